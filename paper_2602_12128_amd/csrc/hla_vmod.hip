// Value modulation (paper Sec. 4.5):  O = T + phi_v1(T) * phi_v2(V), elementwise, with T the
// normalised attention output and phi_v (App. A.1) = Linear d->d, GELU, Linear d->d, LayerNorm.
// Forward and the backward to (dT, dV), as fp32 vector-ALU kernels for any I/O dtype and head dim
// (handles on the matrix-core path with bf16 I/O are served by hla_mfma_vmod.hip instead).
// One workgroup of d threads serves a tile of tokens of one (batch row, head); thread j owns
// hidden unit j of the first layer and channel j of everything after it.  The weights are read
// through the caches ([in][out] order for the forward products, transposed copies for the
// backward ones, so that every read is coalesced over the threads).
#include <algorithm>
#include <cmath>

#include "hla_handle.h"

namespace hla {
namespace {

constexpr int kFwdTile = 32;  // tokens per workgroup, forward
constexpr int kBwdTile = 16;  // tokens per workgroup, backward

__device__ __forceinline__ float gelu_erf(float h) {
  return h * 0.5f * (1.0f + erff(h * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_erf_grad(float h) {
  const float cdf = 0.5f * (1.0f + erff(h * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * expf(-0.5f * h * h);
  return cdf + h * pdf;
}

// fp32 weights of the two maps, densely packed per map m in {0: phi_v1, 1: phi_v2}:
//   W1 [d][d] (in, out), W1T [d][d], W2 [d][d], W2T [d][d], then b1, b2, gamma, beta [d] each
struct VmodW {
  const float* base;
  int d;
  __host__ __device__ int64_t per_map() const { return 4ll * d * d + 4ll * d; }
  __device__ const float* W1(int m) const { return base + m * per_map(); }
  __device__ const float* W1T(int m) const { return W1(m) + d * d; }
  __device__ const float* W2(int m) const { return W1(m) + 2 * d * d; }
  __device__ const float* W2T(int m) const { return W1(m) + 3 * d * d; }
  __device__ const float* b1(int m) const { return W1(m) + 4 * d * d; }
  __device__ const float* b2(int m) const { return b1(m) + d; }
  __device__ const float* gamma(int m) const { return b1(m) + 2 * d; }
  __device__ const float* beta(int m) const { return b1(m) + 3 * d; }
};

template <typename T>
__global__ void k_vmod_pack(const T* W1, const T* b1, const T* W2, const T* b2, const T* gamma,
                            const T* beta, int d, float* __restrict__ out) {
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < d * d; i += gridDim.x * blockDim.x) {
    const int r = i / d, c = i % d;
    out[i] = to_float(W1[i]);
    out[d * d + c * d + r] = to_float(W1[i]);
    out[2 * d * d + i] = to_float(W2[i]);
    out[3 * d * d + c * d + r] = to_float(W2[i]);
    if (i < d) {
      out[4 * d * d + i] = to_float(b1[i]);
      out[4 * d * d + d + i] = to_float(b2[i]);
      out[4 * d * d + 2 * d + i] = to_float(gamma[i]);
      out[4 * d * d + 3 * d + i] = to_float(beta[i]);
    }
  }
}

// One map applied to the TT rows staged in xs ([channel][token], so that a thread reads the TT
// values of one input channel as consecutive floats): h = x W1 + b1 (kept in `hid`),
// u = GELU(h) W2 + b2, then LayerNorm statistics per token through LDS.  On return thread j holds
// u-hat[t][j] in `uhat`, and 1/std of token t sits in rstd_s[t] (LDS, left alone afterwards);
// mean_s [TT] and gs are scratch.
template <int TT>
__device__ __forceinline__ void map_forward(const VmodW& w, int m, int d, int j, const float* xs,
                                            float* gs, float* mean_s, float* rstd_s, float ln_eps,
                                            float (&hid)[TT], float (&uhat)[TT], float* keep_g = nullptr) {
  const float* W1 = w.W1(m);
  const float* W2 = w.W2(m);
#pragma unroll
  for (int t = 0; t < TT; ++t) hid[t] = 0.0f;
  for (int i = 0; i < d; ++i) {
    const float wv = W1[i * d + j];
#pragma unroll
    for (int t = 0; t < TT; ++t) hid[t] += xs[i * TT + t] * wv;
  }
  const float b1 = w.b1(m)[j];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    hid[t] += b1;
    gs[j * TT + t] = gelu_erf(hid[t]);
    if (keep_g != nullptr) keep_g[j * TT + t] = gs[j * TT + t];  // GELU(h), [hidden][token], left alone afterwards
  }
  __syncthreads();
  float u[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) u[t] = 0.0f;
  for (int jj = 0; jj < d; ++jj) {
    const float wv = W2[jj * d + j];
#pragma unroll
    for (int t = 0; t < TT; ++t) u[t] += gs[jj * TT + t] * wv;
  }
  const float b2 = w.b2(m)[j];
  __syncthreads();  // everyone is done reading gs: it now carries u for the statistics
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    u[t] += b2;
    gs[j * TT + t] = u[t];
  }
  __syncthreads();
  if (j < TT) {  // thread t: mean and 1/std of token t over the d channels (two passes, fp32)
    float s = 0.0f;
    for (int c = 0; c < d; ++c) s += gs[c * TT + j];
    const float mean = s / d;
    float v = 0.0f;
    for (int c = 0; c < d; ++c) {
      const float e = gs[c * TT + j] - mean;
      v += e * e;
    }
    mean_s[j] = mean;
    rstd_s[j] = 1.0f / sqrtf(v / d + ln_eps);
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < TT; ++t) uhat[t] = (u[t] - mean_s[t]) * rstd_s[t];
  __syncthreads();  // mean_s and gs are free again
}

template <typename T, int TT>
__device__ __forceinline__ void load_tile(const View& X, int b, int h, int n0, int nt, int d, int j,
                                          float* xs) {
  for (int t = 0; t < TT; ++t) xs[j * TT + t] = t < nt ? to_float(X.row<const T>(b, h, n0 + t)[j]) : 0.0f;
}

// grid (ceil(N / kFwdTile), H, B), block d.  Tin holds T; O receives T + phi_v1(T) * phi_v2(V).
template <typename T>
__global__ void k_vmod_forward(Geom g, VmodW w, float ln_eps, View Tin, View V, View O) {
  constexpr int TT = kFwdTile;
  extern __shared__ float smem[];
  const int d = g.d, j = threadIdx.x;
  float* xs = smem;             // [d][TT]
  float* gs = xs + d * TT;      // [d][TT]
  float* mean_s = gs + d * TT;  // [TT]
  float* rstd_s = mean_s + TT;  // [TT]
  const int n0 = blockIdx.x * TT, h = blockIdx.y, b = blockIdx.z;
  const int nt = min(TT, g.N - n0);
  float hid[TT], uhat[TT], m1[TT], tv[TT];
  load_tile<T, TT>(Tin, b, h, n0, nt, d, j, xs);
  __syncthreads();
#pragma unroll
  for (int t = 0; t < TT; ++t) tv[t] = xs[j * TT + t];
  map_forward<TT>(w, 0, d, j, xs, gs, mean_s, rstd_s, ln_eps, hid, uhat);
  {
    const float ga = w.gamma(0)[j], be = w.beta(0)[j];
#pragma unroll
    for (int t = 0; t < TT; ++t) m1[t] = uhat[t] * ga + be;
  }
  load_tile<T, TT>(V, b, h, n0, nt, d, j, xs);
  __syncthreads();
  map_forward<TT>(w, 1, d, j, xs, gs, mean_s, rstd_s, ln_eps, hid, uhat);
  const float ga = w.gamma(1)[j], be = w.beta(1)[j];
  for (int t = 0; t < nt; ++t)
    O.row<T>(b, h, n0 + t)[j] = from_float<T>(tv[t] + m1[t] * (uhat[t] * ga + be));
}

// Backward of one map for the tile: dm (gradient w.r.t. the map's output, thread j: channel j)
// -> dx (thread j: input channel j).  LayerNorm backward with gg = dm * gamma:
//   du = rstd (gg - mean(gg) - u-hat mean(gg u-hat)),  dg = du W2^T,  dh = dg GELU'(h),  dx = dh W1^T.
// rstd_s [TT] is what map_forward left for this map; a_s, b_s ([d][TT]) and stats ([2][TT]) are scratch.
template <int TT>
__device__ __forceinline__ void map_backward(const VmodW& w, int m, int d, int j, const float (&dm)[TT],
                                             const float (&hid)[TT], const float (&uhat)[TT],
                                             const float* rstd_s, float* a_s, float* b_s, float* stats,
                                             float (&dx)[TT]) {
  const float ga = w.gamma(m)[j];
  float gg[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) {
    gg[t] = dm[t] * ga;
    a_s[j * TT + t] = gg[t];
    b_s[j * TT + t] = gg[t] * uhat[t];
  }
  __syncthreads();
  if (j < TT) {
    float s0 = 0.0f, s1 = 0.0f;
    for (int c = 0; c < d; ++c) {
      s0 += a_s[c * TT + j];
      s1 += b_s[c * TT + j];
    }
    stats[j] = s0 / d;
    stats[TT + j] = s1 / d;
  }
  __syncthreads();
#pragma unroll
  for (int t = 0; t < TT; ++t)
    a_s[j * TT + t] = rstd_s[t] * (gg[t] - stats[t] - uhat[t] * stats[TT + t]);  // du[t][j]
  __syncthreads();
  const float* W2T = w.W2T(m);  // [c][hidden]
  float dg[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) dg[t] = 0.0f;
  for (int c = 0; c < d; ++c) {
    const float wv = W2T[c * d + j];
#pragma unroll
    for (int t = 0; t < TT; ++t) dg[t] += a_s[c * TT + t] * wv;
  }
#pragma unroll
  for (int t = 0; t < TT; ++t) b_s[j * TT + t] = dg[t] * gelu_erf_grad(hid[t]);  // dh[t][j]
  __syncthreads();
  const float* W1T = w.W1T(m);  // [hidden][in]
#pragma unroll
  for (int t = 0; t < TT; ++t) dx[t] = 0.0f;
  for (int jj = 0; jj < d; ++jj) {
    const float wv = W1T[jj * d + j];
#pragma unroll
    for (int t = 0; t < TT; ++t) dx[t] += b_s[jj * TT + t] * wv;
  }
  __syncthreads();
}

// grid (ceil(N / kBwdTile), H, B), block d.  dT = dO + phi_v1'(T)^T (dO * phi_v2(V)),
// dVm = phi_v2'(V)^T (dO * phi_v1(T)); both maps' forward values are recomputed.
template <typename T>
__global__ void k_vmod_backward(Geom g, VmodW w, float ln_eps, View Tin, View V, View dO, View dT,
                                View dVm) {
  constexpr int TT = kBwdTile;
  extern __shared__ float smem[];
  const int d = g.d, j = threadIdx.x;
  float* xs = smem;               // [d][TT]  input rows, then scratch of the backward
  float* gs = xs + d * TT;        // [d][TT]
  float* stats = gs + d * TT;     // [2][TT]
  float* rstd1 = stats + 2 * TT;  // [TT]
  float* rstd2 = rstd1 + TT;      // [TT]
  const int n0 = blockIdx.x * TT, h = blockIdx.y, b = blockIdx.z;
  const int nt = min(TT, g.N - n0);
  float hid1[TT], uhat1[TT], hid2[TT], uhat2[TT];
  load_tile<T, TT>(Tin, b, h, n0, nt, d, j, xs);
  __syncthreads();
  map_forward<TT>(w, 0, d, j, xs, gs, stats, rstd1, ln_eps, hid1, uhat1);
  load_tile<T, TT>(V, b, h, n0, nt, d, j, xs);
  __syncthreads();
  map_forward<TT>(w, 1, d, j, xs, gs, stats, rstd2, ln_eps, hid2, uhat2);
  float dov[TT], dm[TT], dx[TT];
#pragma unroll
  for (int t = 0; t < TT; ++t) dov[t] = t < nt ? to_float(dO.row<const T>(b, h, n0 + t)[j]) : 0.0f;
  const float ga1 = w.gamma(0)[j], be1 = w.beta(0)[j], ga2 = w.gamma(1)[j], be2 = w.beta(1)[j];
#pragma unroll
  for (int t = 0; t < TT; ++t) dm[t] = dov[t] * (uhat2[t] * ga2 + be2);  // d phi_v1(T) = dO * phi_v2(V)
  map_backward<TT>(w, 0, d, j, dm, hid1, uhat1, rstd1, xs, gs, stats, dx);
  for (int t = 0; t < nt; ++t) dT.row<T>(b, h, n0 + t)[j] = from_float<T>(dov[t] + dx[t]);
#pragma unroll
  for (int t = 0; t < TT; ++t) dm[t] = dov[t] * (uhat1[t] * ga1 + be1);  // d phi_v2(V) = dO * phi_v1(T)
  map_backward<TT>(w, 1, d, j, dm, hid2, uhat2, rstd2, xs, gs, stats, dx);
  for (int t = 0; t < nt; ++t) dVm.row<T>(b, h, n0 + t)[j] = from_float<T>(dx[t]);
}

// dst += src over [B, H, N, d] rows (the modulation's share of dV joins the operator's).
template <typename T>
__global__ void k_add_rows(Geom g, View dst, View src) {
  const int64_t idx = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
  const int64_t total = static_cast<int64_t>(g.B) * g.H * g.N * g.d;
  if (idx >= total) return;
  const int c = static_cast<int>(idx % g.d);
  const int64_t th = idx / g.d;
  const int n = static_cast<int>(th % g.N);
  const int64_t bh = th / g.N;
  const int h = static_cast<int>(bh % g.H), b = static_cast<int>(bh / g.H);
  T* p = dst.row<T>(b, h, n) + c;
  *p = from_float<T>(to_float(*p) + to_float(src.row<const T>(b, h, n)[c]));
}

// contiguous [B, H, N, d] view of a workspace array for the current call shape
View ws_view(void* p, const Geom& g) {
  return View{p, static_cast<int64_t>(g.H) * g.N * g.d, static_cast<int64_t>(g.N) * g.d, g.d};
}

// ---- gradients of the modulation's own weights ----------------------------------------------------
// Two steps per map m (0 = phi_v1 applied to T, 1 = phi_v2 applied to V):
//   k_vmod_wgrad_prep  recomputes both maps' forward and this map's backward for every token and
//                      writes the three per-token factors GELU(h), du, dh ([tokens][d] fp32 each);
//                      its workgroups also sum dgamma = sum dm * u-hat and dbeta = sum dm.
//   k_tn_gemm          dW2 = GELU(h)^T du (+ db2 = column sums of du) and dW1 = x^T dh (+ db1),
//                      contractions over the tokens, split over workgroups.
// Partial sums are added in a fixed order by k_sum_parts.

// grid (parts), block d.  Workgroup p serves tiles p, p + parts, .. of the flat list over all
// (batch row, head) pairs; vec_part[p] = [dgamma d | dbeta d].
template <typename T>
__global__ void k_vmod_wgrad_prep(Geom g, VmodW w, float ln_eps, int m, View Tin, View V, View dO,
                                  float* __restrict__ G, float* __restrict__ dU, float* __restrict__ dH,
                                  float* __restrict__ vec_part) {
  constexpr int TT = kBwdTile;
  extern __shared__ float smem[];
  const int d = g.d, j = threadIdx.x;
  float* xs_own = smem;             // [d][TT] input rows of this map
  float* xs_oth = xs_own + d * TT;  // [d][TT] input rows of the other map, then scratch
  float* gs = xs_oth + d * TT;      // [d][TT] scratch
  float* stats = gs + d * TT;       // [2][TT]
  float* rstd_o = stats + 2 * TT;   // [TT]
  float* rstd_s = rstd_o + TT;      // [TT]
  const int tiles_per_row = (g.N + TT - 1) / TT;
  const int total = tiles_per_row * g.B * g.H;
  const float ga_s = w.gamma(m)[j], ga_o = w.gamma(1 - m)[j], be_o = w.beta(1 - m)[j];
  const View& Xs = m == 0 ? Tin : V;
  const View& Xo = m == 0 ? V : Tin;
  float dgam = 0.0f, dbet = 0.0f;
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int row = tile / tiles_per_row, n0 = (tile % tiles_per_row) * TT;
    const int b = row / g.H, h = row % g.H;
    const int nt = min(TT, g.N - n0);
    const int64_t th0 = g.th(b, h, n0);
    load_tile<T, TT>(Xs, b, h, n0, nt, d, j, xs_own);
    load_tile<T, TT>(Xo, b, h, n0, nt, d, j, xs_oth);
    __syncthreads();
    float hid[TT], uhat[TT], mo[TT];
    map_forward<TT>(w, 1 - m, d, j, xs_oth, gs, stats, rstd_o, ln_eps, hid, uhat);
#pragma unroll
    for (int t = 0; t < TT; ++t) mo[t] = uhat[t] * ga_o + be_o;
    map_forward<TT>(w, m, d, j, xs_own, gs, stats, rstd_s, ln_eps, hid, uhat);
    for (int t = 0; t < nt; ++t) G[(th0 + t) * d + j] = gelu_erf(hid[t]);
    // LayerNorm backward (thread j: channel j); rows past the end carry dO = 0
    float gg[TT];
    float* a_s = xs_oth;  // free: the other map is done
#pragma unroll
    for (int t = 0; t < TT; ++t) {
      const float dov = t < nt ? to_float(dO.row<const T>(b, h, n0 + t)[j]) : 0.0f;
      const float dm = dov * mo[t];
      dgam += dm * uhat[t];
      dbet += dm;
      gg[t] = dm * ga_s;
      a_s[j * TT + t] = gg[t];
      gs[j * TT + t] = gg[t] * uhat[t];
    }
    __syncthreads();
    if (j < TT) {
      float s0 = 0.0f, s1 = 0.0f;
      for (int c = 0; c < d; ++c) {
        s0 += a_s[c * TT + j];
        s1 += gs[c * TT + j];
      }
      stats[j] = s0 / d;
      stats[TT + j] = s1 / d;
    }
    __syncthreads();
    float du[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) du[t] = rstd_s[t] * (gg[t] - stats[t] - uhat[t] * stats[TT + t]);
    __syncthreads();  // the statistics pass is done reading a_s
#pragma unroll
    for (int t = 0; t < TT; ++t) a_s[j * TT + t] = du[t];
    for (int t = 0; t < nt; ++t) dU[(th0 + t) * d + j] = du[t];
    __syncthreads();
    const float* W2T = w.W2T(m);
    float dh[TT];
#pragma unroll
    for (int t = 0; t < TT; ++t) dh[t] = 0.0f;
    for (int c = 0; c < d; ++c) {
      const float wv = W2T[c * d + j];
#pragma unroll
      for (int t = 0; t < TT; ++t) dh[t] += a_s[c * TT + t] * wv;
    }
    for (int t = 0; t < nt; ++t) dH[(th0 + t) * d + j] = dh[t] * gelu_erf_grad(hid[t]);
    __syncthreads();
  }
  vec_part[blockIdx.x * 2 * d + j] = dgam;
  vec_part[blockIdx.x * 2 * d + d + j] = dbet;
}

// C[i][j] = sum over tokens of A[t][i] B[t][j] and s[j] = sum over tokens of B[t][j], for A a
// [B, H, N, D] view of element type TA and B a contiguous [tokens][D] fp32 array in the same token
// order.  grid (parts), block 256: thread (ty, tx) = (tid / 16, tid % 16) owns the RT x RT block
// of C at rows ty RT, columns tx RT.  Workgroup p serves the 16-token tiles p, p + parts, ..;
// part[p] = [C D*D | s D].
template <typename TA, int D>
__global__ __launch_bounds__(256) void k_tn_gemm(Geom g, View A, const float* __restrict__ Bm,
                                                 float* __restrict__ part) {
  constexpr int TT = 16, RT = D / 16;
  __shared__ float As[TT][D], Bs[TT][D];
  const int tid = threadIdx.x, ty = tid / 16, tx = tid % 16;
  float acc[RT][RT], bsum[RT];
#pragma unroll
  for (int x = 0; x < RT; ++x) {
    bsum[x] = 0.0f;
#pragma unroll
    for (int y = 0; y < RT; ++y) acc[x][y] = 0.0f;
  }
  const int tiles_per_row = (g.N + TT - 1) / TT;
  const int total = tiles_per_row * g.B * g.H;
  for (int tile = blockIdx.x; tile < total; tile += gridDim.x) {
    const int row = tile / tiles_per_row, n0 = (tile % tiles_per_row) * TT;
    const int b = row / g.H, h = row % g.H;
    const int64_t th0 = g.th(b, h, n0);
    for (int e = tid; e < TT * D; e += 256) {
      const int t = e / D, c = e % D;
      const bool live = n0 + t < g.N;
      As[t][c] = live ? to_float(A.row<const TA>(b, h, n0 + t)[c]) : 0.0f;
      Bs[t][c] = live ? Bm[(th0 + t) * D + c] : 0.0f;
    }
    __syncthreads();
#pragma unroll 4
    for (int t = 0; t < TT; ++t) {
      float av[RT], bv[RT];
#pragma unroll
      for (int x = 0; x < RT; ++x) {
        av[x] = As[t][ty * RT + x];
        bv[x] = Bs[t][tx * RT + x];
      }
#pragma unroll
      for (int x = 0; x < RT; ++x) {
        if (ty == 0) bsum[x] += bv[x];
#pragma unroll
        for (int y = 0; y < RT; ++y) acc[x][y] += av[x] * bv[y];
      }
    }
    __syncthreads();
  }
  float* out = part + static_cast<int64_t>(blockIdx.x) * (D * D + D);
#pragma unroll
  for (int x = 0; x < RT; ++x) {
#pragma unroll
    for (int y = 0; y < RT; ++y) out[(ty * RT + x) * D + tx * RT + y] = acc[x][y];
    if (ty == 0) out[D * D + tx * RT + x] = bsum[x];
  }
}

// dst[k] = sum over p < nparts of part[p * stride + off + k], k < len, in order; nparts = 0 gives zeros
__global__ void k_sum_parts(const float* __restrict__ part, int nparts, int64_t stride, int64_t off,
                            int64_t len, float* __restrict__ dst) {
  const int64_t k = blockIdx.x * static_cast<int64_t>(blockDim.x) + threadIdx.x;
  if (k >= len) return;
  float s = 0.0f;
  for (int p = 0; p < nparts; ++p) s += part[p * stride + off + k];
  dst[k] = s;
}

hla_status sum_parts(hla_handle* hd, hipStream_t s, const float* part, int nparts, int64_t stride,
                     int64_t off, int64_t len, float* dst) {
  return launch(hd, "vmod_weight_grads_reduce", k_sum_parts, dim3(static_cast<unsigned>((len + 255) / 256)),
                dim3(256), 0, s, part, nparts, stride, off, len, dst);
}

template <typename TA, int D>
hla_status tn_gemm_t(hla_handle* hd, hipStream_t s, View A, const float* Bm, int nparts) {
  return launch(hd, "vmod_weight_grads_gemm", k_tn_gemm<TA, D>, dim3(nparts), dim3(256), 0, s, hd->g, A, Bm,
                hd->vmod_wg_partial);
}
template <typename TA>
hla_status tn_gemm(hla_handle* hd, hipStream_t s, View A, const float* Bm, int nparts) {
  switch (hd->g.d) {
    case 32: return tn_gemm_t<TA, 32>(hd, s, A, Bm, nparts);
    case 64: return tn_gemm_t<TA, 64>(hd, s, A, Bm, nparts);
    case 128: return tn_gemm_t<TA, 128>(hd, s, A, Bm, nparts);
    default: return HLA_ERR_UNSUPPORTED;
  }
}

// one map's six gradients; `nparts` = 0: zeros only
template <typename T>
hla_status wgrad_map(hla_handle* hd, const hla_call_args& a, int m, int nparts) {
  const Geom& g = hd->g;
  const int64_t d = g.d, dd = d * d;
  const hla_vmod_weight_grads& o = hd->vmod_wg_out[m];
  hipStream_t s = a.stream;
  float* part = hd->vmod_wg_partial;
  if (nparts == 0) {
    HLA_TRY(sum_parts(hd, s, part, 0, 0, 0, dd, o.dW1));
    HLA_TRY(sum_parts(hd, s, part, 0, 0, 0, d, o.db1));
    HLA_TRY(sum_parts(hd, s, part, 0, 0, 0, dd, o.dW2));
    HLA_TRY(sum_parts(hd, s, part, 0, 0, 0, d, o.db2));
    HLA_TRY(sum_parts(hd, s, part, 0, 0, 0, d, o.dgamma));
    return sum_parts(hd, s, part, 0, 0, 0, d, o.dbeta);
  }
  const VmodW w{hd->vmod_w, g.d};
  const int64_t per = hd->max_th * d;
  float* G = hd->vmod_wg_rows;
  float* dU = G + per;
  float* dH = dU + per;
  const size_t sh = (3 * static_cast<size_t>(d) * kBwdTile + 4 * kBwdTile) * sizeof(float);
  const View Tv = ws_view(hd->vmod_T, g);
  HLA_TRY(launch(hd, "vmod_weight_grads_prep", k_vmod_wgrad_prep<T>, dim3(nparts), dim3(g.d), sh, s, g, w,
                 hd->vmod_ln_eps, m, Tv, a.V, a.dO, G, dU, dH, part));
  HLA_TRY(sum_parts(hd, s, part, nparts, 2 * d, 0, d, o.dgamma));
  HLA_TRY(sum_parts(hd, s, part, nparts, 2 * d, d, d, o.dbeta));
  // dW2 = GELU(h)^T du, db2 = sum du
  const View Gv{G, static_cast<int64_t>(g.H) * g.N * d, static_cast<int64_t>(g.N) * d, d};
  HLA_TRY(tn_gemm<float>(hd, s, Gv, dU, nparts));
  HLA_TRY(sum_parts(hd, s, part, nparts, dd + d, 0, dd, o.dW2));
  HLA_TRY(sum_parts(hd, s, part, nparts, dd + d, dd, d, o.db2));
  // dW1 = x^T dh, db1 = sum dh
  HLA_TRY(tn_gemm<T>(hd, s, m == 0 ? Tv : a.V, dH, nparts));
  HLA_TRY(sum_parts(hd, s, part, nparts, dd + d, 0, dd, o.dW1));
  return sum_parts(hd, s, part, nparts, dd + d, dd, d, o.db1);
}

template <typename T>
hla_status set_weights_t(hla_handle* hd, const hla_vmod_weights* maps, hipStream_t s) {
  const int d = hd->g.d;
  const int64_t per = 4ll * d * d + 4ll * d;
  for (int m = 0; m < 2; ++m)
    HLA_TRY(launch(hd, "vmod_pack", k_vmod_pack<T>, dim3(64), dim3(256), 0, s,
                   static_cast<const T*>(maps[m].W1), static_cast<const T*>(maps[m].b1),
                   static_cast<const T*>(maps[m].W2), static_cast<const T*>(maps[m].b2),
                   static_cast<const T*>(maps[m].gamma), static_cast<const T*>(maps[m].beta), d,
                   hd->vmod_w + m * per));
  return HLA_OK;
}


template <typename T>
hla_status forward_t(hla_handle* hd, const hla_call_args& a) {
  const Geom& g = hd->g;
  const VmodW w{hd->vmod_w, g.d};
  const size_t sh = (2 * static_cast<size_t>(g.d) * kFwdTile + 2 * kFwdTile) * sizeof(float);
  return launch(hd, "vmod_forward", k_vmod_forward<T>, dim3((g.N + kFwdTile - 1) / kFwdTile, g.H, g.B),
                dim3(g.d), sh, a.stream, g, w, hd->vmod_ln_eps, ws_view(hd->vmod_T, g), a.V, a.O);
}

template <typename T>
hla_status backward_t(hla_handle* hd, const hla_call_args& a) {
  const Geom& g = hd->g;
  const VmodW w{hd->vmod_w, g.d};
  const size_t sh = (2 * static_cast<size_t>(g.d) * kBwdTile + 4 * kBwdTile) * sizeof(float);
  return launch(hd, "vmod_backward", k_vmod_backward<T>, dim3((g.N + kBwdTile - 1) / kBwdTile, g.H, g.B),
                dim3(g.d), sh, a.stream, g, w, hd->vmod_ln_eps, ws_view(hd->vmod_T, g), a.V, a.dO,
                ws_view(hd->vmod_dT, g), ws_view(hd->vmod_dV, g));
}

template <typename T>
hla_status add_t(hla_handle* hd, const hla_call_args& a) {
  const Geom& g = hd->g;
  const int64_t total = static_cast<int64_t>(g.B) * g.H * g.N * g.d;
  return launch(hd, "vmod_add_dv", k_add_rows<T>, dim3(static_cast<unsigned>((total + 255) / 256)), dim3(256),
                0, a.stream, g, a.dV, ws_view(hd->vmod_dV, g));
}

}  // namespace

hla_status vmod_set_weights(hla_handle* hd, const hla_vmod_weights* maps, hipStream_t s) {
  if (hd->vmod_wpk != nullptr) HLA_TRY(vmod_mfma_set_weights(hd, maps, s));
  return hd->cfg.io_dtype == HLA_F32 ? set_weights_t<float>(hd, maps, s) : set_weights_t<bf16_t>(hd, maps, s);
}
hla_status vmod_forward(hla_handle* hd, const hla_call_args& a) {
  if (hd->vmod_wpk != nullptr) return vmod_mfma_forward(hd, a);
  return hd->cfg.io_dtype == HLA_F32 ? forward_t<float>(hd, a) : forward_t<bf16_t>(hd, a);
}
hla_status vmod_backward(hla_handle* hd, const hla_call_args& a) {
  if (hd->vmod_wpk != nullptr) return vmod_mfma_backward(hd, a);
  return hd->cfg.io_dtype == HLA_F32 ? backward_t<float>(hd, a) : backward_t<bf16_t>(hd, a);
}
hla_status vmod_add_value_grads(hla_handle* hd, const hla_call_args& a) {
  if (hd->vmod_wpk != nullptr) return vmod_mfma_add_value_grads(hd, a);
  return hd->cfg.io_dtype == HLA_F32 ? add_t<float>(hd, a) : add_t<bf16_t>(hd, a);
}
View vmod_view(void* p, const Geom& g) { return ws_view(p, g); }

int64_t vmod_wgrad_part_floats(int d) { return static_cast<int64_t>(d) * d + d; }

hla_status vmod_weight_grads(hla_handle* hd, const hla_call_args& a, bool empty) {
  const Geom& g = hd->g;
  // matrix-core handles: the backward kernel has left the per-token factors
  if (!empty && hd->vmod_wpk != nullptr) return vmod_mfma_weight_grads(hd, a);
  int nparts = 0;
  if (!empty) {
    const int64_t tiles = static_cast<int64_t>((g.N + kBwdTile - 1) / kBwdTile) * g.B * g.H;
    nparts = static_cast<int>(std::min<int64_t>(tiles, kVmodWgradParts));
  }
  for (int m = 0; m < 2; ++m)
    HLA_TRY(hd->cfg.io_dtype == HLA_F32 ? wgrad_map<float>(hd, a, m, nparts) : wgrad_map<bf16_t>(hd, a, m, nparts));
  return HLA_OK;
}

}  // namespace hla
