// Generic path: fp32 vector-ALU kernels over the literal d_phi^F feature tensor (no matrix
// cores, no algebraic compression).  Serves fp32 I/O, unusual (F, d_phi) and acts as an
// independent GPU cross-check of the MFMA path.  Throughput is not a goal here.
//
// With the augmented state  Chat = [C | z]  ([D, d+1]) and augmented per-token rows
// vhat_j = [v_j | 1], ghat_i = [dO_i/den_i | -<dO_i,o_i>/den_i] every step is one of three
// shapes (Theorem 4.2 and its derivatives):
//   accumulate : Chat  = sum_j T_j (x) yhat_j            (state; d state with T_q, ghat)
//   contract   : out_i = T_i . Chat                       (query side; dV with T_k, dChat)
//   dtensor    : dT_i  = Chat yhat_i, then the chain rule through the outer product
#include <cmath>

#include "hla_handle.h"

namespace hla {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 1024;      // tokens per partial state
constexpr int kAccTile = 8;       // tokens staged per step of accumulate
constexpr int kMaxRows = 128;     // accumulator rows per thread in accumulate: D*d/256 <= 128
constexpr int kTokPerThread = 4;  // contract: tokens per thread
constexpr int kDtTile = 8;        // dtensor: tokens per block
constexpr int kPhiTile = 16;      // feature maps: tokens per block
constexpr int kWgTile = 8;        // weight gradients: tokens staged per step
constexpr int kMaxF = 4;

__device__ __forceinline__ float gelu_erf(float h) {
  return h * 0.5f * (1.0f + erff(h * 0.70710678118654752440f));
}
__device__ __forceinline__ float gelu_erf_grad(float h) {
  const float cdf = 0.5f * (1.0f + erff(h * 0.70710678118654752440f));
  const float pdf = 0.39894228040143267794f * expf(-0.5f * h * h);
  return cdf + h * pdf;
}

// Slot offsets into a feature row: query tensors use phi_q in every slot, key tensors use map f.
__device__ __forceinline__ int slot_offset(bool query, int slot, int dphi) {
  return query ? 0 : (1 + slot) * dphi;
}

// Entry `Di` of the outer product of one token's features (first slot slowest).
__device__ __forceinline__ float outer_entry(const float* frow, bool query, int Di, int F,
                                             int dphi) {
  float p = 1.0f;
  for (int s = F - 1; s >= 0; --s) {
    const int a = Di % dphi;
    Di /= dphi;
    p *= frow[slot_offset(query, s, dphi) + a];
  }
  return p;
}

// ---- weights / features I/O -------------------------------------------------------------------
template <typename T>
__global__ void k_convert_weights(const T* __restrict__ src, int64_t head_stride, float* dst,
                                  int count, int heads_w) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int hw = blockIdx.y;
  if (i < count && hw < heads_w) dst[static_cast<int64_t>(hw) * count + i] = to_float(src[hw * head_stride + i]);
}

// PHI_NONE: copy caller-provided features into the fp32 feature workspace.  One thread per
// token-head: its two feature rows are contiguous in the caller's tensors, and in the tiled
// workspace of the MFMA path 32 consecutive threads write 32 consecutive floats per feature.
template <typename T>
__global__ void k_feat_import(Geom g, View Q, View K, float* __restrict__ feat) {
  const uint32_t th = blockIdx.x * blockDim.x + threadIdx.x;
  if (th >= static_cast<uint32_t>(g.B) * g.H * g.N) return;  // < 2^31 by the create-time check
  const int n = static_cast<int>(th % g.N);
  const uint32_t bh = th / g.N;
  const int h = static_cast<int>(bh % g.H), b = static_cast<int>(bh / g.H);
  const T* q = Q.row<const T>(b, h, n);
  const T* k = K.row<const T>(b, h, n);
  if constexpr (sizeof(T) == 2) {
    // a pair of bf16 features per load and an 8-byte store per pair where the rows allow it: a
    // pair is adjacent in both layouts of the workspace (see fidx), pair p + 1 sits `step` floats on
    const bool pairs = g.dphi % 2 == 0 && ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k)) & 3) == 0;
    if (pairs) {
      const uint32_t* q2 = reinterpret_cast<const uint32_t*>(q);
      const uint32_t* k2 = reinterpret_cast<const uint32_t*>(k);
      float* dst = feat + g.fidx(th, 0);
      const int step = g.feat_tiled ? 64 : 2, nq = g.dphi / 2, np = g.nfeat / 2;
      // eight pairs' loads in flight before the first store (a load next to the store that needs
      // it would cost a memory round trip per pair)
      for (int p0 = 0; p0 < np; p0 += 8) {
        uint32_t w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int p = p0 + i < np ? p0 + i : np - 1;
          w[i] = p < nq ? q2[p] : k2[p - nq];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(w[i]));  // all eight are loaded here: the compiler may not sink a load to its store
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if (p0 + i >= np) break;
          float2 v;
          v.x = __uint_as_float(w[i] << 16);
          v.y = __uint_as_float(w[i] & 0xffff0000u);
          *reinterpret_cast<float2*>(dst + static_cast<int64_t>(p0 + i) * step) = v;
        }
      }
      return;
    }
  }
  for (int j = 0; j < g.dphi; ++j) feat[g.fidx(th, j)] = to_float(q[j]);
  for (int j = g.dphi; j < g.nfeat; ++j) feat[g.fidx(th, j)] = to_float(k[j - g.dphi]);
}

// PHI_NONE: feature gradients are the answer; store them in the I/O dtype.
template <typename T>
__global__ void k_dfeat_export(Geom g, const float* __restrict__ dfeat, View dQ, View dK) {
  const uint32_t th = blockIdx.x * blockDim.x + threadIdx.x;
  if (th >= static_cast<uint32_t>(g.B) * g.H * g.N) return;
  const int n = static_cast<int>(th % g.N);
  const uint32_t bh = th / g.N;
  const int h = static_cast<int>(bh % g.H), b = static_cast<int>(bh / g.H);
  T* q = dQ.row<T>(b, h, n);
  T* k = dK.row<T>(b, h, n);
  if constexpr (sizeof(T) == 2) {
    // two bf16 values per store where the rows allow it
    const bool pairs = g.dphi % 2 == 0 && ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k)) & 3) == 0;
    if (pairs) {
      uint32_t* q2 = reinterpret_cast<uint32_t*>(q);
      uint32_t* k2 = reinterpret_cast<uint32_t*>(k);
      const float* src = dfeat + g.fidx(th, 0);  // pair p: 8 bytes at src + p * step (see fidx)
      const int step = g.feat_tiled ? 64 : 2, nq = g.dphi / 2, np = g.nfeat / 2;
      for (int p0 = 0; p0 < np; p0 += 8) {  // eight pairs' loads in flight before the first store
        float2 v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
          v[i] = *reinterpret_cast<const float2*>(src + static_cast<int64_t>(p0 + i < np ? p0 + i : np - 1) * step);
#pragma unroll
        for (int i = 0; i < 8; ++i) asm volatile("" : "+v"(v[i].x), "+v"(v[i].y));  // as in k_feat_import
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          if (p0 + i >= np) break;
          const uint32_t w = static_cast<uint32_t>(f32_to_bf16_bits(v[i].x)) |
                             (static_cast<uint32_t>(f32_to_bf16_bits(v[i].y)) << 16);
          if (p0 + i < nq) q2[p0 + i] = w; else k2[p0 + i - nq] = w;
        }
      }
      return;
    }
  }
  for (int j = 0; j < g.dphi; ++j) q[j] = from_float<T>(dfeat[g.fidx(th, j)]);
  for (int j = g.dphi; j < g.nfeat; ++j) k[j - g.dphi] = from_float<T>(dfeat[g.fidx(th, j)]);
}

// ---- feature maps (App. A.1) ------------------------------------------------------------------
// grid (ceil(N/kPhiTile), H, B), block d threads.  Thread j owns hidden unit j.
template <typename T>
__global__ void k_phi_forward(Geom g, PhiF32 w, View Q, View K, float* __restrict__ feat) {
  extern __shared__ float smem[];
  const int d = g.d, dphi = g.dphi;
  float* xs = smem;                 // [kPhiTile][d]
  float* gs = smem + kPhiTile * d;  // [kPhiTile][d]
  const int j = threadIdx.x;
  const int n0 = blockIdx.x * kPhiTile, h = blockIdx.y, b = blockIdx.z;
  const int nt = min(kPhiTile, g.N - n0);
  const int hw = w.heads_w == 1 ? 0 : h;
  for (int m = 0; m <= g.F; ++m) {
    if (m <= 1) {
      __syncthreads();
      const View& X = m == 0 ? Q : K;
      for (int t = 0; t < kPhiTile; ++t)
        xs[t * d + j] = t < nt ? to_float(X.row<const T>(b, h, n0 + t)[j]) : 0.0f;
      __syncthreads();
    }
    const int64_t mh = static_cast<int64_t>(m) * w.heads_w + hw;
    const float* W1 = w.W1 + mh * d * d;
    const float* W2 = w.W2 + mh * d * dphi;
    float acc[kPhiTile];
#pragma unroll
    for (int t = 0; t < kPhiTile; ++t) acc[t] = 0.0f;
    for (int i = 0; i < d; ++i) {
      const float wv = W1[i * d + j];
#pragma unroll
      for (int t = 0; t < kPhiTile; ++t) acc[t] += xs[t * d + i] * wv;
    }
    const float bias = w.b1[mh * d + j];
#pragma unroll
    for (int t = 0; t < kPhiTile; ++t) gs[t * d + j] = gelu_erf(acc[t] + bias);
    __syncthreads();
    for (int idx = j; idx < nt * dphi; idx += d) {
      const int t = idx / dphi, c = idx % dphi;
      float u = w.b2[mh * dphi + c];
      for (int jj = 0; jj < d; ++jj) u += gs[t * d + jj] * W2[jj * dphi + c];
      feat[g.fidx(g.th(b, h, n0 + t), m * dphi + c)] = fmaxf(u, 0.0f);
    }
    __syncthreads();
  }
}

// Input gradients through the feature maps; hidden activations are recomputed.  dK sums the F
// key maps.  Thread j owns hidden unit j and input coordinate j.
template <typename T>
__global__ void k_phi_backward(Geom g, PhiF32 w, View Q, View K, const float* __restrict__ feat,
                               const float* __restrict__ dfeat, View dQ, View dK) {
  extern __shared__ float smem[];
  const int d = g.d, dphi = g.dphi;
  float* xs = smem;                   // [kPhiTile][d]
  float* dhs = xs + kPhiTile * d;     // [kPhiTile][d]
  float* dus = dhs + kPhiTile * d;    // [kPhiTile][dphi]
  const int j = threadIdx.x;
  const int n0 = blockIdx.x * kPhiTile, h = blockIdx.y, b = blockIdx.z;
  const int nt = min(kPhiTile, g.N - n0);
  const int hw = w.heads_w == 1 ? 0 : h;
  float dx[kPhiTile];
  for (int m = 0; m <= g.F; ++m) {
    if (m <= 1) {
      __syncthreads();
      const View& X = m == 0 ? Q : K;
      for (int t = 0; t < kPhiTile; ++t)
        xs[t * d + j] = t < nt ? to_float(X.row<const T>(b, h, n0 + t)[j]) : 0.0f;
#pragma unroll
      for (int t = 0; t < kPhiTile; ++t) dx[t] = 0.0f;
    }
    __syncthreads();
    for (int idx = j; idx < kPhiTile * dphi; idx += d) {
      const int t = idx / dphi, c = idx % dphi;
      float du = 0.0f;
      if (t < nt) {
        const int64_t o = g.fidx(g.th(b, h, n0 + t), m * dphi + c);
        du = feat[o] > 0.0f ? dfeat[o] : 0.0f;  // ReLU passes gradient only where it was open
      }
      dus[idx] = du;
    }
    __syncthreads();
    const int64_t mh = static_cast<int64_t>(m) * w.heads_w + hw;
    const float* W1 = w.W1 + mh * d * d;
    const float* W2 = w.W2 + mh * d * dphi;
    float acc[kPhiTile];
#pragma unroll
    for (int t = 0; t < kPhiTile; ++t) acc[t] = 0.0f;
    for (int i = 0; i < d; ++i) {
      const float wv = W1[i * d + j];
#pragma unroll
      for (int t = 0; t < kPhiTile; ++t) acc[t] += xs[t * d + i] * wv;
    }
    const float bias = w.b1[mh * d + j];
#pragma unroll
    for (int t = 0; t < kPhiTile; ++t) {
      float dg = 0.0f;
      for (int c = 0; c < dphi; ++c) dg += dus[t * dphi + c] * W2[j * dphi + c];
      dhs[t * d + j] = dg * gelu_erf_grad(acc[t] + bias);
    }
    __syncthreads();
    for (int jj = 0; jj < d; ++jj) {
      const float wv = W1[j * d + jj];  // dx_j = sum_jj dh_jj W1[j][jj]
#pragma unroll
      for (int t = 0; t < kPhiTile; ++t) dx[t] += dhs[t * d + jj] * wv;
    }
    if (m == 0 || m == g.F) {
      const View& dX = m == 0 ? dQ : dK;
      for (int t = 0; t < nt; ++t) dX.row<T>(b, h, n0 + t)[j] = from_float<T>(dx[t]);
    }
  }
}

// ---- weight gradients of the feature maps -----------------------------------------------------
// dW1 = x^T dh, db1 = sum dh, dW2 = GELU(h)^T du, db2 = sum du over the tokens of a chunk; hidden
// activations are recomputed.  grid (chunks, 1+F, heads_w), block DD = d threads.  Thread j owns
// hidden unit j: column j of dW1, row j of dW2 and entry j of db1 stay in its registers for the
// whole chunk, so nothing is reduced across threads.  The chunk's sums go to
// partial[((map * gridDim.z + hw) * chunks + chunk)][d*d | d | d*dphi | dphi].
// Token tiles: with shared weights (heads_w == 1) the tiles of all (batch row, head) pairs form
// one list; with per-head weights the list of head blockIdx.z holds that head's tiles only.
template <typename T, int DD>
__global__ __launch_bounds__(DD) void k_phi_wgrad(Geom g, PhiF32 w, View Q, View K,
                                                  const float* __restrict__ feat,
                                                  const float* __restrict__ dfeat,
                                                  float* __restrict__ partial) {
  __shared__ float xs[kWgTile][DD];
  __shared__ float dhs[kWgTile][DD];
  __shared__ float dus[kWgTile][16];
  const int dphi = g.dphi;
  const int j = threadIdx.x;
  const int chunk = blockIdx.x, nchunk = gridDim.x, m = blockIdx.y, hw = blockIdx.z;
  const bool shared = w.heads_w == 1;
  const int tpr = (g.N + kWgTile - 1) / kWgTile;
  const int rows = shared ? g.B * g.H : g.B;
  const int total = rows * tpr;
  const int per = (total + nchunk - 1) / nchunk;
  const int t_begin = chunk * per, t_end = min(total, t_begin + per);
  const int64_t mh = static_cast<int64_t>(m) * w.heads_w + hw;
  const float* W1 = w.W1 + mh * DD * DD;
  const float* W2 = w.W2 + mh * DD * dphi;
  const float bias = w.b1[mh * DD + j];
  float w2row[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) w2row[c] = c < dphi ? W2[j * dphi + c] : 0.0f;
  const View& X = m == 0 ? Q : K;
  float dW1c[DD];     // column j of dW1
  float dW2r[16];     // row j of dW2
  float db1 = 0.0f, db2 = 0.0f;
#pragma unroll
  for (int i = 0; i < DD; ++i) dW1c[i] = 0.0f;
#pragma unroll
  for (int c = 0; c < 16; ++c) dW2r[c] = 0.0f;
  for (int tile = t_begin; tile < t_end; ++tile) {
    const int row = tile / tpr, n0 = (tile % tpr) * kWgTile;
    const int b = shared ? row / g.H : row, h = shared ? row % g.H : hw;
    const int nt = min(kWgTile, g.N - n0);
    __syncthreads();
    for (int t = 0; t < kWgTile; ++t) xs[t][j] = t < nt ? to_float(X.row<const T>(b, h, n0 + t)[j]) : 0.0f;
    for (int idx = j; idx < kWgTile * 16; idx += DD) {
      const int t = idx / 16, c = idx % 16;
      float du = 0.0f;
      if (t < nt && c < dphi) {
        const int64_t o = g.fidx(g.th(b, h, n0 + t), m * dphi + c);
        du = feat[o] > 0.0f ? dfeat[o] : 0.0f;  // ReLU passes gradient only where it was open
      }
      dus[t][c] = du;
    }
    __syncthreads();
    float acc[kWgTile];
#pragma unroll
    for (int t = 0; t < kWgTile; ++t) acc[t] = bias;
    for (int i = 0; i < DD; ++i) {
      const float wv = W1[i * DD + j];
#pragma unroll
      for (int t = 0; t < kWgTile; ++t) acc[t] += xs[t][i] * wv;
    }
#pragma unroll
    for (int t = 0; t < kWgTile; ++t) {
      float dg = 0.0f;
#pragma unroll
      for (int c = 0; c < 16; ++c) dg += dus[t][c] * w2row[c];
      const float gv = gelu_erf(acc[t]);
      const float dh = dg * gelu_erf_grad(acc[t]);
      db1 += dh;
#pragma unroll
      for (int c = 0; c < 16; ++c) dW2r[c] += gv * dus[t][c];
      if (j < dphi) db2 += dus[t][j];
      dhs[t][j] = dh;  // read back by this thread only
    }
    // one token at a time, so that only one row of x is in flight beside the DD accumulators
#pragma unroll 1
    for (int t = 0; t < kWgTile; ++t) {
      const float dh = dhs[t][j];
#pragma unroll
      for (int i = 0; i < DD; ++i) dW1c[i] += xs[t][i] * dh;
    }
  }
  float* out = partial + ((static_cast<int64_t>(m) * gridDim.z + hw) * nchunk + chunk) *
                             (static_cast<int64_t>(DD) * DD + DD + DD * dphi + dphi);
#pragma unroll
  for (int i = 0; i < DD; ++i) out[i * DD + j] = dW1c[i];
  out[DD * DD + j] = db1;
#pragma unroll
  for (int c = 0; c < 16; ++c)
    if (c < dphi) out[DD * DD + DD + j * dphi + c] = dW2r[c];
  if (j < dphi) out[DD * DD + DD + DD * dphi + j] = db2;
}

// Sum of the partial weight gradients of one (map, head) in partial order, times the scale of
// its section, into the caller's arrays.  grid (ceil(floats / 256), 1+F, heads), block 256.
struct WgradOut {
  float* dW1[kMaxF + 1];
  float* db1[kMaxF + 1];
  float* dW2[kMaxF + 1];
  float* db2[kMaxF + 1];
};
__global__ void k_wgrad_reduce(int d, int dphi, int nparts,
                               const float* __restrict__ partial, WgradOut out, float sW1, float sb1,
                               float sW2, float sb2) {
  const int nW1 = d * d, nb1 = d, nW2 = d * dphi, nb2 = dphi;
  const int floats = nW1 + nb1 + nW2 + nb2;
  const int e = blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= floats) return;
  const int m = blockIdx.y, hw = blockIdx.z;
  const float* p = partial + (static_cast<int64_t>(m) * gridDim.z + hw) * nparts * floats + e;
  float sum = 0.0f;
  int k = 0;
  for (; k + 8 <= nparts; k += 8) {  // eight loads in flight, added in partial order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = p[static_cast<int64_t>(k + u) * floats];
#pragma unroll
    for (int u = 0; u < 8; ++u) sum += v[u];
  }
  for (; k < nparts; ++k) sum += p[static_cast<int64_t>(k) * floats];
  if (e < nW1) {
    out.dW1[m][static_cast<int64_t>(hw) * nW1 + e] = sW1 * sum;
  } else if (e < nW1 + nb1) {
    out.db1[m][static_cast<int64_t>(hw) * nb1 + (e - nW1)] = sb1 * sum;
  } else if (e < nW1 + nb1 + nW2) {
    out.dW2[m][static_cast<int64_t>(hw) * nW2 + (e - nW1 - nb1)] = sW2 * sum;
  } else {
    out.db2[m][static_cast<int64_t>(hw) * nb2 + (e - nW1 - nb1 - nW2)] = sb2 * sum;
  }
}

template <typename T>
hla_status weight_grads_t(hla_handle* hd, const hla_call_args& a) {
  Geom g = hd->g;
  g.B = a.B;
  g.H = a.H;
  g.N = a.N;
  if (g.dphi > 16) return HLA_ERR_UNSUPPORTED;
  const int nm = 1 + g.F;
  const int heads = hd->phi.heads_w == 1 ? 1 : a.H;
  // about one full grid of workgroups in total, never more partial sums than the workspace holds
  int64_t nchunk = 512 / (static_cast<int64_t>(nm) * heads);
  const int64_t tiles = (hd->phi.heads_w == 1 ? static_cast<int64_t>(a.B) * a.H : a.B) *
                        ((a.N + kWgTile - 1) / kWgTile);
  if (nchunk > tiles) nchunk = tiles;
  if (nchunk < 1) nchunk = 1;
  if (nm * static_cast<int64_t>(heads) * nchunk > hd->wg_parts_cap) return HLA_ERR_STATE;
  const dim3 grid(static_cast<unsigned>(nchunk), nm, heads);
  hipStream_t s = a.stream;
  switch (g.d) {
    case 32:
      HLA_TRY(launch(hd, "phi_weight_grads", k_phi_wgrad<T, 32>, grid, dim3(32), 0, s, g, hd->phi, a.Q, a.K,
                     static_cast<const float*>(hd->feat), static_cast<const float*>(hd->dfeat), hd->wg_partial));
      break;
    case 64:
      HLA_TRY(launch(hd, "phi_weight_grads", k_phi_wgrad<T, 64>, grid, dim3(64), 0, s, g, hd->phi, a.Q, a.K,
                     static_cast<const float*>(hd->feat), static_cast<const float*>(hd->dfeat), hd->wg_partial));
      break;
    case 128:
      HLA_TRY(launch(hd, "phi_weight_grads", k_phi_wgrad<T, 128>, grid, dim3(128), 0, s, g, hd->phi, a.Q, a.K,
                     static_cast<const float*>(hd->feat), static_cast<const float*>(hd->dfeat), hd->wg_partial));
      break;
    default:
      return HLA_ERR_UNSUPPORTED;
  }
  return weight_grads_reduce(hd, static_cast<int>(nchunk), heads, 1.0f, 1.0f, 1.0f, 1.0f, s);
}

// ---- accumulate: partial Chat = sum over a chunk of tokens of T (x) yhat -----------------------
// YIO = true : yhat_j = [V_j | 1] read from the caller's V (I/O dtype, strided)
// YIO = false: yhat_i read from the dense fp32 scratch [th][d+1]
// grid (chunks, H), block 256.  Thread (r, c): column c, rows r + k*R with R = 256/d.
template <typename T, bool YIO>
__global__ void k_accumulate(Geom g, const BlockEnt* __restrict__ chunks,
                             const float* __restrict__ feat, bool query, View Y,
                             const float* __restrict__ ydense, float* __restrict__ partial,
                             int64_t state_stride) {
  extern __shared__ float smem[];
  const int d = g.d, D = g.D;
  const int R = kThreads / d;
  const int nrows = (D + R - 1) / R;
  const int Dpad = nrows * R;
  float* ts = smem;                    // [kAccTile][Dpad]
  float* ys = ts + kAccTile * Dpad;    // [kAccTile][d+1]
  float* fs = ys + kAccTile * (d + 1); // [kAccTile][nfeat]
  const BlockEnt e = chunks[blockIdx.x];
  const int h = blockIdx.y;
  const int tid = threadIdx.x;
  const int c = tid % d, r = tid / d;
  float acc[kMaxRows];
#pragma unroll
  for (int k = 0; k < kMaxRows; ++k) acc[k] = 0.0f;
  float zacc = 0.0f;
  for (int n0 = e.t0; n0 < e.t1; n0 += kAccTile) {
    const int nt = min(kAccTile, e.t1 - n0);
    __syncthreads();
    for (int idx = tid; idx < kAccTile * g.nfeat; idx += kThreads) {
      const int t = idx / g.nfeat;
      fs[idx] = t < nt ? feat[g.th(e.b, h, n0 + t) * g.nfeat + idx % g.nfeat] : 0.0f;
    }
    for (int idx = tid; idx < kAccTile * (d + 1); idx += kThreads) {
      const int t = idx / (d + 1), cc = idx % (d + 1);
      float y = 0.0f;
      if (t < nt) {
        if (YIO)
          y = cc < d ? to_float(Y.row<const T>(e.b, h, n0 + t)[cc]) : 1.0f;
        else
          y = ydense[g.th(e.b, h, n0 + t) * (d + 1) + cc];
      }
      ys[idx] = y;
    }
    __syncthreads();
    for (int idx = tid; idx < kAccTile * Dpad; idx += kThreads) {
      const int t = idx / Dpad, Di = idx % Dpad;
      ts[idx] = Di < D ? outer_entry(fs + t * g.nfeat, query, Di, g.F, g.dphi) : 0.0f;
    }
    __syncthreads();
    for (int t = 0; t < nt; ++t) {
      const float yv = ys[t * (d + 1) + c];
      const float* trow = ts + t * Dpad + r;
#pragma unroll
      for (int k = 0; k < kMaxRows; ++k)
        if (k < nrows) acc[k] += trow[k * R] * yv;
      if (tid < D) zacc += ts[t * Dpad + tid] * ys[t * (d + 1) + d];
    }
  }
  float* out = partial + (static_cast<int64_t>(blockIdx.x) * g.H + h) * state_stride;
#pragma unroll
  for (int k = 0; k < kMaxRows; ++k) {
    const int Di = r + k * R;
    if (k < nrows && Di < D) out[Di * (d + 1) + c] = acc[k];
  }
  if (tid < D) out[tid * (d + 1) + d] = zacc;
}

// Sum the partial states of each (sequence, head) in chunk order (deterministic).
// grid (num_seqs, H), block 256.
__global__ void k_reduce(Geom g, const int32_t* __restrict__ seq_chunk_off,
                         const float* __restrict__ partial, float* __restrict__ state,
                         int64_t state_stride, int count) {
  const int s = blockIdx.x, h = blockIdx.y;
  const int c0 = seq_chunk_off[s], c1 = seq_chunk_off[s + 1];
  float* out = state + (static_cast<int64_t>(s) * g.H + h) * state_stride;
  for (int i = threadIdx.x; i < count; i += blockDim.x) {
    float a = 0.0f;
    for (int ch = c0; ch < c1; ++ch) a += partial[(static_cast<int64_t>(ch) * g.H + h) * state_stride + i];
    out[i] = a;
  }
}

// ---- contract: out_i = T_i . M -----------------------------------------------------------------
// QUERY = true : T = T_q, M = Chat; writes O = num / (eta + eps) and den = eta + eps
// QUERY = false: T = T_k, M = dChat; writes dV = first d columns
// grid (tiles, H), block 256; tile = kTokPerThread * R tokens; thread (r, c) owns column c of
// tokens r + k*R.
template <typename T, bool QUERY>
__global__ void k_contract(Geom g, const BlockEnt* __restrict__ tiles,
                           const float* __restrict__ feat, const float* __restrict__ M,
                           int64_t state_stride, View Out, float* __restrict__ den) {
  extern __shared__ float smem[];
  const int d = g.d, D = g.D;
  const int R = kThreads / d;
  const int tile = kTokPerThread * R;
  float* ts = smem;             // [tile][D]
  float* fs = ts + tile * D;    // [tile][nfeat]
  float* etas = fs + tile * g.nfeat;  // [tile]
  const BlockEnt e = tiles[blockIdx.x];
  const int h = blockIdx.y;
  const int tid = threadIdx.x;
  const int c = tid % d, r = tid / d;
  const int nt = e.t1 - e.t0;
  const float* Mu = M + (static_cast<int64_t>(e.seq) * g.H + h) * state_stride;
  for (int idx = tid; idx < tile * g.nfeat; idx += kThreads) {
    const int t = idx / g.nfeat;
    fs[idx] = t < nt ? feat[g.th(e.b, h, e.t0 + t) * g.nfeat + idx % g.nfeat] : 0.0f;
  }
  __syncthreads();
  for (int idx = tid; idx < tile * D; idx += kThreads) {
    const int t = idx / D, Di = idx % D;
    ts[idx] = outer_entry(fs + t * g.nfeat, QUERY, Di, g.F, g.dphi);
  }
  __syncthreads();
  float acc[kTokPerThread];
#pragma unroll
  for (int k = 0; k < kTokPerThread; ++k) acc[k] = 0.0f;
  for (int Di = 0; Di < D; ++Di) {
    const float mv = Mu[Di * (d + 1) + c];
#pragma unroll
    for (int k = 0; k < kTokPerThread; ++k) acc[k] += ts[(k * R + r) * D + Di] * mv;
  }
  if (QUERY) {
    if (tid < tile) {
      float eta = 0.0f;
      for (int Di = 0; Di < D; ++Di) eta += ts[tid * D + Di] * Mu[Di * (d + 1) + d];
      etas[tid] = eta + g.eps;
      if (tid < nt) den[g.th(e.b, h, e.t0 + tid)] = eta + g.eps;
    }
    __syncthreads();
  }
#pragma unroll
  for (int k = 0; k < kTokPerThread; ++k) {
    const int t = k * R + r;
    if (t < nt) {
      const float o = QUERY ? acc[k] / etas[t] : acc[k];
      Out.row<T>(e.b, h, e.t0 + t)[c] = from_float<T>(o);
    }
  }
}

// ghat_i = [dO_i / den_i | -<dO_i, o_i> / den_i]   (one block row of d threads per token)
// grid (ceil(N/R), H, B), block 256.
template <typename T>
__global__ void k_backward_prep(Geom g, View dO, View O, const float* __restrict__ den,
                                float* __restrict__ yhat) {
  __shared__ float red[kThreads];
  const int d = g.d;
  const int R = kThreads / d;
  const int c = threadIdx.x % d, r = threadIdx.x / d;
  const int n = blockIdx.x * R + r, h = blockIdx.y, b = blockIdx.z;
  const bool live = n < g.N;
  float go = 0.0f, dn = 1.0f, dot = 0.0f;
  if (live) {
    dn = den[g.th(b, h, n)];
    go = to_float(dO.row<const T>(b, h, n)[c]);
    dot = go * to_float(O.row<const T>(b, h, n)[c]);
  }
  red[threadIdx.x] = dot;
  __syncthreads();
  for (int s = d / 2; s > 0; s >>= 1) {
    if (c < s) red[threadIdx.x] += red[threadIdx.x + s];
    __syncthreads();
  }
  if (live) {
    float* y = yhat + g.th(b, h, n) * (d + 1);
    y[c] = go / dn;
    if (c == 0) y[d] = -red[r * d] / dn;
  }
}

// Chain rule from dT [tile][D] (LDS) through the outer product to the feature gradients of the
// tile's tokens: the gradient of slot s, coordinate a, token t is the sum over the entries whose
// digit s equals a of dT[entry] times the product of the other slots' features.  QUERY: all F
// slots hold phi_q and their gradients are summed into dfeat[.., 0:dphi]; otherwise slot f goes
// to dfeat[.., (1+f)*dphi : ..].  Called by all threads of the block; fs = features [tile][nfeat].
template <bool QUERY>
__device__ __forceinline__ void slot_gradients(const Geom& g, const float* fs, const float* dts,
                                               int tile, int nt, int b, int h, int t0,
                                               float* __restrict__ dfeat) {
  const int D = g.D, dphi = g.dphi, F = g.F;
  const int nout = QUERY ? tile * dphi : tile * F * dphi;
  for (int idx = threadIdx.x; idx < nout; idx += blockDim.x) {
    int t, s_lo, s_hi, a;
    if (QUERY) {
      t = idx / dphi;
      a = idx % dphi;
      s_lo = 0;
      s_hi = F;
    } else {
      t = idx / (F * dphi);
      s_lo = (idx / dphi) % F;
      s_hi = s_lo + 1;
      a = idx % dphi;
    }
    if (t >= nt) continue;
    const float* frow = fs + t * g.nfeat;
    float grad = 0.0f;
    for (int s = s_lo; s < s_hi; ++s) {
      for (int Di = 0; Di < D; ++Di) {
        int rem = Di;
        float p = 1.0f;
        bool hit = false;
        for (int sl = F - 1; sl >= 0; --sl) {
          const int dig = rem % dphi;
          rem /= dphi;
          if (sl == s)
            hit = dig == a;
          else
            p *= frow[slot_offset(QUERY, sl, dphi) + dig];
        }
        if (hit) grad += dts[t * D + Di] * p;
      }
    }
    const int col = QUERY ? a : (1 + s_lo) * dphi + a;
    dfeat[g.fidx(g.th(b, h, t0 + t), col)] = grad;
  }
}

// ---- dtensor: dT_i = M yhat_i, then gradients of the outer-product slots -----------------------
// QUERY = true : M = Chat, yhat = ghat (dense scratch), slots all phi_q -> dfeat[.., 0:dphi] (summed)
// QUERY = false: M = dChat, yhat = [V | 1] (caller's V), slot f -> dfeat[.., (1+f)*dphi : ..]
// grid (tiles of kDtTile, H), block 256 (needs D <= 256).
template <typename T, bool QUERY>
__global__ void k_dtensor(Geom g, const BlockEnt* __restrict__ tiles,
                          const float* __restrict__ feat, const float* __restrict__ M,
                          int64_t state_stride, View Y, const float* __restrict__ ydense,
                          float* __restrict__ dfeat) {
  extern __shared__ float smem[];
  const int d = g.d, D = g.D;
  float* ys = smem;                       // [kDtTile][d+1]
  float* fs = ys + kDtTile * (d + 1);     // [kDtTile][nfeat]
  float* dts = fs + kDtTile * g.nfeat;    // [kDtTile][D]
  const BlockEnt e = tiles[blockIdx.x];
  const int h = blockIdx.y;
  const int tid = threadIdx.x;
  const int nt = e.t1 - e.t0;
  const float* Mu = M + (static_cast<int64_t>(e.seq) * g.H + h) * state_stride;
  for (int idx = tid; idx < kDtTile * g.nfeat; idx += kThreads) {
    const int t = idx / g.nfeat;
    fs[idx] = t < nt ? feat[g.th(e.b, h, e.t0 + t) * g.nfeat + idx % g.nfeat] : 0.0f;
  }
  for (int idx = tid; idx < kDtTile * (d + 1); idx += kThreads) {
    const int t = idx / (d + 1), cc = idx % (d + 1);
    float y = 0.0f;
    if (t < nt) {
      if (QUERY)
        y = ydense[g.th(e.b, h, e.t0 + t) * (d + 1) + cc];
      else
        y = cc < d ? to_float(Y.row<const T>(e.b, h, e.t0 + t)[cc]) : 1.0f;
    }
    ys[idx] = y;
  }
  __syncthreads();
  if (tid < D) {
    float dt[kDtTile];
#pragma unroll
    for (int t = 0; t < kDtTile; ++t) dt[t] = 0.0f;
    const float* mrow = Mu + tid * (d + 1);
    for (int cc = 0; cc <= d; ++cc) {
      const float mv = mrow[cc];
#pragma unroll
      for (int t = 0; t < kDtTile; ++t) dt[t] += mv * ys[t * (d + 1) + cc];
    }
#pragma unroll
    for (int t = 0; t < kDtTile; ++t) dts[t * D + tid] = dt[t];
  }
  __syncthreads();
  slot_gradients<QUERY>(g, fs, dts, kDtTile, nt, e.b, h, e.t0, dfeat);
}

// ---- causal variant (Sec. 4.4): one scan over the tokens of a (sequence, head) ------------------
// The sequential state update  Chat^i = decay Chat^{i-1} + T_k,i (x) vhat_i  (and, for the gradient
// of the key side, its mirror image from the back,  dChat^j = decay dChat^{j+1} + T_q,j (x) ghat_j)
// carried through the sequence by ONE workgroup, TT tokens at a time, with the running state in
// LDS.  With a = the tensor that builds the state and ya its augmented rows, b = the tensor that
// reads it and yb its rows, m_tj = decay^|t-j| on the visible side of the mask (j <= t going
// forward, j >= t going back) and c_t the decay of the carried state C as seen from token t:
//   out_t = c_t b_t . C  + sum_j m_tj <b_t, a_j> ya_j          (contract)
//   db_t  = c_t C yb_t   + sum_j m_tj <yb_t, ya_j> a_j         (dtensor, then the chain rule)
//   C    <- decay^TT C   + sum_j u_j a_j (x) ya_j              (u_j: decay from token j to the carry's reference)
// MODE 0: a = T_k, ya = vhat, b = T_q:            O = out[0:d] / (out[d] + eps), den
// MODE 1: same state, yb = ghat:                  d(phi_q) from db
// MODE 2: a = T_q, ya = ghat, b = T_k, yb = vhat, from the back:  dV = out[0:d], d(phi_k) from db
// grid (num_seqs, H), block 256.  Throughput is not a goal: this is the fp32 cross-check of the scan.
template <int TT>
__host__ __device__ constexpr size_t causal_scan_floats(int D, int d, int nfeat) {
  return static_cast<size_t>(D) * (d + 1) + 3 * static_cast<size_t>(TT) * D + 2 * static_cast<size_t>(TT) * (d + 1) +
         static_cast<size_t>(TT) * nfeat + 2 * TT * TT + 3 * TT;
}

template <typename T, int MODE, int TT>
__global__ __launch_bounds__(kThreads) void k_causal_scan(
    Geom g, const BlockEnt* __restrict__ chunks, const int32_t* __restrict__ seq_chunk_off,
    const float* __restrict__ feat, View V, const float* __restrict__ ghat, float decay, View Out,
    float* __restrict__ den, float* __restrict__ dfeat) {
  extern __shared__ float smem[];
  constexpr bool BACK = MODE == 2;
  const int d = g.d, D = g.D, d1 = g.d + 1;
  const int R = kThreads / d;
  float* C = smem;                 // [D][d+1] carried state
  float* A = C + D * d1;           // [TT][D]  state-building tensor
  float* Bt = A + TT * D;          // [TT][D]  reading tensor
  float* dts = Bt + TT * D;        // [TT][D]  db
  float* ya = dts + TT * D;        // [TT][d+1]
  float* yb = ya + TT * d1;        // [TT][d+1]
  float* fs = yb + TT * d1;        // [TT][nfeat]
  float* mp = fs + TT * g.nfeat;   // [TT][TT] m_tj <b_t, a_j>
  float* mw = mp + TT * TT;        // [TT][TT] m_tj <yb_t, ya_j>
  float* cf = mw + TT * TT;        // [TT] c_t
  float* uf = cf + TT;             // [TT] u_j
  float* etas = uf + TT;           // [TT]
  const int s = blockIdx.x, h = blockIdx.y;
  const int tid = threadIdx.x;
  const int c0 = seq_chunk_off[s], c1 = seq_chunk_off[s + 1];
  if (c0 == c1) return;  // empty sequence (uniform over the block)
  const int b = chunks[c0].b, lo = chunks[c0].t0, hi = chunks[c1 - 1].t1;
  const int ntiles = (hi - lo + TT - 1) / TT;
  for (int idx = tid; idx < D * d1; idx += kThreads) C[idx] = 0.0f;
  if (tid < TT) {
    // forward: C is the state at the last token before the tile; back: at the first token behind it
    cf[tid] = powf(decay, static_cast<float>(BACK ? TT - tid : tid + 1));
    uf[tid] = powf(decay, static_cast<float>(BACK ? tid : TT - 1 - tid));
  }
  const float tile_decay = powf(decay, static_cast<float>(TT));
  for (int ti = 0; ti < ntiles; ++ti) {
    const int t0 = lo + (BACK ? ntiles - 1 - ti : ti) * TT;
    const int nt = min(TT, hi - t0);
    __syncthreads();  // the previous tile's readers of fs, A, ya, dts are done; C is up to date
    for (int idx = tid; idx < TT * g.nfeat; idx += kThreads) {
      const int t = idx / g.nfeat;
      fs[idx] = t < nt ? feat[g.fidx(g.th(b, h, t0 + t), idx % g.nfeat)] : 0.0f;
    }
    for (int idx = tid; idx < TT * d1; idx += kThreads) {
      const int t = idx / d1, cc = idx % d1;
      float v = 0.0f, gh = 0.0f;  // rows of tokens beyond the sequence are zero, the 1 included
      if (t < nt) {
        v = cc < d ? to_float(V.row<const T>(b, h, t0 + t)[cc]) : 1.0f;
        if (MODE != 0) gh = ghat[g.th(b, h, t0 + t) * d1 + cc];
      }
      (BACK ? yb : ya)[idx] = v;
      if (MODE != 0) (BACK ? ya : yb)[idx] = gh;
    }
    __syncthreads();
    for (int idx = tid; idx < TT * D; idx += kThreads) {
      const int t = idx / D, Di = idx % D;
      const float tq = outer_entry(fs + t * g.nfeat, true, Di, g.F, g.dphi);
      const float tk = outer_entry(fs + t * g.nfeat, false, Di, g.F, g.dphi);
      A[idx] = BACK ? tq : tk;
      Bt[idx] = BACK ? tk : tq;
    }
    __syncthreads();
    for (int idx = tid; idx < (MODE == 0 ? 1 : 2) * TT * TT; idx += kThreads) {
      const int w = idx / (TT * TT), t = (idx / TT) % TT, j = idx % TT;
      const bool visible = BACK ? j >= t : j <= t;
      float acc = 0.0f;
      if (visible) {
        if (w == 0) {
          for (int Di = 0; Di < D; ++Di) acc += Bt[t * D + Di] * A[j * D + Di];
        } else {
          for (int cc = 0; cc < d1; ++cc) acc += yb[t * d1 + cc] * ya[j * d1 + cc];
        }
        acc *= powf(decay, static_cast<float>(BACK ? j - t : t - j));
      }
      (w == 0 ? mp : mw)[t * TT + j] = acc;
    }
    __syncthreads();
    // contract: thread (r, c) owns column c of tokens r, r + R, ..
    float out[TT];
    if (MODE != 1) {
      const int c = tid % d, r = tid / d;
#pragma unroll
      for (int k = 0; k < TT; ++k) {
        const int t = r + k * R;
        float acc = 0.0f;
        if (t < TT) {
          for (int Di = 0; Di < D; ++Di) acc += Bt[t * D + Di] * C[Di * d1 + c];
          acc *= cf[t];
          for (int j = 0; j < TT; ++j) acc += mp[t * TT + j] * ya[j * d1 + c];
        }
        out[k] = acc;
      }
      if (MODE == 0 && tid < TT) {
        float eta = 0.0f;
        for (int Di = 0; Di < D; ++Di) eta += Bt[tid * D + Di] * C[Di * d1 + d];
        eta *= cf[tid];
        for (int j = 0; j < TT; ++j) eta += mp[tid * TT + j] * ya[j * d1 + d];
        etas[tid] = eta + g.eps;
        if (tid < nt) den[g.th(b, h, t0 + tid)] = eta + g.eps;
      }
    }
    // dtensor: thread Di owns row Di of the state
    if (MODE != 0 && tid < D) {
      float dt[TT];
#pragma unroll
      for (int t = 0; t < TT; ++t) dt[t] = 0.0f;
      for (int cc = 0; cc < d1; ++cc) {
        const float cv = C[tid * d1 + cc];
#pragma unroll
        for (int t = 0; t < TT; ++t) dt[t] += cv * yb[t * d1 + cc];
      }
#pragma unroll
      for (int t = 0; t < TT; ++t) {
        float acc = dt[t] * cf[t];
        for (int j = 0; j < TT; ++j) acc += mw[t * TT + j] * A[j * D + tid];
        dts[t * D + tid] = acc;
      }
    }
    __syncthreads();  // every read of C is done; etas and dts are visible
    if (MODE != 1) {
      const int c = tid % d, r = tid / d;
#pragma unroll
      for (int k = 0; k < TT; ++k) {
        const int t = r + k * R;
        if (t < nt) Out.row<T>(b, h, t0 + t)[c] = from_float<T>(MODE == 0 ? out[k] / etas[t] : out[k]);
      }
    }
    if (MODE == 1) slot_gradients<true>(g, fs, dts, TT, nt, b, h, t0, dfeat);
    if (MODE == 2) slot_gradients<false>(g, fs, dts, TT, nt, b, h, t0, dfeat);
    for (int idx = tid; idx < D * d1; idx += kThreads) {
      const int Di = idx / d1, cc = idx % d1;
      float acc = C[idx] * tile_decay;
      for (int j = 0; j < TT; ++j) acc += uf[j] * A[j * D + Di] * ya[j * d1 + cc];
      C[idx] = acc;
    }
  }
}

template <typename T>
hla_status features_in_t(hla_handle* hd, const hla_call_args& a) {
  Geom g = hd->g;
  hipStream_t s = a.stream;
  const int d = g.d;
  if (hd->cfg.phi_mode == HLA_PHI_NONE) {
    const int64_t total = static_cast<int64_t>(g.B) * g.H * g.N;
    return launch(hd, "generic_feat_import", k_feat_import<T>, dim3((total + 255) / 256), dim3(256),
                  0, s, g, a.Q, a.K, hd->feat);
  }
  const size_t sh = 2 * kPhiTile * d * sizeof(float);
  return launch(hd, "generic_phi_forward", k_phi_forward<T>,
                dim3((g.N + kPhiTile - 1) / kPhiTile, g.H, g.B), dim3(d), sh, s, g, hd->phi, a.Q, a.K,
                hd->feat);
}

template <typename T>
hla_status features_out_t(hla_handle* hd, const hla_call_args& a) {
  Geom g = hd->g;
  hipStream_t s = a.stream;
  const int d = g.d;
  if (hd->cfg.phi_mode == HLA_PHI_NONE) {
    const int64_t total = static_cast<int64_t>(g.B) * g.H * g.N;
    return launch(hd, "generic_dfeat_export", k_dfeat_export<T>, dim3((total + 255) / 256), dim3(256),
                  0, s, g, hd->dfeat, a.dQ, a.dK);
  }
  const size_t sh = (2 * kPhiTile * d + kPhiTile * g.dphi) * sizeof(float);
  return launch(hd, "generic_phi_backward", k_phi_backward<T>,
                dim3((g.N + kPhiTile - 1) / kPhiTile, g.H, g.B), dim3(d), sh, s, g, hd->phi, a.Q, a.K,
                hd->feat, hd->dfeat, a.dQ, a.dK);
}

// The causal scan in one of its three modes; TT = 8 tokens per step where the LDS allows, else 4.
constexpr size_t kLdsLimit = 160 * 1024;
inline int causal_scan_tile(const Geom& g) {
  if (causal_scan_floats<8>(g.D, g.d, g.nfeat) * sizeof(float) <= kLdsLimit) return 8;
  if (causal_scan_floats<4>(g.D, g.d, g.nfeat) * sizeof(float) <= kLdsLimit) return 4;
  return 0;
}

template <typename T, int MODE, int TT>
hla_status causal_scan_launch(hla_handle* hd, const hla_call_args& a, const char* name, View out) {
  const Geom& g = hd->g;
  hla_token_table* chunks = nullptr;
  HLA_TRY(get_table(hd, 0, kChunk, a.stream, &chunks));
  const size_t sh = causal_scan_floats<TT>(g.D, g.d, g.nfeat) * sizeof(float);
  auto kernel = &k_causal_scan<T, MODE, TT>;
  const float dec = hd->cfg.decay > 0.0f && hd->cfg.decay < 1.0f ? hd->cfg.decay : 1.0f;
  return launch(hd, name, kernel, dim3(a.num_seqs, g.H), dim3(kThreads), sh, a.stream, g, chunks->dev,
                chunks->seq_off_dev, static_cast<const float*>(hd->feat), a.V,
                static_cast<const float*>(hd->yhat), dec, out, hd->den, hd->dfeat);
}

// The scan's LDS exceeds the 64 KB a kernel gets without asking: the three modes of a handle's
// dtype and tile are given their size once, when the handle is planned.
template <typename T, int TT>
hla_status causal_scan_allow_lds(const Geom& g) {
  const int sh = static_cast<int>(causal_scan_floats<TT>(g.D, g.d, g.nfeat) * sizeof(float));
  const void* kernels[3] = {reinterpret_cast<const void*>(&k_causal_scan<T, 0, TT>),
                            reinterpret_cast<const void*>(&k_causal_scan<T, 1, TT>),
                            reinterpret_cast<const void*>(&k_causal_scan<T, 2, TT>)};
  for (const void* k : kernels)
    if (hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, sh) != hipSuccess) return HLA_ERR_HIP;
  return HLA_OK;
}

template <typename T, int MODE>
hla_status causal_scan(hla_handle* hd, const hla_call_args& a, const char* name, View out) {
  switch (causal_scan_tile(hd->g)) {
    case 8: return causal_scan_launch<T, MODE, 8>(hd, a, name, out);
    case 4: return causal_scan_launch<T, MODE, 4>(hd, a, name, out);
    default: return HLA_ERR_UNSUPPORTED;
  }
}

template <typename T>
hla_status forward_t(hla_handle* hd, const hla_call_args& a) {
  Geom g = hd->g;
  hipStream_t s = a.stream;
  const int d = g.d;
  const int R = kThreads / d;
  HLA_TRY(features_in_t<T>(hd, a));
  if (hd->cfg.causal) return causal_scan<T, 0>(hd, a, "generic_causal_forward", a.O);
  hla_token_table *chunks = nullptr, *tiles = nullptr;
  HLA_TRY(get_table(hd, 0, kChunk, s, &chunks));
  HLA_TRY(get_table(hd, 1, kTokPerThread * R, s, &tiles));
  const int nrows = (g.D + R - 1) / R;
  const size_t sh_acc = (kAccTile * nrows * R + kAccTile * (d + 1) + kAccTile * g.nfeat) * sizeof(float);
  HLA_TRY(launch(hd, "generic_state_accumulate", k_accumulate<T, true>, dim3(chunks->count, g.H),
                 dim3(kThreads), sh_acc, s, g, chunks->dev, hd->feat, false, a.V,
                 static_cast<const float*>(nullptr), hd->partial, hd->state_stride));
  HLA_TRY(launch(hd, "generic_state_reduce", k_reduce, dim3(a.num_seqs, g.H), dim3(256), 0, s, g,
                 chunks->seq_off_dev, hd->partial, hd->state, hd->state_stride, g.D * (d + 1)));
  const int tile = kTokPerThread * R;
  const size_t sh_c = (static_cast<size_t>(tile) * g.D + tile * g.nfeat + tile) * sizeof(float);
  HLA_TRY(launch(hd, "generic_query_contract", k_contract<T, true>, dim3(tiles->count, g.H),
                 dim3(kThreads), sh_c, s, g, tiles->dev, hd->feat, hd->state, hd->state_stride, a.O,
                 hd->den));
  return HLA_OK;
}

template <typename T>
hla_status backward_t(hla_handle* hd, const hla_call_args& a) {
  Geom g = hd->g;
  hipStream_t s = a.stream;
  const int d = g.d;
  const int R = kThreads / d;
  hla_token_table *chunks = nullptr, *tiles = nullptr, *dtt = nullptr;
  HLA_TRY(get_table(hd, 0, kChunk, s, &chunks));
  HLA_TRY(get_table(hd, 1, kTokPerThread * R, s, &tiles));
  HLA_TRY(get_table(hd, 2, kDtTile, s, &dtt));
  HLA_TRY(launch(hd, "generic_backward_prep", k_backward_prep<T>, dim3((g.N + R - 1) / R, g.H, g.B),
                 dim3(kThreads), 0, s, g, a.dO, a.O, hd->den, hd->yhat));
  if (hd->cfg.causal) {
    // the same state recurrence once more for d(phi_q), its mirror image from the back for
    // d(phi_k) and dV
    HLA_TRY((causal_scan<T, 1>(hd, a, "generic_causal_dquery", a.dV)));
    HLA_TRY((causal_scan<T, 2>(hd, a, "generic_causal_dkey", a.dV)));
    return features_out_t<T>(hd, a);
  }
  const int nrows = (g.D + R - 1) / R;
  const size_t sh_acc = (kAccTile * nrows * R + kAccTile * (d + 1) + kAccTile * g.nfeat) * sizeof(float);
  HLA_TRY(launch(hd, "generic_dstate_accumulate", k_accumulate<T, false>, dim3(chunks->count, g.H),
                 dim3(kThreads), sh_acc, s, g, chunks->dev, hd->feat, true, a.V, hd->yhat, hd->partial,
                 hd->state_stride));
  HLA_TRY(launch(hd, "generic_dstate_reduce", k_reduce, dim3(a.num_seqs, g.H), dim3(256), 0, s, g,
                 chunks->seq_off_dev, hd->partial, hd->dstate, hd->state_stride, g.D * (d + 1)));
  const size_t sh_dt = (kDtTile * (d + 1) + kDtTile * g.nfeat + static_cast<size_t>(kDtTile) * g.D) * sizeof(float);
  HLA_TRY(launch(hd, "generic_dquery_features", k_dtensor<T, true>, dim3(dtt->count, g.H),
                 dim3(kThreads), sh_dt, s, g, dtt->dev, hd->feat, hd->state, hd->state_stride, a.V,
                 hd->yhat, hd->dfeat));
  HLA_TRY(launch(hd, "generic_dkey_features", k_dtensor<T, false>, dim3(dtt->count, g.H),
                 dim3(kThreads), sh_dt, s, g, dtt->dev, hd->feat, hd->dstate, hd->state_stride, a.V,
                 static_cast<const float*>(nullptr), hd->dfeat));
  const int tile = kTokPerThread * R;
  const size_t sh_c = (static_cast<size_t>(tile) * g.D + tile * g.nfeat + tile) * sizeof(float);
  HLA_TRY(launch(hd, "generic_dvalue_contract", k_contract<T, false>, dim3(tiles->count, g.H),
                 dim3(kThreads), sh_c, s, g, tiles->dev, hd->feat, hd->dstate, hd->state_stride, a.dV,
                 static_cast<float*>(nullptr)));
  return features_out_t<T>(hd, a);
}

}  // namespace

hla_status generic_workspace_plan(hla_handle* hd) {
  const Geom& g = hd->g;
  if (g.F > kMaxF || g.D > kThreads) return HLA_ERR_UNSUPPORTED;
  const int R = kThreads / g.d;
  if ((g.D + R - 1) / R > kMaxRows) return HLA_ERR_UNSUPPORTED;
  if (kPhiTile * g.dphi > 64 * 1024) return HLA_ERR_UNSUPPORTED;
  hd->state_stride = static_cast<int64_t>(g.D) * (g.d + 1);
  hd->max_chunks = (hd->cfg.max_tokens + kChunk - 1) / kChunk + hd->cfg.max_seqs;
  hd->yhat_floats = hd->max_th * (g.d + 1);
  hd->tables[0].min_block = kChunk;
  hd->tables[1].min_block = kTokPerThread * R;
  hd->tables[2].min_block = kDtTile;
  // shared-memory budgets (64 KiB static+dynamic without opting in)
  const size_t tile = kTokPerThread * R;
  const size_t sh_c = (tile * g.D + tile * g.nfeat + tile) * sizeof(float);
  if (sh_c > 64 * 1024) return HLA_ERR_UNSUPPORTED;
  if (hd->cfg.causal && causal_scan_tile(g) == 0) return HLA_ERR_UNSUPPORTED;  // the scan's state does not fit LDS
  return HLA_OK;
}

// Kernel attributes a handle on this path needs (once per handle, at creation).
hla_status generic_prepare_kernels(const hla_handle* hd) {
  if (!hd->cfg.causal) return HLA_OK;
  const Geom& g = hd->g;
  const bool f32 = hd->cfg.io_dtype == HLA_F32;
  switch (causal_scan_tile(g)) {
    case 8: return f32 ? causal_scan_allow_lds<float, 8>(g) : causal_scan_allow_lds<bf16_t, 8>(g);
    case 4: return f32 ? causal_scan_allow_lds<float, 4>(g) : causal_scan_allow_lds<bf16_t, 4>(g);
    default: return HLA_ERR_UNSUPPORTED;
  }
}

hla_status convert_weights_to_f32(hla_handle* hd, const hla_phi_weights* maps, hipStream_t s) {
  const Geom& g = hd->g;
  const int nm = 1 + g.F;
  bool shared = true;
  for (int m = 0; m < nm; ++m)
    shared = shared && maps[m].head_stride_W1 == 0 && maps[m].head_stride_b1 == 0 &&
             maps[m].head_stride_W2 == 0 && maps[m].head_stride_b2 == 0;
  const int hw = shared ? 1 : hd->cfg.max_heads;
  const int64_t nW1 = static_cast<int64_t>(g.d) * g.d, nb1 = g.d, nW2 = static_cast<int64_t>(g.d) * g.dphi,
                nb2 = g.dphi;
  float* W1 = hd->w_f32;
  float* b1 = W1 + nm * hw * nW1;
  float* W2 = b1 + nm * hw * nb1;
  float* b2 = W2 + nm * hw * nW2;
  hd->phi = PhiF32{W1, b1, W2, b2, hw};
  for (int m = 0; m < nm; ++m) {
    struct Item {
      const void* src;
      int64_t stride;
      float* dst;
      int64_t count;
    } items[4] = {{maps[m].W1, maps[m].head_stride_W1, W1 + m * hw * nW1, nW1},
                  {maps[m].b1, maps[m].head_stride_b1, b1 + m * hw * nb1, nb1},
                  {maps[m].W2, maps[m].head_stride_W2, W2 + m * hw * nW2, nW2},
                  {maps[m].b2, maps[m].head_stride_b2, b2 + m * hw * nb2, nb2}};
    for (const Item& it : items) {
      dim3 grid(static_cast<unsigned>((it.count + 255) / 256), hw);
      if (hd->cfg.io_dtype == HLA_F32)
        HLA_TRY(launch(hd, "convert_weights", k_convert_weights<float>, grid, dim3(256), 0, s,
                       static_cast<const float*>(it.src), it.stride, it.dst, static_cast<int>(it.count), hw));
      else
        HLA_TRY(launch(hd, "convert_weights", k_convert_weights<bf16_t>, grid, dim3(256), 0, s,
                       static_cast<const bf16_t*>(it.src), it.stride, it.dst, static_cast<int>(it.count), hw));
    }
  }
  return HLA_OK;
}

hla_status generic_set_weights(hla_handle*, hipStream_t) { return HLA_OK; }

hla_status weight_grads_reduce(hla_handle* hd, int nparts, int heads, float sW1, float sb1, float sW2,
                               float sb2, hipStream_t s) {
  const int nm = 1 + hd->g.F;
  WgradOut out{};
  for (int m = 0; m < nm; ++m) {
    out.dW1[m] = hd->wg_out[m].dW1;
    out.db1[m] = hd->wg_out[m].db1;
    out.dW2[m] = hd->wg_out[m].dW2;
    out.db2[m] = hd->wg_out[m].db2;
  }
  const int floats = static_cast<int>(hd->wg_part_floats);
  return launch(hd, "phi_weight_grads_reduce", k_wgrad_reduce, dim3((floats + 255) / 256, nm, heads),
                dim3(256), 0, s, hd->g.d, hd->g.dphi, nparts, static_cast<const float*>(hd->wg_partial), out,
                sW1, sb1, sW2, sb2);
}

hla_status phi_weight_grads(hla_handle* hd, const hla_call_args& a) {
  if (hd->path == HLA_PATH_MFMA && hd->cfg.io_dtype == HLA_BF16) return mfma_phi_weight_grads(hd, a);
  return hd->cfg.io_dtype == HLA_F32 ? weight_grads_t<float>(hd, a) : weight_grads_t<bf16_t>(hd, a);
}

// Features in (feature maps, or import of caller-provided features) and feature gradients out
// (through the maps, or exported as they are); shared with the MFMA path.
hla_status generic_features_in(hla_handle* hd, const hla_call_args& a) {
  return hd->cfg.io_dtype == HLA_F32 ? features_in_t<float>(hd, a) : features_in_t<bf16_t>(hd, a);
}
hla_status generic_features_out(hla_handle* hd, const hla_call_args& a) {
  return hd->cfg.io_dtype == HLA_F32 ? features_out_t<float>(hd, a) : features_out_t<bf16_t>(hd, a);
}

hla_status generic_forward(hla_handle* hd, const hla_call_args& a) {
  return hd->cfg.io_dtype == HLA_F32 ? forward_t<float>(hd, a) : forward_t<bf16_t>(hd, a);
}

hla_status generic_backward(hla_handle* hd, const hla_call_args& a) {
  return hd->cfg.io_dtype == HLA_F32 ? backward_t<float>(hd, a) : backward_t<bf16_t>(hd, a);
}

}  // namespace hla
