// Feature maps phi_q, phi_k1..3 (App. A.1: Linear d->d, GELU, Linear d->d_phi, ReLU) and their
// input gradients on the matrix cores.
//
// A token is an MFMA *column* (lane (r, gl): token r of a 32-token tile, half gl), so the two
// layers chain without any layout change:
//   hidden^T[d x 32] = W1^T X^T      A = W1^T read from one row-major copy of W1 in LDS with
//                                    transpose reads; B = the token's own input channels
//   u^T[d_phi x 32]  = W2^T g^T      B = GELU(hidden) packed straight from the accumulators
// and backward   dg^T = W2 du^T,  dh = dg * GELU'(hidden),  dx^T = W1 dh^T  (A = the same LDS copy
// of W1, plain reads).  The weights of a head stay resident in LDS for the workgroup's lifetime;
// each wave streams its own 32-token tiles, loading them from global memory in operand order.
#include "hla_handle.h"
#include "hla_mfma_common.h"

namespace hla {
namespace {

using namespace mf;

constexpr int kDP = 6;
// waves per workgroup of the query-map and key-map kernels
#ifndef HLA_PHI_WAVES_Q
#define HLA_PHI_WAVES_Q 8
#endif
#ifndef HLA_PHI_WAVES_K
#define HLA_PHI_WAVES_K 4
#endif

// ---- GELU on the vector ALU ------------------------------------------------------------------
// x * Phi(x) with Phi(x) - 1/2 = t * P(t^2), t = clamp(x, +-4)/4: degree-7 minimax fit of the
// normal CDF (|error| <= 2.2e-5 inside, 3.2e-5 beyond the clamp), i.e. |GELU error| <= 4.2e-4,
// an order of magnitude below the bf16 rounding the result receives anyway.
__device__ __forceinline__ float gelu_poly(float x) {
  const float t = __builtin_amdgcn_fmed3f(x, -4.0f, 4.0f) * 0.25f;
  const float u = t * t;
  float p = -1.697353482246399f;
  p = p * u + 8.16788387298584f;
  p = p * u + -17.20026397705078f;
  p = p * u + 21.146461486816406f;
  p = p * u + -17.173776626586914f;
  p = p * u + 9.896830558776855f;
  p = p * u + -4.23522424697876f;
  p = p * u + 1.5953900814056396f;
  return x * (t * p + 0.5f);
}
// d/dx [x Phi(x)] - 1/2 = t * R(t^2): degree-8 fit, |error| <= 5.5e-4.
__device__ __forceinline__ float gelu_grad_poly(float x) {
  const float t = __builtin_amdgcn_fmed3f(x, -4.0f, 4.0f) * 0.25f;
  const float u = t * t;
  float p = 16.82962989807129f;
  p = p * u + -88.24928283691406f;
  p = p * u + 203.22996520996094f;
  p = p * u + -272.4527282714844f;
  p = p * u + 237.85069274902344f;
  p = p * u + -142.80833435058594f;
  p = p * u + 59.85906982421875f;
  p = p * u + -16.94890022277832f;
  p = p * u + 3.1904382705688477f;
  return t * p + 0.5f;
}

// ---- packed weights of one (map, head) in global memory ---------------------------------------
template <int D>
struct Packed {
  static constexpr int kW1 = 0;                       // bf16 [D][D] row-major (row = input channel)
  static constexpr int kW2A = kW1 + D * D * 2;        // bf16 [D/16][64][8]: A operand of u^T = W2^T g^T
  static constexpr int kW2B = kW2A + D * 32 * 2;      // bf16 [D/32][64][8]: A operand of dg^T = W2 du^T
  static constexpr int kB1 = kW2B + D * 16 * 2;       // fp32 [D]
  static constexpr int kB2 = kB1 + D * 4;             // fp32 [8]
  static constexpr int kBytes = kB2 + 32;
};

// hidden unit that k-slot (ks2, gl, j) of the second-layer contraction stands for: the slots
// follow the accumulator layout of the first layer (register i = 8*half + j of row block rb).
__host__ __device__ inline int hidden_of_slot(int ks2, int gl, int j) {
  const int rb = ks2 / 2, half = ks2 % 2;
  return 32 * rb + 16 * half + 8 * (j / 4) + 4 * gl + j % 4;
}

template <int D>
__global__ void k_pack_phi(PhiF32 w, int dphi, unsigned char* __restrict__ out) {
  const int64_t mh = blockIdx.x;  // map * heads_w + head
  unsigned char* base = out + mh * Packed<D>::kBytes;
  const float* W1 = w.W1 + mh * D * D;
  const float* W2 = w.W2 + mh * D * dphi;
  uint16_t* w1 = reinterpret_cast<uint16_t*>(base + Packed<D>::kW1);
  uint16_t* w2a = reinterpret_cast<uint16_t*>(base + Packed<D>::kW2A);
  uint16_t* w2b = reinterpret_cast<uint16_t*>(base + Packed<D>::kW2B);
  float* b1 = reinterpret_cast<float*>(base + Packed<D>::kB1);
  float* b2 = reinterpret_cast<float*>(base + Packed<D>::kB2);
  for (int i = threadIdx.x; i < D * D; i += blockDim.x) w1[i] = f32_to_bf16_bits(W1[i]);
  for (int i = threadIdx.x; i < (D / 16) * 512; i += blockDim.x) {
    const int ks2 = i / 512, lane = (i / 8) % 64, j = i % 8;
    const int r = lane % 32, gl = lane / 32;
    const int n = hidden_of_slot(ks2, gl, j);
    w2a[i] = r < dphi ? f32_to_bf16_bits(W2[n * dphi + r]) : 0;
  }
  for (int i = threadIdx.x; i < (D / 32) * 512; i += blockDim.x) {
    const int rb = i / 512, lane = (i / 8) % 64, j = i % 8;
    const int r = lane % 32, gl = lane / 32;
    const int a = 8 * gl + j;
    w2b[i] = a < dphi ? f32_to_bf16_bits(W2[(32 * rb + r) * dphi + a]) : 0;
  }
  for (int i = threadIdx.x; i < D; i += blockDim.x) b1[i] = w.b1[mh * D + i];
  for (int i = threadIdx.x; i < 8; i += blockDim.x) b2[i] = i < dphi ? w.b2[mh * dphi + i] : 0.0f;
}

// ---- LDS layout ---------------------------------------------------------------------------------
// W1 is kept row-major with its 16-byte chunks XOR-swizzled by the row, so that both the
// transpose reads (4 consecutive rows, same columns) and the plain reads (32 consecutive rows,
// same columns) spread over the banks without padding.  LDS holds weights only: every lane loads
// its token's input channels straight from global memory in operand order.
template <int D>
struct PhiSmem {
  static constexpr int kChunks = D / 8;               // 16-byte chunks per W1 row
  static constexpr int kW1 = D * D * 2;
  static constexpr int kW2 = D * 32 * 2;              // room for W2A (forward) or W2B (backward, half used)
  static constexpr int kMap = kW1 + kW2 + D * 4 + 32;  // + b1 + b2
  static constexpr int total(int nmaps) { return nmaps * kMap; }
  __device__ static __forceinline__ int w1_off(int row, int col) {
    return row * (D * 2) + ((((col >> 3) ^ row) & (kChunks - 1)) << 4) + ((col & 7) << 1);
  }
};

// Copy one (map, head) block of packed weights into LDS (all threads of the workgroup).
template <int D, bool BACKWARD>
__device__ __forceinline__ void load_weights(unsigned char* dst, const unsigned char* src) {
  using SM = PhiSmem<D>;
  using PK = Packed<D>;
  const int nthreads = blockDim.x;
  for (int i = threadIdx.x; i < D * SM::kChunks; i += nthreads) {
    const int row = i / SM::kChunks, ch = i % SM::kChunks;
    *reinterpret_cast<u32x4*>(dst + SM::w1_off(row, ch * 8)) =
        *reinterpret_cast<const u32x4*>(src + PK::kW1 + i * 16);
  }
  const int w2_bytes = BACKWARD ? D * 16 * 2 : D * 32 * 2;
  const unsigned char* w2 = src + (BACKWARD ? PK::kW2B : PK::kW2A);
  for (int i = threadIdx.x; i < w2_bytes / 16; i += nthreads)
    *reinterpret_cast<u32x4*>(dst + SM::kW1 + i * 16) = *reinterpret_cast<const u32x4*>(w2 + i * 16);
  for (int i = threadIdx.x; i < D + 8; i += nthreads)
    *reinterpret_cast<float*>(dst + SM::kW1 + SM::kW2 + i * 4) =
        *reinterpret_cast<const float*>(src + PK::kB1 + i * 4);
}

// The lane's share of its token's input vector as B operands: k-slot (ks, gl, j) is channel
// 16 ks + 8 gl + j, i.e. one 16-byte piece per k-step.  Tokens at or beyond N read as zero.
template <int D>
__device__ __forceinline__ void load_x(const View& X, int b, int h, int n, int N, int gl,
                                       u32x4 (&x)[D / 16]) {
  if (n < N) {
    const bf16_t* row = X.row<const bf16_t>(b, h, n);
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) x[ks] = *reinterpret_cast<const u32x4*>(row + 16 * ks + 8 * gl);
  } else {
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) x[ks][0] = x[ks][1] = x[ks][2] = x[ks][3] = 0u;
  }
}

// hidden^T = b1 + W1^T X^T for one map: acc[rb][i] is hidden unit 32rb + d_row(i, gl) of token r.
template <int D>
__device__ __forceinline__ void first_layer(const unsigned char* wm, const u32x4 (&xb)[D / 16],
                                            int lane, f32x16 (&acc)[D / 32]) {
  using SM = PhiSmem<D>;
  const int gl = lane / 32, L = lane % 16, q = lane / 16;
  const float* b1 = reinterpret_cast<const float*>(wm + SM::kW1 + SM::kW2);
#pragma unroll
  for (int rb = 0; rb < D / 32; ++rb)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      const f32x4 bv = *reinterpret_cast<const f32x4*>(b1 + 32 * rb + 8 * q4 + 4 * gl);
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[rb][4 * q4 + e] = bv[e];
    }
  // A operands are fetched one k-step ahead of the MFMAs that consume them
  auto fetch = [&](int ks, u32x4(&a)[D / 32]) {
    const int krow = 16 * ks + 8 * gl + L / 4;  // input channel (row of W1) this lane addresses
#pragma unroll
    for (int rb = 0; rb < D / 32; ++rb) {
      const int col = 32 * rb + 16 * (q % 2) + 4 * (L % 4);
      const u32x2 lo = lds_read_tr16(wm + SM::w1_off(krow, col));
      const u32x2 hi = lds_read_tr16(wm + SM::w1_off(krow + 4, col));
      a[rb][0] = lo[0];
      a[rb][1] = lo[1];
      a[rb][2] = hi[0];
      a[rb][3] = hi[1];
    }
  };
  u32x4 a[2][D / 32];
  fetch(0, a[0]);
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) {
    if (ks + 1 < D / 16) fetch(ks + 1, a[(ks + 1) & 1]);
    __builtin_amdgcn_sched_barrier(0);  // keep the next step's LDS reads ahead of this step's MFMAs
#pragma unroll
    for (int rb = 0; rb < D / 32; ++rb) acc[rb] = mfma32(a[ks & 1][rb], xb[ks], acc[rb]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// ---- forward ------------------------------------------------------------------------------------
// grid (G, H, B), block WAVES*64.  Maps map0 .. map0+NMAPS-1 of the head are applied to X; the
// features go to the fp32 feature workspace.  Wave w of the grid serves 32-token tiles
// w, w + (total waves), ..; the next tile's inputs are loaded while the current one is computed.
template <int D, int NMAPS, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_phi_fwd(Geom g, View X,
                                                        const unsigned char* __restrict__ wpk,
                                                        int heads_w, int map0,
                                                        float* __restrict__ feat) {
  using SM = PhiSmem<D>;
  constexpr int NRB = D / 32, NKS = D / 16;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int r = lane % 32, gl = lane / 32;
  const int h = blockIdx.y, b = blockIdx.z;
  const int hw = heads_w == 1 ? 0 : h;
  for (int m = 0; m < NMAPS; ++m)  // packed blocks are ordered [map][head]
    load_weights<D, false>(smem + m * SM::kMap,
                           wpk + (static_cast<int64_t>(map0 + m) * heads_w + hw) * Packed<D>::kBytes);
  __syncthreads();
  const int ntiles = (g.N + 31) / 32;
  const int stride = gridDim.x * WAVES;
  int tile = blockIdx.x * WAVES + wave;
  u32x4 xb[NKS], xn[NKS];
  if (tile < ntiles) load_x<D>(X, b, h, tile * 32 + r, g.N, gl, xb);
  for (; tile < ntiles; tile += stride) {
    const int n = tile * 32 + r;
    const bool live = n < g.N;
    if (tile + stride < ntiles) load_x<D>(X, b, h, (tile + stride) * 32 + r, g.N, gl, xn);
#pragma unroll
    for (int m = 0; m < NMAPS; ++m) {
      const unsigned char* wm = smem + m * SM::kMap;
      f32x16 acc[NRB];
      first_layer<D>(wm, xb, lane, acc);
      f32x16 u;
#pragma unroll
      for (int i = 0; i < 16; ++i) u[i] = 0.0f;
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          u32x4 gb;
#pragma unroll
          for (int p = 0; p < 4; ++p)
            gb[p] = pack_bf16(gelu_poly(acc[rb][8 * half + 2 * p]), gelu_poly(acc[rb][8 * half + 2 * p + 1]));
          const u32x4 a2 = *reinterpret_cast<const u32x4*>(wm + SM::kW1 + ((2 * rb + half) * 64 + lane) * 16);
          u = mfma32(a2, gb, u);
        }
      // rows d_row(i, gl) < d_phi: lane gl=0 holds features 0..3, lane gl=1 features 4, 5
      if (live) {
        const float* b2 = reinterpret_cast<const float*>(wm + SM::kW1 + SM::kW2 + D * 4);
        float* f = feat + g.th(b, h, n) * g.nfeat + (map0 + m) * kDP + 4 * gl;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (4 * gl + i < kDP) f[i] = fmaxf(u[i] + b2[4 * gl + i], 0.0f);
      }
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) xb[ks] = xn[ks];
  }
}

// ---- backward -----------------------------------------------------------------------------------
// grid (G, H, B), block WAVES*64.  dX = sum over the NMAPS maps of W1 (GELU'(h) * (W2 du)), with
// du = d(feature) where the ReLU was open.  Hidden activations are recomputed.
template <int D, int NMAPS, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_phi_bwd(Geom g, View X,
                                                        const unsigned char* __restrict__ wpk,
                                                        int heads_w, int map0,
                                                        const float* __restrict__ feat,
                                                        const float* __restrict__ dfeat, View dX) {
  using SM = PhiSmem<D>;
  constexpr int NRB = D / 32, NKS = D / 16;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int r = lane % 32, gl = lane / 32;
  const int h = blockIdx.y, b = blockIdx.z;
  const int hw = heads_w == 1 ? 0 : h;
  for (int m = 0; m < NMAPS; ++m)
    load_weights<D, true>(smem + m * SM::kMap,
                          wpk + (static_cast<int64_t>(map0 + m) * heads_w + hw) * Packed<D>::kBytes);
  __syncthreads();
  const int ntiles = (g.N + 31) / 32;
  const int stride = gridDim.x * WAVES;
  int tile = blockIdx.x * WAVES + wave;
  u32x4 xb[NKS], xn[NKS];
  if (tile < ntiles) load_x<D>(X, b, h, tile * 32 + r, g.N, gl, xb);
  for (; tile < ntiles; tile += stride) {
    const int n = tile * 32 + r;
    const bool live = n < g.N;
    if (tile + stride < ntiles) load_x<D>(X, b, h, (tile + stride) * 32 + r, g.N, gl, xn);
    // du^T as B operand of one 16-slot step: slot (gl, j) is feature 8gl + j (only gl = 0 is used)
    u32x4 dub[NMAPS];
#pragma unroll
    for (int m = 0; m < NMAPS; ++m) {
      dub[m][0] = dub[m][1] = dub[m][2] = dub[m][3] = 0u;
      if (live && gl == 0) {
        const int64_t o = g.th(b, h, n) * g.nfeat + (map0 + m) * kDP;
        float du[8];
#pragma unroll
        for (int a = 0; a < 8; ++a)
          du[a] = (a < kDP && feat[o + (a < kDP ? a : 0)] > 0.0f) ? dfeat[o + (a < kDP ? a : 0)] : 0.0f;
#pragma unroll
        for (int p = 0; p < 4; ++p) dub[m][p] = pack_bf16(du[2 * p], du[2 * p + 1]);
      }
    }
    f32x16 dx[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) dx[rb][i] = 0.0f;
#pragma unroll
    for (int m = 0; m < NMAPS; ++m) {
      const unsigned char* wm = smem + m * SM::kMap;
      f32x16 acc[NRB];
      first_layer<D>(wm, xb, lane, acc);
      u32x4 dhb[NKS];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        f32x16 dg;
#pragma unroll
        for (int i = 0; i < 16; ++i) dg[i] = 0.0f;
        const u32x4 a2 = *reinterpret_cast<const u32x4*>(wm + SM::kW1 + (rb * 64 + lane) * 16);
        dg = mfma32(a2, dub[m], dg);
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const int i = 8 * half + 2 * p;
            dhb[2 * rb + half][p] = pack_bf16(dg[i] * gelu_grad_poly(acc[rb][i]),
                                              dg[i + 1] * gelu_grad_poly(acc[rb][i + 1]));
          }
      }
      // dx^T[in x tok] += W1[in x hidden] dh^T: A rows = input channels, plain reads of the W1 copy
      auto fetch = [&](int ks2, u32x4(&a)[NRB]) {
        const int ncol = 32 * (ks2 / 2) + 16 * (ks2 % 2) + 4 * gl;  // hidden units ncol..+3 and ncol+8..+11
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
          const int row = 32 * rb + r;
          const u32x2 lo = *reinterpret_cast<const u32x2*>(wm + SM::w1_off(row, ncol));
          const u32x2 hi = *reinterpret_cast<const u32x2*>(wm + SM::w1_off(row, ncol + 8));
          a[rb][0] = lo[0];
          a[rb][1] = lo[1];
          a[rb][2] = hi[0];
          a[rb][3] = hi[1];
        }
      };
      u32x4 aw[2][NRB];
      fetch(0, aw[0]);
#pragma unroll
      for (int ks2 = 0; ks2 < NKS; ++ks2) {
        if (ks2 + 1 < NKS) fetch(ks2 + 1, aw[(ks2 + 1) & 1]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) dx[rb] = mfma32(aw[ks2 & 1][rb], dhb[ks2], dx[rb]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (live) {
      bf16_t* orow = dX.row<bf16_t>(b, h, n);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(dx[rb][4 * q4], dx[rb][4 * q4 + 1]);
          w[1] = pack_bf16(dx[rb][4 * q4 + 2], dx[rb][4 * q4 + 3]);
          *reinterpret_cast<u32x2*>(orow + 32 * rb + 8 * q4 + 4 * gl) = w;
        }
    }
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) xb[ks] = xn[ks];
  }
}

template <typename K>
hla_status allow_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
             ? HLA_OK
             : HLA_ERR_HIP;
}

int grid_x(const Geom& g, int waves) {
  // about one workgroup per compute unit in total, at least one per (batch row, head)
  const int units = g.B * g.H;
  const int tiles = (g.N + 32 * waves - 1) / (32 * waves);
  int gx = 256 / units;  // rounding down keeps the whole grid resident in one round
  if (gx > tiles) gx = tiles;
  return gx < 1 ? 1 : gx;
}

constexpr int kWavesQ = HLA_PHI_WAVES_Q, kWavesK = HLA_PHI_WAVES_K;

template <int D>
hla_status forward_t(hla_handle* hd, const hla_call_args& a) {
  using SM = PhiSmem<D>;
  Geom g = hd->g;
  const unsigned char* wpk = static_cast<const unsigned char*>(hd->path_ws) + hd->w_packed_off;
  static bool attr = false;
  if (!attr) {
    HLA_TRY(allow_lds(&k_phi_fwd<D, 1, kWavesQ>, SM::total(1)));
    HLA_TRY(allow_lds(&k_phi_fwd<D, 3, kWavesK>, SM::total(3)));
    attr = true;
  }
  HLA_TRY(launch(hd, "mfma_phi_forward_q", k_phi_fwd<D, 1, kWavesQ>, dim3(grid_x(g, kWavesQ), g.H, g.B),
                 dim3(kWavesQ * 64), SM::total(1), a.stream, g, a.Q, wpk, hd->phi.heads_w, 0, hd->feat));
  HLA_TRY(launch(hd, "mfma_phi_forward_k", k_phi_fwd<D, 3, kWavesK>, dim3(grid_x(g, kWavesK), g.H, g.B),
                 dim3(kWavesK * 64), SM::total(3), a.stream, g, a.K, wpk, hd->phi.heads_w, 1, hd->feat));
  return HLA_OK;
}

template <int D>
hla_status backward_t(hla_handle* hd, const hla_call_args& a) {
  using SM = PhiSmem<D>;
  Geom g = hd->g;
  const unsigned char* wpk = static_cast<const unsigned char*>(hd->path_ws) + hd->w_packed_off;
  static bool attr = false;
  if (!attr) {
    HLA_TRY(allow_lds(&k_phi_bwd<D, 1, kWavesQ>, SM::total(1)));
    HLA_TRY(allow_lds(&k_phi_bwd<D, 3, kWavesK>, SM::total(3)));
    attr = true;
  }
  HLA_TRY(launch(hd, "mfma_phi_backward_q", k_phi_bwd<D, 1, kWavesQ>, dim3(grid_x(g, kWavesQ), g.H, g.B),
                 dim3(kWavesQ * 64), SM::total(1), a.stream, g, a.Q, wpk, hd->phi.heads_w, 0, hd->feat,
                 hd->dfeat, a.dQ));
  HLA_TRY(launch(hd, "mfma_phi_backward_k", k_phi_bwd<D, 3, kWavesK>, dim3(grid_x(g, kWavesK), g.H, g.B),
                 dim3(kWavesK * 64), SM::total(3), a.stream, g, a.K, wpk, hd->phi.heads_w, 1, hd->feat,
                 hd->dfeat, a.dK));
  return HLA_OK;
}

}  // namespace

size_t mfma_phi_packed_bytes(const hla_handle* hd) {
  const size_t per = hd->g.d == 128 ? Packed<128>::kBytes : Packed<64>::kBytes;
  return per * (1 + hd->g.F) * hd->cfg.max_heads;
}

hla_status mfma_phi_set_weights(hla_handle* hd, hipStream_t s) {
  unsigned char* wpk = static_cast<unsigned char*>(hd->path_ws) + hd->w_packed_off;
  const int blocks = (1 + hd->g.F) * hd->phi.heads_w;
  if (hd->g.d == 128)
    return launch(hd, "mfma_pack_phi", k_pack_phi<128>, dim3(blocks), dim3(256), 0, s, hd->phi, hd->g.dphi, wpk);
  return launch(hd, "mfma_pack_phi", k_pack_phi<64>, dim3(blocks), dim3(256), 0, s, hd->phi, hd->g.dphi, wpk);
}

hla_status mfma_phi_forward(hla_handle* hd, const hla_call_args& a) {
  return hd->g.d == 128 ? forward_t<128>(hd, a) : forward_t<64>(hd, a);
}

hla_status mfma_phi_backward(hla_handle* hd, const hla_call_args& a) {
  return hd->g.d == 128 ? backward_t<128>(hd, a) : backward_t<64>(hd, a);
}

}  // namespace hla
