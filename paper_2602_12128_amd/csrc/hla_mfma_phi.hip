// Feature maps phi_q, phi_k1..3 (App. A.1: Linear d->d, GELU, Linear d->d_phi, ReLU) and their
// input gradients on the matrix cores.
//
// A token is an MFMA *column* (lane (r, gl): token r of a 32-token tile, half gl), so the two
// layers chain without any layout change:
//   hidden^T[d x 32] = W1^T X^T      A = rows of W1^T read from LDS with plain 16-byte reads;
//                                    B = the token's own input channels, loaded from global
//                                    memory in operand order
//   u^T[d_phi x 32]  = W2^T g^T      B = GELU(hidden) packed straight from the accumulators
// and backward   dg^T = W2 du^T,  dh = dg * GELU'(hidden),  dx^T = W1 dh^T  (A = the same LDS copy
// of W1^T, transpose reads).  The weights of a head stay resident in LDS while the workgroup
// works through its tiles (first the query map's, then the key maps'); each wave streams its own
// 32-token tiles, and two (backward) or three (forward) waves
// share a SIMD so that one wave's GELU arithmetic overlaps the others' matrix and LDS work.
#include "hla_handle.h"
#include "hla_mfma_common.h"
#include "hla_mfma_gelu.h"

namespace hla {
namespace {

using namespace mf;

struct TrueTag {
  static constexpr bool value = true;
};
struct FalseTag {
  static constexpr bool value = false;
};


// ---- packed weights of one (map, head) in global memory ---------------------------------------
template <int D>
struct Packed {
  static constexpr int kW1T = 0;                      // bf16 [D][D]: row = hidden unit, col = input channel; times 1/4
  static constexpr int kW2A = kW1T + D * D * 2;       // fp16 [D/16][64][8]: A operand of u^T = W2^T g^T; times 4
  static constexpr int kW2B = kW2A + D * 32 * 2;      // bf16 [D/32][64][8]: A operand of dg^T = W2 du^T; times 4
  static constexpr int kB1 = kW2B + D * 16 * 2;       // fp32 [D]; times 1/4
  static constexpr int kB2 = kB1 + D * 4;             // fp32 [16]
  static constexpr int kBytes = kB2 + 64;
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
  uint16_t* w1t = reinterpret_cast<uint16_t*>(base + Packed<D>::kW1T);
  uint16_t* w2a = reinterpret_cast<uint16_t*>(base + Packed<D>::kW2A);
  uint16_t* w2b = reinterpret_cast<uint16_t*>(base + Packed<D>::kW2B);
  float* b1 = reinterpret_cast<float*>(base + Packed<D>::kB1);
  float* b2 = reinterpret_cast<float*>(base + Packed<D>::kB2);
  for (int i = threadIdx.x; i < D * D; i += blockDim.x) {
    const int hid = i / D, in = i % D;
    w1t[i] = f32_to_bf16_bits(kHiddenScale * W1[in * D + hid]);
  }
  for (int i = threadIdx.x; i < (D / 16) * 512; i += blockDim.x) {
    const int ks2 = i / 512, lane = (i / 8) % 64, j = i % 8;
    const int r = lane % 32, gl = lane / 32;
    const int n = hidden_of_slot(ks2, gl, j);
    w2a[i] = r < dphi ? __builtin_bit_cast(uint16_t, static_cast<_Float16>(W2[n * dphi + r] / kHiddenScale)) : 0;
  }
  for (int i = threadIdx.x; i < (D / 32) * 512; i += blockDim.x) {
    const int rb = i / 512, lane = (i / 8) % 64, j = i % 8;
    const int r = lane % 32, gl = lane / 32;
    const int a = 8 * gl + j;
    w2b[i] = a < dphi ? f32_to_bf16_bits(W2[(32 * rb + r) * dphi + a] / kHiddenScale) : 0;
  }
  for (int i = threadIdx.x; i < D; i += blockDim.x) b1[i] = kHiddenScale * w.b1[mh * D + i];
  for (int i = threadIdx.x; i < 16; i += blockDim.x) b2[i] = i < dphi ? w.b2[mh * dphi + i] : 0.0f;
}

// ---- LDS layout ---------------------------------------------------------------------------------
// W1^T is kept row-major (row = hidden unit) with the 16-byte chunks of a row XOR-swizzled by a
// function of the row chosen so that both access patterns spread over all banks without padding:
//   plain 16-byte reads of 16 consecutive rows at one chunk (first-layer A operand), and
//   transpose reads of 4 consecutive rows x 4 consecutive chunks (A operand of dx^T = W1 dh^T).
template <int D, bool BACKWARD = false>
struct PhiSmem {
  static constexpr int kChunks = D / 8;               // 16-byte chunks per row
  static constexpr int kRow = D * 2;                  // bytes per row
  static constexpr int kW1 = D * D * 2;
  static constexpr int kW2 = BACKWARD ? D * 16 * 2 : D * 32 * 2;  // W2B (backward) or W2A (forward)
  static constexpr int kMap = kW1 + kW2 + D * 4 + 64;  // then b1 [D] and b2 [16] in fp32
  // backward adds a 16-row transpose tile per wave for whole-row stores of dX
  static constexpr int total(int nmaps, int waves) {
    return nmaps * kMap + (BACKWARD ? waves * RowTile<D, 16>::kBytes : 0);
  }
  __host__ __device__ static __forceinline__ int swz(int row) {
    return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
  }
  __device__ static __forceinline__ int off(int row, int chunk) {
    return row * kRow + (((chunk ^ swz(row)) & (kChunks - 1)) << 4);
  }
};

// Copy the packed weights of NMAPS (map, head) blocks into LDS (all THREADS threads of the
// workgroup).  All global loads of a map are issued before the first LDS store so that they are
// in flight together: the copy costs one memory round trip per map instead of one per 16 bytes.
template <int D, bool BACKWARD, int THREADS>
__device__ __forceinline__ void load_weights(unsigned char* dst, const unsigned char* src) {
  using SM = PhiSmem<D, BACKWARD>;
  using PK = Packed<D>;
  constexpr int N1 = D * SM::kChunks;                              // 16-byte chunks of W1^T
  constexpr int N2 = (BACKWARD ? D * 16 * 2 : D * 32 * 2) / 16;    // 16-byte chunks of the W2 image
  constexpr int NB = D + 16;                                       // floats of b1 and b2
  constexpr int I1 = (N1 + THREADS - 1) / THREADS, I2 = (N2 + THREADS - 1) / THREADS;
  const unsigned char* w2 = src + (BACKWARD ? PK::kW2B : PK::kW2A);
  const int t = threadIdx.x;
  u32x4 v1[I1], v2[I2];
  float vb = 0.0f;
#pragma unroll
  for (int k = 0; k < I1; ++k)
    if (N1 % THREADS == 0 || t + k * THREADS < N1) v1[k] = *reinterpret_cast<const u32x4*>(src + PK::kW1T + (t + k * THREADS) * 16);
#pragma unroll
  for (int k = 0; k < I2; ++k)
    if (N2 % THREADS == 0 || t + k * THREADS < N2) v2[k] = *reinterpret_cast<const u32x4*>(w2 + (t + k * THREADS) * 16);
  if (t < NB) vb = *reinterpret_cast<const float*>(src + PK::kB1 + t * 4);
#pragma unroll
  for (int k = 0; k < I1; ++k) {
    const int i = t + k * THREADS;
    if (N1 % THREADS == 0 || i < N1) *reinterpret_cast<u32x4*>(dst + SM::off(i / SM::kChunks, i % SM::kChunks)) = v1[k];
  }
#pragma unroll
  for (int k = 0; k < I2; ++k) {
    const int i = t + k * THREADS;
    if (N2 % THREADS == 0 || i < N2) *reinterpret_cast<u32x4*>(dst + SM::kW1 + i * 16) = v2[k];
  }
  if (t < NB) *reinterpret_cast<float*>(dst + SM::kW1 + SM::kW2 + t * 4) = vb;
}

// The lane's share of its token's input vector as B operands: k-slot (ks, gl, j) is channel
// 16 ks + 8 gl + j, i.e. one 16-byte piece per k-step.  Tokens at or beyond N read the last row
// (a token is an MFMA column, so what such a lane computes never reaches another token and is
// not stored).  The loads are unconditional: the same number of loads is in flight on every
// path, which lets the wait counters keep a prefetch in flight across the loop back-edge.
template <int D>
__device__ __forceinline__ void load_x(const View& X, int b, int h, int n, int N, int gl,
                                       u32x4 (&x)[D / 16]) {
  const bf16_t* row = X.row<const bf16_t>(b, h, n < N ? n : N - 1);
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) x[ks] = *reinterpret_cast<const u32x4*>(row + 16 * ks + 8 * gl);
}

// Per-lane byte offsets (inside a map's W1^T block, row block 0) of the first-layer A operand of
// each k-step: row r, chunk 2 ks + gl.  Row blocks add the compile-time constant 32 rows.
template <int D>
__device__ __forceinline__ void first_layer_offsets(int lane, int (&a_off)[D / 16]) {
  using SM = PhiSmem<D>;
  const int r = lane % 32, gl = lane / 32;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) a_off[ks] = SM::off(r, 2 * ks + gl);
}

// Which (batch row, head, first token) a 32-token tile index stands for.  With weights shared by
// all heads the tiles of every (batch row, head) form one flat list that is dealt out evenly to
// all waves of the grid; with per-head weights a workgroup stays on the head of blockIdx.y/z.
struct TileMap {
  int tiles_per_row;  // ceil(N / 32)
  int total;          // tiles this workgroup's list holds
  int H;
  bool flat;
  __device__ __forceinline__ void decode(int t, int& b, int& h, int& n0) const {
    if (flat) {
      const int row = t / tiles_per_row;
      b = row / H;
      h = row % H;
      n0 = (t % tiles_per_row) * 32;
    } else {
      b = blockIdx.z;
      h = blockIdx.y;
      n0 = t * 32;
    }
  }
};
__device__ __forceinline__ TileMap make_tile_map(const Geom& g, int heads_w) {
  TileMap tm;
  tm.tiles_per_row = (g.N + 31) / 32;
  tm.flat = heads_w == 1;
  tm.total = tm.flat ? tm.tiles_per_row * g.B * g.H : tm.tiles_per_row;
  tm.H = g.H;
  return tm;
}

// ---- forward ------------------------------------------------------------------------------------
// block WAVES*64.  Maps map0 .. map0+NMAPS-1 are applied to X; the features go to the fp32
// feature workspace.  Wave w of the grid serves 32-token tiles w, w + (total waves), ..; the next
// tile's inputs are loaded while the current one is computed.
template <int D, int NMAPS, int WAVES, int DPH>
__device__ __forceinline__ void phi_fwd_body(const Geom& g, const View& X,
                                             const unsigned char* __restrict__ wpk, int heads_w,
                                             int map0, int nmaps, float* __restrict__ feat) {
  using SM = PhiSmem<D>;
  constexpr int NRB = D / 32, NKS = D / 16;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  const int r = lane % 32, gl = lane / 32;
  const TileMap tm = make_tile_map(g, heads_w);
  const int hw = heads_w == 1 ? 0 : blockIdx.y;
  for (int m = 0; m < NMAPS; ++m)  // packed blocks are ordered [map][head]
    load_weights<D, false, WAVES * 64>(smem + m * SM::kMap,
                           wpk + (static_cast<int64_t>(map0 + m) * heads_w + hw) * Packed<D>::kBytes);
  __syncthreads();
  int a_off[NKS];
  first_layer_offsets<D>(lane, a_off);
  const int stride = gridDim.x * WAVES;
  int tile = blockIdx.x * WAVES + wave;
  int b = 0, h = 0, n0 = 0;
  // The tile's inputs live in xb only: the next tile's loads are issued into xb as soon as the
  // last first-layer MFMA of the current tile has read it (one and a half stages before the end).
  // The kernel is kept lean in registers (168) so that three waves share a SIMD.
  u32x4 xb[NKS];
  if (tile < tm.total) {
    tm.decode(tile, b, h, n0);
    load_x<D>(X, b, h, n0 + r, g.N, gl, xb);
  }
  // features of the last finished map, not yet stored: accumulator register i of the second layer
  // is feature d_row(i, gl) = 8 (i/4) + 4 gl + i%4; the registers with a feature below d_phi on
  // either lane half are kept
  constexpr int NU = DPH > 8 ? 8 : 4;
  static_assert(DPH <= 16, "one 16-row group of second-layer outputs");
  float pend[NU];
#pragma unroll
  for (int i = 0; i < NU; ++i) pend[i] = 0.0f;
  float* pend_ptr = nullptr;  // feature 4 gl of the token
  auto flush = [&]() {  // a pair of features of 32 consecutive tokens is one contiguous 256-byte run
    if (pend_ptr != nullptr) {
      f32x2* pp = reinterpret_cast<f32x2*>(pend_ptr);
#pragma unroll
      for (int i = 0; i < NU; i += 2) {
        const int a0 = 8 * (i / 4) + i % 4;  // even feature held by lane half 0; half 1 holds a0 + 4
        f32x2 v;
        v[0] = pend[i];
        v[1] = pend[i + 1];
        if (a0 + 4 < DPH) {
          pp[32 * (a0 / 2)] = v;
        } else if (a0 < DPH) {
          if (gl == 0) pp[32 * (a0 / 2)] = v;
        }
      }
    }
    pend_ptr = nullptr;
  };
  // the first layer accumulates on top of its bias: the lane's 16 entries of a 32-row block
  auto bias_acc = [&](const unsigned char* wmap, int rb) {
    f32x16 z;
    const float* b1 = reinterpret_cast<const float*>(wmap + SM::kW1 + SM::kW2) + 32 * rb + 4 * gl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {  // registers 4i..4i+3 are hidden units 32 rb + 8 i + 4 gl + 0..3
      const f32x4 v = *reinterpret_cast<const f32x4*>(b1 + 8 * i);
      z[4 * i] = v[0];
      z[4 * i + 1] = v[1];
      z[4 * i + 2] = v[2];
      z[4 * i + 3] = v[3];
    }
    return z;
  };
  for (; tile < tm.total; tile += stride) {
    const int n = n0 + r;
    const bool live = n < g.N;
    const int64_t th = g.th(b, h, live ? n : 0);
    const bool more_tiles = tile + stride < tm.total;
    if (more_tiles) tm.decode(tile + stride, b, h, n0);  // b, h, n0 now name the next tile
    // Software pipeline over 32-row blocks of the hidden layer (block t = m * NRB + rb): while the
    // vector ALU evaluates GELU on block t, the matrix pipe works on block t + 1, two MFMAs
    // between quarters of the vector work, their LDS operands read one quarter ahead.  Blocks
    // past the last map alias the last map's LDS: their results are never used.
    // hidden blocks alternate between two accumulator sets (NRB is even, so block 0 of every map
    // lands in set 0): no copy from "next" to "current" at the end of a stage
    static_assert(NRB % 2 == 0, "two alternating accumulator sets");
    f32x16 hb[2];
    constexpr int kPer = NKS / 4;  // first-layer MFMAs per slice
    u32x4 an[kPer];                // their A operands, read one slice ahead
    {
      u32x4 a0[NKS];
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) a0[ks] = *reinterpret_cast<const u32x4*>(smem + a_off[ks]);
      hb[0] = bias_acc(smem, 0);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) hb[0] = mfma32(a0[ks], xb[ks], hb[0]);
#pragma unroll
      for (int t = 0; t < kPer; ++t)
        an[t] = *reinterpret_cast<const u32x4*>(smem + (1 % NRB) * 32 * SM::kRow + a_off[t]);
    }
    flush();
#pragma unroll 1
    for (int m = 0; m < nmaps; ++m) {  // nmaps == NMAPS, passed at run time so this stays a loop
      const unsigned char* wm = smem + m * SM::kMap;
      const bool last_map = m + 1 == nmaps;
      f32x16 u;
#pragma unroll
      for (int i = 0; i < 16; ++i) u[i] = 0.0f;
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        // block t+1 (first layer, this stage) and block t+2 (whose first operands the last slice reads)
        const unsigned char* w1 = rb + 1 < NRB ? wm : (last_map ? wm : wm + SM::kMap);
        const unsigned char* w2 = rb + 2 < NRB ? wm : (last_map ? wm : wm + SM::kMap);
        const unsigned char* a1_base = w1 + ((rb + 1) % NRB) * 32 * SM::kRow;
        const unsigned char* a2_base = w2 + ((rb + 2) % NRB) * 32 * SM::kRow;
        f32x16& cur = hb[rb % 2];
        f32x16& nxt = hb[(rb + 1) % 2];
        nxt = bias_acc(w1, (rb + 1) % NRB);
        const u32x4 a20 = *reinterpret_cast<const u32x4*>(wm + SM::kW1 + ((2 * rb) * 64 + lane) * 16);
        const u32x4 a21 = *reinterpret_cast<const u32x4*>(wm + SM::kW1 + ((2 * rb + 1) * 64 + lane) * 16);
        u32x4 gb[2];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          // the empty asm statements pin the order MFMAs -> GELU slice -> next MFMAs: they are
          // volatile (kept in program order) and the values flow through them
          asm volatile("" : "+v"(nxt));
          // first layer of block t+1 (there is none after the last block, and xb already belongs
          // to the next tile's loads by then)
          if (rb + 1 < NRB || !last_map) {
#pragma unroll
            for (int t = 0; t < kPer; ++t) {
              nxt = mfma32(an[t], xb[j * kPer + t], nxt);
              an[t] = j < 3 ? *reinterpret_cast<const u32x4*>(a1_base + a_off[(j + 1) * kPer + t])
                            : *reinterpret_cast<const u32x4*>(a2_base + a_off[t]);
            }
          }
          if (j == 3) u = mfma32_f16(a20, gb[0], u);
          // the next tile's inputs: xb is free once the last first-layer MFMA has been issued
          if (last_map && rb == NRB - 2 && j == 3 && more_tiles) load_x<D>(X, b, h, n0 + r, g.N, gl, xb);
          const float in[4] = {cur[4 * j], cur[4 * j + 1], cur[4 * j + 2], cur[4 * j + 3]};
          __builtin_amdgcn_sched_barrier(0);
          uint32_t out[2];
          gelu_f16<2>(in, out);
          asm volatile("" : "+v"(out[0]), "+v"(out[1]));
          gb[j / 2][2 * (j % 2)] = out[0];
          gb[j / 2][2 * (j % 2) + 1] = out[1];
          __builtin_amdgcn_sched_barrier(0);
        }
        u = mfma32_f16(a21, gb[1], u);
      }
      // The store is held back until the next map (or the next tile's input wait) has been passed:
      // stores count in the same wait counter as loads, and a store issued just before that wait
      // would make the wave sit out the store's full round trip.
      flush();
      {
        const float* b2 = reinterpret_cast<const float*>(wm + SM::kW1 + SM::kW2 + D * 4) + 4 * gl;
#pragma unroll
        for (int i = 0; i < NU; ++i) pend[i] = fmaxf(u[i] + b2[8 * (i / 4) + i % 4], 0.0f);
        pend_ptr = live ? feat + g.fidx(th, (map0 + m) * DPH + 4 * gl) : nullptr;
      }
    }
  }
  flush();
}

// The query map, then the F key maps, in one launch: a workgroup that has finished its share of
// the query tiles swaps the weights in LDS and goes on with the key tiles, so the launch has no
// boundary in between (no drain of the grid, no second cold start).  `nk` is F at run time.
template <int D, int F, int WAVES, int DPH>
__global__ __launch_bounds__(WAVES * 64) void k_phi_fwd(Geom g, View Q, View K,
                                                        const unsigned char* __restrict__ wpk,
                                                        int heads_w, int nk, float* __restrict__ feat) {
  phi_fwd_body<D, 1, WAVES, DPH>(g, Q, wpk, heads_w, 0, 1, feat);
  __syncthreads();  // every wave is done with the query map's weights
  phi_fwd_body<D, F, WAVES, DPH>(g, K, wpk, heads_w, 1, nk, feat);
}

// ---- backward -----------------------------------------------------------------------------------
// block WAVES*64.  dX = sum over the NMAPS maps of W1 (GELU'(h) * (W2 du)), with du = d(feature)
// where the ReLU was open (the form in which the feature-gradient workspace arrives).  Hidden
// activations are recomputed.
template <int D, int NMAPS, int WAVES, int DPH>
__device__ __forceinline__ void phi_bwd_body(const Geom& g, const View& X,
                                             const unsigned char* __restrict__ wpk, int heads_w,
                                             int map0, int nmaps,
                                             const float* __restrict__ dfeat, const View& dX) {
  using SM = PhiSmem<D, true>;
  constexpr int NRB = D / 32, NKS = D / 16;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  const int r = lane % 32, gl = lane / 32;
  const int L = lane % 16, q = lane / 16;
  const TileMap tm = make_tile_map(g, heads_w);
  const int hw = heads_w == 1 ? 0 : blockIdx.y;
  for (int m = 0; m < NMAPS; ++m)
    load_weights<D, true, WAVES * 64>(smem + m * SM::kMap,
                          wpk + (static_cast<int64_t>(map0 + m) * heads_w + hw) * Packed<D>::kBytes);
  __syncthreads();
  unsigned char* ttile = smem + nmaps * SM::kMap + wave * RowTile<D, 16>::kBytes;  // dX transpose tile
  int a_off[NKS];
  first_layer_offsets<D>(lane, a_off);
  // Transpose reads for dx^T[in x tok] += W1[in x hidden] dh^T: k-slots (ks2, gl, j) stand for
  // hidden units 16 ks2 + 4 gl + {0..3} (j < 4) and + 8 (j >= 4); a lane of a 16-lane group
  // addresses hidden row k0 + L/4 and the 4 input channels 32 rb + 16 (q%2) + 4 (L%4) ..+3.
  // swz() ignores the row's bits 4 and up, so the k-step only adds a constant to the address.
  int t_off[2][NRB];
#pragma unroll
  for (int hi = 0; hi < 2; ++hi)
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const int row = 4 * gl + 8 * hi + L / 4;
      const int col = 32 * rb + 16 * (q % 2) + 4 * (L % 4);
      t_off[hi][rb] = SM::off(row, col >> 3) + ((col & 7) << 1);
    }
  const int stride = gridDim.x * WAVES;
  int tile = blockIdx.x * WAVES + wave;
  int b = 0, h = 0, n0 = 0;
  // The tile's inputs live in xb only: the next tile's loads are issued into xb as soon as the
  // last first-layer MFMA of the current tile has read it (one and a half stages before the end).
  u32x4 xb[NKS];
  if (tile < tm.total) {
    tm.decode(tile, b, h, n0);
    load_x<D>(X, b, h, n0 + r, g.N, gl, xb);
  }
  // du^T of one map as B operand of a single 16-slot step: slot (gl, j) is feature 8gl + j (with
  // d_phi <= 8 only gl = 0 is used).  The feature gradients arrive already zeroed where the ReLU
  // was closed (the core backward kernels, which hold the features anyway, write them that way), so
  // this is a plain load.  In two halves: issue_du puts the loads in flight (unconditional, from
  // addresses valid for every lane), finish_du packs them a whole map later.  Anything that looks
  // at the loaded values next to the loads makes the wave sit out the memory round trip there.
  static_assert(DPH % 2 == 0 && DPH <= 16, "features are packed in pairs into one k-step");
  constexpr int NJ = DPH <= 8 ? DPH : 8;  // features per lane half
  auto issue_du = [&](int64_t th, int m, float (&dv)[NJ]) {
    // lane half 1 holds the features from the ninth on (none when d_phi <= 8: it re-reads half 0's);
    // surplus slots re-read the half's first feature
    const int first = DPH <= 8 ? 0 : 8 * gl;
    const int have = DPH <= 8 ? DPH : (gl ? DPH - 8 : 8);
    const f32x2* dp = reinterpret_cast<const f32x2*>(dfeat + g.fidx(th, (map0 + m) * DPH + first));
#pragma unroll
    for (int p = 0; p < NJ / 2; ++p) {
      const f32x2 v = dp[32 * (2 * p < have ? p : 0)];
      dv[2 * p] = v[0];
      dv[2 * p + 1] = v[1];
    }
  };
  auto finish_du = [&](const float (&dv)[NJ], bool live) -> u32x4 {
    const int have = DPH <= 8 ? (gl ? 0 : DPH) : (gl ? DPH - 8 : 8);
    u32x4 d;
    d[0] = d[1] = d[2] = d[3] = 0u;
#pragma unroll
    for (int p = 0; p < NJ / 2; ++p)
      d[p] = pack_bf16(live && 2 * p < have ? dv[2 * p] : 0.0f, live && 2 * p + 1 < have ? dv[2 * p + 1] : 0.0f);
    return d;
  };
  auto zero_acc = []() {  // a constant: becomes the inline 0 of the MFMA's C operand
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.0f;
    return z;
  };
  // the first layer accumulates on top of its bias: the lane's 16 entries of a 32-row block
  auto bias_acc = [&](const unsigned char* wmap, int rb) {
    f32x16 z;
    const float* b1 = reinterpret_cast<const float*>(wmap + SM::kW1 + SM::kW2) + 32 * rb + 4 * gl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {  // registers 4i..4i+3 are hidden units 32 rb + 8 i + 4 gl + 0..3
      const f32x4 v = *reinterpret_cast<const f32x4*>(b1 + 8 * i);
      z[4 * i] = v[0];
      z[4 * i + 1] = v[1];
      z[4 * i + 2] = v[2];
      z[4 * i + 3] = v[3];
    }
    return z;
  };
  // du of the coming tile's first map: loaded during the last map of the tile before, like the
  // later maps' du is loaded a map ahead
  u32x4 dub_first;
  if (tile < tm.total) {
    float dv0[NJ];
    issue_du(g.th(b, h, n0 + r < g.N ? n0 + r : 0), 0, dv0);
    dub_first = finish_du(dv0, n0 + r < g.N);
  }
  for (; tile < tm.total; tile += stride) {
    const int n = n0 + r;
    const bool live = n < g.N;
    const int64_t th = g.th(b, h, live ? n : 0);
    const int ob = b, oh = h, on0 = n0;  // this tile's coordinates
    const bool more_tiles = tile + stride < tm.total;
    if (more_tiles) tm.decode(tile + stride, b, h, n0);  // b, h, n0 now name the next tile
    const bool live_next = more_tiles && n0 + r < g.N;
    const int64_t th_next = g.th(b, h, live_next ? n0 + r : 0);
    f32x16 dx[NRB];  // first written by the second stage of the first map (accumulating onto zero)
    // Software pipeline over 32-row blocks of the hidden layer, block t = m * NRB + rb.  Stage t:
    //   vector ALU : dh(t) = dg(t) * GELU'(hidden(t) + b1), packed as the B operand of dx
    //   matrix pipe: hidden(t+1) = W1^T X^T block (A: 16-byte LDS reads), dg(t) = W2 du^T block,
    //                dx += W1 dh(t-1)^T (A: transpose reads of the same LDS copy),
    // the MFMAs two or three at a time between quarters of the vector-ALU work, their LDS
    // operands read one step ahead.  Blocks before the first / after the last alias valid LDS
    // and meet zero operands or are dropped.
    static_assert(NRB % 2 == 0, "two alternating accumulator sets");
    f32x16 hb[2];  // hidden blocks alternate between two accumulator sets (as in the forward)
    constexpr int kPer = NKS / 4;  // first-layer MFMAs per slice
    u32x4 an[kPer];                // their A operands, read one slice ahead
    {
      u32x4 a0[NKS];
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) a0[ks] = *reinterpret_cast<const u32x4*>(smem + a_off[ks]);
      hb[0] = bias_acc(smem, 0);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) hb[0] = mfma32(a0[ks], xb[ks], hb[0]);
#pragma unroll
      for (int t = 0; t < kPer; ++t)
        an[t] = *reinterpret_cast<const u32x4*>(smem + (1 % NRB) * 32 * SM::kRow + a_off[t]);
    }
    u32x4 dub = dub_first;
    u32x4 dhp[2];  // dh of the previous block (two 16-slot steps)
    // The first map is peeled off the loop over maps: its first stage has no previous block (no dx
    // step at all) and its second stage starts the dx accumulators from the constant zero, which
    // spares clearing them and carrying them into the loop as copies.
    auto run_map = [&](int m, auto first_tag, int64_t th_nx, bool live_nx) {
      constexpr bool FIRST = decltype(first_tag)::value;
      const unsigned char* wm = smem + m * SM::kMap;
      const bool last_map = m + 1 == nmaps;
      float dvn[NJ];  // the next map's du, or the coming tile's first
      issue_du(last_map ? th_nx : th, last_map ? 0 : m + 1, dvn);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        // block t+1 (first layer, this stage) and block t+2 (whose first operands the last slice reads)
        const unsigned char* a1_base = (rb + 1 < NRB ? wm : (last_map ? wm : wm + SM::kMap)) + ((rb + 1) % NRB) * 32 * SM::kRow;
        const unsigned char* a2_base = (rb + 2 < NRB ? wm : (last_map ? wm : wm + SM::kMap)) + ((rb + 2) % NRB) * 32 * SM::kRow;
        const unsigned char* wp = rb > 0 ? wm : (m > 0 ? wm - SM::kMap : wm);
        const int ks2p = 2 * ((rb + NRB - 1) % NRB);  // first of the two 16-slot steps of block t-1
        const u32x4 a2 = *reinterpret_cast<const u32x4*>(wm + SM::kW1 + (rb * 64 + lane) * 16);
        const f32x16 dg = mfma32(a2, dub, zero_acc());
        f32x16& cur = hb[rb % 2];
        f32x16& nxt = hb[(rb + 1) % 2];
        nxt = bias_acc(rb + 1 < NRB ? wm : (last_map ? wm : wm + SM::kMap), (rb + 1) % NRB);
        u32x4 dhc[2];
        // transpose-read operands of the first dx step of this stage
        u32x2 tlo[NRB / 2], thi[NRB / 2];
        const bool has_prev = !(FIRST && rb == 0);  // compile-time after unrolling
        if (has_prev) {
#pragma unroll
          for (int x = 0; x < NRB / 2; ++x) {
            tlo[x] = lds_read_tr16(wp + ks2p * 16 * SM::kRow + t_off[0][x]);
            thi[x] = lds_read_tr16(wp + ks2p * 16 * SM::kRow + t_off[1][x]);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          asm volatile("" : "+v"(nxt));
          // first layer of block t+1 (there is none after the last block, and xb already belongs
          // to the next tile's loads by then)
          if (rb + 1 < NRB || !last_map) {
#pragma unroll
            for (int t = 0; t < kPer; ++t) {
              nxt = mfma32(an[t], xb[j * kPer + t], nxt);
              an[t] = j < 3 ? *reinterpret_cast<const u32x4*>(a1_base + a_off[(j + 1) * kPer + t])
                            : *reinterpret_cast<const u32x4*>(a2_base + a_off[t]);
            }
          }
          // dx += W1[row blocks of this slice, hidden of block t-1] dh(t-1)^T
#pragma unroll
          for (int x = 0; x < NRB / 2; ++x) {
            if (!has_prev) break;
            const int rbx = (j % 2) * (NRB / 2) + x;
            u32x4 a;
            a[0] = tlo[x][0];
            a[1] = tlo[x][1];
            a[2] = thi[x][0];
            a[3] = thi[x][1];
            // each accumulator is touched twice per stage; its very first touch starts from zero
            dx[rbx] = FIRST && rb == 1 && j < 2 ? mfma32(a, dhp[j / 2], zero_acc())
                                                : mfma32(a, dhp[j / 2], dx[rbx]);
            // operands of the next slice's dx step (the last slice reads ahead into valid LDS)
            const int jn = j + 1 < 4 ? j + 1 : 3;
            const int rbn = (jn % 2) * (NRB / 2) + x;
            tlo[x] = lds_read_tr16(wp + (ks2p + jn / 2) * 16 * SM::kRow + t_off[0][rbn]);
            thi[x] = lds_read_tr16(wp + (ks2p + jn / 2) * 16 * SM::kRow + t_off[1][rbn]);
          }
          // the next tile's inputs: xb is free once the last first-layer MFMA has been issued
          if (last_map && rb == NRB - 2 && j == 3 && more_tiles) load_x<D>(X, b, h, n0 + r, g.N, gl, xb);
          const float in[4] = {cur[4 * j], cur[4 * j + 1], cur[4 * j + 2], cur[4 * j + 3]};
          __builtin_amdgcn_sched_barrier(0);
          f16x2 gp[2];
          gelu_grad_f16<2>(in, gp);
          // dg * GELU' in fp32 with the fp16 factor read in place (mixed-precision FMA)
          uint32_t o0 = pack_bf16(__builtin_fmaf(static_cast<float>(gp[0][0]), dg[4 * j], 0.0f),
                                  __builtin_fmaf(static_cast<float>(gp[0][1]), dg[4 * j + 1], 0.0f));
          uint32_t o1 = pack_bf16(__builtin_fmaf(static_cast<float>(gp[1][0]), dg[4 * j + 2], 0.0f),
                                  __builtin_fmaf(static_cast<float>(gp[1][1]), dg[4 * j + 3], 0.0f));
          asm volatile("" : "+v"(o0), "+v"(o1));
          dhc[j / 2][2 * (j % 2)] = o0;
          dhc[j / 2][2 * (j % 2) + 1] = o1;
          __builtin_amdgcn_sched_barrier(0);
        }
        dhp[0] = dhc[0];
        dhp[1] = dhc[1];
      }
      dub = finish_du(dvn, last_map ? live_nx : live);  // after the last map: the coming tile's
    };
    run_map(0, TrueTag{}, th_next, live_next);
#pragma unroll 1
    for (int m = 1; m < nmaps; ++m) run_map(m, FalseTag{}, th_next, live_next);  // nmaps == NMAPS, passed at run time so this stays a loop
    dub_first = dub;
    // dx of the last block
    {
      const unsigned char* wp = smem + (nmaps - 1) * SM::kMap;
      constexpr int ks2p = 2 * (NRB - 1);
#pragma unroll
      for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int rbx = 0; rbx < NRB; ++rbx) {
          const u32x2 lo = lds_read_tr16(wp + (ks2p + hf) * 16 * SM::kRow + t_off[0][rbx]);
          const u32x2 hi = lds_read_tr16(wp + (ks2p + hf) * 16 * SM::kRow + t_off[1][rbx]);
          u32x4 a;
          a[0] = lo[0];
          a[1] = lo[1];
          a[2] = hi[0];
          a[3] = hi[1];
          dx[rbx] = mfma32(a, dhp[hf], dx[rbx]);
        }
    }
    store_rows_bf16<D, 16>(dx, 1.0f, lane, ttile, [&](int t) -> bf16_t* {
      return on0 + t < g.N ? dX.row<bf16_t>(ob, oh, on0 + t) : nullptr;
    });
  }
}

// dQ through the query map, then dK through the F key maps, in one launch (see k_phi_fwd)
template <int D, int F, int WAVES, int DPH>
__global__ __launch_bounds__(WAVES * 64) void k_phi_bwd(Geom g, View Q, View K,
                                                        const unsigned char* __restrict__ wpk,
                                                        int heads_w, int nk,
                                                        const float* __restrict__ dfeat, View dQ,
                                                        View dK) {
  phi_bwd_body<D, 1, WAVES, DPH>(g, Q, wpk, heads_w, 0, 1, dfeat, dQ);
  __syncthreads();  // every wave is done with the query map's weights and its transpose tile
  phi_bwd_body<D, F, WAVES, DPH>(g, K, wpk, heads_w, 1, nk, dfeat, dK);
}

// ---- weight gradients ---------------------------------------------------------------------------
// dW1 = X^T dh, db1 = sum dh, dW2 = GELU(h)^T du, db2 = sum du over tokens, for one map per
// workgroup (blockIdx.y) and, with per-head weights, one head (blockIdx.z).  Both products contract
// over TOKENS, while the forward layout keeps a token in an MFMA column, so every 32-token tile
// goes through two wave-private LDS tiles, [token][input channels | du] and [token][dh | GELU(h)],
// that are read back with transpose reads as operands whose k index is the token.
// Wave w of the workgroup owns hidden block hb = w % (D/32) -- its first-layer weights stay in
// registers, it needs no LDS copy of W1 -- and serves the 32-token tiles th, th + T, .. of the
// workgroup's share, th = w / (D/32), T = WAVES / (D/32).  Its sums end as the hidden-block
// columns of partial number blockIdx.x * T + th of this (map, head):
//   [dW1 D*D | db1 D | dW2 D*d_phi | db2 d_phi] floats, scaled by the packing factors
// (dW1, db1 four times too large, dW2 four times too small); a second kernel adds the partials.
// A workgroup has eight waves, two per SIMD (the live set is kept to 256 registers), and a wave
// takes one tile per iteration, its steps one after the other: what hides the LDS round trip
// between writing a tile and reading it back transposed is the other wave of the SIMD.  (A
// four-wave form with a software pipeline inside the wave -- first layer of tile t+1 and
// contractions of tile t-1 under the vector work of tile t, two sets of LDS tiles, 352 registers --
// took 335 us where this one takes 270, 274 against 235 for twelve features per map.)
template <int D>
struct WgSmem {
  static constexpr int kXStride = (D + 32) * 2 + 32;  // bytes per token row: channels, 32 du columns, pad
  static constexpr int kGStride = 64 * 2 + 32;        // dh (32 columns), GELU(h) (32 columns), pad
  static constexpr int kXBytes = 32 * kXStride;
  static constexpr int kWaveBytes = kXBytes + 32 * kGStride;  // a wave's two tiles
};

template <int D, int WAVES, int DPH>
__global__ __launch_bounds__(WAVES * 64) void k_phi_wgrad(Geom g, View Q, View K,
                                                          const unsigned char* __restrict__ wpk,
                                                          int heads_w,
                                                          const float* __restrict__ feat,
                                                          const float* __restrict__ dfeat,
                                                          float* __restrict__ partial) {
  using SM = WgSmem<D>;
  using PK = Packed<D>;
  constexpr int NRB = D / 32, NKS = D / 16, TH = WAVES / NRB;
  static_assert(WAVES % NRB == 0, "whole groups of hidden blocks");
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  const int r = lane % 32, gl = lane / 32;
  const int L = lane % 16, q = lane / 16;
  const int hb = wave % NRB, th = wave / NRB;
  const int m = blockIdx.y, hw = blockIdx.z;
  unsigned char* xt = smem + wave * SM::kWaveBytes;  // this wave's (X tile, G tile)
  unsigned char* gt = xt + SM::kXBytes;
  const unsigned char* wm = wpk + (static_cast<int64_t>(m) * heads_w + hw) * PK::kBytes;
  const View& X = m == 0 ? Q : K;
  // this wave's first-layer operands: rows 32 hb + r of W1^T, k-slot (ks, gl, j) = channel 16ks + 8gl + j
  u32x4 w1a[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks)
    w1a[ks] = *reinterpret_cast<const u32x4*>(wm + PK::kW1T + ((32 * hb + r) * D + 16 * ks + 8 * gl) * 2);
  const u32x4 w2b = *reinterpret_cast<const u32x4*>(wm + PK::kW2B + (hb * 64 + lane) * 16);
  f32x16 bias;  // first-layer bias of the block in accumulator order
  {
    const float* b1 = reinterpret_cast<const float*>(wm + PK::kB1) + 32 * hb + 4 * gl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f32x4 bv = *reinterpret_cast<const f32x4*>(b1 + 8 * i);
      bias[4 * i] = bv[0];
      bias[4 * i + 1] = bv[1];
      bias[4 * i + 2] = bv[2];
      bias[4 * i + 3] = bv[3];
    }
  }
  // token tiles: one list over all (batch row, head) pairs when the weights are shared
  const bool shared = heads_w == 1;
  const int tpr = (g.N + 31) / 32;
  const int total = (shared ? g.B * g.H : g.B) * tpr;
  f32x16 acc[NRB];   // dW1 rows 32 ib + d_row(i, gl), column 32 hb + r
  f32x16 acc2;       // dW2^T rows = features d_row(i, gl), column 32 hb + r
  float db1[16];     // per-lane (token r) sums of dh for hidden 32 hb + d_row(i, gl)
  float db2[DPH];    // per-lane sums of du (read from the lanes gl == 0)
#pragma unroll
  for (int i = 0; i < 16; ++i) {
#pragma unroll
    for (int ib = 0; ib < NRB; ++ib) acc[ib][i] = 0.0f;
    acc2[i] = 0.0f;
    db1[i] = 0.0f;
  }
#pragma unroll
  for (int a = 0; a < DPH; ++a) db2[a] = 0.0f;
  // The next tile's inputs are loaded as soon as the current tile's have been consumed (the
  // input rows after the copy to LDS, the features once du is formed).  These loads are
  // unconditional with clamped addresses, so that the same number is outstanding on every path;
  // the last tile is simply fetched twice.
  const int step = gridDim.x * TH;
  int tile = blockIdx.x * TH + th;
  u32x4 xb[NKS];  // input rows of the coming tile
  float fv[DPH], dv[DPH];
  auto coords = [&](int t, int& b, int& h, int& n0) {
    const int row = t / tpr;
    n0 = (t % tpr) * 32;
    b = shared ? row / g.H : row;
    h = shared ? row % g.H : hw;
  };
  auto fetch_features = [&](int b, int h, int n0) {
    const int n = n0 + r;
    const int64_t o = g.fidx(g.th(b, h, n < g.N ? n : g.N - 1), m * DPH);
    const f32x2* fp = reinterpret_cast<const f32x2*>(feat + o);
    const f32x2* dp = reinterpret_cast<const f32x2*>(dfeat + o);
#pragma unroll
    for (int p = 0; p < DPH / 2; ++p) {
      const f32x2 f2 = fp[32 * p], d2 = dp[32 * p];
      fv[2 * p] = f2[0];
      fv[2 * p + 1] = f2[1];
      dv[2 * p] = d2[0];
      dv[2 * p + 1] = d2[1];
    }
  };
  // du of the token: zero where the ReLU was closed, and for tokens past the end (whose clamped
  // input row then adds nothing to any sum).  As the B operand of dg = W2 du^T, slot (gl, j) is
  // feature 8 gl + j: with d_phi <= 8 the lanes gl = 1 hold zeros throughout (db2 included), with
  // more features they hold the ninth feature on.
  auto make_du = [&](bool live, u32x4& dub) {
    float du[DPH];
#pragma unroll
    for (int a = 0; a < DPH; ++a) du[a] = live && (DPH > 8 || gl == 0) && fv[a] > 0.0f ? dv[a] : 0.0f;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const float lo0 = 2 * p < DPH ? du[2 * p < DPH ? 2 * p : 0] : 0.0f;
      const float hi0 = 2 * p + 1 < DPH ? du[2 * p + 1 < DPH ? 2 * p + 1 : 0] : 0.0f;
      const float lo1 = 8 + 2 * p < DPH ? du[8 + 2 * p < DPH ? 8 + 2 * p : 0] : 0.0f;
      const float hi1 = 9 + 2 * p < DPH ? du[9 + 2 * p < DPH ? 9 + 2 * p : 0] : 0.0f;
      dub[p] = DPH > 8 ? pack_bf16(gl ? lo1 : lo0, gl ? hi1 : hi0) : pack_bf16(lo0, hi0);
    }
#pragma unroll
    for (int a = 0; a < DPH; ++a) db2[a] += du[a];
  };
  auto put_x_tile = [&](unsigned char* xdst, const u32x4 (&xr)[NKS], const u32x4& dub) {  // [token][channels | du]
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
      *reinterpret_cast<u32x4*>(xdst + r * SM::kXStride + (16 * ks + 8 * gl) * 2) = xr[ks];
    u32x4 z4;
    z4[0] = z4[1] = z4[2] = z4[3] = 0u;
    // du columns D + 8 gl .. + 7 are this lane's operand slots; columns D + 16 .. D + 31 are zero
    *reinterpret_cast<u32x4*>(xdst + r * SM::kXStride + (D + 8 * gl) * 2) = dub;
    *reinterpret_cast<u32x4*>(xdst + r * SM::kXStride + (D + 16 + 8 * gl) * 2) = z4;
  };
  // transpose-read operand: tokens 16 ks + 8 gl + {0..7} of 32 columns starting at col0
  auto operand = [&](const unsigned char* tl, int stride, int ks, int col0) {
    const int krow = 16 * ks + 8 * gl + L / 4;
    const unsigned char* p = tl + krow * stride + (col0 + 16 * (q % 2) + 4 * (L % 4)) * 2;
    const u32x2 lo = lds_read_tr16(p);
    const u32x2 hi = lds_read_tr16(p + 4 * stride);
    u32x4 o;
    o[0] = lo[0];
    o[1] = lo[1];
    o[2] = hi[0];
    o[3] = hi[1];
    return o;
  };
  f32x16 zero;
#pragma unroll
  for (int i = 0; i < 16; ++i) zero[i] = 0.0f;
  // One tile per iteration, its steps one after the other (first layer, dg, the two LDS tiles,
  // GELU and GELU', the contractions over its tokens): the second wave of the SIMD runs while this
  // one waits.  xb, fv, dv always hold the coming tile, loaded as soon as the current tile has used them.
  // (with more than eight features per map the feature loads are not run ahead: their registers
  // are what makes the difference between fitting 256 and spilling)
  constexpr bool kFeatAhead = DPH <= 8;
  if (tile < total) {
    int b, h, n0;
    coords(tile, b, h, n0);
    load_x<D>(X, b, h, n0 + r, g.N, gl, xb);
    if (kFeatAhead) fetch_features(b, h, n0);
  }
  for (; tile < total; tile += step) {
    int b, h, n0;
    coords(tile, b, h, n0);
    if (!kFeatAhead) fetch_features(b, h, n0);
    u32x4 dub;
    make_du(n0 + r < g.N, dub);
    f32x16 cur = bias;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) cur = mfma32(w1a[ks], xb[ks], cur);
    const f32x16 dg = mfma32(w2b, dub, zero);
    put_x_tile(xt, xb, dub);
    {
      const int tn = tile + step < total ? tile + step : tile;
      coords(tn, b, h, n0);
      load_x<D>(X, b, h, n0 + r, g.N, gl, xb);
      if (kFeatAhead) fetch_features(b, h, n0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {  // slice j covers hidden 8j + 4gl .. +3 of the block
      const float in[4] = {cur[4 * j], cur[4 * j + 1], cur[4 * j + 2], cur[4 * j + 3]};
      f16x2 gv[2], gp[2];
      gelu_both_f16<2>(in, gv, gp);
      const float d0 = __builtin_fmaf(static_cast<float>(gp[0][0]), dg[4 * j], 0.0f);
      const float d1 = __builtin_fmaf(static_cast<float>(gp[0][1]), dg[4 * j + 1], 0.0f);
      const float d2 = __builtin_fmaf(static_cast<float>(gp[1][0]), dg[4 * j + 2], 0.0f);
      const float d3 = __builtin_fmaf(static_cast<float>(gp[1][1]), dg[4 * j + 3], 0.0f);
      db1[4 * j] += d0;
      db1[4 * j + 1] += d1;
      db1[4 * j + 2] += d2;
      db1[4 * j + 3] += d3;
      u32x2 dh2, g2;
      dh2[0] = pack_bf16(d0, d1);
      dh2[1] = pack_bf16(d2, d3);
      g2[0] = pack_bf16(static_cast<float>(gv[0][0]), static_cast<float>(gv[0][1]));
      g2[1] = pack_bf16(static_cast<float>(gv[1][0]), static_cast<float>(gv[1][1]));
      *reinterpret_cast<u32x2*>(gt + r * SM::kGStride + (8 * j + 4 * gl) * 2) = dh2;
      *reinterpret_cast<u32x2*>(gt + r * SM::kGStride + (32 + 8 * j + 4 * gl) * 2) = g2;
    }
    wave_lds_sync();
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const u32x4 bdh = operand(gt, SM::kGStride, ks, 0);
      const u32x4 bg = operand(gt, SM::kGStride, ks, 32);
      u32x4 ax[NRB + 1];
#pragma unroll
      for (int ib = 0; ib < NRB; ++ib) ax[ib] = operand(xt, SM::kXStride, ks, 32 * ib);
      ax[NRB] = operand(xt, SM::kXStride, ks, D);
#pragma unroll
      for (int ib = 0; ib < NRB; ++ib) acc[ib] = mfma32(ax[ib], bdh, acc[ib]);
      acc2 = mfma32(ax[NRB], bg, acc2);
    }
    wave_lds_sync();  // the tiles are free for the next tile
  }
  // ---- this wave's share of the partial
  const int nparts = gridDim.x * TH;
  const int64_t floats = static_cast<int64_t>(D) * D + D + D * DPH + DPH;
  float* out = partial + ((static_cast<int64_t>(m) * gridDim.z + hw) * nparts + blockIdx.x * TH + th) * floats;
#pragma unroll
  for (int ib = 0; ib < NRB; ++ib)
#pragma unroll
    for (int i = 0; i < 16; ++i) out[(32 * ib + d_row(i, gl)) * D + 32 * hb + r] = acc[ib][i];
#pragma unroll
  for (int i = 0; i < (DPH > 8 ? 8 : 4); ++i) {
    const int a = d_row(i, gl);
    if (a < DPH) out[D * D + D + (32 * hb + r) * DPH + a] = acc2[i];
  }
  // sums over the 32 tokens of a half-wave (xor offsets below 32 stay inside it)
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    float v = db1[i];
#pragma unroll
    for (int off = 16; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    if (r == 0) out[D * D + 32 * hb + d_row(i, gl)] = v;
  }
  if (hb == 0) {
#pragma unroll
    for (int a = 0; a < DPH; ++a) {
      float v = db2[a];
#pragma unroll
      for (int off = 16; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
      if (lane == 0) out[D * D + D + D * DPH + a] = v;
    }
  }
}

template <typename K>
hla_status allow_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
             ? HLA_OK
             : HLA_ERR_HIP;
}

// One workgroup per compute unit in total.  Shared weights: a flat grid over all tiles; per-head
// weights: (x, H, B) with x workgroups per (batch row, head).
dim3 phi_grid(const hla_handle* hd, int waves) {
  const Geom& g = hd->g;
  const int tiles = (g.N + 31) / 32;
  if (hd->phi.heads_w == 1) {
    const int64_t total = static_cast<int64_t>(tiles) * g.B * g.H;
    const int64_t want = (total + waves - 1) / waves;
    return dim3(static_cast<unsigned>(want < 256 ? (want < 1 ? 1 : want) : 256), 1, 1);
  }
  const int units = g.B * g.H;
  int gx = 256 / units;  // rounding down keeps the whole grid resident in one round
  const int need = (tiles + waves - 1) / waves;
  if (gx > need) gx = need;
  return dim3(gx < 1 ? 1 : gx, g.H, g.B);
}

// waves per workgroup: three per SIMD in the forward kernel (it stays within 168 registers), two
// in the backward one
constexpr int kWavesF = 12, kWavesB = 8;

// F key maps of DPH features each, after the query map
template <int D, int F, int DPH>
hla_status forward_t(hla_handle* hd, const hla_call_args& a) {
  using SM = PhiSmem<D>;
  Geom g = hd->g;
  const unsigned char* wpk = static_cast<const unsigned char*>(hd->path_ws) + hd->w_packed_off;
  const dim3 grid = phi_grid(hd, kWavesF);
  HLA_TRY(launch(hd, "mfma_phi_forward", k_phi_fwd<D, F, kWavesF, DPH>, grid, dim3(kWavesF * 64),
                 SM::total(F, kWavesF), a.stream, g, a.Q, a.K, wpk, hd->phi.heads_w, F, hd->feat));
  return HLA_OK;
}

template <int D, int F, int DPH>
hla_status backward_t(hla_handle* hd, const hla_call_args& a) {
  using SM = PhiSmem<D, true>;
  Geom g = hd->g;
  const unsigned char* wpk = static_cast<const unsigned char*>(hd->path_ws) + hd->w_packed_off;
  const dim3 grid = phi_grid(hd, kWavesB);
  HLA_TRY(launch(hd, "mfma_phi_backward", k_phi_bwd<D, F, kWavesB, DPH>, grid, dim3(kWavesB * 64),
                 SM::total(F, kWavesB), a.stream, g, a.Q, a.K, wpk, hd->phi.heads_w, F, hd->dfeat,
                 a.dQ, a.dK));
  return HLA_OK;
}

constexpr int kWavesW = 8;  // two waves per SIMD

template <int D, int DPH>
hla_status weight_grads_t(hla_handle* hd, const hla_call_args& a) {
  using SM = WgSmem<D>;
  constexpr int TH = kWavesW / (D / 32);
  constexpr int lds = kWavesW * SM::kWaveBytes;  // a set of tiles per wave
  Geom g = hd->g;
  const unsigned char* wpk = static_cast<const unsigned char*>(hd->path_ws) + hd->w_packed_off;
  const int nm = 1 + g.F;
  const bool shared = hd->phi.heads_w == 1;
  const int heads = shared ? 1 : g.H;
  const int64_t tiles = static_cast<int64_t>(shared ? g.B * g.H : g.B) * ((g.N + 31) / 32);
  // one workgroup per compute unit in total, each with at least one tile per wave group
  int64_t nblk = 256 / (static_cast<int64_t>(nm) * heads);
  if (nblk > (tiles + TH - 1) / TH) nblk = (tiles + TH - 1) / TH;
  if (nblk < 1) nblk = 1;
  const int64_t nparts = nblk * TH;
  if (nm * heads * nparts > hd->wg_parts_cap) return HLA_ERR_STATE;
  HLA_TRY(launch(hd, "mfma_phi_weight_grads", k_phi_wgrad<D, kWavesW, DPH>,
                 dim3(static_cast<unsigned>(nblk), nm, heads), dim3(kWavesW * 64), lds, a.stream, g, a.Q, a.K,
                 wpk, hd->phi.heads_w, static_cast<const float*>(hd->feat),
                 static_cast<const float*>(hd->dfeat), hd->wg_partial));
  // undo the packing factors: dh and dg carry 1/kHiddenScale, GELU(h) carries kHiddenScale
  return weight_grads_reduce(hd, static_cast<int>(nparts), heads, kHiddenScale, kHiddenScale,
                             1.0f / kHiddenScale, 1.0f, a.stream);
}

template <int D, int F, int DPH>
hla_status prepare_t() {
  HLA_TRY(allow_lds(&k_phi_fwd<D, F, kWavesF, DPH>, PhiSmem<D>::total(F, kWavesF)));
  HLA_TRY(allow_lds(&k_phi_bwd<D, F, kWavesB, DPH>, PhiSmem<D, true>::total(F, kWavesB)));
  return allow_lds(&k_phi_wgrad<D, kWavesW, DPH>, kWavesW * WgSmem<D>::kWaveBytes);
}

}  // namespace

hla_status mfma_phi_prepare_kernels(const hla_handle* hd) {
  if (hd->g.F == 3) return hd->g.d == 128 ? prepare_t<128, 3, 6>() : prepare_t<64, 3, 6>();
  return hd->g.d == 128 ? prepare_t<128, 2, 12>() : prepare_t<64, 2, 12>();
}

// the two forms the matrix-core path serves: (F, d_phi) = (3, 6) and (2, 12)
bool mfma_phi_supported(const hla_handle* hd) {
  return (hd->g.F == 3 && hd->g.dphi == 6) || (hd->g.F == 2 && hd->g.dphi == 12);
}

hla_status mfma_phi_weight_grads(hla_handle* hd, const hla_call_args& a) {
  if (!mfma_phi_supported(hd)) return HLA_ERR_UNSUPPORTED;
  if (hd->g.F == 3) return hd->g.d == 128 ? weight_grads_t<128, 6>(hd, a) : weight_grads_t<64, 6>(hd, a);
  return hd->g.d == 128 ? weight_grads_t<128, 12>(hd, a) : weight_grads_t<64, 12>(hd, a);
}

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
  if (!mfma_phi_supported(hd)) return HLA_ERR_UNSUPPORTED;
  if (hd->g.F == 3) return hd->g.d == 128 ? forward_t<128, 3, 6>(hd, a) : forward_t<64, 3, 6>(hd, a);
  return hd->g.d == 128 ? forward_t<128, 2, 12>(hd, a) : forward_t<64, 2, 12>(hd, a);
}

hla_status mfma_phi_backward(hla_handle* hd, const hla_call_args& a) {
  if (!mfma_phi_supported(hd)) return HLA_ERR_UNSUPPORTED;
  if (hd->g.F == 3) return hd->g.d == 128 ? backward_t<128, 3, 6>(hd, a) : backward_t<64, 3, 6>(hd, a);
  return hd->g.d == 128 ? backward_t<128, 2, 12>(hd, a) : backward_t<64, 2, 12>(hd, a);
}

}  // namespace hla

