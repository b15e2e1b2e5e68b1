// Value modulation (paper Sec. 4.5) on the matrix cores, bf16 I/O, head dim 64 or 128:
//   O = T + phi_v1(T) * phi_v2(V),   phi_v (App. A.1) = Linear d->d, GELU, Linear d->d, LayerNorm,
// forward and the backward to (dT, dV).
//
// A token is an MFMA column (lane (r, gl): token r of a 32-token tile, half gl), as in the feature
// maps.  Every product takes its A operand from the LDS copy of a weight matrix with lane r
// addressing matrix row swap23(r) (bits 2 and 3 of the row exchanged) instead of row r.  With that
// the accumulator register i of row block b on lane (r, gl) holds row
//        32 b + 16 (i / 8) + 8 gl + i % 8
// of the product: eight CONSECUTIVE rows per lane half, which is at once
//   - the order in which a lane loads its token's input channels (one 16-byte piece per k-step),
//   - the k-slot order of the B operand of the next product (packed straight from the registers,
//     its A operand again a plain 16-byte LDS read at natural columns),
//   - the order of a token row in memory (outputs leave as 16-byte pieces, no lane exchange).
// Forward per map:   y^T = (W1^T/4) X^T + b1/4,  g = GELU(4y)/4 (packed fp16),  u^T = (4 W2^T) g^T + b2,
// LayerNorm over the 128 channels of a token = over 64 registers of a lane and its partner lane.
// Backward per map:  dg^T = W2 du^T,  dh = dg * GELU'(4y),  dx^T = W1 dh^T, with the A operands
// read from the same LDS copies by transpose reads.  du is handed to the matrix cores in fp16
// scaled per token to unit Euclidean norm (the scale goes back on dx, which is linear in du), so
// its range does not depend on the size of the upstream gradient or of 1/std.
// The forward keeps the weights of both maps resident in LDS (one workgroup of four waves per
// compute unit); the backward runs one map per launch (two workgroups per unit).  Each wave streams
// its own 32-token tiles.
#include "hla_handle.h"
#include "hla_mfma_common.h"
#include "hla_mfma_gelu.h"

namespace hla {
namespace {

using namespace mf;

// Workgroups of four waves.  The forward keeps both maps' weights in LDS, so one workgroup fits a
// compute unit and a wave has its SIMD, and all 512 registers, to itself: that is what lets it
// hold a tile's intermediate values and the next tile's inputs at once.  The backward runs one
// map per launch, two workgroups per unit, 256 registers per wave.
constexpr int kWavesV = 4;
constexpr int kRowsOut = 16;  // token rows of a wave's output tile in LDS (a tile leaves in 32/16 passes)

// packed weights of one map in global memory
template <int D>
struct VPacked {
  static constexpr int kW1T = 0;                  // bf16 [D][D]: row = hidden unit, col = input channel; times 1/4
  static constexpr int kW2T = kW1T + D * D * 2;   // fp16 [D][D]: row = output channel, col = hidden unit; times 4
  static constexpr int kB1 = kW2T + D * D * 2;    // fp32 [D]; times 1/4
  static constexpr int kB2 = kB1 + D * 4;         // fp32 [D]
  static constexpr int kGamma = kB2 + D * 4;      // fp32 [D]
  static constexpr int kBeta = kGamma + D * 4;    // fp32 [D]
  static constexpr int kBytes = kBeta + D * 4;
};

template <typename T>
__global__ void k_vmod_pack_mfma(const T* W1, const T* b1, const T* W2, const T* b2, const T* gamma,
                                 const T* beta, int d, unsigned char* __restrict__ out) {
  // W1, W2 are [in][out] row-major
  uint16_t* w1t = reinterpret_cast<uint16_t*>(out);
  uint16_t* w2t = w1t + d * d;
  float* vec = reinterpret_cast<float*>(w2t + d * d);
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < d * d; i += gridDim.x * blockDim.x) {
    const int row = i / d, col = i % d;  // row = output of the layer, col = its input
    w1t[i] = f32_to_bf16_bits(kHiddenScale * to_float(W1[col * d + row]));
    w2t[i] = __builtin_bit_cast(uint16_t, static_cast<_Float16>(to_float(W2[col * d + row]) / kHiddenScale));
    if (i < d) {
      vec[i] = kHiddenScale * to_float(b1[i]);
      vec[d + i] = to_float(b2[i]);
      vec[2 * d + i] = to_float(gamma[i]);
      vec[3 * d + i] = to_float(beta[i]);
    }
  }
}

// LDS: per map the two matrices row-major with swizzled 16-byte chunks (tile_off), then the four
// vectors; after the maps one output tile per wave.
template <int D>
struct VSmem {
  static constexpr int kRowB = D * 2;
  static constexpr int kW1 = 0;
  static constexpr int kW2 = D * D * 2;
  static constexpr int kVec = 2 * D * D * 2;   // b1/4, b2, gamma, beta
  static constexpr int kMap = kVec + 4 * D * 4;
  static constexpr int total(int waves) { return 2 * kMap + waves * RowTile<D, kRowsOut>::kBytes; }
};

__host__ __device__ __forceinline__ int swap23(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

template <int D, int THREADS>
__device__ __forceinline__ void load_map(unsigned char* dst, const unsigned char* src) {
  using SM = VSmem<D>;
  constexpr int CH = D / 8;           // 16-byte chunks per matrix row
  constexpr int NM = 2 * D * CH;      // chunks of both matrices
  constexpr int IT = (NM + THREADS - 1) / THREADS;
  static_assert(NM % THREADS == 0 && D * 4 * 4 / 16 <= THREADS, "copy loops assume whole rounds");
  const int t = threadIdx.x;
  u32x4 v[IT];
#pragma unroll
  for (int k = 0; k < IT; ++k) v[k] = *reinterpret_cast<const u32x4*>(src + (t + k * THREADS) * 16);
  u32x4 vv;
  if (t < D) vv = *reinterpret_cast<const u32x4*>(src + VPacked<D>::kB1 + t * 16);
#pragma unroll
  for (int k = 0; k < IT; ++k) {
    const int i = t + k * THREADS;
    const int mat = i / (D * CH), row = (i / CH) % D, chunk = i % CH;
    *reinterpret_cast<u32x4*>(dst + mat * SM::kW2 + tile_off<SM::kRowB>(row, chunk)) = v[k];
  }
  if (t < D) *reinterpret_cast<u32x4*>(dst + SM::kVec + t * 16) = vv;
}

// the lane's share of a token row as B operands / in accumulator order: one 16-byte piece per
// k-step, channels 16 ks + 8 gl .. + 7.  Rows at or beyond N read the last row.
template <int D>
__device__ __forceinline__ void load_row(const View& X, int b, int h, int n, int N, int gl,
                                         u32x4 (&x)[D / 16]) {
  const bf16_t* row = X.row<const bf16_t>(b, h, n < N ? n : N - 1);
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) x[ks] = *reinterpret_cast<const u32x4*>(row + 16 * ks + 8 * gl);
}

// 16 entries of an fp32 vector in LDS in accumulator order of row block rb
__device__ __forceinline__ f32x16 vec_block(const float* v, int rb, int gl) {
  f32x16 z;
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const f32x4 t = *reinterpret_cast<const f32x4*>(v + 32 * rb + 16 * hf + 8 * gl + 4 * q);
      z[8 * hf + 4 * q] = t[0];
      z[8 * hf + 4 * q + 1] = t[1];
      z[8 * hf + 4 * q + 2] = t[2];
      z[8 * hf + 4 * q + 3] = t[3];
    }
  return z;
}

// entry i of a token row held as packed bf16 pieces (register i of block rb <-> piece 2 rb + i / 8)
template <int D>
__device__ __forceinline__ float row_entry(const u32x4 (&x)[D / 16], int rb, int i) {
  const uint32_t p = x[2 * rb + i / 8][(i % 8) / 2];
  return i % 2 ? bf16_hi(p) : bf16_lo(p);
}

// entry i of a vector held as packed fp16 pieces in the same order
template <int D>
__device__ __forceinline__ float half_entry(const u32x4 (&x)[D / 16], int rb, int i) {
  const uint32_t w = x[2 * rb + i / 8][(i % 8) / 2];  // (a bit_cast applied to the element expression itself reads element 0)
  const f16x2 p = __builtin_bit_cast(f16x2, w);
  return static_cast<float>(p[i % 2]);
}

// 16-byte load through a pointer known to be global memory (after a pointer has been passed
// through an asm statement the compiler no longer knows, and would use the slower generic form)
__device__ __forceinline__ u32x4 load_global16(const void* p) {
  typedef const u32x4 __attribute__((address_space(1))) * gptr;
  return *(gptr)(p);
}

// What the forward keeps of a 32-token tile for the backward: the normalised outputs u-hat of the
// two maps in fp16, [map][piece][lane] 16 bytes (lane-private pieces: the backward's lane reads
// what the forward's lane wrote), then the two 1/std per token, [map][lane] fp32.
template <int D>
struct SavedTile {
  static constexpr int kUhat = 2 * (D / 16) * 1024;
  static constexpr int kBytes = kUhat + 2 * 256;
};

// Per-token factors of the maps' weight gradients, written by the backward kernel when they are
// asked for: bf16 [token-heads][D] arrays per map m (nullptr: not wanted).  With them
//   dW2 = G^T dU, db2 = sum dU;  dW1 = X^T dH, db1 = sum dH.
// The LayerNorm's dgamma = sum over tokens of dm * u-hat and dbeta = sum of dm (dm: gradient w.r.t.
// the map's output) need no arrays: the backward kernel adds them up per lane as it goes and
// leaves one partial per workgroup in gb_part ([workgroup][dgamma | dbeta][D] floats).
struct VmodFactors {
  bf16_t* dU[2];   // gradient w.r.t. the second layer's output
  bf16_t* dH[2];   // gradient w.r.t. the first layer's output
  bf16_t* G[2];    // GELU(h)
  float* gb_part;
};

// eight fp32 values -> a 16-byte piece of a bf16 row
__device__ __forceinline__ u32x4 pack8(const float (&v)[8], float scale) {
  u32x4 w;
#pragma unroll
  for (int p = 0; p < 4; ++p) w[p] = pack_bf16(v[2 * p] * scale, v[2 * p + 1] * scale);
  return w;
}

struct TileWalk {
  int tiles_per_row, total, H;
  __device__ __forceinline__ void decode(int t, int& b, int& h, int& n0) const {
    const int row = t / tiles_per_row;
    b = row / H;
    h = row % H;
    n0 = (t % tiles_per_row) * 32;
  }
};

// First layer of one map for hidden block rb: y = h/4 of the 16 hidden units the lane holds.
// All LDS operands are read before the first MFMA is issued (one exposed LDS round trip per
// block instead of one per MFMA).
template <int D>
__device__ __forceinline__ f32x16 first_layer_block(const unsigned char* wm, const int (&a_off)[D / 16], int gl,
                                                    const u32x4 (&x)[D / 16], int rb) {
  using SM = VSmem<D>;
  constexpr int NKS = D / 16;
  u32x4 a[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks)
    a[ks] = *reinterpret_cast<const u32x4*>(wm + SM::kW1 + rb * 32 * SM::kRowB + a_off[ks]);
  f32x16 hb = vec_block(reinterpret_cast<const float*>(wm + SM::kVec), rb, gl);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) hb = mfma32(a[ks], x[ks], hb);
  return hb;
}

// One map applied to the token rows in x: on return u holds u-hat (the LayerNorm's normalised
// value, before gamma and beta) in accumulator order, rstd the token's 1/std and, if KEEP, yk the
// first layer's y = h/4 as packed fp16 pairs (pair p of block rb = registers 2p, 2p+1).
// The two layers run as a software pipeline over the 32-row blocks of the hidden layer: in stage
// s the vector ALU evaluates GELU on block s while the matrix cores compute the first layer of
// block s + 1 and the second layer's share of block s - 1.  A wave issues in order and has its
// SIMD to itself, so the overlap needs the two kinds of instructions to alternate in program
// order: a stage is cut into four slices (scheduling barriers in between) of four MFMAs, the LDS
// reads of the next slice's operands and a quarter of the block's GELU.
template <int D, bool KEEP>
__device__ __forceinline__ void map_forward(const unsigned char* wm, const int (&a_off)[D / 16], int gl,
                                            const u32x4 (&x)[D / 16], float ln_eps,
                                            f32x16 (&u)[D / 32], f16x2 (&yk)[KEEP ? D / 32 : 1][8],
                                            float& rstd) {
  using SM = VSmem<D>;
  constexpr int NRB = D / 32, NKS = D / 16;
  constexpr int P1 = NKS / 4;       // first-layer MFMAs per slice
  constexpr int P2 = 2 * NRB / 4;   // second-layer MFMAs per slice
  static_assert(NKS % 4 == 0 && (2 * NRB) % 4 == 0, "four slices per stage");
  const float* vec = reinterpret_cast<const float*>(wm + SM::kVec);
#pragma unroll
  for (int ob = 0; ob < NRB; ++ob) u[ob] = vec_block(vec + D, ob, gl);
  // operand of first-layer MFMA i of slice (s, j): block s + 1, k-step P1 j + i
  auto a1 = [&](int s, int j, int i) {
    return *reinterpret_cast<const u32x4*>(wm + SM::kW1 + (s + 1) * 32 * SM::kRowB + a_off[P1 * j + i]);
  };
  // second-layer MFMA i of slice (s, j) is number n = P2 j + i of block s - 1's 2 NRB products:
  // k-step half n / NRB, output block n % NRB
  auto a2 = [&](int s, int j, int i) {
    const int n = P2 * j + i;
    return *reinterpret_cast<const u32x4*>(wm + SM::kW2 + (n % NRB) * 32 * SM::kRowB + a_off[2 * (s - 1) + n / NRB]);
  };
  f32x16 hb[2];
  hb[0] = first_layer_block<D>(wm, a_off, gl, x, 0);
  u32x4 gprev[2], gcur[2], an1[P1], an2[P2];
#pragma unroll
  for (int i = 0; i < P1; ++i) an1[i] = a1(0, 0, i);
#pragma unroll
  for (int s = 0; s <= NRB; ++s) {
    if (s + 1 < NRB) hb[(s + 1) % 2] = vec_block(vec, s + 1, gl);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < NRB) {
#pragma unroll
        for (int i = 0; i < P1; ++i) hb[(s + 1) % 2] = mfma32(an1[i], x[P1 * j + i], hb[(s + 1) % 2]);
      }
      if (s >= 1) {
#pragma unroll
        for (int i = 0; i < P2; ++i) {
          const int n = P2 * j + i;
          u[n % NRB] = mfma32_f16(an2[i], gprev[n / NRB], u[n % NRB]);
        }
      }
      // operands of the next slice
      const int sn = j < 3 ? s : s + 1, jn = j < 3 ? j + 1 : 0;
      if (sn + 1 < NRB) {
#pragma unroll
        for (int i = 0; i < P1; ++i) an1[i] = a1(sn, jn, i);
      }
      if (sn >= 1 && sn <= NRB) {
#pragma unroll
        for (int i = 0; i < P2; ++i) an2[i] = a2(sn, jn, i);
      }
      if (s < NRB) {  // GELU of entries 4j .. 4j+3 of block s -> two dwords of the B operand
        f16x2 y[2];
        y[0] = to_f16x2(hb[s % 2][4 * j], hb[s % 2][4 * j + 1]);
        y[1] = to_f16x2(hb[s % 2][4 * j + 2], hb[s % 2][4 * j + 3]);
        if (KEEP) {
          yk[s][2 * j] = y[0];
          yk[s][2 * j + 1] = y[1];
        }
        uint32_t gp[2];
        gelu_y16<2>(y, gp);
        gcur[j / 2][2 * (j % 2)] = gp[0];
        gcur[j / 2][2 * (j % 2) + 1] = gp[1];
      }
    }
    gprev[0] = gcur[0];
    gprev[1] = gcur[1];
  }
  __builtin_amdgcn_sched_barrier(0);
  // LayerNorm statistics of the token: this lane's D/2 channels and the partner lane's
  float s = 0.0f;
#pragma unroll
  for (int ob = 0; ob < NRB; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += u[ob][i];
  s += partner32(s);
  const float mean = s * (1.0f / D);
  float v = 0.0f;
#pragma unroll
  for (int ob = 0; ob < NRB; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      u[ob][i] -= mean;
      v = __builtin_fmaf(u[ob][i], u[ob][i], v);
    }
  v += partner32(v);
  rstd = 1.0f / sqrtf(v * (1.0f / D) + ln_eps);
#pragma unroll
  for (int ob = 0; ob < NRB; ++ob)
#pragma unroll
    for (int i = 0; i < 16; ++i) u[ob][i] *= rstd;
}

// 16 accumulator entries -> the two 16-byte bf16 pieces of the token row they stand for
__device__ __forceinline__ void pack_block(const f32x16& a, u32x4 (&w)[2]) {
#pragma unroll
  for (int hf = 0; hf < 2; ++hf)
#pragma unroll
    for (int p = 0; p < 4; ++p) w[hf][p] = pack_bf16(a[8 * hf + 2 * p], a[8 * hf + 2 * p + 1]);
}

template <int D, class RowPtr>
__device__ __forceinline__ void store_tile(const u32x4 (&w)[D / 32][2], int lane, unsigned char* lds,
                                           RowPtr&& row_ptr) {
#pragma unroll
  for (int pass = 0; pass < 32 / kRowsOut; ++pass) {
    put_rows<D, kRowsOut>(w, pass, lane, lds);
    flush_rows<D, kRowsOut>(pass, lane, lds, row_ptr);
  }
}

template <int D>
__device__ __forceinline__ void first_layer_offsets(int lane, int (&a_off)[D / 16]) {
  const int r = lane % 32, gl = lane / 32;
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) a_off[ks] = tile_off<D * 2>(swap23(r), 2 * ks + gl);
}

// grid: one workgroup per compute unit, block WAVES*64.  Tin holds T; O receives T + phi_v1(T) * phi_v2(V).
template <int D, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void k_vmod_fwd_mfma(Geom g, const unsigned char* __restrict__ wpk,
                                                              float ln_eps, View Tin, View V, View O,
                                                              unsigned char* __restrict__ saved) {
  using SM = VSmem<D>;
  constexpr int NRB = D / 32, NKS = D / 16;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  const int r = lane % 32, gl = lane / 32;
  load_map<D, WAVES * 64>(smem, wpk);
  load_map<D, WAVES * 64>(smem + SM::kMap, wpk + VPacked<D>::kBytes);
  __syncthreads();
  unsigned char* otile = smem + 2 * SM::kMap + wave * RowTile<D, kRowsOut>::kBytes;
  int a_off[NKS];
  first_layer_offsets<D>(lane, a_off);
  TileWalk tw;
  tw.tiles_per_row = (g.N + 31) / 32;
  tw.total = tw.tiles_per_row * g.B * g.H;
  tw.H = g.H;
  const int stride = gridDim.x * WAVES;
  // u-hat and 1/std of map m for the backward (see SavedTile)
  auto save = [&](int tile_index, int m, const f32x16 (&u)[NRB], float rstd) {
    unsigned char* slot = saved + static_cast<int64_t>(tile_index) * SavedTile<D>::kBytes;
#pragma unroll
    for (int ob = 0; ob < NRB; ++ob)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        u32x4 v;
#pragma unroll
        for (int p = 0; p < 4; ++p)
          v[p] = __builtin_bit_cast(uint32_t, to_f16x2(u[ob][8 * hf + 2 * p], u[ob][8 * hf + 2 * p + 1]));
        __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(slot + (m * NKS + 2 * ob + hf) * 1024 + lane * 16));
      }
    *reinterpret_cast<float*>(slot + SavedTile<D>::kUhat + m * 256 + lane * 4) = rstd;
  };
  // The value map runs first: its input rows were requested during the previous tile, the rows
  // of T are requested at the top of the tile and needed only after it, and the next tile's V
  // rows are requested once the value map is done with the registers -- no wait of the tile
  // loop sits right behind its load, and the tile's stores have a whole map to complete before
  // the next wait on the memory counter.
  int tile = blockIdx.x * WAVES + wave;
  int b = 0, h = 0, n0 = 0;
  u32x4 xv[NKS];
  if (tile < tw.total) {
    tw.decode(tile, b, h, n0);
    load_row<D>(V, b, h, n0 + r, g.N, gl, xv);
  }
  for (; tile < tw.total; tile += stride) {
    u32x4 xt[NKS];
    load_row<D>(Tin, b, h, n0 + r, g.N, gl, xt);
    const int ob_ = b, oh_ = h, on0 = n0;
    f16x2 none[1][8];
    u32x4 m2p[NKS];  // phi_v2(V), packed bf16 in token-row order
    {
      f32x16 m2[NRB];
      float rstd;
      map_forward<D, false>(smem + SM::kMap, a_off, gl, xv, ln_eps, m2, none, rstd);
      save(tile, 1, m2, rstd);
      const float* vec = reinterpret_cast<const float*>(smem + SM::kMap + SM::kVec);
#pragma unroll
      for (int ob = 0; ob < NRB; ++ob) {
        const f32x16 ga = vec_block(vec + 2 * D, ob, gl), be = vec_block(vec + 3 * D, ob, gl);
        f32x16 o;
#pragma unroll
        for (int i = 0; i < 16; ++i) o[i] = __builtin_fmaf(m2[ob][i], ga[i], be[i]);
        u32x4 pk[2];
        pack_block(o, pk);
        m2p[2 * ob] = pk[0];
        m2p[2 * ob + 1] = pk[1];
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (tile + stride < tw.total) {
      tw.decode(tile + stride, b, h, n0);
      load_row<D>(V, b, h, n0 + r, g.N, gl, xv);
    }
    f32x16 m1[NRB];
    float rstd;
    map_forward<D, false>(smem, a_off, gl, xt, ln_eps, m1, none, rstd);
    save(tile, 0, m1, rstd);
    __builtin_amdgcn_sched_barrier(0);
    u32x4 w[NRB][2];
    {
      const float* vec = reinterpret_cast<const float*>(smem + SM::kVec);
#pragma unroll
      for (int ob = 0; ob < NRB; ++ob) {
        const f32x16 ga = vec_block(vec + 2 * D, ob, gl), be = vec_block(vec + 3 * D, ob, gl);
        f32x16 o;
#pragma unroll
        for (int i = 0; i < 16; ++i)
          o[i] = __builtin_fmaf(__builtin_fmaf(m1[ob][i], ga[i], be[i]), row_entry<D>(m2p, ob, i), row_entry<D>(xt, ob, i));
        pack_block(o, w[ob]);
      }
    }
    store_tile<D>(w, lane, otile, [&](int t) -> bf16_t* {
      return on0 + t < g.N ? O.row<bf16_t>(ob_, oh_, on0 + t) : nullptr;
    });
  }
}

// LayerNorm backward of one map for the lane's token, ready for the matrix cores.  With
// gg = dO * m_other * gamma (m_other = the other map's output) and means over the channels,
//   du = rstd (gg - mean(gg) - u-hat mean(gg u-hat)).
// Returns t = (gg - mean(gg) - u-hat mean(gg u-hat)) / |gg|_2 as packed fp16 B operands (k-slot =
// channel) and the factor rstd |gg|_2 that dx must be multiplied with: scaled to unit Euclidean
// norm per token, the operand's range does not depend on the size of dO or of 1/std.
// The row is streamed twice, 16-byte piece by piece (first for the three sums, then for the
// result), through `load(which, ks, pass)`: piece ks of dO (which = 0, packed bf16), of this map's
// u-hat (1) and of the other map's (2, both packed fp16).  Only the result stays in registers; the
// second pass must really load again (its loader is handed pass = 1 so that it can use an address
// the compiler cannot match with the first pass's).
// fDU: this lane's token row of that factor array (see VmodFactors; + 8 gl already applied), or
// nullptr.  ag / ab (D / 2 entries; 1 entry: no sums wanted): the lane's running sums of dm * u-hat and of dm over its
// tokens, entry 8 ks + j for channel 16 ks + 8 gl + j; `live` is 1 for a token of the sequence
// and 0 for the padding of a ragged tile, whose rows must not be counted.
template <int D, int NA, class Load>
__device__ __forceinline__ float norm_backward(const unsigned char* wm_self, const unsigned char* wm_other,
                                               int gl, Load&& load, float rstd, u32x4 (&dub)[D / 16],
                                               bf16_t* fDU, float (&ag)[NA], float (&ab)[NA], float live) {
  static_assert(NA == D / 2 || NA == 1, "the lane's 64 channels, or no sums wanted");
  using SM = VSmem<D>;
  constexpr int NKS = D / 16;
  // a pass requests all its pieces before it looks at the first one: one memory round trip per
  // pass instead of one per piece
  u32x4 dd[NKS], ss[NKS], oo[NKS];
  auto request = [&](int pass) {
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      dd[ks] = load(0, ks, pass);
      ss[ks] = load(1, ks, pass);
      oo[ks] = load(2, ks, pass);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto piece = [&](int ks, int pass, int opaque, float (&gg)[8], float (&uh)[8], float (&dmv)[8]) {
    const u32x4 d = dd[ks], s = ss[ks], o = oo[ks];
    const float* vs = reinterpret_cast<const float*>(wm_self + SM::kVec) + opaque + 16 * ks + 8 * gl;
    const float* vo = reinterpret_cast<const float*>(wm_other + SM::kVec) + opaque + 16 * ks + 8 * gl;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const f32x4 gs = *reinterpret_cast<const f32x4*>(vs + 2 * D + 4 * q);
      const f32x4 go = *reinterpret_cast<const f32x4*>(vo + 2 * D + 4 * q);
      const f32x4 bo = *reinterpret_cast<const f32x4*>(vo + 3 * D + 4 * q);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int j = 4 * q + e;
        const uint32_t dw = d[j / 2], sw = s[j / 2], ow = o[j / 2];
        const f16x2 sp = __builtin_bit_cast(f16x2, sw), op = __builtin_bit_cast(f16x2, ow);
        const float mo = __builtin_fmaf(static_cast<float>(op[j % 2]), go[e], bo[e]);
        dmv[j] = (j % 2 ? bf16_hi(dw) : bf16_lo(dw)) * mo;
        gg[j] = dmv[j] * gs[e];
        uh[j] = static_cast<float>(sp[j % 2]);
      }
    }
  };
  float sa = 0.0f, sb = 0.0f, sc = 0.0f;
  int z1 = 0, z2 = 0;  // zeros the compiler cannot see through: the LDS vectors are read again, too
  asm volatile("" : "+s"(z1));
  request(0);
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    float gg[8], uh[8], dmv[8];
    piece(ks, 0, z1, gg, uh, dmv);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      sa += gg[j];
      sb = __builtin_fmaf(gg[j], uh[j], sb);
      sc = __builtin_fmaf(gg[j], gg[j], sc);
    }
  }
  sa += partner32(sa);
  sb += partner32(sb);
  sc += partner32(sc);
  const float nrm = sqrtf(sc);
  const float inv = nrm > 0.0f ? 1.0f / nrm : 0.0f;
  const float a = sa * (1.0f / D) * inv, bq = sb * (1.0f / D) * inv;
  asm volatile("" : "+s"(z2));
  __builtin_amdgcn_sched_barrier(0);
  request(1);
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    float gg[8], uh[8], dmv[8], tv[8];
    piece(ks, 1, z2, gg, uh, dmv);
#pragma unroll
    for (int j = 0; j < 8; ++j) tv[j] = __builtin_fmaf(gg[j], inv, -a) - uh[j] * bq;
#pragma unroll
    for (int p = 0; p < 4; ++p) dub[ks][p] = __builtin_bit_cast(uint32_t, to_f16x2(tv[2 * p], tv[2 * p + 1]));
    if (fDU != nullptr) *reinterpret_cast<u32x4*>(fDU + 16 * ks) = pack8(tv, rstd * nrm);
    if constexpr (NA == D / 2) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float dl = dmv[j] * live;
        ab[8 * ks + j] += dl;
        ag[8 * ks + j] = __builtin_fmaf(dl, uh[j], ag[8 * ks + j]);
      }
    }
  }
  return rstd * nrm;
}

// dx^T = W1 (GELU'(4y) * (W2 du^T)) for one map: dub = du as fp16 B operands, x = the map's input
// rows (the first layer is computed again, block by block).
// Per 32-row block of the hidden layer: y and dg (NKS MFMAs each, the operands of dg by transpose
// reads, all requested up front), GELU' and the product on the vector ALU, then the block's share
// of dx.
template <int D>
__device__ __forceinline__ void map_backward(const unsigned char* wm, const int (&a_off)[D / 16],
                                             const int (&t_off)[2][D / 32], int gl,
                                             const u32x4 (&x)[D / 16], const u32x4 (&dub)[D / 16],
                                             f32x16 (&dx)[D / 32], bf16_t* fG = nullptr,
                                             bf16_t* fDH = nullptr, float scale = 1.0f) {
  // fG / fDH: this lane's token rows of the factor arrays (+ 8 gl applied) or nullptr; `scale` is
  // the factor the normalised du (and with it dh) is short of
  using SM = VSmem<D>;
  constexpr int NRB = D / 32, NKS = D / 16;
  auto tr_operand = [&](const unsigned char* mat, int blk, int ks) {
    const u32x2 lo = lds_read_tr16(mat + ks * 16 * SM::kRowB + t_off[0][blk]);
    const u32x2 hi = lds_read_tr16(mat + ks * 16 * SM::kRowB + t_off[1][blk]);
    u32x4 a;
    a[0] = lo[0];
    a[1] = lo[1];
    a[2] = hi[0];
    a[3] = hi[1];
    return a;
  };
#pragma unroll
  for (int ib = 0; ib < NRB; ++ib)
#pragma unroll
    for (int i = 0; i < 16; ++i) dx[ib][i] = 0.0f;
  u32x4 ag[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) ag[ks] = tr_operand(wm + SM::kW2, 0, ks);
#pragma unroll
  for (int hb = 0; hb < NRB; ++hb) {
    __builtin_amdgcn_sched_barrier(0);
    // y (first layer again) and dg are two chains of NKS dependent MFMAs each: issued alternately,
    // one fills the other's latency
    u32x4 a1[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
      a1[ks] = *reinterpret_cast<const u32x4*>(wm + SM::kW1 + hb * 32 * SM::kRowB + a_off[ks]);
    f32x16 yb = vec_block(reinterpret_cast<const float*>(wm + SM::kVec), hb, gl);
    f32x16 dg;
#pragma unroll
    for (int i = 0; i < 16; ++i) dg[i] = 0.0f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      yb = mfma32(a1[ks], x[ks], yb);
      dg = mfma32_f16(ag[ks], dub[ks], dg);
    }
    u32x4 ax[2][NRB];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int ib = 0; ib < NRB; ++ib) ax[hf][ib] = tr_operand(wm + SM::kW1, ib, 2 * hb + hf);
    __builtin_amdgcn_sched_barrier(0);
    f16x2 y[8], gp[8];
#pragma unroll
    for (int p = 0; p < 8; ++p) y[p] = to_f16x2(yb[2 * p], yb[2 * p + 1]);
    gelu_grad_y16<8>(y, gp);  // eight independent chains in lockstep: no issue slot waits for its predecessor
    u32x4 dhb[2];
#pragma unroll
    for (int p = 0; p < 8; ++p)
      dhb[p / 4][p % 4] = pack_bf16(static_cast<float>(gp[p][0]) * dg[2 * p], static_cast<float>(gp[p][1]) * dg[2 * p + 1]);
    if (fG != nullptr) {  // registers 8 hf .. 8 hf + 7 of the block are channels 32 hb + 16 hf + 8 gl ..
      uint32_t gq[8];
      gelu_y16<4>(reinterpret_cast<const f16x2(&)[4]>(y[0]), reinterpret_cast<uint32_t(&)[4]>(gq[0]));
      gelu_y16<4>(reinterpret_cast<const f16x2(&)[4]>(y[4]), reinterpret_cast<uint32_t(&)[4]>(gq[4]));
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        float gv[8], hv[8];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
          const f16x2 g2 = __builtin_bit_cast(f16x2, gq[4 * hf + p]);
          gv[2 * p] = static_cast<float>(g2[0]);
          gv[2 * p + 1] = static_cast<float>(g2[1]);
          hv[2 * p] = static_cast<float>(gp[4 * hf + p][0]) * dg[8 * hf + 2 * p];
          hv[2 * p + 1] = static_cast<float>(gp[4 * hf + p][1]) * dg[8 * hf + 2 * p + 1];
        }
        *reinterpret_cast<u32x4*>(fG + 32 * hb + 16 * hf) = pack8(gv, 1.0f / kHiddenScale);
        *reinterpret_cast<u32x4*>(fDH + 32 * hb + 16 * hf) = pack8(hv, scale * kHiddenScale);  // dg carries the packed W2's factor 4
      }
    }
    if (hb + 1 < NRB) {
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) ag[ks] = tr_operand(wm + SM::kW2, hb + 1, ks);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
      for (int ib = 0; ib < NRB; ++ib) dx[ib] = mfma32(ax[hf][ib], dhb[hf], dx[ib]);
  }
  __builtin_amdgcn_sched_barrier(0);
}

// The backward of ONE map per launch (MAP 0: dT = dO + phi_v1'(T)^T (dO * phi_v2(V)), written to dT;
// MAP 1: dV += phi_v2'(V)^T (dO * phi_v1(T)), added to the rows the operator's backward has written).
// Only that map's matrices are in LDS (plus the other map's gamma, beta), so two workgroups share
// a compute unit and one wave's memory and matrix-pipe waits are filled by another's arithmetic.
constexpr int kRowsOutB = 8;
template <int D>
struct VSmemB {
  static constexpr int kOtherVec = VSmem<D>::kMap;            // the other map's four vectors
  static constexpr int kTiles = kOtherVec + 4 * D * 4;
  static constexpr int total(int waves) { return kTiles + waves * RowTile<D, kRowsOutB>::kBytes; }
  // the factor-writing form ends with the sums of dgamma and dbeta over lanes and waves: a
  // [D][33] float tile per wave and 2 x D floats per wave (one workgroup per compute unit)
  static constexpr int kSumTile = D * 33;
  static constexpr int total_factors(int waves) {
    const int sums = (waves * kSumTile + 2 * waves * D) * 4;
    return sums > total(waves) ? sums : total(waves);
  }
};
template <int D, int WAVES, bool FACTORS, int MAP>
__global__ __launch_bounds__(WAVES * 64, FACTORS ? 1 : 2) void k_vmod_bwd_map(Geom g, const unsigned char* __restrict__ wpk,
                                                             View Tin, View V, View dO, View out,
                                                             const unsigned char* __restrict__ saved,
                                                             VmodFactors fac) {
  using SM = VSmem<D>;
  using SB = VSmemB<D>;
  constexpr int NRB = D / 32, NKS = D / 16;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  const int r = lane % 32, gl = lane / 32;
  const int L = lane % 16, q = lane / 16;
  load_map<D, WAVES * 64>(smem, wpk + MAP * VPacked<D>::kBytes);
  if (threadIdx.x < D)
    *reinterpret_cast<u32x4*>(smem + SB::kOtherVec + threadIdx.x * 16) =
        *reinterpret_cast<const u32x4*>(wpk + (1 - MAP) * VPacked<D>::kBytes + VPacked<D>::kB1 + threadIdx.x * 16);
  __syncthreads();
  const unsigned char* wm_other = smem + SB::kOtherVec - SM::kVec;  // only its vectors are there
  unsigned char* otile = smem + SB::kTiles + wave * RowTile<D, kRowsOutB>::kBytes;
  int a_off[NKS];
  first_layer_offsets<D>(lane, a_off);
  // Transpose reads of a [k][m] matrix copy (row = contraction index, 16 per k-step: slot (gl, j)
  // is row 8 gl + j) for the lane's A operand row: lanes 4j'..4j'+3 of a 16-lane group supply row
  // j' of a 4 x 16 block, and lane L receives its column L, which is to be matrix column
  // 32 blk + 16 (q % 2) + swap23(L): the lane that supplies block columns 4c..4c+3 therefore
  // addresses the matrix columns of group c with its two bits exchanged.
  int t_off[2][NRB];
#pragma unroll
  for (int hi = 0; hi < 2; ++hi)
#pragma unroll
    for (int blk = 0; blk < NRB; ++blk) {
      const int c = L % 4, cs = ((c & 1) << 1) | (c >> 1);
      const int row = 8 * gl + 4 * hi + L / 4;
      const int col = 32 * blk + 16 * (q % 2) + 4 * cs;
      t_off[hi][blk] = tile_off<SM::kRowB>(row, col >> 3) + ((col & 7) << 1);
    }
  TileWalk tw;
  tw.tiles_per_row = (g.N + 31) / 32;
  tw.total = tw.tiles_per_row * g.B * g.H;
  tw.H = g.H;
  const int stride = gridDim.x * WAVES;
  const int lane16 = lane * 16;
  const View& X = MAP == 0 ? Tin : V;
  // FACTORS: the lane's sums of dm * u-hat and of dm over its tokens (see norm_backward)
  float ag[FACTORS ? D / 2 : 1], ab[FACTORS ? D / 2 : 1];
#pragma unroll
  for (int i = 0; i < (FACTORS ? D / 2 : 1); ++i) ag[i] = ab[i] = 0.0f;
  for (int tile = blockIdx.x * WAVES + wave; tile < tw.total; tile += stride) {
    int b, h, n0;
    tw.decode(tile, b, h, n0);
    const unsigned char* slot_rd[2] = {saved + static_cast<int64_t>(tile) * SavedTile<D>::kBytes, nullptr};
    slot_rd[1] = slot_rd[0];
    asm volatile("" : "+s"(slot_rd[1]));
    const float rstd = *reinterpret_cast<const float*>(slot_rd[0] + SavedTile<D>::kUhat + MAP * 256 + lane * 4);
    const bf16_t* drow[2] = {dO.row<const bf16_t>(b, h, n0 + r < g.N ? n0 + r : g.N - 1) + 8 * gl, nullptr};
    drow[1] = drow[0];
    asm volatile("" : "+v"(drow[1]));
    auto loader = [&](int which, int ks, int pass) -> u32x4 {
      if (which == 0) return load_global16(drow[pass] + 16 * ks);
      const int m = which == 1 ? MAP : 1 - MAP;
      return load_global16(slot_rd[pass] + (m * NKS + ks) * 1024 + lane16);
    };
    const int64_t frow = FACTORS && n0 + r < g.N ? g.th(b, h, n0 + r) * D + 8 * gl : -1;
    auto frow_of = [&](bf16_t* base) -> bf16_t* { return FACTORS && frow >= 0 ? base + frow : nullptr; };
    u32x4 x[NKS];  // the map's input rows, for the first layer's recomputation
    load_row<D>(X, b, h, n0 + r, g.N, gl, x);
    u32x4 du[NKS];
    const float sc = norm_backward<D>(smem, wm_other, gl, loader, rstd, du, frow_of(fac.dU[MAP]), ag, ab,
                                      frow >= 0 ? 1.0f : 0.0f);
    __builtin_amdgcn_sched_barrier(0);
    f32x16 dx[NRB];
    map_backward<D>(smem, a_off, t_off, gl, x, du, dx, frow_of(fac.G[MAP]), frow_of(fac.dH[MAP]), sc);
    __builtin_amdgcn_sched_barrier(0);
    // what the result is added to: dO (MAP 0) or the operator's own dV (MAP 1), this lane's row
    load_row<D>(MAP == 0 ? dO : out, b, h, n0 + r, g.N, gl, x);
    u32x4 w[NRB][2];
#pragma unroll
    for (int ib = 0; ib < NRB; ++ib) {
      f32x16 o;
#pragma unroll
      for (int i = 0; i < 16; ++i) o[i] = __builtin_fmaf(dx[ib][i], sc, row_entry<D>(x, ib, i));
      pack_block(o, w[ib]);
    }
#pragma unroll
    for (int pass = 0; pass < 32 / kRowsOutB; ++pass) {
      put_rows<D, kRowsOutB>(w, pass, lane, otile);
      flush_rows<D, kRowsOutB>(pass, lane, otile, [&](int t) -> bf16_t* {
        return n0 + t < g.N ? out.row<bf16_t>(b, h, n0 + t) : nullptr;
      });
    }
  }
  if constexpr (FACTORS) {
    // The workgroup's share of dgamma and dbeta: per wave the 32 token lanes of a channel are added
    // in lane order through a [channel][33] LDS tile (the weights are done with), then the four
    // waves in wave order; one partial per workgroup.
    constexpr int kTile = SB::kSumTile;
    __syncthreads();
    float* red = reinterpret_cast<float*>(smem) + wave * kTile;
    float* wsum = reinterpret_cast<float*>(smem) + WAVES * kTile;  // [2][WAVES][D]
    auto wave_sum = [&](const float (&src)[FACTORS ? D / 2 : 1], int which) {
#pragma unroll
      for (int i = 0; i < D / 2; ++i) red[(16 * (i / 8) + 8 * gl + i % 8) * 33 + r] = src[i];
      wave_lds_sync();
      for (int c = lane; c < D; c += kWave) {
        float sum = 0.0f;
#pragma unroll
        for (int k = 0; k < 32; ++k) sum += red[c * 33 + k];
        wsum[(which * WAVES + wave) * D + c] = sum;
      }
      wave_lds_sync();
    };
    wave_sum(ag, 0);
    wave_sum(ab, 1);
    __syncthreads();
    for (int i = threadIdx.x; i < 2 * D; i += WAVES * 64) {
      const int which = i / D, c = i % D;
      float sum = wsum[(which * WAVES) * D + c];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) sum += wsum[(which * WAVES + w) * D + c];
      fac.gb_part[(static_cast<int64_t>(blockIdx.x) * 2 + which) * D + c] = sum;
    }
  }
}

// Adds the `nparts` per-workgroup partials of dgamma and dbeta (see VmodFactors) in order: eight
// slices of the partials per output, each with sixteen loads in flight, then the slices in order.
// grid (2 D / 32), block 256.
__global__ __launch_bounds__(256) void k_vmod_gb_reduce(const float* __restrict__ part, int nparts, int D,
                                                        float* __restrict__ dgamma, float* __restrict__ dbeta) {
  __shared__ float sh[8][32];
  const int o = blockIdx.x * 32 + threadIdx.x % 32, slice = threadIdx.x / 32;  // o = which * D + c
  const int per = (nparts + 7) / 8;
  const int p0 = slice * per, p1 = p0 + per < nparts ? p0 + per : nparts;
  float sum = 0.0f;
  for (int p = p0; p < p1; p += 16) {
    float ld[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) ld[k] = p + k < p1 ? part[static_cast<int64_t>(p + k) * 2 * D + o] : 0.0f;
#pragma unroll
    for (int k = 0; k < 16; ++k) sum += ld[k];
  }
  sh[slice][threadIdx.x % 32] = sum;
  __syncthreads();
  if (slice == 0) {
    float t = sh[0][threadIdx.x];
#pragma unroll
    for (int k = 1; k < 8; ++k) t += sh[k][threadIdx.x];
    (o < D ? dgamma : dbeta)[o % D] = t;
  }
}

// C[i][j] = sum over tokens of A[t][i] B[t][j] and z[i] = sum over tokens of A[t][i] for two bf16
// [B, H, N, D] views, on the matrix cores.  grid (parts, D / 64, jobs), block 256: workgroup half
// blockIdx.y owns rows 64 y .. 64 y + 63 of C; each wave streams 64-token sub-tiles (both row tiles
// through its private LDS, both operands by transpose reads, k = token) of the flat list over all
// (batch row, head) pairs; the workgroup writes one partial:
//   part[(job * parts + blockIdx.x) * (D / 64) + y] = [C rows 64 x D | z 64] floats (the four waves
//   summed in order).  grid.z = jobs: the (A, B) pairs of the list.
template <int D>
struct TnSmem {
  static constexpr int kStride = D * 2 + 32;
  static constexpr int kTile = 64 * kStride;
  static constexpr int kTotal = 4 * 2 * kTile;
};
// The token contractions of one backward as a list: one launch forms them all (blockIdx.z picks
// the job), a second one adds up the partials of each.
constexpr int kTnJobs = 4;
struct TnJob {
  View A, Bv;
  float* M;
  float* v;
};
struct TnJobs {
  TnJob j[kTnJobs];
};
template <int D>
__global__ __launch_bounds__(256) void k_tn_mfma(Geom g, TnJobs jobs, float* __restrict__ part) {
  using SM = TnSmem<D>;
  const View A = jobs.j[blockIdx.z].A, Bv = jobs.j[blockIdx.z].Bv;
  constexpr int NCB = D / 32;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  unsigned char* as = smem + wave * 2 * SM::kTile;
  unsigned char* bs = as + SM::kTile;
  const int r = lane % 32, gq = lane / 32, L = lane % 16, q = lane / 16;
  const int half = blockIdx.y;
  f32x16 acc[2][NCB], zacc[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
    for (int i = 0; i < 16; ++i) zacc[rb][i] = 0.0f;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.0f;
  }
  u32x4 ones;
  ones[0] = ones[1] = ones[2] = ones[3] = 0x3f803f80u;  // bf16 1.0 pairs
  const int per_row = (g.N + 63) / 64;
  const int total = per_row * g.B * g.H;
  const int stride = gridDim.x * 4;
  TileRegs<D, 64> ta, tb;
  auto fetch = [&](int st) {
    const int row = st / per_row, n0 = (st % per_row) * 64;
    fetch_tile<D, 64>(A, row / g.H, row % g.H, n0, g.N, lane, ta);
    fetch_tile<D, 64>(Bv, row / g.H, row % g.H, n0, g.N, lane, tb);
  };
  int st = blockIdx.x * 4 + wave;
  if (st < total) fetch(st);
  for (; st < total; st += stride) {
    put_tile<D, 64>(ta, lane, as, SM::kStride);
    put_tile<D, 64>(tb, lane, bs, SM::kStride);
    if (st + stride < total) fetch(st + stride);
    wave_lds_sync();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int krow = 16 * ks + 8 * gq + L / 4;  // token row this lane addresses for the transpose reads
      u32x4 a[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
        const unsigned char* p = as + krow * SM::kStride + (64 * half + 32 * rb + 16 * (q % 2) + 4 * (L % 4)) * 2;
        const u32x2 lo = lds_read_tr16(p);
        const u32x2 hi = lds_read_tr16(p + 4 * SM::kStride);
        a[rb][0] = lo[0];
        a[rb][1] = lo[1];
        a[rb][2] = hi[0];
        a[rb][3] = hi[1];
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const unsigned char* p = bs + krow * SM::kStride + (32 * cb + 16 * (q % 2) + 4 * (L % 4)) * 2;
        const u32x2 lo = lds_read_tr16(p);
        const u32x2 hi = lds_read_tr16(p + 4 * SM::kStride);
        u32x4 b;
        b[0] = lo[0];
        b[1] = lo[1];
        b[2] = hi[0];
        b[3] = hi[1];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) acc[rb][cb] = mfma32(a[rb], b, acc[rb][cb]);
      }
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) zacc[rb] = mfma32(a[rb], ones, zacc[rb]);
    }
    wave_lds_sync();
  }
  // the four waves' sums through LDS (the row tiles are done with), added in wave order, one
  // partial per workgroup
  constexpr int PW = 64 * D + 64;
  static_assert(4 * PW * 4 <= SM::kTotal, "the waves' tiles fit the LDS the row tiles used");
  __syncthreads();
  float* mine = reinterpret_cast<float*>(smem) + wave * PW;
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int row = 32 * rb + d_row(i, gq);
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) mine[row * D + 32 * cb + r] = acc[rb][cb][i];
      if (r == 0) mine[64 * D + row] = zacc[rb][i];
    }
  __syncthreads();
  const float* all = reinterpret_cast<const float*>(smem);
  float* out = part + ((static_cast<int64_t>(blockIdx.z) * gridDim.x + blockIdx.x) * gridDim.y + half) * PW;
  for (int k = threadIdx.x; k < PW; k += 256) out[k] = ((all[k] + all[PW + k]) + all[2 * PW + k]) + all[3 * PW + k];
}

// Adds the `nparts` partials of k_tn_mfma in order: M[j * D + i] = C[i][j] (the transpose: the
// products are formed with the gradient as the A operand) and v[i] = z[i].
// grid (D * D / 256, jobs), block 256.
template <int D>
__global__ void k_tn_reduce(const float* __restrict__ part, int nparts, TnJobs jobs) {
  constexpr int HALVES = D / 64;
  constexpr int64_t PW = 64 * D + 64;
  float* __restrict__ M = jobs.j[blockIdx.y].M;
  float* __restrict__ v = jobs.j[blockIdx.y].v;
  const int idx = blockIdx.x * 256 + threadIdx.x;  // i * D + j
  const int i = idx / D, j = idx % D;
  const float* base = part + (static_cast<int64_t>(blockIdx.y) * nparts * HALVES + i / 64) * PW;
  // eight partials' loads in flight at a time, added in order
  auto sum = [&](int64_t off) {
    float s = 0.0f;
    for (int p = 0; p < nparts; p += 8) {
      float ld[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) ld[k] = p + k < nparts ? base[static_cast<int64_t>(p + k) * HALVES * PW + off] : 0.0f;
#pragma unroll
      for (int k = 0; k < 8; ++k) s += ld[k];
    }
    return s;
  };
  M[j * D + i] = sum((i % 64) * D + j);
  if (j == 0) v[i] = sum(64 * D + i % 64);
}

template <int D>
hla_status prepare_t() {
  HLA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_vmod_fwd_mfma<D, kWavesV>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, VSmem<D>::total(kWavesV)));
  HLA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_vmod_bwd_map<D, kWavesV, false, 0>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, VSmemB<D>::total(kWavesV)));
  HLA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_vmod_bwd_map<D, kWavesV, false, 1>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, VSmemB<D>::total(kWavesV)));
  HLA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_vmod_bwd_map<D, kWavesV, true, 0>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, VSmemB<D>::total_factors(kWavesV)));
  HLA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_vmod_bwd_map<D, kWavesV, true, 1>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, VSmemB<D>::total_factors(kWavesV)));
  HLA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(k_tn_mfma<D>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, TnSmem<D>::kTotal));
  return HLA_OK;
}

int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  return n;
}

template <int D>
hla_status forward_t(hla_handle* hd, const hla_call_args& a) {
  const Geom& g = hd->g;
  const int64_t tiles = static_cast<int64_t>((g.N + 31) / 32) * g.B * g.H;
  const int grid = static_cast<int>(std::min<int64_t>(compute_units(), (tiles + kWavesV - 1) / kWavesV));
  return launch(hd, "vmod_forward", k_vmod_fwd_mfma<D, kWavesV>, dim3(grid), dim3(kWavesV * 64),
                VSmem<D>::total(kWavesV), a.stream, g, static_cast<const unsigned char*>(hd->vmod_wpk),
                hd->vmod_ln_eps, vmod_view(hd->vmod_T, g), a.V, a.O, hd->vmod_wpk + vmod_mfma_packed_bytes(hd));
}

// the six factor arrays inside hd->vmod_wg_rows (bf16 [max_th][d] each); the workgroups' partial
// sums of dgamma and dbeta go to the head of the contractions' partial buffer, which is free while
// the backward kernels run
VmodFactors factor_arrays(const hla_handle* hd) {
  VmodFactors f;
  bf16_t* base = reinterpret_cast<bf16_t*>(hd->vmod_wg_rows);
  const int64_t per = hd->max_th * hd->g.d;
  for (int m = 0; m < 2; ++m) {
    f.dU[m] = base + (3 * m + 0) * per;
    f.dH[m] = base + (3 * m + 1) * per;
    f.G[m] = base + (3 * m + 2) * per;
  }
  f.gb_part = hd->vmod_wg_partial;
  return f;
}

// the backward of map MAP: MAP 0 writes dT (before the operator's backward), MAP 1 adds the
// modulation's share to the dV the operator's backward has written
template <int D, int MAP>
hla_status backward_map_t(hla_handle* hd, const hla_call_args& a, View out) {
  const Geom& g = hd->g;
  const int64_t tiles = static_cast<int64_t>((g.N + 31) / 32) * g.B * g.H;
  const int grid = static_cast<int>(std::min<int64_t>(2 * compute_units(), (tiles + kWavesV - 1) / kWavesV));
  const unsigned char* saved = hd->vmod_wpk + vmod_mfma_packed_bytes(hd);
  const char* name = MAP == 0 ? "vmod_backward" : "vmod_backward_value";
  if (hd->vmod_wg_on) {
    HLA_TRY(launch(hd, name, k_vmod_bwd_map<D, kWavesV, true, MAP>, dim3(grid), dim3(kWavesV * 64),
                   VSmemB<D>::total_factors(kWavesV), a.stream, g, static_cast<const unsigned char*>(hd->vmod_wpk),
                   vmod_view(hd->vmod_T, g), a.V, a.dO, out, saved, factor_arrays(hd)));
    const hla_vmod_weight_grads& o = hd->vmod_wg_out[MAP];
    return launch(hd, "vmod_weight_grads_norm", k_vmod_gb_reduce, dim3(2 * D / 32), dim3(256), 0, a.stream,
                  static_cast<const float*>(hd->vmod_wg_partial), grid, D, o.dgamma, o.dbeta);
  }
  return launch(hd, name, k_vmod_bwd_map<D, kWavesV, false, MAP>, dim3(grid), dim3(kWavesV * 64),
                VSmemB<D>::total(kWavesV), a.stream, g, static_cast<const unsigned char*>(hd->vmod_wpk),
                vmod_view(hd->vmod_T, g), a.V, a.dO, out, saved, VmodFactors{});
}
template <int D>
hla_status backward_t(hla_handle* hd, const hla_call_args& a) {
  return backward_map_t<D, 0>(hd, a, vmod_view(hd->vmod_dT, hd->g));
}

constexpr int kTnBlocks = 128;  // workgroups (and partials) per row half of a token contraction

template <int D>
hla_status weight_grads_t(hla_handle* hd, const hla_call_args& a) {
  const Geom& g = hd->g;
  const VmodFactors f = factor_arrays(hd);
  TnJobs jobs;
  for (int m = 0; m < 2; ++m) {
    const hla_vmod_weight_grads& o = hd->vmod_wg_out[m];
    jobs.j[2 * m + 0] = TnJob{vmod_view(f.dU[m], g), vmod_view(f.G[m], g), o.dW2, o.db2};
    jobs.j[2 * m + 1] = TnJob{vmod_view(f.dH[m], g), m == 0 ? vmod_view(hd->vmod_T, g) : a.V, o.dW1, o.db1};
  }
  const int64_t subtiles = static_cast<int64_t>((g.N + 63) / 64) * g.B * g.H;
  const int blocks = static_cast<int>(std::min<int64_t>(kTnBlocks, (subtiles + 3) / 4));
  HLA_TRY(launch(hd, "vmod_weight_grads_gemm", k_tn_mfma<D>, dim3(blocks, D / 64, kTnJobs), dim3(256),
                 TnSmem<D>::kTotal, a.stream, g, jobs, hd->vmod_wg_partial));
  return launch(hd, "vmod_weight_grads_reduce", k_tn_reduce<D>, dim3(D * D / 256, kTnJobs), dim3(256), 0, a.stream,
                static_cast<const float*>(hd->vmod_wg_partial), blocks, jobs);
}

template <int D>
hla_status add_t(hla_handle* hd, const hla_call_args& a) {
  return backward_map_t<D, 1>(hd, a, a.dV);
}

}  // namespace

bool vmod_mfma_supported(const hla_handle* hd) {
  return hd->path == HLA_PATH_MFMA && hd->cfg.io_dtype == HLA_BF16 && (hd->g.d == 64 || hd->g.d == 128);
}
size_t vmod_mfma_packed_bytes(const hla_handle* hd) {
  return 2 * static_cast<size_t>(hd->g.d == 64 ? VPacked<64>::kBytes : VPacked<128>::kBytes);
}
// packed weights, then what the forward keeps for the backward: one SavedTile per 32-token tile
size_t vmod_mfma_workspace_bytes(const hla_handle* hd) {
  const int64_t tiles = hd->max_th / 32 + static_cast<int64_t>(hd->cfg.max_heads) * hd->cfg.max_seqs + 1;
  const size_t per = hd->g.d == 64 ? SavedTile<64>::kBytes : SavedTile<128>::kBytes;
  return vmod_mfma_packed_bytes(hd) + static_cast<size_t>(tiles) * per;
}
hla_status vmod_mfma_prepare_kernels(const hla_handle* hd) {
  return hd->g.d == 64 ? prepare_t<64>() : prepare_t<128>();
}
hla_status vmod_mfma_set_weights(hla_handle* hd, const hla_vmod_weights* maps, hipStream_t s) {
  const int d = hd->g.d;
  const size_t per = vmod_mfma_packed_bytes(hd) / 2;
  for (int m = 0; m < 2; ++m)
    HLA_TRY(launch(hd, "vmod_pack", k_vmod_pack_mfma<bf16_t>, dim3(64), dim3(256), 0, s,
                   static_cast<const bf16_t*>(maps[m].W1), static_cast<const bf16_t*>(maps[m].b1),
                   static_cast<const bf16_t*>(maps[m].W2), static_cast<const bf16_t*>(maps[m].b2),
                   static_cast<const bf16_t*>(maps[m].gamma), static_cast<const bf16_t*>(maps[m].beta), d,
                   hd->vmod_wpk + m * per));
  return HLA_OK;
}
hla_status vmod_mfma_forward(hla_handle* hd, const hla_call_args& a) {
  return hd->g.d == 64 ? forward_t<64>(hd, a) : forward_t<128>(hd, a);
}
hla_status vmod_mfma_backward(hla_handle* hd, const hla_call_args& a) {
  return hd->g.d == 64 ? backward_t<64>(hd, a) : backward_t<128>(hd, a);
}
// the modulation's weight gradients from the factors the backward kernel left (it must have run
// with hd->vmod_wg_on)
hla_status vmod_mfma_weight_grads(hla_handle* hd, const hla_call_args& a) {
  return hd->g.d == 64 ? weight_grads_t<64>(hd, a) : weight_grads_t<128>(hd, a);
}
// floats the factor arrays and the partials of the contractions need
int64_t vmod_mfma_factor_floats(const hla_handle* hd) { return 3 * hd->max_th * hd->g.d; }  // six bf16 arrays
int64_t vmod_mfma_partial_floats(const hla_handle* hd) {
  return static_cast<int64_t>(kTnJobs) * kTnBlocks * (hd->g.d / 64) * (64 * hd->g.d + 64);
}
hla_status vmod_mfma_add_value_grads(hla_handle* hd, const hla_call_args& a) {
  return hd->g.d == 64 ? add_t<64>(hd, a) : add_t<128>(hd, a);
}

}  // namespace hla
