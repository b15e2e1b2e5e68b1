// MFMA path: bf16 matrix-core kernels for gfx950 over the symmetric (monomial) form of the
// degree-3 (d_phi = 6) or degree-2 (d_phi = 12) feature tensor (see hla_mfma_common.h; SY below is
// the Sym<F, d_phi> that describes it, MP = SY::MP its padded row count: 64 or 96).  Forward core:
//   k_state   : per chunk of tokens,  Csym += S^T V,  zsym += S^T 1     (contraction over tokens)
//   k_reduce  : sums the chunk partials in fixed order and emits the state as MFMA operands
//   k_query   : O^T = Csym^T Qm^T, eta = Qm . zsym, O = num / (eta + eps)
// Lanes serve tokens: in every token-parallel kernel a token is the MFMA *column*, so per-token
// scalars (eta, den, s) live in one lane pair and never need a cross-lane broadcast.
#include <type_traits>

#include "hla_handle.h"
#include "hla_mfma_common.h"

namespace hla {


namespace {

using namespace mf;


constexpr int kStaggerCore = 5;    // start-up stagger unit of the two core backward kernels (see stagger_start)
constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
// k_query: with a state of 64 rows the workgroup keeps the state's operand image in LDS and three
// workgroups share a compute unit; with more rows the image stays in registers (an LDS copy would
// not buy a third wave per SIMD) and two do.  The grid aims at one resident round.
template <class SY>
constexpr bool query_image_in_lds() {
  return SY::MP <= 64;
}
template <class SY>
constexpr int query_target() {
  return query_image_in_lds<SY>() ? 768 : 496;
}
constexpr int kMinChunk = 256;     // smallest chunk pick_chunk returns
constexpr int kCausalChunk = 256;  // tokens per chunk of the causal scan: eight 32-token tiles
// (128-token chunks, one tile per wave of a four-wave workgroup and two workgroups per compute
// unit, were measured: the tile kernels gain 20-25 % -- a token meets 2.5 tiles of its chunk instead
// of 4.5 -- but the scans, serial in the number of chunks, lose twice that.)
static_assert(kCausalChunk == 256, "the tile kernels' wave-to-tile maps assume eight tiles per chunk");
// Tile `i` (0 or 1) of wave `w` of a four-wave workgroup: w and its mirror image 7 - w, equal
// shares of the triangle of tile pairs.  Eight-wave workgroups give the same two tiles to the two
// waves of a SIMD, w and w + 4.
__device__ __forceinline__ int chunk_tile_of(int w, int i) { return i == 0 ? w : kCausalChunk / 32 - 1 - w; }
constexpr int kMinQueryBlock = 128;  // smallest block pick_query_block returns
constexpr int kChunkTarget = 256;  // workgroups aimed at by the chunked (token-contraction) kernels: one per CU
constexpr int kChunkGrain = 64;    // chunk sizes are multiples of this many tokens (one wave step of k_state)
constexpr int kReduceSlices = 8;   // slices of the state per (sequence, head) in k_reduce

// Where canonical monomial m sits among the (g, slot) pairs.
struct SlotMap {
  int8_t g[128];
  int8_t s[128];
};

template <class SY>
SlotMap make_slot_map() {
  SlotMap sm{};
  for (int m = 0; m < 128; ++m) sm.g[m] = sm.s[m] = -1;
  for (int g = 0; g < 2; ++g)
    for (int s = 0; s < SY::NS; ++s) {
      const int m = SY::slot_canon(g, s);
      if (m < 0) continue;  // padding (the second copy of a self-mirrored monomial)
      sm.g[m] = static_cast<int8_t>(g);
      sm.s[m] = static_cast<int8_t>(s);
    }
  return sm;
}

// Per-unit device state of the MFMA path (all inside hd->path_ws).
template <class SY, int D>
struct StateLayout {
  static constexpr int MP = SY::MP;
  static constexpr int SP = SY::SP;
  static constexpr int64_t kF32 = static_cast<int64_t>(MP) * D + MP;  // canonical C rows, then z
  static constexpr int64_t kOpElems = static_cast<int64_t>(MP) * D;   // bf16 elements per operand array
  // bytes per unit: opA, opB (bf16), zslot (fp32 [2][SP])
  static constexpr int64_t kOpBytes = 2 * kOpElems * 2 + 2 * SP * 4;
};

// ---- sum of per-wave accumulator tiles over the four waves of a workgroup ------------------------
// Every wave holds a [MP rows x D] fp32 tile in MFMA accumulator layout (acc[rb][cb][i]: row
// 32rb + d_row(i, gl), column 32cb + r) and an MP-vector zl (element (MP/2) gl + k, replicated
// over r).  Fixed order (w0 + w1) + (w2 + w3), LDS regions of (MP D + MP) floats;
// the sum (read through summed4 / summed1) has tile row `row` at floats [row * D, row * D + D) and
// the vector at MP D.
template <int D, int MP>
struct WaveSum {
  static constexpr int kRegion = MP * D + MP;          // floats
  // a region per wave where LDS has room for four (one pass, everybody adds); else two regions
  // and the waves add pairwise through their registers
  static constexpr bool kFlat = 4 * kRegion * 4 <= 160 * 1024;
  static constexpr int kBytes = (kFlat ? 4 : 2) * kRegion * 4;
};
template <int D, int MP>
__device__ __forceinline__ void sum_over_waves(f32x16 (&acc)[MP / 32][D / 32], float (&zl)[MP / 2],
                                               float* lds, int wave, int lane) {
  constexpr int NCB = D / 32, NRM = MP / 32, HALF = MP / 2;
  using WS = WaveSum<D, MP>;
  const int r = lane % 32, gl = lane / 32;
  auto put = [&](float* reg) {
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) reg[(32 * rb + d_row(i, gl)) * D + 32 * cb + r] = acc[rb][cb][i];
    if (r == 0) {
#pragma unroll
      for (int k = 0; k < HALF; ++k) reg[MP * D + HALF * gl + k] = zl[k];
    }
  };
  if constexpr (WS::kFlat) {
    // every wave leaves its tile in a region of its own; summed4 / summed1 below form the sum
    __syncthreads();
    put(lds + wave * WS::kRegion);
    __syncthreads();
    return;
  }
  auto add = [&](const float* reg) {
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) acc[rb][cb][i] += reg[(32 * rb + d_row(i, gl)) * D + 32 * cb + r];
#pragma unroll
    for (int k = 0; k < HALF; ++k) zl[k] += reg[MP * D + HALF * gl + k];
  };
  float* reg = lds + (wave / 2) * WS::kRegion;
  __syncthreads();
  if (wave % 2 == 1) put(reg);
  __syncthreads();
  if (wave % 2 == 0) add(reg);
  __syncthreads();
  if (wave == 2) put(lds);
  __syncthreads();
  if (wave == 0) {
    add(lds);
    put(lds);
  }
  __syncthreads();
}

// Entries of the sum after sum_over_waves: floats [4i, 4i + 4) and float i of the summed region.
template <int D, int MP>
__device__ __forceinline__ f32x4 summed4(const float* lds, int i) {
  using WS = WaveSum<D, MP>;
  static_assert(WS::kRegion % 4 == 0, "16-byte pieces");
  const f32x4 a = reinterpret_cast<const f32x4*>(lds)[i];
  if constexpr (!WS::kFlat) return a;
  const f32x4 b = reinterpret_cast<const f32x4*>(lds + WS::kRegion)[i];
  const f32x4 c = reinterpret_cast<const f32x4*>(lds + 2 * WS::kRegion)[i];
  const f32x4 d = reinterpret_cast<const f32x4*>(lds + 3 * WS::kRegion)[i];
  f32x4 v;
#pragma unroll
  for (int x = 0; x < 4; ++x) v[x] = (a[x] + b[x]) + (c[x] + d[x]);
  return v;
}
template <int D, int MP>
__device__ __forceinline__ float summed1(const float* lds, int i) {
  using WS = WaveSum<D, MP>;
  if constexpr (!WS::kFlat) return lds[i];
  return (lds[i] + lds[WS::kRegion + i]) + (lds[2 * WS::kRegion + i] + lds[3 * WS::kRegion + i]);
}

// ---- k_state ----------------------------------------------------------------------------------
template <int D, int MP>
struct StateSmem {
  static constexpr int kVStride = D * 2 + 32;   // bytes per token row of the V tile
  static constexpr int kSStride = MP * 2 + 32;  // bytes per token row of the S tile (MP monomial cols)
  static constexpr int kVBytes = 64 * kVStride;
  static constexpr int kSBytes = 64 * kSStride;
  static constexpr int kWaveBytes = kVBytes + kSBytes;
  static constexpr int kRedBytes = WaveSum<D, MP>::kBytes;
  static constexpr int kTotal = kWaves * kWaveBytes > kRedBytes ? kWaves * kWaveBytes : kRedBytes;
};

// grid (chunks, H), block 256.  Each wave streams 64-token sub-tiles w, w+4, .. of the chunk
// through its private LDS region; the four waves' accumulators are summed in wave order at the
// end and written as one partial state.
// MODE 1 (backward of the causal variant): the same contraction for the gradient state of a chunk,
//   sum_i w_i (Qm_i / den_i) (x) dO_i   and   sum_i w_i (s_i den_i) (Qm_i / den_i),
// with the QUERY monomials of the tokens, V = the dO rows, den / sv the saved denominators and
// the s_i of the query-side kernel, w_i = decay^(i - t0 + 1) (the chunk as seen from the token in
// front of it).
// PER_WAVE (the 256-token chunks of the causal scan): a wave serves a whole chunk of its own
// (chunk blockIdx.x * 4 + wave of the `nchunks`) and writes its accumulators straight to the
// chunk's partial, 128-byte runs per store: no sum over the waves, no barrier.
template <class SY, int D, int MODE = 0, bool PER_WAVE = false>
__global__ __launch_bounds__(kThreads) void k_state(Geom g, const BlockEnt* __restrict__ chunks,
                                                    const float* __restrict__ feat, View V,
                                                    float* __restrict__ partial,
                                                    int64_t partial_stride, float log2_decay,
                                                    const float* __restrict__ den,
                                                    const float* __restrict__ sv, int nchunks) {
  constexpr int DP = SY::DPHI, F = SY::F, MP = SY::MP;
  using SM = StateSmem<D, MP>;
  constexpr int NCB = D / 32;      // column blocks of the state
  constexpr int NRM = MP / 32;     // row blocks of the state
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  unsigned char* vs = smem + wave * SM::kWaveBytes;
  unsigned char* ss = vs + SM::kVBytes;
  const int chunk_index = PER_WAVE ? static_cast<int>(blockIdx.x) * kWaves + wave : static_cast<int>(blockIdx.x);
  BlockEnt e = chunks[PER_WAVE && chunk_index >= nchunks ? 0 : chunk_index];
  if (PER_WAVE && chunk_index >= nchunks) e.t1 = e.t0;  // no chunk for this wave
  const int h = blockIdx.y;
  const int gq = lane / 32;                   // MFMA operand coordinates
  const int L = lane % 16, q = lane / 16;
  const int first = PER_WAVE ? e.t0 : e.t0 + wave * 64, step = PER_WAVE ? 64 : kWaves * 64;

  f32x16 acc[NRM][NCB];
  f32x16 zacc[NRM];
#pragma unroll
  for (int rb = 0; rb < NRM; ++rb) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) zacc[rb][i] = 0.0f;
  }
  u32x4 ones;
  ones[0] = ones[1] = ones[2] = ones[3] = 0x3f803f80u;  // bf16 1.0 pairs
  u32x4 tws[MODE == 1 ? 4 : 1];  // MODE 1: per-token z weights in place of the ones

  // the next sub-tile's V rows and key features are fetched while the current one is consumed
  TileRegs<D, 64> vt;
  constexpr int NFV = MODE == 0 ? F * DP : DP;  // feature values a token needs
  float kf[F * DP];
  float dnf = 1.0f, svf = 0.0f;  // MODE 1: the token's denominator and s
  auto fetch = [&](int n0) {
    fetch_tile<D, 64>(V, e.b, h, n0, e.t1, lane, vt);
    const int n = n0 + lane;
    if (n < e.t1) {
      // pair p of the tile's 32 tokens is one 256-byte run: an 8-byte load per lane and pair
      const int64_t th = g.th(e.b, h, n);
      const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(th, MODE == 0 ? DP : 0));
#pragma unroll
      for (int p = 0; p < NFV / 2; ++p) {
        const f32x2 v = f[32 * p];
        kf[2 * p] = v[0];
        kf[2 * p + 1] = v[1];
      }
      if constexpr (MODE == 1) {
        dnf = den[th];
        svf = sv[th];
      }
    } else {
#pragma unroll
      for (int a = 0; a < NFV; ++a) kf[a] = 0.0f;
      dnf = 1.0f;
      svf = 0.0f;
    }
  };
  if (first < e.t1) fetch(first);
  for (int n0 = first; n0 < e.t1; n0 += step) {
    put_tile<D, 64>(vt, lane, vs, SM::kVStride);
    // ---- key monomials of token n0 + lane (all NM, canonical order), as bf16 row of the S tile
    {
      float kk[F][DP];
#pragma unroll
      for (int f = 0; f < (MODE == 0 ? F : 1); ++f)
#pragma unroll
        for (int a = 0; a < DP; ++a) kk[f][a] = kf[f * DP + a];
      float scale1 = 1.0f, tw = 0.0f;  // MODE 1: weight of the token's monomials, its z weight
      if constexpr (MODE == 0) {
        if (log2_decay != 0.0f) {
          // causal scan with a decay factor: the chunk's state is taken as seen from the first token
          // behind the chunk, token n weighs decay^(t0 + chunk - n); the key tensor is linear in
          // each factor, so the weight goes on the first one
          const float wgt = __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(e.t0 + kCausalChunk - (n0 + lane)));
#pragma unroll
          for (int a = 0; a < DP; ++a) kk[0][a] *= wgt;
        }
      } else {
        scale1 = 1.0f / dnf;
        if (log2_decay != 0.0f) scale1 *= __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(n0 + lane - e.t0 + 1));
        tw = svf * dnf;
      }
      if (n0 + step < e.t1) fetch(n0 + step);
      float sm[SY::NM];
      if constexpr (MODE == 0) {
        sym_key_monomials_all<SY>(kk, sm);
      } else {
        sym_query_monomials_all<SY>(kk[0], sm);
#pragma unroll
        for (int m = 0; m < SY::NM; ++m) sm[m] *= scale1;
        // the z weights of the sub-tile's tokens as B operands: k-slot (ks, gq, j) is token 16 ks + 8 gq + j
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
          for (int p = 0; p < 4; ++p)
            tws[ks][p] = pack_bf16(__shfl(tw, 16 * ks + 8 * gq + 2 * p, 64), __shfl(tw, 16 * ks + 8 * gq + 2 * p + 1, 64));
      }
      uint32_t packed[MP / 2];
#pragma unroll
      for (int p = 0; p < MP / 2; ++p) {
        const float lo = 2 * p < SY::NM ? sm[2 * p < SY::NM ? 2 * p : 0] : 0.0f;
        const float hi = 2 * p + 1 < SY::NM ? sm[2 * p + 1 < SY::NM ? 2 * p + 1 : 0] : 0.0f;
        packed[p] = pack_bf16(lo, hi);
      }
#pragma unroll
      for (int p = 0; p < MP / 8; ++p) {
        u32x4 w;
        w[0] = packed[4 * p];
        w[1] = packed[4 * p + 1];
        w[2] = packed[4 * p + 2];
        w[3] = packed[4 * p + 3];
        *reinterpret_cast<u32x4*>(ss + lane * SM::kSStride + p * 16) = w;
      }
    }
    wave_lds_sync();
    // ---- Csym[MP x D] += S^T[MP x 64 tokens] V[64 tokens x D]; zsym += S^T 1
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int krow = 16 * ks + 8 * gq + L / 4;  // token row this lane addresses for the transpose read
      u32x4 a[NRM];
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb) {
        const unsigned char* p = ss + krow * SM::kSStride + (32 * rb + 16 * (q % 2) + 4 * (L % 4)) * 2;
        const u32x2 lo = lds_read_tr16(p);
        const u32x2 hi = lds_read_tr16(p + 4 * SM::kSStride);
        a[rb][0] = lo[0];
        a[rb][1] = lo[1];
        a[rb][2] = hi[0];
        a[rb][3] = hi[1];
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const unsigned char* p = vs + krow * SM::kVStride + (32 * cb + 16 * (q % 2) + 4 * (L % 4)) * 2;
        const u32x2 lo = lds_read_tr16(p);
        const u32x2 hi = lds_read_tr16(p + 4 * SM::kVStride);
        u32x4 b;
        b[0] = lo[0];
        b[1] = lo[1];
        b[2] = hi[0];
        b[3] = hi[1];
#pragma unroll
        for (int rb = 0; rb < NRM; ++rb) acc[rb][cb] = mfma32(a[rb], b, acc[rb][cb]);
      }
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb) zacc[rb] = mfma32(a[rb], MODE == 1 ? tws[ks] : ones, zacc[rb]);
    }
    wave_lds_sync();
  }
  if constexpr (PER_WAVE) {
    if (chunk_index >= nchunks) return;
    float* out = partial + (static_cast<int64_t>(chunk_index) * g.H + h) * partial_stride;
    const int r = lane % 32;
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int row = 32 * rb + d_row(i, gq);
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) out[row * D + 32 * cb + r] = acc[rb][cb][i];
        if (r == 0) out[MP * D + row] = zacc[rb][i];
      }
    return;
  }
  // ---- sum the four waves through LDS, then write the partial state (rows = canonical monomials)
  float zl[MP / 2];
#pragma unroll
  for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
    for (int i = 0; i < 16; ++i) zl[16 * rb + i] = zacc[rb][i];
  float* red = reinterpret_cast<float*>(smem);
  sum_over_waves<D, MP>(acc, zl, red, wave, lane);
  float* out = partial + (static_cast<int64_t>(blockIdx.x) * g.H + h) * partial_stride;
  for (int i = threadIdx.x; i < MP * D / 4; i += kThreads)
    reinterpret_cast<f32x4*>(out)[i] = summed4<D, MP>(red, i);
  // vector element (MP/2) gl + 16 rb + i is state row 32 rb + d_row(i, gl)
  if (threadIdx.x < MP) {
    const int gg = threadIdx.x / (MP / 2), k = threadIdx.x % (MP / 2);
    out[MP * D + 32 * (k / 16) + d_row(k % 16, gg)] = summed1<D, MP>(red, MP * D + threadIdx.x);
  }
}

// ---- k_reduce ---------------------------------------------------------------------------------
// grid (num_seqs, H, kReduceSlices), block 256.  Sums the chunk partials of one (sequence, head)
// in chunk order and scatters the bf16 copy of the state into the two operand layouts:
//   opA[rb][ks][lane=(r,gl)][j] = Csym[mono(gl, 8ks+j)][32rb + r]           (rows = channels)
//   opB[rb][ks][lane=(r,gl)][j] = Csym[mono of row 32rb + r][16ks + 8gl + j]  (rows = monomials)
// where state row rho = 32rb + r belongs to (g, s) with rho%32 = 8*(i/4) + 4g + i%4, s = 16rb + i.
// SLOT_ROWS = false: partial rows are canonical monomials (k_state); true: partial row SP g + s is
// slot (g, s) already (k_bwd_query).  A thread owns four consecutive channels of one row; the
// loads of sixteen chunks are in flight together, the additions stay in chunk order.
template <class SY, int D, bool SLOT_ROWS>
__global__ __launch_bounds__(256) void k_reduce(Geom g, const int32_t* __restrict__ seq_chunk_off,
                                                const float* __restrict__ partial,
                                                int64_t partial_stride,
                                                unsigned char* __restrict__ ops, SlotMap sm) {
  using SL = StateLayout<SY, D>;
  constexpr int MP = SL::MP, SP = SL::SP;
  constexpr int VPR = D / 4;                         // float4 per state row
  static_assert(MP * VPR % kReduceSlices == 0, "slices cover the state evenly");
  constexpr int PER = MP * VPR / kReduceSlices;      // float4 per slice
  const int s = blockIdx.x, h = blockIdx.y, sl = blockIdx.z;
  const int c0 = seq_chunk_off[s], c1 = seq_chunk_off[s + 1];
  const int64_t u = static_cast<int64_t>(s) * g.H + h;
  uint16_t* opA = reinterpret_cast<uint16_t*>(ops + u * SL::kOpBytes);
  uint16_t* opB = opA + SL::kOpElems;
  float* zslot = reinterpret_cast<float*>(opB + SL::kOpElems);
  const float* base = partial + static_cast<int64_t>(h) * partial_stride;
  const int64_t cstride = static_cast<int64_t>(g.H) * partial_stride;
  // sixteen chunk loads in flight at a time, the ragged last batch included (its surplus loads
  // repeat the last chunk and are not added): a batch costs one memory round trip, a chunk
  // loaded on its own would cost one each
  auto sum_chunks = [&](const float* p0, auto& acc, auto load) {
    constexpr int NB = 16;
    for (int ch = c0; ch < c1; ch += NB) {
      decltype(load(p0)) v[NB];
#pragma unroll
      for (int k = 0; k < NB; ++k) v[k] = load(p0 + (ch + k < c1 ? ch + k : c1 - 1) * cstride);
#pragma unroll
      for (int k = 0; k < NB; ++k)
        if (ch + k < c1) acc += v[k];
    }
  };
  for (int idx = threadIdx.x; idx < PER; idx += blockDim.x) {
    const int v = sl * PER + idx;
    const int m = v / VPR, c = (v % VPR) * 4;
    f32x4 a;
    a[0] = a[1] = a[2] = a[3] = 0.0f;
    sum_chunks(base + m * D + c, a, [](const float* p) { return *reinterpret_cast<const f32x4*>(p); });
    const int mg = SLOT_ROWS ? m / SP : sm.g[m];
    const int ms = SLOT_ROWS ? m % SP : sm.s[m];
    if (mg >= 0) {
      uint16_t bits[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) bits[e] = f32_to_bf16_bits(a[e]);
      {  // opA: channel c+e is the row, slot (mg, ms) the contraction index
        const int ks = ms / 8, j = ms % 8;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int rb = (c + e) / 32, r = (c + e) % 32;
          opA[((rb * (MP / 16) + ks) * 64 + 32 * mg + r) * 8 + j] = bits[e];
        }
      }
      {  // opB: monomial row from (mg, ms), channels c..c+3 the contraction index (4 consecutive j)
        const int rb = ms / 16, i = ms % 16;
        const int r = 8 * (i / 4) + 4 * mg + i % 4;
        const int ks = c / 16, gl = (c % 16) / 8, j = c % 8;
        u32x2 w;
        w[0] = bits[0] | (static_cast<uint32_t>(bits[1]) << 16);
        w[1] = bits[2] | (static_cast<uint32_t>(bits[3]) << 16);
        *reinterpret_cast<u32x2*>(opB + ((rb * (D / 16) + ks) * 64 + 32 * gl + r) * 8 + j) = w;
      }
    }
  }
  if (sl == 0) {
    for (int m = threadIdx.x; m < MP; m += blockDim.x) {
      float a = 0.0f;
      sum_chunks(base + MP * D + m, a, [](const float* p) { return *p; });
      const int mg = SLOT_ROWS ? m / SP : sm.g[m];
      const int ms = SLOT_ROWS ? m % SP : sm.s[m];
      if (mg >= 0) zslot[mg * SP + ms] = a;
    }
  }
}

// A block-wide copy of BYTES (a multiple of 16) from global memory to LDS in two halves: request()
// puts the loads in flight, commit() writes what arrived to LDS.  Kernels request everything their
// start-up needs from memory in one go and only then consume it, so that the start-up costs one
// round trip to memory instead of one per item.
template <int BYTES, int THREADS>
struct ImageCopy {
  static constexpr int N16 = BYTES / 16, N = (N16 + THREADS - 1) / THREADS;
  u32x4 v[N];
  __device__ __forceinline__ void request(const unsigned char* src) {
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const int i = threadIdx.x + k * THREADS;
      if (N16 % THREADS == 0 || i < N16) v[k] = reinterpret_cast<const u32x4*>(src)[i];
    }
  }
  __device__ __forceinline__ void commit(unsigned char* dst) const {
#pragma unroll
    for (int k = 0; k < N; ++k) {
      const int i = threadIdx.x + k * THREADS;
      if (N16 % THREADS == 0 || i < N16) reinterpret_cast<u32x4*>(dst)[i] = v[k];
    }
  }
};

// ---- k_query ----------------------------------------------------------------------------------
// grid (blocks of pick_query_block tokens, H), block 256.  Wave w serves 32-token tiles w, w+4, ..;
// lane (r, gl): token r of the tile, slot half gl (gl = 1 works on the reversed feature vector).
template <class SY, int D>
__global__ __launch_bounds__(kThreads, query_image_in_lds<SY>() ? 3 : 2) void k_query(Geom g, const BlockEnt* __restrict__ blocks,
                                                    const float* __restrict__ feat,
                                                    const unsigned char* __restrict__ ops, View O,
                                                    float* __restrict__ den) {
  using SL = StateLayout<SY, D>;
  constexpr int SP = SY::SP, MP = SY::MP, DP = SY::DPHI;
  constexpr int NRB = D / 32, NKS = MP / 16;
  // The operand image of the state (rows = channels): shared by the workgroup's waves through LDS
  // and read per product (in registers it would cost 64 of them per lane and one of the three
  // waves a SIMD holds of this kernel), or in registers (see query_image_in_lds).
  constexpr bool kImgLds = query_image_in_lds<SY>();
  constexpr int kImgBytes = kImgLds ? NRB * NKS * 64 * 16 : 0;
  __shared__ __align__(16) unsigned char smem[kImgBytes + kWaves * RowTile<D>::kBytes];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  unsigned char* tile = smem + kImgBytes + wave * RowTile<D>::kBytes;
  const int r = lane % 32, gl = lane / 32;
  const BlockEnt e = blocks[blockIdx.x];
  const int h = blockIdx.y;
  const int64_t u = static_cast<int64_t>(e.seq) * g.H + h;
  const u32x4* opA = reinterpret_cast<const u32x4*>(ops + u * SL::kOpBytes);
  const float* zslot = reinterpret_cast<const float*>(ops + u * SL::kOpBytes + 2 * SL::kOpElems * 2) + gl * SP;
  u32x4 areg[kImgLds ? 1 : NRB * NKS];
  if constexpr (kImgLds) {
    ImageCopy<NRB * NKS * 64 * 16, kThreads> img;
    img.request(reinterpret_cast<const unsigned char*>(opA));
    img.commit(smem);
    __syncthreads();
  } else {
#pragma unroll
    for (int k = 0; k < NRB * NKS; ++k) areg[k] = opA[k * 64 + lane];
  }
  auto state_op = [&](int rb, int ks) -> u32x4 {
    if constexpr (kImgLds)
      return reinterpret_cast<const u32x4*>(smem)[(rb * NKS + ks) * 64 + lane];
    else
      return areg[rb * NKS + ks];
  };
  // The normaliser vector of this lane's half: in registers, or -- when the state has more than 64
  // rows and the registers would no longer allow two waves per SIMD -- in LDS, read per tile.
  constexpr bool kZInLds = SP > 32;
  __shared__ __align__(16) float zs[kZInLds ? 2 * SP : 4];
  float z[kZInLds ? 1 : SP];
  if constexpr (kZInLds) {
    if (threadIdx.x < 2 * SP) zs[threadIdx.x] = (zslot - gl * SP)[threadIdx.x];
    __syncthreads();
  } else {
#pragma unroll
    for (int s = 0; s < SP; ++s) z[s] = zslot[s];
  }
  auto zval = [&](int s) -> float {
    if constexpr (kZInLds)
      return zs[gl * SP + s];
    else
      return z[s];
  };

  // The features of the next tile are loaded while the current one is computed; the loads are
  // unconditional (token clamped into the block) so that they stay in flight across the loop
  // back-edge, and a lane past the block's end zeroes its copy instead.
  float qn[DP];
  auto fetch = [&](int n0) {
    const int n = n0 + r < e.t1 ? n0 + r : e.t1 - 1;
    const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(g.th(e.b, h, n), 0));
#pragma unroll
    for (int p = 0; p < DP / 2; ++p) {  // lane half 1 takes the pairs, and each pair, in reverse
      const f32x2 v = f[32 * (gl ? DP / 2 - 1 - p : p)];
      qn[2 * p] = gl ? v[1] : v[0];
      qn[2 * p + 1] = gl ? v[0] : v[1];
    }
  };
  if (e.t0 + wave * 32 < e.t1) fetch(e.t0 + wave * 32);
  for (int n0 = e.t0 + wave * 32; n0 < e.t1; n0 += kWaves * 32) {
    const int n = n0 + r;
    const bool live = n < e.t1;
    float qf[DP];
#pragma unroll
    for (int c = 0; c < DP; ++c) qf[c] = live ? qn[c] : 0.0f;
    fetch(n0 + kWaves * 32);
    float qm[SP];
    sym_query_monomials<SY>(qf, qm, gl);
    u32x4 b[NKS];
    float eta = 0.0f;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int s = 8 * ks + 2 * p;
        const uint32_t pk = pack_bf16(qm[s], qm[s + 1]);
        b[ks][p] = pk;
        eta += bf16_lo(pk) * zval(s) + bf16_hi(pk) * zval(s + 1);  // the same rounded values the MFMA sees
      }
    eta += partner32(eta);
    const float dn = eta + g.eps;
    const float inv = 1.0f / dn;
    if (live && gl == 0) den[g.th(e.b, h, n)] = dn;
    f32x16 acc[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][i] = 0.0f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) acc[rb] = mfma32(state_op(rb, ks), b[ks], acc[rb]);
    }
    store_rows_bf16<D>(acc, inv, lane, tile, [&](int t) -> bf16_t* {
      return n0 + t < e.t1 ? O.row<bf16_t>(e.b, h, n0 + t) : nullptr;
    });
  }
}


// ---- causal variant (Sec. 4.4): chunked scan -------------------------------------------------------
// Token i attends to tokens j <= i of its sequence.  The sequence is cut into chunks of
// kCausalChunk tokens: k_state gives every chunk's own state, k_prefix turns them into the state
// BEFORE each chunk (exclusive running sum in chunk order, emitted as the query kernel's operand
// image), and k_query_causal adds, for every query tile, the contribution of the earlier tiles of
// its own chunk through the masked score tile  P^T = S Qm^T  (keys x queries) and  O^T += V^T P.

template <class SY, int D>
struct PrefixLayout {
  static constexpr int64_t kOpElems = static_cast<int64_t>(SY::MP) * D;   // bf16: rows = channels image
  static constexpr int64_t kBytes = kOpElems * 2 + 2 * SY::SP * 4;        // then the normaliser by slot
};

// canonical monomial of slot (g, s), -1 for padding slots: the inverse of SlotMap
struct CanonMap {
  int8_t m[2][64];
};
template <class SY>
CanonMap make_canon_map() {
  CanonMap cm{};
  for (int g = 0; g < 2; ++g)
    for (int s = 0; s < 64; ++s) cm.m[g][s] = static_cast<int8_t>(s < SY::SP ? SY::slot_canon(g, s) : -1);
  return cm;
}

// grid (num_seqs, H, kScanParts * 2 * NKS * D / kScanThreads + 1), block kScanThreads.  A piece is the eight slots (g, 8 ks .. 8 ks + 7)
// of one channel c, shared by kScanParts threads (see there): eight running sums, read from the eight partial rows of those monomials at
// column c (consecutive threads: consecutive floats), written for chunk ch -- before chunk ch's own
// partial is added -- as the 16 bytes these eight slots occupy in the operand image (consecutive
// threads of a 32-channel block: consecutive 16-byte pieces).  Padding slots are written as zeros.
// With a decay factor the chunks' partials arrive weighted as seen from the first token behind
// their chunk, and the running sum is multiplied by chunk_decay = decay^chunk from one chunk to the
// next (1 without decay): the state before chunk ch as seen from its first token.
// REVERSE: the running sum goes from the sequence's last chunk to its first, and chunk ch receives
// the sum over the chunks behind it (the gradient states of the backward).  Images are written
// `stride` bytes apart, the normaliser vector z_off bytes into an image.
constexpr int kScanThreads = 64;  // one wave per workgroup: the scans are a few thousand threads in all, spread over as many compute units as possible
// A scan is a chain of memory round trips, one per batch of chunks, and a wave can have only 63
// loads outstanding: the eight values of a 16-byte piece of the image by channels (eight scalar
// loads per chunk) are shared by two neighbouring threads, whose stores still fall side by side, so
// that a batch of sixteen chunks is one round trip (measured: 41 / 40 us for the two scans against
// 43 / 45; four threads per piece 58; the image by monomial rows, two 16-byte loads per chunk, is
// best left with one thread per piece and sixteen chunks per batch: 50 and 46 us otherwise).
constexpr int kScanParts = 2;      // image by channels: threads per piece (four slots each)
constexpr int kScanPartsRows = 1;  // image by monomial rows: threads per piece
constexpr int kScanBatchRows = 16; // its chunks in flight
template <class SY, int D, bool REVERSE>
__device__ __forceinline__ void prefix_body(int zidx, int zcount, const Geom& g,
                                            const int32_t* __restrict__ seq_chunk_off,
                                            const float* __restrict__ partial, int64_t partial_stride,
                                            unsigned char* __restrict__ pfx, const CanonMap& cm,
                                            float chunk_decay, int64_t stride, int64_t z_off) {
  constexpr int MP = SY::MP, SP = SY::SP, NKS = MP / 16;
  constexpr int NV = 8 / kScanParts;  // slots per thread
  const int s = blockIdx.x, h = blockIdx.y;
  const int c0 = seq_chunk_off[s], c1 = seq_chunk_off[s + 1], nc = c1 - c0;
  auto chunk_at = [&](int pos) { return REVERSE ? c1 - 1 - pos : c0 + pos; };  // pos-th chunk in scan order
  const int64_t cstride = static_cast<int64_t>(g.H) * partial_stride;
  // the last workgroup in z carries the normaliser vector (one thread per eight slots), the others
  // the operand image
  const bool zblock = zidx == zcount - 1;
  if (!zblock) {
    const int item = zidx * kScanThreads + threadIdx.x;  // (mg, ks, c, part)
    const int part = item % kScanParts, rest = item / kScanParts;
    const int c = rest % D, ks = (rest / D) % NKS, mg = rest / (D * NKS);
    const float* base = partial + static_cast<int64_t>(h) * partial_stride + c;
    int row[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) row[j] = cm.m[mg][8 * ks + NV * part + j];
    float acc[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) acc[j] = 0.0f;
    const int rb = c / 32, r = c % 32;
    constexpr int NB = 16;  // chunks in flight (one memory round trip per batch)
    for (int pos = 0; pos < nc; pos += NB) {
      float ld[NB][NV];
#pragma unroll
      for (int k = 0; k < NB; ++k) {
        const float* p = base + chunk_at(pos + k < nc ? pos + k : nc - 1) * cstride;
#pragma unroll
        for (int j = 0; j < NV; ++j) ld[k][j] = row[j] >= 0 ? p[row[j] * D] : 0.0f;
      }
#pragma unroll
      for (int k = 0; k < NB; ++k) {
        if (pos + k >= nc) break;
        u32x4* opA = reinterpret_cast<u32x4*>(pfx + (static_cast<int64_t>(chunk_at(pos + k)) * g.H + h) * stride);
        uint32_t* piece = reinterpret_cast<uint32_t*>(opA + (rb * NKS + ks) * 64 + 32 * mg + r) + (NV / 2) * part;
        if constexpr (NV == 8) {
          u32x4 w;
#pragma unroll
          for (int p = 0; p < 4; ++p) w[p] = pack_bf16(acc[2 * p], acc[2 * p + 1]);
          *reinterpret_cast<u32x4*>(piece) = w;
        } else if constexpr (NV == 4) {
          u32x2 w;
          w[0] = pack_bf16(acc[0], acc[1]);
          w[1] = pack_bf16(acc[2], acc[3]);
          *reinterpret_cast<u32x2*>(piece) = w;
        } else {
          piece[0] = pack_bf16(acc[0], acc[1]);
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) acc[j] = __builtin_fmaf(acc[j], chunk_decay, ld[k][j]);
      }
    }
    return;
  }
  // the normaliser vector by slot: thread (mg, ks) carries eight slots; loads batched like the
  // rows above (a load per chunk issued next to the store that needs it would cost one memory
  // round trip per chunk)
  if (threadIdx.x >= 2 * NKS) return;
  const int ks = threadIdx.x % NKS, mg = threadIdx.x / NKS;
  int row[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) row[j] = cm.m[mg][8 * ks + j];
  float z[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) z[j] = 0.0f;
  const float* zb = partial + static_cast<int64_t>(h) * partial_stride + MP * D;
  constexpr int NZ = 16;
  for (int pos = 0; pos < nc; pos += NZ) {
    float ld[NZ][8];
#pragma unroll
    for (int k = 0; k < NZ; ++k) {
      const float* p = zb + chunk_at(pos + k < nc ? pos + k : nc - 1) * cstride;
#pragma unroll
      for (int j = 0; j < 8; ++j) ld[k][j] = row[j] >= 0 ? p[row[j]] : 0.0f;
    }
#pragma unroll
    for (int k = 0; k < NZ; ++k) {
      if (pos + k >= nc) break;
      float* zslot = reinterpret_cast<float*>(pfx + (static_cast<int64_t>(chunk_at(pos + k)) * g.H + h) * stride + z_off);
      f32x4 lo, hi;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        lo[j] = z[j];
        hi[j] = z[4 + j];
      }
      *reinterpret_cast<f32x4*>(zslot + mg * SP + 8 * ks) = lo;
      *reinterpret_cast<f32x4*>(zslot + mg * SP + 8 * ks + 4) = hi;
#pragma unroll
      for (int j = 0; j < 8; ++j) z[j] = __builtin_fmaf(z[j], chunk_decay, ld[k][j]);
    }
  }
}

// The same scan emitting the image whose rows are monomials (the A operand of products that
// contract over the channels, used by the backward): image row rho = 32 rbm + r is slot
// (g, s) = ((rho >> 2) & 1, 16 (rho >> 5) + 4 ((rho >> 3) & 3) + (rho & 3)), so that accumulator
// register i of row block rbm on lane half gl is the lane's own slot 16 rbm + i.
// grid (num_seqs, H, kScanPartsRows * (MP / 32) * (D / 16) * 64 / kScanThreads), block kScanThreads; a
// piece is eight consecutive channels of one row; the image starts `img_off` bytes into a chunk's block.
template <class SY, int D, bool REVERSE>
__device__ __forceinline__ void prefix_rows_body(int zidx, const Geom& g,
                                                 const int32_t* __restrict__ seq_chunk_off,
                                                 const float* __restrict__ partial, int64_t partial_stride,
                                                 unsigned char* __restrict__ pfx, const CanonMap& cm,
                                                 float chunk_decay, int64_t stride, int64_t img_off) {
  constexpr int NKD = D / 16;
  constexpr int PR = kScanPartsRows, NQ = 2 / PR;  // threads per piece, 16-byte loads per thread and chunk
  static_assert(PR == 1 || PR == 2, "a thread carries eight or four channels of a piece");
  const int s = blockIdx.x, h = blockIdx.y;
  const int c0 = seq_chunk_off[s], c1 = seq_chunk_off[s + 1], nc = c1 - c0;
  auto chunk_at = [&](int pos) { return REVERSE ? c1 - 1 - pos : c0 + pos; };
  const int item = zidx * kScanThreads + threadIdx.x;  // (rbm, kd, lane, part)
  const int part = item % PR, rest = item / PR;
  const int lane = rest % 64, kd = (rest / 64) % NKD, rbm = rest / (64 * NKD);
  const int rho = 32 * rbm + lane % 32, gl = lane / 32;
  const int m = cm.m[(rho >> 2) & 1][16 * (rho >> 5) + 4 * ((rho >> 3) & 3) + (rho & 3)];
  const float* base = partial + static_cast<int64_t>(h) * partial_stride + (m >= 0 ? m : 0) * D + 16 * kd + 8 * gl + 4 * NQ * part;
  const int64_t cstride = static_cast<int64_t>(g.H) * partial_stride;
  float acc[4 * NQ];
#pragma unroll
  for (int j = 0; j < 4 * NQ; ++j) acc[j] = 0.0f;
  constexpr int NB = kScanBatchRows;
  for (int pos = 0; pos < nc; pos += NB) {
    f32x4 ld[NB][NQ];
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      const f32x4* p = reinterpret_cast<const f32x4*>(base + chunk_at(pos + k < nc ? pos + k : nc - 1) * cstride);
#pragma unroll
      for (int x = 0; x < NQ; ++x) ld[k][x] = p[x];
    }
#pragma unroll
    for (int k = 0; k < NB; ++k) {
      if (pos + k >= nc) break;
      u32x4* img = reinterpret_cast<u32x4*>(pfx + (static_cast<int64_t>(chunk_at(pos + k)) * g.H + h) * stride + img_off);
      uint32_t* piece = reinterpret_cast<uint32_t*>(img + (rbm * NKD + kd) * 64 + lane) + 2 * NQ * part;
      if constexpr (NQ == 2) {
        u32x4 w;
#pragma unroll
        for (int p = 0; p < 4; ++p) w[p] = pack_bf16(acc[2 * p], acc[2 * p + 1]);
        *reinterpret_cast<u32x4*>(piece) = w;
      } else {
        u32x2 w;
        w[0] = pack_bf16(acc[0], acc[1]);
        w[1] = pack_bf16(acc[2], acc[3]);
        *reinterpret_cast<u32x2*>(piece) = w;
      }
      if (m >= 0) {
#pragma unroll
        for (int j = 0; j < 4 * NQ; ++j) acc[j] = __builtin_fmaf(acc[j], chunk_decay, ld[k][j / 4][j % 4]);
      }
    }
  }
}

template <class SY, int D, bool REVERSE>
__global__ __launch_bounds__(kScanThreads) void k_prefix(Geom g, const int32_t* __restrict__ seq_chunk_off,
                                                         const float* __restrict__ partial,
                                                         int64_t partial_stride, unsigned char* __restrict__ pfx,
                                                         CanonMap cm, float chunk_decay, int64_t stride,
                                                         int64_t z_off) {
  prefix_body<SY, D, REVERSE>(blockIdx.z, gridDim.z, g, seq_chunk_off, partial, partial_stride, pfx, cm,
                              chunk_decay, stride, z_off);
}
template <class SY, int D, bool REVERSE>
__global__ __launch_bounds__(kScanThreads) void k_prefix_rows(Geom g, const int32_t* __restrict__ seq_chunk_off,
                                                              const float* __restrict__ partial,
                                                              int64_t partial_stride, unsigned char* __restrict__ pfx,
                                                              CanonMap cm, float chunk_decay, int64_t stride,
                                                              int64_t img_off) {
  prefix_rows_body<SY, D, REVERSE>(blockIdx.z, g, seq_chunk_off, partial, partial_stride, pfx, cm, chunk_decay,
                                   stride, img_off);
}
// both images in one launch: the first `za` workgroups in z carry the image by channels and the
// normaliser (into `pfx`), the rest the image by monomial rows (into `rows`, img_off bytes into a
// chunk's block there)
template <class SY, int D, bool REVERSE>
__global__ __launch_bounds__(kScanThreads) void k_prefix_both(Geom g, const int32_t* __restrict__ seq_chunk_off,
                                                              const float* __restrict__ partial,
                                                              int64_t partial_stride, unsigned char* __restrict__ pfx,
                                                              CanonMap cm, float chunk_decay, int64_t stride,
                                                              int64_t z_off, unsigned char* __restrict__ rows,
                                                              int64_t rows_stride, int64_t img_off, int za) {
  if (static_cast<int>(blockIdx.z) < za)
    prefix_body<SY, D, REVERSE>(blockIdx.z, za, g, seq_chunk_off, partial, partial_stride, pfx, cm, chunk_decay,
                                stride, z_off);
  else
    prefix_rows_body<SY, D, REVERSE>(blockIdx.z - za, g, seq_chunk_off, partial, partial_stride, rows, cm,
                                     chunk_decay, rows_stride, img_off);
}

// Waves per workgroup of k_query_causal: eight (two per SIMD, 256 registers each) where the live
// set allows it, one query tile per wave; else four with two tiles each.
template <class SY>
constexpr int causal_query_waves() {
  return SY::MP <= 64 ? 8 : 4;
}

template <class SY, int D>
struct CausalSmem {
  static constexpr int kTiles = kCausalChunk / 32;
  static constexpr int NKS = SY::MP / 16;
  static constexpr int kWavesQ = causal_query_waves<SY>();
  static constexpr int kVStride = D * 2 + 32;                  // bytes per token row of the V tile
  static constexpr int kVBytes = kCausalChunk * kVStride;
  static constexpr int kSBytes = kTiles * NKS * 64 * 16;       // key-monomial operand images of the chunk
  static constexpr int kOutRows = kWavesQ == 4 ? 32 : 16;  // rows of a wave's store tile
  static constexpr int kBase = kVBytes + kSBytes + kWavesQ * RowTile<D, kOutRows>::kBytes;
  // the operand image of the state in front of the chunk, read by every wave: an LDS copy where
  // it fits, each wave's own loads from memory otherwise
  static constexpr int kImgBytes = SY::MP * D * 2 + 2 * SY::SP * 4;  // with the normaliser by slot behind it
  static constexpr bool kImgLds = kBase + kImgBytes <= 160 * 1024;
  static constexpr int kTotal = kBase + (kImgLds ? kImgBytes : 0);
};

// grid (chunks of kCausalChunk tokens, H), block of 4 or 8 waves.  The workgroup stages the chunk's
// V rows and the key monomials of its tokens (as MFMA A-operand images, one per 32-key tile) in
// LDS; with four waves, wave w then serves query tiles w and 7 - w (equal numbers of key tiles per
// wave); with eight, waves w and w + 4 (which share a SIMD) serve tiles w and 7 - w, so that every
// SIMD still sees nine key tiles but has a second wave to run while one waits.  Lane (r, gl):
// query r of the tile, slot half gl, as in k_query.
template <class SY, int D>
__global__ __launch_bounds__(causal_query_waves<SY>() * 64) void k_query_causal(Geom g, const BlockEnt* __restrict__ chunks,
                                                           const float* __restrict__ feat, View V,
                                                           const unsigned char* __restrict__ pfx, View O,
                                                           float* __restrict__ den, float log2_decay,
                                                           int nchunks) {
  using SM = CausalSmem<SY, D>;
  using PL = PrefixLayout<SY, D>;
  constexpr int SP = SY::SP, MP = SY::MP, DP = SY::DPHI, F = SY::F;
  constexpr int NRB = D / 32, NKS = MP / 16, NF = F * DP;
  constexpr int WAVES = SM::kWavesQ;
  constexpr int kRowsPW = kCausalChunk / WAVES;       // rows a wave stages
  constexpr int kTilesPW = kCausalChunk / 32 / WAVES;  // tiles a wave stages and serves
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  unsigned char* vs = smem;
  u32x4* simg = reinterpret_cast<u32x4*>(smem + SM::kVBytes);
  unsigned char* tile = smem + SM::kVBytes + SM::kSBytes + wave * RowTile<D, SM::kOutRows>::kBytes;
  const int r = lane % 32, gl = lane / 32;
  const int L = lane % 16, q = lane / 16;
  static_assert(SM::kImgBytes == PL::kBytes, "the staged image is the prefix record of the chunk");
  // A workgroup walks the (chunk, head) items blockIdx.x, blockIdx.x + gridDim.x, .. (item = head *
  // nchunks + chunk): what the next item's start needs from memory is requested while the current
  // one is worked on (and its table entry an item earlier still), so that only the copy into LDS
  // stands between two items.
  struct Staged {  // an item's start as it arrives from memory
    ImageCopy<SM::kImgLds ? SM::kImgBytes : 16, WAVES * 64> image;  // state in front of the chunk, its normaliser
    TileRegs<D, kRowsPW> vt;                                        // this wave's share of the V rows
    f32x2 kraw[kTilesPW][NF / 2];                                   // key features of the tiles it stages
    f32x2 qraw0[DP / 2];                                            // features of its first query tile
  };
  const int qt_first = WAVES == 8 ? (wave < 4 ? wave : 11 - wave) : chunk_tile_of(wave, 0);
  // a query tile's features (tokens beyond the chunk read its last token and are zeroed when used)
  auto request_query = [&](const BlockEnt& e, int h, int qt, f32x2 (&qraw)[DP / 2]) {
    const int n = e.t0 + 32 * qt + r;
    const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(g.th(e.b, h, n < e.t1 ? n : e.t1 - 1), 0));
#pragma unroll
    for (int p = 0; p < DP / 2; ++p) qraw[p] = f[32 * (gl ? DP / 2 - 1 - p : p)];  // lane half 1: pairs in reverse
  };
  auto request = [&](const BlockEnt& e, int ci, int h, Staged& st) {
    if constexpr (SM::kImgLds) st.image.request(pfx + (static_cast<int64_t>(ci) * g.H + h) * PL::kBytes);
    fetch_tile<D, kRowsPW>(V, e.b, h, e.t0 + kRowsPW * wave, e.t1, lane, st.vt);
#pragma unroll
    for (int tt = 0; tt < kTilesPW; ++tt) {
      const int n = e.t0 + 32 * (kTilesPW * wave + tt) + r;
      const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(g.th(e.b, h, n < e.t1 ? n : e.t1 - 1), DP));
#pragma unroll
      for (int p = 0; p < NF / 2; ++p) st.kraw[tt][p] = f[32 * p];
    }
    request_query(e, h, qt_first, st.qraw0);
  };
  // the staged tiles: state image, V rows, key-monomial images
  auto commit = [&](const BlockEnt& e, const Staged& st) {
    if constexpr (SM::kImgLds) st.image.commit(smem + SM::kBase);
    put_tile<D, kRowsPW>(st.vt, lane, vs + kRowsPW * wave * SM::kVStride, SM::kVStride);
#pragma unroll
    for (int tt = 0; tt < kTilesPW; ++tt) {
      const int t = kTilesPW * wave + tt;
      const bool live_k = e.t0 + 32 * t + r < e.t1;
      float kf[NF], kr[NF];
#pragma unroll
      for (int p = 0; p < NF / 2; ++p) {
        kf[2 * p] = live_k ? st.kraw[tt][p][0] : 0.0f;
        kf[2 * p + 1] = live_k ? st.kraw[tt][p][1] : 0.0f;
      }
      float kk[F][DP];
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int c = 0; c < DP; ++c) kr[f * DP + c] = kf[(f + 1) * DP - 1 - c];
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int c = 0; c < DP; ++c) kk[f][c] = gl ? kr[f * DP + c] : kf[f * DP + c];
      float sm[SP];
      sym_key_monomials_slots<SY>(kk, sm, gl);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        u32x4 w;
#pragma unroll
        for (int p = 0; p < 4; ++p) w[p] = pack_bf16(sm[8 * ks + 2 * p], sm[8 * ks + 2 * p + 1]);
        simg[(t * NKS + ks) * 64 + lane] = w;
      }
    }
  };
  float rowfac[16];  // decay^(31 - key row of accumulator register i)
#pragma unroll
  for (int i = 0; i < 16; ++i)
    rowfac[i] = log2_decay != 0.0f ? __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(31 - d_row(i, gl))) : 1.0f;
  const int nitems = nchunks * g.H, stride_i = gridDim.x;
  int item = blockIdx.x;  // < nitems: the grid is never larger
  int ci = item % nchunks, h = item / nchunks;
  BlockEnt e = chunks[ci];
  BlockEnt e_next = chunks[(item + stride_i < nitems ? item + stride_i : item) % nchunks];
  Staged st;
  request(e, ci, h, st);
  while (true) {
    f32x2 qraw0[DP / 2];
#pragma unroll
    for (int p = 0; p < DP / 2; ++p) qraw0[p] = st.qraw0[p];
    commit(e, st);
    __syncthreads();
    const int item_n = item + stride_i;
    const bool more = item_n < nitems;  // the same for the whole workgroup
    const int cn = item_n % nchunks, hn = item_n / nchunks;
    if (more) request(e_next, cn, hn, st);
    const BlockEnt e_next2 = chunks[(item_n + stride_i < nitems ? item_n + stride_i : item) % nchunks];
    const unsigned char* pu = pfx + (static_cast<int64_t>(ci) * g.H + h) * PL::kBytes;
    const u32x4* opA = reinterpret_cast<const u32x4*>(SM::kImgLds ? smem + SM::kBase : pu);
    const float* zslot = reinterpret_cast<const float*>((SM::kImgLds ? smem + SM::kBase : pu) + PL::kOpElems * 2) + gl * SP;
  #pragma unroll 1
    for (int qi = 0; qi < kTilesPW; ++qi) {
      const int qt = WAVES == 8 ? (wave < 4 ? wave : 11 - wave) : chunk_tile_of(wave, qi);
      const int n0 = e.t0 + 32 * qt;
      if (n0 >= e.t1) continue;
      const int n = n0 + r;
      const bool live = n < e.t1;
      float qf[DP];
      {
        f32x2 qraw[DP / 2];
        if (qi == 0) {
  #pragma unroll
          for (int p = 0; p < DP / 2; ++p) qraw[p] = qraw0[p];
        } else {
          request_query(e, h, qt, qraw);
        }
  #pragma unroll
        for (int p = 0; p < DP / 2; ++p) {  // and each pair in reverse
          qf[2 * p] = live ? (gl ? qraw[p][1] : qraw[p][0]) : 0.0f;
          qf[2 * p + 1] = live ? (gl ? qraw[p][0] : qraw[p][1]) : 0.0f;
        }
      }
      float qm[SP];
      sym_query_monomials<SY>(qf, qm, gl);
      u32x4 b[NKS];
      float eta = 0.0f;
  #pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const f32x4 z0 = *reinterpret_cast<const f32x4*>(zslot + 8 * ks);
        const f32x4 z1 = *reinterpret_cast<const f32x4*>(zslot + 8 * ks + 4);
  #pragma unroll
        for (int p = 0; p < 4; ++p) {
          const int s = 8 * ks + 2 * p;
          const uint32_t pk = pack_bf16(qm[s], qm[s + 1]);
          b[ks][p] = pk;
          const float za = p < 2 ? z0[2 * p] : z1[2 * p - 4], zb = p < 2 ? z0[2 * p + 1] : z1[2 * p - 3];
          eta += bf16_lo(pk) * za + bf16_hi(pk) * zb;  // the same rounded values the MFMA sees
        }
      }
      // everything before the chunk: the prefix state
      f32x16 acc[NRB];
  #pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
  #pragma unroll
        for (int i = 0; i < 16; ++i) acc[rb][i] = 0.0f;
  #pragma unroll
        for (int ks = 0; ks < NKS; ++ks) acc[rb] = mfma32(opA[(rb * NKS + ks) * 64 + lane], b[ks], acc[rb]);
      }
      if (log2_decay != 0.0f) {  // the prefix state is as seen from the chunk's first token
        const float wq = __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(32 * qt + r));
        eta *= wq;
  #pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
  #pragma unroll
          for (int i = 0; i < 16; ++i) acc[rb][i] *= wq;
      }
      // the chunk's own tokens up to the query: key tiles 0 .. qt
  #pragma unroll 1
      for (int kt = 0; kt <= qt; ++kt) {
        f32x16 P;
  #pragma unroll
        for (int i = 0; i < 16; ++i) P[i] = 0.0f;
        {
          u32x4 sa[NKS];  // all operands requested before the first MFMA
  #pragma unroll
          for (int ks = 0; ks < NKS; ++ks) sa[ks] = simg[(kt * NKS + ks) * 64 + lane];
          __builtin_amdgcn_sched_barrier(0);
  #pragma unroll
          for (int ks = 0; ks < NKS; ++ks) P = mfma32(sa[ks], b[ks], P);
        }
        if (log2_decay != 0.0f) {  // decay^(query position - key position); masked entries get 0 below
          if (kt < qt) {  // distance >= 1: a per-lane factor times a per-register one (both at most 1)
            const float cw = __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(32 * (qt - kt) + r - 31));
  #pragma unroll
            for (int i = 0; i < 16; ++i) P[i] *= cw * rowfac[i];
          } else {
  #pragma unroll
            for (int i = 0; i < 16; ++i)
              P[i] *= __builtin_amdgcn_exp2f(log2_decay * fmaxf(static_cast<float>(r - d_row(i, gl)), 0.0f));
          }
        }
        if (kt == qt) {  // key d_row(i, gl) of the tile against query r: later keys are masked
  #pragma unroll
          for (int i = 0; i < 16; ++i)
            if (d_row(i, gl) > r) P[i] = 0.0f;
        }
        u32x4 pb[2];
  #pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
  #pragma unroll
          for (int p = 0; p < 4; ++p) {
            const uint32_t pk = pack_bf16(P[8 * ks2 + 2 * p], P[8 * ks2 + 2 * p + 1]);
            pb[ks2][p] = pk;
            eta += bf16_lo(pk) + bf16_hi(pk);
          }
        // O^T += V^T P: k-slot (ks2, gl, j) is key 16 ks2 + 8 (j / 4) + 4 gl + j % 4 of the tile, the
        // order in which the score accumulators hold the keys
        u32x4 va[2][NRB];
  #pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          const int krow = 32 * kt + 16 * ks2 + 4 * gl + L / 4;
  #pragma unroll
          for (int rb = 0; rb < NRB; ++rb) {
            const unsigned char* p = vs + krow * SM::kVStride + (32 * rb + 16 * (q % 2) + 4 * (L % 4)) * 2;
            const u32x2 lo = lds_read_tr16(p);
            const u32x2 hi = lds_read_tr16(p + 8 * SM::kVStride);
            va[ks2][rb][0] = lo[0];
            va[ks2][rb][1] = lo[1];
            va[ks2][rb][2] = hi[0];
            va[ks2][rb][3] = hi[1];
          }
        }
        __builtin_amdgcn_sched_barrier(0);
  #pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
  #pragma unroll
          for (int rb = 0; rb < NRB; ++rb) acc[rb] = mfma32(va[ks2][rb], pb[ks2], acc[rb]);
      }
      eta += partner32(eta);
      const float dn = eta + g.eps;
      const float inv = 1.0f / dn;
      if (live && gl == 0) den[g.th(e.b, h, n)] = dn;
      store_rows_bf16<D, SM::kOutRows>(acc, inv, lane, tile, [&](int t) -> bf16_t* {
        return n0 + t < e.t1 ? O.row<bf16_t>(e.b, h, n0 + t) : nullptr;
      });
    }
    if (!more) break;
    __syncthreads();  // every wave is done with this item's tiles
    item = item_n;
    ci = cn;
    h = hn;
    e = e_next;
    e_next = e_next2;
  }
}

// ---- k_bwd_query ------------------------------------------------------------------------------
template <int D, int MP>
struct BwdQSmem {
  static constexpr int kDoBytes = 32 * D * 2;   // dO tile [32 tokens][D] bf16, swizzled, unpadded
  // scaled-monomial tile [32 tokens][MP slot columns] bf16, swizzled; rows of 128 or 256 bytes
  static constexpr int kQRow = MP <= 64 ? 128 : 256;
  static constexpr int kQBytes = 32 * kQRow;
  static constexpr int kWaveBytes = kDoBytes + kQBytes;
  // With more than 64 state rows the monomial-row operand image of the state does not fit the
  // register file next to the accumulators: the workgroup keeps one copy in LDS instead.
  static constexpr bool kOpsInLds = MP > 64;
  static constexpr int kOpBytes = kOpsInLds ? MP * D * 2 + MP * 4 : 0;  // image, then the normaliser vector
  static constexpr int kStream = kOpBytes + kWaves * kWaveBytes;
  static constexpr int kRedBytes = WaveSum<D, MP>::kBytes;
  static constexpr int kTotal = kStream > kRedBytes ? kStream : kRedBytes;
};

// grid (chunks, H), block 256.  Per 32-token tile and lane (token r, slot half gl), with
// inv = 1/den and the raw upstream gradient rows dO as the operand of both contractions:
//   X^T = Csym dO^T               (contraction over channels; dO loaded in B-operand order)
//   s   = -inv^2 <Qm, X>          (= -<dO, o>/den, because o = Csym^T Qm / den: O is not re-read)
//   dM  = inv X + s zsym   -> chain rule to d(phi_q)
//   dCsym += (inv Qm)^T dO        (contraction over the tile's tokens: both operands through LDS
//                                  with transpose reads),   dzsym += s Qm.
// Taking s from the same X that feeds dM makes the component of dM along Qm cancel exactly, which
// is where the query gradient loses its precision otherwise.  The chunk's dCsym/dzsym are summed
// over the four waves in wave order and written as one partial whose row SP g + s is slot (g, s).
template <class SY, int D>
__global__ __launch_bounds__(kThreads) void k_bwd_query(
    Geom g, const BlockEnt* __restrict__ chunks, const float* __restrict__ feat,
    const float* __restrict__ den, const unsigned char* __restrict__ ops, View dO,
    float* __restrict__ dfeat, float* __restrict__ partial, int64_t partial_stride, int relu_mask) {
  using SL = StateLayout<SY, D>;
  using SM = BwdQSmem<D, SY::MP>;
  constexpr int SP = SY::SP, MP = SY::MP, DP = SY::DPHI;
  constexpr int NCB = D / 32, NKD = D / 16, NRM = MP / 32;
  constexpr int DROW = D * 2;  // bytes per dO tile row
  constexpr int QROW = SM::kQRow;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  unsigned char* ds = smem + SM::kOpBytes + wave * SM::kWaveBytes;
  unsigned char* qs = ds + SM::kDoBytes;
  const BlockEnt e = chunks[blockIdx.x];
  const int h = blockIdx.y;
  const int r = lane % 32, gl = lane / 32;
  const int L = lane % 16, q = lane / 16;
  const int64_t u = static_cast<int64_t>(e.seq) * g.H + h;
  const u32x4* opB = reinterpret_cast<const u32x4*>(ops + u * SL::kOpBytes + SL::kOpElems * 2);
  const float* zslot = reinterpret_cast<const float*>(ops + u * SL::kOpBytes + 2 * SL::kOpElems * 2) + gl * SP;
  u32x4 a_mo[SM::kOpsInLds ? 1 : NRM][SM::kOpsInLds ? 1 : NKD];
  if constexpr (SM::kOpsInLds) {
    constexpr int N16 = MP * D * 2 / 16;
    static_assert(N16 % kThreads == 0, "the operand image is copied in whole rounds");
#pragma unroll
    for (int k = 0; k < N16 / kThreads; ++k)
      reinterpret_cast<u32x4*>(smem)[threadIdx.x + k * kThreads] = opB[threadIdx.x + k * kThreads];
    if (threadIdx.x < MP) reinterpret_cast<float*>(smem + MP * D * 2)[threadIdx.x] = (zslot - gl * SP)[threadIdx.x];
    __syncthreads();
  } else {
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int ks = 0; ks < NKD; ++ks) a_mo[rb][ks] = opB[(rb * NKD + ks) * 64 + lane];
  }
  auto state_op = [&](int rb, int ks) -> u32x4 {
    if constexpr (SM::kOpsInLds)
      return reinterpret_cast<const u32x4*>(smem)[(rb * NKD + ks) * 64 + lane];
    else
      return a_mo[rb][ks];
  };
  float z[SM::kOpsInLds ? 1 : SP];  // this half's normaliser entries (in LDS next to the image otherwise)
  if constexpr (!SM::kOpsInLds) {
#pragma unroll
    for (int s4 = 0; s4 < SP / 4; ++s4) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(zslot + 4 * s4);
#pragma unroll
      for (int i = 0; i < 4; ++i) z[4 * s4 + i] = v[i];
    }
  }
  auto zval = [&](int s) -> float {
    if constexpr (SM::kOpsInLds)
      return reinterpret_cast<const float*>(smem + MP * D * 2)[gl * SP + s];
    else
      return z[s];
  };
  // per-lane LDS offsets: own-row writes, and transpose reads of token rows 8gl + L/4 (+4) at the
  // 4 columns 32x + 16(q%2) + 4(L%4) ..+3 (x = row block of Qm^T or column block of dO)
  int dw_off[NKD];
#pragma unroll
  for (int ks = 0; ks < NKD; ++ks) dw_off[ks] = tile_off<DROW>(r, 2 * ks + gl);
  int qw_off[SP / 8];
#pragma unroll
  for (int p4 = 0; p4 < SP / 8; ++p4) qw_off[p4] = tile_off<QROW>(r, (SP / 8) * gl + p4);
  int qa_off[2][NRM], db_off[2][NCB];
#pragma unroll
  for (int hi = 0; hi < 2; ++hi) {
    const int row = 8 * gl + 4 * hi + L / 4;
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
      qa_off[hi][rb] = tile_off<QROW>(row, 4 * rb + 2 * (q % 2) + (L % 4) / 2) + (L % 2) * 8;
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
      db_off[hi][cb] = tile_off<DROW>(row, 4 * cb + 2 * (q % 2) + (L % 4) / 2) + (L % 2) * 8;
  }

  f32x16 dC[NRM][NCB];
#pragma unroll
  for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) dC[rb][cb][i] = 0.0f;
  float dzacc[SP];
#pragma unroll
  for (int s = 0; s < SP; ++s) dzacc[s] = 0.0f;

  // one tile's inputs: the dO row pieces (B operand, k-slot (ks, gl, j) = channel 16ks + 8gl + j),
  // the query features of this lane's half (gl = 1: reversed) and the denominator
  u32x4 xb[NKD], xn[NKD];
  float fb[DP], fn[DP];
  float denb = 1.0f, denn = 1.0f;
  auto fetch = [&](int n0, u32x4(&x)[NKD], float(&f)[DP], float& dn) {
    const int n = n0 + r;
    if (n < e.t1) {
      const bf16_t* row = dO.row<const bf16_t>(e.b, h, n);
#pragma unroll
      for (int ks = 0; ks < NKD; ++ks) x[ks] = *reinterpret_cast<const u32x4*>(row + 16 * ks + 8 * gl);
      const int64_t th = g.th(e.b, h, n);
      const f32x2* fp = reinterpret_cast<const f32x2*>(feat + g.fidx(th, 0));
#pragma unroll
      for (int p = 0; p < DP / 2; ++p) {
        const f32x2 v = fp[32 * p];
        f[2 * p] = v[0];
        f[2 * p + 1] = v[1];
      }
      dn = den[th];
    } else {
#pragma unroll
      for (int ks = 0; ks < NKD; ++ks) x[ks][0] = x[ks][1] = x[ks][2] = x[ks][3] = 0u;
#pragma unroll
      for (int a = 0; a < DP; ++a) f[a] = 0.0f;
      dn = 1.0f;
    }
  };
  // X^T = Csym dO^T of one tile: NKD dependent MFMAs per row block that everything else in the
  // tile waits for.  They run one tile ahead, at the end of the previous iteration (the rows are
  // prefetched by then), so that they complete in the shadow of the next tile's monomial
  // arithmetic.
  f32x16 X[NRM];
  auto x_product = [&](const u32x4(&x)[NKD]) {
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) X[rb][i] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < NKD; ++ks)
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb) X[rb] = mfma32(state_op(rb, ks), x[ks], X[rb]);
  };
  stagger_start(wave, blockIdx.x, kStaggerCore);
  int n0 = e.t0 + wave * 32;
  if (n0 < e.t1) {
    fetch(n0, xb, fb, denb);
    x_product(xb);
  }
  for (; n0 < e.t1; n0 += kWaves * 32) {
    const int n = n0 + r;
    const bool live = n < e.t1;
    const int64_t th = g.th(e.b, h, live ? n : e.t0);
    if (n0 + kWaves * 32 < e.t1) fetch(n0 + kWaves * 32, xn, fn, denn);
    // dO tile for the token contraction
#pragma unroll
    for (int ks = 0; ks < NKD; ++ks) *reinterpret_cast<u32x4*>(ds + dw_off[ks]) = xb[ks];
    // monomials of this lane's slots and their scaled bf16 copy (a row of the A^T tile)
    const float inv = live ? 1.0f / denb : 0.0f;
    float qf[DP];
    {
      float fr[DP];  // reversed copy first: see the note on selects in k_bwd_key
#pragma unroll
      for (int c = 0; c < DP; ++c) fr[c] = fb[DP - 1 - c];
#pragma unroll
      for (int c = 0; c < DP; ++c) qf[c] = gl ? fr[c] : fb[c];
    }
    float qm[SP];
    sym_query_monomials<SY>(qf, qm, gl);
#pragma unroll
    for (int p4 = 0; p4 < SP / 8; ++p4) {
      u32x4 w;
#pragma unroll
      for (int p = 0; p < 4; ++p) w[p] = pack_bf16(qm[8 * p4 + 2 * p] * inv, qm[8 * p4 + 2 * p + 1] * inv);
      *reinterpret_cast<u32x4*>(qs + qw_off[p4]) = w;
    }
    float dot = 0.0f;
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) dot += qm[16 * rb + i] * X[rb][i];
    dot += partner32(dot);
    const float si = -(inv * inv) * dot;
    float dm[SP];
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        dm[16 * rb + i] = inv * X[rb][i] + si * zval(16 * rb + i);
        dzacc[16 * rb + i] += si * qm[16 * rb + i];
      }
    float dq[DP];
#pragma unroll
    for (int c = 0; c < DP; ++c) dq[c] = 0.0f;
    sym_query_monomials_grad<SY>(qf, dm, dq, gl);
    float other[DP];
#pragma unroll
    for (int c = 0; c < DP; ++c) other[c] = partner32(dq[c]);
    if (live && gl == 0) {
      // relu_mask: the features came out of a ReLU, and what the feature-map backward needs is
      // the gradient of its input: zero where the feature is zero
      f32x2* df = reinterpret_cast<f32x2*>(dfeat + g.fidx(th, 0));
#pragma unroll
      for (int c = 0; c < DP; c += 2) {
        f32x2 v;
        v[0] = (!relu_mask || fb[c] > 0.0f) ? dq[c] + other[DP - 1 - c] : 0.0f;
        v[1] = (!relu_mask || fb[c + 1] > 0.0f) ? dq[c + 1] + other[DP - 2 - c] : 0.0f;
        df[32 * (c / 2)] = v;
      }
    }
    wave_lds_sync();
    // dCsym[(g,s) rows x D] += (inv Qm)^T[MP x 32 tokens] dO[32 tokens x D]
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      u32x4 a[NRM];
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb) {
        const u32x2 lo = lds_read_tr16(qs + ks * 16 * QROW + qa_off[0][rb]);
        const u32x2 hi = lds_read_tr16(qs + ks * 16 * QROW + qa_off[1][rb]);
        a[rb][0] = lo[0];
        a[rb][1] = lo[1];
        a[rb][2] = hi[0];
        a[rb][3] = hi[1];
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const u32x2 lo = lds_read_tr16(ds + ks * 16 * DROW + db_off[0][cb]);
        const u32x2 hi = lds_read_tr16(ds + ks * 16 * DROW + db_off[1][cb]);
        u32x4 b;
        b[0] = lo[0];
        b[1] = lo[1];
        b[2] = hi[0];
        b[3] = hi[1];
#pragma unroll
        for (int rb = 0; rb < NRM; ++rb) dC[rb][cb] = mfma32(a[rb], b, dC[rb][cb]);
      }
    }
    wave_lds_sync();
    x_product(xn);  // the next tile's (after the last tile: unused)
#pragma unroll
    for (int ks = 0; ks < NKD; ++ks) xb[ks] = xn[ks];
#pragma unroll
    for (int a = 0; a < DP; ++a) fb[a] = fn[a];
    denb = denn;
  }
  // dz: sum over the 32 token lanes of each half
#pragma unroll
  for (int s = 0; s < SP; ++s) {
    float v = dzacc[s];
#pragma unroll
    for (int m = 1; m < 32; m <<= 1) v += __shfl_xor(v, m, 64);
    dzacc[s] = v;
  }
  // sum the four waves: row 32rb + d_row(i, gl) of the accumulators is column SP g' + s' of the
  // monomial tile, i.e. slot (g', s'); the vector element SP gl + s is slot (gl, s) as well
  float* red = reinterpret_cast<float*>(smem);
  sum_over_waves<D, MP>(dC, dzacc, red, wave, lane);
  f32x4* out = reinterpret_cast<f32x4*>(partial + (static_cast<int64_t>(blockIdx.x) * g.H + h) * partial_stride);
  for (int i = threadIdx.x; i < (MP * D + MP) / 4; i += kThreads) out[i] = summed4<D, MP>(red, i);
}

// ---- k_bwd_key --------------------------------------------------------------------------------
// grid (chunks, H), block 256.  Per 32-token tile and lane (token r, gl):
//   dS^T = dCsym V^T (+ dzsym) -> chain rule to d(phi_k1..F);  dV^T = dCsym^T S^T.
// LDS only serves the transpose of the dV tile for whole-row stores.
// Both contractions run over channels or monomials, never over tokens, so a lane loads its own
// token's V row straight into B-operand order; the next tile's row and features are fetched while
// the current tile is computed.
template <class SY, int D>
__global__ __launch_bounds__(kThreads) void k_bwd_key(Geom g, const BlockEnt* __restrict__ blocks,
                                                      const float* __restrict__ feat,
                                                      const unsigned char* __restrict__ dops, View V,
                                                      float* __restrict__ dfeat, View dV,
                                                      int relu_mask) {
  using SL = StateLayout<SY, D>;
  constexpr int SP = SY::SP, MP = SY::MP, DP = SY::DPHI, F = SY::F;
  constexpr int NRB = D / 32, NKS = MP / 16, NKD = D / 16, NRM = MP / 32;
  constexpr int NF = F * DP;  // key features per token
  // LDS: the two operand images of the state gradient (shared by the four waves, read per use:
  // holding them in registers would leave no room for the software pipeline below), then one
  // transpose tile per wave for whole-row stores of dV
  constexpr int kOpImg = static_cast<int>(SL::kOpElems) * 2;  // bytes of one operand image
  __shared__ __align__(16) unsigned char smem[2 * kOpImg + kWaves * RowTile<D>::kBytes];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  unsigned char* tile = smem + 2 * kOpImg + wave * RowTile<D>::kBytes;
  const int r = lane % 32, gl = lane / 32;
  const BlockEnt e = blocks[blockIdx.x];
  const int h = blockIdx.y;
  const int64_t u = static_cast<int64_t>(e.seq) * g.H + h;
  {
    const u32x4* src = reinterpret_cast<const u32x4*>(dops + u * SL::kOpBytes);
    constexpr int N16 = 2 * kOpImg / 16, PER = N16 / kThreads;
    static_assert(N16 % kThreads == 0, "operand images are copied in whole rounds");
    u32x4 v[PER];
#pragma unroll
    for (int k = 0; k < PER; ++k) v[k] = src[threadIdx.x + k * kThreads];
#pragma unroll
    for (int k = 0; k < PER; ++k) reinterpret_cast<u32x4*>(smem)[threadIdx.x + k * kThreads] = v[k];
  }
  const u32x4* opA = reinterpret_cast<const u32x4*>(smem) + lane;            // [rb * NKS + ks] * 64
  const u32x4* opB = reinterpret_cast<const u32x4*>(smem + kOpImg) + lane;   // [rb * NKD + ks] * 64
  const float* dzslot = reinterpret_cast<const float*>(dops + u * SL::kOpBytes + 2 * SL::kOpElems * 2) + gl * SP;
  float dz[SP];
#pragma unroll
  for (int s4 = 0; s4 < SP / 4; ++s4) {
    const f32x4 v = *reinterpret_cast<const f32x4*>(dzslot + 4 * s4);
#pragma unroll
    for (int i = 0; i < 4; ++i) dz[4 * s4 + i] = v[i];
  }
  __syncthreads();

  // One tile's inputs: the V row pieces (B operand, k-slot (ks, gl, j) = channel 16ks + 8gl + j;
  // the 32-byte runs of a row that one load instruction touches are merged by the vector cache)
  // and the F d_phi key features of the token.  vn/kn always hold the loads in flight for the coming
  // tile (rows past the chunk read its last row and are masked below) and are copied at the top
  // of the loop.  Memory instructions are spread through the iteration instead of issued in
  // bursts: the next tile's loads go out one at a time between the MFMAs of the first half, the
  // previous tile's outputs (dV rows staged in LDS, feature gradients held in registers) leave
  // between quarters of the chain rule.  All waves of the grid run the same schedule, and
  // back-to-back bursts from all of them at once stall on the memory pipeline's queues.
  constexpr int PIECES = D / 8, RPI = 64 / PIECES, NST = 32 / RPI;  // dV row stores per tile
  u32x4 vb[NKD], vn[NKD];
  float kb[NF], kn[NF];
  stagger_start(wave, blockIdx.x, kStaggerCore);
  int n0 = e.t0 + wave * 32;
  const bf16_t* nrow = nullptr;   // the coming tile's V row and feature address of this lane
  const f32x2* nfeat = nullptr;  // feature pairs
  auto next_addr = [&](int t0) {
    const int n = t0 + r < e.t1 ? t0 + r : e.t1 - 1;
    nrow = V.row<const bf16_t>(e.b, h, n);
    nfeat = reinterpret_cast<const f32x2*>(feat + g.fidx(g.th(e.b, h, n), DP));
  };
  if (n0 < e.t1) {
    next_addr(n0);
#pragma unroll
    for (int ks = 0; ks < NKD; ++ks) vn[ks] = *reinterpret_cast<const u32x4*>(nrow + 16 * ks + 8 * gl);
#pragma unroll
    for (int p = 0; p < NF / 2; ++p) {
      const f32x2 v = nfeat[32 * p];
      kn[2 * p] = v[0];
      kn[2 * p + 1] = v[1];
    }
  }
  int pend_n0 = -1;            // first token of the tile staged in LDS, -1: none
  float pend_df[NF];           // its feature gradients (this lane's token)
#pragma unroll
  for (int a = 0; a < NF; ++a) pend_df[a] = 0.0f;
  // one dV row store of the staged tile
  auto flush_piece = [&](int i) {
    const int row = i * RPI + lane / PIECES, piece = lane % PIECES;
    const u32x4 v = *reinterpret_cast<const u32x4*>(tile + row * RowTile<D, 32>::kStride + piece * 16);
    if (pend_n0 >= 0 && pend_n0 + row < e.t1)
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dV.row<bf16_t>(e.b, h, pend_n0 + row) + piece * 8));
  };
  // feature-gradient pairs a0 .. a1-1 of the staged tile
  auto flush_df = [&](int a0, int a1) {
    if (pend_n0 >= 0 && pend_n0 + r < e.t1 && gl == 0) {
      f32x2* df = reinterpret_cast<f32x2*>(dfeat + g.fidx(g.th(e.b, h, pend_n0 + r), DP));
#pragma unroll
      for (int p = 0; p < NF / 2; ++p)
        if (p >= a0 && p < a1) {
          f32x2 v;
          v[0] = pend_df[2 * p];
          v[1] = pend_df[2 * p + 1];
          df[32 * p] = v;
        }
    }
  };
  for (; n0 < e.t1; n0 += kWaves * 32) {
    const bool live = n0 + r < e.t1;
#pragma unroll
    for (int ks = 0; ks < NKD; ++ks) vb[ks] = vn[ks];
#pragma unroll
    for (int a = 0; a < NF; ++a) kb[a] = kn[a];
    next_addr(n0 + kWaves * 32 < e.t1 ? n0 + kWaves * 32 : n0);
    f32x16 dS[NRM];
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) dS[rb][i] = 0.0f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < NKD; ++ks) {
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb) dS[rb] = mfma32(opB[(rb * NKD + ks) * 64], vb[ks], dS[rb]);
      vn[ks] = *reinterpret_cast<const u32x4*>(nrow + 16 * ks + 8 * gl);
      __builtin_amdgcn_sched_barrier(0);
    }
    // features of this lane's half: gl = 1 works on the reversed vectors; lanes past the chunk
    // work on zeros
    float kk[F][DP];
    {
      // the reversed copy is a renaming of registers; selecting between the two arrays element by
      // element costs one v_cndmask each (a select between two elements of ONE array may be turned
      // into a run-time index, which is lowered to a compare-and-select chain over the whole array)
      float kf[NF], kr[NF];
#pragma unroll
      for (int a = 0; a < NF; ++a) kf[a] = live ? kb[a] : 0.0f;
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int c = 0; c < DP; ++c) kr[f * DP + c] = kf[(f + 1) * DP - 1 - c];
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int c = 0; c < DP; ++c) kk[f][c] = gl ? kr[f * DP + c] : kf[f * DP + c];
    }
    // dV^T = dCsym^T S^T
    float sm[SP];
    sym_key_monomials_slots<SY>(kk, sm, gl);
    f32x16 acc[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][i] = 0.0f;
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      u32x4 b;
#pragma unroll
      for (int p = 0; p < 4; ++p) b[p] = pack_bf16(sm[8 * ks + 2 * p], sm[8 * ks + 2 * p + 1]);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        acc[rb] = mfma32(opA[(rb * NKS + ks) * 64], b, acc[rb]);
        // the coming tile's feature pairs, a few per MFMA
        constexpr int kPerM = (NF / 2 + NKS * NRB - 1) / (NKS * NRB);
#pragma unroll
        for (int t = 0; t < kPerM; ++t) {
          const int p = (ks * NRB + rb) * kPerM + t;
          if (p < NF / 2) {
            const f32x2 v = nfeat[32 * p];
            kn[2 * p] = v[0];
            kn[2 * p + 1] = v[1];
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    float dk[F][DP];
    {
      float ds[SP];
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) ds[16 * rb + i] = dS[rb][i] + dz[16 * rb + i];
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int c = 0; c < DP; ++c) dk[f][c] = 0.0f;
      // chain rule in four quarters, the previous tile's outputs leaving in between
      KeyGradAcc<SY> kacc;
      kacc.clear();
      static_for<0, 4>([&](auto Q) {
        constexpr int qd = decltype(Q)::value;
        constexpr int NS = SY::NS, S0 = qd * ((NS + 3) / 4), S1 = (qd + 1) * ((NS + 3) / 4);
        sym_key_monomials_grad_range<SY, S0, S1>(kk, ds, dk, kacc, gl);
        if constexpr (qd == 3) sym_key_monomials_grad_finish<SY>(kk, dk, kacc);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = qd * NST / 4; i < (qd + 1) * NST / 4; ++i) flush_piece(i);
        constexpr int NP = NF / 2;
        flush_df(qd * ((NP + 3) / 4), (qd + 1) * ((NP + 3) / 4) < NP ? (qd + 1) * ((NP + 3) / 4) : NP);
        __builtin_amdgcn_sched_barrier(0);
      });
    }
    {
      float other[F][DP];
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int c = 0; c < DP; ++c) other[f][c] = partner32(dk[f][c]);
#pragma unroll
      for (int f = 0; f < F; ++f)
#pragma unroll
        for (int c = 0; c < DP; ++c) {
          const float v = dk[f][c] + other[f][DP - 1 - c];
          pend_df[f * DP + c] = (!relu_mask || kb[f * DP + c] > 0.0f) ? v : 0.0f;  // see k_bwd_query
        }
    }
    {
      wave_lds_sync();  // the flush above has read the whole staged tile
      u32x4 w[NRB][2];
      pack_rows<D>(acc, 1.0f, w);
      put_rows<D, 32>(w, 0, lane, tile);
      pend_n0 = n0;
    }
  }
  // the last tile's outputs
#pragma unroll
  for (int i = 0; i < NST; ++i) flush_piece(i);
  flush_df(0, NF / 2);
}

inline int pick_chunk(const hla_handle* hd, const Geom& g, int num_seqs) {
  // The chunked kernels hold one workgroup per compute unit, so a grid of more than one round is
  // mostly a second, nearly empty round, and the longest chunk sets the kernel's time: take the
  // smallest chunk (a multiple of kChunkGrain tokens) whose chunks, counted sequence by sequence
  // and times H, stay within kChunkTarget -- or one chunk per sequence when even that is too many.
  int64_t total = 0, longest = 0;
  auto len = [&](int s) -> int64_t {
    return hd->sig_packed ? hd->cu_host[s + 1] - hd->cu_host[s] : g.N;
  };
  for (int s = 0; s < num_seqs; ++s) {
    total += len(s);
    longest = len(s) > longest ? len(s) : longest;
  }
  auto count = [&](int64_t chunk) {
    int64_t c = 0;
    for (int s = 0; s < num_seqs; ++s) c += (len(s) + chunk - 1) / chunk;
    return c * g.H;
  };
  const int64_t H = g.H > 0 ? g.H : 1;
  int64_t chunk = ((total * H + kChunkTarget - 1) / kChunkTarget + kChunkGrain - 1) / kChunkGrain * kChunkGrain;
  if (chunk < kMinChunk) chunk = kMinChunk;
  while (count(chunk) > kChunkTarget && chunk < longest)
    chunk += (chunk / 64 + kChunkGrain - 1) / kChunkGrain * kChunkGrain;
  return static_cast<int>(chunk);
}

inline int pick_query_block(const Geom& g, int num_seqs, int target) {
  // The query kernel keeps two or three workgroups per compute unit (`target` in all): aim at one
  // resident round of them, in multiples of the 128 tokens a workgroup consumes per step.
  const int units = num_seqs * g.H > 0 ? num_seqs * g.H : 1;
  const int per_unit = target / units > 0 ? target / units : 1;
  const int64_t mean_len = (static_cast<int64_t>(g.B) * g.N + num_seqs - 1) / (num_seqs > 0 ? num_seqs : 1);
  const int64_t blk = ((mean_len + per_unit - 1) / per_unit + 127) / 128 * 128;
  return static_cast<int>(blk < kMinQueryBlock ? kMinQueryBlock : blk);
}

template <typename K>
hla_status allow_big_lds(K kernel, int bytes) {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                             hipFuncAttributeMaxDynamicSharedMemorySize, bytes) == hipSuccess
             ? HLA_OK
             : HLA_ERR_HIP;
}

// ---- backward of the causal variant -----------------------------------------------------------------
// With w_ij = decay^(i-j) for j <= i, den_i = eta_i + eps, Qm'_i = Qm_i / den_i, t_i = s_i den_i:
//   query side  X_i = sum_{j<=i} w_ij <dO_i, v_j> S_j,   Z_i = sum_{j<=i} w_ij S_j,
//               s_i = -<Qm_i, X_i> / den_i^2,            dQm_i = X_i / den_i + s_i Z_i
//   key side    dS_j = sum_{i>=j} w_ij (<dO_i, v_j> + t_i) Qm'_i,
//               dv_j = sum_{i>=j} w_ij <Qm'_i, S_j> dO_i
// Each sum splits into the other chunks (a state: the prefix of sum S (x) v for the queries, the
// suffix of sum w Qm' (x) dO for the keys, from the scans above as per-chunk operand images) and the
// tokens of the own chunk, which go through 32 x 32 tiles E = (other rows) (own rows)^T masked and
// weighted entry by entry, as in k_query_causal.  The two kernels below are mirror images: a
// workgroup stages the rows and the monomials of the chunk's OTHER side in LDS, then each wave
// serves two tiles of the OWN side, a token per MFMA column.
// The monomial tile is [token][MP] bf16 with its columns in the row order rho of the operand images
// (see k_prefix_rows), so that the accumulators of  X^T += M^T (W * E)  hold a lane's own slots.
template <class SY, int D>
struct CgSmem {
  static constexpr int kTiles = kCausalChunk / 32;
  static constexpr int kRStride = D * 2 + 32;          // bytes per token row of the row tile
  // bytes per token row of the monomial tile: rows 36 (52) dwords apart keep both its 8-byte row
  // reads and its transpose reads (four rows of 32 bytes per 16 lanes) off each other's banks
  static constexpr int kMStride = SY::MP * 2 + 16;
  static constexpr int kRBytes = kCausalChunk * kRStride;
  static constexpr int kMBytes = kCausalChunk * kMStride;
  static constexpr int kTBytes = kCausalChunk * 4;     // t_i of the chunk's queries (key side)
  static constexpr int kImgBytes = SY::MP * D * 2;     // one operand image of a state
  static constexpr int kLdsLimit = 160 * 1024;
  // The images of the state in front of / behind the chunk are read by every wave, for each of
  // its tiles: from an LDS copy where that fits, from memory otherwise (each wave's own loads:
  // eight times the traffic, and measured at a third of the key-side kernel's time).
  static constexpr int kBaseQ = kRBytes + kMBytes;
  static constexpr bool kImgLdsQ = kBaseQ + kImgBytes <= kLdsLimit;
  static constexpr int kTotalQ = kBaseQ + (kImgLdsQ ? kImgBytes : 0);
  static constexpr int kBaseK = kRBytes + kMBytes + kTBytes + kWaves * RowTile<D, 16>::kBytes;
  static constexpr bool kImgLdsK = kBaseK + 2 * kImgBytes <= kLdsLimit;
  static constexpr int kTotalK = kBaseK + (kImgLdsK ? 2 * kImgBytes : 0);
};


// column (in elements) of slot (g, s) in the monomial tile
__device__ __forceinline__ int rho_of(int g, int s) { return 32 * (s / 16) + 8 * ((s % 16) / 4) + 4 * g + s % 4; }

// this lane's SP monomials -> row `row` of the monomial tile (groups of four slots are four
// consecutive columns)
template <class SY>
__device__ __forceinline__ void put_monomials(unsigned char* mt, int stride, int row, int gl,
                                              const float (&m)[SY::SP], float scale) {
#pragma unroll
  for (int q4 = 0; q4 < SY::SP / 4; ++q4) {
    u32x2 w;
    w[0] = pack_bf16(m[4 * q4] * scale, m[4 * q4 + 1] * scale);
    w[1] = pack_bf16(m[4 * q4 + 2] * scale, m[4 * q4 + 3] * scale);
    *reinterpret_cast<u32x2*>(mt + row * stride + rho_of(gl, 4 * q4) * 2) = w;
  }
}

// E[other token d_row(i, gl) of tile u][own token r] = <row_other, row_own>: A = plain 16-byte reads
// of the row tile, B = the own rows in operand order
template <int D>
__device__ __forceinline__ f32x16 rows_product(const unsigned char* rt, int stride, int u, int lane,
                                               const u32x4 (&bown)[D / 16]) {
  const int r = lane % 32, gl = lane / 32;
  // all operands are requested before the first MFMA: one exposed LDS round trip per product
  u32x4 a[D / 16];
#pragma unroll
  for (int kd = 0; kd < D / 16; ++kd)
    a[kd] = *reinterpret_cast<const u32x4*>(rt + (32 * u + r) * stride + (16 * kd + 8 * gl) * 2);
  __builtin_amdgcn_sched_barrier(0);
  f32x16 E;
#pragma unroll
  for (int i = 0; i < 16; ++i) E[i] = 0.0f;
#pragma unroll
  for (int kd = 0; kd < D / 16; ++kd) E = mfma32(a[kd], bown[kd], E);
  return E;
}

// acc[blk]^T[32 blk + .. x own] += tile(u)^T B for the NB 32-column blocks of a [token][columns]
// tile: k-slot (ks2, gl, j) of B is token 16 ks2 + 8 (j / 4) + 4 gl + j % 4 of tile u, the order
// in which a product's accumulators hold its rows
template <int NB>
__device__ __forceinline__ void transposed_product(const unsigned char* tile, int stride, int u, int lane,
                                                   const u32x4 (&b)[2], f32x16 (&acc)[NB]) {
  const int gl = lane / 32, L = lane % 16, q = lane / 16;
  u32x4 a[2][NB];  // all operands are requested before the first MFMA
#pragma unroll
  for (int ks2 = 0; ks2 < 2; ++ks2) {
    const int krow = 32 * u + 16 * ks2 + 4 * gl + L / 4;
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
      const unsigned char* p = tile + krow * stride + (32 * blk + 16 * (q % 2) + 4 * (L % 4)) * 2;
      const u32x2 lo = lds_read_tr16(p);
      const u32x2 hi = lds_read_tr16(p + 8 * stride);
      a[ks2][blk][0] = lo[0];
      a[ks2][blk][1] = lo[1];
      a[ks2][blk][2] = hi[0];
      a[ks2][blk][3] = hi[1];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) acc[blk] = mfma32(a[ks2][blk], b[ks2], acc[blk]);
}

// grid (chunks of kCausalChunk tokens, H), block 256.  Query side: writes the query part of the
// feature gradients and s_i (sv) for the key side.  rows_img / z_img: per (chunk, head) the
// monomial-row image of the state in front of the chunk and its normaliser by slot.
template <class SY, int D>
__global__ __launch_bounds__(causal_query_waves<SY>() * 64) void k_cgrad_q(Geom g, const BlockEnt* __restrict__ chunks,
                                                      const float* __restrict__ feat,
                                                      const float* __restrict__ den, View V, View dO,
                                                      const unsigned char* __restrict__ rows_img,
                                                      int64_t rows_stride,
                                                      const unsigned char* __restrict__ z_img,
                                                      int64_t z_stride, float* __restrict__ dfeat,
                                                      float* __restrict__ sv, float log2_decay,
                                                      int relu_mask) {
  using SM = CgSmem<SY, D>;
  constexpr int SP = SY::SP, MP = SY::MP, DP = SY::DPHI, F = SY::F;
  constexpr int NKD = D / 16, NRM = MP / 32, NF = F * DP;
  constexpr int WAVES = causal_query_waves<SY>();      // see k_query_causal
  constexpr int kRowsPW = kCausalChunk / WAVES;        // rows a wave stages
  constexpr int kTilesPW = kCausalChunk / 32 / WAVES;  // tiles a wave stages and serves
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  unsigned char* rt = smem;
  unsigned char* mt = smem + SM::kRBytes;
  const int r = lane % 32, gl = lane / 32;
  const BlockEnt e = chunks[blockIdx.x];
  const int h = blockIdx.y;
  const int64_t ch_h = static_cast<int64_t>(blockIdx.x) * g.H + h;
  // the monomial-row image of the state in front of the chunk: an LDS copy where it fits
  // a query tile's inputs: its dO row in operand order, its features and den (tokens beyond the
  // chunk read its last token and are zeroed when used)
  auto request_query = [&](int qt, u32x4 (&bdo)[NKD], f32x2 (&fraw)[DP / 2], float& dn) {
    const int n = e.t0 + 32 * qt + r;
    const int nc = n < e.t1 ? n : e.t1 - 1;
    const bf16_t* row = dO.row<const bf16_t>(e.b, h, nc);
#pragma unroll
    for (int kd = 0; kd < NKD; ++kd) bdo[kd] = *reinterpret_cast<const u32x4*>(row + 16 * kd + 8 * gl);
    const int64_t th = g.th(e.b, h, nc);
    const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(th, 0));
#pragma unroll
    for (int p = 0; p < DP / 2; ++p) fraw[p] = f[32 * p];
    dn = den[th];
  };
  const int qt_first = WAVES == 8 ? (wave < 4 ? wave : 11 - wave) : chunk_tile_of(wave, 0);
  // ---- everything the start needs from memory, requested at once: the monomial-row image of the
  // state in front of the chunk (an LDS copy where it fits), the chunk's V rows and the key features
  // of the tiles this wave stages (an equal share per wave), the inputs of its first query tile
  ImageCopy<SM::kImgLdsQ ? SM::kImgBytes : 16, WAVES * 64> image;
  if constexpr (SM::kImgLdsQ) image.request(rows_img + ch_h * rows_stride);
  TileRegs<D, kRowsPW> vt;
  fetch_tile<D, kRowsPW>(V, e.b, h, e.t0 + kRowsPW * wave, e.t1, lane, vt);
  f32x2 kraw[kTilesPW][NF / 2];
#pragma unroll
  for (int tt = 0; tt < kTilesPW; ++tt) {
    const int n = e.t0 + 32 * (kTilesPW * wave + tt) + r;
    const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(g.th(e.b, h, n < e.t1 ? n : e.t1 - 1), DP));
#pragma unroll
    for (int p = 0; p < NF / 2; ++p) kraw[tt][p] = f[32 * p];
  }
  u32x4 bdo0[NKD];
  f32x2 fraw0[DP / 2];
  float dn0;
  request_query(qt_first, bdo0, fraw0, dn0);
  // ---- the staged tiles: V rows and key monomials
  if constexpr (SM::kImgLdsQ) image.commit(smem + SM::kBaseQ);
  put_tile<D, kRowsPW>(vt, lane, rt + kRowsPW * wave * SM::kRStride, SM::kRStride);
#pragma unroll
  for (int tt = 0; tt < kTilesPW; ++tt) {
    const int t = kTilesPW * wave + tt;
    const bool live_k = e.t0 + 32 * t + r < e.t1;
    float kf[NF], kr[NF];
#pragma unroll
    for (int p = 0; p < NF / 2; ++p) {
      kf[2 * p] = live_k ? kraw[tt][p][0] : 0.0f;
      kf[2 * p + 1] = live_k ? kraw[tt][p][1] : 0.0f;
    }
    float kk[F][DP];
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
      for (int c = 0; c < DP; ++c) kr[f * DP + c] = kf[(f + 1) * DP - 1 - c];
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
      for (int c = 0; c < DP; ++c) kk[f][c] = gl ? kr[f * DP + c] : kf[f * DP + c];
    float sm[SP];
    sym_key_monomials_slots<SY>(kk, sm, gl);
    put_monomials<SY>(mt, SM::kMStride, 32 * t + r, gl, sm, 1.0f);
  }
  __syncthreads();
  // decay^(31 - key row of accumulator register i): the per-register part of an off-diagonal
  // tile's weights (at most 1; 1 without decay)
  float rowfac[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
    rowfac[i] = log2_decay != 0.0f ? __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(31 - d_row(i, gl))) : 1.0f;
  const u32x4* opB = reinterpret_cast<const u32x4*>(SM::kImgLdsQ ? smem + SM::kBaseQ : rows_img + ch_h * rows_stride);
  const float* zslot = reinterpret_cast<const float*>(z_img + ch_h * z_stride) + gl * SP;
#pragma unroll 1
  for (int qi = 0; qi < kTilesPW; ++qi) {
    const int qt = WAVES == 8 ? (wave < 4 ? wave : 11 - wave) : chunk_tile_of(wave, qi);
    const int n0 = e.t0 + 32 * qt;
    if (n0 >= e.t1) continue;
    const int n = n0 + r;
    const bool live = n < e.t1;
    const int64_t th = g.th(e.b, h, live ? n : e.t1 - 1);
    u32x4 bdo[NKD];
    f32x2 fraw[DP / 2];
    float dn;
    if (qi == 0) {  // requested before the staging
#pragma unroll
      for (int kd = 0; kd < NKD; ++kd) bdo[kd] = bdo0[kd];
#pragma unroll
      for (int p = 0; p < DP / 2; ++p) fraw[p] = fraw0[p];
      dn = dn0;
    } else {
      request_query(qt, bdo, fraw, dn);
    }
    if (!live) {
#pragma unroll
      for (int kd = 0; kd < NKD; ++kd) bdo[kd][0] = bdo[kd][1] = bdo[kd][2] = bdo[kd][3] = 0u;
    }
    float fb[DP], qf[DP];
    {
#pragma unroll
      for (int p = 0; p < DP / 2; ++p) {
        fb[2 * p] = live ? fraw[p][0] : 0.0f;
        fb[2 * p + 1] = live ? fraw[p][1] : 0.0f;
      }
      float fr[DP];
#pragma unroll
      for (int c = 0; c < DP; ++c) fr[c] = fb[DP - 1 - c];
#pragma unroll
      for (int c = 0; c < DP; ++c) qf[c] = gl ? fr[c] : fb[c];
    }
    const float inv = live ? 1.0f / dn : 0.0f;
    float qm[SP];
    sym_query_monomials<SY>(qf, qm, gl);
    // the chunks in front: X = (state) dO^T, Z = its normaliser, both as seen from the chunk's
    // first token
    f32x16 X[NRM], Z[NRM];
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb) {
#pragma unroll
      for (int i = 0; i < 16; ++i) X[rb][i] = 0.0f;
#pragma unroll
      for (int kd = 0; kd < NKD; ++kd) X[rb] = mfma32(opB[(rb * NKD + kd) * 64 + lane], bdo[kd], X[rb]);
#pragma unroll
      for (int i4 = 0; i4 < 4; ++i4) {
        const f32x4 z = *reinterpret_cast<const f32x4*>(zslot + 16 * rb + 4 * i4);
#pragma unroll
        for (int i = 0; i < 4; ++i) Z[rb][4 * i4 + i] = z[i];
      }
    }
    if (log2_decay != 0.0f) {
      const float wq = __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(32 * qt + r));
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          X[rb][i] *= wq;
          Z[rb][i] *= wq;
        }
    }
    // the chunk's own keys up to the query: key tiles 0 .. qt
#pragma unroll 1
    for (int kt = 0; kt <= qt; ++kt) {
      const f32x16 E = rows_product<D>(rt, SM::kRStride, kt, lane, bdo);
      // weights of the tile's entries (key d_row(i, gl) of tile kt against query r): 1 in front of
      // the diagonal tile, there 0 behind the query; with a decay factor decay^(distance), which
      // in front of the diagonal tile (distance >= 1) factors into a per-lane and a per-register
      // part
      u32x4 bE[2], bW[2];
      if (kt < qt) {
        const float cw = log2_decay != 0.0f ? __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(32 * (qt - kt) + r - 31)) : 1.0f;
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const int i = 8 * ks2 + 2 * p;
            const float w0 = cw * rowfac[i], w1 = cw * rowfac[i + 1];
            bE[ks2][p] = pack_bf16(E[i] * w0, E[i + 1] * w1);
            bW[ks2][p] = pack_bf16(w0, w1);
          }
      } else {
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            float wv[2];
#pragma unroll
            for (int x = 0; x < 2; ++x) {
              const float dist = static_cast<float>(r - d_row(8 * ks2 + 2 * p + x, gl));
              wv[x] = dist < 0.0f ? 0.0f : (log2_decay != 0.0f ? __builtin_amdgcn_exp2f(log2_decay * dist) : 1.0f);
            }
            bE[ks2][p] = pack_bf16(E[8 * ks2 + 2 * p] * wv[0], E[8 * ks2 + 2 * p + 1] * wv[1]);
            bW[ks2][p] = pack_bf16(wv[0], wv[1]);
          }
      }
      transposed_product<NRM>(mt, SM::kMStride, kt, lane, bE, X);
      transposed_product<NRM>(mt, SM::kMStride, kt, lane, bW, Z);
    }
    // s_i from the same X that feeds dQm (the component along Qm cancels exactly), chain rule
    float dot = 0.0f;
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) dot += qm[16 * rb + i] * X[rb][i];
    dot += partner32(dot);
    const float si = -(inv * inv) * dot;
    float dm[SP];
#pragma unroll
    for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
      for (int i = 0; i < 16; ++i) dm[16 * rb + i] = inv * X[rb][i] + si * Z[rb][i];
    float dq[DP];
#pragma unroll
    for (int c = 0; c < DP; ++c) dq[c] = 0.0f;
    sym_query_monomials_grad<SY>(qf, dm, dq, gl);
    float other[DP];
#pragma unroll
    for (int c = 0; c < DP; ++c) other[c] = partner32(dq[c]);
    if (live && gl == 0) {
      f32x2* df = reinterpret_cast<f32x2*>(dfeat + g.fidx(th, 0));
#pragma unroll
      for (int c = 0; c < DP; c += 2) {
        f32x2 v;
        v[0] = (!relu_mask || fb[c] > 0.0f) ? dq[c] + other[DP - 1 - c] : 0.0f;
        v[1] = (!relu_mask || fb[c + 1] > 0.0f) ? dq[c + 1] + other[DP - 2 - c] : 0.0f;
        df[32 * (c / 2)] = v;
      }
      sv[th] = si;
    }
  }
}

// grid (chunks of kCausalChunk tokens, H), block of eight waves.  Key side: writes the key part of
// the feature gradients and dV.  dops: per (chunk, head) the images of the gradient state behind
// the chunk.  A key tile has two results, dS (-> the feature gradients) and dv, which share nothing
// but the tile's weights: wave w < 4 computes dS and wave w + 4 (same SIMD) dv of key tiles w and
// 7 - w, twelve MFMAs per query tile each, so that a SIMD always has a second wave to run while one
// waits for LDS, and each role's live set fits the 256 registers a wave then has.
constexpr int kWavesCK = 8;
static_assert(kCausalChunk / 32 == kWavesCK, "one staged tile per wave, two key tiles per wave pair");

// weights of a tile's entries (query d_row(i, gl) of tile qt against key r of tile kt): 1 behind
// the diagonal tile, there 0 for queries in front of the key; with a decay factor
// decay^(distance), factored behind the diagonal tile (distance >= 1) into a per-lane and a
// per-register part (rowfac[i] = decay^d_row(i, gl))
__device__ __forceinline__ void key_tile_weights(int qt, int kt, int r, int gl, float log2_decay,
                                                 const float (&rowfac)[16], float (&wv)[16]) {
  const float cw = qt > kt && log2_decay != 0.0f
                       ? __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(32 * (qt - kt) - r))
                       : 1.0f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (qt > kt) {
      wv[i] = cw * rowfac[i];
    } else {
      const float dist = static_cast<float>(d_row(i, gl) - r);
      wv[i] = dist < 0.0f ? 0.0f : (log2_decay != 0.0f ? __builtin_amdgcn_exp2f(log2_decay * dist) : 1.0f);
    }
  }
}

template <class SY, int D>
__global__ __launch_bounds__(kWavesCK * 64) void k_cgrad_k(
    Geom g, const BlockEnt* __restrict__ chunks, const float* __restrict__ feat,
    const float* __restrict__ den, const float* __restrict__ sv, View V, View dO,
    const unsigned char* __restrict__ dops, float* __restrict__ dfeat, View dV, float log2_decay,
    int relu_mask) {
  using SM = CgSmem<SY, D>;
  using SL = StateLayout<SY, D>;
  constexpr int SP = SY::SP, MP = SY::MP, DP = SY::DPHI, F = SY::F;
  constexpr int NRB = D / 32, NKD = D / 16, NRM = MP / 32, NKS = MP / 16, NF = F * DP;
  constexpr int kRowsPW = kCausalChunk / kWavesCK;  // rows a wave stages
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = wave_index();
  const int wt = wave % 4;  // this wave's share of the key tiles: wt and 7 - wt
  unsigned char* rt = smem;
  unsigned char* mt = smem + SM::kRBytes;
  float* tq = reinterpret_cast<float*>(smem + SM::kRBytes + SM::kMBytes);
  unsigned char* tile = smem + SM::kRBytes + SM::kMBytes + SM::kTBytes + wt * RowTile<D, 16>::kBytes;
  const int r = lane % 32, gl = lane / 32;
  const BlockEnt e = chunks[blockIdx.x];
  const int h = blockIdx.y;
  const unsigned char* pu = dops + (static_cast<int64_t>(blockIdx.x) * g.H + h) * SL::kOpBytes;
  const u32x4* opA = reinterpret_cast<const u32x4*>(SM::kImgLdsK ? smem + SM::kBaseK : pu);
  const u32x4* opB = reinterpret_cast<const u32x4*>(SM::kImgLdsK ? smem + SM::kBaseK + SM::kImgBytes : pu + SL::kOpElems * 2);
  // a key tile's inputs: its key features and, for the dS role, its V row in operand order
  // (tokens beyond the chunk read the chunk's last token and are zeroed when used)
  auto request_key = [&](int kt, f32x2 (&kraw)[NF / 2], u32x4 (&bv)[NKD]) {
    const int n = e.t0 + 32 * kt + r;
    const int nc = n < e.t1 ? n : e.t1 - 1;
    const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(g.th(e.b, h, nc), DP));
#pragma unroll
    for (int p = 0; p < NF / 2; ++p) kraw[p] = f[32 * p];
    if (wave < 4) {
      const bf16_t* row = V.row<const bf16_t>(e.b, h, nc);
#pragma unroll
      for (int kd = 0; kd < NKD; ++kd) bv[kd] = *reinterpret_cast<const u32x4*>(row + 16 * kd + 8 * gl);
    }
  };
  // ---- everything the start needs from memory, requested at once: the two images of the gradient
  // state behind the chunk (channel rows for dv, monomial rows for dS), the chunk's dO rows, the
  // query features, den and s of the 32 tokens this wave stages, the first key tile's inputs
  ImageCopy<SM::kImgLdsK ? 2 * SM::kImgBytes : 16, kWavesCK * 64> images;
  if constexpr (SM::kImgLdsK) images.request(pu);
  TileRegs<D, kRowsPW> vt;
  fetch_tile<D, kRowsPW>(dO, e.b, h, e.t0 + kRowsPW * wave, e.t1, lane, vt);
  const int ns = e.t0 + 32 * wave + r;  // the token whose monomials this lane stages
  const bool live_s = ns < e.t1;
  const int64_t th_s = g.th(e.b, h, live_s ? ns : e.t1 - 1);
  f32x2 qraw[DP / 2];
  {
    const f32x2* f = reinterpret_cast<const f32x2*>(feat + g.fidx(th_s, 0));
#pragma unroll
    for (int p = 0; p < DP / 2; ++p) qraw[p] = f[32 * (gl ? DP / 2 - 1 - p : p)];  // lane half 1: pairs in reverse
  }
  const float dn_s = den[th_s], sv_s = sv[th_s];
  f32x2 kraw0[NF / 2];
  u32x4 bv0[NKD];
  request_key(wt, kraw0, bv0);
  // ---- the staged tiles: dO rows, scaled query monomials Qm / den and t = s den
  if constexpr (SM::kImgLdsK) images.commit(smem + SM::kBaseK);
  put_tile<D, kRowsPW>(vt, lane, rt + kRowsPW * wave * SM::kRStride, SM::kRStride);
  {
    float qf[DP];
#pragma unroll
    for (int p = 0; p < DP / 2; ++p) {  // and each pair in reverse
      qf[2 * p] = live_s ? (gl ? qraw[p][1] : qraw[p][0]) : 0.0f;
      qf[2 * p + 1] = live_s ? (gl ? qraw[p][0] : qraw[p][1]) : 0.0f;
    }
    float qm[SP];
    sym_query_monomials<SY>(qf, qm, gl);
    put_monomials<SY>(mt, SM::kMStride, 32 * wave + r, gl, qm, live_s ? 1.0f / dn_s : 0.0f);
    if (gl == 0) tq[32 * wave + r] = live_s ? sv_s * dn_s : 0.0f;
  }
  __syncthreads();
  float rowfac[16];
#pragma unroll
  for (int i = 0; i < 16; ++i)
    rowfac[i] = log2_decay != 0.0f ? __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(d_row(i, gl))) : 1.0f;
  const int last = (e.t1 - e.t0 + 31) / 32 - 1;  // the chunk's last query tile
  // one key tile; FIRST: the wave's first, whose inputs were requested before the staging
  auto key_tile = [&](int kt, auto first_tag) {
    constexpr bool FIRST = decltype(first_tag)::value;
    const int n0 = e.t0 + 32 * kt;
    if (n0 >= e.t1) return;
    const int n = n0 + r;
    const bool live = n < e.t1;
    const int64_t th = g.th(e.b, h, live ? n : e.t1 - 1);
    f32x2 kraw[NF / 2];
    u32x4 bv[NKD];
    if constexpr (FIRST) {
#pragma unroll
      for (int p = 0; p < NF / 2; ++p) kraw[p] = kraw0[p];
#pragma unroll
      for (int kd = 0; kd < NKD; ++kd) bv[kd] = bv0[kd];
    } else {
      request_key(kt, kraw, bv);
    }
    // the key's features: lane half 1 holds every map's reversed
    float kk[F][DP];
    {
      float kb[NF], kr[NF];
#pragma unroll
      for (int p = 0; p < NF / 2; ++p) {
        kb[2 * p] = live ? kraw[p][0] : 0.0f;
        kb[2 * p + 1] = live ? kraw[p][1] : 0.0f;
      }
#pragma unroll
      for (int f2 = 0; f2 < F; ++f2)
#pragma unroll
        for (int c = 0; c < DP; ++c) kr[f2 * DP + c] = kb[(f2 + 1) * DP - 1 - c];
#pragma unroll
      for (int f2 = 0; f2 < F; ++f2)
#pragma unroll
        for (int c = 0; c < DP; ++c) kk[f2][c] = gl ? kr[f2 * DP + c] : kb[f2 * DP + c];
    }
    // the chunks behind enter as seen from the chunk's last token
    const float wk = log2_decay != 0.0f
                         ? __builtin_amdgcn_exp2f(log2_decay * static_cast<float>(kCausalChunk - 1 - (32 * kt + r)))
                         : 1.0f;
    if (wave < 4) {
      // ---- dS^T = (gradient state) v + dz  +  sum over the chunk's queries, then the chain rule
      const float* dzslot = reinterpret_cast<const float*>(pu + 2 * SL::kOpElems * 2) + gl * SP;
      if (!live) {
#pragma unroll
        for (int kd = 0; kd < NKD; ++kd) bv[kd][0] = bv[kd][1] = bv[kd][2] = bv[kd][3] = 0u;
      }
      f32x16 Y[NRM];
#pragma unroll
      for (int rb = 0; rb < NRM; ++rb) {
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4) {
          const f32x4 z = *reinterpret_cast<const f32x4*>(dzslot + 16 * rb + 4 * i4);
#pragma unroll
          for (int i = 0; i < 4; ++i) Y[rb][4 * i4 + i] = z[i];
        }
#pragma unroll
        for (int kd = 0; kd < NKD; ++kd) Y[rb] = mfma32(opB[(rb * NKD + kd) * 64 + lane], bv[kd], Y[rb]);
      }

      if (log2_decay != 0.0f) {
#pragma unroll
        for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
          for (int i = 0; i < 16; ++i) Y[rb][i] *= wk;
      }
#pragma unroll 1
      for (int qt = kt; qt <= last; ++qt) {
        float wv[16];
        key_tile_weights(qt, kt, r, gl, log2_decay, rowfac, wv);
        const f32x16 E = rows_product<D>(rt, SM::kRStride, qt, lane, bv);  // <dO_i, v_j>
        u32x4 bE[2];
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
          // t of query d_row(i, gl) = 16 ks2 + 8 (p / 2) + 4 gl + (2 p + x) % 4, i = 8 ks2 + 2 p + x
          const f32x4 t0 = *reinterpret_cast<const f32x4*>(tq + 32 * qt + 16 * ks2 + 4 * gl);
          const f32x4 t1 = *reinterpret_cast<const f32x4*>(tq + 32 * qt + 16 * ks2 + 4 * gl + 8);
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const int i = 8 * ks2 + 2 * p;
            const float ta = p < 2 ? t0[(2 * p) % 4] : t1[(2 * p) % 4];
            const float tb = p < 2 ? t0[(2 * p + 1) % 4] : t1[(2 * p + 1) % 4];
            bE[ks2][p] = pack_bf16((E[i] + ta) * wv[i], (E[i + 1] + tb) * wv[i + 1]);
          }
        }
        transposed_product<NRM>(mt, SM::kMStride, qt, lane, bE, Y);
      }
      float dk[F][DP];
      {
        float ds[SP];
#pragma unroll
        for (int rb = 0; rb < NRM; ++rb)
#pragma unroll
          for (int i = 0; i < 16; ++i) ds[16 * rb + i] = Y[rb][i];
#pragma unroll
        for (int f2 = 0; f2 < F; ++f2)
#pragma unroll
          for (int c = 0; c < DP; ++c) dk[f2][c] = 0.0f;
        KeyGradAcc<SY> kacc;
        kacc.clear();
        sym_key_monomials_grad_range<SY, 0, SY::NS>(kk, ds, dk, kacc, gl);
        sym_key_monomials_grad_finish<SY>(kk, dk, kacc);
      }
      float other[F][DP];
#pragma unroll
      for (int f2 = 0; f2 < F; ++f2)
#pragma unroll
        for (int c = 0; c < DP; ++c) other[f2][c] = partner32(dk[f2][c]);
      if (live && gl == 0) {
        f32x2* df = reinterpret_cast<f32x2*>(dfeat + g.fidx(th, DP));
#pragma unroll
        for (int p = 0; p < NF / 2; ++p) {
          f32x2 v;
#pragma unroll
          for (int x = 0; x < 2; ++x) {
            const int a = 2 * p + x, f2 = a / DP, c = a % DP;
            const float val = dk[f2][c] + other[f2][DP - 1 - c];
            v[x] = (!relu_mask || kk[f2][c] > 0.0f) ? val : 0.0f;  // gl == 0: the features in order
          }
          df[32 * p] = v;
        }
      }
    } else {
      // ---- dv^T = (gradient state)^T S  +  sum over the chunk's queries of w <Qm'_i, S_j> dO_i
      u32x4 bS[NKS];
      {
        float sm[SP];
        sym_key_monomials_slots<SY>(kk, sm, gl);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
          for (int p = 0; p < 4; ++p) bS[ks][p] = pack_bf16(sm[8 * ks + 2 * p], sm[8 * ks + 2 * p + 1]);
      }
      f32x16 dvT[NRB];
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int i = 0; i < 16; ++i) dvT[rb][i] = 0.0f;
#pragma unroll 1
      for (int qt = kt; qt <= last; ++qt) {
        float wv[16];
        key_tile_weights(qt, kt, r, gl, log2_decay, rowfac, wv);
        // <Qm'_i, S_j>: A = row reads of the monomial tile, the eight k-slots (g, 8 ks + j) of a
        // k-step as two runs of four columns
        u32x4 am[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          const unsigned char* p = mt + (32 * qt + r) * SM::kMStride + rho_of(gl, 8 * ks) * 2;
          const u32x2 lo = *reinterpret_cast<const u32x2*>(p);
          const u32x2 hi = *reinterpret_cast<const u32x2*>(p + 16);
          am[ks][0] = lo[0];
          am[ks][1] = lo[1];
          am[ks][2] = hi[0];
          am[ks][3] = hi[1];
        }
        f32x16 A;
#pragma unroll
        for (int i = 0; i < 16; ++i) A[i] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) A = mfma32(am[ks], bS[ks], A);
        u32x4 bA[2];
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
          for (int p = 0; p < 4; ++p) {
            const int i = 8 * ks2 + 2 * p;
            bA[ks2][p] = pack_bf16(A[i] * wv[i], A[i + 1] * wv[i + 1]);
          }
        transposed_product<NRB>(rt, SM::kRStride, qt, lane, bA, dvT);
      }
      // the chunks behind (the key's weight wk goes into the B operand)
      {
        u32x4 bSw[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
          for (int p = 0; p < 4; ++p)
            bSw[ks][p] = log2_decay != 0.0f ? pack_bf16(bf16_lo(bS[ks][p]) * wk, bf16_hi(bS[ks][p]) * wk) : bS[ks][p];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
          for (int ks = 0; ks < NKS; ++ks) dvT[rb] = mfma32(opA[(rb * NKS + ks) * 64 + lane], bSw[ks], dvT[rb]);
      }
      store_rows_bf16<D, 16>(dvT, 1.0f, lane, tile, [&](int t) -> bf16_t* {
        return n0 + t < e.t1 ? dV.row<bf16_t>(e.b, h, n0 + t) : nullptr;
      });
    }
  };
  key_tile(wt, std::true_type{});
  key_tile(kCausalChunk / 32 - 1 - wt, std::false_type{});
}

template <class SY, int D>
hla_status backward_causal(hla_handle* hd, const hla_call_args& a) {
  using SL = StateLayout<SY, D>;
  using SM = StateSmem<D, SY::MP>;
  using SG = CgSmem<SY, D>;
  Geom g = hd->g;
  hipStream_t s = a.stream;
  hla_token_table* cch = nullptr;
  HLA_TRY(get_table(hd, 2, kCausalChunk, s, &cch));
  if (static_cast<int64_t>(cch->count) * g.H > hd->max_chunks * hd->cfg.max_heads) return HLA_ERR_INVALID_ARG;
  // images of the state in front of every chunk, then of the gradient state behind it
  unsigned char* ops = static_cast<unsigned char*>(hd->path_ws) + hd->causal_bwd_off;
  unsigned char* dops = ops + SL::kOpBytes * hd->max_chunks * hd->cfg.max_heads;
  const float dec = hd->cfg.decay > 0.0f && hd->cfg.decay < 1.0f ? hd->cfg.decay : 1.0f;
  const float l2d = dec < 1.0f ? std::log2(dec) : 0.0f;
  const float chunk_decay = dec < 1.0f ? std::pow(dec, static_cast<float>(kCausalChunk)) : 1.0f;
  const int relu_mask = hd->cfg.phi_mode == HLA_PHI_MLP ? 1 : 0;
  const CanonMap cm = make_canon_map<SY>();
  const int64_t stride = SL::kOpBytes, z_off = 2 * SL::kOpElems * 2, b_off = SL::kOpElems * 2;
  const dim3 sgrid(a.num_seqs, g.H, kScanParts * 2 * (SY::MP / 16) * D / kScanThreads + 1);
  const dim3 rgrid(a.num_seqs, g.H, kScanPartsRows * (SY::MP / 32) * (D / 16) * 64 / kScanThreads);
  static_assert((SY::MP / 32) * (D / 16) * 64 % kScanThreads == 0, "whole workgroups of row-image items");
  const float* nof = nullptr;
  using PL = PrefixLayout<SY, D>;
  const unsigned char* pfx = static_cast<unsigned char*>(hd->path_ws) + hd->causal_off;
  // The forward left the chunks' own states in the partial buffer and their running sum (operand
  // image by channels, normaliser) in its prefix images; what the query side needs on top is the
  // image by monomial rows.  A second backward after the same forward finds the partial buffer
  // holding gradient states and computes the chunk states again.
  // A handle that has run a backward before has its forwards write that image too (one scan
  // launch for both, see forward_causal), and it stays valid until the next forward.
  if (!hd->causal_rows_valid) {
    if (!hd->causal_partials_valid)
      HLA_TRY(launch(hd, "mfma_state", k_state<SY, D, 0, true>, dim3((cch->count + kWaves - 1) / kWaves, g.H),
                     dim3(kThreads), SM::kTotal, s, g, cch->dev, hd->feat, a.V, hd->partial, SL::kF32, l2d, nof, nof,
                     cch->count));
    HLA_TRY(launch(hd, "mfma_state_prefix_rows", k_prefix_rows<SY, D, false>, rgrid, dim3(kScanThreads), 0, s, g,
                   cch->seq_off_dev, hd->partial, SL::kF32, ops, cm, chunk_decay, stride, b_off));
    hd->causal_rows_valid = true;
  }
  hd->causal_seen_backward = true;
  HLA_TRY(launch(hd, "mfma_causal_grad_query", k_cgrad_q<SY, D>, dim3(cch->count, g.H), dim3(causal_query_waves<SY>() * 64),
                 SG::kTotalQ, s, g, cch->dev, hd->feat, hd->den, a.V, a.dO,
                 static_cast<const unsigned char*>(ops + b_off), stride,
                 pfx + PL::kOpElems * 2, static_cast<int64_t>(PL::kBytes), hd->dfeat, hd->yhat, l2d, relu_mask));
  hd->causal_partials_valid = false;
  // gradient states of the chunks, summed from the back
  HLA_TRY(launch(hd, "mfma_dstate", k_state<SY, D, 1, true>, dim3((cch->count + kWaves - 1) / kWaves, g.H),
                 dim3(kThreads), SM::kTotal, s, g, cch->dev, hd->feat, a.dO, hd->partial, SL::kF32, l2d,
                 static_cast<const float*>(hd->den), static_cast<const float*>(hd->yhat), cch->count));
  HLA_TRY(launch(hd, "mfma_dstate_suffix", k_prefix_both<SY, D, true>, dim3(a.num_seqs, g.H, sgrid.z + rgrid.z),
                 dim3(kScanThreads), 0, s, g, cch->seq_off_dev, hd->partial, SL::kF32, dops, cm, chunk_decay, stride,
                 z_off, dops, stride, b_off, static_cast<int>(sgrid.z)));
  HLA_TRY(launch(hd, "mfma_causal_grad_key", k_cgrad_k<SY, D>, dim3(cch->count, g.H), dim3(kWavesCK * 64),
                 SG::kTotalK, s, g, cch->dev, hd->feat, hd->den, static_cast<const float*>(hd->yhat), a.V, a.dO,
                 dops, hd->dfeat, a.dV, l2d, relu_mask));
  return HLA_OK;
}

template <class SY, int D>
hla_status backward_core(hla_handle* hd, const hla_call_args& a) {
  using SL = StateLayout<SY, D>;
  using SQ = BwdQSmem<D, SY::MP>;
  Geom g = hd->g;
  hipStream_t s = a.stream;
  const int chunk = pick_chunk(hd, g, a.num_seqs);
  hla_token_table* chunks = nullptr;
  HLA_TRY(get_table(hd, 0, chunk, s, &chunks));
  unsigned char* ops = static_cast<unsigned char*>(hd->path_ws);
  unsigned char* dops = ops + SL::kOpBytes * hd->max_units;
  const int relu_mask = hd->cfg.phi_mode == HLA_PHI_MLP ? 1 : 0;
  HLA_TRY(launch(hd, "mfma_bwd_query", k_bwd_query<SY, D>, dim3(chunks->count, g.H), dim3(kThreads),
                 SQ::kTotal, s, g, chunks->dev, hd->feat, hd->den, ops, a.dO, hd->dfeat,
                 hd->partial, SL::kF32, relu_mask));
  HLA_TRY(launch(hd, "mfma_dstate_reduce", k_reduce<SY, D, true>, dim3(a.num_seqs, g.H, kReduceSlices),
                 dim3(256), 0, s, g, chunks->seq_off_dev, hd->partial, SL::kF32, dops,
                 make_slot_map<SY>()));
  HLA_TRY(launch(hd, "mfma_bwd_key", k_bwd_key<SY, D>, dim3(chunks->count, g.H), dim3(kThreads),
                 0, s, g, chunks->dev, hd->feat, dops, a.V, hd->dfeat, a.dV, relu_mask));
  return HLA_OK;
}

template <class SY, int D>
hla_status forward_core(hla_handle* hd, const hla_call_args& a) {
  using SL = StateLayout<SY, D>;
  using SM = StateSmem<D, SY::MP>;
  Geom g = hd->g;
  hipStream_t s = a.stream;
  const int chunk = pick_chunk(hd, g, a.num_seqs);
  hla_token_table *chunks = nullptr, *qblocks = nullptr;
  HLA_TRY(get_table(hd, 0, chunk, s, &chunks));
  HLA_TRY(get_table(hd, 1, pick_query_block(g, a.num_seqs, query_target<SY>()), s, &qblocks));
  if (static_cast<int64_t>(chunks->count) * g.H > hd->max_chunks * hd->cfg.max_heads)
    return HLA_ERR_INVALID_ARG;
  HLA_TRY(launch(hd, "mfma_state", k_state<SY, D>, dim3(chunks->count, g.H), dim3(kThreads),
                 SM::kTotal, s, g, chunks->dev, hd->feat, a.V, hd->partial, SL::kF32, 0.0f, static_cast<const float*>(nullptr), static_cast<const float*>(nullptr), 0));
  const SlotMap sm = make_slot_map<SY>();
  unsigned char* ops = static_cast<unsigned char*>(hd->path_ws);
  HLA_TRY(launch(hd, "mfma_state_reduce", k_reduce<SY, D, false>, dim3(a.num_seqs, g.H, kReduceSlices),
                 dim3(256), 0, s, g, chunks->seq_off_dev, hd->partial, SL::kF32, ops, sm));
  HLA_TRY(launch(hd, "mfma_query", k_query<SY, D>, dim3(qblocks->count, g.H), dim3(kThreads), 0, s,
                 g, qblocks->dev, hd->feat, ops, a.O, hd->den));
  return HLA_OK;
}

template <class SY, int D>
hla_status forward_causal(hla_handle* hd, const hla_call_args& a) {
  using SL = StateLayout<SY, D>;
  using SM = StateSmem<D, SY::MP>;
  using SC = CausalSmem<SY, D>;
  Geom g = hd->g;
  hipStream_t s = a.stream;
  hla_token_table* cch = nullptr;
  HLA_TRY(get_table(hd, 2, kCausalChunk, s, &cch));
  if (static_cast<int64_t>(cch->count) * g.H > hd->max_chunks * hd->cfg.max_heads) return HLA_ERR_INVALID_ARG;
  unsigned char* pfx = static_cast<unsigned char*>(hd->path_ws) + hd->causal_off;
  // decay factor: log2 for the per-token weights, its power over a whole chunk for the scan
  const float dec = hd->cfg.decay > 0.0f && hd->cfg.decay < 1.0f ? hd->cfg.decay : 1.0f;
  const float l2d = dec < 1.0f ? std::log2(dec) : 0.0f;
  const float chunk_decay = dec < 1.0f ? std::pow(dec, static_cast<float>(kCausalChunk)) : 1.0f;
  HLA_TRY(launch(hd, "mfma_state", k_state<SY, D, 0, true>, dim3((cch->count + kWaves - 1) / kWaves, g.H),
                 dim3(kThreads), SM::kTotal, s, g, cch->dev, hd->feat, a.V, hd->partial, SL::kF32, l2d,
                 static_cast<const float*>(nullptr), static_cast<const float*>(nullptr), cch->count));
  static_assert(2 * (SY::MP / 16) * D % kScanThreads == 0, "whole workgroups of prefix items");
  using PL = PrefixLayout<SY, D>;
  const int za = kScanParts * 2 * (SY::MP / 16) * D / kScanThreads + 1;
  if (hd->causal_seen_backward) {
    // a handle in training use: the backward's image of the same running sum (rows = monomials)
    // comes out of the same launch, which spares the backward a scan of its own
    unsigned char* ops = static_cast<unsigned char*>(hd->path_ws) + hd->causal_bwd_off;
    const int zr = kScanPartsRows * (SY::MP / 32) * (D / 16) * 64 / kScanThreads;
    HLA_TRY(launch(hd, "mfma_state_prefix", k_prefix_both<SY, D, false>, dim3(a.num_seqs, g.H, za + zr),
                   dim3(kScanThreads), 0, s, g, cch->seq_off_dev, hd->partial, SL::kF32, pfx, make_canon_map<SY>(),
                   chunk_decay, static_cast<int64_t>(PL::kBytes), static_cast<int64_t>(PL::kOpElems * 2), ops,
                   static_cast<int64_t>(SL::kOpBytes), static_cast<int64_t>(SL::kOpElems * 2), za));
  } else {
    HLA_TRY(launch(hd, "mfma_state_prefix", k_prefix<SY, D, false>, dim3(a.num_seqs, g.H, za),
                   dim3(kScanThreads), 0, s, g, cch->seq_off_dev, hd->partial, SL::kF32, pfx, make_canon_map<SY>(), chunk_decay,
                   static_cast<int64_t>(PL::kBytes), static_cast<int64_t>(PL::kOpElems * 2)));
  }
  hd->causal_rows_valid = hd->causal_seen_backward;
  // one resident workgroup per compute unit, each walking its share of the (chunk, head) items
  const int64_t items = static_cast<int64_t>(cch->count) * g.H;
  HLA_TRY(launch(hd, "mfma_query_causal", k_query_causal<SY, D>, dim3(static_cast<unsigned>(items < kChunkTarget ? items : kChunkTarget)),
                 dim3(SC::kWavesQ * 64), SC::kTotal, s, g, cch->dev, hd->feat, a.V, pfx, a.O, hd->den, l2d,
                 static_cast<int>(cch->count)));
  hd->causal_partials_valid = true;  // the partial buffer holds this forward's chunk states
  return HLA_OK;
}

template <class SY, int D>
hla_status prepare_core() {
  HLA_TRY(allow_big_lds(&k_query_causal<SY, D>, CausalSmem<SY, D>::kTotal));
  HLA_TRY(allow_big_lds(&k_cgrad_q<SY, D>, CgSmem<SY, D>::kTotalQ));
  HLA_TRY(allow_big_lds(&k_cgrad_k<SY, D>, CgSmem<SY, D>::kTotalK));
  HLA_TRY(allow_big_lds(&k_state<SY, D, 0, true>, StateSmem<D, SY::MP>::kTotal));
  HLA_TRY(allow_big_lds(&k_state<SY, D, 1, true>, StateSmem<D, SY::MP>::kTotal));
  HLA_TRY(allow_big_lds(&k_state<SY, D>, StateSmem<D, SY::MP>::kTotal));
  return allow_big_lds(&k_bwd_query<SY, D>, BwdQSmem<D, SY::MP>::kTotal);
}

bool aligned16(const View& v) {
  return (reinterpret_cast<uintptr_t>(v.ptr) % 16 == 0) && v.sb % 8 == 0 && v.sh % 8 == 0 && v.sn % 8 == 0;
}

}  // namespace

using Sym36 = Sym<3, 6>;    // three factors of six features: 56 monomials in 64 rows
using Sym212 = Sym<2, 12>;  // two factors of twelve features: 78 monomials in 96 rows

// every canonical monomial is served by exactly one (lane half, slot) pair
template <class SY>
constexpr bool slots_cover_monomials() {
  int seen[SY::NM] = {};
  for (int g = 0; g < 2; ++g)
    for (int s = 0; s < SY::SP; ++s) {
      const int m = SY::slot_canon(g, s);
      if (m >= SY::NM) return false;
      if (m >= 0) ++seen[m];
    }
  for (int m = 0; m < SY::NM; ++m)
    if (seen[m] != 1) return false;
  return true;
}
static_assert(Sym36::NM == 56 && Sym36::MP == 64 && slots_cover_monomials<Sym36>(), "degree-3 slot table");
static_assert(Sym212::NM == 78 && Sym212::MP == 96 && slots_cover_monomials<Sym212>(), "degree-2 slot table");

bool mfma_supported(const hla_config& c) {
  const bool form = (c.degree == 3 && c.feature_dim == 6) || (c.degree == 2 && c.feature_dim == 12);
  return c.io_dtype == HLA_BF16 && form && (c.head_dim == 64 || c.head_dim == 128);
}

hla_status mfma_workspace_plan(hla_handle* hd) {
  const Geom& g = hd->g;
  const int64_t MP = g.F == 3 ? Sym36::MP : Sym212::MP, SP = MP / 2;
  hd->state_stride = MP * g.d + MP;
  // pick_chunk keeps chunks * H <= kChunkTarget + num_seqs * H (it only ever grows the chunk)
  hd->max_chunks = (kChunkTarget + hd->cfg.max_heads - 1) / hd->cfg.max_heads + hd->cfg.max_seqs + 1;
  hd->yhat_floats = 1;
  hd->tables[0].min_block = kMinChunk;
  hd->tables[1].min_block = kMinQueryBlock;
  if (hd->cfg.causal) {  // one partial state and one prefix image per chunk of kCausalChunk tokens
    hd->tables[2].min_block = kCausalChunk;
    const int64_t cc = (hd->cfg.max_tokens + kCausalChunk - 1) / kCausalChunk + hd->cfg.max_seqs;
    if (cc > hd->max_chunks) hd->max_chunks = cc;
  }
  // per unit: opA + opB (bf16) + zslot, for the state and for its gradient
  const int64_t op_bytes = 2 * MP * g.d * 2 + 2 * SP * 4;
  hd->path_ws_bytes = static_cast<size_t>(2 * op_bytes * hd->max_units);
  hd->w_packed_off = hd->path_ws_bytes;
  if (hd->cfg.phi_mode == HLA_PHI_MLP) hd->path_ws_bytes += mfma_phi_packed_bytes(hd);
  hd->causal_off = hd->path_ws_bytes;
  if (hd->cfg.causal) {
    hd->path_ws_bytes += static_cast<size_t>(hd->max_chunks * hd->cfg.max_heads * (MP * g.d * 2 + 2 * SP * 4));
    // backward: per chunk the images (opA, opB, z) of the state in front and of the gradient state behind
    hd->path_ws_bytes = (hd->path_ws_bytes + 255) / 256 * 256;
    hd->causal_bwd_off = hd->path_ws_bytes;
    hd->path_ws_bytes += static_cast<size_t>(2 * op_bytes * hd->max_chunks * hd->cfg.max_heads);
    hd->yhat_floats = hd->max_th;  // s_i of the query-side kernel
  }
  return HLA_OK;
}

hla_status mfma_prepare_kernels(const hla_handle* hd) {
  if (hd->g.F == 3)
    HLA_TRY(hd->g.d == 128 ? (prepare_core<Sym36, 128>()) : (prepare_core<Sym36, 64>()));
  else
    HLA_TRY(hd->g.d == 128 ? (prepare_core<Sym212, 128>()) : (prepare_core<Sym212, 64>()));
  return hd->cfg.phi_mode == HLA_PHI_MLP ? mfma_phi_prepare_kernels(hd) : HLA_OK;
}

hla_status mfma_set_weights(hla_handle* hd, hipStream_t s) { return mfma_phi_set_weights(hd, s); }

template <class SY>
static hla_status forward_sym(hla_handle* hd, const hla_call_args& a) {
  if (hd->cfg.causal) return hd->g.d == 128 ? forward_causal<SY, 128>(hd, a) : forward_causal<SY, 64>(hd, a);
  return hd->g.d == 128 ? forward_core<SY, 128>(hd, a) : forward_core<SY, 64>(hd, a);
}
template <class SY>
static hla_status backward_sym(hla_handle* hd, const hla_call_args& a) {
  if (hd->cfg.causal) return hd->g.d == 128 ? backward_causal<SY, 128>(hd, a) : backward_causal<SY, 64>(hd, a);
  return hd->g.d == 128 ? backward_core<SY, 128>(hd, a) : backward_core<SY, 64>(hd, a);
}

hla_status mfma_forward(hla_handle* hd, const hla_call_args& a) {
  if (!aligned16(a.V) || !aligned16(a.O)) return HLA_ERR_UNSUPPORTED;
  if (hd->cfg.phi_mode == HLA_PHI_MLP) {
    if (!aligned16(a.Q) || !aligned16(a.K)) return HLA_ERR_UNSUPPORTED;
    HLA_TRY(mfma_phi_forward(hd, a));
  } else {
    HLA_TRY(generic_features_in(hd, a));
  }
  return hd->g.F == 3 ? forward_sym<Sym36>(hd, a) : forward_sym<Sym212>(hd, a);
}

hla_status mfma_backward(hla_handle* hd, const hla_call_args& a) {
  if (!aligned16(a.V) || !aligned16(a.O) || !aligned16(a.dO) || !aligned16(a.dV))
    return HLA_ERR_UNSUPPORTED;
  HLA_TRY(hd->g.F == 3 ? backward_sym<Sym36>(hd, a) : backward_sym<Sym212>(hd, a));
  if (hd->cfg.phi_mode == HLA_PHI_MLP) {
    if (!aligned16(a.Q) || !aligned16(a.K) || !aligned16(a.dQ) || !aligned16(a.dK))
      return HLA_ERR_UNSUPPORTED;
    return mfma_phi_backward(hd, a);
  }
  return generic_features_out(hd, a);
}

}  // namespace hla
