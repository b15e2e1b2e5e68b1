// MFMA path: bf16 matrix-core kernels for gfx950 over the symmetric (monomial) form of the
// degree-3 feature tensor (see hla_mfma_common.h).  Forward core:
//   k_state   : per chunk of tokens,  Csym += S^T V,  zsym += S^T 1     (contraction over tokens)
//   k_reduce  : sums the chunk partials in fixed order and emits the state as MFMA operands
//   k_query   : O^T = Csym^T Qm^T, eta = Qm . zsym, O = num / (eta + eps)
// Lanes serve tokens: in every token-parallel kernel a token is the MFMA *column*, so per-token
// scalars (eta, den, s) live in one lane pair and never need a cross-lane broadcast.
#include "hla_handle.h"
#include "hla_mfma_common.h"

namespace hla {


namespace {

using namespace mf;

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kQueryBlock = 1024;  // tokens per workgroup in token-parallel kernels
constexpr int kReduceSlices = 8;

// Where canonical monomial m sits among the (g, slot) pairs.
struct SlotMap {
  int8_t g[64];
  int8_t s[64];
};

template <int DP>
SlotMap make_slot_map() {
  SlotMap sm{};
  for (int m = 0; m < 64; ++m) sm.g[m] = sm.s[m] = -1;
  for (int g = 0; g < 2; ++g)
    for (int s = 0; s < Sym3<DP>::NS; ++s) {
      const int m = sym3_slot_canon(DP, g, s);
      sm.g[m] = static_cast<int8_t>(g);
      sm.s[m] = static_cast<int8_t>(s);
    }
  return sm;
}

// Per-unit device state of the MFMA path (all inside hd->path_ws).
template <int DP, int D>
struct StateLayout {
  static constexpr int MP = Sym3<DP>::MP;
  static constexpr int SP = Sym3<DP>::SP;
  static constexpr int64_t kF32 = static_cast<int64_t>(MP) * D + MP;  // canonical C rows, then z
  static constexpr int64_t kOpElems = static_cast<int64_t>(MP) * D;   // bf16 elements per operand array
  // bytes per unit: opA, opB (bf16), zslot (fp32 [2][SP])
  static constexpr int64_t kOpBytes = 2 * kOpElems * 2 + 2 * SP * 4;
};

// ---- k_state ----------------------------------------------------------------------------------
template <int D>
struct StateSmem {
  static constexpr int kVStride = D * 2 + 32;   // bytes per token row of the V tile
  static constexpr int kSStride = 64 * 2 + 32;  // bytes per token row of the S tile (64 monomial cols)
  static constexpr int kVBytes = 64 * kVStride;
  static constexpr int kSBytes = 64 * kSStride;
  static constexpr int kWaveBytes = kVBytes + kSBytes;
  static constexpr int kRedBytes = (64 * D + 64) * 4;
  static constexpr int kTotal = kWaves * kWaveBytes > kRedBytes ? kWaves * kWaveBytes : kRedBytes;
};

// grid (chunks, H), block 256.  Each wave streams 64-token sub-tiles w, w+4, .. of the chunk
// through its private LDS region; the four waves' accumulators are summed in wave order at the
// end and written as one partial state.
template <int DP, int D>
__global__ __launch_bounds__(kThreads) void k_state(Geom g, const BlockEnt* __restrict__ chunks,
                                                    const float* __restrict__ feat, View V,
                                                    float* __restrict__ partial,
                                                    int64_t partial_stride) {
  using SY = Sym3<DP>;
  using SM = StateSmem<D>;
  static_assert(SY::MP == 64, "state kernel is laid out for a 64-row padded state");
  constexpr int NCB = D / 32;      // column blocks of the state
  constexpr int NVL = D * 2 / 16 * 64 / 64;  // 16-byte pieces per token row = D/8
  constexpr int PIECES = D / 8;    // 16-byte pieces per row
  constexpr int ROWS_PER_LD = 64 / PIECES;   // token rows covered by one wave-wide 16 B load
  constexpr int NLD = 64 / ROWS_PER_LD;      // loads per 64-token tile
  (void)NVL;
  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  unsigned char* vs = smem + wave * SM::kWaveBytes;
  unsigned char* ss = vs + SM::kVBytes;
  const BlockEnt e = chunks[blockIdx.x];
  const int h = blockIdx.y;
  const int r = lane % 32, gq = lane / 32;   // MFMA operand coordinates
  const int L = lane % 16, q = lane / 16;

  f32x16 acc[2][NCB];
  f32x16 zacc[2];
#pragma unroll
  for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[rb][cb][i] = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) zacc[rb][i] = 0.0f;
  }
  u32x4 ones;
  ones[0] = ones[1] = ones[2] = ones[3] = 0x3f803f80u;  // bf16 1.0 pairs

  const int prow = lane / PIECES, pcol = lane % PIECES;
  for (int n0 = e.t0 + wave * 64; n0 < e.t1; n0 += kWaves * 64) {
    // ---- V tile: coalesced 16-byte loads, rows beyond the chunk are zero
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int row = i * ROWS_PER_LD + prow;
      const int n = n0 + row;
      u32x4 v;
      v[0] = v[1] = v[2] = v[3] = 0u;
      if (n < e.t1) v = *reinterpret_cast<const u32x4*>(V.row<const bf16_t>(e.b, h, n) + pcol * 8);
      *reinterpret_cast<u32x4*>(vs + row * SM::kVStride + pcol * 16) = v;
    }
    // ---- key monomials of token n0 + lane (all NM, canonical order), as bf16 row of the S tile
    {
      float k1[DP], k2[DP], k3[DP];
      const int n = n0 + lane;
      if (n < e.t1) {
        const float* f = feat + g.th(e.b, h, n) * g.nfeat + DP;
#pragma unroll
        for (int a = 0; a < DP; ++a) {
          k1[a] = f[a];
          k2[a] = f[DP + a];
          k3[a] = f[2 * DP + a];
        }
      } else {
#pragma unroll
        for (int a = 0; a < DP; ++a) k1[a] = k2[a] = k3[a] = 0.0f;
      }
      float sm[SY::NM];
      key_monomials_all<DP>(k1, k2, k3, sm);
      uint32_t packed[32];
#pragma unroll
      for (int p = 0; p < 32; ++p) {
        const float lo = 2 * p < SY::NM ? sm[2 * p < SY::NM ? 2 * p : 0] : 0.0f;
        const float hi = 2 * p + 1 < SY::NM ? sm[2 * p + 1 < SY::NM ? 2 * p + 1 : 0] : 0.0f;
        packed[p] = pack_bf16(lo, hi);
      }
#pragma unroll
      for (int p = 0; p < 8; ++p) {
        u32x4 w;
        w[0] = packed[4 * p];
        w[1] = packed[4 * p + 1];
        w[2] = packed[4 * p + 2];
        w[3] = packed[4 * p + 3];
        *reinterpret_cast<u32x4*>(ss + lane * SM::kSStride + p * 16) = w;
      }
    }
    wave_lds_sync();
    // ---- Csym[64 x D] += S^T[64 x 64 tokens] V[64 tokens x D]; zsym += S^T 1
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int krow = 16 * ks + 8 * gq + L / 4;  // token row this lane addresses for the transpose read
      u32x4 a[2];
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
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
        for (int rb = 0; rb < 2; ++rb) acc[rb][cb] = mfma32(a[rb], b, acc[rb][cb]);
      }
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) zacc[rb] = mfma32(a[rb], ones, zacc[rb]);
    }
    wave_lds_sync();
  }
  // ---- sum the four waves in wave order through LDS, then write the partial state
  float* red = reinterpret_cast<float*>(smem);
  for (int w = 0; w < kWaves; ++w) {
    __syncthreads();
    if (wave == w) {
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int row = 32 * rb + d_row(i, gq);
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb) {
            float* p = red + row * D + 32 * cb + r;
            *p = (w == 0 ? 0.0f : *p) + acc[rb][cb][i];
          }
          if (r == 0) {
            float* p = red + 64 * D + row;
            *p = (w == 0 ? 0.0f : *p) + zacc[rb][i];
          }
        }
      }
    }
  }
  __syncthreads();
  float* out = partial + (static_cast<int64_t>(blockIdx.x) * g.H + h) * partial_stride;
  for (int i = threadIdx.x; i < 64 * D + 64; i += kThreads) out[i] = red[i];
}

// ---- k_reduce ---------------------------------------------------------------------------------
// grid (num_seqs, H, kReduceSlices), block 256.  Sums the chunk partials of one (sequence, head)
// in chunk order, writes the fp32 state and scatters its bf16 copy into the two operand layouts:
//   opA[rb][ks][lane=(r,gl)][j] = Csym[mono(gl, 8ks+j)][32rb + r]           (rows = channels)
//   opB[rb][ks][lane=(r,gl)][j] = Csym[mono of row 32rb + r][16ks + 8gl + j]  (rows = monomials)
// where state row rho = 32rb + r belongs to (g, s) with rho%32 = 8*(i/4) + 4g + i%4, s = 16rb + i.
template <int DP, int D>
__global__ void k_reduce(Geom g, const int32_t* __restrict__ seq_chunk_off,
                         const float* __restrict__ partial, int64_t partial_stride,
                         float* __restrict__ state, unsigned char* __restrict__ ops, SlotMap sm) {
  using SL = StateLayout<DP, D>;
  constexpr int MP = SL::MP, SP = SL::SP;
  constexpr int CW = D / kReduceSlices;  // channels per slice
  const int s = blockIdx.x, h = blockIdx.y, sl = blockIdx.z;
  const int c0 = seq_chunk_off[s], c1 = seq_chunk_off[s + 1];
  const int64_t u = static_cast<int64_t>(s) * g.H + h;
  float* st = state + u * SL::kF32;
  uint16_t* opA = reinterpret_cast<uint16_t*>(ops + u * SL::kOpBytes);
  uint16_t* opB = opA + SL::kOpElems;
  float* zslot = reinterpret_cast<float*>(opB + SL::kOpElems);
  for (int idx = threadIdx.x; idx < MP * CW; idx += blockDim.x) {
    const int m = idx / CW, c = sl * CW + idx % CW;
    float a = 0.0f;
    for (int ch = c0; ch < c1; ++ch)
      a += partial[(static_cast<int64_t>(ch) * g.H + h) * partial_stride + m * D + c];
    st[m * D + c] = a;
    const int mg = m < 64 ? sm.g[m] : -1;
    if (mg >= 0) {
      const int ms = sm.s[m];
      const uint16_t bits = f32_to_bf16_bits(a);
      {  // opA: channel c is the row, slot (mg, ms) the contraction index
        const int rb = c / 32, r = c % 32, ks = ms / 8, j = ms % 8;
        opA[((rb * (MP / 16) + ks) * 64 + 32 * mg + r) * 8 + j] = bits;
      }
      {  // opB: monomial row from (mg, ms), channel c the contraction index
        const int rb = ms / 16, i = ms % 16;
        const int r = 8 * (i / 4) + 4 * mg + i % 4;
        const int ks = c / 16, gl = (c % 16) / 8, j = c % 8;
        opB[((rb * (D / 16) + ks) * 64 + 32 * gl + r) * 8 + j] = bits;
      }
    }
  }
  if (sl == 0) {
    for (int m = threadIdx.x; m < MP; m += blockDim.x) {
      float a = 0.0f;
      for (int ch = c0; ch < c1; ++ch)
        a += partial[(static_cast<int64_t>(ch) * g.H + h) * partial_stride + MP * D + m];
      st[MP * D + m] = a;
      const int mg = m < 64 ? sm.g[m] : -1;
      if (mg >= 0) zslot[mg * SP + sm.s[m]] = a;
    }
  }
}

// ---- k_query ----------------------------------------------------------------------------------
// grid (blocks of kQueryBlock tokens, H), block 256.  Wave w serves 32-token tiles w, w+4, ..;
// lane (r, gl): token r of the tile, slot half gl (gl = 1 works on the reversed feature vector).
template <int DP, int D>
__global__ __launch_bounds__(kThreads) void k_query(Geom g, const BlockEnt* __restrict__ blocks,
                                                    const float* __restrict__ feat,
                                                    const unsigned char* __restrict__ ops, View O,
                                                    float* __restrict__ den) {
  using SY = Sym3<DP>;
  using SL = StateLayout<DP, D>;
  constexpr int SP = SY::SP, MP = SY::MP;
  constexpr int NRB = D / 32, NKS = MP / 16;
  const int lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
  const int r = lane % 32, gl = lane / 32;
  const BlockEnt e = blocks[blockIdx.x];
  const int h = blockIdx.y;
  const int64_t u = static_cast<int64_t>(e.seq) * g.H + h;
  const u32x4* opA = reinterpret_cast<const u32x4*>(ops + u * SL::kOpBytes);
  const float* zslot = reinterpret_cast<const float*>(ops + u * SL::kOpBytes + 2 * SL::kOpElems * 2) + gl * SP;
  u32x4 a[NRB][NKS];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) a[rb][ks] = opA[(rb * NKS + ks) * 64 + lane];
  float z[SP];
#pragma unroll
  for (int s = 0; s < SP; ++s) z[s] = zslot[s];

  for (int n0 = e.t0 + wave * 32; n0 < e.t1; n0 += kWaves * 32) {
    const int n = n0 + r;
    const bool live = n < e.t1;
    float qf[DP];
    if (live) {
      const float* f = feat + g.th(e.b, h, n) * g.nfeat;
#pragma unroll
      for (int c = 0; c < DP; ++c) qf[c] = f[gl ? DP - 1 - c : c];
    } else {
#pragma unroll
      for (int c = 0; c < DP; ++c) qf[c] = 0.0f;
    }
    float qm[SP];
    query_monomials<DP>(qf, qm);
    u32x4 b[NKS];
    float eta = 0.0f;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const int s = 8 * ks + 2 * p;
        const uint32_t pk = pack_bf16(qm[s], qm[s + 1]);
        b[ks][p] = pk;
        eta += bf16_lo(pk) * z[s] + bf16_hi(pk) * z[s + 1];  // the same rounded values the MFMA sees
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
      for (int ks = 0; ks < NKS; ++ks) acc[rb] = mfma32(a[rb][ks], b[ks], acc[rb]);
    }
    if (live) {
      bf16_t* orow = O.row<bf16_t>(e.b, h, n);
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(acc[rb][4 * q4] * inv, acc[rb][4 * q4 + 1] * inv);
          w[1] = pack_bf16(acc[rb][4 * q4 + 2] * inv, acc[rb][4 * q4 + 3] * inv);
          *reinterpret_cast<u32x2*>(orow + 32 * rb + 8 * q4 + 4 * gl) = w;
        }
    }
  }
}

template <int DP, int D>
hla_status forward_core(hla_handle* hd, const hla_call_args& a) {
  using SL = StateLayout<DP, D>;
  using SM = StateSmem<D>;
  Geom g = hd->g;
  hipStream_t s = a.stream;
  // chunk size: smallest power of two >= 256 that keeps the grid at or under ~3 workgroups per CU
  int chunk = 256;
  const int64_t tokens = static_cast<int64_t>(g.B) * g.N;
  while ((tokens / chunk + a.num_seqs) * g.H > 768 && chunk < (1 << 20)) chunk *= 2;
  hla_token_table *chunks = nullptr, *qblocks = nullptr;
  HLA_TRY(get_table(hd, chunk, s, &chunks));
  HLA_TRY(get_table(hd, kQueryBlock, s, &qblocks));
  if (static_cast<int64_t>(chunks->count) * g.H > hd->max_chunks * hd->cfg.max_heads)
    return HLA_ERR_INVALID_ARG;
  static bool attr_set = false;
  if (!attr_set) {
    HLA_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_state<DP, D>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, SM::kTotal));
    attr_set = true;
  }
  HLA_TRY(launch(hd, "mfma_state", k_state<DP, D>, dim3(chunks->count, g.H), dim3(kThreads),
                 SM::kTotal, s, g, chunks->dev, hd->feat, a.V, hd->partial, SL::kF32));
  const SlotMap sm = make_slot_map<DP>();
  unsigned char* ops = static_cast<unsigned char*>(hd->path_ws);
  HLA_TRY(launch(hd, "mfma_state_reduce", k_reduce<DP, D>, dim3(a.num_seqs, g.H, kReduceSlices),
                 dim3(256), 0, s, g, chunks->seq_off_dev, hd->partial, SL::kF32, hd->state, ops, sm));
  HLA_TRY(launch(hd, "mfma_query", k_query<DP, D>, dim3(qblocks->count, g.H), dim3(kThreads), 0, s,
                 g, qblocks->dev, hd->feat, ops, a.O, hd->den));
  return HLA_OK;
}

bool aligned16(const View& v) {
  return (reinterpret_cast<uintptr_t>(v.ptr) % 16 == 0) && v.sb % 8 == 0 && v.sh % 8 == 0 && v.sn % 8 == 0;
}

}  // namespace

bool mfma_supported(const hla_config& c) {
  return c.io_dtype == HLA_BF16 && c.degree == 3 && c.feature_dim == 6 &&
         (c.head_dim == 64 || c.head_dim == 128);
}

hla_status mfma_workspace_plan(hla_handle* hd) {
  const Geom& g = hd->g;
  const int64_t MP = 64, SP = 32;
  hd->state_stride = MP * g.d + MP;
  // forward_core keeps chunks * H <= 768 unless the sequences alone exceed that
  hd->max_chunks = (768 + hd->cfg.max_heads - 1) / hd->cfg.max_heads + hd->cfg.max_seqs +
                   hd->cfg.max_tokens / (1 << 20) + 2;
  hd->yhat_floats = 1;
  // per unit: opA + opB (bf16) + zslot, for the state and for its gradient
  const int64_t op_bytes = 2 * MP * g.d * 2 + 2 * SP * 4;
  hd->path_ws_bytes = static_cast<size_t>(2 * op_bytes * hd->max_units);
  for (int sz = 256; sz <= (1 << 20); sz *= 2) hd->tables[sz];
  hd->tables[kQueryBlock];
  return HLA_OK;
}

hla_status mfma_set_weights(hla_handle*, hipStream_t) { return HLA_OK; }

hla_status mfma_forward(hla_handle* hd, const hla_call_args& a) {
  if (!aligned16(a.V) || !aligned16(a.O)) return HLA_ERR_UNSUPPORTED;
  HLA_TRY(generic_features_in(hd, a));
  if (hd->g.d == 128) return forward_core<6, 128>(hd, a);
  return forward_core<6, 64>(hd, a);
}

hla_status mfma_backward(hla_handle*, const hla_call_args&) { return HLA_ERR_UNSUPPORTED; }

}  // namespace hla
