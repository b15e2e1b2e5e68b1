// Device helpers for the matrix-core (MFMA) path on gfx950: operand types, MFMA wrappers with
// their lane layouts, LDS transpose reads, wave-level LDS ordering, and the compile-time tables
// of the symmetric (monomial) form of the degree-3 feature tensor.
#ifndef HLA_MFMA_COMMON_H_
#define HLA_MFMA_COMMON_H_

#include <type_traits>
#include <utility>

#include "hla_common.h"

namespace hla {
namespace mf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));  // one pair of features in the tiled workspace
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

// ---- v_mfma_f32_32x32x16_bf16 ---------------------------------------------------------------
// D[32x32] += A[32x16] * B[16x32].  Lane l = (r, g) with r = l % 32, g = l / 32:
//   A operand: row r,   k = 8g .. 8g+7      (8 bf16 = 4 VGPRs)
//   B operand: col r,   k = 8g .. 8g+7
//   D: column r; register i (0..15) holds row 8*(i/4) + 4*g + (i%4).
// The contraction only needs A and B to agree on what k-slot (g, j) means, so kernels are free
// to map k-slots to tokens / channels / monomials in whatever order suits their loads.
__device__ __forceinline__ f32x16 mfma32(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ int d_row(int i, int g) { return 8 * (i / 4) + 4 * g + (i % 4); }
// v_mfma_f32_32x32x16_f16: the same lane layout with fp16 operands
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ f32x16 mfma32_f16(u32x4 a, u32x4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a),
                                                __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// two fp32 -> packed bf16 pair (lo = a, hi = b), round-to-nearest-even
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 v;
  v[0] = static_cast<__bf16>(a);
  v[1] = static_cast<__bf16>(b);
  return __builtin_bit_cast(uint32_t, v);
}
__device__ __forceinline__ float bf16_lo(uint32_t p) { return __uint_as_float(p << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t p) { return __uint_as_float(p & 0xffff0000u); }

// ---- ds_read_b64_tr_b16 ---------------------------------------------------------------------
// Within each group of 16 lanes the 16 x (4 bf16) values are treated as a 4 x 16 matrix whose row
// j is supplied by lanes 4j..4j+3 (4 elements each); lane n of the group receives column n.
// With a row-major [k][n] tile in LDS, lane L passing the address of (row k0 + L/4, cols
// n0 + 4*(L%4) .. +3) receives (k0..k0+3, n0 + L): four consecutive k for one n, which is half of
// an MFMA operand whose contraction index runs along the tile's rows.
__device__ __forceinline__ u32x2 lds_read_tr16(const void* lds_ptr) {
  typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds_ptr));
  return __builtin_bit_cast(u32x2, v);
}

// The wave's index in its workgroup as a scalar: what is derived from it (tile numbers, their
// decoding into batch row / head / token with integer divisions, LDS region bases) then runs on
// the scalar unit instead of costing vector-ALU slots in every lane.
__device__ __forceinline__ int wave_index() {
  return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x) / kWave);
}

// Orders this wave's earlier LDS writes before its later LDS reads by other lanes of the same
// wave (no s_barrier: waves of a workgroup run independent pipelines over private LDS regions).
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ---- swizzled LDS tiles --------------------------------------------------------------------------
// A [rows][ROWB bytes] tile (ROWB = 256 or 128) whose 16-byte chunks are XOR-swizzled by a function
// of the row, so that both access patterns the kernels use are bank-conflict free without padding:
// 16-byte accesses of 16 consecutive rows at one chunk, and transpose reads of 4 consecutive rows
// (starting at a multiple of 4) x 4 consecutive chunks (starting at a multiple of 4).
template <int ROWB>
__host__ __device__ __forceinline__ int tile_swz(int row) {
  return ROWB == 256 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}
template <int ROWB>
__host__ __device__ __forceinline__ int tile_off(int row, int chunk) {
  return row * ROWB + (((chunk ^ tile_swz<ROWB>(row)) & (ROWB / 16 - 1)) << 4);
}

// All waves of a streaming kernel run the same schedule; started together they reach their LDS,
// vector-memory and matrix phases at the same moment and queue on the units a compute unit
// shares.  A start-up delay that differs per wave (and per workgroup) spreads the phases out.
// `unit` is in steps of 64 * 8 cycles.
__device__ __forceinline__ void stagger_start(int wave, int block, int unit) {
  const int n = wave * unit + (block & 3);
  for (int i = 0; i < n; ++i) __builtin_amdgcn_s_sleep(8);
}

// value held by the lane 32 away (the other half of a (token, g) lane pair)
__device__ __forceinline__ float partner32(float v) { return __shfl_xor(v, 32, 64); }

// Stage a [32 tokens x D] bf16 tile row-major into LDS with coalesced 16-byte loads; rows at or
// beyond t1 are zero.  Row stride `stride` bytes.
template <int D>
__device__ __forceinline__ void stage_tile32(const View& X, int b, int h, int n0, int t1, int lane,
                                             unsigned char* dst, int stride) {
  constexpr int PIECES = D / 8;
  constexpr int RPL = 64 / PIECES;
  constexpr int NLD = 32 / RPL;
  const int prow = lane / PIECES, pcol = lane % PIECES;
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int row = i * RPL + prow;
    const int n = n0 + row;
    u32x4 v;
    v[0] = v[1] = v[2] = v[3] = 0u;
    if (n < t1) v = *reinterpret_cast<const u32x4*>(X.row<const bf16_t>(b, h, n) + pcol * 8);
    *reinterpret_cast<u32x4*>(dst + row * stride + pcol * 16) = v;
  }
}

// The same staging split in two so that the global loads of the NEXT tile can be in flight while
// the current tile is being consumed: fetch_tile issues the loads into registers, put_tile writes
// them to LDS.  ROWS = tokens per tile (32 or 64).
template <int D, int ROWS>
struct TileRegs {
  static constexpr int PIECES = D / 8;        // 16-byte pieces per token row
  static constexpr int RPL = 64 / PIECES;     // rows covered by one wave-wide load
  static constexpr int NLD = ROWS / RPL;      // loads per tile
  u32x4 v[NLD];
};
template <int D, int ROWS>
__device__ __forceinline__ void fetch_tile(const View& X, int b, int h, int n0, int t1, int lane,
                                           TileRegs<D, ROWS>& t) {
  using T = TileRegs<D, ROWS>;
  const int prow = lane / T::PIECES, pcol = lane % T::PIECES;
#pragma unroll
  for (int i = 0; i < T::NLD; ++i) {
    const int n = n0 + i * T::RPL + prow;
    t.v[i][0] = t.v[i][1] = t.v[i][2] = t.v[i][3] = 0u;
    if (n < t1) t.v[i] = *reinterpret_cast<const u32x4*>(X.row<const bf16_t>(b, h, n) + pcol * 8);
  }
}
template <int D, int ROWS>
__device__ __forceinline__ void put_tile(const TileRegs<D, ROWS>& t, int lane, unsigned char* dst,
                                         int stride) {
  using T = TileRegs<D, ROWS>;
  const int prow = lane / T::PIECES, pcol = lane % T::PIECES;
#pragma unroll
  for (int i = 0; i < T::NLD; ++i)
    *reinterpret_cast<u32x4*>(dst + (i * T::RPL + prow) * stride + pcol * 16) = t.v[i];
}

// ---- coalesced row stores of a token-per-lane accumulator tile ---------------------------------
// acc[rb][i] holds channel 32rb + d_row(i, gl) of token r (lane (r, gl)).  The tile is rounded to
// bf16, exchanged between the two lanes of a token (v_permlane32_swap) so that each lane owns two
// runs of 8 consecutive channels per row block, written to a wave-private LDS tile and read back
// with 16 consecutive lanes covering one token row, so that every global store instruction
// writes whole 2D-byte rows.  `row_ptr(t)` returns the destination of tile row t or nullptr.
template <int D, int ROWS = 32>
struct RowTile {
  static constexpr int kStride = D * 2 + 16;   // bytes; 16-byte reads and writes stay conflict-free
  static constexpr int kBytes = ROWS * kStride;
};
// ROWS (32 or 16) = token rows the LDS tile holds; with 16 the tile goes out in two passes.
// pack_rows rounds and exchanges, put_rows writes one pass into the LDS tile, flush_rows stores
// that pass to global memory.  Kernels that stream tiles split the two: a tile is staged at the
// end of its iteration and flushed at the top of the next one, right after the wait for that
// iteration's inputs.  Stores count in the same wait counter as loads, so a store issued just
// before such a wait would cost its whole round trip.
template <int D>
__device__ __forceinline__ void pack_rows(const f32x16 (&acc)[D / 32], float scale,
                                          u32x4 (&w)[D / 32][2]) {
#pragma unroll
  for (int rb = 0; rb < D / 32; ++rb)
#pragma unroll
    for (int pr = 0; pr < 2; ++pr) {
      const int x = 8 * pr, y = 8 * pr + 4;  // accumulator registers of the two 4-channel groups
      const uint32_t x0 = pack_bf16(acc[rb][x] * scale, acc[rb][x + 1] * scale);
      const uint32_t x1 = pack_bf16(acc[rb][x + 2] * scale, acc[rb][x + 3] * scale);
      const uint32_t y0 = pack_bf16(acc[rb][y] * scale, acc[rb][y + 1] * scale);
      const uint32_t y1 = pack_bf16(acc[rb][y + 2] * scale, acc[rb][y + 3] * scale);
      // upper lanes of x swap with lower lanes of y: lane gl = 0 ends with channels +0..7 of the
      // 16-channel group, lane gl = 1 with channels +8..15
      const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
      const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
      w[rb][pr][0] = s0[0];
      w[rb][pr][1] = s1[0];
      w[rb][pr][2] = s0[1];
      w[rb][pr][3] = s1[1];
    }
}
template <int D, int ROWS>
__device__ __forceinline__ void put_rows(const u32x4 (&w)[D / 32][2], int pass, int lane,
                                         unsigned char* lds) {
  using RT = RowTile<D, ROWS>;
  const int r = lane % 32, gl = lane / 32;
  if (ROWS == 32 || r / ROWS == pass) {
#pragma unroll
    for (int rb = 0; rb < D / 32; ++rb)
#pragma unroll
      for (int pr = 0; pr < 2; ++pr)
        *reinterpret_cast<u32x4*>(lds + (r % ROWS) * RT::kStride + (32 * rb + 16 * pr + 8 * gl) * 2) = w[rb][pr];
  }
  wave_lds_sync();
}
// row_ptr(t) returns the destination of tile row t (0..31) or nullptr
template <int D, int ROWS, class RowPtr>
__device__ __forceinline__ void flush_rows(int pass, int lane, const unsigned char* lds, RowPtr&& row_ptr) {
  using RT = RowTile<D, ROWS>;
  constexpr int PIECES = D / 8;        // 16-byte pieces per row
  constexpr int RPI = 64 / PIECES;     // rows per store instruction
#pragma unroll
  for (int i = 0; i < ROWS / RPI; ++i) {
    const int row = i * RPI + lane / PIECES, piece = lane % PIECES;
    const u32x4 v = *reinterpret_cast<const u32x4*>(lds + row * RT::kStride + piece * 16);
    bf16_t* dst = row_ptr(pass * ROWS + row);
    // nontemporal: the outputs are not read again by the library; stored plainly they push the
    // inputs of the following kernels out of the caches
    if (dst != nullptr) __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(dst + piece * 8));
  }
  wave_lds_sync();
}
template <int D, int ROWS = 32, class RowPtr>
__device__ __forceinline__ void store_rows_bf16(const f32x16 (&acc)[D / 32], float scale, int lane,
                                                unsigned char* lds, RowPtr&& row_ptr) {
  u32x4 w[D / 32][2];
  pack_rows<D>(acc, scale, w);
#pragma unroll
  for (int pass = 0; pass < 32 / ROWS; ++pass) {
    put_rows<D, ROWS>(w, pass, lane, lds);
    flush_rows<D, ROWS>(pass, lane, lds, row_ptr);
  }
}

template <int I, int N, class Fn>
__device__ __forceinline__ void static_for(Fn&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// ---- symmetric form of the degree-3 feature tensor -------------------------------------------
// T_q = q (x) q (x) q is symmetric, so contracting it with the state only sees the state summed
// over index permutations.  Both sides are therefore kept over the C(dphi+2, 3) monomials
// {x <= y <= z}:   query feature  Qm[m] = q_x q_y q_z,
//                  key feature    S[m]  = sum over distinct orderings (a,b,c) of (x,y,z) of
//                                         k1_a k2_b k3_c,
// and  sum_D T_q[D] C[D,:] = sum_m Qm[m] Csym[m,:]  with  Csym = sum_j S_j (x) v_j  exactly.
//
// Index reversal a -> dphi-1-a maps monomials to monomials without fixed points when dphi is
// even, so they split into NS = NM/2 mirror pairs.  A token is served by two lanes (g = 0, 1):
// lane g = 0 evaluates the pair's first member from the features as they are, lane g = 1 runs
// the SAME instructions on the reversed feature vector and thereby evaluates the mirror member.
// "Slot" s (0..NS-1, padded to SP) names a pair; (g, s) names a monomial.
struct Tri {
  int x, y, z;
};
constexpr int sym3_num_mono(int dp) { return dp * (dp + 1) * (dp + 2) / 6; }
constexpr Tri sym3_mono(int dp, int m) {
  int c = 0;
  for (int x = 0; x < dp; ++x)
    for (int y = x; y < dp; ++y)
      for (int z = y; z < dp; ++z) {
        if (c == m) return Tri{x, y, z};
        ++c;
      }
  return Tri{-1, -1, -1};
}
constexpr int sym3_canon(int dp, Tri t) {
  int c = 0;
  for (int x = 0; x < dp; ++x)
    for (int y = x; y < dp; ++y)
      for (int z = y; z < dp; ++z) {
        if (x == t.x && y == t.y && z == t.z) return c;
        ++c;
      }
  return -1;
}
constexpr Tri sym3_mirror(int dp, Tri t) { return Tri{dp - 1 - t.z, dp - 1 - t.y, dp - 1 - t.x}; }
// s-th monomial (in canonical order) that precedes its own mirror image
constexpr Tri sym3_slot(int dp, int s) {
  int c = 0;
  for (int m = 0; m < sym3_num_mono(dp); ++m) {
    const Tri t = sym3_mono(dp, m);
    if (m < sym3_canon(dp, sym3_mirror(dp, t))) {
      if (c == s) return t;
      ++c;
    }
  }
  return Tri{-1, -1, -1};
}
// canonical monomial index served by (g, s); -1 for padding slots
constexpr int sym3_slot_canon(int dp, int g, int s) {
  if (s >= sym3_num_mono(dp) / 2) return -1;
  const Tri t = sym3_slot(dp, s);
  return g == 0 ? sym3_canon(dp, t) : sym3_canon(dp, sym3_mirror(dp, t));
}

template <int DP>
struct Sym3 {
  static_assert(DP % 2 == 0, "mirror pairing needs an even feature dim");
  static constexpr int NM = sym3_num_mono(DP);   // monomials
  static constexpr int NS = NM / 2;              // mirror pairs (slots actually used)
  static constexpr int SP = (NS + 15) / 16 * 16; // slots per lane half, padded
  static constexpr int MP = 2 * SP;              // rows of the padded symmetric state
};

// Query monomials of this lane's slots from its (possibly reversed) features.
template <int DP>
__device__ __forceinline__ void query_monomials(const float (&q)[DP], float (&qm)[Sym3<DP>::SP]) {
  static_for<0, Sym3<DP>::SP>([&](auto S) {
    constexpr int s = decltype(S)::value;
    if constexpr (s < Sym3<DP>::NS) {
      constexpr Tri t = sym3_slot(DP, s);
      qm[s] = (q[t.x] * q[t.y]) * q[t.z];
    } else {
      qm[s] = 0.0f;
    }
  });
}

// dq[a] += sum_s dm[s] * d(q_x q_y q_z)/dq_a  (one term per position, which also covers
// repeated indices).
template <int DP>
__device__ __forceinline__ void query_monomials_grad(const float (&q)[DP],
                                                     const float (&dm)[Sym3<DP>::SP],
                                                     float (&dq)[DP]) {
  static_for<0, Sym3<DP>::NS>([&](auto S) {
    constexpr int s = decltype(S)::value;
    constexpr Tri t = sym3_slot(DP, s);
    dq[t.x] += dm[s] * (q[t.y] * q[t.z]);
    dq[t.y] += dm[s] * (q[t.x] * q[t.z]);
    dq[t.z] += dm[s] * (q[t.x] * q[t.y]);
  });
}

// Distinct orderings of a monomial, enumerated at compile time.
struct Perm3 {
  int n;
  int a[6], b[6], c[6];
};
constexpr Perm3 sym3_perms(Tri t) {
  Perm3 p{0, {0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0}, {0, 0, 0, 0, 0, 0}};
  const int v[3] = {t.x, t.y, t.z};
  const int idx[6][3] = {{0, 1, 2}, {0, 2, 1}, {1, 0, 2}, {1, 2, 0}, {2, 0, 1}, {2, 1, 0}};
  for (int k = 0; k < 6; ++k) {
    const int a = v[idx[k][0]], b = v[idx[k][1]], c = v[idx[k][2]];
    bool dup = false;
    for (int e = 0; e < p.n; ++e) dup = dup || (p.a[e] == a && p.b[e] == b && p.c[e] == c);
    if (!dup) {
      p.a[p.n] = a;
      p.b[p.n] = b;
      p.c[p.n] = c;
      ++p.n;
    }
  }
  return p;
}

// Key monomial feature of one monomial: S = sum over distinct orderings of k1_a k2_b k3_c.
template <int DP, int X, int Y, int Z>
__device__ __forceinline__ float key_monomial(const float (&k1)[DP], const float (&k2)[DP],
                                              const float (&k3)[DP]) {
  constexpr Perm3 p = sym3_perms(Tri{X, Y, Z});
  float acc = 0.0f;
  static_for<0, p.n>([&](auto E) {
    constexpr int e = decltype(E)::value;
    acc += k1[p.a[e]] * (k2[p.b[e]] * k3[p.c[e]]);
  });
  return acc;
}

// All NM key monomials in canonical order (one lane serves one token).
template <int DP>
__device__ __forceinline__ void key_monomials_all(const float (&k1)[DP], const float (&k2)[DP],
                                                  const float (&k3)[DP],
                                                  float (&sm)[Sym3<DP>::NM]) {
  static_for<0, Sym3<DP>::NM>([&](auto M) {
    constexpr int m = decltype(M)::value;
    constexpr Tri t = sym3_mono(DP, m);
    sm[m] = key_monomial<DP, t.x, t.y, t.z>(k1, k2, k3);
  });
}

// Key monomials of this lane's slots (features possibly reversed).
template <int DP>
__device__ __forceinline__ void key_monomials_slots(const float (&k1)[DP], const float (&k2)[DP],
                                                    const float (&k3)[DP],
                                                    float (&sm)[Sym3<DP>::SP]) {
  static_for<0, Sym3<DP>::SP>([&](auto S) {
    constexpr int s = decltype(S)::value;
    if constexpr (s < Sym3<DP>::NS) {
      constexpr Tri t = sym3_slot(DP, s);
      sm[s] = key_monomial<DP, t.x, t.y, t.z>(k1, k2, k3);
    } else {
      sm[s] = 0.0f;
    }
  });
}

// Chain rule of key_monomials_slots: every distinct ordering (a,b,c) of slot s feeds
// dk1[a] += ds * k2_b k3_c, dk2[b] += ds * k1_a k3_c, dk3[c] += ds * k1_a k2_b.
// Evaluated through U[a][b] = sum over the orderings of ds * k3_c, which serves two of the three:
//   dk1[a] = sum_b U[a][b] k2_b,   dk2[b] = sum_a U[a][b] k1_a,   dk3[c] += ds * (k1_a k2_b),
// two multiply-adds per ordering plus 2 DP^2 at the end instead of three and three products.
// Slots S0 .. S1-1 per call, so that callers can interleave other work between ranges; U is
// cleared by the caller before the first range and folded in by key_monomials_grad_finish after
// the last.
constexpr bool sym3_pair_used(int dp, int a, int b) {  // does any slot have an ordering (a, b, .)?
  for (int s = 0; s < sym3_num_mono(dp) / 2; ++s) {
    const Perm3 p = sym3_perms(sym3_slot(dp, s));
    for (int e = 0; e < p.n; ++e)
      if (p.a[e] == a && p.b[e] == b) return true;
  }
  return false;
}
template <int DP, int S0, int S1>
__device__ __forceinline__ void key_monomials_grad_range(const float (&k1)[DP], const float (&k2)[DP],
                                                         const float (&k3)[DP],
                                                         const float (&ds)[Sym3<DP>::SP],
                                                         float (&U)[DP][DP], float (&dk3)[DP]) {
  static_for<S0, (S1 < Sym3<DP>::NS ? S1 : Sym3<DP>::NS)>([&](auto S) {
    constexpr int s = decltype(S)::value;
    constexpr Tri t = sym3_slot(DP, s);
    constexpr Perm3 p = sym3_perms(t);
    static_for<0, p.n>([&](auto E) {
      constexpr int e = decltype(E)::value;
      U[p.a[e]][p.b[e]] += ds[s] * k3[p.c[e]];
      dk3[p.c[e]] += ds[s] * (k1[p.a[e]] * k2[p.b[e]]);
    });
  });
}
template <int DP>
__device__ __forceinline__ void key_monomials_grad_finish(const float (&k1)[DP], const float (&k2)[DP],
                                                          const float (&U)[DP][DP], float (&dk1)[DP],
                                                          float (&dk2)[DP]) {
  static_for<0, DP * DP>([&](auto AB) {
    constexpr int a = decltype(AB)::value / DP, b = decltype(AB)::value % DP;
    if constexpr (sym3_pair_used(DP, a, b)) {
      dk1[a] += U[a][b] * k2[b];
      dk2[b] += U[a][b] * k1[a];
    }
  });
}
template <int DP>
__device__ __forceinline__ void key_monomials_grad(const float (&k1)[DP], const float (&k2)[DP],
                                                   const float (&k3)[DP],
                                                   const float (&ds)[Sym3<DP>::SP],
                                                   float (&dk1)[DP], float (&dk2)[DP],
                                                   float (&dk3)[DP]) {
  float U[DP][DP];
#pragma unroll
  for (int a = 0; a < DP; ++a)
#pragma unroll
    for (int b = 0; b < DP; ++b) U[a][b] = 0.0f;
  key_monomials_grad_range<DP, 0, Sym3<DP>::NS>(k1, k2, k3, ds, U, dk3);
  key_monomials_grad_finish<DP>(k1, k2, U, dk1, dk2);
}


// ---- symmetric form of the degree-2 feature tensor -------------------------------------------
// The same construction for T_q = q (x) q: monomials {x <= y}, query feature q_x q_y, key feature
// k1_x k2_y + k1_y k2_x (one term when x == y).  Index reversal maps (x, y) to
// (dphi-1-y, dphi-1-x) and fixes the dphi/2 monomials with x + y = dphi - 1, so the slots are the
// NPAIR mirror pairs followed by the NFIX self-mirrored monomials.  Lane g = 0 serves a
// self-mirrored monomial; on lane g = 1 the same instructions would produce it a second time, so
// that lane multiplies those slots (values and gradients) by zero: (1, s) is padding there.
struct Duo {
  int x, y;
};
constexpr int sym2_num_mono(int dp) { return dp * (dp + 1) / 2; }
constexpr Duo sym2_mono(int dp, int m) {
  int c = 0;
  for (int x = 0; x < dp; ++x)
    for (int y = x; y < dp; ++y) {
      if (c == m) return Duo{x, y};
      ++c;
    }
  return Duo{-1, -1};
}
constexpr int sym2_canon(int dp, Duo t) {
  int c = 0;
  for (int x = 0; x < dp; ++x)
    for (int y = x; y < dp; ++y) {
      if (x == t.x && y == t.y) return c;
      ++c;
    }
  return -1;
}
constexpr Duo sym2_mirror(int dp, Duo t) { return Duo{dp - 1 - t.y, dp - 1 - t.x}; }
constexpr int sym2_num_pairs(int dp) { return (sym2_num_mono(dp) - dp / 2) / 2; }
// slot s: first the monomials that precede their mirror image, then the self-mirrored ones
constexpr Duo sym2_slot(int dp, int s) {
  int c = 0;
  for (int pass = 0; pass < 2; ++pass)
    for (int m = 0; m < sym2_num_mono(dp); ++m) {
      const Duo t = sym2_mono(dp, m);
      const int mm = sym2_canon(dp, sym2_mirror(dp, t));
      if (pass == 0 ? m < mm : m == mm) {
        if (c == s) return t;
        ++c;
      }
    }
  return Duo{-1, -1};
}
constexpr int sym2_slot_canon(int dp, int g, int s) {
  const int np = sym2_num_pairs(dp);
  if (s >= np + dp / 2) return -1;
  const Duo t = sym2_slot(dp, s);
  if (s >= np) return g == 0 ? sym2_canon(dp, t) : -1;
  return g == 0 ? sym2_canon(dp, t) : sym2_canon(dp, sym2_mirror(dp, t));
}

// Degree-generic view of the symmetric form: F = 3 is Sym3 above.
template <int F_, int DP>
struct Sym;
template <int DP>
struct Sym<3, DP> : Sym3<DP> {
  static constexpr int F = 3;
  static constexpr int DPHI = DP;
  static constexpr int slot_canon(int g, int s) { return sym3_slot_canon(DP, g, s); }
};
template <int DP>
struct Sym<2, DP> {
  static_assert(DP % 2 == 0, "mirror pairing needs an even feature dim");
  static constexpr int F = 2;
  static constexpr int DPHI = DP;
  static constexpr int NM = sym2_num_mono(DP);
  static constexpr int NPAIR = sym2_num_pairs(DP);
  static constexpr int NFIX = DP / 2;
  static constexpr int NS = NPAIR + NFIX;
  static constexpr int SP = (NS + 15) / 16 * 16;
  static constexpr int MP = 2 * SP;
  static constexpr int slot_canon(int g, int s) { return sym2_slot_canon(DP, g, s); }
};

// The monomial helpers below take the features of a token as f[map][DP] (already reversed on the
// lanes of half gl = 1) and dispatch on the degree.
template <class SY>
__device__ __forceinline__ void sym_query_monomials(const float (&q)[SY::DPHI], float (&qm)[SY::SP],
                                                    int gl) {
  constexpr int DP = SY::DPHI;
  if constexpr (SY::F == 3) {
    query_monomials<DP>(q, qm);
  } else {
    const float fx = gl ? 0.0f : 1.0f;
    static_for<0, SY::SP>([&](auto S) {
      constexpr int s = decltype(S)::value;
      if constexpr (s < SY::NS) {
        constexpr Duo t = sym2_slot(DP, s);
        qm[s] = s < SY::NPAIR ? q[t.x] * q[t.y] : (q[t.x] * q[t.y]) * fx;
      } else {
        qm[s] = 0.0f;
      }
    });
  }
}
template <class SY>
__device__ __forceinline__ void sym_query_monomials_grad(const float (&q)[SY::DPHI],
                                                         const float (&dm)[SY::SP],
                                                         float (&dq)[SY::DPHI], int gl) {
  constexpr int DP = SY::DPHI;
  if constexpr (SY::F == 3) {
    query_monomials_grad<DP>(q, dm, dq);
  } else {
    const float fx = gl ? 0.0f : 1.0f;
    static_for<0, SY::NS>([&](auto S) {
      constexpr int s = decltype(S)::value;
      constexpr Duo t = sym2_slot(DP, s);
      const float w = s < SY::NPAIR ? dm[s] : dm[s] * fx;
      dq[t.x] += w * q[t.y];
      dq[t.y] += w * q[t.x];
    });
  }
}
// all NM query monomials in canonical order (one lane serves one token, features not reversed)
template <class SY>
__device__ __forceinline__ void sym_query_monomials_all(const float (&q)[SY::DPHI], float (&qm)[SY::NM]) {
  constexpr int DP = SY::DPHI;
  static_for<0, SY::NM>([&](auto M) {
    constexpr int m = decltype(M)::value;
    if constexpr (SY::F == 3) {
      constexpr Tri t = sym3_mono(DP, m);
      qm[m] = (q[t.x] * q[t.y]) * q[t.z];
    } else {
      constexpr Duo t = sym2_mono(DP, m);
      qm[m] = q[t.x] * q[t.y];
    }
  });
}
// all NM key monomials in canonical order (one lane serves one token, features not reversed)
template <class SY>
__device__ __forceinline__ void sym_key_monomials_all(const float (&k)[SY::F][SY::DPHI],
                                                      float (&sm)[SY::NM]) {
  constexpr int DP = SY::DPHI;
  if constexpr (SY::F == 3) {
    key_monomials_all<DP>(k[0], k[1], k[2], sm);
  } else {
    static_for<0, SY::NM>([&](auto M) {
      constexpr int m = decltype(M)::value;
      constexpr Duo t = sym2_mono(DP, m);
      if constexpr (t.x == t.y)
        sm[m] = k[0][t.x] * k[1][t.x];
      else
        sm[m] = k[0][t.x] * k[1][t.y] + k[0][t.y] * k[1][t.x];
    });
  }
}
template <class SY>
__device__ __forceinline__ void sym_key_monomials_slots(const float (&k)[SY::F][SY::DPHI],
                                                        float (&sm)[SY::SP], int gl) {
  constexpr int DP = SY::DPHI;
  if constexpr (SY::F == 3) {
    key_monomials_slots<DP>(k[0], k[1], k[2], sm);
  } else {
    const float fx = gl ? 0.0f : 1.0f;
    static_for<0, SY::SP>([&](auto S) {
      constexpr int s = decltype(S)::value;
      if constexpr (s < SY::NS) {
        constexpr Duo t = sym2_slot(DP, s);
        if constexpr (t.x == t.y)
          sm[s] = k[0][t.x] * k[1][t.x];
        else
          sm[s] = k[0][t.x] * k[1][t.y] + k[0][t.y] * k[1][t.x];
        if constexpr (s >= SY::NPAIR) sm[s] *= fx;
      } else {
        sm[s] = 0.0f;
      }
    });
  }
}
// chain rule of sym_key_monomials_slots over slots S0 .. S1-1: clear a KeyGradAcc, call the ranges
// in any split, then sym_key_monomials_grad_finish (three factors: see key_monomials_grad_range;
// two factors: nothing is carried between the calls)
template <class SY>
struct KeyGradAcc {
  static constexpr int N = SY::F == 3 ? SY::DPHI : 1;
  float U[N][N];
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int a = 0; a < N; ++a)
#pragma unroll
      for (int b = 0; b < N; ++b) U[a][b] = 0.0f;
  }
};
template <class SY, int S0, int S1>
__device__ __forceinline__ void sym_key_monomials_grad_range(const float (&k)[SY::F][SY::DPHI],
                                                             const float (&ds)[SY::SP],
                                                             float (&dk)[SY::F][SY::DPHI],
                                                             KeyGradAcc<SY>& acc, int gl) {
  constexpr int DP = SY::DPHI;
  if constexpr (SY::F == 3) {
    key_monomials_grad_range<DP, S0, S1>(k[0], k[1], k[2], ds, acc.U, dk[2]);
  } else {
    const float fx = gl ? 0.0f : 1.0f;
    static_for<S0, (S1 < SY::NS ? S1 : SY::NS)>([&](auto S) {
      constexpr int s = decltype(S)::value;
      constexpr Duo t = sym2_slot(DP, s);
      const float w = s < SY::NPAIR ? ds[s] : ds[s] * fx;
      dk[0][t.x] += w * k[1][t.y];
      dk[1][t.y] += w * k[0][t.x];
      if constexpr (t.x != t.y) {
        dk[0][t.y] += w * k[1][t.x];
        dk[1][t.x] += w * k[0][t.y];
      }
    });
  }
}
template <class SY>
__device__ __forceinline__ void sym_key_monomials_grad_finish(const float (&k)[SY::F][SY::DPHI],
                                                              float (&dk)[SY::F][SY::DPHI],
                                                              const KeyGradAcc<SY>& acc) {
  if constexpr (SY::F == 3) key_monomials_grad_finish<SY::DPHI>(k[0], k[1], acc.U, dk[0], dk[1]);
}

}  // namespace mf
}  // namespace hla

#endif  // HLA_MFMA_COMMON_H_
