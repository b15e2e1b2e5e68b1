// Shared host/device definitions of libhla (internal; the public boundary is include/hla.h).
#ifndef HLA_COMMON_H_
#define HLA_COMMON_H_

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "hla.h"

namespace hla {

// ---- element types ---------------------------------------------------------------------------
struct bf16_t {
  uint16_t bits;
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) {
  return __uint_as_float(static_cast<uint32_t>(x.bits) << 16);
}
// round-to-nearest-even, NaN kept quiet
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<uint16_t>(u >> 16);
}
template <typename T>
__device__ __forceinline__ T from_float(float f);
template <>
__device__ __forceinline__ float from_float<float>(float f) {
  return f;
}
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float f) {
  bf16_t r;
  r.bits = f32_to_bf16_bits(f);
  return r;
}

// ---- views and tables ------------------------------------------------------------------------
// Strided [B,H,N,width] view, innermost contiguous (mirrors hla_tensor, device side).
struct View {
  void* ptr;
  int64_t sb, sh, sn;
  template <typename T>
  __device__ __forceinline__ T* row(int b, int h, int n) const {
    return static_cast<T*>(ptr) + b * sb + h * sh + static_cast<int64_t>(n) * sn;
  }
};
inline View make_view(const hla_tensor& t) { return View{t.ptr, t.stride_b, t.stride_h, t.stride_n}; }

// A run of consecutive tokens [t0, t1) of one sequence, living in batch row b.
struct BlockEnt {
  int32_t b;
  int32_t seq;
  int32_t t0;
  int32_t t1;
};

// Problem geometry shared by all kernels of one call.
struct Geom {
  int32_t B, H, N;       // as passed by the caller (N = tokens per batch row)
  int32_t d, dphi, F, D;  // head dim, feature dim, degree, dphi^F
  int32_t nfeat;          // (1+F)*dphi, features per token-head in the feature workspace
  int32_t feat_tiled;     // layout of the feature workspaces, see fidx()
  float eps;
  __host__ __device__ __forceinline__ int64_t th(int b, int h, int n) const {
    return (static_cast<int64_t>(b) * H + h) * N + n;
  }
  // Index of feature a of token-head th in the feature / feature-gradient workspace.  Plain:
  // [th][nfeat].  Tiled (matrix-core path, nfeat even): [th / 32][nfeat / 2][32][2], so that the 32
  // lanes that hold one PAIR of features (2p, 2p + 1) of 32 consecutive token-heads read and write
  // one contiguous 256-byte run with one 8-byte access each.
  __host__ __device__ __forceinline__ int64_t fidx(int64_t th, int a) const {
    return feat_tiled ? (th >> 5) * (static_cast<int64_t>(nfeat) * 32) + (a >> 1) * 64 + ((th & 31) << 1) + (a & 1)
                      : th * nfeat + a;
  }
};

// Feature-map weights converted to fp32 and densely packed per map:
//   W1 [maps][heads_w][d][d], b1 [maps][heads_w][d], W2 [maps][heads_w][d][dphi], b2 [..][dphi]
// heads_w is 1 when the weights are shared by all heads.
struct PhiF32 {
  const float* W1;
  const float* b1;
  const float* W2;
  const float* b2;
  int32_t heads_w;
};

// ---- launch bookkeeping ----------------------------------------------------------------------
struct ProfileRecord {
  const char* name;
  hipEvent_t start, stop;
};

struct Profiler {
  bool on = false;
  std::vector<ProfileRecord> records;     // used prefix: n_used
  size_t n_used = 0;
  bool pending = false;
  const char* begin(const char* name, hipStream_t s);
  void end(hipStream_t s);
  void clear_records();
  void destroy();
};

}  // namespace hla

#define HLA_HIP_TRY(expr)                      \
  do {                                         \
    hipError_t _e = (expr);                    \
    if (_e != hipSuccess) return HLA_ERR_HIP;  \
  } while (0)

#endif  // HLA_COMMON_H_
