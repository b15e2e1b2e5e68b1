// GELU and its derivative on the vector ALU in packed fp16, shared by the matrix-core kernels
// that apply Linear -> GELU -> Linear maps (the feature maps of App. A.1 and the value-modulation
// maps of Sec. 4.5).
#ifndef HLA_MFMA_GELU_H_
#define HLA_MFMA_GELU_H_

#include "hla_mfma_common.h"

namespace hla {
namespace mf {

// ---- GELU on the vector ALU, two values per instruction in packed fp16 -------------------------
// The first layer is computed at a quarter of its scale (W1 and b1 are packed times 1/4, an exact
// scaling), so the vector ALU sees y = x/4.  With yc = clamp(y, +-1) and v = yc^2 - 1/2 in
// [-1/2, 1/2]:   Phi(x) - 1/2 = yc * P(v),   GELU(x)/4 = y * (1/2 + yc * P(v)),
// GELU'(x) = 1/2 + yc * Q(v); the factor 4 is folded into the packed second-layer weights.  In this
// variable v costs one FMA, and a Horner chain of fp16 FMAs keeps its rounding error near 2^-12
// per step.  Evaluated end to end in fp16 the absolute GELU error is at most 5.2e-3 (rms 5.1e-4
// for standard-normal inputs; fp16 rounding, not the fit, sets it: one degree more gains 1.5e-3
// at most): a third of what rounding an exact GELU to bf16 would cost, which is why the hidden
// layer is handed to the second layer in fp16.
// Pre-activations must stay below four times the fp16 range (65504) in magnitude.
constexpr float kHiddenScale = 0.25f;
__device__ __forceinline__ f16x2 splat16(float v) {
  f16x2 r;
  r[0] = static_cast<_Float16>(v);
  r[1] = r[0];
  return r;
}
__device__ __forceinline__ f16x2 to_f16x2(float a, float b) {
  f16x2 r;
  r[0] = static_cast<_Float16>(a);  // round to nearest even (v_cvt_pk_f16_f32)
  r[1] = static_cast<_Float16>(b);
  return r;
}
__device__ __forceinline__ f16x2 clamp1(f16x2 x) {
  return __builtin_elementwise_min(__builtin_elementwise_max(x, splat16(-1.0f)), splat16(1.0f));
}
// NCH independent chains are advanced in lockstep: a packed-fp16 instruction cannot issue right
// behind the one that produces its input, so a single Horner chain would leave every other issue
// slot empty.
// GELU(x)/4 of 2*NCH values y = x/4 held as packed fp16 pairs: degree-5 fit of (Phi - 1/2)/yc in v
template <int NCH>
__device__ __forceinline__ void gelu_y16(const f16x2 (&y)[NCH], uint32_t (&out)[NCH]) {
  constexpr float c[6] = {0.70459f, -0.672363f, 0.841797f, -1.19434f, 2.07227f, -1.90039f};
  f16x2 yc[NCH], v[NCH], p[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) yc[i] = clamp1(y[i]);
#pragma unroll
  for (int i = 0; i < NCH; ++i) v[i] = __builtin_elementwise_fma(yc[i], yc[i], splat16(-0.5f));
#pragma unroll
  for (int i = 0; i < NCH; ++i) p[i] = __builtin_elementwise_fma(splat16(c[5]), v[i], splat16(c[4]));
#pragma unroll
  for (int k = 3; k >= 0; --k)
#pragma unroll
    for (int i = 0; i < NCH; ++i) p[i] = __builtin_elementwise_fma(p[i], v[i], splat16(c[k]));
#pragma unroll
  for (int i = 0; i < NCH; ++i) p[i] = __builtin_elementwise_fma(yc[i], p[i], splat16(0.5f));
#pragma unroll
  for (int i = 0; i < NCH; ++i) out[i] = __builtin_bit_cast(uint32_t, y[i] * p[i]);
}
// the same from fp32 values (rounded to fp16 first)
template <int NCH>
__device__ __forceinline__ void gelu_f16(const float (&in)[2 * NCH], uint32_t (&out)[NCH]) {
  f16x2 y[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) y[i] = to_f16x2(in[2 * i], in[2 * i + 1]);
  gelu_y16<NCH>(y, out);
}
// d/dx [x Phi(x)] at x = 4y for 2*NCH values y held as packed fp16 pairs: degree-6 fit of
// (GELU' - 1/2)/yc in v, |error| <= 2.1e-3 (the rounding of the product with dg to bf16 costs
// twice that)
template <int NCH>
__device__ __forceinline__ void gelu_grad_y16(const f16x2 (&y)[NCH], f16x2 (&out)[NCH]) {
  constexpr float c[7] = {0.733398f, -0.930664f, 1.80273f, -2.875f, 6.35938f, -16.375f, 16.4062f};
  f16x2 yc[NCH], v[NCH], p[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) yc[i] = clamp1(y[i]);
#pragma unroll
  for (int i = 0; i < NCH; ++i) v[i] = __builtin_elementwise_fma(yc[i], yc[i], splat16(-0.5f));
#pragma unroll
  for (int i = 0; i < NCH; ++i) p[i] = __builtin_elementwise_fma(splat16(c[6]), v[i], splat16(c[5]));
#pragma unroll
  for (int k = 4; k >= 0; --k)
#pragma unroll
    for (int i = 0; i < NCH; ++i) p[i] = __builtin_elementwise_fma(p[i], v[i], splat16(c[k]));
#pragma unroll
  for (int i = 0; i < NCH; ++i) out[i] = __builtin_elementwise_fma(yc[i], p[i], splat16(0.5f));
}
template <int NCH>
__device__ __forceinline__ void gelu_grad_f16(const float (&in)[2 * NCH], f16x2 (&out)[NCH]) {
  f16x2 y[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) y[i] = to_f16x2(in[2 * i], in[2 * i + 1]);
  gelu_grad_y16<NCH>(y, out);
}

// GELU(x)/4 and GELU'(x) of the same 2*NCH values y = x/4 (the two fits share yc and v)
template <int NCH>
__device__ __forceinline__ void gelu_both_f16(const float (&in)[2 * NCH], f16x2 (&gout)[NCH],
                                              f16x2 (&dout)[NCH]) {
  constexpr float c[6] = {0.70459f, -0.672363f, 0.841797f, -1.19434f, 2.07227f, -1.90039f};
  constexpr float e[7] = {0.733398f, -0.930664f, 1.80273f, -2.875f, 6.35938f, -16.375f, 16.4062f};
  f16x2 y[NCH], yc[NCH], v[NCH], p[NCH], q[NCH];
#pragma unroll
  for (int i = 0; i < NCH; ++i) y[i] = to_f16x2(in[2 * i], in[2 * i + 1]);
#pragma unroll
  for (int i = 0; i < NCH; ++i) yc[i] = clamp1(y[i]);
#pragma unroll
  for (int i = 0; i < NCH; ++i) v[i] = __builtin_elementwise_fma(yc[i], yc[i], splat16(-0.5f));
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    p[i] = __builtin_elementwise_fma(splat16(c[5]), v[i], splat16(c[4]));
    q[i] = __builtin_elementwise_fma(splat16(e[6]), v[i], splat16(e[5]));
  }
#pragma unroll
  for (int i = 0; i < NCH; ++i) q[i] = __builtin_elementwise_fma(q[i], v[i], splat16(e[4]));
#pragma unroll
  for (int k = 3; k >= 0; --k)
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      p[i] = __builtin_elementwise_fma(p[i], v[i], splat16(c[k]));
      q[i] = __builtin_elementwise_fma(q[i], v[i], splat16(e[k]));
    }
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    p[i] = __builtin_elementwise_fma(yc[i], p[i], splat16(0.5f));
    dout[i] = __builtin_elementwise_fma(yc[i], q[i], splat16(0.5f));
    gout[i] = y[i] * p[i];
  }
}

}  // namespace mf
}  // namespace hla

#endif  // HLA_MFMA_GELU_H_
