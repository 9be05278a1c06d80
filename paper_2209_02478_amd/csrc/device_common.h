// Device-side helpers shared by the kernels: storage types, conversions, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mk {

typedef uint16_t bf16_t;   // raw bfloat16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
  return __uint_as_float(((uint32_t)v) << 16);
}
// round to nearest, ties to even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  return __builtin_bit_cast(bf16_t, (__bf16)f);
}
// two values in one conversion: a in the low half, b in the high half
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> __device__ __forceinline__ float ld(const T* p);
template <> __device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }

template <typename T> __device__ __forceinline__ void st(T* p, float v);
template <> __device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// value a T would hold after a store (used where a kernel must behave as if it re-read its output)
template <typename T> __device__ __forceinline__ float rnd(float v);
template <> __device__ __forceinline__ float rnd<float>(float v) { return v; }
template <> __device__ __forceinline__ float rnd<bf16_t>(float v) { return bf16_to_f32(f32_to_bf16(v)); }

// Sums (maxima) over the 64 lanes of a wave, the result in every lane.  Inside a row of 16 lanes
// four rotating DPP adds (by 8, 4, 2, 1) leave the row's total in each of its lanes; the four
// rows are then read through scalar registers and combined in row order.  A butterfly of
// cross-lane shuffles costs six dependent trips through the LDS crossbar instead, which is what
// the row-wise kernels spent most of their time on.  The order of the additions is fixed.
template <int CTRL>
__device__ __forceinline__ float dpp_rotate(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_rotate<0x128>(v);   // row_ror:8
  v += dpp_rotate<0x124>(v);   // row_ror:4
  v += dpp_rotate<0x122>(v);   // row_ror:2
  v += dpp_rotate<0x121>(v);   // row_ror:1
  return ((lane_value(v, 0) + lane_value(v, 16)) + lane_value(v, 32)) + lane_value(v, 48);
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_rotate<0x128>(v));
  v = fmaxf(v, dpp_rotate<0x124>(v));
  v = fmaxf(v, dpp_rotate<0x122>(v));
  v = fmaxf(v, dpp_rotate<0x121>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}

__device__ __forceinline__ float gelu_erf(float x) {
  return 0.5f * x * (1.0f + erff(x * 0.70710678118654752440f));
}
// erf by the rational approximation of Abramowitz & Stegun 7.1.26 (absolute error < 1.5e-7),
// one exponential and one reciprocal: used where the result is rounded to bf16 anyway
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __frcp_rn(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(t, 1.061405429f, -1.453152027f);
  p = fmaf(t, p, 1.421413741f);
  p = fmaf(t, p, -0.284496736f);
  p = fmaf(t, p, 0.254829592f);
  const float r = 1.0f - p * t * __expf(-ax * ax);
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_erf_bf16(float x) {
  return 0.5f * x * (1.0f + erf_as(x * 0.70710678118654752440f));
}
// tanh form with tanh(u) = 1 - 2 / (1 + exp(2u)): exact limits at both ends, relative error ~1e-6
__device__ __forceinline__ float gelu_tanh_bf16(float x) {
  const float c = 0.79788456080286535588f;
  const float u = c * (x + 0.044715f * x * x * x);
  const float t = 1.0f - 2.0f * __frcp_rn(1.0f + __expf(2.0f * u));
  return 0.5f * x * (1.0f + t);
}
__device__ __forceinline__ float gelu_tanh(float x) {
  const float c = 0.79788456080286535588f;
  return 0.5f * x * (1.0f + tanhf(c * (x + 0.044715f * x * x * x)));
}
__device__ __forceinline__ float gelu_erf_grad(float x) {
  float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752440f));
  float pdf = 0.39894228040143267794f * __expf(-0.5f * x * x);
  return cdf + x * pdf;
}
// the same with the rational erf above: its exponential, exp(-x^2 / 2), is also the density's, so
// the derivative costs one exponential and one reciprocal (used where the result is rounded to bf16)
__device__ __forceinline__ float gelu_erf_grad_bf16(float x) {
  const float ax = fabsf(x) * 0.70710678118654752440f;
  const float t = __frcp_rn(fmaf(0.3275911f, ax, 1.0f));
  float p = fmaf(t, 1.061405429f, -1.453152027f);
  p = fmaf(t, p, 1.421413741f);
  p = fmaf(t, p, -0.284496736f);
  p = fmaf(t, p, 0.254829592f);
  const float e = __expf(-ax * ax);
  const float erf_x = copysignf(1.0f - p * t * e, x);
  return 0.5f * (1.0f + erf_x) + x * 0.39894228040143267794f * e;
}
__device__ __forceinline__ float gelu_tanh_grad(float x) {
  const float c = 0.79788456080286535588f;
  float t = tanhf(c * (x + 0.044715f * x * x * x));
  return 0.5f * (1.0f + t) + 0.5f * x * (1.0f - t * t) * c * (1.0f + 0.134145f * x * x);
}

}  // namespace mk
