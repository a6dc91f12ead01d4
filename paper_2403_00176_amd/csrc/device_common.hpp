// Device helpers shared by the kernel files: bf16 conversion, activations, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "launch.hpp"

namespace sod2 {

typedef uint16_t bf16_t;
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
// round to nearest, ties to even: the conversion instruction of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values in one instruction: lo in bits 0..15, hi in bits 16..31
__device__ __forceinline__ uint32_t f2bf2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
template <class T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf2f(v); }
template <class T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return f2bf(v); }

// GELU in its erf form, 0.5 x (1 + erf(x / sqrt 2)) = h + |h| erf(|z|) with h = x / 2, z = x / sqrt 2.
// erf(z) for z >= 0 is evaluated as 1 - 2^(-z P(z)) with P of degree 5, the weighted least-squares fit of
// -log2(erfc(z)) / z on [0, 4] (beyond 4, erfc < 1.6e-8 is held constant); absolute error of erf below 3.2e-7 in
// fp32, far inside the rounding of the bf16 or fp32 value the GELU is stored as.  One v_exp_f32, no reciprocal, no
// division: 15 issue slots per element against 24 for the rational-times-Gaussian form (the epilogue of a
// contraction that ends in GELU is bound by these instructions).
__device__ __forceinline__ float erf_pos(float z) {           // z >= 0
  z = fminf(z, 4.0f);
  float p = fmaf(-0.00014206966f, z, 0.0036644198f);
  p = fmaf(p, z, -0.030896446f);
  p = fmaf(p, z, 0.14969963f);
  p = fmaf(p, z, 0.91816539f);
  p = fmaf(p, z, 1.6279250f);
  return 1.f - __builtin_amdgcn_exp2f(-(p * z));
}
__device__ __forceinline__ float gelu_erf(float v) {
  const float h = 0.5f * v;
  return fmaf(fabsf(h), erf_pos(fabsf(v) * 0.70710678118654752f), h);
}

__device__ __forceinline__ float apply_act(float v, int act) {
  if (act == ACT_RELU) return fmaxf(v, 0.f);
  if (act == ACT_GELU) return gelu_erf(v);
  if (act == ACT_SIGMOID) return 1.f / (1.f + __expf(-v));
  return v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

union V16 {
  uint4 u;
  bf16x8_t b;
  bf16_t h[8];
  uint32_t w[4];
};
__device__ __forceinline__ uint4 zero4() { return make_uint4(0, 0, 0, 0); }

}  // namespace sod2
