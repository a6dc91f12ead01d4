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

// Reductions over the 64 lanes of a wave (all of them active), through the data-parallel-primitive lane moves: no LDS
// round trip per step as with a lane permute (a chain of six of those is ~0.3 us; three such chains made up a sixth
// of the one-row LayerNorm + contraction kernel).  Steps: lane ^ 1 and lane ^ 2 inside a quad, the mirror inside a
// half row of 8 and inside a row of 16, then lane 15 of rows 0 and 2 into rows 1 and 3 and lane 31 into the upper
// half: lane 63 holds the result, which every lane reads.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp_move(float old, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v), CTRL,
                                                               ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1>(0.f, v);                    // quad_perm [1, 0, 3, 2]
  v += dpp_move<0x4E>(0.f, v);                    // quad_perm [2, 3, 0, 1]
  v += dpp_move<0x141>(0.f, v);                   // row_half_mirror
  v += dpp_move<0x140>(0.f, v);                   // row_mirror
  v += dpp_move<0x142, 0xA>(0.f, v);              // row_bcast15 into rows 1 and 3
  v += dpp_move<0x143, 0xC>(0.f, v);              // row_bcast31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<0xB1>(v, v));
  v = fmaxf(v, dpp_move<0x4E>(v, v));
  v = fmaxf(v, dpp_move<0x141>(v, v));
  v = fmaxf(v, dpp_move<0x140>(v, v));
  v = fmaxf(v, dpp_move<0x142, 0xA>(v, v));
  v = fmaxf(v, dpp_move<0x143, 0xC>(v, v));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
// sum over the 8 lanes 8 q .. 8 q + 7, in every one of them
__device__ __forceinline__ float octet_sum(float v) {
  v += dpp_move<0xB1>(0.f, v);
  v += dpp_move<0x4E>(0.f, v);
  v += dpp_move<0x141>(0.f, v);
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
