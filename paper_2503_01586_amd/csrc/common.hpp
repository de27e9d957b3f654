// Shared device helpers of libelitekv: storage types, conversions, wave reductions.
// gfx950 only: 64-wide wavefronts are assumed everywhere.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ekv {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;

// bf16 is kept as raw bits; arithmetic is always fp32.
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
  return __builtin_bit_cast(uint16_t, (__bf16)f);   // the hardware conversion of gfx950
}

__device__ __forceinline__ float ld(const float* p, int64_t i) { return p[i]; }
__device__ __forceinline__ float ld(const bf16_t* p, int64_t i) { return bf16_bits_to_f32(p[i].bits); }
__device__ __forceinline__ void st(float* p, int64_t i, float v) { p[i] = v; }
__device__ __forceinline__ void st(bf16_t* p, int64_t i, float v) { p[i].bits = f32_to_bf16_bits(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// theta_i = base^(-2i/d_h) in double (Section 2.2; RoFormer's frequencies)
__device__ __forceinline__ double rope_theta(double base, int i, int head_dim) {
  return pow(base, -2.0 * (double)i / (double)head_dim);
}

}  // namespace ekv
