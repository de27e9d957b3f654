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

// 16 bytes of a weight matrix that a decode step reads once (the next layer brings its own weights):
// a non-temporal load, which streams from HBM about 15 % faster than a plain one
typedef uint32_t ekv_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const void* p) {
  const ekv_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const ekv_u32x4*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

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

// Layout of the absorbed query in the workspace of the matrix-core decode path: element (b, h, k) of
// q~ [B, n_h, d_q] is stored so that what one wave of the attention kernel loads with one instruction,
// the MFMA operand of 16 heads x 32 latent columns (lane l: head 16*hh + l%16, columns 8*(l/16) .. +8),
// is one contiguous KiB: blocks [b][head group of 32][column slice of qs][32-column step][head half],
// inside a block lane-major, 8 columns per lane.  Head groups are padded to 32 heads (slots of heads
// beyond n_h are never written or used).
__host__ __device__ inline int64_t qt_packed_index(int b, int h, int k, int head_groups, int d_q, int qs) {
  const int hg = h >> 5, hh = (h >> 4) & 1, i = h & 15;
  const int w = k / qs, kk = k - w * qs;
  const int64_t blk = ((((int64_t)b * head_groups + hg) * (d_q / qs) + w) * (qs / 32) + (kk >> 5)) * 2 + hh;
  return (blk * 64 + ((kk >> 3) & 3) * 16 + i) * 8 + (kk & 7);
}

// Column n of the append's output Y = x [W_ke | W_dkv | W_dkv2]: which weight matrix holds it, at
// which column, with which row stride.  NE = 2 r n_h elite columns, then d_ck columns of W_dkv,
// then d_c - d_ck columns of W_dkv2 (separated latents; d_ck == d_c for the joint latent).
template <typename T>
__device__ __forceinline__ void weight_column(int n, int NE, int d_ck, int d_c, const T* W_ke, const T* W_dkv,
                                              const T* W_dkv2, const T** base, int64_t* stride) {
  if (n < NE) { *base = W_ke + n; *stride = NE; }
  else if (n - NE < d_ck) { *base = W_dkv + (n - NE); *stride = d_ck; }
  else { *base = W_dkv2 + (n - NE - d_ck); *stride = d_c - d_ck; }
}

// theta_i = base^(-2i/d_h) (Section 2.2; RoFormer's frequencies), computed once per call on the
// host in double and handed to the kernels by value (head_dim <= 256: at most 128 chunks).
struct RopeTable {
  double theta[128];
};
inline RopeTable make_rope_table(double base, int head_dim) {
  RopeTable t;
  for (int i = 0; i < 128; ++i) t.theta[i] = (2 * i < head_dim) ? pow(base, -2.0 * (double)i / (double)head_dim) : 0.0;
  return t;
}

// The table of the calling thread's last (base, head_dim): a decode loop asks for the same one at
// every launch, and 128 pow() calls are several microseconds of host time.
inline const RopeTable& rope_table(double base, int head_dim) {
  thread_local RopeTable table;
  thread_local double have_base = 0.0;
  thread_local int have_dim = 0;
  if (have_base != base || have_dim != head_dim) {
    table = make_rope_table(base, head_dim);
    have_base = base;
    have_dim = head_dim;
  }
  return table;
}

// sin and cos of pos * theta.  The angle is formed and reduced to [-pi/4, pi/4] in double
// (two-term Cody-Waite, exact for the |k| < 2^20 quadrants that positions up to 2^31 with
// theta <= 1 can reach in practice); only the reduced argument goes through fp32 sin/cos.
__device__ __forceinline__ void rope_sincos(int32_t pos, double theta, float* sn, float* cs) {
  const double a = (double)pos * theta;
  const double k = rint(a * 0.63661977236758134308);        // a / (pi/2)
  double r = fma(-k, 1.57079632679489655800e+00, a);        // pi/2, high part
  r = fma(-k, 6.12323399573676603587e-17, r);               // pi/2, low part
  const float rf = (float)r;
  const float s = sinf(rf), c = cosf(rf);
  const int q = (int)((long long)k & 3);
  *sn = (q == 0) ? s : (q == 1) ? c : (q == 2) ? -s : -c;
  *cs = (q == 0) ? c : (q == 1) ? -s : (q == 2) ? -c : s;
}

// The same with sin and cos of the reduced argument from their Taylor polynomials (|r| <= pi/4:
// truncation below 3e-8, i.e. fp32 rounding level) instead of the library routines, whose
// instruction count dominates the epilogue of the matrix-core append (16 to 64 rotations per lane).
__device__ __forceinline__ void rope_sincos_poly(int32_t pos, double theta, float* sn, float* cs) {
  const double a = (double)pos * theta;
  const double k = rint(a * 0.63661977236758134308);        // a / (pi/2)
  double r = fma(-k, 1.57079632679489655800e+00, a);        // pi/2, high part
  r = fma(-k, 6.12323399573676603587e-17, r);               // pi/2, low part
  const float x = (float)r, x2 = x * x;
  float ps = fmaf(x2, 2.7557319e-6f, -1.9841270e-4f);       // x^9/9! - x^7/7! ...
  ps = fmaf(ps, x2, 8.3333333e-3f);
  ps = fmaf(ps, x2, -1.6666667e-1f);
  const float s = fmaf(ps * x2, x, x);
  float pc = fmaf(x2, 2.4801587e-5f, -1.3888889e-3f);       // x^8/8! - x^6/6! ...
  pc = fmaf(pc, x2, 4.1666667e-2f);
  pc = fmaf(pc, x2, -0.5f);
  const float c = fmaf(pc, x2, 1.0f);
  const int q = (int)((long long)k & 3);
  *sn = (q == 0) ? s : (q == 1) ? c : (q == 2) ? -s : -c;
  *cs = (q == 0) ? c : (q == 1) ? -s : (q == 2) ? -c : s;
}

}  // namespace ekv
