// Measurement-only kernels that sit beside the EliteKV path:
//   * ordinary RoPE multi-head decode attention over an uncompressed cache (Section 2.2: a RoPE
//     model caches all d_h rotated key dims and the value), split over the sequence;
//   * a streaming-read probe that gives the achievable HBM read rate.
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

constexpr int kMhaThreads = 256;

template <typename T> struct Vec16;
template <> struct Vec16<float> { static constexpr int n = 4; };
template <> struct Vec16<bf16_t> { static constexpr int n = 8; };

// 16 bytes of a plane that is read once per step: a non-temporal load (streams from HBM about 15 % faster)
typedef uint32_t ck_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ ck_u32x4 stream16(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const ck_u32x4*>(p));
}
template <typename T>
__device__ __forceinline__ void load16(const T* p, float (&out)[Vec16<T>::n]);
template <>
__device__ __forceinline__ void load16<float>(const float* p, float (&out)[4]) {
  const ck_u32x4 v = stream16(p);
  out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y); out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
}
template <>
__device__ __forceinline__ void load16<bf16_t>(const bf16_t* p, float (&out)[8]) {
  const ck_u32x4 v = stream16(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    out[2 * i] = __uint_as_float(w[i] << 16);
    out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}

// One work-group per (split, head, batch row).  LPR lanes share one cached row (16 bytes each);
// a wave therefore covers 64/LPR tokens per step.  Each lane group runs its own online softmax;
// the groups are merged through LDS at the end.
template <typename T, int LPR>
__global__ __launch_bounds__(kMhaThreads) void mha_attn_kernel(
    const T* __restrict__ q, const int32_t* __restrict__ q_pos, const int32_t* __restrict__ seq_len,
    const T* __restrict__ k_plane, const T* __restrict__ v_plane, float* __restrict__ part_m,
    float* __restrict__ part_l, float* __restrict__ part_o, int n_h, int d_h, RopeTable rope,
    float scale_log2e, int64_t max_seq_len, int64_t batch_stride_rows, int64_t plane_rows,
    int n_splits, int chunk) {
  constexpr int VEC = Vec16<T>::n;
  constexpr int TPW = 64 / LPR;            // tokens per wave step
  constexpr int GROUPS = 4 * TPW;          // lane groups in the work-group
  extern __shared__ float smem[];
  float* q_s = smem;                       // [d_h]
  float* g_m = q_s + d_h;                  // [GROUPS]
  float* g_l = g_m + GROUPS;               // [GROUPS]
  float* g_o = g_l + GROUPS;               // [GROUPS][d_h]

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sub = lane % LPR, grp = lane / LPR;

  const int64_t row0 = (int64_t)b * batch_stride_rows;
  int64_t len = seq_len[b];
  len = min(len, max_seq_len);
  len = min(len, plane_rows - row0);
  len = max(len, (int64_t)0);
  const int64_t t0 = (int64_t)split * chunk;
  const int64_t t1 = min(t0 + chunk, len);

  const T* qrow = q + ((int64_t)b * n_h + h) * d_h;
  for (int i = tid; i < d_h / 2; i += kMhaThreads) {
    float s, c;
    rope_sincos(q_pos[b], rope.theta[i], &s, &c);
    const float u = ld(qrow, 2 * i), v = ld(qrow, 2 * i + 1);
    q_s[2 * i] = (u * c - v * s) * scale_log2e;
    q_s[2 * i + 1] = (u * s + v * c) * scale_log2e;
  }
  __syncthreads();
  float qv[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) qv[i] = q_s[sub * VEC + i];

  float acc[VEC];
#pragma unroll
  for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int64_t t = t0 + wave * TPW + grp; t < t1; t += 4 * TPW) {
    const int64_t off = ((row0 + t) * n_h + h) * d_h + sub * VEC;
    float kv[VEC], vv[VEC];
    load16<T>(k_plane + off, kv);
    load16<T>(v_plane + off, vv);
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < VEC; ++i) s = fmaf(qv[i], kv[i], s);
#pragma unroll
    for (int o = LPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, kWave);
    const float m_new = fmaxf(m, s);
    const float alpha = exp2f(m - m_new);
    const float p = exp2f(s - m_new);
    l = l * alpha + p;
#pragma unroll
    for (int i = 0; i < VEC; ++i) acc[i] = fmaf(p, vv[i], acc[i] * alpha);
    m = m_new;
  }

  const int g = wave * TPW + grp;
  if (sub == 0) { g_m[g] = m; g_l[g] = l; }
#pragma unroll
  for (int i = 0; i < VEC; ++i) g_o[g * d_h + sub * VEC + i] = acc[i];
  __syncthreads();

  const int64_t pi = ((int64_t)b * n_splits + split) * n_h + h;
  float M = -INFINITY;
  for (int gg = 0; gg < GROUPS; ++gg) M = fmaxf(M, g_m[gg]);
  float L = 0.f;
  for (int gg = 0; gg < GROUPS; ++gg) L += (g_l[gg] > 0.f) ? g_l[gg] * exp2f(g_m[gg] - M) : 0.f;
  for (int j = tid; j < d_h; j += kMhaThreads) {
    float o = 0.f;
    for (int gg = 0; gg < GROUPS; ++gg)
      if (g_l[gg] > 0.f) o = fmaf(exp2f(g_m[gg] - M), g_o[gg * d_h + j], o);
    part_o[pi * d_h + j] = o;
  }
  if (tid == 0) { part_m[pi] = M; part_l[pi] = L; }
}

template <typename T>
__global__ __launch_bounds__(kMhaThreads) void mha_merge_kernel(
    const float* __restrict__ part_m, const float* __restrict__ part_l,
    const float* __restrict__ part_o, T* __restrict__ out, int n_h, int d_h, int n_splits) {
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int64_t base = (int64_t)b * n_splits * n_h + h;
  float M = -INFINITY;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, part_m[base + (int64_t)s * n_h]);
  float L = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float ls = part_l[base + (int64_t)s * n_h];
    L += (ls > 0.f) ? ls * exp2f(part_m[base + (int64_t)s * n_h] - M) : 0.f;
  }
  const float inv = L > 0.f ? 1.f / L : 0.f;
  for (int j = tid; j < d_h; j += kMhaThreads) {
    float o = 0.f;
    for (int s = 0; s < n_splits; ++s) {
      const int64_t pi = base + (int64_t)s * n_h;
      if (part_l[pi] > 0.f) o = fmaf(exp2f(part_m[pi] - M), part_o[pi * d_h + j], o);
    }
    st(out, ((int64_t)b * n_h + h) * d_h + j, o * inv);
  }
}

template <typename T, int LPR>
static void launch_mha_t(const MhaArgs& a, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int n_h = d.n_heads, d_h = d.head_dim;
  const size_t np = (size_t)a.B * a.n_splits * n_h;
  float* pm = (float*)a.ws;
  float* pl = pm + np;
  float* po = pl + np;
  constexpr int GROUPS = 4 * (64 / LPR);
  const size_t sm = sizeof(float) * (size_t)(d_h + 2 * GROUPS + GROUPS * d_h);
  const float scale_log2e = kLog2e / sqrtf((float)d_h);
  mha_attn_kernel<T, LPR><<<dim3(a.n_splits, n_h, (unsigned)a.B), kMhaThreads, sm, stream>>>(
      (const T*)a.q, a.q_pos, a.seq_len, (const T*)a.k_plane, (const T*)a.v_plane, pm, pl, po, n_h,
      d_h, rope_table(d.rope_base, d.head_dim), scale_log2e, a.max_seq_len, a.batch_stride_rows, a.plane_rows, a.n_splits,
      a.chunk);
  mha_merge_kernel<T><<<dim3(n_h, (unsigned)a.B), kMhaThreads, 0, stream>>>(pm, pl, po, (T*)a.out, n_h,
                                                                         d_h, a.n_splits);
}

hipError_t launch_mha_decode(const MhaArgs& a, hipStream_t stream) {
  const int d_h = a.dims.head_dim;
  const bool f32 = a.dims.dtype == ELITEKV_FP32;
  const int lpr = d_h / (f32 ? 4 : 8);
#define EKV_MHA(L)                                      \
  do {                                                  \
    if (f32) launch_mha_t<float, L>(a, stream);         \
    else launch_mha_t<bf16_t, L>(a, stream);            \
  } while (0)
  switch (lpr) {
    case 2: EKV_MHA(2); break;
    case 4: EKV_MHA(4); break;
    case 8: EKV_MHA(8); break;
    case 16: EKV_MHA(16); break;
    case 32: EKV_MHA(32); break;
    case 64: EKV_MHA(64); break;
    default: return hipErrorInvalidValue;
  }
#undef EKV_MHA
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
constexpr int kStreamThreads = 256;
constexpr int kStreamGrid = 2048;

// NT: the loads carry the non-temporal bit
template <bool NT>
__global__ __launch_bounds__(kStreamThreads) void stream_read_kernel(const uint4* __restrict__ src,
                                                                     size_t n16, uint32_t* sink) {
  // every block streams one contiguous share, eight 16-byte loads per thread in flight
  auto ld = [](const uint4* p) -> ck_u32x4 { return NT ? stream16(p) : *reinterpret_cast<const ck_u32x4*>(p); };
  uint32_t acc = 0;
  const size_t per = (n16 + gridDim.x - 1) / gridDim.x;
  const size_t lo = per * blockIdx.x, hi = min(lo + per, n16);
  size_t i = lo + threadIdx.x;
  for (; i + 7 * kStreamThreads < hi; i += 8 * kStreamThreads) {
    ck_u32x4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = ld(src + i + u * kStreamThreads);
#pragma unroll
    for (int u = 0; u < 8; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < hi; i += kStreamThreads) {
    const ck_u32x4 a = ld(src + i);
    acc ^= a.x ^ a.y ^ a.z ^ a.w;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o, kWave);
  if ((threadIdx.x & 63) == 0) atomicXor(&sink[blockIdx.x], acc);
}

// The same stream through direct global->LDS loads (what the attention kernel's tiles come in by): every wave
// keeps two groups of eight 1 KiB loads in flight in an LDS area of its own; nothing reads the LDS.  Whole
// 8 KiB groups only: the last bytes % (grid * 4 waves * 8 KiB) bytes are left out (the caller accounts for them).
constexpr int kStreamLdsGrid = 512;
constexpr int kStreamLdsBytes = 4 * 16384;
constexpr size_t kStreamLdsUnit = (size_t)kStreamLdsGrid * 4 * 8192;

template <bool NT>
__global__ __launch_bounds__(kStreamThreads) void stream_read_lds_kernel(const char* __restrict__ src, size_t groups,
                                                                         uint32_t* sink) {
  extern __shared__ __attribute__((aligned(16))) char ssm[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const char* p = src + ((size_t)blockIdx.x * 4 + wave) * groups * 8192 + lane * 16;
  const uint32_t base = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)ssm + wave * 16384);
  for (size_t g = 0; g < groups; ++g) {
    const uint32_t b = base + (uint32_t)(g & 1) * 8192;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (NT)
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off nt" : : "s"(b + u * 1024), "v"(p + u * 1024) : "memory", "m0");
      else
        asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(b + u * 1024), "v"(p + u * 1024) : "memory", "m0");
    }
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");         // the group before this one has landed
    p += 8192;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) atomicXor(&sink[blockIdx.x], (uint32_t)(unsigned char)ssm[0]);
}

// mode bit 0: non-temporal loads; bit 1: direct global->LDS loads instead of loads into registers
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int mode, size_t* bytes_read,
                              hipStream_t stream) {
  if (mode & 2) {
    const size_t groups = bytes / kStreamLdsUnit;            // 8 KiB groups per wave
    if (bytes_read) *bytes_read = groups * kStreamLdsUnit;
    if (groups == 0) return hipSuccess;
    static LdsLimit lim0, lim1;
    hipError_t e = (mode & 1) ? raise_lds_limit(lim1, reinterpret_cast<const void*>(&stream_read_lds_kernel<true>), kStreamLdsBytes)
                              : raise_lds_limit(lim0, reinterpret_cast<const void*>(&stream_read_lds_kernel<false>), kStreamLdsBytes);
    if (e != hipSuccess) return e;
    if (mode & 1) stream_read_lds_kernel<true><<<kStreamLdsGrid, kStreamThreads, kStreamLdsBytes, stream>>>((const char*)src, groups, sink);
    else stream_read_lds_kernel<false><<<kStreamLdsGrid, kStreamThreads, kStreamLdsBytes, stream>>>((const char*)src, groups, sink);
    return hipGetLastError();
  }
  if (bytes_read) *bytes_read = bytes;
  if (mode & 1) stream_read_kernel<true><<<kStreamGrid, kStreamThreads, 0, stream>>>((const uint4*)src, bytes / 16, sink);
  else stream_read_kernel<false><<<kStreamGrid, kStreamThreads, 0, stream>>>((const uint4*)src, bytes / 16, sink);
  return hipGetLastError();
}

}  // namespace ekv
