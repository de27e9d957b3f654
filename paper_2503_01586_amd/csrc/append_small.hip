// Cache append for a handful of tokens (the per-step append of a decoding batch): the weights
// [W_ke | W_dkv] are streamed from HBM exactly once, split over column blocks and over the
// contraction dimension so that every compute unit pulls a share; a second small kernel sums
// the contraction splits, applies the selective RoPE and writes the cache rows.
//   (Section 3.1, cache contents of a RoPElite model; Section 3.2, c = x A^{kv}, W^k_{e,h}.)
#include "common.hpp"
#include "launch.hpp"
#include "append_small.hpp"

namespace ekv {

template <int TT>
__global__ __launch_bounds__(kAsThreads) void append_small_kernel(const AppendSmallParams P) {
  extern __shared__ __attribute__((aligned(16))) float xs[];   // [kc][TT]
  append_small_body<TT, 8>(P, blockIdx.x, blockIdx.y, blockIdx.z, xs);
}

// grid (T, column blocks of 256): sum the contraction splits, rotate the elite pairs, store
__global__ __launch_bounds__(256) void append_finish_kernel(
    const float* __restrict__ partial, const int32_t* __restrict__ pos, const int64_t* __restrict__ slot,
    int64_t T, const int32_t* __restrict__ elite_idx, bf16_t* __restrict__ ke_plane,
    bf16_t* __restrict__ c_plane, int64_t plane_rows, int n_h, int d_h, int r, int d_c, int ksplit,
    RopeTable rope) {
  const int NE = 2 * r * n_h, N = NE + d_c;
  const int64_t t = blockIdx.x;
  const int n = blockIdx.y * 256 + threadIdx.x;
  const bool col_ok = n < N;
  float mine = 0.f;
  if (col_ok) {
    // eight independent loads in flight per round; the sum keeps the split order
    for (int s0 = 0; s0 < ksplit; s0 += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (s0 + u < ksplit) ? partial[((int64_t)(s0 + u) * T + t) * N + n] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) mine += v[u];
    }
  }
  const float other = __shfl_xor(mine, 1, kWave);
  if (!col_ok) return;
  const int64_t row = slot[t];
  if (row < 0 || row >= plane_rows) return;
  if (n < NE) {
    const int h = n / (2 * r), j = (n % (2 * r)) >> 1;
    int chunk = elite_idx[h * r + j];
    chunk = min(max(chunk, 0), d_h / 2 - 1);
    float s, c;
    rope_sincos(pos[t], rope.theta[chunk], &s, &c);
    const float o = (n & 1) ? (other * s + mine * c) : (mine * c - other * s);
    st(ke_plane, row * NE + n, o);
  } else {
    st(c_plane, row * d_c + (n - NE), mine);
  }
}

bool append_small_supported(const elitekv_dims& d, int64_t T, int d_ck) {
  if (d.dtype != ELITEKV_BF16 || T > 64) return false;
  const int NE = 2 * d.r * d.n_heads;
  return NE % kAsCols == 0 && d.d_c % kAsCols == 0 && d_ck % kAsCols == 0;
}

// contraction splits so that (column blocks x splits) is about two work-groups per compute unit
static int append_small_ksplit(const elitekv_dims& d) {
  const int blocks = (2 * d.r * d.n_heads + d.d_c) / kAsCols;
  int ks = 1;
  while (ks < 64 && blocks * ks < 512 && (d.d_model + ks * 2 - 1) / (ks * 2) >= 64) ks <<= 1;
  return ks;
}

size_t append_small_workspace(const elitekv_dims& d, int64_t T) {
  return (size_t)append_small_ksplit(d) * (size_t)T * (size_t)(2 * d.r * d.n_heads + d.d_c) * sizeof(float);
}

hipError_t launch_append_small(const AppendArgs& a, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int NE = 2 * d.r * d.n_heads, N = NE + d.d_c;
  const int ks = append_small_ksplit(d);
  int kc = (d.d_model + ks - 1) / ks;
  kc = (kc + 31) / 32 * 32;
  float* partial = (float*)a.ws;
  AppendSmallParams P;
  P.x = (const bf16_t*)a.x; P.T = a.T; P.W_ke = (const bf16_t*)a.W_ke; P.W_dkv = (const bf16_t*)a.W_dkv;
  P.W_dkv2 = (const bf16_t*)a.W_dkv2; P.partial = partial; P.d_ck = a.d_ck; P.d = d.d_model; P.NE = NE; P.d_c = d.d_c;
  P.kc = kc;
  P.W_q = nullptr; P.q_cols = 0; P.x_opart = nullptr; P.x_heads = 0; P.x_chunks = 0; P.x_dh = 1;
#define EKV_AS(TT)                                                                                   \
  append_small_kernel<TT><<<dim3(N / kAsCols, ks, (unsigned)((a.T + TT - 1) / TT)), kAsThreads,      \
                            (size_t)kc * TT * sizeof(float), stream>>>(P)
  if (a.T == 1) EKV_AS(1);
  else if (a.T == 2) EKV_AS(2);
  else if (a.T <= 4) EKV_AS(4);
  else EKV_AS(kAsTokens);
#undef EKV_AS
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_append_finish(a, partial, ks, stream);
}

// out[t, n] = sum over the contraction splits of partial[s][t][n], rounded to the storage type
__global__ __launch_bounds__(256) void dense_finish_kernel(const float* __restrict__ partial, bf16_t* __restrict__ out,
                                                           int ksplit, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over [T, N]
  if (e >= total) return;
  float a = 0.f;
  for (int s0 = 0; s0 < ksplit; s0 += 8) {                      // eight independent loads in flight; split order kept
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = (s0 + u < ksplit) ? partial[(int64_t)(s0 + u) * total + e] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) a += v[u];
  }
  st(out, e, a);
}

hipError_t launch_append_finish(const AppendArgs& a, const float* partial, int ksplit, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int N = 2 * d.r * d.n_heads + d.d_c;
  if (a.dense_out) {
    const int64_t total = a.T * (int64_t)N;
    dense_finish_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(partial, (bf16_t*)a.dense_out, ksplit, total);
    return hipGetLastError();
  }
  append_finish_kernel<<<dim3((unsigned)a.T, (N + 255) / 256), 256, 0, stream>>>(
      partial, a.pos, a.slot, a.T, a.elite_idx, (bf16_t*)a.ke_plane, (bf16_t*)a.c_plane, a.plane_rows,
      d.n_heads, d.head_dim, d.r, d.d_c, ksplit, rope_table(d.rope_base, d.head_dim));
  return hipGetLastError();
}

}  // namespace ekv
