// Generic (any shape, fp32 or bf16 storage, fp32 VALU arithmetic) cache append:
//   Y = X [W_ke | W_dkv]; the 2r*n_h elite columns are rotated by pos * theta_{I_h[j]} and written
//   to the elite-key plane, the d_c latent columns go to the latent plane
//   (Section 3.1, cache contents of a RoPElite model; Section 3.2, c = x A^{kv}, W^k_{e,h}).
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

constexpr int kApThreads = 256;
constexpr int kApTokens = 8;     // tokens per work-group
constexpr int kApK = 128;        // contraction chunk staged in LDS

template <typename T>
__global__ __launch_bounds__(kApThreads) void append_generic_kernel(
    const T* __restrict__ x, const int32_t* __restrict__ pos, const int64_t* __restrict__ slot,
    int64_t T_tokens, const T* __restrict__ W_ke, const T* __restrict__ W_dkv, const T* __restrict__ W_dkv2, int d_ck,
    const int32_t* __restrict__ elite_idx, T* __restrict__ ke_plane, T* __restrict__ c_plane,
    int64_t plane_rows, int d, int n_h, int d_h, int r, int d_c, RopeTable rope) {
  __shared__ float xs[kApTokens][kApK];
  const int tid = threadIdx.x;
  const int NE = 2 * r * n_h;
  const int N = NE + d_c;
  const int n = blockIdx.y * kApThreads + tid;
  const int64_t t0 = (int64_t)blockIdx.x * kApTokens;
  const bool col_ok = n < N;
  const T* wcol;
  int64_t wstride;
  weight_column(col_ok ? n : 0, NE, d_ck, d_c, W_ke, W_dkv, W_dkv2, &wcol, &wstride);

  float acc[kApTokens];
#pragma unroll
  for (int i = 0; i < kApTokens; ++i) acc[i] = 0.f;

  for (int k0 = 0; k0 < d; k0 += kApK) {
    for (int e = tid; e < kApTokens * kApK; e += kApThreads) {
      const int tt = e / kApK, kk = e % kApK;
      const int64_t t = t0 + tt;
      xs[tt][kk] = (t < T_tokens && k0 + kk < d) ? ld(x, t * d + k0 + kk) : 0.f;
    }
    __syncthreads();
    if (col_ok) {
      const int kmax = min(kApK, d - k0);
      for (int kk = 0; kk < kmax; ++kk) {
        const float w = ld(wcol, (int64_t)(k0 + kk) * wstride);
#pragma unroll
        for (int tt = 0; tt < kApTokens; ++tt) acc[tt] = fmaf(xs[tt][kk], w, acc[tt]);
      }
    }
    __syncthreads();
  }

  // epilogue.  Elite columns come in (lane 0, lane 1) pairs held by neighbouring threads.
  const bool is_elite = n < NE;
  int chunk = 0;
  if (is_elite) {
    const int h = n / (2 * r), j = (n % (2 * r)) >> 1;
    chunk = elite_idx[h * r + j];
    chunk = min(max(chunk, 0), d_h / 2 - 1);
  }
  const double theta = is_elite ? rope.theta[chunk] : 0.0;
#pragma unroll
  for (int tt = 0; tt < kApTokens; ++tt) {
    const int64_t t = t0 + tt;
    const float mine = acc[tt];
    const float other = __shfl_xor(mine, 1, kWave);
    if (t >= T_tokens || !col_ok) continue;
    const int64_t row = slot[t];
    if (row < 0 || row >= plane_rows) continue;
    if (is_elite) {
      float s, c;
      rope_sincos(pos[t], theta, &s, &c);
      // (u, v) -> (u c - v s, u s + v c)
      const float o = (n & 1) ? (other * s + mine * c) : (mine * c - other * s);
      st(ke_plane, row * NE + n, o);
    } else {
      st(c_plane, row * d_c + (n - NE), mine);
    }
  }
}

hipError_t launch_append_generic(const AppendArgs& a, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int N = 2 * d.r * d.n_heads + d.d_c;
  const dim3 grid((unsigned)((a.T + kApTokens - 1) / kApTokens), (N + kApThreads - 1) / kApThreads);
  if (d.dtype == ELITEKV_FP32) {
    append_generic_kernel<float><<<grid, kApThreads, 0, stream>>>(
        (const float*)a.x, a.pos, a.slot, a.T, (const float*)a.W_ke, (const float*)a.W_dkv,
        (const float*)a.W_dkv2, a.d_ck, a.elite_idx, (float*)a.ke_plane, (float*)a.c_plane, a.plane_rows, d.d_model, d.n_heads,
        d.head_dim, d.r, d.d_c, rope_table(d.rope_base, d.head_dim));
  } else {
    append_generic_kernel<bf16_t><<<grid, kApThreads, 0, stream>>>(
        (const bf16_t*)a.x, a.pos, a.slot, a.T, (const bf16_t*)a.W_ke, (const bf16_t*)a.W_dkv,
        (const bf16_t*)a.W_dkv2, a.d_ck, a.elite_idx, (bf16_t*)a.ke_plane, (bf16_t*)a.c_plane, a.plane_rows, d.d_model, d.n_heads,
        d.head_dim, d.r, d.d_c, rope_table(d.rope_base, d.head_dim));
  }
  return hipGetLastError();
}

}  // namespace ekv
