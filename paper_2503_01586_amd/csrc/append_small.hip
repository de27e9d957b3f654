// Cache append for a handful of tokens (the per-step append of a decoding batch): the weights
// [W_ke | W_dkv] are streamed from HBM exactly once, split over column blocks and over the
// contraction dimension so that every compute unit pulls a share; a second small kernel sums
// the contraction splits, applies the selective RoPE and writes the cache rows.
//   (Section 3.1, cache contents of a RoPElite model; Section 3.2, c = x A^{kv}, W^k_{e,h}.)
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

constexpr int kAsThreads = 256;
constexpr int kAsCols = 64;       // output columns per work-group: one 128-byte line of a bf16 weight row
constexpr int kAsTokens = 8;      // most tokens per work-group pass

// grid (column blocks, contraction splits, token tiles); TT = tokens per work-group pass
template <int TT>
__global__ __launch_bounds__(kAsThreads) void append_small_kernel(
    const bf16_t* __restrict__ x, int64_t T, const bf16_t* __restrict__ W_ke,
    const bf16_t* __restrict__ W_dkv, const bf16_t* __restrict__ W_dkv2, int d_ck, float* __restrict__ partial,
    int d, int NE, int d_c, int kc) {
  extern __shared__ __attribute__((aligned(16))) float xs[];   // [kc][TT]
  __shared__ float red[4][8][TT][8];                    // [wave][column chunk][token][8 cols]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = lane >> 3, cchunk = lane & 7;
  const int N = NE + d_c;
  const int n0 = blockIdx.x * kAsCols;
  const int k0 = blockIdx.y * kc;
  const int64_t t0 = (int64_t)blockIdx.z * TT;

  const bf16_t* wbase;
  int64_t wstride;
  weight_column(n0, NE, d_ck, d_c, W_ke, W_dkv, W_dkv2, &wbase, &wstride);   // a block lies in one matrix
  wbase += cchunk * 8;

  // the weight rows of the first batch are requested before anything else: they are the long pole
  constexpr int kBatch = 8;
  const int steps = kc / 32;
  uint4 wq[kBatch];
  auto load_batch = [&](int s0) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const int k = k0 + (s0 + u) * 32 + wave * 8 + rg;
      wq[u] = make_uint4(0, 0, 0, 0);
      if (s0 + u < steps && k < d) wq[u] = *reinterpret_cast<const uint4*>(wbase + (int64_t)k * wstride);
    }
  };
  // stage x[t0 .. t0+TT, k0 .. k0+kc) as xs[k][token]: per pass a thread takes one k for all tokens.
  // The first pass of these small loads is requested ahead of the weight rows (behind 16 MB of
  // queued weight traffic they would return late); the weight rows follow at once.
  auto load_x = [&](int kk, float (&xv)[TT]) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
      xv[tt] = (kk < kc && t0 + tt < T && k0 + kk < d) ? ld(x, (t0 + tt) * d + k0 + kk) : 0.f;
  };
  float xfirst[TT];
  load_x(tid, xfirst);
  load_batch(0);
  for (int kk = tid; kk < kc; kk += kAsThreads) {
    float xv[TT];
    if (kk == tid) {
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) xv[tt] = xfirst[tt];
    } else {
      load_x(kk, xv);
    }
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) xs[kk * TT + tt] = xv[tt];
  }
  __syncthreads();

  float acc[TT][8];
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[t][i] = 0.f;

  for (int s0 = 0; s0 < steps; s0 += kBatch) {
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      if (s0 + u < steps) {
        const int kk = (s0 + u) * 32 + wave * 8 + rg;
        const uint32_t ww[4] = {wq[u].x, wq[u].y, wq[u].z, wq[u].w};
        float w[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          w[2 * i] = __uint_as_float(ww[i] << 16);
          w[2 * i + 1] = __uint_as_float(ww[i] & 0xffff0000u);
        }
        float xv[TT];
#pragma unroll
        for (int t = 0; t < TT; ++t) xv[t] = xs[kk * TT + t];
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
          for (int i = 0; i < 8; ++i) acc[t][i] = fmaf(xv[t], w[i], acc[t][i]);
      }
    }
    if (s0 + kBatch < steps) load_batch(s0 + kBatch);
  }
  // sum over the 8 row groups of the wave, then over the 4 waves
#pragma unroll
  for (int t = 0; t < TT; ++t)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float v = acc[t][i];
      v += __shfl_xor(v, 8, kWave);
      v += __shfl_xor(v, 16, kWave);
      v += __shfl_xor(v, 32, kWave);
      acc[t][i] = v;
    }
  if (rg == 0) {
#pragma unroll
    for (int t = 0; t < TT; ++t)
#pragma unroll
      for (int i = 0; i < 8; ++i) red[wave][cchunk][t][i] = acc[t][i];
  }
  __syncthreads();
  for (int e = tid; e < TT * kAsCols; e += kAsThreads) {
    const int tt = e / kAsCols, c = e % kAsCols;
    const int64_t t = t0 + tt;
    if (t < T) {
      const float v = red[0][c >> 3][tt][c & 7] + red[1][c >> 3][tt][c & 7] + red[2][c >> 3][tt][c & 7] +
                      red[3][c >> 3][tt][c & 7];
      partial[((int64_t)blockIdx.y * T + t) * N + n0 + c] = v;
    }
  }
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
#define EKV_AS(TT)                                                                                   \
  append_small_kernel<TT><<<dim3(N / kAsCols, ks, (unsigned)((a.T + TT - 1) / TT)), kAsThreads,      \
                            (size_t)kc * TT * sizeof(float), stream>>>(                             \
      (const bf16_t*)a.x, a.T, (const bf16_t*)a.W_ke, (const bf16_t*)a.W_dkv, (const bf16_t*)a.W_dkv2, a.d_ck,  \
      partial, d.d_model, NE, d.d_c, kc)
  if (a.T == 1) EKV_AS(1);
  else if (a.T == 2) EKV_AS(2);
  else if (a.T <= 4) EKV_AS(4);
  else EKV_AS(kAsTokens);
#undef EKV_AS
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_append_finish(a, partial, ks, stream);
}

hipError_t launch_append_finish(const AppendArgs& a, const float* partial, int ksplit, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int N = 2 * d.r * d.n_heads + d.d_c;
  append_finish_kernel<<<dim3((unsigned)a.T, (N + 255) / 256), 256, 0, stream>>>(
      partial, a.pos, a.slot, a.T, a.elite_idx, (bf16_t*)a.ke_plane, (bf16_t*)a.c_plane, a.plane_rows,
      d.n_heads, d.head_dim, d.r, d.d_c, ksplit, make_rope_table(d.rope_base, d.head_dim));
  return hipGetLastError();
}

}  // namespace ekv
