// Cache append for a handful of tokens, first pass: the weights [W_ke | W_dkv] are streamed from HBM
// exactly once, split over column blocks and over the contraction dimension so that every compute
// unit pulls a share; the sums of the contraction splits are added up later (append_finish, or the
// new-token role of the attention kernel in the fused decode step).
//   (Section 3.1, cache contents of a RoPElite model; Section 3.2, c = x A^{kv}, W^k_{e,h}.)
// The body is a device function: it is the whole of append_small_kernel and one of the two roles of
// the decode step's front kernel.
#pragma once
#include "common.hpp"

namespace ekv {

constexpr int kAsThreads = 256;
constexpr int kAsCols = 64;       // output columns per work-group: one 128-byte line of a bf16 weight row
constexpr int kAsTokens = 8;      // most tokens per work-group pass

struct AppendSmallParams {
  const bf16_t* x;
  int64_t T;
  const bf16_t* W_ke;
  const bf16_t* W_dkv;
  const bf16_t* W_dkv2;
  float* partial;         // [contraction splits][T][N] sums of this call
  int d_ck, d, NE, d_c, kc;
  // optional fourth block of output columns behind the cache row: x W_q (q_cols = n_h d_h, a multiple
  // of 64; 0 = none).  N = NE + d_c + q_cols.
  const bf16_t* W_q;
  int q_cols;
  // XS = 1 only: x is not given as bf16 rows but as the column-chunk partials of the attention's
  // up-projection, x[t, h d_h + j] = bf16(sum_c x_opart[t, h, c, j])  (what out_reduce would store)
  const float* x_opart;
  int x_heads, x_chunks, x_dh;
};

// Work-group (bx, by, bz) = (column block, contraction split, token tile); TT = tokens per pass,
// KB = weight rows per thread requested at once (all loads of a work-group are in flight together
// when kc <= 32 KB); XS = where x comes from (see AppendSmallParams); xs = dynamic LDS of kc * TT floats.
template <int TT, int KB, int XS = 0>
__device__ __forceinline__ void append_small_body(const AppendSmallParams& P, int bx, int by, int bz, float* xs) {
  const bf16_t* __restrict__ x = P.x;
  const int64_t T = P.T;
  const bf16_t* __restrict__ W_ke = P.W_ke;
  const bf16_t* __restrict__ W_dkv = P.W_dkv;
  const bf16_t* __restrict__ W_dkv2 = P.W_dkv2;
  float* __restrict__ partial = P.partial;
  const int d_ck = P.d_ck, d = P.d, NE = P.NE, d_c = P.d_c, kc = P.kc;
  __shared__ float red[4][8][TT][8];                    // [wave][column chunk][token][8 cols]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int rg = lane >> 3, cchunk = lane & 7;
  const int N = NE + d_c + P.q_cols;
  const int n0 = bx * kAsCols;
  const int k0 = by * kc;
  const int64_t t0 = (int64_t)bz * TT;

  const bf16_t* wbase;
  int64_t wstride;
  if (n0 < NE + d_c) {
    weight_column(n0, NE, d_ck, d_c, W_ke, W_dkv, W_dkv2, &wbase, &wstride);   // a block lies in one matrix
  } else {
    wbase = P.W_q + (n0 - NE - d_c);
    wstride = P.q_cols;
  }
  wbase += cchunk * 8;

  // the weight rows of the first batch are requested before anything else: they are the long pole
  constexpr int kBatch = KB;
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
    for (int tt = 0; tt < TT; ++tt) {
      const bool ok = kk < kc && t0 + tt < T && k0 + kk < d;
      if (XS == 0) {
        xv[tt] = ok ? ld(x, (t0 + tt) * d + k0 + kk) : 0.f;
      } else {
        float v = 0.f;
        if (ok) {
          const int k = k0 + kk, h = k / P.x_dh, j = k - h * P.x_dh;
          const float* op = P.x_opart + (((t0 + tt) * P.x_heads + h) * (int64_t)P.x_chunks) * P.x_dh + j;
          for (int c = 0; c < P.x_chunks; ++c) v += op[(int64_t)c * P.x_dh];
          v = bf16_bits_to_f32(f32_to_bf16_bits(v));
        }
        xv[tt] = v;
      }
    }
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
      partial[((int64_t)by * T + t) * N + n0 + c] = v;
    }
  }
}

}  // namespace ekv
