// Cache append for a decoding batch (8 <= T <= 64 tokens) on the matrix cores, first pass.
//   Y = X [W_ke | W_dkv]   (Section 3.2: c = x A^{kv} and the elite key rows W^k_{e,h}; Section 3.1:
//   what a RoPElite model caches), computed transposed, Y^T[n, t] = sum_k W^T[n, k] X^T[k, t]:
//     A (32 x 16 per step) = W^T: the weight tile sits in LDS as stored ([k][n], n contiguous) and
//                            is read transposed (ds_read_b64_tr_b16),
//     B (16 x 32)          = X^T: a lane's eight consecutive k of one token are contiguous in x,
//     D[n, t]              : a lane ends up with ONE token and groups of four consecutive columns.
// The weights are the traffic; they are streamed once, split over column blocks and over the
// contraction dimension so that every compute unit pulls a share.  fp32 partials go to the
// workspace; append_finish sums the contraction splits, rotates and stores.
// The body is a device function: it is the whole of append_skinny_kernel and one of the two roles
// of the decode step's front kernel for batches.
#pragma once
#include "common.hpp"

namespace ekv {

typedef __attribute__((ext_vector_type(8))) __bf16 am_bf16x8;
typedef __attribute__((ext_vector_type(8))) short am_s16x8;
typedef __attribute__((ext_vector_type(4))) short am_s16x4;
typedef __attribute__((ext_vector_type(16))) float am_f32x16;
typedef __attribute__((address_space(3))) am_s16x4 am_lds_s16x4_t;

constexpr int kSkCols = 64;                    // output columns per work-group (two 32-column MFMA tiles)
constexpr int kSkStage = 128;                  // contraction rows per LDS stage
constexpr int kSkRow = kSkCols * 2 + 32;       // bytes of one staged weight row; the padding spreads the
                                               // four rows of a transposed read over all banks

struct AppendSkinnyParams {
  const bf16_t* x;
  int T;
  const bf16_t* W_ke;
  const bf16_t* W_dkv;
  const bf16_t* W_dkv2;
  float* partial;          // [contraction splits][T][N] sums of this call
  int d_ck, d, NE, d_c, kc;
};

constexpr int kSkLds = 2 * kSkStage * kSkRow;   // LDS bytes of the body: two weight stages

// Work-group (bx, by) = (column block, contraction split); waves = (column tile nt, half kh of every
// stage); TT = 32-token tiles (1 or 2); wsm = kSkLds bytes of 16-byte aligned LDS.
template <int TT>
__device__ __forceinline__ void append_skinny_body(const AppendSkinnyParams& P, int bx, int by, char* wsm_base) {
  const bf16_t* __restrict__ x = P.x;
  const int T = P.T;
  const bf16_t* __restrict__ W_ke = P.W_ke;
  const bf16_t* __restrict__ W_dkv = P.W_dkv;
  const bf16_t* __restrict__ W_dkv2 = P.W_dkv2;
  float* __restrict__ partial = P.partial;
  const int d_ck = P.d_ck, d = P.d, NE = P.NE, d_c = P.d_c, kc = P.kc;
  char (*wsm)[kSkStage * kSkRow] = reinterpret_cast<char (*)[kSkStage * kSkRow]>(wsm_base);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nt = wave & 1, kh = wave >> 1;
  const int n32 = lane & 31, hi = lane >> 5, i16 = lane & 15, q16 = lane >> 4;
  const int N = NE + d_c;
  const int n0 = bx * kSkCols;
  const int k_begin = by * kc;
  const int k_end = min(d, k_begin + kc);
  const int nstages = (k_end - k_begin + kSkStage - 1) / kSkStage;

  const bf16_t* wbase;
  int64_t wstride;
  weight_column(n0, NE, d_ck, d_c, W_ke, W_dkv, W_dkv2, &wbase, &wstride);   // a block lies in one matrix

  // weight loader: a stage is 128 rows x 8 pieces of 16 bytes; thread <-> 4 of them
  uint4 wreg[4];
  auto load_w = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = i * 256 + tid, k = k0 + (e >> 3), ch = e & 7;
      wreg[i] = make_uint4(0, 0, 0, 0);
      if (k < k_end) wreg[i] = *reinterpret_cast<const uint4*>(wbase + (int64_t)k * wstride + ch * 8);
    }
  };
  auto store_w = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = i * 256 + tid;
      *reinterpret_cast<uint4*>(&wsm[buf][(e >> 3) * kSkRow + (e & 7) * 16]) = wreg[i];
    }
  };
  // token operand: k-step ks of this wave's stage half, token tile tt
  auto load_x = [&](int k0, am_bf16x8 (&xr)[4][TT]) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int k = k0 + kh * 64 + ks * 16 + hi * 8;
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) {
        const int t = tt * 32 + n32;
        am_s16x8 v = (am_s16x8)(0);
        if (t < T && k < k_end) v = *reinterpret_cast<const am_s16x8*>(x + (int64_t)t * d + k);
        xr[ks][tt] = __builtin_bit_cast(am_bf16x8, v);
      }
    }
  };

  // transposed-read offsets inside a stage: 16-lane group q16 serves rows 8*(q16/2) + 4e + i16/4 of a
  // k-step and columns 32*nt + 16*(q16%2) + 4*(i16%4) ..
  const int tr0 = (kh * 64 + 8 * (q16 >> 1) + (i16 >> 2)) * kSkRow + nt * 64 + 32 * (q16 & 1) + 8 * (i16 & 3);

  am_f32x16 acc[TT];
#pragma unroll
  for (int tt = 0; tt < TT; ++tt) acc[tt] = (am_f32x16)(0.f);

  am_bf16x8 xa[4][TT], xb[4][TT];
  load_w(k_begin);
  load_x(k_begin, xa);
  store_w(0);
  __syncthreads();
  auto compute = [&](int buf, am_bf16x8 (&xr)[4][TT]) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const char* base = &wsm[buf][tr0 + ks * 16 * kSkRow];
      const am_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((am_lds_s16x4_t*)(base));
      const am_s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((am_lds_s16x4_t*)(base + 4 * kSkRow));
      const am_s16x8 a16 = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
      const am_bf16x8 a = __builtin_bit_cast(am_bf16x8, a16);
#pragma unroll
      for (int tt = 0; tt < TT; ++tt) acc[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, xr[ks][tt], acc[tt], 0, 0, 0);
    }
  };
  // two stages per trip so that the register sets of the token operand alternate at compile time
  for (int s = 0; s < nstages; s += 2) {
    const bool more1 = s + 1 < nstages, more2 = s + 2 < nstages;
    if (more1) { load_w(k_begin + (s + 1) * kSkStage); load_x(k_begin + (s + 1) * kSkStage, xb); }
    compute(0, xa);
    if (!more1) break;
    store_w(1);
    __syncthreads();
    if (more2) { load_w(k_begin + (s + 2) * kSkStage); load_x(k_begin + (s + 2) * kSkStage, xa); }
    compute(1, xb);
    if (!more2) break;
    store_w(0);
    __syncthreads();
  }

  // the two stage halves meet in LDS; then one lane owns token t and 4 consecutive columns per group
  __syncthreads();
  float* red = reinterpret_cast<float*>(&wsm[0][0]);          // [nt][tt][16][64]
  if (kh == 1) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[((nt * TT + tt) * 16 + v) * 64 + lane] = acc[tt][v];
  }
  __syncthreads();
  if (kh == 0) {
#pragma unroll
    for (int tt = 0; tt < TT; ++tt) {
      const int t = tt * 32 + n32;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[tt][v] += red[((nt * TT + tt) * 16 + v) * 64 + lane];
      if (t < T) {
        float* prow = partial + ((int64_t)by * T + t) * N + n0 + nt * 32 + 4 * hi;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
          *reinterpret_cast<float4*>(prow + 8 * g4) =
              make_float4(acc[tt][4 * g4], acc[tt][4 * g4 + 1], acc[tt][4 * g4 + 2], acc[tt][4 * g4 + 3]);
      }
    }
  }
}

}  // namespace ekv
