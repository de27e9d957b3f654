// Cache append on the matrix cores (bf16 in, fp32 accumulate).
//   Y = X [W_ke | W_dkv]   (Section 3.2: c = x A^{kv} and the elite key rows W^k_{e,h}; Section 3.1:
//   what a RoPElite model caches), computed transposed, Y^T[n, t] = sum_k W^T[n, k] X^T[k, t]:
//     A (32 x 16 per step) = W^T: the weight tile sits in LDS as stored ([k][n], n contiguous) and
//                            is read transposed (ds_read_b64_tr_b16),
//     B (16 x 32)          = X^T: a lane's eight consecutive k of one token are contiguous in x,
//     D[n, t]              : a lane ends up with ONE token and groups of four consecutive output
//                            columns, so the (even, odd) pairs that RoPE rotates stay in one lane.
//
// append_skinny: a decoding batch (8 <= T <= 64 tokens).  The weights are the traffic; they are
// streamed once, split over column blocks and over the contraction dimension so that every
// compute unit pulls a share.  fp32 partials go to the workspace; the finish kernel of the
// small-batch path sums the contraction splits, rotates and stores.
#include "common.hpp"
#include "launch.hpp"
#include "append_skinny.hpp"

namespace ekv {

template <int TT>   // 32-token tiles (1 or 2)
__global__ __launch_bounds__(256) void append_skinny_kernel(const AppendSkinnyParams P) {
  __shared__ __attribute__((aligned(16))) char wsm[kSkLds];
  append_skinny_body<TT>(P, blockIdx.x, blockIdx.y, wsm);
}

AppendSkinnyParams make_append_skinny_params(const AppendArgs& a, float* partial, int kc) {
  const elitekv_dims& d = a.dims;
  AppendSkinnyParams P;
  P.x = (const bf16_t*)a.x; P.T = (int)a.T; P.W_ke = (const bf16_t*)a.W_ke; P.W_dkv = (const bf16_t*)a.W_dkv;
  P.W_dkv2 = (const bf16_t*)a.W_dkv2; P.partial = partial; P.d_ck = a.d_ck; P.d = d.d_model;
  P.NE = 2 * d.r * d.n_heads; P.d_c = d.d_c; P.kc = kc;
  return P;
}

bool append_skinny_supported(const elitekv_dims& d, int64_t T, int d_ck) {
  if (d.dtype != ELITEKV_BF16 || T < 8 || T > 64) return false;
  const int NE = 2 * d.r * d.n_heads;
  return NE % kSkCols == 0 && d.d_c % kSkCols == 0 && d_ck % kSkCols == 0 && d.d_model % 8 == 0;
}

// contraction splits: about one work-group per compute unit, whole stages per split
int append_skinny_ksplit(const elitekv_dims& d) {
  const int blocks = (2 * d.r * d.n_heads + d.d_c) / kSkCols;
  int ks = (256 + blocks - 1) / blocks;
  const int max_ks = (d.d_model + kSkStage - 1) / kSkStage;
  if (ks > max_ks) ks = max_ks;
  return ks < 1 ? 1 : ks;
}

int append_skinny_kc(const elitekv_dims& d, int ks) {
  const int kc = (d.d_model + ks - 1) / ks;
  return (kc + kSkStage - 1) / kSkStage * kSkStage;
}

size_t append_skinny_workspace(const elitekv_dims& d, int64_t T) {
  return (size_t)append_skinny_ksplit(d) * (size_t)T * (size_t)(2 * d.r * d.n_heads + d.d_c) * sizeof(float);
}

hipError_t launch_append_skinny(const AppendArgs& a, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int NE = 2 * d.r * d.n_heads, N = NE + d.d_c;
  int ks = append_skinny_ksplit(d);
  const int kc = append_skinny_kc(d, ks);
  ks = (d.d_model + kc - 1) / kc;            // splits that still have rows; never more than planned
  float* partial = (float*)a.ws;
  const dim3 grid(N / kSkCols, ks);
  const AppendSkinnyParams P = make_append_skinny_params(a, partial, kc);
  if (a.T <= 32) append_skinny_kernel<1><<<grid, 256, 0, stream>>>(P);
  else append_skinny_kernel<2><<<grid, 256, 0, stream>>>(P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_append_finish(a, partial, ks, stream);
}

// ---------------------------------------------------------------------------------------------
// append_gemm: prefill-sized appends (T > 64).  A dense contraction bounded by the matrix cores.
// Work-group tile: 128 output columns x (64 * WN) tokens, 2 x 2 waves, each wave 64 columns x
// (32 * WN) tokens = 2 x WN accumulator tiles of 32 x 32.  Both operands go through LDS in
// double-buffered stages of 64 contraction rows (global -> registers -> LDS, the loads of stage
// s+1 in flight while stage s is multiplied).  The epilogue rotates the elite pairs in registers
// (a lane holds one token and four consecutive columns per group) and stores bf16 rows straight
// into the cache planes.
// ---------------------------------------------------------------------------------------------
constexpr int kGmCols = 128;                   // output columns per work-group
constexpr int kGmStage = 64;                   // contraction rows per stage
constexpr int kGmARow = kGmCols * 2 + 32;      // bytes of a staged weight row [k][128 n] (+ bank spread)
constexpr int kGmBRow = kGmStage * 2 + 16;     // bytes of a staged token row [t][64 k] (+ bank spread)

template <int WN>
struct GemmLayout {
  static constexpr int BN = 64 * WN;                          // tokens per work-group
  static constexpr int A_BYTES = kGmStage * kGmARow;
  static constexpr int B_BYTES = BN * kGmBRow;
  static constexpr int STAGE = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static constexpr int NB = BN * 8 / 256;                     // 16-byte token pieces per thread per stage
};

// Epilogue of the GEMM kernels: lane <-> token; registers 4*g4 .. 4*g4+3 of accumulator tile (i, j)
// are the output columns n0 + wm*64 + i*32 + 8*g4 + 4*hi + {0, 1, 2, 3} of token
// t0 + wn*32*WN + j*32 + n32.  Elite pairs are rotated in registers; bf16 rows go to the planes.
template <int WN>
__device__ __forceinline__ void gemm_epilogue(am_f32x16 (&acc)[2][WN], int n0, int64_t t0, int wm, int wn, int n32,
                                              int hi, int64_t T, const int32_t* __restrict__ pos,
                                              const int64_t* __restrict__ slot, const int32_t* __restrict__ elite_idx,
                                              bf16_t* __restrict__ ke_plane, bf16_t* __restrict__ c_plane,
                                              int64_t plane_rows, int n_h, int d_h, int r, int d_c,
                                              const RopeTable& rope) {
  const int NE = 2 * r * n_h;
#pragma unroll
  for (int j = 0; j < WN; ++j) {
    const int64_t t = t0 + wn * 32 * WN + j * 32 + n32;
    if (t >= T) continue;
    const int64_t row = slot ? slot[t] : t;                  // no slot list: rows are written in place
    if (row < 0 || row >= plane_rows) continue;
    const int32_t p = pos ? pos[t] : 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int n = n0 + wm * 64 + i * 32 + 8 * g4 + 4 * hi;
        const bool elite_block = n < NE;                       // uniform over the wave's 64-column half
        float v0 = acc[i][j][4 * g4], v1 = acc[i][j][4 * g4 + 1], v2 = acc[i][j][4 * g4 + 2], v3 = acc[i][j][4 * g4 + 3];
        bf16_t* dst;
        if (elite_block) {
          // two (even, odd) pairs: slots (n % 2r)/2 and the next one of the same head (2r is even and
          // n is a multiple of 4, so a group of four never straddles a head when 2r % 4 == 0; with
          // 2r % 4 == 2 the second pair may belong to the next head: both are looked up separately)
          float sn, cs;
          {
            const int hh = n / (2 * r), jj = (n % (2 * r)) >> 1;
            int ch = elite_idx[hh * r + jj];
            ch = min(max(ch, 0), d_h / 2 - 1);
            rope_sincos_poly(p, rope.theta[ch], &sn, &cs);
            const float a0 = v0 * cs - v1 * sn, a1 = v0 * sn + v1 * cs;
            v0 = a0; v1 = a1;
          }
          {
            const int n2 = n + 2;
            const int hh = n2 / (2 * r), jj = (n2 % (2 * r)) >> 1;
            int ch = elite_idx[hh * r + jj];
            ch = min(max(ch, 0), d_h / 2 - 1);
            rope_sincos_poly(p, rope.theta[ch], &sn, &cs);
            const float a2 = v2 * cs - v3 * sn, a3 = v2 * sn + v3 * cs;
            v2 = a2; v3 = a3;
          }
          dst = ke_plane + row * NE + n;
        } else {
          dst = c_plane + row * d_c + (n - NE);
        }
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16_bits(v0) | ((uint32_t)f32_to_bf16_bits(v1) << 16);
        pk.y = (uint32_t)f32_to_bf16_bits(v2) | ((uint32_t)f32_to_bf16_bits(v3) << 16);
        *reinterpret_cast<uint2*>(dst) = pk;
      }
    }
  }
}

template <int WN>
__global__ __launch_bounds__(256) void append_gemm_kernel(
    const bf16_t* __restrict__ x, const int32_t* __restrict__ pos, const int64_t* __restrict__ slot, int64_t T,
    const bf16_t* __restrict__ W_ke, const bf16_t* __restrict__ W_dkv, const bf16_t* __restrict__ W_dkv2, int d_ck,
    const int32_t* __restrict__ elite_idx, bf16_t* __restrict__ ke_plane, bf16_t* __restrict__ c_plane, int64_t plane_rows, int d, int n_h, int d_h,
    int r, int d_c, RopeTable rope) {
  using L = GemmLayout<WN>;
  extern __shared__ __attribute__((aligned(16))) char gsm[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave & 1, wn = wave >> 1;                    // wave's 64-column half, token half
  const int n32 = lane & 31, hi = lane >> 5, i16 = lane & 15, q16 = lane >> 4;
  const int NE = 2 * r * n_h;
  const int n0 = blockIdx.x * kGmCols;
  const int64_t t0 = (int64_t)blockIdx.y * L::BN;
  const int nstages = (d + kGmStage - 1) / kGmStage;

  // this thread always loads the same 8-column piece (tid % 16) of a weight row; each 64-column
  // half of the block lies in one of the weight matrices
  const bf16_t* wbase;
  int64_t wstride;
  weight_column(n0 + ((tid & 8) ? 64 : 0), NE, d_ck, d_c, W_ke, W_dkv, W_dkv2, &wbase, &wstride);
  wbase += (tid & 7) * 8;

  uint4 areg[4], breg[L::NB];
  auto load_stage = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {               // weights: 64 rows x 16 pieces
      const int e = i * 256 + tid, k = k0 + (e >> 4);
      areg[i] = make_uint4(0, 0, 0, 0);
      if (k < d) areg[i] = *reinterpret_cast<const uint4*>(wbase + (int64_t)k * wstride);
    }
#pragma unroll
    for (int i = 0; i < L::NB; ++i) {           // tokens: BN rows x 8 pieces
      const int e = i * 256 + tid, ch = e & 7;
      const int64_t t = t0 + (e >> 3);
      const int k = k0 + ch * 8;
      breg[i] = make_uint4(0, 0, 0, 0);
      if (t < T && k < d) breg[i] = *reinterpret_cast<const uint4*>(x + t * d + k);
    }
  };
  auto store_stage = [&](int buf) {
    char* As = gsm + buf * L::STAGE;
    char* Bs = As + L::A_BYTES;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = i * 256 + tid;
      *reinterpret_cast<uint4*>(As + (e >> 4) * kGmARow + (e & 15) * 16) = areg[i];
    }
#pragma unroll
    for (int i = 0; i < L::NB; ++i) {
      const int e = i * 256 + tid;
      *reinterpret_cast<uint4*>(Bs + (e >> 3) * kGmBRow + (e & 7) * 16) = breg[i];
    }
  };

  am_f32x16 acc[2][WN];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j) acc[i][j] = (am_f32x16)(0.f);

  // operand offsets inside a stage
  const int a_off = (8 * (q16 >> 1) + (i16 >> 2)) * kGmARow + wm * 128 + 32 * (q16 & 1) + 8 * (i16 & 3);
  const int b_off = (wn * 32 * WN + n32) * kGmBRow + hi * 16;

  auto compute = [&](int buf) {
    const char* As = gsm + buf * L::STAGE;
    const char* Bs = As + L::A_BYTES;
#pragma unroll
    for (int ks = 0; ks < kGmStage / 16; ++ks) {
      am_bf16x8 a[2], b[WN];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const char* base = As + a_off + ks * 16 * kGmARow + i * 64;
        const am_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((am_lds_s16x4_t*)(base));
        const am_s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((am_lds_s16x4_t*)(base + 4 * kGmARow));
        a[i] = __builtin_bit_cast(am_bf16x8, __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
      }
#pragma unroll
      for (int j = 0; j < WN; ++j)
        b[j] = *reinterpret_cast<const am_bf16x8*>(Bs + b_off + j * 32 * kGmBRow + ks * 32);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  load_stage(0);
  store_stage(0);
  __syncthreads();
  for (int s = 0; s < nstages; ++s) {
    const bool more = s + 1 < nstages;
    if (more) load_stage((s + 1) * kGmStage);
    compute(s & 1);
    if (more) store_stage((s + 1) & 1);
    __syncthreads();
  }

  gemm_epilogue<WN>(acc, n0, t0, wm, wn, n32, hi, T, pos, slot, elite_idx, ke_plane, c_plane, plane_rows, n_h, d_h,
                    r, d_c, rope);
}

// ---------------------------------------------------------------------------------------------
// append_gemm_dma: the same GEMM with both operands brought in by direct global->LDS loads into a
// ring of NS stages of 32 contraction rows (no register staging, one barrier per stage, the loads
// of the next NS-2 stages in flight while a stage is multiplied).  CM x WNW waves: CM along the
// 64 CM columns, WNW along the tokens; the widest tiles run eight waves, two per SIMD.  A direct load writes 1 KiB
// (64 lanes x 16 bytes) contiguously, so the LDS layouts are made of 1 KiB blocks:
//   weights  [32 k][64 CM n]: blocks of 8 rows x 128 bytes, 16-byte pieces XOR-swizzled by row
//            (conflict-free transposed reads), block (kb, nb) at (kb*CM + nb) KiB;
//   tokens   [BN t][32 k]:  blocks of 16 rows x 64 bytes, pieces XOR-swizzled by row.
// Needs d_model % 32 == 0 (whole stages); other shapes take append_gemm_kernel.
// ---------------------------------------------------------------------------------------------
constexpr int kGdStage = 32;                    // contraction rows per stage

__device__ __forceinline__ int gd_swz8(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }
// token blocks (16 rows x 64 bytes): a 16-byte read of 16 lanes = 16 rows at one logical piece; the four
// rows r, r+4, r+8, r+12 that share a 64-byte bank window take four different pieces
__device__ __forceinline__ int gd_swz4(int row) { return (row >> 2) & 3; }

__device__ __forceinline__ void gd_dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory", "m0");
}

// WN = 32-token tiles per wave, WNW = waves along the tokens, CM = waves along the columns (64 columns each)
template <int WN, int NS, int WNW, int CM>
struct GemmDmaLayout {
  static constexpr int BN = 32 * WN * WNW;                    // tokens per work-group
  static constexpr int COLS = 64 * CM;                        // output columns per work-group
  static constexpr int NWAVES = CM * WNW;
  static constexpr int A_BYTES = kGdStage * COLS * 2;         // weight stage
  static constexpr int WB = A_BYTES / 1024;                   // ... in 1 KiB blocks (kb = 0..3, nb = 0..CM-1)
  static constexpr int B_BYTES = BN * 64;                     // token stage
  static constexpr int STAGE = A_BYTES + B_BYTES;
  static constexpr int LDS_BYTES = NS * STAGE;
  static constexpr int LOADS = STAGE / 1024;                  // direct loads per stage per work-group
  static constexpr int LPW = LOADS / NWAVES;                  // ... per wave
  static_assert(LOADS % NWAVES == 0, "the loads of a stage are divided evenly among the waves");
  static_assert(LDS_BYTES <= 160 * 1024, "exceeds the LDS of a compute unit");
  static_assert(NS >= 3 && NS <= 12 && (NS - 2) * LPW <= 63, "ring depth outside what the load counter can express");
};

// SPB = stages consumed per barrier (1 or 2).  With 2 the work-group synchronises once per 64 contraction rows:
// half as many barriers and load waits, the operands of the second stage of a pair read while the first is
// multiplied, NS - 2 stages in flight behind the pair.
// KG = groups of waves that split the contraction rows of every stage between them (1 or 2).  With 2 (eight waves on
// a 128 x 128 tile) the waves of a group own 64 x 64 outputs each instead of 64 x 32 and take one of the two 16-row
// k-steps of every stage: a wave then reads 4 KB instead of 6 KB of operands from LDS per four MFMAs (the LDS, not the
// matrix cores, is the busiest unit of this tile: 48 KB read + 16 KB written per stage against 128 B per cycle), and the
// two groups add their halves through LDS once, before the epilogue.
template <int WN, int NS, int WNW, int CM, int SPB, int KG>
__global__ __launch_bounds__(64 * CM * WNW) void append_gemm_dma_kernel(
    const bf16_t* __restrict__ x, const int32_t* __restrict__ pos, const int64_t* __restrict__ slot, int64_t T,
    const bf16_t* __restrict__ W_ke, const bf16_t* __restrict__ W_dkv, const bf16_t* __restrict__ W_dkv2, int d_ck,
    const int32_t* __restrict__ elite_idx, bf16_t* __restrict__ ke_plane, bf16_t* __restrict__ c_plane,
    int64_t plane_rows, int d, int n_h, int d_h, int r, int d_c, RopeTable rope, int64_t x_ld, int x_off2, int d2) {
  using L = GemmDmaLayout<WN, NS, WNW, CM>;
  extern __shared__ __attribute__((aligned(16))) char gsm[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  static_assert(KG == 1 || (KG == 2 && WN == 1 && WNW == 4 && CM == 2), "contraction groups: eight waves on 128 x 128");
  constexpr int WNC = KG * WN;                     // 32-token tiles a wave accumulates
  constexpr int KSN = 2 / KG;                      // k-steps of a stage a wave multiplies
  const int kg = KG == 2 ? wave >> 2 : 0;          // contraction group of this wave
  const int wv = KG == 2 ? wave & 3 : wave;        // wave inside its group
  const int wm = wv % CM, wn = wv / CM;
  const int n32 = lane & 31, hi = lane >> 5, i16 = lane & 15, q16 = lane >> 4;
  const int NE = 2 * r * n_h;
  // Work-groups go to the eight XCDs round-robin by linear index.  All column blocks of one token
  // block are given to the SAME XCD, one after the other, so the token tile is fetched into that
  // XCD's L2 once and re-used by every column block instead of being fetched by eight L2s.
  const int col_blocks = (NE + d_c) / L::COLS;
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int64_t tblock = (int64_t)(seq / col_blocks) * 8 + xcd;
  const int n0 = (seq % col_blocks) * L::COLS;
  const int64_t t0 = tblock * L::BN;
  if (t0 >= T) return;
  // a column block inside W_dkv2 may contract a different column slice of the input rows (d2 > 0; the host
  // makes sure that no block straddles the two matrices then)
  const bool second = d2 > 0 && n0 - NE >= d_ck;
  const bf16_t* xs = second ? x + x_off2 : x;
  const int nstages = (second ? d2 : d) / kGdStage;

  // ---- loader.  Wave w issues loads w*LPW .. w*LPW+LPW-1 of a stage; load index < WB is weight block
  // (kb = idx / CM, nb = idx % CM), the others are token blocks of 16 rows.
  const char* gsrc[L::LPW];      // this lane's global address for the next stage to be requested
  int64_t gstep[L::LPW];         // bytes to advance per stage
#pragma unroll
  for (int u = 0; u < L::LPW; ++u) {
    const int idx = wave * L::LPW + u;
    if (idx < L::WB) {
      const int kb = idx / CM, nb = idx % CM, row = lane >> 3, pc = (lane & 7) ^ gd_swz8(row);
      const bf16_t* wb;
      int64_t ws;
      weight_column(n0 + nb * 64, NE, d_ck, d_c, W_ke, W_dkv, W_dkv2, &wb, &ws);
      gsrc[u] = reinterpret_cast<const char*>(wb + (int64_t)(kb * 8 + row) * ws + pc * 8);
      gstep[u] = (int64_t)kGdStage * ws * 2;
    } else {
      const int tb = idx - L::WB, row = lane >> 2, pc = (lane & 3) ^ gd_swz4(row);
      const int64_t t = min(t0 + tb * 16 + row, T - 1);        // rows past the end repeat the last token
      gsrc[u] = reinterpret_cast<const char*>(xs + t * x_ld + pc * 8);
      gstep[u] = (int64_t)kGdStage * 2;
    }
  }
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)gsm);
  int issue_slot = 0;            // ring slot of the next stage to be requested; stages are requested in order
  auto issue = [&]() {
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds0 + issue_slot * L::STAGE + wave * L::LPW * 1024);
#pragma unroll
    for (int u = 0; u < L::LPW; ++u) {
      gd_dma16(gsrc[u], base + u * 1024);
      gsrc[u] += gstep[u];
    }
    issue_slot = (issue_slot + 1 == NS) ? 0 : issue_slot + 1;
  };

  am_f32x16 acc[2][WNC];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < WNC; ++j) acc[i][j] = (am_f32x16)(0.f);

  // ---- operand read offsets inside a stage
  // weights, transposed read: k rows 8*(q16/2) + 4e + i16/4 of a k-step (block kb = 2*ks + q16/2 ...)
  int a_off[2][2];               // [i: 32-column tile of the wave's 64-column half][e: rows 0-3 | 4-7]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const int r8 = 4 * e + (i16 >> 2);
      const int piece = (i << 2) | ((q16 & 1) << 1) | ((i16 & 3) >> 1);       // 16-byte piece inside the 128-byte row
      a_off[i][e] = ((q16 >> 1) * CM + wm) * 1024 + r8 * 128 + ((piece ^ gd_swz8(r8)) << 4) + ((i16 & 1) << 3);
    }
  // tokens: row n32 of tile j (block 2*(wn*WN + j) + n32/16), piece 2*ks + hi
  int b_off[2];                  // [ks]
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int row = n32 & 15;
    b_off[ks] = L::A_BYTES + (wn * WNC * 2 + (n32 >> 4)) * 1024 + row * 64 + (((2 * ks + hi) ^ gd_swz4(row)) << 4);
  }

  const int b_off_g = kg ? b_off[1] : b_off[0];   // contraction groups: the group's k-step
  // wait until this wave's direct loads have landed except those of the `ahead` most recent stages
  auto wait_loads = [&](int ahead) {
    switch (ahead) {
      case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
#define EKV_WAIT(K) case K: if constexpr (K <= NS - 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(K * L::LPW) : "memory"); break;
      EKV_WAIT(1) EKV_WAIT(2) EKV_WAIT(3) EKV_WAIT(4) EKV_WAIT(5) EKV_WAIT(6) EKV_WAIT(7) EKV_WAIT(8) EKV_WAIT(9) EKV_WAIT(10)
#undef EKV_WAIT
      default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
  };
  // operands of one stage in registers: both 16-row k-steps
  struct StageOps {
    am_bf16x8 a[KSN][2];         // [k-step][32-column tile]
    am_bf16x8 b[KSN][WNC];       // [k-step][32-token tile]
  };
  int read_slot = 0;             // ring slot of the next stage to be read into registers; stages are read in order
  auto read_ops = [&](StageOps& o) {
    const char* st = gsm + read_slot * L::STAGE;
    read_slot = (read_slot + 1 == NS) ? 0 : read_slot + 1;
#pragma unroll
    for (int kq = 0; kq < KSN; ++kq) {
      const int ks = KG == 2 ? kg : kq;            // the group's k-step of the stage
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        // a k-step is two 8-row weight blocks per 64-column block: 2 * CM KiB
        const am_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((am_lds_s16x4_t*)(st + ks * 2048 * CM + a_off[i][0]));
        const am_s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((am_lds_s16x4_t*)(st + ks * 2048 * CM + a_off[i][1]));
        o.a[kq][i] = __builtin_bit_cast(am_bf16x8, __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
      }
#pragma unroll
      for (int j = 0; j < WNC; ++j) o.b[kq][j] = *reinterpret_cast<const am_bf16x8*>(st + (KG == 2 ? b_off_g : b_off[kq]) + j * 2048);
    }
  };
  auto multiply = [&](const StageOps& o) {
#pragma unroll
    for (int ks = 0; ks < KSN; ++ks)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < WNC; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(o.a[ks][i], o.b[ks][j], acc[i][j], 0, 0, 0);
  };

  if constexpr (SPB == 1) {
#pragma unroll
    for (int s = 0; s < NS - 1; ++s)
      if (s < nstages) issue();
    // Ring pipeline: stages s+1 .. s+NS-2 stay in flight while stage s is consumed.  (A version skewed
    // by one stage -- the operands of stage s+1 read into a second register set while stage s is
    // multiplied -- hides the LDS latency and the barrier but keeps one stage less in flight; it
    // measured 5 % slower with eight waves and 20 % slower with four.)
    for (int s = 0; s < nstages; ++s) {
      wait_loads(min(nstages - 1 - s, NS - 2));                   // this wave's loads of stage s have landed
      __syncthreads();             // every wave's part of stage s is in LDS; everyone is done with stage s-1
      if (s + NS - 1 < nstages) issue();                          // into the buffer stage s-1 occupied
      StageOps ops;
      read_ops(ops);
      multiply(ops);
    }
  } else {
    static_assert(SPB == 2 && NS >= 4, "pairs of stages need a ring of at least four");
#pragma unroll
    for (int s = 0; s < NS - 2; ++s)
      if (s < nstages) issue();
    // Stages s and s+1 are consumed behind one barrier; before it NS-4 later stages may still be in flight,
    // after it the two buffers of stages s-2 and s-1 are refilled (NS-2 stages in flight behind the pair).
    for (int s = 0; s < nstages; s += 2) {
      wait_loads(max(min(nstages, s + NS - 2) - (s + 2), 0));     // this wave's loads of stages s, s+1 have landed
      __syncthreads();
      if (s + NS - 2 < nstages) issue();
      if (s + NS - 1 < nstages) issue();
      StageOps o0, o1;
      read_ops(o0);
      if (s + 1 < nstages) read_ops(o1);
      multiply(o0);
      if (s + 1 < nstages) multiply(o1);
    }
  }

  if constexpr (KG == 2) {
    // The two groups hold sums over different contraction rows of the same 64 x 64 outputs.  Group g finishes the
    // g-th 32-token tile: every wave leaves the tile it does not finish in LDS (the ring is free now), adds what its
    // partner of the other group left for it, and runs the epilogue on 64 columns x 32 tokens.
    static_assert(8 * 2 * 16 * 64 * 4 <= L::LDS_BYTES, "the exchange reuses the ring");
    __syncthreads();
    float* xb = reinterpret_cast<float*>(gsm);
    auto put = [&](int writer, const am_f32x16 (&t)[2]) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) xb[((writer * 2 + i) * 16 + v) * 64 + lane] = t[i][v];
    };
    am_f32x16 fin[2][1];
    if (kg == 0) {
      const am_f32x16 other[2] = {acc[0][1], acc[1][1]};
      put(wv * 2 + 0, other);
      fin[0][0] = acc[0][0]; fin[1][0] = acc[1][0];
    } else {
      const am_f32x16 other[2] = {acc[0][0], acc[1][0]};
      put(wv * 2 + 1, other);
      fin[0][0] = acc[0][1]; fin[1][0] = acc[1][1];
    }
    __syncthreads();
    const int partner = wv * 2 + (1 - kg);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) fin[i][0][v] += xb[((partner * 2 + i) * 16 + v) * 64 + lane];
    gemm_epilogue<1>(fin, n0, t0, wm, wn * 2 + kg, n32, hi, T, pos, slot, elite_idx, ke_plane, c_plane, plane_rows, n_h,
                     d_h, r, d_c, rope);
  } else {
    gemm_epilogue<WN>(acc, n0, t0, wm, wn, n32, hi, T, pos, slot, elite_idx, ke_plane, c_plane, plane_rows, n_h, d_h,
                      r, d_c, rope);
  }
}

bool append_gemm_supported(const elitekv_dims& d, int64_t T, int d_ck) {
  if (d.dtype != ELITEKV_BF16 || T <= 64) return false;
  const int NE = 2 * d.r * d.n_heads;
  // 128-column blocks in all, each 64-column half inside one weight matrix
  return (NE + d.d_c) % kGmCols == 0 && NE % 64 == 0 && d.d_c % 64 == 0 && d_ck % 64 == 0 && d.d_model % 8 == 0;
}

template <int WN>
static hipError_t launch_gemm_wn(const AppendArgs& a, hipStream_t stream) {
  using L = GemmLayout<WN>;
  const elitekv_dims& d = a.dims;
  const int N = 2 * d.r * d.n_heads + d.d_c;
  static LdsLimit lds_limit;
  const hipError_t le = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&append_gemm_kernel<WN>), L::LDS_BYTES);
  if (le != hipSuccess) return le;
  const dim3 grid(N / kGmCols, (unsigned)((a.T + L::BN - 1) / L::BN));
  append_gemm_kernel<WN><<<grid, 256, L::LDS_BYTES, stream>>>(
      (const bf16_t*)a.x, a.pos, a.slot, a.T, (const bf16_t*)a.W_ke, (const bf16_t*)a.W_dkv,
      (const bf16_t*)a.W_dkv2, a.d_ck, a.elite_idx, (bf16_t*)a.ke_plane, (bf16_t*)a.c_plane, a.plane_rows, d.d_model, d.n_heads, d.head_dim, d.r, d.d_c,
      rope_table(d.rope_base, d.head_dim));
  return hipGetLastError();
}

template <int WN, int NS, int WNW, int CM, int SPB = 1, int KG = 1>
static hipError_t launch_gemm_dma(const AppendArgs& a, hipStream_t stream) {
  using L = GemmDmaLayout<WN, NS, WNW, CM>;
  const elitekv_dims& d = a.dims;
  const int N = 2 * d.r * d.n_heads + d.d_c;
  static LdsLimit lds_limit;
  const hipError_t le = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&append_gemm_dma_kernel<WN, NS, WNW, CM, SPB, KG>),
                                        L::LDS_BYTES);
  if (le != hipSuccess) return le;
  const int64_t tblocks = (a.T + L::BN - 1) / L::BN;
  const dim3 grid((unsigned)((tblocks + 7) / 8 * 8 * (N / L::COLS)));   // token blocks padded to whole rounds of 8 XCDs
  append_gemm_dma_kernel<WN, NS, WNW, CM, SPB, KG><<<grid, 64 * CM * WNW, L::LDS_BYTES, stream>>>(
      (const bf16_t*)a.x, a.pos, a.slot, a.T, (const bf16_t*)a.W_ke, (const bf16_t*)a.W_dkv,
      (const bf16_t*)a.W_dkv2, a.d_ck, a.elite_idx, (bf16_t*)a.ke_plane, (bf16_t*)a.c_plane, a.plane_rows,
      d.d_model, d.n_heads, d.head_dim, d.r, d.d_c, rope_table(d.rope_base, d.head_dim),
      a.x_ld ? a.x_ld : (int64_t)d.d_model, a.x_off2, a.d2);
  return hipGetLastError();
}

hipError_t launch_append_gemm(const AppendArgs& a, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int64_t col_blocks = (2 * d.r * d.n_heads + d.d_c) / kGmCols;
  // the widest token tile that still gives every compute unit work
  const int split = 2 * d.r * d.n_heads + a.d_ck;              // first column of W_dkv2
  if (a.d2 > 0 || a.x_ld > 0) {
    // column slices of wider rows: only the direct-load kernels take them, with whole stages in both slices
    // and no 128-column block across the two matrices
    if (d.d_model % kGdStage || a.d2 % kGdStage || a.x_off2 % 8 || a.x_ld % 8 || (a.d2 > 0 && split % kGmCols))
      return hipErrorInvalidValue;
  }
  if (d.d_model % kGdStage == 0) {
    const int N = 2 * d.r * d.n_heads + d.d_c;
    // 256 x 256 tiles, one work-group per compute unit: a third fewer operand bytes per flop, 13 % faster
    // than 256 x 128 whenever its work-groups fill the 256 compute units evenly -- one full round, or
    // enough rounds that the ragged last one costs less than that (measured: slower at 260-320
    // work-groups and at 128, faster at 224-256 and from 360 on)
    const int64_t wide = N % 256 == 0 && (a.d2 == 0 || split % 256 == 0) ? (N / 256) * ((a.T + 255) / 256) : 0;
    if (wide >= 352 || (wide >= 224 && wide <= 256)) return launch_gemm_dma<4, 4, 2, 4>(a, stream);
    if (col_blocks * ((a.T + 255) / 256) >= 512) return launch_gemm_dma<2, 6, 4, 2>(a, stream);
    // 128 x 128 tiles: with about one work-group per compute unit eight waves (two per SIMD, 32 tokens x 64
    // columns each) hide a little more of the stage latency than four (595 against 549 TFLOP/s at 2048 tokens
    // x 2048 columns; two ring stages per barrier: 626; the waves as two contraction groups: 688); with more rounds the four-wave form and its larger share of the tile per wave is kept
    const int64_t wgs128 = col_blocks * ((a.T + 127) / 128);
    if (wgs128 >= 256 && wgs128 <= 384) return launch_gemm_dma<1, 6, 4, 2, 2, 2>(a, stream);
    if (wgs128 >= 256) return launch_gemm_dma<2, 4, 2, 2>(a, stream);
    return launch_gemm_dma<1, 6, 2, 2>(a, stream);
  }
  if (col_blocks * ((a.T + 255) / 256) >= 1024) return launch_gemm_wn<4>(a, stream);
  return launch_gemm_wn<1>(a, stream);
}

}  // namespace ekv
