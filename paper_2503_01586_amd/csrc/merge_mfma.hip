// merge_up_mfma: log-sum-exp merge of the sequence splits, normalisation and the W_uv up-projection
// for a decoding batch (Section 2.1, exact softmax identity; Section 3.2, B^v_J; Section 5).
// One work-group per (chunk of 128 latent columns, head, tile of up to 32 batch rows):
//   1. every global load of the work-group is requested up front: the split maxima and sums, the
//      chunk of W_uv[:, head, :] (staged in LDS as stored, [k][j]), and the first sixteen split
//      accumulators of every thread, so the kernel pays one round of memory latency;
//   2. merge weights per row  w_s = exp2(m_s - max m), 1 / sum w_s l_s  (eight lanes per row);
//   3. merged latent of the chunk, thread <-> ((row, slice of the splits), eight columns), slices
//      added in a fixed order and normalised into ubar [rows][128] (fp32);
//   4. o[row, j] += ubar[row, :] W_uv[:, j] on the matrix cores: M = 32 batch rows, one 32-column
//      tile of the head's d_h outputs per wave, K = the chunk's 128 columns in eight steps; ubar goes
//      in as bf16 high part + bf16 remainder (two MFMAs per step: 16 mantissa bits), W_uv is read
//      transposed from LDS (ds_read_b64_tr_b16);
//   5. the chunk's partial outputs go to opart; out_reduce adds the chunks in a fixed order.
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

typedef __attribute__((ext_vector_type(8))) __bf16 mm_bf16x8;
typedef __attribute__((ext_vector_type(8))) short mm_s16x8;
typedef __attribute__((ext_vector_type(4))) short mm_s16x4;
typedef __attribute__((ext_vector_type(16))) float mm_f32x16;
typedef __attribute__((address_space(3))) mm_s16x4 mm_lds_s16x4_t;

constexpr int kMmRows = 32;              // batch rows per work-group (the M of the MFMA)
constexpr int kMmCols = 128;             // latent columns per work-group
constexpr int kMmWeightFloats = 4096;    // most (rows x splits) merge weights a work-group keeps in LDS
constexpr int kMmPre = 16;               // split accumulators per thread requested up front

template <int DH>
struct MergeMfmaLayout {
  static constexpr int WROW = DH * 2 + 32;                 // bytes of a staged W_uv row; the padding spreads
                                                           // the four rows of a transposed read over all banks
  static constexpr int WST = kMmCols * WROW;
  static constexpr int UROW = kMmCols + 4;                 // floats per latent row (padded)
  // merged latents of a tile's rows; with several slices per row (a tile of at most 8 rows, possibly
  // the last one of a batch cut into larger tiles) the 16 per-slice sums sit behind them
  static __host__ __device__ int u_rows(int rows_per_wg) { return rows_per_wg <= 8 ? rows_per_wg + 16 : (rows_per_wg < 24 ? 24 : rows_per_wg); }
  static size_t lds_bytes(int rows, int n_splits) {
    return (size_t)WST + (size_t)u_rows(rows) * UROW * 4 + kMmRows * 4 + (size_t)2 * rows * n_splits * 4;
  }
};

template <int DH>
__global__ __launch_bounds__(256) void merge_up_mfma_kernel(
    const float* __restrict__ part_m, const float* __restrict__ part_l, const bf16_t* __restrict__ part_u,
    const bf16_t* __restrict__ W_uv, float* __restrict__ opart, int B, int n_h, int nhp, int d_u, int n_splits,
    int rows_per_wg) {
  using L = MergeMfmaLayout<DH>;
  constexpr int WROW = L::WROW, UROW = L::UROW;
  extern __shared__ __attribute__((aligned(16))) char msm2[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, head = blockIdx.y, b0 = blockIdx.z * rows_per_wg;
  const int n_chunks = gridDim.x;
  const int rows = min(rows_per_wg, B - b0);                               // 1 .. 32
  char* wst = msm2;                                                        // [128 k][WROW]
  float* ubar = reinterpret_cast<float*>(msm2 + L::WST);                   // [rows][UROW] merged latents
  float* uitem = ubar + rows * UROW;                                       // [16 items][UROW], only when rows <= 8
  float* invl = ubar + L::u_rows(rows_per_wg) * UROW;                      // [32]
  float* wsp = invl + kMmRows;                                             // [rows][n_splits] maxima, then weights
  float* lsp = wsp + rows * n_splits;                                      // [rows][n_splits] split sums
  const int col0 = chunk * kMmCols;

  // ---- (1) all loads.  Small ones first: behind the bulk they would return late.
  //      split maxima and sums of every (row, split) of this head (thread <-> one of the first 256)
  const int ml_n = rows * n_splits;
  float m_first = -INFINITY, l_first = 0.f;
  if (tid < ml_n) {
    const int64_t gi = ((int64_t)b0 * n_splits + tid) * nhp + head;
    l_first = part_l[gi];
    m_first = part_m[gi];
  }
  //      the chunk of W_uv[:, head, :]: coalesced 16-byte loads
  constexpr int CPR = DH / 8;                      // 16-byte pieces per W_uv row
  constexpr int WPASS = kMmCols * CPR / 256;       // loads per thread
  uint4 wld[WPASS];
#pragma unroll
  for (int i = 0; i < WPASS; ++i) {
    const int e = i * 256 + tid, k = e / CPR, c = e % CPR;
    wld[i] = ld16_stream(W_uv + ((int64_t)(col0 + k) * n_h + head) * DH + c * 8);
  }
  //      split accumulators: thread <-> (item g [+16], 16-byte piece cl); item = (row rl, slice sl);
  //      slice sl of SL takes the splits sl, sl + SL, ...
  const int SL = rows <= 8 ? 16 / rows : 1;        // slices per row (several only with at most 8 rows)
  const int n_items = rows * SL;                   // <= 32; above 16 a thread takes two items
  const bool two = n_items > 16;
  const int cl = tid & 15, g = tid >> 4;
  const int64_t sstep = (int64_t)nhp * d_u;
  const bf16_t* ub[2];
  int sl_of[2], rl_of[2];
  bool item_ok[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int item = g + 16 * e;
    item_ok[e] = item < n_items;
    rl_of[e] = item_ok[e] ? item % rows : 0;
    sl_of[e] = item_ok[e] ? item / rows : 0;
    ub[e] = part_u + (((int64_t)(b0 + rl_of[e]) * n_splits) * nhp + head) * (int64_t)d_u + col0 + cl * 8;
  }
  // request p of a thread: with two items they alternate (item p % 2, its split number p / 2),
  // with one item all sixteen requests are its first sixteen splits
  uint4 pre[kMmPre];
#pragma unroll
  for (int p = 0; p < kMmPre; ++p) {
    const int e = two ? (p & 1) : 0, q = two ? (p >> 1) : p;
    const int s = sl_of[e] + q * SL;
    pre[p] = make_uint4(0, 0, 0, 0);
    if (item_ok[e] && s < n_splits) pre[p] = *reinterpret_cast<const uint4*>(ub[e] + s * sstep);
  }
  const int pre_q = two ? kMmPre / 2 : kMmPre;     // splits per item that were requested up front

  // ---- (2) merge weights
  for (int it = tid; it < ml_n; it += 256) {
    float ls = l_first, ms = m_first;
    if (it != tid) {
      const int64_t gi = ((int64_t)b0 * n_splits + it) * nhp + head;
      ls = part_l[gi];
      ms = part_m[gi];
    }
    wsp[it] = (ls > 0.f) ? ms : -INFINITY;                     // an empty split has weight 0
    lsp[it] = ls;
  }
#pragma unroll
  for (int i = 0; i < WPASS; ++i) {
    const int e = i * 256 + tid, k = e / CPR, c = e % CPR;
    *reinterpret_cast<uint4*>(wst + k * WROW + c * 16) = wld[i];
  }
  __syncthreads();
  {                                                            // eight lanes <-> batch row (rows <= 32)
    const int row = tid >> 3, l8 = tid & 7;
    const bool row_ok = row < rows;
    float* wr = wsp + (row_ok ? row : 0) * n_splits;
    const float* lr = lsp + (row_ok ? row : 0) * n_splits;
    float m = -INFINITY;
    if (row_ok)
      for (int s = l8; s < n_splits; s += 8) m = fmaxf(m, wr[s]);
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
    float lsum = 0.f;
    if (row_ok)
      for (int s = l8; s < n_splits; s += 8) {
        const float w = (wr[s] > -INFINITY) ? exp2f(wr[s] - m) : 0.f;
        wr[s] = w;
        lsum += w * lr[s];
      }
#pragma unroll
    for (int o = 1; o < 8; o <<= 1) lsum += __shfl_xor(lsum, o, kWave);   // fixed order: the same tree in every lane
    if (row_ok && l8 == 0) invl[row] = (lsum > 0.f) ? 1.f / lsum : 0.f;
  }
  __syncthreads();

  // ---- (3) merged latent of the chunk
  auto fma8 = [](float (&acc)[8], float w, const uint4& u) {
    const uint32_t uu[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[2 * i] = fmaf(w, __uint_as_float(uu[i] << 16), acc[2 * i]);
      acc[2 * i + 1] = fmaf(w, __uint_as_float(uu[i] & 0xffff0000u), acc[2 * i + 1]);
    }
  };
  float acc[2][8];
#pragma unroll
  for (int e = 0; e < 2; ++e)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[e][i] = 0.f;
#pragma unroll
  for (int p = 0; p < kMmPre; ++p) {
    const int q = two ? (p >> 1) : p;
    if (two && (p & 1)) {
      const int s = sl_of[1] + q * SL;
      if (item_ok[1] && s < n_splits) fma8(acc[1], wsp[rl_of[1] * n_splits + s], pre[p]);
    } else {
      const int s = sl_of[0] + q * SL;
      if (item_ok[0] && s < n_splits) fma8(acc[0], wsp[rl_of[0] * n_splits + s], pre[p]);
    }
  }
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    if (!item_ok[e]) continue;
    const float* wr = wsp + rl_of[e] * n_splits;
    for (int s0 = sl_of[e] + pre_q * SL; s0 < n_splits; s0 += 8 * SL) {        // more splits than were requested up front
      uint4 u[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        u[q] = make_uint4(0, 0, 0, 0);
        if (s0 + q * SL < n_splits) u[q] = *reinterpret_cast<const uint4*>(ub[e] + (s0 + q * SL) * sstep);
      }
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (s0 + q * SL < n_splits) fma8(acc[e], wr[s0 + q * SL], u[q]);
    }
    // one slice per row: the item is the row, normalised in place; otherwise the slice sums wait for the pass below
    const float sc = (SL == 1) ? invl[rl_of[e]] : 1.f;
    float* ur = (SL == 1 ? ubar : uitem) + (g + 16 * e) * UROW + cl * 8;
    *reinterpret_cast<float4*>(ur) = make_float4(acc[e][0] * sc, acc[e][1] * sc, acc[e][2] * sc, acc[e][3] * sc);
    *reinterpret_cast<float4*>(ur + 4) = make_float4(acc[e][4] * sc, acc[e][5] * sc, acc[e][6] * sc, acc[e][7] * sc);
  }
  __syncthreads();
  if (SL > 1) {        // slices of a row added in a fixed order, normalised
    for (int e = tid; e < rows * kMmCols; e += 256) {
      const int rl = e / kMmCols, c = e % kMmCols;
      float a = 0.f;
      for (int sl = 0; sl < SL; ++sl) a += uitem[(sl * rows + rl) * UROW + c];
      ubar[rl * UROW + c] = a * invl[rl];
    }
    __syncthreads();
  }

  // ---- (4) up-projection on the matrix cores: wave <-> 32 of the head's d_h output columns
  if (wave < DH / 32) {
    const int nt = wave;
    const int n32 = lane & 31, hi = lane >> 5, i16 = lane & 15, q16 = lane >> 4;
    // transposed read of W_uv[k][j]: 16-lane group q16 serves rows 8*(q16/2) + i16/4 (+4) of a k-step
    // and columns 32*nt + 16*(q16%2) + 4*(i16%4) ..; the lane ends up with column 32*nt + n32 and the
    // eight k of its half (8*hi ..)
    const int tr0 = (8 * (q16 >> 1) + (i16 >> 2)) * WROW + nt * 64 + 32 * (q16 & 1) + 8 * (i16 & 3);
    mm_f32x16 acc = (mm_f32x16)(0.f);
#pragma unroll
    for (int ks = 0; ks < kMmCols / 16; ++ks) {
      const float* up = ubar + min(n32, rows - 1) * UROW + ks * 16 + hi * 8;   // row n32, columns ks*16 + 8*hi ..
      float4 f0 = *reinterpret_cast<const float4*>(up);
      float4 f1 = *reinterpret_cast<const float4*>(up + 4);
      if (n32 >= rows) f0 = f1 = make_float4(0.f, 0.f, 0.f, 0.f);           // rows past the tile
      const float f[8] = {f0.x, f0.y, f0.z, f0.w, f1.x, f1.y, f1.z, f1.w};
      mm_bf16x8 a_hi, a_lo;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const __bf16 h = (__bf16)f[i];
        a_hi[i] = h;
        a_lo[i] = (__bf16)(f[i] - (float)h);
      }
      const char* base = wst + tr0 + ks * 16 * WROW;
      const mm_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((mm_lds_s16x4_t*)(base));
      const mm_s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((mm_lds_s16x4_t*)(base + 4 * WROW));
      const mm_bf16x8 b = __builtin_bit_cast(mm_bf16x8, __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_hi, b, acc, 0, 0, 0);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_lo, b, acc, 0, 0, 0);
    }
    // D[row, j]: this lane holds column j = 32*nt + n32 and rows 8*g4 + 4*hi + {0..3}
    const int j = nt * 32 + n32;
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int rl = 8 * g4 + 4 * hi + v;
        if (rl < rows) opart[(((int64_t)(b0 + rl) * n_h + head) * n_chunks + chunk) * DH + j] = acc[4 * g4 + v];
      }
  }
}

bool merge_mfma_supported(const elitekv_dims& d, int d_u, int64_t B, int64_t n_splits) {
  if (B < 2 || d_u % kMmCols || (d.head_dim != 128 && d.head_dim != 64)) return false;
  return (B < kMmRows ? B : kMmRows) * n_splits <= kMmWeightFloats;   // (any smaller row tile fits too)
}

template <int DH>
static hipError_t launch_merge_mfma_dh(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  using L = MergeMfmaLayout<DH>;
  const elitekv_dims& d = a.dims;
  // rows per work-group: all of them (up to 32) unless that leaves compute units idle
  int rows = (int)(a.B < kMmRows ? a.B : kMmRows);
  const int64_t groups = (int64_t)(p.d_u / kMmCols) * d.n_heads;
  while (rows > 8 && groups * ((a.B + rows - 1) / rows) < 256) rows = (rows + 1) / 2;
  const size_t sm = L::lds_bytes(rows, p.n_part);
  static LdsLimit lds_limit;
  const hipError_t le = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&merge_up_mfma_kernel<DH>), sm);
  if (le != hipSuccess) return le;
  const dim3 grid(p.d_u / kMmCols, d.n_heads, (unsigned)((a.B + rows - 1) / rows));
  merge_up_mfma_kernel<DH><<<grid, 256, sm, stream>>>(
      (const float*)(a.ws + p.off_m), (const float*)(a.ws + p.off_l), (const bf16_t*)(a.ws + p.off_u),
      (const bf16_t*)a.W_uv, (float*)(a.ws + p.off_opart), (int)a.B, d.n_heads, p.head_groups * 32, p.d_u,
      p.n_part, rows);
  return hipGetLastError();
}

hipError_t launch_merge_mfma(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  return a.dims.head_dim == 128 ? launch_merge_mfma_dh<128>(a, p, stream) : launch_merge_mfma_dh<64>(a, p, stream);
}

}  // namespace ekv
