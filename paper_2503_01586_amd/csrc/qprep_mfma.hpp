// Query preparation of the decode step for a batch (eight rows and up), on the matrix cores.
// The body is a device function: it is the whole of qprep_mfma_kernel and one of the two roles of
// the decode step's front kernel for batches.
#pragma once
#include "common.hpp"
#include "qprep_rows.hpp"   // QprepRowsParams

namespace ekv {

// ---------------------------------------------------------------------------------------------
// qprep_mfma: the same absorption for a decoding batch, on the matrix cores.  Per head h it is the
// small GEMM  qt[b, k] = sum_j W_uk[k, h, j] q_ne[b, j]  with the batch as the N dimension:
//   A (32 x 16 per step) = 32 rows of W_uk[:, h, :], read straight from memory (a lane's eight
//                          consecutive j are contiguous), kept in registers for every batch tile
//   B (16 x 32)          = the compacted non-elite query of 32 batch rows, from LDS
// One wave per 32 latent columns, four waves (128 columns) per work-group, all batch rows: W_uk is
// read once.  Work-groups of the first column block also write the rotated elite query.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 qp_bf16x8;
typedef __attribute__((ext_vector_type(8))) short qp_s16x8;
typedef __attribute__((ext_vector_type(16))) float qp_f32x16;
constexpr int kQmRows = 64;     // batch rows staged in LDS per pass

// LDS bytes of the body: the compacted non-elite query of kQmRows batch rows + the chunk list
inline size_t qprep_mfma_lds(int head_dim, int r) { return (size_t)kQmRows * (head_dim - 2 * r + 8) * 2 + 64 * sizeof(int); }

// bx = block of 128 latent columns, by = head; qms = qprep_mfma_lds(...) bytes of 16-byte aligned LDS;
// KS = contraction steps of 16 non-elite dims (the tail is zero-filled).  P.sincos (optional) is written by the
// work-groups that rotate the elite query.
template <int KS>
__device__ __forceinline__ void qprep_mfma_body(const QprepRowsParams& P, const RopeTable& rope, int bx, int by,
                                                char* qms) {
  const bf16_t* __restrict__ q = P.q;
  const int32_t* __restrict__ q_pos = P.q_pos;
  const bf16_t* __restrict__ W_uk = P.W_uk;
  const int32_t* __restrict__ elite_idx = P.elite_idx;
  float* __restrict__ qe = P.qe;
  bf16_t* __restrict__ qt = P.qt;
  const int B = P.B, n_h = P.n_h, d_h = P.d_h, r = P.r, d_c = P.d_c;
  const float scale_log2e = P.scale_log2e;
  const int nd = d_h - 2 * r, half = d_h / 2, ndp = nd + 8;
  uint16_t* qne = reinterpret_cast<uint16_t*>(qms);                       // [kQmRows][ndp] bf16 bits
  int* ne = reinterpret_cast<int*>(qms + (size_t)kQmRows * ndp * 2);      // [64] non-elite chunks, ascending
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = by;
  const int k0 = bx * 128 + wave * 32;
  const int n32 = lane & 31, hi = lane >> 5;

  // this lane's pieces of W_uk row (k0 + n32, h): chunks 2*ks + hi
  qp_bf16x8 A[KS];
  {
    const bf16_t* wrow = W_uk + ((int64_t)(k0 + n32) * n_h + h) * nd;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int c = 2 * ks + hi;
      qp_s16x8 v = (qp_s16x8)(0);
      if (c * 8 < nd) v = *reinterpret_cast<const qp_s16x8*>(wrow + c * 8);
      A[ks] = __builtin_bit_cast(qp_bf16x8, v);
    }
  }
  // the non-elite chunks of this head in ascending order
  if (wave == 0) {
    bool elite = false;
    for (int j = 0; j < r; ++j) elite |= (elite_idx[h * r + j] == lane);
    const bool live = lane < half && !elite;
    const uint64_t mask = __ballot(live);
    if (live) ne[__popcll(mask & ((1ull << lane) - 1ull))] = lane;
  }
  __syncthreads();
  const uint32_t* q32 = reinterpret_cast<const uint32_t*>(q);
  const int my_chunk = (lane < nd / 2) ? ne[lane] : 0;

  for (int b0 = 0; b0 < B; b0 += kQmRows) {
    const int rows = min(kQmRows, B - b0);
    if (b0 > 0) __syncthreads();                        // the previous rows have been consumed
    // compacted non-elite query: lane <-> chunk position, wave <-> rows wave, wave + 4, ...
    for (int bl = wave; bl < kQmRows; bl += 4) {
      uint32_t* dst = reinterpret_cast<uint32_t*>(qne + bl * ndp);
      if (lane < nd / 2) dst[lane] = (bl < rows) ? q32[((int64_t)(b0 + bl) * n_h + h) * half + my_chunk] : 0u;
      else if (lane < nd / 2 + 4) dst[lane] = 0u;       // the padding doubles as the zero tail of K
    }
    if (bx == 0) {                              // rotated elite query of these rows
      for (int e = tid; e < rows * r; e += 256) {
        const int j = e % r, b = b0 + e / r;
        int i = elite_idx[h * r + j];
        i = min(max(i, 0), half - 1);
        float sn, cs;
        rope_sincos(q_pos[b], rope.theta[i], &sn, &cs);
        const bf16_t* qrow = q + ((int64_t)b * n_h + h) * d_h;
        const float u = ld(qrow, 2 * i), v = ld(qrow, 2 * i + 1);
        float* o = qe + ((int64_t)b * n_h + h) * 2 * r;
        o[2 * j] = (u * cs - v * sn) * scale_log2e;
        o[2 * j + 1] = (u * sn + v * cs) * scale_log2e;
        if (P.sincos) P.sincos[((int64_t)b * n_h + h) * r + j] = make_float2(sn, cs);
      }
    }
    __syncthreads();
    for (int bt = 0; bt < rows; bt += 32) {
      qp_f32x16 acc = (qp_f32x16)(0.f);
      const uint16_t* brow = qne + (bt + n32) * ndp + hi * 8;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const qp_bf16x8 bop = *reinterpret_cast<const qp_bf16x8*>(brow + ks * 16);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[ks], bop, acc, 0, 0, 0);
      }
      // D[k, b]: this lane holds batch row bt + n32 and latent columns k0 + 8*g4 + 4*hi + {0..3}.  The two
      // lanes of a batch row (hi = 0, 1) hold the two halves of each 8-column lane slot of the operand
      // layout (qt_packed_index): the upper half is fetched from lane + 32 and the slot stored as 16 bytes.
      const int b = b0 + bt + n32;
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16_bits(acc[4 * g4] * scale_log2e) |
               ((uint32_t)f32_to_bf16_bits(acc[4 * g4 + 1] * scale_log2e) << 16);
        pk.y = (uint32_t)f32_to_bf16_bits(acc[4 * g4 + 2] * scale_log2e) |
               ((uint32_t)f32_to_bf16_bits(acc[4 * g4 + 3] * scale_log2e) << 16);
        uint4 slot;
        slot.x = pk.x; slot.y = pk.y;
        slot.z = __shfl_xor(pk.x, 32, kWave);
        slot.w = __shfl_xor(pk.y, 32, kWave);
        if (b < B && hi == 0)
          *reinterpret_cast<uint4*>(qt + qt_packed_index(b, h, k0 + 8 * g4, P.head_groups, d_c, P.q_slice)) = slot;
      }
    }
  }
}

}  // namespace ekv
