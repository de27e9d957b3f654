// Query preparation of the decode step for fewer than eight batch rows: the rotated elite query and
// W_uk absorbed into the rest of the query (Section 3.1 score equation, first sum; Section 5,
// absorption of B^k).  The body is a device function: it is the whole of qprep_rows_kernel, and one
// of the two roles of the decode step's front kernel.
#pragma once
#include "common.hpp"

namespace ekv {

// ---------------------------------------------------------------------------------------------
// qprep_rows.  W_uk [d_c, n_h, nd] is a row-major matrix with one row of nd = d_h - 2r weights
// per (latent column k, head h); thread <-> row, so a work-group streams 256 consecutive rows.
//   qt[b, h, k] = scale * sum_j q[b, h, nonelite_j] * W_uk[k, h, j]
// The rows of a work-group are one contiguous piece of memory; it is brought into LDS by direct
// global->LDS loads of consecutive 16-byte pieces (fully coalesced; a thread reading its own
// 224-byte row from memory touches a different cache line in every lane) and laid out with an odd
// row pitch so that the threads' 16-byte reads of their rows are bank-conflict free.
// The compacted non-elite query of the batch tile sits in LDS (bf16, as given).
// ---------------------------------------------------------------------------------------------
constexpr int kQpThreads = 256;
constexpr int kQpBatchTile = 8;

struct QprepRowsParams {
  const bf16_t* q;
  const int32_t* q_pos;
  const bf16_t* W_uk;
  const int32_t* elite_idx;
  float* qe;
  bf16_t* qt;
  float2* sincos;         // optional [B][n_h * r]: (sin, cos) of every rotated chunk, for the key of the same position
  int B, n_h, d_h, r, d_c;
  int q_slice, head_groups;   // layout of qt (qt_packed_index): the attention kernel's column slice per wave, groups of 32 heads
  float scale_log2e;
};

// LDS bytes of the body for a batch tile of bt rows: query staging + elite masks + weight image
inline size_t qprep_rows_lds(int n_heads, int head_dim, int r, int bt) {
  const int nd = head_dim - 2 * r;
  return (((size_t)bt * n_heads * (nd + 8) * 2 + (size_t)n_heads * 8 + 15) & ~(size_t)15) +
         (size_t)kQpThreads * ((nd / 8) | 1) * 16;
}

// BT = batch rows handled per work-group pass (1, 2, 4 or 8), a template parameter so that the
// single-row decode does no work for absent rows.  bx = index of this work-group among the nbx of
// the query preparation (the last one rotates the elite query), by = batch tile, qsm = LDS.
template <int BT>
__device__ __forceinline__ void qprep_rows_body(const QprepRowsParams& P, const RopeTable& rope, int bx, int nbx,
                                                int by, char* qsm) {
  const bf16_t* __restrict__ q = P.q;
  const int32_t* __restrict__ q_pos = P.q_pos;
  const bf16_t* __restrict__ W_uk = P.W_uk;
  const int32_t* __restrict__ elite_idx = P.elite_idx;
  float* __restrict__ qe = P.qe;
  bf16_t* __restrict__ qt = P.qt;
  const int B = P.B, n_h = P.n_h, d_h = P.d_h, r = P.r, d_c = P.d_c;
  const float scale_log2e = P.scale_log2e;
  const int nd = d_h - 2 * r;
  const int ndp = nd + 8;                                  // padded row: breaks the LDS bank period
  const int half = d_h / 2;                                // <= 64 (checked on the host)
  uint16_t* qne = reinterpret_cast<uint16_t*>(qsm);        // [BT][n_h][ndp] bf16 bits
  uint64_t* emask = reinterpret_cast<uint64_t*>(qsm + (size_t)BT * n_h * ndp * 2);   // [n_h]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = by * BT;
  const int bt_n = min(BT, B - b0);

  // The rotated elite query is the work of one extra work-group (the last one), so that its chain of
  // dependent loads and the sin/cos do not lengthen a work-group that also streams weight rows.
  if (bx == nbx - 1) {
    for (int e = tid; e < bt_n * n_h * r; e += kQpThreads) {
      const int j = e % r, h = (e / r) % n_h, b = b0 + e / (r * n_h);
      int i = elite_idx[h * r + j];
      i = min(max(i, 0), half - 1);
      float s, c;
      rope_sincos(q_pos[b], rope.theta[i], &s, &c);
      const bf16_t* qrow = q + ((int64_t)b * n_h + h) * d_h;
      const float u = ld(qrow, 2 * i), v = ld(qrow, 2 * i + 1);
      float* o = qe + ((int64_t)b * n_h + h) * 2 * r;
      o[2 * j] = (u * c - v * s) * scale_log2e;
      o[2 * j + 1] = (u * s + v * c) * scale_log2e;
      if (P.sincos) P.sincos[((int64_t)b * n_h + h) * r + j] = make_float2(s, c);
    }
    return;
  }
  // this thread's weight row (latent column k, head h) is requested before anything else
  const int64_t row = (int64_t)bx * kQpThreads + tid;
  const bool row_ok = row < (int64_t)d_c * n_h;
  const int nchunk = nd / 8;                               // 16-byte pieces per row, <= 16
  const int pitch = nchunk | 1;                            // LDS row pitch in pieces (odd)
  char* wl = qsm + (((size_t)BT * n_h * ndp * 2 + (size_t)n_h * 8 + 15) & ~(size_t)15);   // [256][pitch] pieces
  // The small loads the prologue depends on (elite indices, the first pass of query rows) are
  // requested BEFORE the weight image: behind 11 MB of queued weight traffic they would return late.
  const uint32_t* q32 = reinterpret_cast<const uint32_t*>(q);
  const int e_first = (tid < n_h * r) ? elite_idx[tid] : -1;
  auto load_q = [&](int h0, uint32_t (&qv)[8][BT]) {       // eight heads per pass, all loads issued together
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int h = h0 + i * (kQpThreads / 64);
#pragma unroll
      for (int bt = 0; bt < BT; ++bt)
        qv[i][bt] = (h < n_h && bt < bt_n && lane < half) ? q32[((int64_t)(b0 + bt) * n_h + h) * half + lane] : 0u;
    }
  };
  uint32_t qv[8][BT];
  load_q(wave, qv);
  {
    // piece m = 64 j + lane of the LDS image is (row m / pitch, piece m % pitch); wave w issues j = w, w+4, ..
    const uint32_t lbase = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)wl);
    const int64_t rows_total = (int64_t)d_c * n_h;
    const int64_t r0 = (int64_t)bx * kQpThreads;
    const int total = kQpThreads * pitch;                  // pieces in the image
    int m = wave * 64 + lane;
    int rr = m / pitch, cc = m % pitch;
    const int dq = 256 / pitch, dr = 256 % pitch;
    for (int j = wave; j * 64 < total; j += 4) {
      const bool real = cc < nchunk && r0 + rr < rows_total && m < total;
      const bf16_t* src = W_uk + (real ? (r0 + rr) * nd + cc * 8 : 0);        // padding pieces fetch piece 0
      asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
                   :
                   : "s"(__builtin_amdgcn_readfirstlane(lbase + j * 1024)), "v"(src)
                   : "memory", "m0");
      m += 256; rr += dq; cc += dr;
      if (cc >= pitch) { cc -= pitch; ++rr; }
    }
  }

  // elite mask per head, then the compacted non-elite query: wave <-> head, lane <-> chunk; a
  // ballot gives every non-elite chunk its position
  for (int h = tid; h < n_h; h += kQpThreads) emask[h] = 0ull;
  __syncthreads();
  for (int e = tid; e < n_h * r; e += kQpThreads) {
    const int i = (e == tid) ? e_first : elite_idx[e];
    if (i >= 0 && i < half) atomicOr(reinterpret_cast<unsigned long long*>(&emask[e / r]), 1ull << i);
  }
  __syncthreads();
  for (int h0 = wave; h0 < n_h; h0 += 8 * (kQpThreads / 64)) {
    if (h0 != wave) load_q(h0, qv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int h = h0 + i * (kQpThreads / 64);
      if (h < n_h) {                                      // uniform over the wave
        const bool live = lane < half && !((emask[h] >> lane) & 1ull);
        const uint64_t mask = __ballot(live);
        const int pos = __popcll(mask & ((1ull << lane) - 1ull));
        if (live) {
#pragma unroll
          for (int bt = 0; bt < BT; ++bt)
            reinterpret_cast<uint32_t*>(qne + ((size_t)bt * n_h + h) * ndp)[pos] = qv[i][bt];
        }
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");        // this wave's pieces of the weight image have landed
  __syncthreads();

  if (!row_ok) return;
  const int k = (int)((uint32_t)row / (uint32_t)n_h), h = (int)((uint32_t)row % (uint32_t)n_h);
  const uint4* wrow = reinterpret_cast<const uint4*>(wl + (size_t)tid * pitch * 16);
  float acc[BT];
#pragma unroll
  for (int bt = 0; bt < BT; ++bt) acc[bt] = 0.f;
#pragma unroll
  for (int c = 0; c < 16; ++c) {
    if (c < nchunk) {
      const uint4 wv = wrow[c];
      const uint32_t ww[4] = {wv.x, wv.y, wv.z, wv.w};
      float w[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        w[2 * i] = __uint_as_float(ww[i] << 16);
        w[2 * i + 1] = __uint_as_float(ww[i] & 0xffff0000u);
      }
#pragma unroll
      for (int bt = 0; bt < BT; ++bt) {
        const uint4 qv = *reinterpret_cast<const uint4*>(qne + ((size_t)bt * n_h + h) * ndp + 8 * c);
        const uint32_t qq[4] = {qv.x, qv.y, qv.z, qv.w};
        float a = acc[bt];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a = fmaf(w[2 * i], __uint_as_float(qq[i] << 16), a);
          a = fmaf(w[2 * i + 1], __uint_as_float(qq[i] & 0xffff0000u), a);
        }
        acc[bt] = a;
      }
    }
  }
#pragma unroll
  for (int bt = 0; bt < BT; ++bt)
    if (bt < bt_n) st(qt, qt_packed_index(b0 + bt, h, k, P.head_groups, d_c, P.q_slice), acc[bt] * scale_log2e);
}

}  // namespace ekv
