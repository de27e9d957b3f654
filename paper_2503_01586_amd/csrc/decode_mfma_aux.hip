// The kernels around the bf16 MFMA attention kernel:
//   qprep_rows   : rotated elite query + W_uk absorbed into the rest of the query
//                  (Section 3.1 score equation, first sum; Section 5, absorption of B^k)
//   merge_up     : exact log-sum-exp merge of the sequence splits, normalisation, and the W_uv
//                  up-projection of a chunk of latent columns (Section 3.2, B^v_J), one batch row
//                  (the version for a batch is merge_mfma.hip)
//                  the last work-group of a head to finish adds the chunks' partials (chunk_sum.hpp)
#include "common.hpp"
#include "chunk_sum.hpp"
#include "launch.hpp"
#include "qprep_rows.hpp"
#include "qprep_mfma.hpp"

namespace ekv {

template <int BT>
__global__ __launch_bounds__(kQpThreads) void qprep_rows_kernel(const QprepRowsParams P, const RopeTable rope) {
  extern __shared__ __attribute__((aligned(16))) char qsm[];
  qprep_rows_body<BT>(P, rope, blockIdx.x, gridDim.x, blockIdx.y, qsm);
}

QprepRowsParams make_qprep_rows_params(const DecodeArgs& a, const DecodePlan& p, float* qe, bf16_t* qt) {
  const elitekv_dims& d = a.dims;
  QprepRowsParams P;
  P.q = (const bf16_t*)a.q; P.q_pos = a.q_pos; P.W_uk = (const bf16_t*)a.W_uk; P.elite_idx = a.elite_idx;
  P.qe = qe; P.qt = qt; P.sincos = p.fresh ? (float2*)(a.ws + p.off_sincos) : nullptr; P.B = (int)a.B; P.n_h = d.n_heads; P.d_h = d.head_dim; P.r = d.r; P.d_c = p.d_q;
  P.q_slice = decode_mfma_slice_width(d.d_c); P.head_groups = p.head_groups;
  P.scale_log2e = kLog2e / sqrtf((float)d.head_dim);
  return P;
}

template <int BT>
static hipError_t launch_qprep_bt(const DecodeArgs& a, const DecodePlan& p, float* qe, bf16_t* qt, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const size_t sm = qprep_rows_lds(d.n_heads, d.head_dim, d.r, BT);
  const int64_t rows = (int64_t)p.d_q * d.n_heads;
  const dim3 grid((unsigned)((rows + kQpThreads - 1) / kQpThreads) + 1, (unsigned)((a.B + BT - 1) / BT));   // + the rotation group
  static LdsLimit lds_limit;
  const hipError_t le = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&qprep_rows_kernel<BT>), sm);
  if (le != hipSuccess) return le;
  qprep_rows_kernel<BT><<<grid, kQpThreads, sm, stream>>>(make_qprep_rows_params(a, p, qe, qt),
                                                          rope_table(d.rope_base, d.head_dim));
  return hipGetLastError();
}

template <int KS>
__global__ __launch_bounds__(256) void qprep_mfma_kernel(const QprepRowsParams P, const RopeTable rope) {
  extern __shared__ __attribute__((aligned(16))) char qms[];
  qprep_mfma_body<KS>(P, rope, blockIdx.x, blockIdx.y, qms);
}

bool qprep_mfma_supported(const elitekv_dims& d, int d_q, int64_t B) {
  const int nd = d.head_dim - 2 * d.r;
  return B >= 8 && d_q % 128 == 0 && nd % 8 == 0 && nd >= 16 && nd <= 128 && d.head_dim <= 128;
}

static hipError_t launch_qprep_mfma(const DecodeArgs& a, const DecodePlan& p, float* qe, bf16_t* qt, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int nd = d.head_dim - 2 * d.r;
  const int ks = (nd + 15) / 16;
  const size_t sm = qprep_mfma_lds(d.head_dim, d.r);
  const dim3 grid(p.d_q / 128, d.n_heads);
  const QprepRowsParams P = make_qprep_rows_params(a, p, qe, qt);
  const RopeTable rope = rope_table(d.rope_base, d.head_dim);
#define EKV_QM(KSV) qprep_mfma_kernel<KSV><<<grid, 256, sm, stream>>>(P, rope)
  switch (ks) {
    case 1: EKV_QM(1); break;
    case 2: EKV_QM(2); break;
    case 3: EKV_QM(3); break;
    case 4: EKV_QM(4); break;
    case 5: EKV_QM(5); break;
    case 6: EKV_QM(6); break;
    case 7: EKV_QM(7); break;
    default: EKV_QM(8); break;
  }
#undef EKV_QM
  return hipGetLastError();
}

hipError_t launch_qprep_rows(const DecodeArgs& a, const DecodePlan& p, float* qe, bf16_t* qt, hipStream_t stream) {
  if (qprep_mfma_supported(a.dims, p.d_q, a.B)) return launch_qprep_mfma(a, p, qe, qt, stream);
  // batch rows per work-group: as many as the batch has (up to 8) and as the LDS holds
  int bt = a.B == 1 ? 1 : a.B == 2 ? 2 : a.B <= 4 ? 4 : kQpBatchTile;
  while (bt > 1 && qprep_rows_lds(a.dims.n_heads, a.dims.head_dim, a.dims.r, bt) > 150 * 1024) bt >>= 1;
  if (qprep_rows_lds(a.dims.n_heads, a.dims.head_dim, a.dims.r, bt) > 150 * 1024) return hipErrorInvalidValue;   // more heads than an LDS holds
  if (bt == 1) return launch_qprep_bt<1>(a, p, qe, qt, stream);
  if (bt == 2) return launch_qprep_bt<2>(a, p, qe, qt, stream);
  if (bt == 4) return launch_qprep_bt<4>(a, p, qe, qt, stream);
  return launch_qprep_bt<kQpBatchTile>(a, p, qe, qt, stream);
}

// ---------------------------------------------------------------------------------------------
// merge_up.  One work-group per (chunk of CW latent columns, head, batch row):
//   * exact log-sum-exp merge of the sequence splits for this head (weights from m, l),
//   * the merged, normalised latent of the chunk's columns,
//   * its contribution to the up-projection  o[h, :] = ubar[h, :] W_uv[:, h, :]   (B^v_J),
//   * written as a partial per chunk; the last work-group of the head to arrive adds the chunk
//     partials in chunk order and writes out[b, head, :] (chunk_sum.hpp); fuse_out == 0 leaves the
//     partials for a caller that consumes them itself.
// Partials: part_m / part_l [P, NHP], part_u [P, NHP, d_c] bf16 with P = b * n_splits + s.
// All global loads that do not depend on earlier results (the W_uv rows, the first batch of
// split accumulators) are requested at the top so that their latency overlaps the merge weights.
// ---------------------------------------------------------------------------------------------
template <int CW, int DH>
__global__ __launch_bounds__(256) void merge_up_kernel(
    const float* __restrict__ part_m, const float* __restrict__ part_l,
    const bf16_t* __restrict__ part_u, const bf16_t* __restrict__ W_uv, float* opart,
    bf16_t* __restrict__ out, int* chunk_counters, int fuse_out, int n_h, int nhp, int d_c, int n_splits) {
  constexpr int LPR = CW / 8;              // lanes that cover one split's row chunk (16 bytes each)
  constexpr int NG = 256 / LPR;            // split groups working in parallel
  constexpr int LPW = DH / 8;              // lanes that cover one W_uv row
  constexpr int RPI = 64 / LPW;            // W_uv rows per wave instruction
  constexpr int NWI = CW / (4 * RPI);      // W_uv rows per thread
  constexpr int UB = 28;                   // split accumulators requested per batch
  // all arguments in one round trip of the scalar cache (else: three, one after the other, before the first load)
  asm volatile("" ::"s"(part_m), "s"(part_l), "s"(part_u), "s"(W_uv), "s"(opart), "s"(out), "s"(chunk_counters),
               "s"(fuse_out), "s"(n_h), "s"(nhp), "s"(d_c), "s"(n_splits), "s"(gridDim.x));
  extern __shared__ __attribute__((aligned(16))) float msm[];
  float* wsp = msm;                        // [n_splits] merge weights of this head
  float* red = wsp + n_splits;             // [256] scratch
  float* big = red + 256;                  // [NG][CW], later [4][DH]
  float* ubar = big + NG * CW;             // [CW]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int chunk = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  const int n_chunks = gridDim.x;
  const int64_t p0 = (int64_t)b * n_splits;
  const int col0 = chunk * CW;

  // (0) the split maxima and sums this thread will need first (split tid of the first 256): requested
  //     before the bulk loads, behind which they would return late
  const bool first_ok = tid < n_splits;
  const float m_first = first_ok ? part_m[(p0 + tid) * nhp + head] : -INFINITY;
  const float l_first = first_ok ? part_l[(p0 + tid) * nhp + head] : 0.f;

  // (1) this thread's W_uv rows: k = col0 + wave*RPI + rr + i*4*RPI
  const int jl = lane % LPW, rr = lane / LPW;
  uint4 wreg[NWI];
  {
    const bf16_t* wb = W_uv + ((int64_t)(col0 + wave * RPI + rr) * n_h + head) * DH + jl * 8;
#pragma unroll
    for (int i = 0; i < NWI; ++i)
      wreg[i] = ld16_stream(wb + (int64_t)i * 4 * RPI * n_h * DH);
  }
  // (2) first batch of split accumulators: group sg takes splits sg, sg + NG, ...
  const int cl = tid % LPR, sg = tid / LPR;
  const bool grp_ok = sg < NG;
  const bf16_t* ub = part_u + (p0 * nhp + head) * (int64_t)d_c + col0 + cl * 8;
  const int64_t sstep = (int64_t)nhp * d_c;
  uint4 ureg[UB];
  auto load_batch = [&](int s0) {
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int s = s0 + sg + u * NG;
      ureg[u] = make_uint4(0, 0, 0, 0);
      if (grp_ok && s < n_splits) ureg[u] = *reinterpret_cast<const uint4*>(ub + s * sstep);
    }
  };
  load_batch(0);

  // (3) merge weights  w_s = exp2(m_s - max m),  L = sum w_s l_s   (an empty split has l = 0)
  float m = m_first;
  for (int s = tid + 256; s < n_splits; s += 256) m = fmaxf(m, part_m[(p0 + s) * nhp + head]);
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  float lsum = 0.f;
  for (int s = tid; s < n_splits; s += 256) {
    const float ls = (s == tid) ? l_first : part_l[(p0 + s) * nhp + head];
    const float ms = (s == tid) ? m_first : part_m[(p0 + s) * nhp + head];
    const float w = (ls > 0.f) ? exp2f(ms - m) : 0.f;
    wsp[s] = w;
    lsum += w * ls;
  }
  lsum = wave_sum(lsum);
  if (lane == 0) red[wave] = lsum;
  __syncthreads();
  const float Lsum = (red[0] + red[1]) + (red[2] + red[3]);
  const float inv = (Lsum > 0.f) ? 1.f / Lsum : 0.f;

  // (4) merged latent of this chunk (an empty split has weight 0 and a zero accumulator)
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int s0 = 0; s0 < n_splits; s0 += UB * NG) {
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int s = s0 + sg + u * NG;
      const float w = (grp_ok && s < n_splits) ? wsp[s] : 0.f;
      const uint32_t uu[4] = {ureg[u].x, ureg[u].y, ureg[u].z, ureg[u].w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        acc[2 * i] = fmaf(w, __uint_as_float(uu[i] << 16), acc[2 * i]);
        acc[2 * i + 1] = fmaf(w, __uint_as_float(uu[i] & 0xffff0000u), acc[2 * i + 1]);
      }
    }
    if (s0 + UB * NG < n_splits) load_batch(s0 + UB * NG);
  }
  if (grp_ok) {
#pragma unroll
    for (int i = 0; i < 8; ++i) big[sg * CW + cl * 8 + i] = acc[i];
  }
  __syncthreads();
  for (int c = tid; c < CW; c += 256) {
    float a = 0.f;
#pragma unroll 4
    for (int gq = 0; gq < NG; ++gq) a += big[gq * CW + c];
    ubar[c] = a * inv;
  }
  __syncthreads();

  // (5) up-projection of this chunk with the prefetched rows
  float o[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = 0.f;
#pragma unroll
  for (int i = 0; i < NWI; ++i) {
    const float u = ubar[wave * RPI + rr + i * 4 * RPI];
    const uint32_t ww[4] = {wreg[i].x, wreg[i].y, wreg[i].z, wreg[i].w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      o[2 * q] = fmaf(u, __uint_as_float(ww[q] << 16), o[2 * q]);
      o[2 * q + 1] = fmaf(u, __uint_as_float(ww[q] & 0xffff0000u), o[2 * q + 1]);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float v = o[i];
#pragma unroll
    for (int off = LPW; off < 64; off <<= 1) v += __shfl_xor(v, off, kWave);
    o[i] = v;
  }
  float* wred = big;                         // [4][DH]
  if (rr == 0) {
#pragma unroll
    for (int i = 0; i < 8; ++i) wred[wave * DH + jl * 8 + i] = o[i];
  }
  __syncthreads();
  float* op = opart + (((int64_t)b * n_h + head) * n_chunks + chunk) * DH;
  if (tid < DH)
    store_partial_device_scope(op + tid, (wred[tid] + wred[DH + tid]) + (wred[2 * DH + tid] + wred[3 * DH + tid]));
  if (fuse_out)
    sum_chunks_by_last_arrival<DH>(opart, out, chunk_counters + (int64_t)b * n_h + head, n_h, n_chunks, head, b, 1,
                                   reinterpret_cast<int*>(red));
}

// out[b, h, j] = sum over the latent chunks of the up-projection partials, in chunk order: the launch that
// follows the batched merge.  (There a last-arrival sum inside the merge, as the single-row merge has it, was
// measured 1 to 3 us slower than this launch: one work-group then adds up to 32 rows x d_h x chunks values behind
// a chain of store acknowledgement, counter and device-scope loads.)
__global__ __launch_bounds__(256) void out_reduce_kernel(const float* __restrict__ opart,
                                                         bf16_t* __restrict__ out, int d_h,
                                                         int n_chunks, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over [B * n_h, d_h]
  if (e >= total) return;
  const int64_t bh = e / d_h;
  const int j = (int)(e % d_h);
  const float* p = opart + bh * n_chunks * d_h + j;
  float a = 0.f;
#pragma unroll 8
  for (int c = 0; c < n_chunks; ++c) a += p[(int64_t)c * d_h];
  st(out, e, a);
}

hipError_t launch_merge_up(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  if (p.merge_batch) {
    hipError_t e = launch_merge_mfma(a, p, stream);
    if (e != hipSuccess || a.no_out_reduce) return e;
    const int64_t total = (int64_t)a.B * d.n_heads * d.head_dim;
    out_reduce_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(
        (const float*)(a.ws + p.off_opart), (bf16_t*)a.out, d.head_dim, p.d_u / 128, total);
    return hipGetLastError();
  }
  const float* pm = (const float*)(a.ws + p.off_m);
  const float* pl = (const float*)(a.ws + p.off_l);
  const bf16_t* pu = (const bf16_t*)(a.ws + p.off_u);
  float* opart = (float*)(a.ws + p.off_opart);
  const int cw = p.up_cw;
  const dim3 grid(p.d_u / cw, d.n_heads, (unsigned)a.B);
  const int nhp = p.head_groups * 32;
#define EKV_MU(CW, DH)                                                                              \
  do {                                                                                              \
    const size_t sm = sizeof(float) * ((size_t)p.n_part + 256 + (size_t)(256 / (CW / 8)) * CW + CW); \
    merge_up_kernel<CW, DH><<<grid, 256, sm, stream>>>(pm, pl, pu, (const bf16_t*)a.W_uv, opart,    \
                                                       (bf16_t*)a.out, (int*)(a.ws + p.off_cnt),    \
                                                       a.no_out_reduce ? 0 : 1, d.n_heads, nhp,     \
                                                       p.d_u, p.n_part);                            \
  } while (0)
  if (cw == 192) { if (d.head_dim == 128) EKV_MU(192, 128); else EKV_MU(192, 64); }
  else { if (d.head_dim == 128) EKV_MU(64, 128); else EKV_MU(64, 64); }
#undef EKV_MU
  return hipGetLastError();
}

}  // namespace ekv
