// Front kernel of the fused decode step.  The step's two first pieces of work do not depend on each
// other: the cache append of the step's tokens (x [W_ke | W_dkv]; Sections 3.1 and 3.2) and the
// query preparation (rotated elite query, W_uk absorbed into the rest; Section 3.1 score equation,
// Section 5).  Both are a single pass over a weight matrix of a few megabytes, far too short to
// amortise a launch each, so one launch runs both: the first work-groups take the rows of W_uk, the
// others the (column block, contraction split) pieces of the append.  The append's split sums are
// added up, rotated and stored by the new-token work-groups of the attention kernel that follows in
// the stream (they need the prepared query anyway), so the step has no separate finishing launch.
#include "common.hpp"
#include "launch.hpp"
#include "append_small.hpp"
#include "append_skinny.hpp"
#include "qprep_rows.hpp"
#include "qprep_mfma.hpp"

namespace ekv {

QprepRowsParams make_qprep_rows_params(const DecodeArgs& a, const DecodePlan& p, float* qe, bf16_t* qt);
AppendSkinnyParams make_append_skinny_params(const AppendArgs& a, float* partial, int kc);
int append_skinny_ksplit(const elitekv_dims& d);
int append_skinny_kc(const elitekv_dims& d, int ks);

constexpr int kFrontBatch = 16;   // weight rows per thread in flight in the append role

// token / batch-row tile (template parameter) that covers B rows
static int front_tile(int64_t B) { return B == 1 ? 1 : B == 2 ? 2 : B <= 4 ? 4 : 8; }

// BT = token / batch-row tile of both roles (the step appends one token per batch row)
template <int BT>
__global__ __launch_bounds__(256) void decode_front_kernel(const AppendSmallParams A, const QprepRowsParams Q,
                                                           const RopeTable rope, int n_qprep, int n_blocks) {
  extern __shared__ __attribute__((aligned(16))) char fsm[];
  static_assert(kAsThreads == 256 && kQpThreads == 256, "both roles use 256 threads");
  // the arguments of both roles are fetched in one round trip of the scalar cache, ahead of the first branch
  // (fetched where they are first used they cost three trips of about 0.4 us each before the first load goes out)
  asm volatile("" ::"s"(A.x), "s"(A.T), "s"(A.W_ke), "s"(A.W_dkv), "s"(A.W_dkv2), "s"(A.partial), "s"(A.d_ck), "s"(A.d),
               "s"(A.NE), "s"(A.d_c), "s"(A.kc), "s"(A.W_q), "s"(A.q_cols), "s"(n_qprep), "s"(n_blocks), "s"(Q.q), "s"(Q.q_pos), "s"(Q.W_uk),
               "s"(Q.elite_idx), "s"(Q.qe), "s"(Q.qt), "s"(Q.sincos), "s"(Q.B), "s"(Q.n_h), "s"(Q.d_h), "s"(Q.r),
               "s"(Q.d_c), "s"(Q.q_slice), "s"(Q.head_groups), "s"(Q.scale_log2e));
  const int wg = blockIdx.x;
  if (wg < n_qprep) {
    qprep_rows_body<BT>(Q, rope, wg, n_qprep, 0, fsm);
  } else {
    const int e = wg - n_qprep;
    append_small_body<BT, kFrontBatch>(A, e % n_blocks, e / n_blocks, 0, reinterpret_cast<float*>(fsm));
  }
}

bool decode_front_plan(const elitekv_dims& d, int d_ck, int d_q, int64_t B, int* ks_out, int* kc_out) {
  if (d.dtype != ELITEKV_BF16 || B < 1 || B > kAsTokens) return false;
  if (qprep_mfma_supported(d, d_q, B)) return false;                 // eight rows and up: matrix-core kernels
  const int nd = d.head_dim - 2 * d.r;
  if (d.r < 1 || nd < 8 || nd % 8 || d.head_dim > 128) return false;
  if (!append_small_supported(d, B, d_ck > 0 ? d_ck : d.d_c)) return false;
  const size_t lds = qprep_rows_lds(d.n_heads, d.head_dim, d.r, front_tile(B));
  if (lds > 150 * 1024) return false;
  // contraction splits: as many as keep every work-group of the launch resident at once
  const int resident = 256 * (lds + 2048 <= 80 * 1024 ? 2 : 1);
  const int n_qprep = (int)(((int64_t)d_q * d.n_heads + kQpThreads - 1) / kQpThreads) + 1;
  const int n_blocks = (2 * d.r * d.n_heads + d.d_c) / kAsCols;
  int ks = 16;
  while (ks > 2 && (n_qprep + n_blocks * ks > resident || (d.d_model + ks - 1) / ks < 64)) ks >>= 1;
  int kc = (d.d_model + ks - 1) / ks;
  kc = (kc + 31) / 32 * 32;
  *ks_out = ks; *kc_out = kc;
  return true;
}

template <int BT>
static hipError_t launch_front_bt(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const size_t sm_a = (size_t)p.fr_kc * BT * sizeof(float), sm_q = qprep_rows_lds(d.n_heads, d.head_dim, d.r, BT);
  const size_t sm = sm_a > sm_q ? sm_a : sm_q;
  static LdsLimit lds_limit;
  const hipError_t le = raise_lds_limit(lds_limit, reinterpret_cast<const void*>(&decode_front_kernel<BT>), sm);
  if (le != hipSuccess) return le;
  const int NE = 2 * d.r * d.n_heads;
  AppendSmallParams A;
  A.x = (const bf16_t*)ap.x; A.T = ap.T; A.W_ke = (const bf16_t*)ap.W_ke; A.W_dkv = (const bf16_t*)ap.W_dkv;
  A.W_dkv2 = (const bf16_t*)ap.W_dkv2; A.partial = (float*)(a.ws + p.off_apart); A.d_ck = ap.d_ck; A.d = d.d_model;
  A.NE = NE; A.d_c = d.d_c; A.kc = p.fr_kc;
  A.W_q = nullptr; A.q_cols = 0; A.x_opart = nullptr; A.x_heads = 0; A.x_chunks = 0; A.x_dh = 1;
  const int n_blocks = (NE + d.d_c) / kAsCols;
  const int n_qprep = (int)(((int64_t)p.d_q * d.n_heads + kQpThreads - 1) / kQpThreads) + 1;   // + the rotation group
  decode_front_kernel<BT><<<n_qprep + n_blocks * p.fr_ks, 256, sm, stream>>>(
      A, make_qprep_rows_params(a, p, (float*)(a.ws + p.off_qe), (bf16_t*)(a.ws + p.off_qt)),
      rope_table(d.rope_base, d.head_dim), n_qprep, n_blocks);
  return hipGetLastError();
}

hipError_t launch_decode_front(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const int bt = front_tile(a.B);
  return bt == 1 ? launch_front_bt<1>(ap, a, p, stream) : bt == 2 ? launch_front_bt<2>(ap, a, p, stream)
       : bt == 4 ? launch_front_bt<4>(ap, a, p, stream) : launch_front_bt<8>(ap, a, p, stream);
}

// ---- whole attention block of a step (Section 2.1: q = x W^q in front, [o_0 .. o_{n_h-1}] W^o behind).
// block_front: the first pass of the append and of the query projection in one weight-streaming
// launch (the same x, the columns of W_q simply follow the cache row's columns); q_finish adds the
// query's split sums and rounds them (every q-prep work-group needs the whole query: summing the
// splits there, 193 times over, was measured at 25 us).  oproj: y = out W^o by the same
// weight-streaming body, whose x is read as the sum of the merge's column-chunk partials, so the
// merge needs no reduction launch; y_finish adds the contraction splits of y.
template <int TT>
__global__ __launch_bounds__(kAsThreads) void block_front_kernel(const AppendSmallParams P) {
  extern __shared__ __attribute__((aligned(16))) float bfx[];
  append_small_body<TT, kFrontBatch, 0>(P, blockIdx.x, blockIdx.y, 0, bfx);
}

template <int TT>
__global__ __launch_bounds__(kAsThreads) void oproj_kernel(const AppendSmallParams P) {
  extern __shared__ __attribute__((aligned(16))) float opx[];
  append_small_body<TT, kFrontBatch, 1>(P, blockIdx.x, blockIdx.y, 0, opx);
}

// q[b, c] = bf16(sum over the contraction splits of the x W_q columns of the front pass)
__global__ __launch_bounds__(256) void q_finish_kernel(const float* __restrict__ partial, bf16_t* __restrict__ q, int ks,
                                                       int64_t B, int stride, int col0, int q_cols) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over [B, q_cols]
  if (e >= B * q_cols) return;
  const int64_t b = e / q_cols;
  const int c = (int)(e - b * q_cols);
  float a = 0.f;
  for (int s = 0; s < ks; ++s) a += partial[((int64_t)s * B + b) * stride + col0 + c];
  st(q, e, a);
}

__global__ __launch_bounds__(256) void y_finish_kernel(const float* __restrict__ partial, bf16_t* __restrict__ y,
                                                       int ks, int64_t total) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;   // over [B, d_model]
  if (e >= total) return;
  float a = 0.f;
  for (int s = 0; s < ks; ++s) a += partial[(int64_t)s * total + e];
  st(y, e, a);
}

// contraction splits of a weight-streaming pass over `rows` weight rows: at most 512 rows per split
// (sixteen per thread, all in flight at once), whole 32-row steps
static void stream_splits(int rows, int* ks, int* kc) {
  int s = (rows + 511) / 512;
  if (s < 1) s = 1;
  int c = (rows + s - 1) / s;
  c = (c + 31) / 32 * 32;
  *ks = (rows + c - 1) / c;
  *kc = c;
}

bool block_step_plan(const elitekv_dims& d, int64_t B, int* fr_ks, int* fr_kc, int* y_ks, int* y_kc) {
  if (B < 1 || B > kAsTokens || d.d_model % kAsCols || (d.n_heads * d.head_dim) % kAsCols) return false;
  stream_splits(d.d_model, fr_ks, fr_kc);
  stream_splits(d.n_heads * d.head_dim, y_ks, y_kc);
  return true;
}

template <int TT>
static hipError_t launch_block_front_tt(const AppendArgs& ap, const void* W_q, const DecodeArgs& a, const DecodePlan& p,
                                        hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int NE = 2 * d.r * d.n_heads, q_cols = d.n_heads * d.head_dim;
  AppendSmallParams A;
  A.x = (const bf16_t*)ap.x; A.T = ap.T; A.W_ke = (const bf16_t*)ap.W_ke; A.W_dkv = (const bf16_t*)ap.W_dkv;
  A.W_dkv2 = (const bf16_t*)ap.W_dkv2; A.partial = (float*)(a.ws + p.off_apart); A.d_ck = ap.d_ck; A.d = d.d_model;
  A.NE = NE; A.d_c = d.d_c; A.kc = p.fr_kc;
  A.W_q = (const bf16_t*)W_q; A.q_cols = q_cols; A.x_opart = nullptr; A.x_heads = 0; A.x_chunks = 0; A.x_dh = 1;
  const dim3 grid((NE + d.d_c + q_cols) / kAsCols, p.fr_ks);
  block_front_kernel<TT><<<grid, kAsThreads, (size_t)p.fr_kc * TT * sizeof(float), stream>>>(A);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t total = ap.T * (int64_t)q_cols;
  q_finish_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>(A.partial, (bf16_t*)(a.ws + p.off_qfin), p.fr_ks,
                                                                     ap.T, p.fr_stride, NE + d.d_c, q_cols);
  return hipGetLastError();
}

hipError_t launch_block_front(const AppendArgs& ap, const void* W_q, const DecodeArgs& a, const DecodePlan& p,
                              hipStream_t stream) {
  const int tt = front_tile(a.B);
  return tt == 1 ? launch_block_front_tt<1>(ap, W_q, a, p, stream) : tt == 2 ? launch_block_front_tt<2>(ap, W_q, a, p, stream)
       : tt == 4 ? launch_block_front_tt<4>(ap, W_q, a, p, stream) : launch_block_front_tt<8>(ap, W_q, a, p, stream);
}

template <int TT>
static hipError_t launch_oproj_tt(const DecodeArgs& a, const DecodePlan& p, const void* W_o, void* y, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  AppendSmallParams A;
  A.x = nullptr; A.T = a.B; A.W_ke = nullptr; A.W_dkv = (const bf16_t*)W_o; A.W_dkv2 = nullptr;
  A.partial = (float*)(a.ws + p.off_ypart); A.d_ck = d.d_model; A.d = d.n_heads * d.head_dim; A.NE = 0; A.d_c = d.d_model;
  A.kc = p.y_kc; A.W_q = nullptr; A.q_cols = 0;
  A.x_opart = (const float*)(a.ws + p.off_opart); A.x_heads = d.n_heads; A.x_chunks = p.d_u / p.up_cw; A.x_dh = d.head_dim;
  const dim3 grid(d.d_model / kAsCols, p.y_ks);
  oproj_kernel<TT><<<grid, kAsThreads, (size_t)p.y_kc * TT * sizeof(float), stream>>>(A);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t total = a.B * (int64_t)d.d_model;
  y_finish_kernel<<<(unsigned)((total + 255) / 256), 256, 0, stream>>>((const float*)(a.ws + p.off_ypart), (bf16_t*)y,
                                                                     p.y_ks, total);
  return hipGetLastError();
}

hipError_t launch_oproj(const DecodeArgs& a, const DecodePlan& p, const void* W_o, void* y, hipStream_t stream) {
  const int tt = front_tile(a.B);
  return tt == 1 ? launch_oproj_tt<1>(a, p, W_o, y, stream) : tt == 2 ? launch_oproj_tt<2>(a, p, W_o, y, stream)
       : tt == 4 ? launch_oproj_tt<4>(a, p, W_o, y, stream) : launch_oproj_tt<8>(a, p, W_o, y, stream);
}

// ---- batches of eight rows and up: the matrix-core versions of the two roles in one launch; the
// append's split sums are then added, rotated and stored by append_finish (with many sequences the
// new-token work-groups of the attention kernel would take compute units from its tile work-groups).
template <int KS, int TT>
__global__ __launch_bounds__(256) void decode_front_mfma_kernel(const AppendSkinnyParams A, const QprepRowsParams Q,
                                                                const RopeTable rope, int n_qprep, int q_blocks,
                                                                int n_blocks) {
  extern __shared__ __attribute__((aligned(16))) char fsm[];
  const int wg = blockIdx.x;
  if (wg < n_qprep) {
    qprep_mfma_body<KS>(Q, rope, wg % q_blocks, wg / q_blocks, fsm);          // (block of 128 latent columns, head)
  } else {
    const int e = wg - n_qprep;
    append_skinny_body<TT>(A, e % n_blocks, e / n_blocks, fsm);               // (column block, contraction split)
  }
}

bool decode_front_mfma_supported(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p) {
  const elitekv_dims& d = a.dims;
  if (!p.mfma || p.fresh == 1 || ap.T != a.B) return false;
  return qprep_mfma_supported(d, p.d_q, a.B) && append_skinny_supported(d, ap.T, ap.d_ck);
}

// Fused step for 8 to 64 sequences: the contraction splits and the rows of a split that the batched front launch
// leaves for the attention kernel's owner work-groups (no finishing launch).
bool decode_front_mfma_plan(const elitekv_dims& d, int d_ck, int d_q, int64_t B, int* ks_out, int* kc_out) {
  if (!qprep_mfma_supported(d, d_q, B) || !append_skinny_supported(d, B, d_ck > 0 ? d_ck : d.d_c)) return false;
  int ks = append_skinny_ksplit(d);
  const int kc = append_skinny_kc(d, ks);
  ks = (d.d_model + kc - 1) / kc;
  *ks_out = ks; *kc_out = kc;
  return true;
}

template <int KS>
static hipError_t launch_front_mfma_ks(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int N = 2 * d.r * d.n_heads + d.d_c;
  int ks = append_skinny_ksplit(d);
  const int kc = append_skinny_kc(d, ks);
  ks = (d.d_model + kc - 1) / kc;            // splits that still have rows; never more than planned
  float* partial = p.fresh == 2 ? (float*)(a.ws + p.off_apart) : (float*)ap.ws;
  const size_t sm_q = qprep_mfma_lds(d.head_dim, d.r);
  const size_t sm = sm_q > (size_t)kSkLds ? sm_q : (size_t)kSkLds;
  const int q_blocks = p.d_q / 128, n_qprep = q_blocks * d.n_heads, n_blocks = N / kSkCols;
  const AppendSkinnyParams A = make_append_skinny_params(ap, partial, kc);
  const QprepRowsParams Q = make_qprep_rows_params(a, p, (float*)(a.ws + p.off_qe), (bf16_t*)(a.ws + p.off_qt));
  const RopeTable rope = rope_table(d.rope_base, d.head_dim);
  const unsigned grid = (unsigned)(n_qprep + n_blocks * ks);
  if (ap.T <= 32) decode_front_mfma_kernel<KS, 1><<<grid, 256, sm, stream>>>(A, Q, rope, n_qprep, q_blocks, n_blocks);
  else decode_front_mfma_kernel<KS, 2><<<grid, 256, sm, stream>>>(A, Q, rope, n_qprep, q_blocks, n_blocks);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.fresh == 2) return e;            // fused step: the attention launch finishes the new rows
  return launch_append_finish(ap, partial, ks, stream);
}

hipError_t launch_decode_front_mfma(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const int nd = a.dims.head_dim - 2 * a.dims.r;
  switch ((nd + 15) / 16) {
    case 1: return launch_front_mfma_ks<1>(ap, a, p, stream);
    case 2: return launch_front_mfma_ks<2>(ap, a, p, stream);
    case 3: return launch_front_mfma_ks<3>(ap, a, p, stream);
    case 4: return launch_front_mfma_ks<4>(ap, a, p, stream);
    case 5: return launch_front_mfma_ks<5>(ap, a, p, stream);
    case 6: return launch_front_mfma_ks<6>(ap, a, p, stream);
    case 7: return launch_front_mfma_ks<7>(ap, a, p, stream);
    default: return launch_front_mfma_ks<8>(ap, a, p, stream);
  }
}

}  // namespace ekv
