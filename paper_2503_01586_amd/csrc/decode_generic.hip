// Generic (any shape, fp32 or bf16 storage, fp32 VALU arithmetic) decode attention over the
// EliteKV cache.  This is the path of the fp32 dtype and of bf16 shapes the MFMA kernels do not
// cover.  Three kernels on one stream:
//   qprep  : rotate the query's elite chunks at q_pos, absorb W_uk into the rest of the query
//            (Section 3.1 score equation, first sum; Section 5, absorption of B^k)
//   attn   : per (split, head, batch row) online softmax over both score terms with values
//            accumulated in latent space (Section 2.1 softmax; Section 3.2 shared latent)
//   merge  : exact log-sum-exp merge of the splits, then the W_uv up-projection (B^v_J)
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

constexpr int kGenThreads = 256;
constexpr int kGenTile = 64;   // cached tokens per inner tile

template <typename T>
__global__ __launch_bounds__(kGenThreads) void qprep_generic_kernel(
    const T* __restrict__ q, const int32_t* __restrict__ q_pos, const T* __restrict__ W_uk,
    const int32_t* __restrict__ elite_idx, float* __restrict__ qe, float* __restrict__ qt,
    int n_h, int d_h, int r, int d_c, RopeTable rope, float scale_log2e) {
  __shared__ float q_ne[256];     // d_h <= 256 checked on the host
  __shared__ int is_elite[128];
  const int h = blockIdx.x;
  const int b = blockIdx.y;
  const int tid = threadIdx.x;
  const int nd = d_h - 2 * r;
  const T* qrow = q + ((int64_t)b * n_h + h) * d_h;

  for (int i = tid; i < d_h / 2; i += kGenThreads) is_elite[i] = 0;
  __syncthreads();
  for (int j = tid; j < r; j += kGenThreads) {
    int i = elite_idx[h * r + j];
    if (i >= 0 && i < d_h / 2) is_elite[i] = 1;
  }
  __syncthreads();
  if (tid == 0) {
    int n = 0;
    for (int i = 0; i < d_h / 2; ++i) {
      if (!is_elite[i]) {
        if (n + 1 < nd) {             // overflows only if the caller passed repeated indices
          q_ne[n] = ld(qrow, 2 * i) * scale_log2e;
          q_ne[n + 1] = ld(qrow, 2 * i + 1) * scale_log2e;
        }
        n += 2;
      }
    }
    for (; n < nd; ++n) q_ne[n] = 0.f;
  }
  for (int j = tid; j < r; j += kGenThreads) {
    int i = elite_idx[h * r + j];
    i = min(max(i, 0), d_h / 2 - 1);
    float s, c;
    rope_sincos(q_pos[b], rope.theta[i], &s, &c);
    float u = ld(qrow, 2 * i), v = ld(qrow, 2 * i + 1);
    float* o = qe + ((int64_t)b * n_h + h) * 2 * r;
    o[2 * j] = (u * c - v * s) * scale_log2e;
    o[2 * j + 1] = (u * s + v * c) * scale_log2e;
  }
  __syncthreads();
  float* qt_row = qt + ((int64_t)b * n_h + h) * d_c;
  for (int k = tid; k < d_c; k += kGenThreads) {
    const T* w = W_uk + ((int64_t)k * n_h + h) * nd;
    float acc = 0.f;
    for (int j = 0; j < nd; ++j) acc = fmaf(q_ne[j], ld(w, j), acc);
    qt_row[k] = acc;
  }
}

// One work-group per (split, head, batch row).  CPT = latent columns per thread.
template <typename T, int CPT>
__global__ __launch_bounds__(kGenThreads) void attn_generic_kernel(
    const T* __restrict__ ke_plane, const T* __restrict__ c_plane, const float* __restrict__ qe,
    const float* __restrict__ qt, const int32_t* __restrict__ seq_len, float* __restrict__ part_m,
    float* __restrict__ part_l, float* __restrict__ part_u, int n_h, int two_r, int d_c, int d_q, int d_u,
    int64_t max_seq_len, int64_t batch_stride_rows, int64_t plane_rows, int n_splits, int chunk, int q_per_seq) {
  extern __shared__ float smem[];
  // a cache row holds d_c latent columns: the first d_q of them enter the scores, the last d_u are
  // accumulated as values (joint latent: d_q = d_u = d_c, the same columns serve both)
  float* qt_s = smem;                 // [d_q]
  float* qe_s = qt_s + d_q;           // [two_r]
  float* s_tile = qe_s + two_r;       // [kGenTile]
  float* p_tile = s_tile + kGenTile;  // [kGenTile]

  const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  const int64_t row0 = (int64_t)(b / q_per_seq) * batch_stride_rows;
  int64_t len = seq_len[b];
  len = min(len, max_seq_len);
  len = min(len, plane_rows - row0);
  len = max(len, (int64_t)0);
  const int64_t t0 = (int64_t)split * chunk;
  const int64_t t1 = min(t0 + chunk, len);

  const int v0 = d_c - d_u;
  for (int k = tid; k < d_q; k += kGenThreads) qt_s[k] = qt[((int64_t)b * n_h + h) * d_q + k];
  for (int e = tid; e < two_r; e += kGenThreads) qe_s[e] = qe[((int64_t)b * n_h + h) * two_r + e];
  __syncthreads();

  float acc[CPT];
#pragma unroll
  for (int i = 0; i < CPT; ++i) acc[i] = 0.f;
  float m = -INFINITY, l = 0.f;

  for (int64_t tile = t0; tile < t1; tile += kGenTile) {
    const int nt = (int)min((int64_t)kGenTile, t1 - tile);
    // scores: each wave takes 16 tokens, lanes split the contraction
    for (int tt = 0; tt < kGenTile / 4; ++tt) {
      const int ti = wave * (kGenTile / 4) + tt;
      float part = 0.f;
      if (ti < nt) {
        const int64_t row = row0 + tile + ti;
        const T* crow = c_plane + row * d_c;
        for (int k = lane; k < d_q; k += 64) part = fmaf(qt_s[k], ld(crow, k), part);
        const T* krow = ke_plane + (row * n_h + h) * two_r;
        for (int e = lane; e < two_r; e += 64) part = fmaf(qe_s[e], ld(krow, e), part);
      }
      part = wave_sum(part);
      if (lane == 0) s_tile[ti] = (ti < nt) ? part : -INFINITY;
    }
    __syncthreads();
    const float sv = s_tile[lane];
    const float m_new = fmaxf(m, wave_max(sv));
    const float alpha = exp2f(m - m_new);   // m = -inf on the first tile gives 0
    const float p = exp2f(sv - m_new);      // -inf score gives 0
    l = l * alpha + wave_sum(p);
    if (wave == 0) p_tile[lane] = p;
    __syncthreads();
#pragma unroll
    for (int cc = 0; cc < CPT; ++cc) {
      const int k = tid + cc * kGenThreads;
      if (k < d_u) {
        float a = acc[cc] * alpha;
        const T* col = c_plane + (row0 + tile) * d_c + v0 + k;
        for (int tt = 0; tt < nt; ++tt) a = fmaf(p_tile[tt], ld(col, (int64_t)tt * d_c), a);
        acc[cc] = a;
      }
    }
    m = m_new;
    __syncthreads();
  }

  const int64_t pi = ((int64_t)b * n_splits + split) * n_h + h;
  if (tid == 0) {
    part_m[pi] = m;
    part_l[pi] = l;
  }
#pragma unroll
  for (int cc = 0; cc < CPT; ++cc) {
    const int k = tid + cc * kGenThreads;
    if (k < d_u) part_u[pi * d_u + k] = acc[cc];
  }
}

// One work-group per (head, batch row): merge the splits, normalise, apply W_uv.
template <typename T>
__global__ __launch_bounds__(kGenThreads) void merge_upproj_generic_kernel(
    const float* __restrict__ part_m, const float* __restrict__ part_l,
    const float* __restrict__ part_u, const T* __restrict__ W_uv, T* __restrict__ out, int n_h,
    int d_h, int d_c, int n_splits) {
  extern __shared__ float smem[];
  float* ubar = smem;            // [d_c]
  float* w = ubar + d_c;         // [n_splits]
  float* red = w + n_splits;     // [kGenThreads]
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
  const int64_t base = (int64_t)b * n_splits * n_h + h;

  float m = -INFINITY;
  for (int s = tid; s < n_splits; s += kGenThreads) m = fmaxf(m, part_m[base + (int64_t)s * n_h]);
  red[tid] = m;
  __syncthreads();
  for (int o = kGenThreads / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] = fmaxf(red[tid], red[tid + o]);
    __syncthreads();
  }
  m = red[0];
  __syncthreads();
  float lsum = 0.f;
  for (int s = tid; s < n_splits; s += kGenThreads) {
    const float ls = part_l[base + (int64_t)s * n_h];
    const float ws = (ls > 0.f) ? exp2f(part_m[base + (int64_t)s * n_h] - m) : 0.f;
    w[s] = ws;
    lsum += ws * ls;
  }
  red[tid] = lsum;
  __syncthreads();
  for (int o = kGenThreads / 2; o > 0; o >>= 1) {
    if (tid < o) red[tid] += red[tid + o];
    __syncthreads();
  }
  const float L = red[0];
  const float inv = (L > 0.f) ? 1.f / L : 0.f;
  __syncthreads();
  for (int k = tid; k < d_c; k += kGenThreads) {
    float a = 0.f;
    for (int s = 0; s < n_splits; ++s) {
      const float ws = w[s];
      if (ws != 0.f) a = fmaf(ws, part_u[(base + (int64_t)s * n_h) * d_c + k], a);
    }
    ubar[k] = a * inv;
  }
  __syncthreads();
  // out[b,h,j] = sum_k ubar[k] W_uv[k,h,j]; thread groups split k (d_h <= 256 checked on the host)
  const int groups = kGenThreads / d_h;
  const int j = tid % d_h, g = tid / d_h;
  float a = 0.f;
  if (g < groups)
    for (int k = g; k < d_c; k += groups) a = fmaf(ubar[k], ld(W_uv, ((int64_t)k * n_h + h) * d_h + j), a);
  red[tid] = a;
  __syncthreads();
  if (tid < d_h) {
    float tot = 0.f;
    for (int gg = 0; gg < groups; ++gg) tot += red[gg * d_h + tid];
    st(out, ((int64_t)b * n_h + h) * d_h + tid, tot);
  }
}

template <typename T>
static hipError_t launch_decode_generic_t(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int n_h = d.n_heads, d_h = d.head_dim, r = d.r, d_c = d.d_c, d_q = p.d_q, d_u = p.d_u;
  float* qe = (float*)(a.ws + p.off_qe);
  float* qt = (float*)(a.ws + p.off_qt);
  float* pm = (float*)(a.ws + p.off_m);
  float* pl = (float*)(a.ws + p.off_l);
  float* pu = (float*)(a.ws + p.off_u);
  const float scale_log2e = kLog2e / sqrtf((float)d_h);

  if (a.stages & 1)
    qprep_generic_kernel<T><<<dim3(n_h, (unsigned)a.B), kGenThreads, 0, stream>>>(
        (const T*)a.q, a.q_pos, (const T*)a.W_uk, a.elite_idx, qe, qt, n_h, d_h, r, d_q,
        rope_table(d.rope_base, d.head_dim), scale_log2e);

  const dim3 grid(p.n_splits, n_h, (unsigned)a.B);
  const size_t sm = sizeof(float) * (size_t)(d_q + 2 * r + 2 * kGenTile);
  const int cpt = (d_u + kGenThreads - 1) / kGenThreads;
#define EKV_ATTN(C)                                                                               \
  attn_generic_kernel<T, C><<<grid, kGenThreads, sm, stream>>>(                                   \
      (const T*)a.ke_plane, (const T*)a.c_plane, qe, qt, a.seq_len, pm, pl, pu, n_h, 2 * r, d_c, d_q, d_u, \
      a.max_seq_len, a.batch_stride_rows, a.plane_rows, p.n_splits, p.chunk, a.q_per_seq)
  if (!(a.stages & 2)) {}
  else if (cpt <= 1) EKV_ATTN(1);
  else if (cpt <= 2) EKV_ATTN(2);
  else if (cpt <= 4) EKV_ATTN(4);
  else if (cpt <= 8) EKV_ATTN(8);
  else EKV_ATTN(16);
#undef EKV_ATTN

  if (!(a.stages & 4)) return hipGetLastError();
  const size_t sm2 = sizeof(float) * (size_t)(d_u + p.n_splits + kGenThreads);
  merge_upproj_generic_kernel<T><<<dim3(n_h, (unsigned)a.B), kGenThreads, sm2, stream>>>(
      pm, pl, pu, (const T*)a.W_uv, (T*)a.out, n_h, d_h, d_u, p.n_splits);
  return hipGetLastError();
}

hipError_t launch_decode_generic(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  if (a.dims.dtype == ELITEKV_FP32) return launch_decode_generic_t<float>(a, p, stream);
  return launch_decode_generic_t<bf16_t>(a, p, stream);
}

}  // namespace ekv
