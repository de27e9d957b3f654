// C-ABI entry points of libelitekv: host-side validation, split planning, workspace layout.
// Nothing here touches the device except through the launchers, and nothing allocates.
#include <math.h>
#include <string.h>

#include "launch.hpp"

// Built-in scratch of elitekv_decode_attn_noalloc: device memory that belongs to the library's code
// object (every GPU the library runs on holds its own copy until the process ends).  In host code the
// array's NAME is only a handle for hipGetSymbolAddress; kernels are given the looked-up address.
static __device__ __align__(256) unsigned char scratch[ELITEKV_NOALLOC_SCRATCH_BYTES];

namespace ekv {

// Device address of `scratch` on the current device, looked up once per device; nullptr on error.
static void* scratch_ptr() {
  static std::atomic<void*> addr[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = addr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  addr[dev].store(p, std::memory_order_release);
  return p;
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return (((uintptr_t)p) & 15u) == 0; }

static int check_dims(const elitekv_dims* d) {
  if (!d) return ELITEKV_ENULL;
  if (d->d_model <= 0 || d->n_heads <= 0 || d->head_dim <= 0 || (d->head_dim & 1)) return ELITEKV_EINVAL;
  if (d->r < 0 || 2 * d->r > d->head_dim || d->d_c <= 0) return ELITEKV_EINVAL;
  if (d->dtype != ELITEKV_FP32 && d->dtype != ELITEKV_BF16) return ELITEKV_EINVAL;
  if (!(d->rope_base > 0.0) || !isfinite(d->rope_base)) return ELITEKV_EINVAL;
  return ELITEKV_OK;
}

static inline size_t elem_bytes(const elitekv_dims* d) { return d->dtype == ELITEKV_FP32 ? 4 : 2; }

constexpr int kMaxSplits = 1024;
constexpr int kComputeUnits = 256;  // MI355X
constexpr int kTargetGroups = 1024;   // generic path: work-groups wanted in flight

static int32_t auto_splits_generic(const elitekv_dims* d, int64_t B, int64_t max_seq) {
  const int64_t per_split_min = 64;
  int64_t want = (kTargetGroups + B * d->n_heads - 1) / (B * d->n_heads);
  int64_t cap = (max_seq + per_split_min - 1) / per_split_min;
  if (want > cap) want = cap;
  if (want > kMaxSplits) want = kMaxSplits;
  if (want < 1) want = 1;
  return (int32_t)want;
}

// Decide the path and lay the workspace out.  Returns a status.
// d_ck = 0: joint latent; d_ck > 0: separated latents, a cache row is [c^k (d_ck) | c^v (d_c - d_ck)]
// want_fresh: plan the fused decode step (the newest token enters as one more split) if the kernels cover it
// block: plan the whole-block step (EUNSUPPORTED unless the fused step's kernels cover the shape)
static int plan_decode(const elitekv_dims* d, int32_t d_ck, int64_t B, int64_t max_seq, int32_t n_splits,
                       DecodePlan* p, bool want_fresh = false, bool block = false) {
  int st = check_dims(d);
  if (st) return st;
  if (B < 0 || max_seq < 0 || n_splits < 0) return ELITEKV_EINVAL;
  if (d_ck < 0 || d_ck >= d->d_c) return ELITEKV_EINVAL;
  if (d->d_c > 4096 || d->head_dim > 256 || n_splits > kMaxSplits) return ELITEKV_EUNSUPPORTED;
  if (B > 65535) return ELITEKV_EUNSUPPORTED;
  memset(p, 0, sizeof(*p));
  const int64_t Bq = B > 0 ? B : 1;
  const int64_t seq = max_seq > 0 ? max_seq : 1;
  const size_t nh = d->n_heads, Bz = (size_t)B;
  p->d_q = d_ck > 0 ? d_ck : d->d_c;
  p->d_u = d_ck > 0 ? d->d_c - d_ck : d->d_c;
  const size_t dq = p->d_q, du = p->d_u;
  size_t off = 0;
  p->off_qe = off; off = align_up(off + Bz * nh * 2 * d->r * sizeof(float), 256);
  if (decode_mfma_supported(*d, d_ck)) {
    // one work-group per (split, group of 32 heads, batch row); one group fills a compute unit
    p->mfma = 1;
    p->head_groups = (d->n_heads + 31) / 32;
    int ks = 0, kc = 0;
    if (want_fresh && B > 0 && decode_front_plan(*d, d_ck, p->d_q, B, &ks, &kc)) {
      p->fresh = 1; p->fr_ks = ks; p->fr_kc = kc;
      p->fr_stride = 2 * d->r * d->n_heads + d->d_c;
    } else if (want_fresh && !block && B > 0 && decode_front_mfma_plan(*d, d_ck, p->d_q, B, &ks, &kc)) {
      p->fresh = 2; p->fr_ks = ks; p->fr_kc = kc;
      p->fr_stride = 2 * d->r * d->n_heads + d->d_c;
    }
    if (block) {
      int yks = 0, ykc = 0;
      if (!p->fresh || d_ck != 0 || !block_step_plan(*d, B, &ks, &kc, &yks, &ykc)) return ELITEKV_EUNSUPPORTED;
      p->fr_ks = ks; p->fr_kc = kc; p->y_ks = yks; p->y_kc = ykc;
      p->fr_stride += d->n_heads * d->head_dim;            // x W_q is computed alongside the cache row
    }
    int64_t ns = n_splits;
    if (ns == 0) {
      // the narrow-latent instantiations run two work-groups per compute unit; with many batch rows
      // it pays to give every compute unit two (more splits also mean more partials to merge)
      const int64_t want = (decode_mfma_groups_per_cu(*d) == 2 && Bq * p->head_groups >= 16) ? 2 * kComputeUnits
                                                                                            : kComputeUnits;
      ns = (want + Bq * p->head_groups - 1) / (Bq * p->head_groups);
      const int64_t cap = (seq + 15) / 16;
      if (ns > cap) ns = cap;
      if (ns > kMaxSplits) ns = kMaxSplits;
      if (ns < 1) ns = 1;
    }
    p->n_splits = (int32_t)ns;
    p->n_part = (int32_t)ns;
    int64_t chunk = (seq + ns - 1) / ns;
    chunk = (chunk + 31) / 32 * 32;
    p->chunk = (int32_t)chunk;
    const size_t np = Bz * (size_t)p->n_part * p->head_groups;
    p->off_qt = off; off = align_up(off + Bz * (size_t)p->head_groups * 32 * dq * 2, 256);   // head groups padded to 32
    p->off_m = off;  off = align_up(off + np * 32 * sizeof(float), 256);
    p->off_l = off;  off = align_up(off + np * 32 * sizeof(float), 256);
    p->off_u = off;  off = align_up(off + np * 32 * du * 2, 256);
    p->merge_batch = merge_mfma_supported(*d, p->d_u, B, p->n_part) ? 1 : 0;
    p->up_cw = p->merge_batch ? 128 : (p->d_u % 192 == 0) ? 192 : 64;
    p->off_opart = off;
    off = align_up(off + Bz * nh * (size_t)(p->d_u / p->up_cw) * d->head_dim * sizeof(float), 256);
    p->off_cnt = off;
    off = align_up(off + Bz * nh * sizeof(int32_t), 256);
    if (p->fresh) {
      p->off_apart = off;
      off = align_up(off + (size_t)p->fr_ks * Bz * (size_t)p->fr_stride * sizeof(float), 256);
      p->off_sincos = off;
      off = align_up(off + Bz * nh * (size_t)d->r * 2 * sizeof(float), 256);
    }
    if (block) {
      p->off_qfin = off;
      off = align_up(off + Bz * nh * (size_t)d->head_dim * 2, 256);
      p->off_ypart = off;
      off = align_up(off + (size_t)p->y_ks * Bz * (size_t)d->d_model * sizeof(float), 256);
    }
  } else {
    if (block) return ELITEKV_EUNSUPPORTED;
    p->mfma = 0;
    p->head_groups = 1;
    p->n_splits = n_splits > 0 ? n_splits : auto_splits_generic(d, Bq, seq);
    p->n_part = p->n_splits;
    int64_t chunk = (seq + p->n_splits - 1) / p->n_splits;
    if (chunk < 1) chunk = 1;
    p->chunk = (int32_t)chunk;
    const size_t ns = p->n_splits;
    p->off_qt = off; off = align_up(off + Bz * nh * dq * sizeof(float), 256);
    p->off_m = off;  off = align_up(off + Bz * ns * nh * sizeof(float), 256);
    p->off_l = off;  off = align_up(off + Bz * ns * nh * sizeof(float), 256);
    p->off_u = off;  off = align_up(off + Bz * ns * nh * du * sizeof(float), 256);
  }
  p->total = off;
  return ELITEKV_OK;
}

static int plan_mha(const elitekv_dims* d, int64_t B, int64_t max_seq, int32_t n_splits, int32_t* ns_out,
                    int32_t* chunk_out, size_t* bytes) {
  int st = check_dims(d);
  if (st) return st;
  if (B < 0 || max_seq < 0 || n_splits < 0) return ELITEKV_EINVAL;
  if (n_splits > kMaxSplits || d->head_dim > 256) return ELITEKV_EUNSUPPORTED;
  const int vec = d->dtype == ELITEKV_FP32 ? 4 : 8;
  const int lpr = d->head_dim / vec;
  if (d->head_dim % vec || lpr < 2 || lpr > 64 || (lpr & (lpr - 1))) return ELITEKV_EUNSUPPORTED;
  const int64_t Bq = B > 0 ? B : 1;
  int32_t ns = n_splits > 0 ? n_splits : auto_splits_generic(d, Bq, max_seq > 0 ? max_seq : 1);
  int64_t chunk = (max_seq + ns - 1) / ns;
  if (chunk < 1) chunk = 1;
  *ns_out = ns;
  *chunk_out = (int32_t)chunk;
  *bytes = align_up((size_t)B * ns * d->n_heads * (2 + d->head_dim) * sizeof(float), 256);
  return ELITEKV_OK;
}

}  // namespace ekv

using namespace ekv;

extern "C" {

const char* elitekv_strerror(int status) {
  switch (status) {
    case ELITEKV_OK: return "ok";
    case ELITEKV_EINVAL: return "invalid dimensions or counts";
    case ELITEKV_EINDEX: return "elite index out of range or repeated within a head";
    case ELITEKV_ENULL: return "required pointer is NULL";
    case ELITEKV_EALIGN: return "pointer or stride is not 16-byte aligned";
    case ELITEKV_EWORKSPACE: return "workspace too small";
    case ELITEKV_EUNSUPPORTED: return "shape not covered by the kernels";
    case ELITEKV_EHIP: return "HIP launch error";
    case ELITEKV_ESCRATCH: return "call needs more than the built-in scratch buffer holds";
    default: return "unknown status";
  }
}

int elitekv_cache_row_elems(const elitekv_dims* dims, int64_t* ke_elems, int64_t* c_elems) {
  int st = check_dims(dims);
  if (st) return st;
  if (!ke_elems || !c_elems) return ELITEKV_ENULL;
  *ke_elems = 2LL * dims->r * dims->n_heads;
  *c_elems = dims->d_c;
  return ELITEKV_OK;
}

int elitekv_param_count(const elitekv_dims* dims, int64_t* n_params) {
  int st = check_dims(dims);
  if (st) return st;
  if (!n_params) return ELITEKV_ENULL;
  const int64_t d = dims->d_model, nh = dims->n_heads, dh = dims->head_dim, r = dims->r, dc = dims->d_c;
  *n_params = 2 * r * nh * d + dc * (d + 2 * dh * nh - 2 * r * nh);
  return ELITEKV_OK;
}

int elitekv_validate_elite_idx(const elitekv_dims* dims, const int32_t* idx_host) {
  int st = check_dims(dims);
  if (st) return st;
  if (dims->r == 0) return ELITEKV_OK;
  if (!idx_host) return ELITEKV_ENULL;
  const int half = dims->head_dim / 2, r = dims->r;
  for (int h = 0; h < dims->n_heads; ++h) {
    for (int j = 0; j < r; ++j) {
      const int32_t i = idx_host[h * r + j];
      if (i < 0 || i >= half) return ELITEKV_EINDEX;
      for (int k = 0; k < j; ++k)
        if (idx_host[h * r + k] == i) return ELITEKV_EINDEX;
    }
  }
  return ELITEKV_OK;
}

// d_ck = columns of the first latent weight matrix (d_c for the joint latent)
static size_t append_ws_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t T) {
  if (check_dims(dims) || T < 0) return 0;
  if (T > 0 && append_gemm_supported(*dims, T, d_ck)) return 0;
  if (T > 0 && append_skinny_supported(*dims, T, d_ck)) return align_up(append_skinny_workspace(*dims, T), 256);
  if (T > 0 && append_small_supported(*dims, T, d_ck)) return align_up(append_small_workspace(*dims, T), 256);
  return 0;
}

// argument checks of an append; ws_needed = 0 skips the workspace check
static int append_check(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                        const int64_t* slot, int64_t T, const void* W_ke, const void* W_dkv, const void* W_dkv2,
                        const int32_t* elite_idx, const void* ke_plane, const void* c_plane, int64_t plane_rows,
                        const void* ws, size_t ws_bytes, size_t ws_needed) {
  int st = check_dims(dims);
  if (st) return st;
  if (T < 0 || plane_rows < 0 || d_ck <= 0 || d_ck > dims->d_c) return ELITEKV_EINVAL;
  if (dims->head_dim > 256) return ELITEKV_EUNSUPPORTED;     // the kernels' RoPE table holds 128 chunk frequencies
  if (T == 0) return ELITEKV_OK;
  if (!x || !pos || !slot || !W_dkv || !c_plane) return ELITEKV_ENULL;
  if (d_ck < dims->d_c && !W_dkv2) return ELITEKV_ENULL;
  if (dims->r > 0 && (!W_ke || !elite_idx || !ke_plane)) return ELITEKV_ENULL;
  if (!aligned16(x) || !aligned16(W_dkv) || !aligned16(W_dkv2) || !aligned16(c_plane) || !aligned16(W_ke) ||
      !aligned16(ke_plane) || !aligned16(ws))
    return ELITEKV_EALIGN;
  if (ws_needed > 0 && (!ws || ws_bytes < ws_needed)) return ws ? ELITEKV_EWORKSPACE : ELITEKV_ENULL;
  if ((T + 7) / 8 > 2147483647LL) return ELITEKV_EUNSUPPORTED;
  return ELITEKV_OK;
}

static AppendArgs append_args(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                              const int64_t* slot, int64_t T, const void* W_ke, const void* W_dkv,
                              const void* W_dkv2, const int32_t* elite_idx, void* ke_plane, void* c_plane,
                              int64_t plane_rows, void* ws) {
  AppendArgs a;
  a.dims = *dims; a.d_ck = d_ck; a.x = x; a.pos = pos; a.slot = slot; a.T = T; a.W_ke = W_ke; a.W_dkv = W_dkv;
  a.W_dkv2 = W_dkv2; a.elite_idx = elite_idx; a.ke_plane = ke_plane; a.c_plane = c_plane;
  a.plane_rows = plane_rows; a.ws = (char*)ws;
  return a;
}

static hipError_t append_dispatch(const AppendArgs& a, hipStream_t stream) {
  const elitekv_dims* dims = &a.dims;
  return append_gemm_supported(*dims, a.T, a.d_ck)     ? launch_append_gemm(a, stream)
         : append_skinny_supported(*dims, a.T, a.d_ck) ? launch_append_skinny(a, stream)
         : append_small_supported(*dims, a.T, a.d_ck)  ? launch_append_small(a, stream)
                                                       : launch_append_generic(a, stream);
}

static int append_impl(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                       const int64_t* slot, int64_t T, const void* W_ke, const void* W_dkv, const void* W_dkv2,
                       const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows, void* ws,
                       size_t ws_bytes, void* hip_stream) {
  const int st = append_check(dims, d_ck, x, pos, slot, T, W_ke, W_dkv, W_dkv2, elite_idx, ke_plane, c_plane,
                              plane_rows, ws, ws_bytes, dims ? append_ws_bytes(dims, d_ck, T) : 0);
  if (st || T == 0) return st;
  const AppendArgs a = append_args(dims, d_ck, x, pos, slot, T, W_ke, W_dkv, W_dkv2, elite_idx, ke_plane,
                                   c_plane, plane_rows, ws);
  return append_dispatch(a, (hipStream_t)hip_stream) == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

size_t elitekv_append_workspace_bytes(const elitekv_dims* dims, int64_t T) {
  return dims ? append_ws_bytes(dims, dims->d_c, T) : 0;
}

int elitekv_append(const elitekv_dims* dims, const void* x, const int32_t* pos, const int64_t* slot,
                   int64_t T, const void* W_ke, const void* W_dkv, const int32_t* elite_idx,
                   void* ke_plane, void* c_plane, int64_t plane_rows, void* ws, size_t ws_bytes,
                   void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  return append_impl(dims, dims->d_c, x, pos, slot, T, W_ke, W_dkv, nullptr, elite_idx, ke_plane, c_plane,
                     plane_rows, ws, ws_bytes, hip_stream);
}

int elitekv_decode_path(const elitekv_dims* dims, int32_t d_ck) {
  DecodePlan p;
  const int st = plan_decode(dims, d_ck, 1, 16, 0, &p);
  if (st) return st;
  return p.mfma ? ELITEKV_PATH_MATRIX_CORE : ELITEKV_PATH_GENERIC;
}

int32_t elitekv_decode_auto_splits(const elitekv_dims* dims, int64_t B, int64_t max_seq_len) {
  DecodePlan p;
  if (plan_decode(dims, 0, B, max_seq_len, 0, &p)) return 0;
  return p.n_splits;
}

size_t elitekv_decode_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len,
                                      int32_t n_splits) {
  DecodePlan p;
  if (plan_decode(dims, 0, B, max_seq_len, n_splits, &p)) return 0;
  return p.total;
}

static int decode_check(const elitekv_dims* dims, const DecodePlan& p, const void* q, const int32_t* q_pos,
                        const int32_t* seq_len, int64_t B, int64_t batch_stride_rows, const void* W_uk,
                        const void* W_uv, const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                        int64_t plane_rows, const void* out, const void* ws, size_t ws_bytes) {
  if (batch_stride_rows < 0 || plane_rows < 0) return ELITEKV_EINVAL;
  if (B == 0) return ELITEKV_OK;
  if (B > 65535) return ELITEKV_EUNSUPPORTED;
  if (!q || !q_pos || !seq_len || !W_uv || !c_plane || !out || !ws) return ELITEKV_ENULL;
  if (dims->r > 0 && (!elite_idx || !ke_plane)) return ELITEKV_ENULL;
  if (2 * dims->r < dims->head_dim && !W_uk) return ELITEKV_ENULL;
  if (!aligned16(q) || !aligned16(W_uk) || !aligned16(W_uv) || !aligned16(ke_plane) ||
      !aligned16(c_plane) || !aligned16(out) || !aligned16(ws))
    return ELITEKV_EALIGN;
  if (ws_bytes < p.total) return ELITEKV_EWORKSPACE;
  return ELITEKV_OK;
}

static DecodeArgs decode_args(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                              const int32_t* seq_len, int64_t B, int64_t max_seq_len, int64_t batch_stride_rows,
                              const void* W_uk, const void* W_uv, const int32_t* elite_idx, const void* ke_plane,
                              const void* c_plane, int64_t plane_rows, void* out, void* ws, int32_t stages,
                              int32_t q_per_seq) {
  DecodeArgs a;
  a.dims = *dims; a.d_ck = d_ck; a.q = q; a.q_pos = q_pos; a.seq_len = seq_len; a.B = B;
  a.max_seq_len = max_seq_len; a.batch_stride_rows = batch_stride_rows; a.W_uk = W_uk; a.W_uv = W_uv;
  a.elite_idx = elite_idx; a.ke_plane = ke_plane; a.c_plane = c_plane; a.plane_rows = plane_rows; a.out = out;
  a.ws = (char*)ws; a.stages = stages; a.q_per_seq = q_per_seq;
  a.fr_slot = nullptr; a.fr_ke_out = nullptr; a.fr_c_out = nullptr;
  a.no_out_reduce = 0;
  return a;
}

static int decode_impl(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                       const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                       int64_t batch_stride_rows, const void* W_uk, const void* W_uv,
                       const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                       int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                       void* hip_stream, int32_t stages, int32_t q_per_seq = 1) {
  DecodePlan p;
  int st = plan_decode(dims, d_ck, B, max_seq_len, n_splits, &p);
  if (st) return st;
  st = decode_check(dims, p, q, q_pos, seq_len, B, batch_stride_rows, W_uk, W_uv, elite_idx, ke_plane, c_plane,
                    plane_rows, out, ws, ws_bytes);
  if (st || B == 0) return st;
  const DecodeArgs a = decode_args(dims, d_ck, q, q_pos, seq_len, B, max_seq_len, batch_stride_rows, W_uk, W_uv,
                                   elite_idx, ke_plane, c_plane, plane_rows, out, ws, stages, q_per_seq);
  const hipError_t e = p.mfma ? launch_decode_mfma(a, p, (hipStream_t)hip_stream)
                             : launch_decode_generic(a, p, (hipStream_t)hip_stream);
  return e == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

/* ---- fused decode step: append of the step's tokens + attention ---- */

// workspace = [decode workspace (with the fused step's extra pieces) | append workspace of B tokens]
static size_t step_ws_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t max_seq_len, int32_t n_splits) {
  DecodePlan p;
  if (plan_decode(dims, d_ck, B, max_seq_len, n_splits, &p, true)) return 0;
  return p.total + (p.fresh ? 0 : append_ws_bytes(dims, d_ck > 0 ? d_ck : dims->d_c, B));
}

static int step_impl(const elitekv_dims* dims, int32_t d_ck, const void* x, const void* q, const int32_t* pos,
                     const int64_t* slot, const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                     int64_t batch_stride_rows, const void* W_ke, const void* W_dkv, const void* W_dkv2,
                     const void* W_uk, const void* W_uv, const int32_t* elite_idx, void* ke_plane, void* c_plane,
                     int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits, void* hip_stream) {
  DecodePlan p;
  int st = plan_decode(dims, d_ck, B, max_seq_len, n_splits, &p, true);
  if (st) return st;
  const int32_t a_ck = d_ck > 0 ? d_ck : dims->d_c;          // columns of the first latent weight matrix
  st = append_check(dims, a_ck, x, pos, slot, B, W_ke, W_dkv, W_dkv2, elite_idx, ke_plane, c_plane, plane_rows, ws,
                    ws_bytes, 0);
  if (st) return st;
  st = decode_check(dims, p, q, pos, seq_len, B, batch_stride_rows, W_uk, W_uv, elite_idx, ke_plane, c_plane,
                    plane_rows, out, ws, ws_bytes);
  if (st || B == 0) return st;
  const size_t need = p.total + (p.fresh ? 0 : append_ws_bytes(dims, a_ck, B));
  if (ws_bytes < need) return ELITEKV_EWORKSPACE;
  const hipStream_t stream = (hipStream_t)hip_stream;
  const AppendArgs ap = append_args(dims, a_ck, x, pos, slot, B, W_ke, W_dkv, W_dkv2, elite_idx, ke_plane, c_plane,
                                    plane_rows, (char*)ws + p.total);
  DecodeArgs a = decode_args(dims, d_ck, q, pos, seq_len, B, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                             ke_plane, c_plane, plane_rows, out, ws, 7, 1);
  hipError_t e;
  if (p.fresh) {
    // front kernel (first pass of the append + query preparation), then attention (whose owner
    // work-groups finish the append), merge and up-projection
    a.fr_slot = slot; a.fr_ke_out = ke_plane; a.fr_c_out = c_plane;
    e = p.fresh == 2 ? launch_decode_front_mfma(ap, a, p, stream) : launch_decode_front(ap, a, p, stream);
    a.stages = 6;
    if (e == hipSuccess) e = launch_decode_mfma(a, p, stream);
  } else if (decode_front_mfma_supported(ap, a, p)) {
    // batches: first pass of the append + query preparation in one launch, the append's finishing
    // launch, then attention, merge and up-projection
    e = launch_decode_front_mfma(ap, a, p, stream);
    a.stages = 6;
    if (e == hipSuccess) e = launch_decode_mfma(a, p, stream);
  } else {
    e = append_dispatch(ap, stream);
    if (e == hipSuccess) e = p.mfma ? launch_decode_mfma(a, p, stream) : launch_decode_generic(a, p, stream);
  }
  return e == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

size_t elitekv_decode_step_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len,
                                           int32_t n_splits) {
  return step_ws_bytes(dims, 0, B, max_seq_len, n_splits);
}

int elitekv_decode_step(const elitekv_dims* dims, const void* x, const void* q, const int32_t* pos,
                        const int64_t* slot, const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                        int64_t batch_stride_rows, const void* W_ke, const void* W_dkv, const void* W_uk,
                        const void* W_uv, const int32_t* elite_idx, void* ke_plane, void* c_plane,
                        int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                        void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  return step_impl(dims, 0, x, q, pos, slot, seq_len, B, max_seq_len, batch_stride_rows, W_ke, W_dkv, nullptr, W_uk,
                   W_uv, elite_idx, ke_plane, c_plane, plane_rows, out, ws, ws_bytes, n_splits, hip_stream);
}

/* ---- whole attention block of a decode step ---- */

// Plain projection out = in W of up to 64 rows (in [T, d_in], W [d_in, N], out [T, N], all bf16) through the
// weight-streaming append kernels (r = 0: no elite columns, no rotation; the latent columns are the output).
static elitekv_dims projection_dims(const elitekv_dims* dims, int d_in, int N) {
  elitekv_dims pd = *dims;
  pd.d_model = d_in; pd.n_heads = 1; pd.head_dim = 2; pd.r = 0; pd.d_c = N;
  return pd;
}
static bool projection_supported(const elitekv_dims* dims, int64_t T, int d_in, int N) {
  const elitekv_dims pd = projection_dims(dims, d_in, N);
  return T >= 1 && T <= 64 && (append_skinny_supported(pd, T, N) || append_small_supported(pd, T, N));
}
static size_t projection_ws_bytes(const elitekv_dims* dims, int64_t T, int d_in, int N) {
  const elitekv_dims pd = projection_dims(dims, d_in, N);
  return append_ws_bytes(&pd, N, T);
}
static hipError_t launch_projection(const elitekv_dims* dims, const void* in, const void* W, int64_t T, int d_in, int N,
                                    void* out, void* ws, hipStream_t stream) {
  const elitekv_dims pd = projection_dims(dims, d_in, N);
  AppendArgs a = append_args(&pd, N, in, nullptr, nullptr, T, nullptr, W, nullptr, nullptr, nullptr, nullptr, 0, ws);
  a.dense_out = out;
  return append_skinny_supported(pd, T, N) ? launch_append_skinny(a, stream) : launch_append_small(a, stream);
}

// The composed form of the block step, for what the fused form does not cover (eight sequences and more, separated
// latents): q = x W_q, the decode step, y = out W_o as launches of their own, q and out staying in the workspace.
// Workspace: [decode-step workspace | q bf16 [B, n_h d_h] | out bf16 [B, n_h d_h] | projection partial sums].
struct BlockLayout { size_t step, off_q, off_o, off_proj, total; };
static bool block_composed_layout(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t max_seq_len,
                                  int32_t n_splits, BlockLayout* L) {
  if (check_dims(dims) || dims->dtype != ELITEKV_BF16 || B < 1 || B > 64) return false;
  const int hd = dims->n_heads * dims->head_dim;
  if (!projection_supported(dims, B, dims->d_model, hd) || !projection_supported(dims, B, hd, dims->d_model)) return false;
  L->step = step_ws_bytes(dims, d_ck, B, max_seq_len, n_splits);
  if (L->step == 0) return false;
  size_t off = align_up(L->step, 256);
  L->off_q = off; off = align_up(off + (size_t)B * hd * 2, 256);
  L->off_o = off; off = align_up(off + (size_t)B * hd * 2, 256);
  L->off_proj = off;
  const size_t pq = projection_ws_bytes(dims, B, dims->d_model, hd), po = projection_ws_bytes(dims, B, hd, dims->d_model);
  L->total = align_up(off + (pq > po ? pq : po), 256);
  return true;
}

static int block_composed_impl(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                               const int64_t* slot, const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                               int64_t batch_stride_rows, const void* W_q, const void* W_ke, const void* W_dkv,
                               const void* W_dkv2, const void* W_uk, const void* W_uv, const void* W_o,
                               const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows, void* y,
                               void* ws, size_t ws_bytes, int32_t n_splits, void* hip_stream) {
  BlockLayout L;
  if (!block_composed_layout(dims, d_ck, B, max_seq_len, n_splits, &L)) return ELITEKV_EUNSUPPORTED;
  if (!x || !W_q || !W_o || !y || !ws) return ELITEKV_ENULL;
  if (!aligned16(x) || !aligned16(W_q) || !aligned16(W_o) || !aligned16(y) || !aligned16(ws)) return ELITEKV_EALIGN;
  if (ws_bytes < L.total) return ELITEKV_EWORKSPACE;
  char* w = (char*)ws;
  const int hd = dims->n_heads * dims->head_dim;
  const hipStream_t stream = (hipStream_t)hip_stream;
  // the step's own argument checks come first (nothing is enqueued on an error): a dry plan + check
  {
    DecodePlan p;
    int st = plan_decode(dims, d_ck, B, max_seq_len, n_splits, &p, true);
    if (st) return st;
    const int32_t a_ck = d_ck > 0 ? d_ck : dims->d_c;
    st = append_check(dims, a_ck, x, pos, slot, B, W_ke, W_dkv, W_dkv2, elite_idx, ke_plane, c_plane, plane_rows, ws,
                      ws_bytes, 0);
    if (st) return st;
    st = decode_check(dims, p, x, pos, seq_len, B, batch_stride_rows, W_uk, W_uv, elite_idx, ke_plane, c_plane,
                      plane_rows, y, ws, ws_bytes);
    if (st) return st;
  }
  if (launch_projection(dims, x, W_q, B, dims->d_model, hd, w + L.off_q, w + L.off_proj, stream) != hipSuccess)
    return ELITEKV_EHIP;
  const int st = step_impl(dims, d_ck, x, w + L.off_q, pos, slot, seq_len, B, max_seq_len, batch_stride_rows, W_ke, W_dkv,
                           W_dkv2, W_uk, W_uv, elite_idx, ke_plane, c_plane, plane_rows, w + L.off_o, ws, L.step, n_splits,
                           hip_stream);
  if (st) return st;
  if (launch_projection(dims, w + L.off_o, W_o, B, hd, dims->d_model, y, w + L.off_proj, stream) != hipSuccess)
    return ELITEKV_EHIP;
  return ELITEKV_OK;
}

size_t elitekv_block_step_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len, int32_t n_splits) {
  DecodePlan p;
  if (plan_decode(dims, 0, B, max_seq_len, n_splits, &p, true, true) == ELITEKV_OK) return p.total;
  BlockLayout L;
  return block_composed_layout(dims, 0, B, max_seq_len, n_splits, &L) ? L.total : 0;
}

int elitekv_block_step(const elitekv_dims* dims, const void* x, const int32_t* pos, const int64_t* slot,
                       const int32_t* seq_len, int64_t B, int64_t max_seq_len, int64_t batch_stride_rows,
                       const void* W_q, const void* W_ke, const void* W_dkv, const void* W_uk, const void* W_uv,
                       const void* W_o, const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows,
                       void* y, void* ws, size_t ws_bytes, int32_t n_splits, void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  if (B == 0) return check_dims(dims);                       // nothing to do
  DecodePlan p;
  int st = plan_decode(dims, 0, B, max_seq_len, n_splits, &p, true, true);
  if (st == ELITEKV_EUNSUPPORTED)                            // eight sequences and more, ...: the composed form
    return block_composed_impl(dims, 0, x, pos, slot, seq_len, B, max_seq_len, batch_stride_rows, W_q, W_ke, W_dkv,
                               nullptr, W_uk, W_uv, W_o, elite_idx, ke_plane, c_plane, plane_rows, y, ws, ws_bytes,
                               n_splits, hip_stream);
  if (st) return st;
  st = append_check(dims, dims->d_c, x, pos, slot, B, W_ke, W_dkv, nullptr, elite_idx, ke_plane, c_plane, plane_rows,
                    ws, ws_bytes, 0);
  if (st) return st;
  // the query and the attention output stay inside the workspace: x stands in for q and y for out in the checks
  st = decode_check(dims, p, x, pos, seq_len, B, batch_stride_rows, W_uk, W_uv, elite_idx, ke_plane, c_plane,
                    plane_rows, y, ws, ws_bytes);
  if (st || B == 0) return st;
  if (!W_q || !W_o) return ELITEKV_ENULL;
  if (!aligned16(W_q) || !aligned16(W_o)) return ELITEKV_EALIGN;
  const hipStream_t stream = (hipStream_t)hip_stream;
  const AppendArgs ap = append_args(dims, dims->d_c, x, pos, slot, B, W_ke, W_dkv, nullptr, elite_idx, ke_plane,
                                    c_plane, plane_rows, nullptr);
  DecodeArgs a = decode_args(dims, 0, (const char*)ws + p.off_qfin, pos, seq_len, B, max_seq_len, batch_stride_rows, W_uk,
                             W_uv, elite_idx, ke_plane, c_plane, plane_rows, nullptr, ws, 6, 1);
  a.fr_slot = slot; a.fr_ke_out = ke_plane; a.fr_c_out = c_plane;
  a.no_out_reduce = 1;
  // (1) first pass of the append and of x W_q  (2) the query's contraction splits summed, rounded
  // (3) q-prep  (4) attention, which also finishes and stores the new rows  (5) merge +
  // up-projection, chunk partials kept  (6) out W_o from the chunk partials  (7) sum of its splits
  hipError_t e = launch_block_front(ap, W_q, a, p, stream);
  if (e == hipSuccess) e = launch_qprep_rows(a, p, (float*)(a.ws + p.off_qe), (bf16_t*)(a.ws + p.off_qt), stream);
  if (e == hipSuccess) e = launch_decode_mfma(a, p, stream);
  if (e == hipSuccess) e = launch_oproj(a, p, W_o, y, stream);
  return e == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

size_t elitekv_slrd_block_step_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t max_seq_len,
                                               int32_t n_splits) {
  BlockLayout L;
  if (!dims || d_ck <= 0 || d_ck >= dims->d_c) return 0;
  return block_composed_layout(dims, d_ck, B, max_seq_len, n_splits, &L) ? L.total : 0;
}

int elitekv_slrd_block_step(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                            const int64_t* slot, const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                            int64_t batch_stride_rows, const void* W_q, const void* W_ke, const void* A_k,
                            const void* A_v, const void* B_k, const void* B_v, const void* W_o,
                            const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows, void* y,
                            void* ws, size_t ws_bytes, int32_t n_splits, void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  int st = check_dims(dims);
  if (st) return st;
  if (d_ck <= 0 || d_ck >= dims->d_c || B < 0) return ELITEKV_EINVAL;
  if (B == 0) return ELITEKV_OK;
  return block_composed_impl(dims, d_ck, x, pos, slot, seq_len, B, max_seq_len, batch_stride_rows, W_q, W_ke, A_k, A_v,
                             B_k, B_v, W_o, elite_idx, ke_plane, c_plane, plane_rows, y, ws, ws_bytes, n_splits,
                             hip_stream);
}

size_t elitekv_slrd_decode_step_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B,
                                                int64_t max_seq_len, int32_t n_splits) {
  if (!dims || d_ck <= 0 || d_ck >= dims->d_c) return 0;
  return step_ws_bytes(dims, d_ck, B, max_seq_len, n_splits);
}

int elitekv_slrd_decode_step(const elitekv_dims* dims, int32_t d_ck, const void* x, const void* q,
                             const int32_t* pos, const int64_t* slot, const int32_t* seq_len, int64_t B,
                             int64_t max_seq_len, int64_t batch_stride_rows, const void* W_ke, const void* A_k,
                             const void* A_v, const void* B_k, const void* B_v, const int32_t* elite_idx,
                             void* ke_plane, void* c_plane, int64_t plane_rows, void* out, void* ws,
                             size_t ws_bytes, int32_t n_splits, void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  if (d_ck <= 0 || d_ck >= dims->d_c) return ELITEKV_EINVAL;
  return step_impl(dims, d_ck, x, q, pos, slot, seq_len, B, max_seq_len, batch_stride_rows, W_ke, A_k, A_v, B_k,
                   B_v, elite_idx, ke_plane, c_plane, plane_rows, out, ws, ws_bytes, n_splits, hip_stream);
}

/* ---- RoPElite search ---- */

static int check_search(int64_t T, int32_t n_h, int32_t head_dim, int32_t r, double rope_base) {
  if (T < 1 || n_h < 1 || head_dim < 2 || (head_dim & 1) || r < 1 || 2 * r > head_dim) return ELITEKV_EINVAL;
  if (!(rope_base > 0.0) || !isfinite(rope_base)) return ELITEKV_EINVAL;
  if (head_dim > 128 || n_h > 65535 || T > (1 << 20)) return ELITEKV_EUNSUPPORTED;
  return ELITEKV_OK;
}

size_t elitekv_ropelite_search_workspace_bytes(int64_t T, int32_t n_heads, int32_t head_dim, int32_t r) {
  if (check_search(T, n_heads, head_dim, r, 10000.0)) return 0;
  return search_workspace_bytes(T, n_heads, head_dim);
}

int elitekv_ropelite_search(const float* q, const float* k, const int32_t* pos, int64_t T, int32_t n_heads,
                            int32_t head_dim, int32_t r, double rope_base, int32_t* elite_out, float* dist_out,
                            void* ws, size_t ws_bytes, void* hip_stream) {
  int st = check_search(T, n_heads, head_dim, r, rope_base);
  if (st) return st;
  if (!q || !k || !pos || !elite_out || !ws) return ELITEKV_ENULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(ws)) return ELITEKV_EALIGN;
  if (ws_bytes < search_workspace_bytes(T, n_heads, head_dim)) return ELITEKV_EWORKSPACE;
  const hipError_t e = launch_ropelite_search(q, k, pos, T, n_heads, head_dim, r, rope_base, elite_out, dist_out,
                                              (char*)ws, (hipStream_t)hip_stream);
  return e == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

/* ---- several queries per sequence ---- */

size_t elitekv_multiquery_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t T, int64_t max_seq_len,
                                          int32_t n_splits) {
  DecodePlan p;
  if (B < 0 || T < 1 || B * T > 65535 || plan_decode(dims, 0, B * T, max_seq_len, n_splits, &p)) return 0;
  return p.total;
}

int elitekv_multiquery_attn(const elitekv_dims* dims, const void* q, const int32_t* q_pos, const int32_t* kv_len,
                            int64_t B, int64_t T, int64_t max_seq_len, int64_t batch_stride_rows,
                            const void* W_uk, const void* W_uv, const int32_t* elite_idx, const void* ke_plane,
                            const void* c_plane, int64_t plane_rows, void* out, void* ws, size_t ws_bytes,
                            int32_t n_splits, void* hip_stream) {
  if (B < 0 || T < 1) return dims ? ELITEKV_EINVAL : ELITEKV_ENULL;
  if (B * T > 65535) return ELITEKV_EUNSUPPORTED;
  return decode_impl(dims, 0, q, q_pos, kv_len, B * T, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                     ke_plane, c_plane, plane_rows, out, ws, ws_bytes, n_splits, hip_stream, 7, (int32_t)T);
}

/* ---- many queries per sequence (prefill): K and V rebuilt once per cached row, then flash attention ---- */

static size_t prefill_ws_impl(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t T, int64_t max_seq_len) {
  if (check_dims(dims) || B < 0 || T < 1 || max_seq_len < 0) return 0;
  if (prefill_flash_supported(*dims, d_ck, T, max_seq_len)) return prefill_flash_workspace(*dims, B, T, max_seq_len);
  return d_ck ? elitekv_slrd_multiquery_workspace_bytes(dims, d_ck, B, T, max_seq_len, 0)
              : elitekv_multiquery_workspace_bytes(dims, B, T, max_seq_len, 0);
}

static int prefill_impl(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                        const int32_t* kv_len, int64_t B, int64_t T, int64_t max_seq_len, int64_t batch_stride_rows,
                        const void* W_uk, const void* W_uv, const int32_t* elite_idx, const void* ke_plane,
                        const void* c_plane, int64_t plane_rows, void* out, void* ws, size_t ws_bytes,
                        void* hip_stream) {
  int st = check_dims(dims);
  if (st) return st;
  if (B < 0 || T < 1 || max_seq_len < 0 || batch_stride_rows < 0 || plane_rows < 0) return ELITEKV_EINVAL;
  if (!prefill_flash_supported(*dims, d_ck, T, max_seq_len)) {     // other shapes: every query as a decode query
    if (d_ck)
      return elitekv_slrd_multiquery_attn(dims, d_ck, q, q_pos, kv_len, B, T, max_seq_len, batch_stride_rows, W_uk,
                                          W_uv, elite_idx, ke_plane, c_plane, plane_rows, out, ws, ws_bytes, 0,
                                          hip_stream);
    return elitekv_multiquery_attn(dims, q, q_pos, kv_len, B, T, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                                   ke_plane, c_plane, plane_rows, out, ws, ws_bytes, 0, hip_stream);
  }
  if (B == 0) return ELITEKV_OK;
  if (B * T > (1LL << 24) || B * dims->n_heads > (1 << 20)) return ELITEKV_EUNSUPPORTED;
  if (!q || !q_pos || !kv_len || !W_uk || !W_uv || !elite_idx || !ke_plane || !c_plane || !out || !ws) return ELITEKV_ENULL;
  if (!aligned16(q) || !aligned16(W_uk) || !aligned16(W_uv) || !aligned16(ke_plane) || !aligned16(c_plane) ||
      !aligned16(out) || !aligned16(ws))
    return ELITEKV_EALIGN;
  if (ws_bytes < prefill_flash_workspace(*dims, B, T, max_seq_len)) return ELITEKV_EWORKSPACE;
  const DecodeArgs a = decode_args(dims, d_ck, q, q_pos, kv_len, B * T, max_seq_len, batch_stride_rows, W_uk, W_uv,
                                   elite_idx, ke_plane, c_plane, plane_rows, out, ws, 7, (int32_t)T);
  return launch_prefill_flash(a, B, T, (hipStream_t)hip_stream) == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

size_t elitekv_prefill_attn_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t T, int64_t max_seq_len) {
  return prefill_ws_impl(dims, 0, B, T, max_seq_len);
}

int elitekv_prefill_attn(const elitekv_dims* dims, const void* q, const int32_t* q_pos, const int32_t* kv_len,
                         int64_t B, int64_t T, int64_t max_seq_len, int64_t batch_stride_rows, const void* W_uk,
                         const void* W_uv, const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                         int64_t plane_rows, void* out, void* ws, size_t ws_bytes, void* hip_stream) {
  return prefill_impl(dims, 0, q, q_pos, kv_len, B, T, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx, ke_plane,
                      c_plane, plane_rows, out, ws, ws_bytes, hip_stream);
}

size_t elitekv_slrd_prefill_attn_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t T,
                                                 int64_t max_seq_len) {
  if (!dims || d_ck <= 0 || d_ck >= dims->d_c) return 0;
  return prefill_ws_impl(dims, d_ck, B, T, max_seq_len);
}

int elitekv_slrd_prefill_attn(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                              const int32_t* kv_len, int64_t B, int64_t T, int64_t max_seq_len,
                              int64_t batch_stride_rows, const void* B_k, const void* B_v, const int32_t* elite_idx,
                              const void* ke_plane, const void* c_plane, int64_t plane_rows, void* out, void* ws,
                              size_t ws_bytes, void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  if (d_ck <= 0 || d_ck >= dims->d_c) return ELITEKV_EINVAL;
  return prefill_impl(dims, d_ck, q, q_pos, kv_len, B, T, max_seq_len, batch_stride_rows, B_k, B_v, elite_idx,
                      ke_plane, c_plane, plane_rows, out, ws, ws_bytes, hip_stream);
}

/* ---- separated low-rank decomposition (two latents per token, stored side by side) ---- */

int elitekv_slrd_param_count(const elitekv_dims* dims, int32_t d_ck, int64_t* n_params) {
  int st = check_dims(dims);
  if (st) return st;
  if (d_ck <= 0 || d_ck >= dims->d_c) return ELITEKV_EINVAL;
  if (!n_params) return ELITEKV_ENULL;
  const int64_t d = dims->d_model, nh = dims->n_heads, dh = dims->head_dim, r = dims->r;
  const int64_t dck = d_ck, dcv = dims->d_c - d_ck;
  *n_params = 2 * r * nh * d + dck * (d + dh * nh - 2 * r * nh) + dcv * (d + dh * nh);
  return ELITEKV_OK;
}

size_t elitekv_slrd_append_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t T) {
  if (!dims || d_ck <= 0 || d_ck >= dims->d_c) return 0;
  return append_ws_bytes(dims, d_ck, T);
}

int elitekv_slrd_append(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                        const int64_t* slot, int64_t T, const void* W_ke, const void* A_k, const void* A_v,
                        const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows, void* ws,
                        size_t ws_bytes, void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  if (d_ck <= 0 || d_ck >= dims->d_c) return ELITEKV_EINVAL;
  return append_impl(dims, d_ck, x, pos, slot, T, W_ke, A_k, A_v, elite_idx, ke_plane, c_plane, plane_rows, ws,
                     ws_bytes, hip_stream);
}

size_t elitekv_slrd_decode_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B,
                                           int64_t max_seq_len, int32_t n_splits) {
  DecodePlan p;
  if (d_ck <= 0 || plan_decode(dims, d_ck, B, max_seq_len, n_splits, &p)) return 0;
  return p.total;
}

int elitekv_slrd_decode_attn(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                             const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                             int64_t batch_stride_rows, const void* B_k, const void* B_v,
                             const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                             int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                             void* hip_stream) {
  if (d_ck <= 0) return dims ? ELITEKV_EINVAL : ELITEKV_ENULL;
  return decode_impl(dims, d_ck, q, q_pos, seq_len, B, max_seq_len, batch_stride_rows, B_k, B_v, elite_idx,
                     ke_plane, c_plane, plane_rows, out, ws, ws_bytes, n_splits, hip_stream, 7);
}

size_t elitekv_slrd_multiquery_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t T,
                                               int64_t max_seq_len, int32_t n_splits) {
  DecodePlan p;
  if (d_ck <= 0 || B < 0 || T < 1 || B * T > 65535 || plan_decode(dims, d_ck, B * T, max_seq_len, n_splits, &p))
    return 0;
  return p.total;
}

int elitekv_slrd_multiquery_attn(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                                 const int32_t* kv_len, int64_t B, int64_t T, int64_t max_seq_len,
                                 int64_t batch_stride_rows, const void* B_k, const void* B_v,
                                 const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                                 int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                                 void* hip_stream) {
  if (!dims) return ELITEKV_ENULL;
  if (d_ck <= 0 || B < 0 || T < 1) return ELITEKV_EINVAL;
  if (B * T > 65535) return ELITEKV_EUNSUPPORTED;
  return decode_impl(dims, d_ck, q, q_pos, kv_len, B * T, max_seq_len, batch_stride_rows, B_k, B_v, elite_idx,
                     ke_plane, c_plane, plane_rows, out, ws, ws_bytes, n_splits, hip_stream, 7, (int32_t)T);
}

int elitekv_decode_attn(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                        const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                        int64_t batch_stride_rows, const void* W_uk, const void* W_uv,
                        const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                        int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                        void* hip_stream) {
  return decode_impl(dims, 0, q, q_pos, seq_len, B, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                     ke_plane, c_plane, plane_rows, out, ws, ws_bytes, n_splits, hip_stream, 7);
}

int elitekv_decode_attn_noalloc(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                                const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                                int64_t batch_stride_rows, const void* W_uk, const void* W_uv,
                                const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                                int64_t plane_rows, void* out, int32_t n_splits, void* hip_stream) {
  DecodePlan p;
  const int st = plan_decode(dims, 0, B, max_seq_len, n_splits, &p);
  if (st) return st;
  if (p.total > (size_t)ELITEKV_NOALLOC_SCRATCH_BYTES) return ELITEKV_ESCRATCH;
  void* ws = scratch_ptr();
  if (!ws) return ELITEKV_EHIP;
  // every kernel of the call writes the part of the scratch it later reads (empty splits included),
  // so nothing needs clearing between calls
  return decode_impl(dims, 0, q, q_pos, seq_len, B, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                     ke_plane, c_plane, plane_rows, out, ws, ELITEKV_NOALLOC_SCRATCH_BYTES, n_splits, hip_stream, 7);
}

int elitekv_decode_attn_stages(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                               const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                               int64_t batch_stride_rows, const void* W_uk, const void* W_uv,
                               const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                               int64_t plane_rows, void* out, void* ws, size_t ws_bytes,
                               int32_t n_splits, void* hip_stream, int32_t stages, int32_t d_ck) {
  if (stages < 1 || stages > 7) return ELITEKV_EINVAL;
  return decode_impl(dims, d_ck, q, q_pos, seq_len, B, max_seq_len, batch_stride_rows, W_uk, W_uv, elite_idx,
                     ke_plane, c_plane, plane_rows, out, ws, ws_bytes, n_splits, hip_stream, stages);
}

size_t elitekv_mha_decode_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len,
                                          int32_t n_splits) {
  int32_t ns, chunk;
  size_t bytes;
  if (plan_mha(dims, B, max_seq_len, n_splits, &ns, &chunk, &bytes)) return 0;
  return bytes;
}

int elitekv_mha_decode(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                       const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                       int64_t batch_stride_rows, const void* k_plane, const void* v_plane,
                       int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                       void* hip_stream) {
  int32_t ns, chunk;
  size_t bytes;
  int st = plan_mha(dims, B, max_seq_len, n_splits, &ns, &chunk, &bytes);
  if (st) return st;
  if (batch_stride_rows < 0 || plane_rows < 0) return ELITEKV_EINVAL;
  if (B == 0) return ELITEKV_OK;
  if (B > 65535) return ELITEKV_EUNSUPPORTED;
  if (!q || !q_pos || !seq_len || !k_plane || !v_plane || !out || !ws) return ELITEKV_ENULL;
  if (!aligned16(q) || !aligned16(k_plane) || !aligned16(v_plane) || !aligned16(out) || !aligned16(ws))
    return ELITEKV_EALIGN;
  if (ws_bytes < bytes) return ELITEKV_EWORKSPACE;
  MhaArgs a;
  a.dims = *dims; a.q = q; a.q_pos = q_pos; a.seq_len = seq_len; a.B = B; a.max_seq_len = max_seq_len;
  a.batch_stride_rows = batch_stride_rows; a.k_plane = k_plane; a.v_plane = v_plane;
  a.plane_rows = plane_rows; a.out = out; a.ws = (char*)ws; a.n_splits = ns; a.chunk = chunk;
  const hipError_t e = launch_mha_decode(a, (hipStream_t)hip_stream);
  return e == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

int elitekv_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream) {
  if (!src || !sink) return ELITEKV_ENULL;
  if (!aligned16(src) || (bytes & 15u)) return ELITEKV_EALIGN;
  if (bytes == 0) return ELITEKV_OK;
  const hipError_t e = launch_stream_read(src, bytes, sink, 1, nullptr, (hipStream_t)hip_stream);
  return e == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

int elitekv_stream_read_mode(const void* src, size_t bytes, uint32_t* sink, int32_t mode, size_t* bytes_read,
                             void* hip_stream) {
  if (!src || !sink) return ELITEKV_ENULL;
  if (mode < 0 || mode > 3) return ELITEKV_EINVAL;
  if (!aligned16(src) || (bytes & 15u)) return ELITEKV_EALIGN;
  if (bytes_read) *bytes_read = 0;
  if (bytes == 0) return ELITEKV_OK;
  const hipError_t e = launch_stream_read(src, bytes, sink, mode, bytes_read, (hipStream_t)hip_stream);
  return e == hipSuccess ? ELITEKV_OK : ELITEKV_EHIP;
}

}  // extern "C"
