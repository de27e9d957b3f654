// Internal interface between the C-ABI entry points (host validation and planning) and the
// kernel launchers.  Every launcher only enqueues work on `stream`.
#pragma once
#include <atomic>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/elitekv.h"

namespace ekv {

// Raising a kernel's dynamic-LDS limit (the default is 64 KiB, static LDS included) is a per-device setting; it is made
// once per (kernel instantiation, device, largest size asked for so far).  One LdsLimit per
// instantiation (a function-local static: zero-initialised, safe to use from several threads).
constexpr int kMaxDevices = 64;
struct LdsLimit {
  std::atomic<size_t> have[kMaxDevices];
};
inline hipError_t raise_lds_limit(LdsLimit& st, const void* kernel, size_t bytes) {
  if (bytes <= 48 * 1024) return hipSuccess;     // with the kernels' static LDS still below the default limit
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < kMaxDevices;
  if (tracked && st.have[dev].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && tracked) st.have[dev].store(bytes, std::memory_order_relaxed);
  return e;
}


// Where each intermediate of one decode call lives inside the caller's workspace.
struct DecodePlan {
  int32_t n_splits;     // sequence splits per batch row
  int32_t chunk;        // cached tokens per split
  int32_t mfma;         // 1: bf16 MFMA kernels, 0: generic VALU kernels
  int32_t head_groups;  // MFMA path: groups of up to 32 heads
  int32_t up_cw;        // MFMA path: latent columns per merge/up-projection work-group
  int32_t merge_batch;  // MFMA path: 1 = the merge kernel that takes all batch rows per work-group
  int32_t d_q;          // width of the absorbed query: d_c (joint latent) or d_ck (separated latents)
  int32_t d_u;          // width of the latent accumulators: d_c (joint) or d_cv (separated)
  size_t off_qe;        // rotated, scaled elite query      fp32 [B, n_h, 2r]
  size_t off_qt;        // absorbed, scaled latent query    fp32 [B, n_h, d_c] (generic) / bf16 (mfma)
  size_t off_m;         // split maxima (log2 domain)       fp32 [B, n_splits, n_h_pad]
  size_t off_l;         // split sums                       fp32 [B, n_splits, n_h_pad]
  size_t off_u;         // split latent accumulators        fp32 [B, n_splits, ...]
  size_t off_opart;     // up-projection partials           fp32
  size_t off_cnt;       // MFMA path: arrival counters of the merge kernels' chunk groups   int32 [B, n_h]
  // fused decode step (fresh != 0): the cache row of the newest token of every sequence is finished (summed,
  // rotated, stored) inside the attention kernel, by the work-group whose tiles include its position,
  // from the append's contraction-split sums.  1: fewer than eight sequences (weight-streaming front launch),
  // 2: eight to 64 sequences (matrix-core front launch)
  int32_t fresh;
  int32_t n_part;       // partials per batch row (= n_splits)
  int32_t fr_ks;        // contraction splits of the step's append
  int32_t fr_kc;        // ... rows of the weight matrices per split (a multiple of 32)
  size_t off_apart;     // the append's split sums           fp32 [fr_ks, B, fr_stride]
  int32_t fr_stride;    // floats per token in them: 2 r n_h + d_c, + n_h d_h when x W_q is computed alongside
  size_t off_qfin;      // whole-block step: the query x W_q, summed over the splits   bf16 [B, n_h, d_h]
  size_t off_ypart;     // whole-block step: split sums of the output projection  fp32 [y_ks, B, d_model]
  int32_t y_ks, y_kc;
  size_t off_sincos;    // (sin, cos) of the rotated chunks  fp32 [B, n_h r, 2]
  size_t total;
};

struct DecodeArgs {
  elitekv_dims dims;
  int32_t d_ck;         // separated latents: a cache row is [c^k (d_ck) | c^v (d_c - d_ck)]; 0 = joint latent
  const void* q;
  const int32_t* q_pos;
  const int32_t* seq_len;
  int64_t B, max_seq_len, batch_stride_rows;
  const void* W_uk;
  const void* W_uv;
  const int32_t* elite_idx;
  const void* ke_plane;
  const void* c_plane;
  int64_t plane_rows;
  void* out;
  char* ws;
  int32_t q_per_seq;                // queries per sequence: row b of q belongs to sequence b / q_per_seq
  int32_t stages;                   // bit 0 q-prep, bit 1 split attention, bit 2 merge + up-projection
  // fused decode step only: destination rows of the new tokens and the planes, writable
  const int64_t* fr_slot;
  void* fr_ke_out;
  void* fr_c_out;
  // whole-block step only: the merge leaves its column-chunk partials for the output projection (no out_reduce)
  int32_t no_out_reduce;
};

struct AppendArgs {
  elitekv_dims dims;
  int32_t d_ck;         // columns of W_dkv; the remaining d_c - d_ck latent columns come from W_dkv2
  const void* W_dkv2;   // separated latents: A^v [d, d_c - d_ck]; unused when d_ck == d_c
  const void* x;
  const int32_t* pos;
  const int64_t* slot;
  int64_t T;
  const void* W_ke;
  const void* W_dkv;
  const int32_t* elite_idx;
  void* ke_plane;
  void* c_plane;
  int64_t plane_rows;
  char* ws;
  // Matrix-core GEMM only (launch_append_gemm), for inputs that are column slices of wider rows:
  int64_t x_ld = 0;     // elements between two rows of x; 0: dims.d_model
  int32_t x_off2 = 0;   // the W_dkv2 columns contract x[:, x_off2 : x_off2 + d2] with W_dkv2 [d2, d_c - d_ck] ...
  int32_t d2 = 0;       // ... 0: the same dims.d_model columns of x as the others
  // Plain projection (the q and output projections of the whole-block step, Section 2.1): with dense_out set the
  // T <= 64 append kernels run with r = 0 and leave x W_dkv as dense rows [T, d_c] of the storage type there;
  // no rotation, no planes, pos / slot / elite_idx unused.
  void* dense_out = nullptr;
};

struct MhaArgs {
  elitekv_dims dims;
  const void* q;
  const int32_t* q_pos;
  const int32_t* seq_len;
  int64_t B, max_seq_len, batch_stride_rows;
  const void* k_plane;
  const void* v_plane;
  int64_t plane_rows;
  void* out;
  char* ws;
  int32_t n_splits, chunk;
};

hipError_t launch_append_generic(const AppendArgs& a, hipStream_t stream);
bool append_small_supported(const elitekv_dims& d, int64_t T, int d_ck);
size_t append_small_workspace(const elitekv_dims& d, int64_t T);
hipError_t launch_append_small(const AppendArgs& a, hipStream_t stream);
hipError_t launch_append_finish(const AppendArgs& a, const float* partial, int ksplit, hipStream_t stream);
bool append_skinny_supported(const elitekv_dims& d, int64_t T, int d_ck);
size_t append_skinny_workspace(const elitekv_dims& d, int64_t T);
hipError_t launch_append_skinny(const AppendArgs& a, hipStream_t stream);
bool append_gemm_supported(const elitekv_dims& d, int64_t T, int d_ck);
hipError_t launch_append_gemm(const AppendArgs& a, hipStream_t stream);
hipError_t launch_decode_generic(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream);
bool decode_mfma_supported(const elitekv_dims& d, int d_ck);
int decode_mfma_groups_per_cu(const elitekv_dims& d);
int decode_mfma_slice_width(int d_c);     // latent columns per wave of the attention kernel for rows of d_c columns; 0 = none
struct bf16_t;
hipError_t launch_qprep_rows(const DecodeArgs& a, const DecodePlan& p, float* qe, bf16_t* qt,
                             hipStream_t stream);
bool qprep_mfma_supported(const elitekv_dims& d, int d_q, int64_t B);
// Fused decode step: its front kernel runs the first pass of the append of the step's B tokens and the
// query preparation in one launch.  decode_front_plan says whether the kernels cover the shape and
// how the append's contraction is split (ks splits of kc weight rows).
bool decode_front_plan(const elitekv_dims& d, int d_ck, int d_q, int64_t B, int* ks, int* kc);
hipError_t launch_decode_front(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p, hipStream_t stream);
// whole-block step: the split plans of its two weight-streaming passes, its first launch (append + x W_q)
// and its last two (out W_o from the merge's chunk partials, then the sum of the splits)
bool block_step_plan(const elitekv_dims& d, int64_t B, int* fr_ks, int* fr_kc, int* y_ks, int* y_kc);
hipError_t launch_block_front(const AppendArgs& ap, const void* W_q, const DecodeArgs& a, const DecodePlan& p,
                              hipStream_t stream);   // + the sum of the query's contraction splits into ws + off_qfin
hipError_t launch_oproj(const DecodeArgs& a, const DecodePlan& p, const void* W_o, void* y, hipStream_t stream);
// ... for batches of eight rows and up (matrix-core roles; includes the append's finishing launch)
bool decode_front_mfma_supported(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p);
bool decode_front_mfma_plan(const elitekv_dims& d, int d_ck, int d_q, int64_t B, int* ks, int* kc);
hipError_t launch_decode_front_mfma(const AppendArgs& ap, const DecodeArgs& a, const DecodePlan& p, hipStream_t stream);
bool merge_mfma_supported(const elitekv_dims& d, int d_u, int64_t B, int64_t n_splits);
hipError_t launch_merge_mfma(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream);
hipError_t launch_merge_up(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream);
hipError_t launch_decode_mfma(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream);
// many queries per sequence: keys and values rebuilt from the latent once per cached row (with the append's
// matrix-core GEMM), then flash attention; a.B = B * T query rows, a.seq_len = the visible rows of each
bool prefill_flash_supported(const elitekv_dims& d, int d_ck, int64_t T, int64_t max_seq_len);
size_t prefill_flash_workspace(const elitekv_dims& d, int64_t B, int64_t T, int64_t max_seq_len);
hipError_t launch_prefill_flash(const DecodeArgs& a, int64_t B, int64_t T, hipStream_t stream);
hipError_t launch_mha_decode(const MhaArgs& a, hipStream_t stream);
size_t search_workspace_bytes(int64_t T, int n_h, int d_h);
hipError_t launch_ropelite_search(const float* q, const float* k, const int32_t* pos, int64_t T, int n_h, int d_h,
                                  int r, double rope_base, int32_t* elite_out, float* dist_out, char* ws,
                                  hipStream_t stream);
hipError_t launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int mode, size_t* bytes_read,
                              hipStream_t stream);

}  // namespace ekv
