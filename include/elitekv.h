/*
 * libelitekv — decode hot path of EliteKV (RoPElite + joint low-rank KV compression)
 * for AMD MI355X (gfx950).  Plain C ABI: pointers and sizes only.
 *
 * The library is stateless: it allocates nothing, keeps no handles and never synchronises.
 * Every call only validates its arguments on the host and enqueues kernels on the HIP stream
 * it is given; results are valid once the caller has synchronised that stream.  All buffers
 * are owned by the caller.  Unless a parameter says "host", array pointers are DEVICE pointers.
 *
 * Notation follows the paper: d (hidden size), n_h (heads), d_h (head dim), r (elite 2-D chunks
 * per head, Section 3.1), I_h (head h's elite chunk indices, each in [0, d_h/2)), d_c (rank of the
 * joint latent, Section 3.2 "Joint Low-Rank Decomposition"), W_ke (W^k_{e,h}, Section 3.2),
 * W_dkv = A^{kv}, W_uk = B^k_J, W_uv = B^v_J.
 *
 * Conventions fixed here where the paper is silent:
 *   - theta_i = rope_base^(-2i/d_h); a chunk is the ADJACENT dim pair (2i, 2i+1) (Section 2.2);
 *   - R(a) maps a row pair (u, v) to (u cos a - v sin a, u sin a + v cos a);
 *   - column order inside a head: elite slots in the caller's I_h order, each slot as its two
 *     lanes; non-elite dims in ascending original index;
 *   - softmax scale is 1/sqrt(d_h) (Section 2.1).
 *
 * Return value of every int function: 0 on success, a negative elitekv_status otherwise.
 * Validation happens before any launch; on error nothing has been enqueued.
 */
#ifndef ELITEKV_H
#define ELITEKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum elitekv_status {
  ELITEKV_OK = 0,
  ELITEKV_EINVAL = -1,        /* bad dims: odd head_dim, r < 0 or r > d_h/2, d_c <= 0, negative counts, bad dtype */
  ELITEKV_EINDEX = -2,        /* elite index out of range or repeated inside a head (host check only) */
  ELITEKV_ENULL = -3,         /* a required pointer is NULL */
  ELITEKV_EALIGN = -4,        /* a pointer or stride misses the 16-byte alignment the kernels need */
  ELITEKV_EWORKSPACE = -5,    /* workspace smaller than the matching *_workspace_bytes() */
  ELITEKV_EUNSUPPORTED = -6,  /* shape outside what the kernels cover (see each call) */
  ELITEKV_EHIP = -7,          /* the HIP runtime reported a launch error */
  ELITEKV_ESCRATCH = -8       /* elitekv_decode_attn_noalloc: the call needs more than the built-in scratch holds */
};

enum elitekv_dtype {
  ELITEKV_FP32 = 0,           /* fp32 storage, fp32 arithmetic */
  ELITEKV_BF16 = 1            /* bf16 storage (weights, activations, cache), fp32 accumulation */
};

/* Problem dimensions.  MHA only (one key/value head per query head). */
typedef struct elitekv_dims {
  int32_t d_model;    /* d, hidden size of x */
  int32_t n_heads;    /* n_h */
  int32_t head_dim;   /* d_h, even */
  int32_t r;          /* elite chunks per head, 0 <= r <= d_h/2 */
  int32_t d_c;        /* latent rank, > 0 */
  int32_t dtype;      /* elitekv_dtype of x, q, weights, cache planes and out */
  double rope_base;   /* > 0, e.g. 10000 */
} elitekv_dims;

/* Human-readable name of a status code.  Never NULL. */
const char* elitekv_strerror(int status);

/* Per-token cache row sizes in elements: *ke_elems = 2*r*n_h, *c_elems = d_c.
 * (Section 3.2, J-LRD: the cache holds 2*r*n_h + d_c elements per token per layer.) */
int elitekv_cache_row_elems(const elitekv_dims* dims, int64_t* ke_elems, int64_t* c_elems);

/* Total parameters of the four weight blocks this ABI takes:
 * 2*r*n_h*d + d_c*(d + 2*d_h*n_h - 2*r*n_h)  (Section 3.2, storage cost of RoPElite with J-LRD). */
int elitekv_param_count(const elitekv_dims* dims, int64_t* n_params);

/* Host-only check of the index sets I_h (Section 3.1): idx_host is a HOST array [n_h, r];
 * every entry must lie in [0, d_h/2) and be distinct within its head.  EINDEX otherwise. */
int elitekv_validate_elite_idx(const elitekv_dims* dims, const int32_t* idx_host);

/* Workspace (device bytes) elitekv_append needs for T tokens.  0 on bad dims. */
size_t elitekv_append_workspace_bytes(const elitekv_dims* dims, int64_t T);

/*
 * Cache append (Section 3.1, what a RoPElite model adds to its cache at step t; Section 3.2,
 * c_t = x_t A^{kv} and W^k_{e,h}).  For every token t < T:
 *     c_plane[slot[t], :]            = x_t W_dkv
 *     ke_plane[slot[t], h, 2j:2j+2]  = (x_t W_ke[:, h, 2j:2j+2]) R(pos[t] * theta_{I_h[j]})
 * The rotation angle is formed in double precision.  Old cache rows are never read.
 *
 *   x          [T, d_model]                 dims->dtype, row-major
 *   pos        [T] int32                    position of each token
 *   slot       [T] int64                    destination row in both planes; a slot outside
 *                                           [0, plane_rows) makes that token a no-op
 *   W_ke       [d_model, n_h, 2r]           dims->dtype
 *   W_dkv      [d_model, d_c]               dims->dtype
 *   elite_idx  [n_h, r] int32               DEVICE copy of I_h (validate on the host beforehand)
 *   ke_plane   [plane_rows, n_h, 2r]        written, dims->dtype (may be NULL when r == 0)
 *   c_plane    [plane_rows, d_c]            written, dims->dtype
 *   ws         workspace of at least elitekv_append_workspace_bytes(dims, T) (may be NULL if 0)
 *   hip_stream a hipStream_t (NULL = the default stream)
 *
 * T == 0 is a successful no-op.  Errors: EINVAL, ENULL, EALIGN (pointers must be 16-byte aligned),
 * EWORKSPACE, EUNSUPPORTED (head_dim > 256), EHIP.
 */
int elitekv_append(const elitekv_dims* dims, const void* x, const int32_t* pos, const int64_t* slot,
                   int64_t T, const void* W_ke, const void* W_dkv, const int32_t* elite_idx,
                   void* ke_plane, void* c_plane, int64_t plane_rows, void* ws, size_t ws_bytes,
                   void* hip_stream);

/* Which kernels the decode entry points (elitekv_decode_attn, _decode_step, _multiquery_attn and their slrd_
 * forms; Sections 3.1, 3.2 and 5 as cited there) run for a shape: ELITEKV_PATH_MATRIX_CORE, the tuned bf16 MFMA
 * kernels (bf16; d_h 64 or 128; r = 4, 8 or 16 elite chunks per head; (d_h - 2r) a multiple of 8; d_c a
 * multiple of 128 up to 2048, or 1920; r = 16 only up to d_c 1792, the widest row whose tiles fit the LDS next to
 * 2 r = 32 elite values per head; separated latents: d_ck and d_c - d_ck whole wave slices / 64-column chunks),
 * or ELITEKV_PATH_GENERIC, the untuned fp32 vector kernels that cover every other shape (all fp32 shapes,
 * other r or d_c).  Results are the same to rounding; only the speed differs, so a caller that cares asks here.
 * d_ck = 0: joint latent; d_ck > 0: separated latents.  Host only.  Negative status on bad dims. */
enum elitekv_path { ELITEKV_PATH_GENERIC = 0, ELITEKV_PATH_MATRIX_CORE = 1 };
int elitekv_decode_path(const elitekv_dims* dims, int32_t d_ck);

/* Number of sequence splits elitekv_decode_attn uses when n_splits == 0 ("auto") for this shape.
 * Returns <= 0 on bad dims. */
int32_t elitekv_decode_auto_splits(const elitekv_dims* dims, int64_t B, int64_t max_seq_len);

/* Workspace (device bytes) elitekv_decode_attn needs.  n_splits == 0 means "auto". 0 on bad dims. */
size_t elitekv_decode_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len,
                                      int32_t n_splits);

/*
 * Single-token decode attention over the compressed cache (Section 3.1, the RoPElite score
 * equation; Section 2.1, softmax attention; Section 3.2, B^{kv} = [B^k_J, B^v_J]; Section 5,
 * absorption of B^k and B^v into the neighbouring products).  For batch row b and head h, over
 * the cached rows j in [b*batch_stride_rows, b*batch_stride_rows + seq_len[b]):
 *     s_j = ( rot(q[b,h,I_h], q_pos[b]) . ke_plane[j,h,:]  +  q[b,h,non-elite] . (c_plane[j,:] W_uk[:,h,:]) ) / sqrt(d_h)
 *     p   = softmax_j(s),      out[b,h,:] = sum_j p_j (c_plane[j,:] W_uv[:,h,:])
 * computed as: W_uk absorbed into the query, one online softmax over both score terms, values
 * accumulated in latent space, split over the sequence with an exact log-sum-exp merge, then
 * W_uv applied once.  The cached elite keys are used as stored (no re-rotation).
 *
 *   q          [B, n_h, d_h]        un-rotated query, original dim order, dims->dtype
 *   q_pos      [B] int32            position of each query token
 *   seq_len    [B] int32            cached rows each batch row attends to; values above
 *                                   max_seq_len, or reaching past plane_rows, are clamped
 *                                   on the device; seq_len[b] == 0 gives a zero output row
 *   max_seq_len                     HOST upper bound on seq_len[] (plans the split).  Of every batch row
 *                                   the first min(max_seq_len, rows left in the planes) rows may be READ
 *                                   whatever seq_len[b] says (a kernel requests its first rows before
 *                                   seq_len[b] has arrived); rows at or beyond seq_len[b] never reach a
 *                                   result, whatever they hold
 *   batch_stride_rows               plane rows between consecutive batch rows' first row
 *   W_uk       [d_c, n_h, d_h-2r]   dims->dtype
 *   W_uv       [d_c, n_h, d_h]      dims->dtype
 *   elite_idx  [n_h, r] int32       DEVICE copy of I_h
 *   ke_plane   [plane_rows, n_h, 2r], c_plane [plane_rows, d_c]   read only, dims->dtype
 *   out        [B, n_h, d_h]        written, dims->dtype
 *   ws         at least elitekv_decode_workspace_bytes(dims, B, max_seq_len, n_splits)
 *   n_splits   sequence splits per batch row; 0 = auto.  The result does not depend on it
 *              beyond rounding.
 *
 * B == 0 is a successful no-op.  Errors: EINVAL, ENULL, EALIGN, EWORKSPACE, EUNSUPPORTED
 * (d_c > 4096, head_dim > 256, or n_splits > 1024), EHIP.
 */
int elitekv_decode_attn(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                        const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                        int64_t batch_stride_rows, const void* W_uk, const void* W_uv,
                        const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                        int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                        void* hip_stream);

/*
 * elitekv_decode_attn for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (without ws / ws_bytes), same kernels and bit-for-bit the same result as elitekv_decode_attn; the
 * intermediates live in a buffer of ELITEKV_NOALLOC_SCRATCH_BYTES that is part of the library's device
 * image (one copy per GPU, held until the process ends).  The call allocates and frees nothing.
 *   - ESCRATCH (nothing enqueued) when elitekv_decode_workspace_bytes(dims, B, max_seq_len, n_splits)
 *     exceeds ELITEKV_NOALLOC_SCRATCH_BYTES; 32 MiB covers the 7B shape at 25 % cache, one sequence,
 *     32768 cached tokens with the automatic split count.
 *   - All calls on one GPU share that GPU's buffer: two calls whose kernels may overlap (different
 *     streams, no ordering between them) race.  Calls on one stream are ordered and safe.  Nothing in
 *     the buffer has to be cleared between calls.
 *   - The buffer's address is looked up on the first call on each device (hipGetSymbolAddress); make
 *     that first call outside a graph capture.
 * Other errors as elitekv_decode_attn; EHIP also if the buffer's address cannot be obtained.
 */
#define ELITEKV_NOALLOC_SCRATCH_BYTES (32u << 20)
int elitekv_decode_attn_noalloc(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                                const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                                int64_t batch_stride_rows, const void* W_uk, const void* W_uv,
                                const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                                int64_t plane_rows, void* out, int32_t n_splits, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * RoPElite search (Section 3.1, Algorithm 1): the greedy choice of every head's r elite chunks from
 * a sample of UN-ROTATED queries and keys of one layer.  In each of r rounds every chunk that is
 * not yet elite is tried as the one additional rotated chunk; the chunk whose pre-softmax scores
 * (Section 2.1's s, over the causal pairs key step <= query step, scaled by 1/sqrt(d_h)) have the
 * smallest L1 distance to the scores of full RoPE is appended; the lowest index wins a tie.
 *   q, k      [T, n_heads, head_dim] float32, device      pos [T] int32, device
 *   elite_out [n_heads, r] int32, device: chunk indices in selection order (usable as elite_idx)
 *   dist_out  [n_heads, r] float32, device, or NULL: the winning distance of every round
 * Arithmetic is fp32 (angles reduced in double); a near-tie between two chunks may resolve
 * differently from exact arithmetic.  head_dim <= 128.  Workspace: the _workspace_bytes function.
 * Enqueues 2 r + 2 kernels on hip_stream; no host synchronisation.
 * ------------------------------------------------------------------------------------------- */
size_t elitekv_ropelite_search_workspace_bytes(int64_t T, int32_t n_heads, int32_t head_dim, int32_t r);
int elitekv_ropelite_search(const float* q, const float* k, const int32_t* pos, int64_t T, int32_t n_heads,
                            int32_t head_dim, int32_t r, double rope_base, int32_t* elite_out, float* dist_out,
                            void* ws, size_t ws_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Several queries per sequence (a prefill chunk, the verification of drafted tokens): T query
 * tokens of each of B sequences attend over the cache rows of their own sequence.  Section 2.1
 * builds K_t, V_t from the tokens up to step t, so query (b, t) sees a prefix of sequence b's rows;
 * the caller states its length in kv_len (causal decoding: the query's position + 1, after the
 * chunk's own tokens have been appended).  Each query is computed exactly as by elitekv_decode_attn.
 *   q      [B, T, n_h, d_h]   q_pos [B * T]   kv_len [B * T]   out [B, T, n_h, d_h]
 * Sequence b owns plane rows [b * batch_stride_rows, ...); max_seq_len bounds every kv_len.
 * Other arguments, workspace rules and errors as elitekv_decode_attn; EINVAL if T < 1,
 * EUNSUPPORTED if B * T > 65535.
 * ------------------------------------------------------------------------------------------- */
size_t elitekv_multiquery_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t T, int64_t max_seq_len,
                                          int32_t n_splits);
int elitekv_multiquery_attn(const elitekv_dims* dims, const void* q, const int32_t* q_pos, const int32_t* kv_len,
                            int64_t B, int64_t T, int64_t max_seq_len, int64_t batch_stride_rows,
                            const void* W_uk, const void* W_uv, const int32_t* elite_idx, const void* ke_plane,
                            const void* c_plane, int64_t plane_rows, void* out, void* ws, size_t ws_bytes,
                            int32_t n_splits, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Many queries per sequence (a prefill, a long prompt chunk).  Same arguments, layouts, meaning of
 * kv_len and result as elitekv_multiquery_attn (Section 2.1: query t sees the keys and values of
 * the tokens up to step t), but the multiplications are ordered for many queries: the keys
 * [stored rotated elite dims | c B^k_J,h] and values c B^v_J,h (Section 3.1 score equation,
 * Section 3.2 J-LRD) of the first max_seq_len rows of every sequence are rebuilt ONCE into the
 * workspace, and every query then runs ordinary attention (Section 2.1) against them, instead of
 * absorbing B^k into each query (Section 5), which costs d_c / d_h times more per (query, key).
 *   q [B, T, n_h, d_h]   q_pos [B * T]   kv_len [B * T]   out [B, T, n_h, d_h]   (device pointers)
 * bf16, head_dim 128, r in {4, 8}, d_c a multiple of 32, n_h (2 d_h - 2 r) a multiple of 128,
 * T >= 48 and max_seq_len > 64 run this path; every other call is handed to elitekv_multiquery_attn
 * (and its limits apply): with fewer queries per sequence the absorbed form is the cheaper order.
 * Rows of a sequence beyond the largest kv_len of its queries are never read by the attention, but
 * the first max_seq_len rows of the latent plane are read by the rebuild.
 * Workspace: the _workspace_bytes function (about B * max_seq_len * n_h * (2 d_h - 2 r) * 2 bytes).
 * Errors as elitekv_decode_attn; EUNSUPPORTED if B * T > 2^24.
 * ------------------------------------------------------------------------------------------- */
size_t elitekv_prefill_attn_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t T, int64_t max_seq_len);
int elitekv_prefill_attn(const elitekv_dims* dims, const void* q, const int32_t* q_pos, const int32_t* kv_len,
                         int64_t B, int64_t T, int64_t max_seq_len, int64_t batch_stride_rows, const void* W_uk,
                         const void* W_uv, const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                         int64_t plane_rows, void* out, void* ws, size_t ws_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Separated low-rank decomposition (Section 3.2, "Separated Low-Rank Decomposition"):
 *     W^k_{e^,0:n_h-1} ~ A^k B^k_S,   W^v_{0:n_h-1} ~ A^v B^v_S,
 * a token caches two latents, c^k = x A^k (d_ck columns) and c^v = x A^v (d_cv columns), next to its
 * rotated elite keys; 2 r n_h + d_ck + d_cv cache elements per token.  The two latents are stored
 * SIDE BY SIDE in one row of the latent plane: c_plane [rows, d_ck + d_cv] = [c^k | c^v], so
 * dims->d_c = d_ck + d_cv is the row width and d_ck says where c^v starts.  Everything else
 * (planes, positions, slots, elite indices, workspace rules, streams, error codes) is as in the
 * joint entry points above.  EINVAL unless 0 < d_ck < dims->d_c.
 * ------------------------------------------------------------------------------------------- */

/* Section 3.2, storage cost with S-LRD: 2 r n_h d + d_ck (d + d_h n_h - 2 r n_h) + d_cv (d + d_h n_h). */
int elitekv_slrd_param_count(const elitekv_dims* dims, int32_t d_ck, int64_t* n_params);

/* Workspace bytes elitekv_slrd_append needs for T tokens (host only; may be 0). */
size_t elitekv_slrd_append_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t T);

/*
 * Append T tokens: elite keys as in elitekv_append; latent row = [x A^k | x A^v].
 * A_k [d_model, d_ck] and A_v [d_model, d_c - d_ck], row-major, device pointers.
 */
int elitekv_slrd_append(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                        const int64_t* slot, int64_t T, const void* W_ke, const void* A_k, const void* A_v,
                        const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows, void* ws,
                        size_t ws_bytes, void* hip_stream);

/* Workspace bytes of elitekv_slrd_decode_attn (host only).  n_splits == 0 means "auto"
 * (elitekv_decode_auto_splits gives the count). */
size_t elitekv_slrd_decode_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B,
                                           int64_t max_seq_len, int32_t n_splits);

/*
 * Single-token decode attention of an S-LRD model: keys are [rotated elite dims | c^k B^k_S,h],
 * values are c^v B^v_S,h.  B_k [d_ck, n_h, d_h - 2r], B_v [d_c - d_ck, n_h, d_h], device pointers;
 * the remaining arguments as in elitekv_decode_attn.  B^k_S is absorbed into the query and B^v_S is
 * applied after the attention sum, so scores only touch the c^k columns of a cache row and the value
 * accumulation only its c^v columns.
 */
int elitekv_slrd_decode_attn(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                             const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                             int64_t batch_stride_rows, const void* B_k, const void* B_v,
                             const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                             int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                             void* hip_stream);

/*
 * Several queries per sequence of an S-LRD model: elitekv_multiquery_attn (Section 2.1: query (b, t)
 * sees the first kv_len rows of sequence b) with the keys and values of elitekv_slrd_decode_attn
 * (Section 3.2).  q [B, T, n_h, d_h], q_pos and kv_len [B * T], out [B, T, n_h, d_h]; B_k, B_v and
 * the planes as in elitekv_slrd_decode_attn; workspace from the _workspace_bytes function.
 * EINVAL if T < 1 or d_ck is out of range, EUNSUPPORTED if B * T > 65535.
 */
size_t elitekv_slrd_multiquery_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t T,
                                               int64_t max_seq_len, int32_t n_splits);
int elitekv_slrd_multiquery_attn(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                                 const int32_t* kv_len, int64_t B, int64_t T, int64_t max_seq_len,
                                 int64_t batch_stride_rows, const void* B_k, const void* B_v,
                                 const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                                 int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                                 void* hip_stream);

/*
 * Many queries per sequence of an S-LRD model: elitekv_prefill_attn with the keys
 * [stored rotated elite dims | c^k B^k_S,h] and values c^v B^v_S,h of Section 3.2 rebuilt once per
 * cached row (keys from the first d_ck columns of a latent row, values from the others), then ordinary
 * attention (Section 2.1).  Arguments as elitekv_slrd_multiquery_attn, result the same.
 * Runs this path under the conditions of elitekv_prefill_attn and, in addition, d_ck a multiple of 32
 * and n_h (d_h - 2 r) a multiple of 128; every other call is handed to elitekv_slrd_multiquery_attn
 * (and its limits apply).  Workspace: the _workspace_bytes function.
 */
size_t elitekv_slrd_prefill_attn_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t T,
                                                 int64_t max_seq_len);
int elitekv_slrd_prefill_attn(const elitekv_dims* dims, int32_t d_ck, const void* q, const int32_t* q_pos,
                              const int32_t* kv_len, int64_t B, int64_t T, int64_t max_seq_len,
                              int64_t batch_stride_rows, const void* B_k, const void* B_v, const int32_t* elite_idx,
                              const void* ke_plane, const void* c_plane, int64_t plane_rows, void* out, void* ws,
                              size_t ws_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * One decode step in one call: the B new tokens (one per sequence) are appended to the cache and
 * each sequence's query attends to its cached tokens and to its new token.  With
 * slot[b] = b * batch_stride_rows + seq_len[b] - 1 the result is that of elitekv_append (T = B; x,
 * pos, slot) followed by elitekv_decode_attn (q, q_pos = pos, seq_len) on the same stream
 * (Sections 3.1, 3.2 and 5 as cited there); sums may be taken in a different order, so results agree
 * to rounding, not bit for bit.
 *   seq_len[b] counts the tokens the query of sequence b attends to, the new one included: rows
 *   b * batch_stride_rows + [0, seq_len[b] - 1) of the planes, then the new token, whose row is
 *   slot[b] = b * batch_stride_rows + seq_len[b] - 1.  For a sequence whose slot[b] is anything
 *   else (out of range: the token is not stored; another row) the row is stored as elitekv_append
 *   stores it but out[b] is unspecified: depending on the shape the new token is attended to from
 *   its fresh row or from whatever row seq_len[b] - 1 of the plane holds.  seq_len[b] <= 0:
 *   nothing is attended, out[b] is 0, and the token is still stored at slot[b] if that is in range.
 *   For up to 64 sequences (bf16 shapes of the matrix-core path) the step is three launches (four
 *   from eight sequences on): the first pass of the append together with the query preparation; the
 *   attention, in which the work-group that owns the tile of a sequence's newest position first adds
 *   up the append's partial sums, rotates and stores the new row; the merge with the up-projection
 *   (from two sequences on followed by the launch that adds its column-chunk partials).  Other shapes
 *   run the two entry points' kernels one after the other.
 *   All other arguments, layouts, ownership and errors as in elitekv_append and
 *   elitekv_decode_attn.  ws: elitekv_decode_step_workspace_bytes bytes (EWORKSPACE if smaller).
 * ------------------------------------------------------------------------------------------- */
size_t elitekv_decode_step_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len,
                                           int32_t n_splits);
int elitekv_decode_step(const elitekv_dims* dims, const void* x, const void* q, const int32_t* pos,
                        const int64_t* slot, const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                        int64_t batch_stride_rows, const void* W_ke, const void* W_dkv, const void* W_uk,
                        const void* W_uv, const int32_t* elite_idx, void* ke_plane, void* c_plane,
                        int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                        void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * The whole attention block of one decode step (Section 2.1: q_t = x_t W^q per head in front, the
 * concatenated heads times W^o behind; Section 5: B^k and B^v stay absorbed into the neighbouring
 * products, nothing is materialised).  For every sequence b:
 *     q[b]  = x[b] W_q                      (rounded to dims->dtype, as a model would hold it)
 *     the token is appended as in elitekv_append (x[b], pos[b], slot[b])
 *     o[b]  = elitekv_decode_attn over the sequence's cached tokens and the new one (q_pos = pos)
 *     y[b]  = [o[b,0,:] .. o[b,n_h-1,:]] W_o
 * with the meaning of seq_len and slot of elitekv_decode_step (the new token is the last one
 * attended to and slot[b] = b * batch_stride_rows + seq_len[b] - 1).
 *   W_q   [d_model, n_h, d_h]      dims->dtype
 *   W_o   [n_h, d_h, d_model]      dims->dtype
 *   y     [B, d_model]             written, dims->dtype
 *   the other arguments as in elitekv_decode_step; ws: elitekv_block_step_workspace_bytes bytes.
 * Fewer than eight sequences (bf16 shapes of the matrix-core path): seven launches -- the first pass of
 * the append and of x W_q in one weight-streaming launch; the sum of the query's contraction splits; the
 * query preparation; the attention, which also finishes and stores the new rows; the merge with the
 * up-projection; out W_o read straight from the merge's column-chunk partials; the sum of its
 * contraction splits.  Eight to 64 sequences, and bf16 shapes outside the matrix-core path: the composed
 * form -- q = x W_q and y = out W_o as weight-streaming launches of their own around the kernels of
 * elitekv_decode_step, q and out (rounded to dims->dtype) staying in the workspace.
 * EUNSUPPORTED unless bf16, B <= 64 and d_model and n_h d_h are multiples of 64; other errors as
 * elitekv_decode_step.
 * ------------------------------------------------------------------------------------------- */
size_t elitekv_block_step_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len,
                                          int32_t n_splits);
int elitekv_block_step(const elitekv_dims* dims, const void* x, const int32_t* pos, const int64_t* slot,
                       const int32_t* seq_len, int64_t B, int64_t max_seq_len, int64_t batch_stride_rows,
                       const void* W_q, const void* W_ke, const void* W_dkv, const void* W_uk, const void* W_uv,
                       const void* W_o, const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows,
                       void* y, void* ws, size_t ws_bytes, int32_t n_splits, void* hip_stream);

/* The whole attention block of a decode step of an S-LRD model (Section 2.1 projections around Section 3.2's
 * separated decomposition): elitekv_block_step with the cache rows, keys and values of elitekv_slrd_append /
 * elitekv_slrd_decode_attn (A_k [d_model, d_ck], A_v [d_model, d_c - d_ck], B_k [d_ck, n_h, d_h - 2r],
 * B_v [d_c - d_ck, n_h, d_h]; a latent row is [c^k | c^v]).  Always the composed form (see elitekv_block_step).
 * EINVAL unless 0 < d_ck < dims->d_c; EUNSUPPORTED unless bf16, B <= 64, d_model and n_h d_h multiples of 64. */
size_t elitekv_slrd_block_step_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B, int64_t max_seq_len,
                                               int32_t n_splits);
int elitekv_slrd_block_step(const elitekv_dims* dims, int32_t d_ck, const void* x, const int32_t* pos,
                            const int64_t* slot, const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                            int64_t batch_stride_rows, const void* W_q, const void* W_ke, const void* A_k,
                            const void* A_v, const void* B_k, const void* B_v, const void* W_o,
                            const int32_t* elite_idx, void* ke_plane, void* c_plane, int64_t plane_rows, void* y,
                            void* ws, size_t ws_bytes, int32_t n_splits, void* hip_stream);

/* The same step for separated latents: elitekv_slrd_append followed by elitekv_slrd_decode_attn. */
size_t elitekv_slrd_decode_step_workspace_bytes(const elitekv_dims* dims, int32_t d_ck, int64_t B,
                                                int64_t max_seq_len, int32_t n_splits);
int elitekv_slrd_decode_step(const elitekv_dims* dims, int32_t d_ck, const void* x, const void* q,
                             const int32_t* pos, const int64_t* slot, const int32_t* seq_len, int64_t B,
                             int64_t max_seq_len, int64_t batch_stride_rows, const void* W_ke, const void* A_k,
                             const void* A_v, const void* B_k, const void* B_v, const int32_t* elite_idx,
                             void* ke_plane, void* c_plane, int64_t plane_rows, void* out, void* ws,
                             size_t ws_bytes, int32_t n_splits, void* hip_stream);

/* ---------------------------------------------------------------------------------------------
 * Measurement-only companions (not part of the method).
 * ------------------------------------------------------------------------------------------- */

/*
 * Measurement only: elitekv_decode_attn restricted to the stages named in `stages`
 * (bit 0: query preparation, bit 1: split attention over the cache planes, bit 2: merge of the
 * splits + up-projection).  A stage that is left out reads what an earlier call with the same
 * arguments left in the workspace, so a full call must come first; the benchmark uses it to time
 * back-to-back launches of one stage with nothing else on the stream.  Same arguments and errors as
 * elitekv_decode_attn; EINVAL if stages is outside 1..7.  `out` is written only by stage bit 2.
 * d_ck = 0: the joint latent (elitekv_decode_attn); d_ck > 0: separated latents with W_uk = B^k_S and
 * W_uv = B^v_S (elitekv_slrd_decode_attn).
 */
int elitekv_decode_attn_stages(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                               const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                               int64_t batch_stride_rows, const void* W_uk, const void* W_uv,
                               const int32_t* elite_idx, const void* ke_plane, const void* c_plane,
                               int64_t plane_rows, void* out, void* ws, size_t ws_bytes,
                               int32_t n_splits, void* hip_stream, int32_t stages, int32_t d_ck);

/* Workspace bytes of elitekv_mha_decode.  n_splits == 0 means "auto". */
size_t elitekv_mha_decode_workspace_bytes(const elitekv_dims* dims, int64_t B, int64_t max_seq_len,
                                          int32_t n_splits);

/*
 * Comparator: ordinary RoPE multi-head decode attention over an UNCOMPRESSED cache at the same
 * (B, S, n_h, d_h) (Section 2.2: a RoPE model caches every chunk of k rotated, plus v).
 *   q [B, n_h, d_h] un-rotated (all d_h/2 chunks are rotated at q_pos[b] here);
 *   k_plane, v_plane [plane_rows, n_h, d_h], keys already rotated; out [B, n_h, d_h].
 * Only dims->n_heads, head_dim, dtype and rope_base are used.  head_dim must be <= 256.
 */
int elitekv_mha_decode(const elitekv_dims* dims, const void* q, const int32_t* q_pos,
                       const int32_t* seq_len, int64_t B, int64_t max_seq_len,
                       int64_t batch_stride_rows, const void* k_plane, const void* v_plane,
                       int64_t plane_rows, void* out, void* ws, size_t ws_bytes, int32_t n_splits,
                       void* hip_stream);

/*
 * Streaming-read probe: reads `bytes` bytes at `src` (16-byte aligned, bytes % 16 == 0) once with
 * wide coalesced non-temporal loads (the kind the attention kernel uses for cache rows) and folds them
 * into sink[0..grid) so the reads cannot be elided.  Gives the achievable HBM read rate to compare the
 * decode kernel against; launches of a gigabyte show the ceiling, launches of a plane's size include the
 * start-up of a launch.  sink: >= 4096 uint32.
 */
int elitekv_stream_read(const void* src, size_t bytes, uint32_t* sink, void* hip_stream);

/*
 * The same probe with the kind of load chosen by the caller, to show what the cache hint and the load
 * path are worth on this machine.  mode bit 0: the loads carry the non-temporal bit; bit 1: direct
 * global->LDS loads (the path the attention kernel's tiles take; 512 work-groups, every wave keeps 16 KiB in
 * flight, nothing reads the LDS) instead of loads into registers.  The direct form reads whole units of
 * 16 MiB only; *bytes_read (host pointer, may be NULL) receives the number of bytes the launch reads.
 * EINVAL unless 0 <= mode <= 3; other errors as elitekv_stream_read (mode 1 is that call).
 */
int elitekv_stream_read_mode(const void* src, size_t bytes, uint32_t* sink, int32_t mode, size_t* bytes_read,
                             void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* ELITEKV_H */
