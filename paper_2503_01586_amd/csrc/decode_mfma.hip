// bf16 decode attention over the EliteKV cache on the gfx950 matrix cores.
//
// One work-group handles one (sequence split, group of up to 32 heads, batch row).  All heads of
// the group are one MFMA dimension against the SHARED latent tile (Section 3.2: key and value
// share the latent c), so each cached row is read from HBM exactly once and serves both the key
// role (scores) and the value role (latent accumulation):
//
//   scores   S^T[token, head] = C[token, :] . Qt[head, :]      16x16x32 MFMA, A = latent tile rows,
//            B = absorbed query;  + per-head elite term ke[token, head, :] . qe[head, :]  (VALU)
//            (Section 3.1 score equation with W_uk absorbed into the query, Section 5)
//   softmax  online, in the log2 domain (the query is pre-scaled by log2(e)/sqrt(d_h))
//   values   U^T[col, head] += C^T[col, token] . P^T[token, head]   32x32x16 MFMA, A = the SAME
//            tile read transposed from LDS, B = the probabilities
//
// The latent dimension is split over the NW waves of the group (DC_W columns each): a wave keeps
// its slice of the absorbed query and of U in registers and computes partial scores over its
// slice; the waves exchange partial scores through LDS once per 16-token tile.  Tiles come in
// through direct global->LDS loads into a private slice per wave, double-buffered: the loads of
// tile i+1 are in flight while tile i is computed.
#include <type_traits>

#include "common.hpp"
#include "launch.hpp"

namespace ekv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4_t;

constexpr int kTile = 16;   // cached tokens per tile

struct AttnMfmaParams {
  const bf16_t* ke_plane;
  const bf16_t* c_plane;
  const float* qe;        // [B, n_h, 2r]   rotated, scaled elite query
  const bf16_t* qt;       // absorbed, scaled latent query q~ [B, n_h, d_q] in operand order (qt_packed_index)
  const int32_t* seq_len;
  float* part_m;          // [B, n_splits, HG*32]        split maxima (log2 domain)
  float* part_l;          // [B, n_splits, HG*32]        split sums
  bf16_t* part_u;         // [B, n_splits, HG*32, d_c]   split latent accumulators, head-major
  int n_h, d_c, n_splits, chunk, head_groups;
  int batch, pair_map;    // pair_map: 1-D grid, the two head groups of an item share an XCD (2: one head group, every batch row on one XCD)
  int q_per_seq;          // query rows per sequence (several queries share the cache rows of a sequence)
  int d_q, d_u;           // widths of the absorbed query and of the latent accumulators (d_c when joint)
  int q_slice;            // column slice per wave (DC_W), as the query preparation laid qt out
  int64_t max_seq_len, batch_stride_rows, plane_rows;
  // Fused decode step: the cache row of the newest token of every sequence (position seq_len - 1) is
  // still a set of partial sums (the append's contraction splits) when the launch begins.  The
  // work-group whose tiles include that position adds them up and stores the row before it requests
  // its first tile (both head groups of a 40-head shape do, each for itself); every other tile of the
  // launch lies below that position.  n_part = partials per batch row (= n_splits).
  int n_part;
  int fresh;              // 1: fused decode step
  const float* fr_partial;   // [fr_ks][batch][fr_stride] sums of the append's contraction splits (a cache row first)
  int fr_stride;
  const float2* fr_sincos;   // [batch][n_h * r]  (sin, cos) of the new token's elite chunks
  const int64_t* fr_slot;    // [batch] destination rows
  int fr_ks;
  bf16_t* fr_ke_out;         // the planes, writable
  bf16_t* fr_c_out;
  // arrival counters of the merge kernels that follow in the same call ([batch, n_h] ints): cleared here
  int* chunk_counters;
};

// LDS layout of one wave's tile slice (16 tokens x DC_W latent columns, bf16): blocks of
// 8 rows x 128 bytes (1 KiB, exactly what one direct-to-LDS load of 64 lanes x 16 bytes fills),
// block (rb, cb) at ((rb * NCB) + cb) KiB.  Inside a block the 16-byte chunk index is XOR-ed with
// swz(row) = ((row & 3) << 1) | ((row >> 2) & 1): eight rows read at one logical chunk hit eight
// different bank groups (row-wise b128 reads), and the 4 rows x 32 bytes a transposed b64 read
// covers hit four different 32-byte bank groups.
// A slice whose width is an odd multiple of 32 columns ends in one half-width block of
// 16 rows x 64 bytes (again 1 KiB, one load) behind the full blocks, chunk index XOR-ed with
// half_swz(row).
// The elite keys of a tile are double-buffered like the latent tile when the LDS has room for it;
// otherwise there is one buffer, refilled for the next tile as soon as the wave has read it.
template <int NW, int DC_W, int TWO_R>
struct AttnMfmaLayout {
  static_assert(DC_W % 32 == 0, "a wave's latent slice must be a whole number of 32-column MFMA steps");
  static_assert(NW == 2 || NW == 4 || NW == 8, "16 tokens are divided evenly among the waves");
  static constexpr int KS = DC_W / 32;                      // score k-steps per wave (K = 32)
  static constexpr int CT = DC_W / 32;                      // 32-column accumulator tiles per wave
  static constexpr int NCB = DC_W / 64;                     // full 128-byte column blocks per row
  static constexpr int HALF = (DC_W % 64) / 32;             // 1: a trailing half-width block
  static constexpr int NLOAD = 2 * NCB + HALF;              // direct-to-LDS loads per tile per wave
  static constexpr int HALF_OFF = 2 * NCB * 1024;           // the half-width block inside the slice
  static constexpr int WTILE = NLOAD * 1024;                // LDS bytes of one wave's tile slice
  static constexpr int TILE_BYTES = NW * WTILE;             // one buffer
  static constexpr int TPW = kTile / NW;                    // tokens each wave finalises
  static constexpr int EPL = TPW / 2;                       // ... per lane (lanes 0-31 / 32-63 alternate)
  static constexpr int X1_ROW = 33;                         // floats per token row (padded)
  static constexpr int X1 = NW * kTile * X1_ROW * 4;        // stage 1: every wave's partial scores
  static constexpr int X2_ROW = 20;                         // floats per head row (16 tokens, padded)
  static constexpr int X2 = 32 * X2_ROW * 4;                // stage 2: the final scores
  // elite keys of a tile: per wave the TPW tokens it finalises x the 32 heads of the group
  static constexpr int KE_ROW = 32 * TWO_R * 2;             // bytes of one token's group row
  static constexpr int KE_CPT = KE_ROW / 16;                // 16-byte chunks per token
  static constexpr int NKE = (TPW * KE_CPT + 63) / 64;      // direct-to-LDS loads per tile per wave
  static constexpr int KE_W = NKE * 1024;                   // LDS bytes of one wave's elite slice
  static constexpr int KE_BYTES = NW * KE_W;                // one buffer
  static constexpr int kLdsMax = 160 * 1024;                // LDS of a gfx950 compute unit
  static constexpr int X1_PAD = (X1 + 15) / 16 * 16;
  static constexpr int KE_BUFS = (2 * TILE_BYTES + 2 * KE_BYTES + X1_PAD + X2 <= kLdsMax) ? 2 : 1;
  static constexpr int KE_OFF = 2 * TILE_BYTES;
  static constexpr int X1_OFF = KE_OFF + KE_BUFS * KE_BYTES;
  static constexpr int X2_OFF = X1_OFF + X1_PAD;
  static constexpr int LDS_BYTES = X2_OFF + X2;
  // else: not compiled (the shape runs the generic kernels); 64 elite values per head beside a 128-column latent
  // (more elite than latent columns, two waves with eight tokens each to finalise) is not a shape worth a kernel
  static constexpr bool kFits = LDS_BYTES <= kLdsMax && !(TWO_R == 64 && NW == 2);
  // four waves with slices of up to 192 columns leave room for a second work-group on the compute unit (then at most
  // 256 registers per lane) -- unless the elite rows are so wide that the LDS holds one work-group only
  static constexpr int kGroupsPerCu = (NW == 4 && DC_W <= 192 && 2 * LDS_BYTES <= kLdsMax) ? 2 : 1;
};

__device__ __forceinline__ int tile_swz(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }
// half-width block (16 rows x 4 chunks): rows two apart differ in the 32-byte pair they use
__device__ __forceinline__ int half_swz(int row) { return (((row >> 1) & 1) << 1) | ((row >> 2) & 1); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// One direct global->LDS load: every lane fetches 16 bytes from its own global address; lane l's
// data lands at lds_base + l*16.  Issued through inline assembly so that the waits on these loads
// stay entirely under the kernel's control (vmcnt counting, see the tile loop).
// STREAM marks the load non-temporal: cache rows that are read once per step stream from HBM
// about 15 % faster that way (a plain read of 1 GiB through these loads: 6.0 TB/s, marked: 6.9 TB/s).
// Rows that a second work-group is about to re-read from the L2 (head-group pairs) are loaded unmarked.
template <int OFF, bool STREAM>
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_base) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off offset:%2 nt"
                 :
                 : "s"(lds_base), "v"(gptr), "n"(OFF)
                 : "memory", "m0");
  else
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off offset:%2"
                 :
                 : "s"(lds_base), "v"(gptr), "n"(OFF)
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// log2-domain slack before the running maximum is raised: probabilities stay below 2^8
constexpr float kRescaleSlack = 8.f;

// The newest token of sequence b in a fused decode step (NT threads): its cache row = the sum of the
// append's contraction splits (in split order, as append_finish adds them), the elite pairs rotated
// with the (sin, cos) the query preparation left behind (same position, same chunks), rounded to the
// cache type and stored at slot[b].  Run by the work-group(s) that own the tile the token lies in,
// before they request anything from the planes: the tile loads then bring the row in like any other.
template <int NT, int TWO_R>
__device__ __forceinline__ void store_new_token_row(const AttnMfmaParams& p, int b, int64_t slot) {
  const int tid = threadIdx.x;
  const int NE = p.n_h * TWO_R, N = NE + p.d_c;
  if (slot < 0 || slot >= p.plane_rows) return;            // a token without a row is not stored
  for (int pr = tid; pr < N / 2; pr += NT) {
    const int n = 2 * pr;
    float a0 = 0.f, a1 = 0.f;
    for (int s0 = 0; s0 < p.fr_ks; s0 += 8) {              // eight independent loads in flight; split order kept
      float2 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        v[u] = (s0 + u < p.fr_ks)
                   ? *reinterpret_cast<const float2*>(p.fr_partial + ((int64_t)(s0 + u) * p.batch + b) * p.fr_stride + n)
                   : make_float2(0.f, 0.f);
#pragma unroll
      for (int u = 0; u < 8; ++u) { a0 += v[u].x; a1 += v[u].y; }
    }
    if (n < NE) {                                          // pair index pr = h * r + j
      const float2 sc = p.fr_sincos[(int64_t)b * (NE / 2) + pr];
      const float o0 = a0 * sc.y - a1 * sc.x, o1 = a1 * sc.y + a0 * sc.x;
      a0 = o0; a1 = o1;
    }
    const uint32_t pk = pack_bf16x2(a0, a1);
    if (n < NE) *reinterpret_cast<uint32_t*>(p.fr_ke_out + slot * NE + n) = pk;
    else *reinterpret_cast<uint32_t*>(p.fr_c_out + slot * (int64_t)p.d_c + (n - NE)) = pk;
  }
}

// SEP = separated latents (Section 3.2, S-LRD): a cache row is [c^k (d_q columns) | c^v (d_u columns)];
// the waves whose slice lies in c^k only compute scores, the waves whose slice lies in c^v only
// accumulate values (d_q is a multiple of DC_W).  SEP = false is the joint latent: every wave does both.
// (Four-wave instantiations with slices of up to 192 columns that use at most 80 KB of LDS are
// compiled for two work-groups per compute unit, i.e. at most 256 registers per lane: kGroupsPerCu.)
// SMODE: which loads of cache rows are marked non-temporal (see dma16): 1 = all (nobody else reads the rows),
// 2 = those of the odd steps only (head-group pairs: at odd steps a work-group is the second and last reader of its tile).
template <int NW, int DC_W, int TWO_R, bool SEP, int SMODE>
__global__ __launch_bounds__(NW * 64, (AttnMfmaLayout<NW, DC_W, TWO_R>::kGroupsPerCu)) void attn_mfma_kernel(const AttnMfmaParams p) {
  using L = AttnMfmaLayout<NW, DC_W, TWO_R>;
  constexpr int KS = L::KS, CT = L::CT, NCB = L::NCB, EPL = L::EPL, TPW = L::TPW;
  constexpr int KCH = TWO_R / 8;                 // 16-byte chunks of one head's elite key
  // One wave per SIMD (512 registers per lane, half of them accumulation registers): the accumulators are pinned to
  // the AGPRs by hand.  Left to the compiler, such a kernel keeps the accumulators in VGPRs and parks the absorbed
  // query in AGPRs instead -- copying its registers right after the loads below were issued, before they have landed.
  constexpr bool ACC_AGPR = NW == 4 && L::kGroupsPerCu == 1;
  constexpr bool KE2 = L::KE_BUFS == 2 || TWO_R == 0;
  // direct-to-LDS loads that may still be in flight when a tile is consumed: with two elite-key
  // buffers the whole next tile, with one only its latent part (its elite keys are requested in
  // the middle of the current tile, before the latent loads of the tile after)
  constexpr int IN_FLIGHT = KE2 ? L::NLOAD + (TWO_R > 0 ? L::NKE : 0) : L::NLOAD;

  // Every kernel argument the start-up uses is fetched now, in one round trip of the scalar cache (left to
  // itself the compiler fetches them block by block where they are first used: three trips of about 0.4 us
  // each, one after the other, before the first load of the launch can go out).
  asm volatile("" ::"s"(p.ke_plane), "s"(p.c_plane), "s"(p.qe), "s"(p.qt), "s"(p.seq_len), "s"(p.n_h), "s"(p.d_c),
               "s"(p.n_splits), "s"(p.head_groups), "s"(p.batch), "s"(p.pair_map), "s"(p.q_per_seq), "s"(p.d_q),
               "s"(p.max_seq_len), "s"(p.batch_stride_rows), "s"(p.plane_rows), "s"(p.fresh), "s"(p.chunk_counters),
               "s"(p.n_part), "s"(p.fr_partial), "s"(p.fr_stride), "s"(p.fr_sincos), "s"(p.fr_slot), "s"(p.fr_ks),
               "s"(p.fr_ke_out), "s"(p.fr_c_out), "s"(gridDim.x), "s"(gridDim.y));
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  // Which DC_W-column slice of the latent row this wave works on: rotated from work-group to
  // work-group.  The work-groups of an XCD run in step and all fetch the same absorbed query from its
  // L2; when they all ask for the same lines at the same moment the L2 serves them one after the
  // other (a compute unit then gets a fifth of the rate of independent streams).  Rotated, eight
  // groups of them ask for eight different parts of the query at any moment.  Partial scores are
  // exchanged by slice index and summed in slice order, so the result does not depend on the rotation.
  const int lin_wg = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
  const int cw = (wave + (lin_wg >> 3)) & (NW - 1);
  const int nwk = SEP ? p.d_q / DC_W : NW;               // slices that enter the scores
  const bool do_s = !SEP || cw < nwk;                    // this wave's slice enters the scores
  const bool do_v = !SEP || cw >= nwk;                   // this wave's slice is accumulated as values
  const int vwave = SEP ? cw - nwk : cw;                 // position of the slice among the value slices
  int split = blockIdx.x, hg = blockIdx.y, b = blockIdx.z;
  if (p.pair_map == 2) {
    // One head group, a multiple of eight batch rows: all splits of batch row b run on XCD b % 8 (work-groups go to
    // the XCDs round-robin by linear index), so an XCD's L2 fetches the absorbed queries of its own rows only
    // instead of every row's (at 64 rows that is 3 MB per XCD, which the streamed cache rows keep evicting:
    // 294 MB fetched per launch against 268 MB of cache).
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    b = (slot / p.n_splits) * 8 + xcd;
    split = slot % p.n_splits;
    if (b >= p.batch) return;
  } else if (p.pair_map) {
    // Two head groups read the same latent rows.  Work-groups go to the eight XCDs round-robin by
    // linear index, so indices i and i + 8 land on the same XCD back to back: they are given the
    // two head groups of one (split, batch row) item, and the second reader of a row finds it in
    // that XCD's L2 instead of fetching it from HBM again.
    // (3: a multiple of eight batch rows, and every row's splits on XCD b % 8 as above)
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int per_row = p.n_splits;
    hg = slot & 1;
    if (p.pair_map == 3) {
      b = ((slot >> 1) / per_row) * 8 + xcd;
      split = (slot >> 1) % per_row;
      if (b >= p.batch) return;
    } else {
      const int item = (slot >> 1) * 8 + xcd;
      if (item >= per_row * p.batch) return;
      split = item % per_row;
      b = item / per_row;
    }
  }
  if (split == 0 && hg == 0)
    for (int i = tid; i < p.n_h; i += NW * 64) p.chunk_counters[(int64_t)b * p.n_h + i] = 0;
  // ---- the query
  // This wave's slice of the absorbed query as the B operand of the 16x16x32 score MFMAs (lane l holds
  // head hh*16 + l%16, latent columns 32*ks + 8*(l/16) .. +8) and the lane's head's rotated elite
  // query.  A compute unit keeps only so many memory requests in flight and serves them in the order
  // they were issued, so the 128 KB of query (quick: they come from the L2) are requested right behind
  // the first tile (slow: HBM; see the start-up below) and ahead of the second: they land with the first
  // tile and never queue up behind later ones.  The loads are issued
  // from assembly, like the tile loads: a load the compiler knows of makes it wait, before the
  // first use of the value, with a count that ignores the tile loads issued behind it, i.e. for all
  // of them.  The registers are first read in compute(), after the loop's wait for the first tile.
  // Heads beyond n_h (second head group of 40 heads) read the last
  // head's query: their results are never stored.
  const int head = hg * 32 + n;
  const bool head_ok = head < p.n_h;
  const int head_c = head_ok ? head : p.n_h - 1;
  const int i16 = lane & 15, q16 = lane >> 4;
  u32x4 Qb[KS][2];
  // the lane's head's rotated elite query, four floats per register quad; the quads are read in place (element by
  // element) and never copied: a copy made before the loads below have landed would take stale registers with it
  // and leave the loaded values to land in registers the compiler has already given to something else
  f32x4 qv[TWO_R > 0 ? TWO_R / 4 : 1];
  int32_t len_raw;                                       // seq_len[b] through the scalar cache: not behind the vector loads
  asm volatile("s_load_dword %0, %1, 0x0" : "=s"(len_raw) : "s"(p.seq_len + __builtin_amdgcn_readfirstlane(b)) : "memory");
  // fr_slot[b] (fused step: the row of the newest token) in the same trip: fetched by the owner work-group where it
  // finishes that row, it would be one more trip to memory (about 1.5 us) ahead of the split sums' loads.  Outside
  // a fused step the host points fr_slot at readable workspace bytes and the value is not used.
  int64_t slot_raw;
  asm volatile("s_load_dwordx2 %0, %1, 0x0" : "=s"(slot_raw) : "s"(p.fr_slot + __builtin_amdgcn_readfirstlane(b)) : "memory");
  auto load_query = [&]() {
    {
      // every wave loads a slice, also the waves of a separated latent that only accumulate values (they read slice 0
      // and never use it): a load under a condition would reach the loop through a merge of two register versions,
      // which the compiler may realise as copies made right behind the loads, before they have landed
      const int cq = do_s ? cw : 0;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int hq = min(hg * 32 + hh * 16 + i16, p.n_h - 1);
        const bf16_t* qrow = p.qt + qt_packed_index(b, hq, cq * DC_W + 8 * q16, p.head_groups, p.d_q, DC_W);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)                      // one contiguous KiB per instruction
          asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(Qb[ks][hh]) : "v"(qrow + ks * 1024) : "memory");
      }
    }
    if constexpr (TWO_R > 0) {
      const float* qer = p.qe + ((int64_t)b * p.n_h + head_c) * TWO_R;
#pragma unroll
      for (int j = 0; j < TWO_R / 4; ++j) asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(qv[j]) : "v"(qer + 4 * j) : "memory");
    }
  };
  const int64_t row0 = (int64_t)(b / p.q_per_seq) * p.batch_stride_rows;

  char* ctile0 = smem + wave * L::WTILE;                 // buffer 0; buffer 1 is TILE_BYTES further
  char* ketile0 = smem + L::KE_OFF + wave * L::KE_W;     // buffer 0; buffer 1 (if any) is KE_BYTES further
  float* x1 = reinterpret_cast<float*>(smem + L::X1_OFF);
  float* x2 = reinterpret_cast<float*>(smem + L::X2_OFF);

  // Split s takes the 16-token tiles s, s + n_splits, s + 2 n_splits, ...: at any moment the
  // work-groups of a batch row read one contiguous window of the planes that moves through the
  // sequence (DRAM-page friendly); the softmax does not care about token order.
  const int64_t t0 = (int64_t)split * kTile;
  const int64_t t_step = (int64_t)p.n_splits * kTile;
  const int64_t pidx = ((int64_t)b * p.n_part + split) * (p.head_groups * 32) + hg * 32;
  // Rows the tile loads may touch: until seq_len[b] has arrived, the bound the host knows (the planes'
  // extent); afterwards the sequence's length.
  const int64_t t_cap = min(p.max_seq_len, p.plane_rows - row0);
  int64_t t_end = t_cap;

  f32x16 uacc[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) uacc[ct] = (f32x16)(0.f);
  float m_run = -INFINITY, l_run = 0.f;

  const int64_t crow_bytes = (int64_t)p.d_c * 2;
  const int64_t krow_bytes = (int64_t)p.n_h * TWO_R * 2;
  // loader: lane l fills slot (row l/8, position l%8) of every block; it fetches the logical
  // chunk that the swizzle puts there
  const int ld_row = lane >> 3;
  const char* cbase = reinterpret_cast<const char*>(p.c_plane) + (int64_t)cw * DC_W * 2 +
                      (((lane & 7) ^ tile_swz(ld_row)) << 4);
  const char* hbase = reinterpret_cast<const char*>(p.c_plane) + ((int64_t)cw * DC_W + NCB * 64) * 2 +
                      (((lane & 3) ^ half_swz(lane >> 2)) << 4);
  // elite-key loader: slot c = i*64 + lane of the wave's slice is (token c / KE_CPT, chunk c % KE_CPT)
  const char* kbase = reinterpret_cast<const char*>(p.ke_plane);

  // LDS read offsets (inside a wave's tile slice) that do not change from tile to tile.
  // score A operand: token row i16, logical chunk 4*ks + q16 -> block (i16/8, ks/2)
  const int a_off = (i16 >> 3) * (NCB * 1024) + (i16 & 7) * 128;
  const int a_swz = tile_swz(i16 & 7);
  const int a_c0 = a_off + ((q16 ^ a_swz) << 4);                // even ks: in-block chunks 0..3
  const int a_c1 = a_off + (((4 | q16) ^ a_swz) << 4);          // odd ks:  in-block chunks 4..7
  // value A operand (transposed b64 read): 16-lane group q16 serves tokens 8*(q16/2) + {0..3 | 4..7}
  // and columns 32*ct + 16*(q16%2) + ..; source lane s supplies row s/4, 4 columns at 4*(s%4)
  const int tr_lo = ((q16 & 1) << 1) | ((i16 & 3) >> 1);        // 16-byte chunk inside the 32 columns
  const int tr_base = (q16 >> 1) * (NCB * 1024) + ((i16 & 1) << 3);
  int tr_off[2][2];                                             // [rows 0-3 | 4-7][ct parity]
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int r8 = 4 * e + (i16 >> 2);
#pragma unroll
    for (int par = 0; par < 2; ++par)
      tr_off[e][par] = tr_base + r8 * 128 + ((((par << 2) | tr_lo) ^ tile_swz(r8)) << 4);
  }
  // the same two reads inside the half-width block (row-major 16 x 64 bytes)
  const int ah_off = L::HALF_OFF + i16 * 64 + ((q16 ^ half_swz(i16)) << 4);
  int trh_off[2];
#pragma unroll
  for (int e = 0; e < 2; ++e) {
    const int row = 8 * (q16 >> 1) + 4 * e + (i16 >> 2);
    trh_off[e] = L::HALF_OFF + row * 64 + ((tr_lo ^ half_swz(row)) << 4) + ((i16 & 1) << 3);
  }
  // stage-2 ownership: this wave finalises tokens wave*TPW + g + 2*e (e < EPL) for head n
  const int own_t0 = wave * TPW + g;

  auto issue_c = [&](int64_t tile_t0, char* ctile, auto nt) {
    constexpr bool STREAM = decltype(nt)::value;
    const uint32_t cl = __builtin_amdgcn_readfirstlane(lds_addr(ctile));
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
      const int64_t t = min(tile_t0 + rb * 8 + ld_row, t_end - 1);
      const char* gp = cbase + (row0 + t) * crow_bytes;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) dma16<0, STREAM>(gp + cb * 128, cl + (rb * NCB + cb) * 1024);
    }
    if (L::HALF) {   // lane l fills slot (row l/4, position l%4) of the half-width block
      const int hr = lane >> 2;
      const int64_t t = min(tile_t0 + hr, t_end - 1);
      dma16<0, STREAM>(hbase + (row0 + t) * crow_bytes, cl + L::HALF_OFF);
    }
  };
  auto issue_ke = [&](int64_t tile_t0, char* ketile, auto nt) {
    constexpr bool STREAM = decltype(nt)::value;
    if (TWO_R > 0) {
      const uint32_t kl = __builtin_amdgcn_readfirstlane(lds_addr(ketile));
#pragma unroll
      for (int i = 0; i < L::NKE; ++i) {
        const int c = i * 64 + lane;
        const int tl = min(c / L::KE_CPT, TPW - 1), ch = c % L::KE_CPT;
        const int hd = min(hg * 32 + ch / KCH, p.n_h - 1);
        const int64_t t = min(tile_t0 + wave * TPW + tl, t_end - 1);
        dma16<0, STREAM>(kbase + (row0 + t) * krow_bytes + ((int64_t)hd * KCH + ch % KCH) * 16, kl + i * 1024);
      }
    }
  };
  auto issue = [&](int64_t tile_t0, char* ctile, char* ketile, auto nt) {
    issue_c(tile_t0, ctile, nt);
    if (KE2) issue_ke(tile_t0, ketile, nt);
  };
  using NtEven = std::integral_constant<bool, SMODE == 1>;   // even steps (buffer 0)
  using NtOdd = std::integral_constant<bool, SMODE != 0>;    // odd steps (buffer 1)

  auto compute = [&](int64_t tile, const char* ctile, char* ketile, int64_t next_tile, auto nt_next) {
    // ---- partial scores over this wave's latent slice, two head halves
    f32x4 sd[2] = {(f32x4)(0.f), (f32x4)(0.f)};
    if (do_s) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      if (KS > 8 && ks % 4 == 0) asm volatile("" ::: "memory");   // wide slices: bound the operand look-ahead
      const int aoff = (L::HALF && ks == 2 * NCB) ? ah_off : (ks >> 1) * 1024 + ((ks & 1) ? a_c1 : a_c0);
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(ctile + aoff);
      sd[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, Qb[ks][0]), sd[0], 0, 0, 0);
      sd[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, Qb[ks][1]), sd[1], 0, 0, 0);
    }
    }
    // ---- stage 1: publish them as x1[slice][token][head]; lane holds tokens 4*q16 + v, head hh*16 + i16
    if (do_s) {
      float* xw = x1 + (cw * kTile + 4 * q16) * L::X1_ROW + i16;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int v = 0; v < 4; ++v) xw[v * L::X1_ROW + hh * 16] = sd[hh][v];
    }
    // elite term of the (token, head) pairs this wave finalises (overlaps the barrier)
    float fin[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      float d = 0.f;
      if (TWO_R > 0) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
          const uint4 kv = *reinterpret_cast<const uint4*>(ketile + (((g + 2 * e) * L::KE_CPT + n * KCH + c) << 4));
          const uint32_t w[4] = {kv.x, kv.y, kv.z, kv.w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            d = fmaf(qv[2 * c + i / 2][2 * (i % 2)], __uint_as_float(w[i] << 16), d);
            d = fmaf(qv[2 * c + i / 2][2 * (i % 2) + 1], __uint_as_float(w[i] & 0xffff0000u), d);
          }
        }
      }
      fin[e] = d;
    }
    __syncthreads();
    if (!KE2 && next_tile < t_end) {   // single elite-key buffer: this wave has read its slice
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      issue_ke(next_tile, ketile, nt_next);
    }
    // ---- stage 2: sum the NW partials in a fixed order, publish as x2[head][token]
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const int tok = own_t0 + 2 * e;
#pragma unroll
      for (int w2 = 0; w2 < NW; ++w2)
        if (!SEP || w2 < nwk) fin[e] += x1[(w2 * kTile + tok) * L::X1_ROW + n];
      x2[n * L::X2_ROW + tok] = fin[e];
    }
    __syncthreads();
    // ---- online softmax; lane = head n, tokens 8*g + j
    float s[8];
    {
      const f32x4 lo = *reinterpret_cast<const f32x4*>(x2 + n * L::X2_ROW + 8 * g);
      const f32x4 hi = *reinterpret_cast<const f32x4*>(x2 + n * L::X2_ROW + 8 * g + 4);
      s[0] = lo[0]; s[1] = lo[1]; s[2] = lo[2]; s[3] = lo[3];
      s[4] = hi[0]; s[5] = hi[1]; s[6] = hi[2]; s[7] = hi[3];
    }
    float tmax = -INFINITY;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      s[j] = (tile + 8 * g + j < t_end) ? s[j] : -INFINITY;
      tmax = fmaxf(tmax, s[j]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    // the reference maximum is raised only when a score exceeds it by more than the slack
    const float m_new = (tmax > m_run + kRescaleSlack || m_run == -INFINITY) ? tmax : m_run;
    const float alpha = exp2f(m_run - m_new);
    float psum = 0.f;
    bf16x8 P;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float pv = exp2f(s[j] - m_new);
      psum += pv;
      P[j] = (__bf16)pv;
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__any(alpha != 1.f)) {
      if (ACC_AGPR) {
        // One wave per SIMD: the accumulator tiles are kept in the accumulation registers (AGPRs).
        // Rescaling them as ordinary vector arithmetic would make the compiler hold every tile in
        // VGPRs across the whole loop; the explicit moves pin them to AGPRs instead.
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
          for (int j = 0; j < 16; ++j) {
            float y, z;
            asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(y) : "a"(uacc[ct][j]));
            y *= alpha;
            asm volatile("v_accvgpr_write_b32 %0, %1\n\ts_nop 2" : "=a"(z) : "v"(y));   // + wait states before an MFMA reads it
            uacc[ct][j] = z;
          }
        }
      } else {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) uacc[ct] *= alpha;
      }
    }
    // ---- latent accumulation: U^T += C^T P^T, the tile read transposed from LDS
    if (do_v) {
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      if (CT > 8 && ct % 4 == 0) asm volatile("" ::: "memory");
      const bool in_half = L::HALF && ct == 2 * NCB;
      const char* trp = ctile + (in_half ? 0 : (ct >> 1) * 1024);
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_t*)(trp + (in_half ? trh_off[0] : tr_off[0][ct & 1])));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (lds_s16x4_t*)(trp + (in_half ? trh_off[1] : tr_off[1][ct & 1])));
      const s16x8 a16 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      uacc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a16), P, uacc[ct], 0, 0, 0);
    }
    }
  };

  // two tiles per trip so that buffer and register-set indices are compile-time
  char* ctile1 = ctile0 + L::TILE_BYTES;
  char* ketile1 = KE2 ? ketile0 + L::KE_BYTES : ketile0;
  // The second work-group of a head-group pair swaps neighbouring tiles (see tile_at below).
  const int swp = ((p.pair_map & 1) && hg) ? 1 : 0;

  // ---- start-up.  seq_len[b] takes a trip to memory (about 1.5 us after a launch); the first tile does not wait
  // for it.  Its rows are requested at once, on the assumption that the tile lies wholly inside the sequence:
  // the rows are inside the planes whatever seq_len says (t_cap), and when the assumption holds -- every split
  // but the one at the sequence's end -- these are exactly the loads the tile needs.  The query follows (it comes
  // from the L2 and is first read together with the tile).  A work-group whose first tile turns out to be cut by
  // the sequence's end, to hold the newest token's row (fused step), or not to exist, lets the loads land,
  // discards them and starts over with the length known.
  const int64_t spec_t = t0 + swp * t_step;
  const bool spec = spec_t + kTile <= t_cap;
  if (spec) {
    issue_c(spec_t, ctile0, NtEven{});
    issue_ke(spec_t, ketile0, NtEven{});
  }
  if (!p.fresh) load_query();
  asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(len_raw), "+s"(slot_raw) : : "memory");
  {
    int64_t len = len_raw;
    len = min(len, t_cap);
    t_end = max(len, (int64_t)0);
  }
  // rows the speculative loads may have covered: all below the sequence's end, and below the newest token's row,
  // which is still being put together when a fused step begins
  const bool spec_ok = spec && spec_t + kTile <= t_end - (p.fresh ? 1 : 0);
  if (spec && !spec_ok) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  if (p.fresh) {
    // Fused decode step: the work-group whose tiles include the newest token's position (both head groups
    // of it, each for itself) finishes that token's cache row and stores it, and waits for the stores,
    // before any wave of it requests that tile; with nothing attended the row is still stored, by one group.
    // This comes before the query loads: nothing may touch their registers until they have landed.
    const bool own = t_end > 0 ? split == (int)(((t_end - 1) / kTile) % p.n_splits) : (split == 0 && hg == 0);
    if (own) {
      store_new_token_row<NW * 64, TWO_R>(p, b, slot_raw);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    load_query();
  }
  __builtin_amdgcn_s_barrier();                          // a new row is stored before any wave asks for its tile

  if (t0 >= t_end) {   // empty split: weight 0 in the merge (l == 0), accumulator rows zeroed
    if (wave == 0 && g == 0) {
      p.part_m[pidx + n] = -INFINITY;
      p.part_l[pidx + n] = 0.f;
    }
    uint4* z = reinterpret_cast<uint4*>(p.part_u + pidx * (int64_t)p.d_u);
    for (int i = tid; i < 4 * p.d_u; i += NW * 64) z[i] = make_uint4(0, 0, 0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // the query loads (and the stores) are done with the registers
    return;
  }

  // The i-th tile this work-group processes.  The second work-group of a head-group pair swaps
  // neighbouring tiles: at any moment the two fetch DIFFERENT rows from HBM, and each finds the
  // tile its partner fetched one step earlier in the XCD's L2 (twice as many independent streams
  // as when both ask for the same rows at the same time).
  const int n_my = (int)((t_end - t0 + t_step - 1) / t_step);
  auto tile_at = [&](int i) -> int64_t {     // t_end stands for "no such tile"
    if (i >= n_my) return t_end;
    const int j = i ^ swp;
    return t0 + (int64_t)(j < n_my ? j : i) * t_step;
  };
  const int64_t first = tile_at(0), second = tile_at(1);
  // query loads of a wave that stand behind the speculative tile loads in the order of return
  constexpr int NQ = 2 * KS + TWO_R / 4;
  if (!spec_ok) {
    issue_c(first, ctile0, NtEven{});
    issue_ke(first, ketile0, NtEven{});
  }
  if (second < t_end) {
    // All work-groups start together.  Requests for the second tile go out once half of the first has
    // arrived: the first tile is then complete (and being computed) after one tile's worth of bus time
    // instead of two, while the bus still never runs dry.
    if (spec_ok) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L::NLOAD / 2 + (TWO_R > 0 ? L::NKE : 0) + NQ) : "memory");
    else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(L::NLOAD / 2 + (TWO_R > 0 ? L::NKE : 0)) : "memory");
    issue(second, ctile1, ketile1, NtOdd{});
  }
  for (int i = 0; i < n_my; i += 2) {
    const int64_t ta = tile_at(i), tb = tile_at(i + 1), tc = tile_at(i + 2), td = tile_at(i + 3);
    if (tb < t_end) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(IN_FLIGHT) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    compute(ta, ctile0, ketile0, tb, NtOdd{});
    if (tb >= t_end) break;
    if (tc < t_end) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // buffer 0 was last read one tile ago
      issue(tc, ctile0, ketile0, NtEven{});
      asm volatile("s_waitcnt vmcnt(%0)" ::"n"(IN_FLIGHT) : "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    compute(tb, ctile1, ketile1, tc, NtEven{});
    if (td < t_end) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      issue(td, ctile1, ketile1, NtOdd{});
    }
  }

  // ---- write this split's partial (m, l, U)
  const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
  if (wave == 0 && g == 0) {
    p.part_m[pidx + n] = m_run;
    p.part_l[pidx + n] = head_ok ? l_tot : 0.f;
  }
  // U goes out head-major in bf16.  The accumulators hold, per lane, one head and scattered
  // columns; they are transposed through LDS (free now) so that global stores are row-contiguous.
  constexpr int TSTR = DC_W * 2 + 16;                       // bytes per head row in LDS
  static_assert(NW * 32 * TSTR <= L::LDS_BYTES, "transpose staging exceeds the LDS allocation");
  __syncthreads();                                          // every wave is done with its tile slices
  char* tt = smem + wave * (32 * TSTR);
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint2 pk;
      pk.x = pack_bf16x2(uacc[ct][4 * j], uacc[ct][4 * j + 1]);
      pk.y = pack_bf16x2(uacc[ct][4 * j + 2], uacc[ct][4 * j + 3]);
      *reinterpret_cast<uint2*>(tt + n * TSTR + (ct * 32 + 8 * j + 4 * g) * 2) = pk;
    }
  }
  constexpr int CPRW = DC_W * 2 / 16;                       // 16-byte chunks per head row
  char* ubase = reinterpret_cast<char*>(p.part_u) + (pidx * (int64_t)p.d_u + (int64_t)(do_v ? vwave : 0) * DC_W) * 2;
#pragma unroll
  for (int i = 0; i < 32 * CPRW / 64; ++i) {
    const int idx = i * 64 + lane;
    const int row = idx / CPRW, ch = idx % CPRW;
    const uint4 v = *reinterpret_cast<const uint4*>(tt + row * TSTR + ch * 16);
    // non-temporal: the 25 MB of partials of a launch are on their way to memory while other work-groups still
    // stream, instead of leaving the eight L2s in one burst when the kernel ends
    if (do_v && hg * 32 + row < p.n_h) {
      __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(ubase + (int64_t)row * p.d_u * 2 + ch * 16));
    }
  }
}

// ---------------------------------------------------------------------------------------------
template <int NW, int DC_W, int TWO_R, bool SEP, int SMODE>
static hipError_t launch_attn_as(const AttnMfmaParams& prm, int64_t B, hipStream_t stream) {
  using L = AttnMfmaLayout<NW, DC_W, TWO_R>;
  static LdsLimit lds_limit;
  const hipError_t le = raise_lds_limit(
      lds_limit, reinterpret_cast<const void*>(&attn_mfma_kernel<NW, DC_W, TWO_R, SEP, SMODE>), L::LDS_BYTES);
  if (le != hipSuccess) return le;
  const int per_row = prm.n_splits;
  const dim3 grid = prm.pair_map == 2 ? dim3((unsigned)((B + 7) / 8 * 8 * per_row), 1, 1)
                  : prm.pair_map == 3 ? dim3((unsigned)((B + 7) / 8 * 16 * per_row), 1, 1)
                  : prm.pair_map ? dim3((unsigned)((per_row * B + 7) / 8 * 16), 1, 1)
                                 : dim3(per_row, prm.head_groups, (unsigned)B);
  attn_mfma_kernel<NW, DC_W, TWO_R, SEP, SMODE><<<grid, NW * 64, L::LDS_BYTES, stream>>>(prm);
  return hipGetLastError();
}

template <int NW, int DC_W, int TWO_R, bool SEP>
static hipError_t launch_attn(const AttnMfmaParams& prm, int64_t B, hipStream_t stream) {
  if constexpr (AttnMfmaLayout<NW, DC_W, TWO_R>::kFits) {
    // head-group pairs share their rows through the L2; every other launch reads a row once
    return (prm.pair_map & 1) ? launch_attn_as<NW, DC_W, TWO_R, SEP, 2>(prm, B, stream)
                        : launch_attn_as<NW, DC_W, TWO_R, SEP, 1>(prm, B, stream);
  } else {
    return hipErrorInvalidValue;                            // decode_mfma_supported() keeps such shapes away
  }
}

// does the tile set of (waves, slice width) hold its LDS layout with elite rows of 2r values?
template <int NW, int DC_W>
static bool layout_fits(int two_r) {
  return two_r == 8 ? AttnMfmaLayout<NW, DC_W, 8>::kFits
       : two_r == 16 ? AttnMfmaLayout<NW, DC_W, 16>::kFits
       : two_r == 32 ? AttnMfmaLayout<NW, DC_W, 32>::kFits
       : two_r == 64 ? AttnMfmaLayout<NW, DC_W, 64>::kFits : false;
}

// wave slice of the compiled instantiation for a latent row of d_c columns; 0 = none
// The compiled instantiations: every latent width that is a multiple of 128 up to 2048 (the
// hardware-friendly widths of Appendix C) and 1920 (the 13B benchmark shape), as
// X(d_c, waves, columns per wave).  Eight waves x <= 192 columns run two waves per SIMD; four waves
// with wider slices run one wave per SIMD with the accumulators in AGPRs.
#define EKV_ATTN_SHAPES(X)                                                                            \
  X(2048, 4, 512) X(1920, 4, 480) X(1792, 4, 448) X(1664, 4, 416) X(1536, 8, 192) X(1408, 4, 352)     \
  X(1280, 8, 160) X(1152, 4, 288) X(1024, 8, 128) X(896, 4, 224) X(768, 4, 192) X(640, 4, 160)        \
  X(512, 4, 128) X(384, 4, 96) X(256, 4, 64) X(128, 2, 64)

static void shape_of(int d_c, int* nw, int* dcw) {
  *nw = 0; *dcw = 0;
#define X(DC, NWV, DCW) if (d_c == DC) { *nw = NWV; *dcw = DCW; }
  EKV_ATTN_SHAPES(X)
#undef X
}
static int slice_width(int d_c) { int nw, w; shape_of(d_c, &nw, &w); return w; }
int decode_mfma_slice_width(int d_c) { return slice_width(d_c); }

// work-groups of the attention kernel that fit one compute unit (see the launch bounds of the kernel)
int decode_mfma_groups_per_cu(const elitekv_dims& d) {
  int g = 1;
  const int two_r = 2 * d.r;
#define X(DC, NWV, DCW)                                                                         \
  if (d.d_c == DC)                                                                              \
    g = two_r == 8 ? AttnMfmaLayout<NWV, DCW, 8>::kGroupsPerCu                                  \
      : two_r == 16 ? AttnMfmaLayout<NWV, DCW, 16>::kGroupsPerCu                                \
      : two_r == 32 ? AttnMfmaLayout<NWV, DCW, 32>::kGroupsPerCu                                \
      : two_r == 64 ? AttnMfmaLayout<NWV, DCW, 64>::kGroupsPerCu : 1;
  EKV_ATTN_SHAPES(X)
#undef X
  return g;
}

bool decode_mfma_supported(const elitekv_dims& d, int d_ck) {
  if (d.dtype != ELITEKV_BF16) return false;
  if ((d.head_dim != 128 && d.head_dim != 64) || (d.head_dim - 2 * d.r) % 8) return false;
  const int two_r = 2 * d.r;
  if (two_r != 8 && two_r != 16 && two_r != 32 && two_r != 64) return false;   // r = 4, 8, 16, 32 elite chunks per head
  const int w = slice_width(d.d_c);
  if (w == 0) return false;
  bool fits = false;                                      // 2r = 32 and 64 with the widest rows do not fit the LDS
#define X(DC, NWV, DCW) if (d.d_c == DC) fits = layout_fits<NWV, DCW>(two_r);
  EKV_ATTN_SHAPES(X)
#undef X
  if (!fits) return false;
  if (d_ck > 0 && w > 256) return false;    // the one-wave-per-SIMD instantiations are compiled for the joint latent only
  // separated latents with 64 elite values per head, or 32 beside 224-column slices: the compiled code parks query
  // registers in AGPRs right behind their loads (before they have landed), so these shapes take the generic kernels
  if (d_ck > 0 && (two_r == 64 || (two_r == 32 && w == 224))) return false;
  // separated latents: whole wave slices on either side of the boundary
  // (and the value part a whole number of the merge kernels' 64-column chunks)
  return d_ck == 0 || (d_ck > 0 && d_ck < d.d_c && d_ck % w == 0 && (d.d_c - d_ck) % 64 == 0);
}

hipError_t launch_decode_mfma(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  float* qe = (float*)(a.ws + p.off_qe);
  bf16_t* qt = (bf16_t*)(a.ws + p.off_qt);
  AttnMfmaParams prm;
  prm.ke_plane = (const bf16_t*)a.ke_plane; prm.c_plane = (const bf16_t*)a.c_plane;
  prm.qe = qe; prm.qt = qt; prm.seq_len = a.seq_len;
  prm.part_m = (float*)(a.ws + p.off_m); prm.part_l = (float*)(a.ws + p.off_l);
  prm.part_u = (bf16_t*)(a.ws + p.off_u);
  prm.n_h = d.n_heads; prm.d_c = d.d_c; prm.n_splits = p.n_splits; prm.chunk = p.chunk;
  prm.head_groups = p.head_groups; prm.max_seq_len = a.max_seq_len;
  prm.batch_stride_rows = a.batch_stride_rows; prm.plane_rows = a.plane_rows;
  prm.batch = (int)a.B;
  const bool rows_to_xcds = a.B >= 8 && a.B % 8 == 0 && a.q_per_seq == 1;
  prm.pair_map = p.head_groups == 2 ? (rows_to_xcds ? 3 : 1) : rows_to_xcds ? 2 : 0;
  prm.d_q = p.d_q; prm.d_u = p.d_u; prm.q_per_seq = a.q_per_seq; prm.q_slice = slice_width(d.d_c);
  prm.n_part = p.n_part; prm.fresh = p.fresh;
  // fr_slot is read (through the scalar cache) by every work-group of every launch; outside a fused step it points
  // at the first bytes of the workspace (the elite queries: at least 32 bytes per batch row) and the value is ignored
  prm.fr_partial = nullptr; prm.fr_sincos = nullptr; prm.fr_slot = (const int64_t*)(a.ws + p.off_qe); prm.fr_ks = 0; prm.fr_stride = 0;
  prm.fr_ke_out = nullptr; prm.fr_c_out = nullptr;
  prm.chunk_counters = (int*)(a.ws + p.off_cnt);
  if (p.fresh) {
    prm.fr_partial = (const float*)(a.ws + p.off_apart); prm.fr_sincos = (const float2*)(a.ws + p.off_sincos);
    prm.fr_slot = a.fr_slot; prm.fr_ks = p.fr_ks; prm.fr_stride = p.fr_stride;
    prm.fr_ke_out = (bf16_t*)a.fr_ke_out; prm.fr_c_out = (bf16_t*)a.fr_c_out;
  }

  hipError_t e = hipSuccess;
  if (a.stages & 1) e = launch_qprep_rows(a, p, qe, qt, stream);
  if (e != hipSuccess) return e;
  if (!(a.stages & 2)) return (a.stages & 4) ? launch_merge_up(a, p, stream) : hipSuccess;

  e = hipErrorInvalidValue;
  const int two_r = 2 * d.r;
  const bool sep = a.d_ck > 0;
#define X(DC, NWV, DCW)                                                                                \
  if (d.d_c == DC) {                                                                                   \
    if constexpr (DCW <= 256) {                                                                        \
      if (sep && two_r == 32) {                                                                        \
        if constexpr (DCW != 224) e = launch_attn<NWV, DCW, 32, true>(prm, a.B, stream);               \
      } else if (sep) {                                                                                \
        e = two_r == 16 ? launch_attn<NWV, DCW, 16, true>(prm, a.B, stream)                            \
                        : launch_attn<NWV, DCW, 8, true>(prm, a.B, stream);                            \
      }                                                                                                \
    }                                                                                                  \
    if (!sep) e = two_r == 64 ? launch_attn<NWV, DCW, 64, false>(prm, a.B, stream)                     \
                  : two_r == 32 ? launch_attn<NWV, DCW, 32, false>(prm, a.B, stream)                   \
                  : two_r == 16 ? launch_attn<NWV, DCW, 16, false>(prm, a.B, stream)                   \
                                : launch_attn<NWV, DCW, 8, false>(prm, a.B, stream);                   \
  }
  EKV_ATTN_SHAPES(X)
#undef X
  if (e != hipSuccess) return e;
  return (a.stages & 4) ? launch_merge_up(a, p, stream) : hipSuccess;
}

}  // namespace ekv
