// Attention of MANY queries per sequence over the EliteKV cache (a prefill, a long prompt chunk):
// bf16 on the gfx950 matrix cores, fp32 accumulation.
//
// With one query the cheapest order of the multiplications absorbs B^k into the query and applies
// B^v after the attention sum (Section 5), at 4 d_c flops per (query, cached token, head).  With T
// queries it is cheaper to undo the low-rank compression ONCE per cached token and let every query
// use the result: keys  k_j,h = [ke_j,h (stored rotated, Section 3.1) | c_j B^k_J,h]  and values
// v_j,h = c_j B^v_J,h  (Section 3.2, J-LRD), 2 d_c (2 d_h - 2r) flops per (token, head), then
// ordinary attention (Section 2.1) at 4 d_h flops per (query, token, head).  Three steps:
//
//   1. the matrix-core GEMM of the cache append (launch_append_gemm) run on the latent rows:
//                          KV[j, :] = c_j [B^k_J | B^v_J]   (no elite columns, no rotation)
//   2. prefill_attn_kernel flash attention: S^T = K Q^T, online softmax, O^T += V^T P^T, with the
//                          query packed on the way in: q^ = [R(pos theta_i) q_i for i in I_h (slot
//                          order) | q's non-elite dims, ascending], scaled by log2(e)/sqrt(d_h)
//                          (Section 3.1 score equation)
//
// Step 2, one work-group = 4 waves x 32 or 64 queries of one (sequence, head); a 64-key tile of K and V
// comes in by direct global->LDS loads, double-buffered.  Per wave and tile:
//   S^T[key, query]   32x32x16 MFMA, A = key rows from LDS (16-byte reads), B = the wave's queries,
//                     held in registers for the whole pass;
//   softmax           a lane owns ONE query (the MFMA output column) and 16 keys per 32-key block,
//                     its partner lane (l ^ 32) the other 16: the row maximum is an in-lane
//                     reduction plus one shuffle;
//   O^T[dim, query]   32x32x16 MFMA, B = the probabilities straight from the score registers (the
//                     keys of a k-step are taken in the order the score tile leaves them in a lane),
//                     A = V read transposed from LDS (ds_read_b64_tr_b16) in that same key order.
// Query blocks are handed out in pairs (i, last - i): under a causal mask every work-group then
// has the same number of key tiles.  Work-groups of one (sequence, head) share an XCD, so the
// tiles the later query blocks re-read come from that XCD's L2.
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

typedef __attribute__((ext_vector_type(8))) __bf16 pf_bf16x8;
typedef __attribute__((ext_vector_type(16))) float pf_f32x16;
typedef __attribute__((ext_vector_type(4))) short pf_s16x4;
typedef __attribute__((ext_vector_type(8))) short pf_s16x8;
typedef __attribute__((address_space(3))) pf_s16x4 pf_lds_s16x4_t;

constexpr int kPfDh = 128;                       // head dim of the compiled kernel
constexpr int kPfTile = 64;                      // keys per tile
constexpr int kPfRow = kPfDh * 2;                // bytes of a staged K or V row
constexpr int kPfPlane = kPfTile * kPfRow;       // one K (or V) tile: 16 KiB
constexpr int kPfStage = 2 * kPfPlane;           // K + V
constexpr int kPfLds = 2 * kPfStage + 64 + 256;  // two stages + the block's reduction scratch + the head's chunk order

struct PrefillParams {
  const bf16_t* q;           // [B * T, n_h, d_h]  queries as the caller holds them (un-rotated)
  const int32_t* q_pos;      // [B * T]
  const int32_t* elite_idx;  // [n_h, r]
  const bf16_t* ke_plane;    // [plane_rows, n_h, 2r]
  const bf16_t* kv;          // [B, S, NKV]  rebuilt [non-elite key dims of every head | values of every head]
  const int32_t* kv_len;     // [B * T] rows of its sequence each query attends to
  bf16_t* out;               // [B * T, n_h, d_h]
  int n_h, T, B;
  int nqb;                   // query blocks per sequence
  int npair;                 // work-groups per (sequence, head): pairs of query blocks, or single blocks
  int paired;                // 1: a work-group takes the blocks (last - i, i) one after the other; 0: block last - i only
  float scale;               // log2(e) / sqrt(d_h)
  int64_t S;                 // rows per sequence in kv
  int64_t NKV, NK;           // row width of kv; first value column
  int64_t batch_stride_rows, plane_rows, max_seq_len;
  RopeTable rope;
};

// staged rows are 16 chunks of 16 bytes; chunk c of row `row` sits at chunk c ^ pf_swz(row): 16 rows read at
// one logical chunk cover all 64 banks, and the 4 rows x 32 bytes of a transposed read cover 4 different
// 64-byte windows
__device__ __forceinline__ int pf_swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

__device__ __forceinline__ void pf_dma16(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory", "m0");
}

__device__ __forceinline__ uint32_t pf_pack2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// log2-domain slack before a query's running maximum is raised: probabilities stay below 2^8
constexpr float kPfSlack = 8.f;

// QB = 32-query blocks per wave: a work-group handles 4 * 32 * QB queries.  QB = 1 is what is launched:
// two work-groups share a compute unit, so a SIMD has one wave's softmax arithmetic to run beside the
// other wave's MFMAs.  (QB = 2: every K and V fragment read from LDS would feed two MFMAs, at one wave per SIMD.)
template <int TWO_R, int QB>
__global__ __launch_bounds__(256, QB == 1 ? 2 : 1) void prefill_attn_kernel(const PrefillParams p) {
  constexpr int KCH = TWO_R / 8;                 // leading 16-byte chunks of a key row that come from the elite plane
  constexpr int R = TWO_R / 2;
  constexpr int QBLK = 128 * QB;                 // queries per work-group pass
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int* red = reinterpret_cast<int*>(smem + 2 * kPfStage);
  int* order = red + 16;                         // order[pp]: the chunk of q that is pair pp of the packed query
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n32 = lane & 31, g = lane >> 5, i16 = lane & 15, q16 = lane >> 4;

  // work-groups go to the eight XCDs round-robin by linear index: all query blocks of one
  // (sequence, head) get indices that are equal modulo 8
  const int xcd = blockIdx.x & 7, seqi = blockIdx.x >> 3;
  const int ph = (seqi / p.npair) * 8 + xcd;
  if (ph >= p.B * p.n_h) return;
  const int pr = seqi % p.npair;
  const int b = ph / p.n_h, h = ph % p.n_h;
  const int64_t row0 = (int64_t)b * p.batch_stride_rows;
  const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem);

  // ---- the packed query's dim order (Section 3.1 score equation): the head's elite chunks in slot
  // order, then the other chunks ascending -- the order of a rebuilt key row [ke | c B^k]
  if (wave == 0) {
    int slot = -1;
    for (int j = 0; j < R; ++j)
      if (p.elite_idx[h * R + j] == lane) slot = j;
    const unsigned long long elite = __ballot(slot >= 0);
    const int rank = __popcll(~elite & ((1ull << lane) - 1ull));   // non-elite chunks below this one
    const int pp = slot >= 0 ? slot : R + rank;
    order[lane] = 0;                                               // (repeated elite indices leave holes: keep them in range)
    if (pp < kPfDh / 2) order[pp] = lane;
  }

  // ---- loader: wave w fills rows 16w .. 16w+15 of the K tile and of the V tile, four rows per load;
  // lane l fills (row l/16, chunk position l%16) and fetches the logical chunk the swizzle puts there
  const int ld_r = lane >> 4;
  const char* kv_seq = reinterpret_cast<const char*>(p.kv) + (int64_t)b * p.S * p.NKV * 2;
  const char* ke_seq = reinterpret_cast<const char*>(p.ke_plane) + (row0 * p.n_h + h) * (int64_t)(TWO_R * 2);

  // ---- LDS read offsets
  // keys as the A operand of S^T: row kb*32 + n32, logical chunk 2*ks + g
  const int k_row_off = n32 * kPfRow;
  const int k_swz = pf_swz(n32);                 // the same for row n32 + 32
  // values, transposed: for a k-step (kb, s2) the lane's 16-lane group supplies keys
  // kb*32 + 16*s2 + 4*g + i16/4 (+ 8 for the upper half) and dims 32*dt + 16*(q16%2) + 4*(i16%4) ..
  const int v_r = 4 * g + (i16 >> 2);
  const int v_ch = ((q16 & 1) << 1) | ((i16 & 3) >> 1);
  const int v_lo_swz = ((i16 >> 2) << 2) | g;
  const int v_hi_swz = ((i16 >> 2) << 2) | ((g + 2) & 3);
  const int v_byte = (i16 & 1) << 3;

  for (int half = 0; half < 2; ++half) {
    const int qblk = half == 0 ? p.nqb - 1 - pr : pr;
    if (half == 1 && (!p.paired || qblk == p.nqb - 1 - pr)) break;   // single blocks; the middle block of an odd count
    int len[QB];
    int64_t qrow[QB];
    bool q_ok[QB];
    int wmax = 0;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const int tq = qblk * QBLK + (wave * QB + qb) * 32 + n32;   // this lane's query of block qb
      q_ok[qb] = tq < p.T;
      qrow[qb] = (int64_t)b * p.T + (q_ok[qb] ? tq : p.T - 1);
      int64_t len64 = q_ok[qb] ? (int64_t)p.kv_len[qrow[qb]] : 0;
      len64 = min(len64, p.max_seq_len);
      len64 = min(len64, p.plane_rows - row0);
      len64 = min(len64, p.S);
      len[qb] = (int)max(len64, (int64_t)0);
      wmax = max(wmax, len[qb]);
    }
    // the block's largest visible length bounds the key loop
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) wmax = max(wmax, __shfl_xor(wmax, o, kWave));
    __syncthreads();                                          // the previous block is done with red[] and the tiles
    if (lane == 0) red[wave] = wmax;
    __syncthreads();                                          // (also: order[] is complete)
    const int kv_hi = max(max(red[0], red[1]), max(red[2], red[3]));
    const int ntiles = (kv_hi + kPfTile - 1) / kPfTile;

    // the loads of a tile in four parts (u = 0..3: four rows of K and of V per wave each); a tile index past the
    // last one stands for the last one (such copies are never read)
    auto issue_part = [&](int tile, int buf, int u) {
      const uint32_t kl = __builtin_amdgcn_readfirstlane(lds0 + buf * kPfStage + wave * 4096);
      tile = min(tile, ntiles - 1);
      {
        const int row = wave * 16 + u * 4 + ld_r;
        const int lc = (lane & 15) ^ pf_swz(row);
        const int64_t t = min(tile * kPfTile + row, kv_hi - 1);   // rows past the end repeat the last visible one
        const char* krow = kv_seq + t * p.NKV * 2 + ((int64_t)h * (kPfDh - TWO_R) + (lc - KCH) * 8) * 2;
        const char* erow = ke_seq + t * (int64_t)p.n_h * (TWO_R * 2) + lc * 16;
        pf_dma16((KCH > 0 && lc < KCH) ? erow : krow, kl + u * 1024);
        const char* vrow = kv_seq + t * p.NKV * 2 + (p.NK + (int64_t)h * kPfDh + lc * 8) * 2;
        pf_dma16(vrow, kl + kPfPlane + u * 1024);
      }
    };
    auto issue = [&](int tile, int buf) {
#pragma unroll
      for (int u = 0; u < 4; ++u) issue_part(tile, buf, u);
    };
    if (ntiles > 0) issue(0, 0);                              // in flight while the queries are prepared

    // the wave's queries as the B operand: lane = query n32, packed dims 16*ks + 8*g .. of block qb,
    // gathered pair by pair from q in the packed order; elite pairs (the first R) rotated to the
    // query's position (Section 2.2, eq. 1a); everything scaled by log2(e)/sqrt(d_h)
    pf_bf16x8 Qb[QB][kPfDh / 16];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const bf16_t* qsrc = p.q + (qrow[qb] * p.n_h + h) * kPfDh;
      const int32_t qp = p.q_pos[qrow[qb]];
#pragma unroll
      for (int ks = 0; ks < kPfDh / 16; ++ks) {
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int pp = 8 * ks + 4 * g + j;
          const int ch = order[pp];
          const uint32_t raw = *reinterpret_cast<const uint32_t*>(qsrc + 2 * ch);
          float a = bf16_bits_to_f32(raw & 0xffffu), c = bf16_bits_to_f32(raw >> 16);
          if (8 * ks < R) {                                   // k-steps that can hold elite pairs (compile-time)
            if (pp < R) {
              float sn, cs;
              rope_sincos_poly(qp, p.rope.theta[ch], &sn, &cs);
              const float a2 = a * cs - c * sn, c2 = a * sn + c * cs;
              a = a2; c = c2;
            }
          }
          w[j] = pf_pack2(a * p.scale, c * p.scale);
        }
        Qb[qb][ks] = __builtin_bit_cast(pf_bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
      }
    }

    pf_f32x16 oacc[QB][kPfDh / 32];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
      for (int dt = 0; dt < kPfDh / 32; ++dt) oacc[qb][dt] = (pf_f32x16)(0.f);
      m_run[qb] = -INFINITY;
      l_run[qb] = 0.f;
    }

    for (int it = 0; it < ntiles; ++it) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // this wave's part of tile `it` has landed
      __syncthreads();                                        // ... everyone's; and tile it-1 has been read by all
      const char* Kt = smem + (it & 1) * kPfStage;
      const char* Vt = Kt + kPfPlane;
      const int key0 = it * kPfTile;

      // ---- scores: two 32-key blocks per query block.  All key fragments of the tile are requested
      // before the first MFMA (the compiler would otherwise read each one right before its use and
      // expose the LDS latency sixteen times); sched_barrier keeps the requests where they are.
      pf_bf16x8 kf[kPfDh / 16][2];
#pragma unroll
      for (int ks = 0; ks < kPfDh / 16; ++ks) {
        const int off = k_row_off + (((2 * ks + g) ^ k_swz) << 4);
        kf[ks][0] = *reinterpret_cast<const pf_bf16x8*>(Kt + off);
        kf[ks][1] = *reinterpret_cast<const pf_bf16x8*>(Kt + off + 32 * kPfRow);
      }
      __builtin_amdgcn_sched_barrier(0);
      pf_f32x16 sacc[QB][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) { sacc[qb][0] = (pf_f32x16)(0.f); sacc[qb][1] = (pf_f32x16)(0.f); }
      // The next tile's loads are requested BEHIND the first score MFMAs: vector work (here the address
      // arithmetic) overlaps MFMAs of the same wave that were issued before it, not those of the other wave.
#pragma unroll
      for (int ks = 0; ks < kPfDh / 16; ++ks) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
          sacc[qb][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks][0], Qb[qb][ks], sacc[qb][0], 0, 0, 0);
          sacc[qb][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks][1], Qb[qb][ks], sacc[qb][1], 0, 0, 0);
        }
        if (ks < 4) {
          asm volatile("" : "+v"(sacc[0][1]));                // (keeps the MFMAs above the requests below)
          issue_part(it + 1, (it + 1) & 1, ks);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // ---- value fragments of the first 32 keys, requested ahead of the softmax arithmetic.
      // k-slot (g, j) of k-step (kb, s2) is key kb*32 + 16*s2 + 8*(j/4) + 4*g + j%4
      pf_bf16x8 vf[2][2][kPfDh / 32];
      auto read_v = [&](int kb) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const char* vlo = Vt + (kb * 32 + 16 * s2 + v_r) * kPfRow + v_byte;
#pragma unroll
          for (int dt = 0; dt < kPfDh / 32; ++dt) {
            const int ch = 4 * dt + v_ch;
            const pf_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pf_lds_s16x4_t*)(vlo + ((ch ^ v_lo_swz) << 4)));
            const pf_s16x4 hi =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((pf_lds_s16x4_t*)(vlo + 8 * kPfRow + ((ch ^ v_hi_swz) << 4)));
            vf[kb][s2][dt] = __builtin_bit_cast(pf_bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          }
        }
      };
      read_v(0);
      __builtin_amdgcn_sched_barrier(0);
      pf_bf16x8 Pb[QB][2][2];
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        // register v of block kb is key key0 + kb*32 + 8*(v/4) + 4*g + v%4 for this lane's query
        if (__any(key0 + kPfTile > len[qb])) {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = key0 + kb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
              sacc[qb][kb][v] = key < len[qb] ? sacc[qb][kb][v] : -INFINITY;
            }
        }
        // ---- online softmax (log2 domain: the packed query carries log2(e)/sqrt(d_h))
        float t0 = fmaxf(sacc[qb][0][0], sacc[qb][1][0]);
#pragma unroll
        for (int v = 1; v < 16; ++v) t0 = fmaxf(t0, fmaxf(sacc[qb][0][v], sacc[qb][1][v]));
        const float tmax = fmaxf(t0, __shfl_xor(t0, 32, kWave));
        // the reference maximum is raised only when a score exceeds it by more than the slack
        const float m_new = (tmax > m_run[qb] + kPfSlack || m_run[qb] == -INFINITY) ? tmax : m_run[qb];
        const float m_use = m_new == -INFINITY ? 0.f : m_new;  // nothing visible yet: every exponential below is 0
        const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_use);
        m_run[qb] = m_new;
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const float pv = __builtin_amdgcn_exp2f(sacc[qb][kb][8 * s2 + j] - m_use);
              psum += pv;
              Pb[qb][kb][s2][j] = (__bf16)pv;
            }
        l_run[qb] = l_run[qb] * alpha + psum;
        if (__any(alpha != 1.f)) {
#pragma unroll
          for (int dt = 0; dt < kPfDh / 32; ++dt) oacc[qb][dt] *= alpha;
        }
      }
      // ---- values: the fragments of the second 32 keys are requested before the first MFMAs
      read_v(1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int dt = 0; dt < kPfDh / 32; ++dt)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
              oacc[qb][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[kb][s2][dt], Pb[qb][kb][s2], oacc[qb][dt], 0, 0, 0);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the spare copy of the last tile has landed before the stages are reused

    // ---- normalise and store: register 4*j + i of tile dt is dim 32*dt + 8*j + 4*g + i of the lane's query
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, kWave);
      const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;     // a query that sees nothing gets a zero row
      if (q_ok[qb]) {
        bf16_t* orow = p.out + (qrow[qb] * p.n_h + h) * kPfDh + 4 * g;
#pragma unroll
        for (int dt = 0; dt < kPfDh / 32; ++dt)
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            uint2 pk;
            pk.x = pf_pack2(oacc[qb][dt][4 * j] * inv, oacc[qb][dt][4 * j + 1] * inv);
            pk.y = pf_pack2(oacc[qb][dt][4 * j + 2] * inv, oacc[qb][dt][4 * j + 3] * inv);
            *reinterpret_cast<uint2*>(orow + 32 * dt + 8 * j) = pk;
          }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
static elitekv_dims rebuild_dims(const elitekv_dims& d) {
  elitekv_dims g = d;
  g.d_model = d.d_c;                                         // contraction over the latent
  g.r = 0;                                                   // no elite columns, nothing is rotated
  g.d_c = d.n_heads * (2 * d.head_dim - 2 * d.r);            // [non-elite key dims | values] of every head
  return g;
}

// Below this many queries per sequence the absorbed form (every query through the decode kernels) is the
// cheaper order: rebuilding a row costs 2 d_c (2 d_h - 2r) flops per head, about what 60-70 absorbed queries
// cost on it at their measured rates.
constexpr int kPfMinQueries = 48;

bool prefill_flash_supported(const elitekv_dims& d, int d_ck, int64_t T, int64_t max_seq_len) {
  if (d.dtype != ELITEKV_BF16 || d.head_dim != kPfDh) return false;
  // separated latents: keys are rebuilt from the first d_ck columns of a latent row and values from the rest,
  // each slice in whole contraction stages, and no 128-column block of the rebuilt row lies across the two
  if (d_ck < 0 || d_ck >= d.d_c || d_ck % 32) return false;
  if (d_ck > 0 && (d.n_heads * (d.head_dim - 2 * d.r)) % 128) return false;
  if (T < kPfMinQueries) return false;
  if (2 * d.r != 8 && 2 * d.r != 16) return false;
  if (d.d_c % 32 || T < 1 || max_seq_len <= 64 || max_seq_len > (1 << 30)) return false;
  const elitekv_dims g = rebuild_dims(d);
  return append_gemm_supported(g, max_seq_len, d.n_heads * (d.head_dim - 2 * d.r));
}

static size_t pf_align(size_t v) { return (v + 255) / 256 * 256; }

// workspace: the rebuilt K/V rows of all sequences
size_t prefill_flash_workspace(const elitekv_dims& d, int64_t B, int64_t T, int64_t max_seq_len) {
  (void)T;
  return pf_align((size_t)B * (size_t)max_seq_len * (size_t)rebuild_dims(d).d_c * 2);
}

template <int TWO_R, int QB>
static hipError_t launch_pf(PrefillParams& p, int64_t B, int64_t T, hipStream_t stream) {
  p.nqb = (int)((T + 128 * QB - 1) / (128 * QB));
  const int64_t pairs = (B * p.n_h + 7) / 8 * 8;             // (sequence, head) pairs, padded to whole rounds of the XCDs
  // Pairs of blocks give every work-group the same number of key tiles, but a work-group runs its two blocks one
  // after the other.  When single blocks still make at most one work-group per compute unit (a prompt of up to 1024
  // tokens of one 32-head sequence), the pairs would leave half of the compute units idle: then every block gets a
  // work-group of its own, heaviest first (0.085 -> 0.073 ms at 1024 tokens, 7B 25 %).  With more blocks than compute
  // units the pairs are faster (2048 tokens: 0.138 against 0.153 ms with single blocks, whose heaviest two share a
  // compute unit and set the launch's length).
  p.paired = pairs * p.nqb > 256 ? 1 : 0;
  p.npair = p.paired ? (p.nqb + 1) / 2 : p.nqb;
  static LdsLimit lim;
  const hipError_t e = raise_lds_limit(lim, reinterpret_cast<const void*>(&prefill_attn_kernel<TWO_R, QB>), kPfLds);
  if (e != hipSuccess) return e;
  prefill_attn_kernel<TWO_R, QB><<<(unsigned)(pairs * p.npair), 256, kPfLds, stream>>>(p);
  return hipGetLastError();
}

hipError_t launch_prefill_flash(const DecodeArgs& a, int64_t B, int64_t T, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int64_t S = a.max_seq_len;
  const elitekv_dims gd = rebuild_dims(d);
  const int64_t NK = (int64_t)d.n_heads * (d.head_dim - 2 * d.r), NKV = gd.d_c;
  bf16_t* kv = reinterpret_cast<bf16_t*>(a.ws);

  // K/V of every sequence's first S rows (rows past the end of the planes are left out)
  // Sequences that lie back to back in the planes (stride == max_seq_len) are one GEMM over all their rows;
  // otherwise one launch per sequence.
  const bool packed = a.batch_stride_rows == S && B > 1;
  hipError_t e = hipSuccess;
  for (int64_t b = 0; b < (packed ? 1 : B); ++b) {
    const int64_t row0 = b * a.batch_stride_rows;
    const int64_t want = packed ? B * S : S;
    const int64_t rows = want < a.plane_rows - row0 ? want : a.plane_rows - row0;
    if (rows <= 0) continue;
    AppendArgs g;
    g.dims = gd; g.d_ck = (int32_t)NK; g.W_dkv = a.W_uk; g.W_dkv2 = a.W_uv; g.W_ke = nullptr;
    if (a.d_ck > 0) {                                          // [c^k | c^v] rows: keys from c^k, values from c^v
      g.dims.d_model = a.d_ck; g.x_ld = d.d_c; g.x_off2 = a.d_ck; g.d2 = d.d_c - a.d_ck;
    }
    g.x = (const bf16_t*)a.c_plane + row0 * d.d_c; g.pos = nullptr; g.slot = nullptr; g.T = rows;   // rows written in place
    g.elite_idx = nullptr; g.ke_plane = nullptr; g.c_plane = kv + b * S * NKV; g.plane_rows = want; g.ws = nullptr;
    e = launch_append_gemm(g, stream);
    if (e != hipSuccess) return e;
  }

  PrefillParams p;
  p.q = (const bf16_t*)a.q; p.q_pos = a.q_pos; p.elite_idx = a.elite_idx;
  p.ke_plane = (const bf16_t*)a.ke_plane; p.kv = kv; p.kv_len = a.seq_len; p.out = (bf16_t*)a.out;
  p.n_h = d.n_heads; p.T = (int)T; p.B = (int)B;
  p.scale = kLog2e / sqrtf((float)d.head_dim);
  p.S = S; p.NKV = NKV; p.NK = NK;
  p.batch_stride_rows = a.batch_stride_rows; p.plane_rows = a.plane_rows; p.max_seq_len = a.max_seq_len;
  p.rope = rope_table(d.rope_base, d.head_dim);
  // one 32-query block per wave: with two (every LDS fragment feeding two MFMAs, one wave per SIMD) the
  // compiler does not interleave one block's softmax with the other's MFMAs, and it measured 20 % slower
  return 2 * d.r == 16 ? launch_pf<16, 1>(p, B, T, stream) : launch_pf<8, 1>(p, B, T, stream);
}

}  // namespace ekv
