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
//   1. pack_query_kernel   q^ = [R(pos theta_i) q_i for i in I_h (slot order) | q's non-elite dims,
//                          ascending], scaled by log2(e)/sqrt(d_h), bf16          (Section 3.1 score equation)
//   2. the matrix-core GEMM of the cache append (launch_append_gemm) run on the latent rows:
//                          KV[j, :] = c_j [B^k_J | B^v_J]   (no elite columns, no rotation)
//   3. prefill_attn_kernel flash attention: S^T = K Q^T, online softmax, O^T += V^T P^T.
//
// Step 3, one work-group = 4 waves x 32 queries of one (sequence, head); a 64-key tile of K and V
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
constexpr int kPfQB = 128;                       // queries per block (4 waves x 32)
constexpr int kPfTile = 64;                      // keys per tile
constexpr int kPfRow = kPfDh * 2;                // bytes of a staged K or V row
constexpr int kPfPlane = kPfTile * kPfRow;       // one K (or V) tile: 16 KiB
constexpr int kPfStage = 2 * kPfPlane;           // K + V
constexpr int kPfLds = 2 * kPfStage + 64;        // two stages + the block's reduction scratch

struct PrefillParams {
  const bf16_t* qp;          // [B * T, n_h, d_h]  packed queries
  const bf16_t* ke_plane;    // [plane_rows, n_h, 2r]
  const bf16_t* kv;          // [B, S, NKV]  rebuilt [non-elite key dims of every head | values of every head]
  const int32_t* kv_len;     // [B * T] rows of its sequence each query attends to
  bf16_t* out;               // [B * T, n_h, d_h]
  int n_h, T, B;
  int nqb;                   // query blocks per sequence
  int npair;                 // work-groups per (sequence, head): pairs of query blocks
  int64_t S;                 // rows per sequence in kv
  int64_t NKV, NK;           // row width of kv; first value column
  int64_t batch_stride_rows, plane_rows, max_seq_len;
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

template <int TWO_R>
__global__ __launch_bounds__(256, 2) void prefill_attn_kernel(const PrefillParams p) {
  constexpr int KCH = TWO_R / 8;                 // leading 16-byte chunks of a key row that come from the elite plane
  extern __shared__ __attribute__((aligned(16))) char smem[];
  int* red = reinterpret_cast<int*>(smem + 2 * kPfStage);
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
    if (half == 1 && qblk == p.nqb - 1 - pr) break;          // the middle block of an odd count
    const int tq = qblk * kPfQB + wave * 32 + n32;            // this lane's query
    const bool q_ok = tq < p.T;
    const int64_t qrow = (int64_t)b * p.T + (q_ok ? tq : p.T - 1);
    int64_t len64 = q_ok ? (int64_t)p.kv_len[qrow] : 0;
    len64 = min(len64, p.max_seq_len);
    len64 = min(len64, p.plane_rows - row0);
    len64 = min(len64, p.S);
    const int len = (int)max(len64, (int64_t)0);
    // the block's largest visible length bounds the key loop
    int wmax = len;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) wmax = max(wmax, __shfl_xor(wmax, o, kWave));
    __syncthreads();                                          // the previous block is done with red[] and the tiles
    if (lane == 0) red[wave] = wmax;
    __syncthreads();
    const int kv_hi = max(max(red[0], red[1]), max(red[2], red[3]));
    const int ntiles = (kv_hi + kPfTile - 1) / kPfTile;

    // the wave's queries as the B operand: lane = query n32, dims 16*ks + 8*g ..
    pf_bf16x8 Qb[kPfDh / 16];
    {
      const bf16_t* qsrc = p.qp + (qrow * p.n_h + h) * kPfDh + 8 * g;
#pragma unroll
      for (int ks = 0; ks < kPfDh / 16; ++ks)
        Qb[ks] = __builtin_bit_cast(pf_bf16x8, *reinterpret_cast<const pf_s16x8*>(qsrc + 16 * ks));
    }

    auto issue = [&](int tile, int buf) {
      const uint32_t kl = __builtin_amdgcn_readfirstlane(lds0 + buf * kPfStage + wave * 4096);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
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

    pf_f32x16 oacc[kPfDh / 32];
#pragma unroll
    for (int dt = 0; dt < kPfDh / 32; ++dt) oacc[dt] = (pf_f32x16)(0.f);
    float m_run = -INFINITY, l_run = 0.f;

    if (ntiles > 0) issue(0, 0);
    for (int it = 0; it < ntiles; ++it) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // this wave's part of tile `it` has landed
      __syncthreads();                                        // ... everyone's; and tile it-1 has been read by all
      if (it + 1 < ntiles) issue(it + 1, (it + 1) & 1);
      const char* Kt = smem + (it & 1) * kPfStage;
      const char* Vt = Kt + kPfPlane;
      const int key0 = it * kPfTile;

      // ---- scores: two 32-key blocks
      pf_f32x16 sacc[2] = {(pf_f32x16)(0.f), (pf_f32x16)(0.f)};
#pragma unroll
      for (int ks = 0; ks < kPfDh / 16; ++ks) {
        const int off = k_row_off + (((2 * ks + g) ^ k_swz) << 4);
        const pf_bf16x8 a0 = *reinterpret_cast<const pf_bf16x8*>(Kt + off);
        const pf_bf16x8 a1 = *reinterpret_cast<const pf_bf16x8*>(Kt + off + 32 * kPfRow);
        sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, Qb[ks], sacc[0], 0, 0, 0);
        sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, Qb[ks], sacc[1], 0, 0, 0);
      }
      // register v of block kb is key key0 + kb*32 + 8*(v/4) + 4*g + v%4 for this lane's query
      if (__any(key0 + kPfTile > len)) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int key = key0 + kb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
            sacc[kb][v] = key < len ? sacc[kb][v] : -INFINITY;
          }
      }
      // ---- online softmax (log2 domain: the packed query carries log2(e)/sqrt(d_h))
      float tmax = -INFINITY;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int v = 0; v < 16; ++v) tmax = fmaxf(tmax, sacc[kb][v]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
      const float m_new = fmaxf(m_run, tmax);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;  // nothing visible yet: every exponential below is 0
      const float alpha = exp2f(m_run - m_use);
      m_run = m_new;
      float psum = 0.f;
      pf_bf16x8 Pb[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const float pv = exp2f(sacc[kb][8 * s2 + j] - m_use);
            psum += pv;
            Pb[kb][s2][j] = (__bf16)pv;
          }
      l_run = l_run * alpha + psum;
      if (__any(alpha != 1.f)) {
#pragma unroll
        for (int dt = 0; dt < kPfDh / 32; ++dt) oacc[dt] *= alpha;
      }
      // ---- values: k-slot (g, j) of k-step (kb, s2) is key kb*32 + 16*s2 + 8*(j/4) + 4*g + j%4
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const char* vlo = Vt + (kb * 32 + 16 * s2 + v_r) * kPfRow + v_byte;
#pragma unroll
          for (int dt = 0; dt < kPfDh / 32; ++dt) {
            const int ch = 4 * dt + v_ch;
            const pf_s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((pf_lds_s16x4_t*)(vlo + ((ch ^ v_lo_swz) << 4)));
            const pf_s16x4 hi =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((pf_lds_s16x4_t*)(vlo + 8 * kPfRow + ((ch ^ v_hi_swz) << 4)));
            const pf_s16x8 a16 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(pf_bf16x8, a16), Pb[kb][s2], oacc[dt], 0, 0, 0);
          }
        }
    }

    // ---- normalise and store: register 4*j + i of tile dt is dim 32*dt + 8*j + 4*g + i of the lane's query
    const float l_tot = l_run + __shfl_xor(l_run, 32, kWave);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;       // a query that sees nothing gets a zero row
    if (q_ok) {
      bf16_t* orow = p.out + (qrow * p.n_h + h) * kPfDh + 4 * g;
#pragma unroll
      for (int dt = 0; dt < kPfDh / 32; ++dt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint2 pk;
          pk.x = pf_pack2(oacc[dt][4 * j] * inv, oacc[dt][4 * j + 1] * inv);
          pk.y = pf_pack2(oacc[dt][4 * j + 2] * inv, oacc[dt][4 * j + 3] * inv);
          *reinterpret_cast<uint2*>(orow + 32 * dt + 8 * j) = pk;
        }
    }
  }
}

// One wave per (query row, head): lane l owns chunk l of the head (dims 2l, 2l+1).
__global__ __launch_bounds__(256) void pack_query_kernel(const bf16_t* __restrict__ q, const int32_t* __restrict__ q_pos,
                                                         const int32_t* __restrict__ elite_idx, bf16_t* __restrict__ qp,
                                                         int64_t rows, int n_h, int d_h, int r, RopeTable rope, float scale) {
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (item >= rows * n_h) return;                            // uniform over the wave
  const int64_t row = item / n_h;
  const int h = (int)(item % n_h);
  const bool live = lane < d_h / 2;
  int slot = -1;
  for (int j = 0; j < r; ++j)
    if (elite_idx[h * r + j] == lane) slot = j;
  const unsigned long long elite = __ballot(slot >= 0);
  const int rank = __popcll(~elite & ((1ull << lane) - 1ull));   // non-elite chunks below this one
  if (!live) return;
  const uint32_t w = *reinterpret_cast<const uint32_t*>(q + item * d_h + 2 * lane);
  float a = bf16_bits_to_f32(w & 0xffffu), c = bf16_bits_to_f32(w >> 16);
  int dst;
  if (slot >= 0) {
    float sn, cs;
    rope_sincos(q_pos[row], rope.theta[lane], &sn, &cs);
    const float a2 = a * cs - c * sn, c2 = a * sn + c * cs;
    a = a2; c = c2;
    dst = 2 * slot;
  } else {
    dst = 2 * r + 2 * rank;
  }
  if (dst + 1 < d_h) *reinterpret_cast<uint32_t*>(qp + item * d_h + dst) = pf_pack2(a * scale, c * scale);
}

// rows of the rebuilt K/V buffer are written in place: slot[t] = t; the GEMM's epilogue also reads a
// position per row, which nothing uses without elite columns
__global__ void prefill_rows_kernel(int64_t* slot, int32_t* pos, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) { slot[i] = i; pos[i] = 0; }
}

// ---------------------------------------------------------------------------------------------
static elitekv_dims rebuild_dims(const elitekv_dims& d) {
  elitekv_dims g = d;
  g.d_model = d.d_c;                                         // contraction over the latent
  g.r = 0;                                                   // no elite columns, nothing is rotated
  g.d_c = d.n_heads * (2 * d.head_dim - 2 * d.r);            // [non-elite key dims | values] of every head
  return g;
}

bool prefill_flash_supported(const elitekv_dims& d, int64_t T, int64_t max_seq_len) {
  if (d.dtype != ELITEKV_BF16 || d.head_dim != kPfDh) return false;
  if (2 * d.r != 8 && 2 * d.r != 16) return false;
  if (d.d_c % 32 || T < 1 || max_seq_len <= 64 || max_seq_len > (1 << 30)) return false;
  const elitekv_dims g = rebuild_dims(d);
  return append_gemm_supported(g, max_seq_len, d.n_heads * (d.head_dim - 2 * d.r));
}

static size_t pf_align(size_t v) { return (v + 255) / 256 * 256; }

// workspace: [slot int64 S][pos int32 S][packed queries][rebuilt K/V of all sequences]
size_t prefill_flash_workspace(const elitekv_dims& d, int64_t B, int64_t T, int64_t max_seq_len) {
  const size_t S = (size_t)max_seq_len;
  return pf_align(S * 8) + pf_align(S * 4) + pf_align((size_t)B * T * d.n_heads * d.head_dim * 2) +
         pf_align((size_t)B * S * (size_t)rebuild_dims(d).d_c * 2);
}

hipError_t launch_prefill_flash(const DecodeArgs& a, int64_t B, int64_t T, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int64_t S = a.max_seq_len;
  const elitekv_dims gd = rebuild_dims(d);
  const int64_t NK = (int64_t)d.n_heads * (d.head_dim - 2 * d.r), NKV = gd.d_c;
  char* ws = a.ws;
  int64_t* slot = reinterpret_cast<int64_t*>(ws);   ws += pf_align((size_t)S * 8);
  int32_t* pos = reinterpret_cast<int32_t*>(ws);    ws += pf_align((size_t)S * 4);
  bf16_t* qp = reinterpret_cast<bf16_t*>(ws);       ws += pf_align((size_t)B * T * d.n_heads * d.head_dim * 2);
  bf16_t* kv = reinterpret_cast<bf16_t*>(ws);

  prefill_rows_kernel<<<(unsigned)((S + 255) / 256), 256, 0, stream>>>(slot, pos, S);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int64_t items = B * T * d.n_heads;
  pack_query_kernel<<<(unsigned)((items + 3) / 4), 256, 0, stream>>>(
      (const bf16_t*)a.q, a.q_pos, a.elite_idx, qp, B * T, d.n_heads, d.head_dim, d.r,
      rope_table(d.rope_base, d.head_dim), kLog2e / sqrtf((float)d.head_dim));
  e = hipGetLastError();
  if (e != hipSuccess) return e;

  // K/V of every sequence's first S rows (rows past the end of the planes are left out)
  for (int64_t b = 0; b < B; ++b) {
    const int64_t row0 = b * a.batch_stride_rows;
    const int64_t rows = S < a.plane_rows - row0 ? S : a.plane_rows - row0;
    if (rows <= 0) continue;
    AppendArgs g;
    g.dims = gd; g.d_ck = (int32_t)NK; g.W_dkv = a.W_uk; g.W_dkv2 = a.W_uv; g.W_ke = nullptr;
    g.x = (const bf16_t*)a.c_plane + row0 * d.d_c; g.pos = pos; g.slot = slot; g.T = rows;
    g.elite_idx = nullptr; g.ke_plane = nullptr; g.c_plane = kv + b * S * NKV; g.plane_rows = S; g.ws = nullptr;
    e = launch_append_gemm(g, stream);
    if (e != hipSuccess) return e;
  }

  PrefillParams p;
  p.qp = qp; p.ke_plane = (const bf16_t*)a.ke_plane; p.kv = kv; p.kv_len = a.seq_len; p.out = (bf16_t*)a.out;
  p.n_h = d.n_heads; p.T = (int)T; p.B = (int)B;
  p.nqb = (int)((T + kPfQB - 1) / kPfQB);
  p.npair = (p.nqb + 1) / 2;
  p.S = S; p.NKV = NKV; p.NK = NK;
  p.batch_stride_rows = a.batch_stride_rows; p.plane_rows = a.plane_rows; p.max_seq_len = a.max_seq_len;
  const int64_t pairs = (B * d.n_heads + 7) / 8 * 8;         // (sequence, head) pairs, padded to whole rounds of the XCDs
  const int64_t groups = pairs * p.npair;
  static LdsLimit lim8, lim16;
  if (2 * d.r == 16) {
    e = raise_lds_limit(lim16, reinterpret_cast<const void*>(&prefill_attn_kernel<16>), kPfLds);
    if (e != hipSuccess) return e;
    prefill_attn_kernel<16><<<(unsigned)groups, 256, kPfLds, stream>>>(p);
  } else {
    e = raise_lds_limit(lim8, reinterpret_cast<const void*>(&prefill_attn_kernel<8>), kPfLds);
    if (e != hipSuccess) return e;
    prefill_attn_kernel<8><<<(unsigned)groups, 256, kPfLds, stream>>>(p);
  }
  return hipGetLastError();
}

}  // namespace ekv
