// bf16 decode attention over the EliteKV cache on the gfx950 matrix cores.
//
// One work-group handles one (sequence split, group of up to 32 heads, batch row).  All heads of
// the group are one MFMA dimension against the SHARED latent tile (Section 3.2: key and value
// share the latent c), so each cached row is read from HBM exactly once and serves both the key
// role (scores) and the value role (latent accumulation):
//
//   scores   S^T[token, head] = C[token, :] . Qt[head, :]        A = latent tile, B = absorbed query
//            + per-head elite term  ke[token, head, :] . qe[head, :]   (VALU, 2r-wide)
//            (Section 3.1 score equation with W_uk absorbed into the query, Section 5)
//   softmax  online, in the log2 domain (the query is pre-scaled by log2(e)/sqrt(d_h))
//   values   U^T[col, head] += C^T[col, token] . P^T[token, head]   A = the SAME tile read
//            transposed from LDS, B = the probabilities straight from the score registers
//
// The latent dimension is split over the NW waves of the group (DC_W columns each): a wave holds
// its slice of the absorbed query and of U in registers, computes partial scores over its slice,
// and the waves exchange partial scores through LDS once per 32-token tile.  Tiles are brought in
// with direct global->LDS loads (16 bytes per lane), one private LDS slice per wave.
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4_t;

constexpr int kTile = 32;   // cached tokens per tile = the MFMA M dimension

struct AttnMfmaParams {
  const bf16_t* ke_plane;
  const bf16_t* c_plane;
  const float* qe;        // [B, n_h, 2r]   rotated, scaled elite query
  const bf16_t* qt;       // [B, n_h, d_c]  absorbed, scaled latent query
  const int32_t* seq_len;
  float* part_m;          // [B, n_splits, HG*32]        split maxima (log2 domain)
  float* part_l;          // [B, n_splits, HG*32]        split sums
  bf16_t* part_u;         // [B, n_splits, HG*32, d_c]   split latent accumulators, head-major
  int n_h, d_c, n_splits, chunk, head_groups;
  int64_t max_seq_len, batch_stride_rows, plane_rows;
};

// LDS layout of one wave's tile slice (32 tokens x DC_W latent columns, bf16): blocks of
// 8 rows x 128 bytes (1 KiB, exactly what one direct-to-LDS load of 64 lanes x 16 bytes fills),
// block (rb, cb) at ((rb * NCB) + cb) KiB.  Inside a block the 16-byte chunk index is XOR-ed with
// swz(row) = ((row & 3) << 1) | ((row >> 2) & 1): eight rows read at one logical chunk hit eight
// different bank groups (row-wise b128 reads), and the 4 rows x 32 bytes a transposed b64 read
// covers hit four different 32-byte bank groups.
template <int NW, int DC_W>
struct AttnMfmaLayout {
  static_assert(DC_W % 64 == 0, "a wave's latent slice must be a whole number of 128-byte blocks");
  static_assert(16 % NW == 0, "the 16 score registers are divided evenly among the waves");
  static constexpr int KS = DC_W / 16;                      // score k-steps per wave
  static constexpr int CT = DC_W / 32;                      // 32-column accumulator tiles per wave
  static constexpr int NCB = DC_W / 64;                     // 128-byte column blocks per row
  static constexpr int NLOAD = 4 * NCB;                     // direct-to-LDS loads per tile per wave
  static constexpr int WTILE = NLOAD * 1024;                // LDS bytes of one wave's tile slice
  static constexpr int VPW = 16 / NW;                       // score registers each wave finalises
  static constexpr int X1 = NW * 16 * 64 * 4;               // stage-1 exchange: every wave's partials
  static constexpr int X2 = 16 * 64 * 4;                    // stage-2 exchange: the final scores
  static constexpr int LDS_BYTES = NW * WTILE + X1 + X2;
  static_assert(LDS_BYTES <= 160 * 1024, "exceeds the 160 KiB of LDS of a gfx950 compute unit");
};

__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int tile_swz(int row) { return ((row & 3) << 1) | ((row >> 2) & 1); }

// log2-domain slack before the running maximum is raised: probabilities stay below 2^8
constexpr float kRescaleSlack = 8.f;

template <int NW, int DC_W, int TWO_R>
__global__ __launch_bounds__(NW * 64) void attn_mfma_kernel(const AttnMfmaParams p) {
  using L = AttnMfmaLayout<NW, DC_W>;
  constexpr int KS = L::KS, CT = L::CT, NCB = L::NCB, VPW = L::VPW;
  constexpr int KCH = TWO_R / 8;                 // 16-byte chunks of one head's elite key

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, g = lane >> 5;
  const int split = blockIdx.x, hg = blockIdx.y, b = blockIdx.z;
  char* ctile = smem + wave * L::WTILE;
  float* x1 = reinterpret_cast<float*>(smem + NW * L::WTILE);
  float* x2 = reinterpret_cast<float*>(smem + NW * L::WTILE + L::X1);

  const int64_t row0 = (int64_t)b * p.batch_stride_rows;
  int64_t len = p.seq_len[b];
  len = min(len, p.max_seq_len);
  len = min(len, p.plane_rows - row0);
  len = max(len, (int64_t)0);
  const int64_t t0 = (int64_t)split * p.chunk;
  const int64_t t_end = min(t0 + p.chunk, len);
  const int64_t pidx = ((int64_t)b * p.n_splits + split) * (p.head_groups * 32) + hg * 32;

  if (t0 >= t_end) {   // empty split: the merge skips it (l == 0)
    if (wave == 0 && g == 0) {
      p.part_m[pidx + n] = -INFINITY;
      p.part_l[pidx + n] = 0.f;
    }
    return;
  }

  const int head = hg * 32 + n;
  const bool head_ok = head < p.n_h;
  const int head_c = head_ok ? head : p.n_h - 1;

  // this wave's slice of the absorbed query, as the B operand of the score MFMAs
  bf16x8 Qb[KS];
  {
    const bf16_t* qrow = p.qt + ((int64_t)b * p.n_h + head_c) * p.d_c + wave * DC_W + 8 * g;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      s16x8 v = *reinterpret_cast<const s16x8*>(qrow + 16 * ks);
      if (!head_ok) v = (s16x8)(0);
      Qb[ks] = __builtin_bit_cast(bf16x8, v);
    }
  }
  float qe[TWO_R > 0 ? TWO_R : 1];
  if (TWO_R > 0) {
    const float* qer = p.qe + ((int64_t)b * p.n_h + head_c) * TWO_R;
#pragma unroll
    for (int j = 0; j < TWO_R; ++j) qe[j] = head_ok ? qer[j] : 0.f;
  }

  f32x16 uacc[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) uacc[ct] = (f32x16)(0.f);
  float m_run = -INFINITY, l_run = 0.f;

  const int64_t crow_bytes = (int64_t)p.d_c * 2;
  const int64_t krow_bytes = (int64_t)p.n_h * TWO_R * 2;
  // loader: lane l fills slot (row l/8, position l%8) of every block; it fetches the logical
  // chunk that the swizzle puts there
  const int ld_row = lane >> 3;
  const char* cbase = reinterpret_cast<const char*>(p.c_plane) + (int64_t)wave * DC_W * 2 +
                      (((lane & 7) ^ tile_swz(ld_row)) << 4);
  const char* kbase = reinterpret_cast<const char*>(p.ke_plane) + (int64_t)head_c * TWO_R * 2;

  // LDS read addresses that do not change from tile to tile
  // score A operand: row n, logical chunk 2*ks + g  ->  block (n/8, ks/4), in-block chunk 2*(ks%4)+g
  const char* a_row = ctile + (n >> 3) * (NCB * 1024) + (n & 7) * 128;
  const int a_swz = tile_swz(n & 7);
  // value A operand (transposed b64 read): lane (q16, s16) addresses row 8*j + 4*(q16/2) + s16/4,
  // 4 columns at 32*ct + 16*(q16%2) + 4*(s16%4)
  const int q16 = lane >> 4, s16 = lane & 15;
  const int tr_r8 = 4 * (q16 >> 1) + (s16 >> 2);                  // row inside its 8-row block
  const int tr_swz = tile_swz(tr_r8);
  const int tr_lo = ((q16 & 1) << 1) | ((s16 & 3) >> 1);          // chunk inside a 32-column group
  const char* tr_row = ctile + tr_r8 * 128 + ((s16 & 1) << 3);
  const int tr_c0 = (tr_lo ^ tr_swz) << 4;                        // even ct: in-block chunks 0..3
  const int tr_c1 = ((4 | tr_lo) ^ tr_swz) << 4;                  // odd ct: in-block chunks 4..7

  uint4 kreg[VPW][KCH > 0 ? KCH : 1];

  auto issue_tile = [&](int64_t tile_t0) {
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
      const int64_t t = min(tile_t0 + rb * 8 + ld_row, t_end - 1);
      const char* gp = cbase + (row0 + t) * crow_bytes;
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
        __builtin_amdgcn_global_load_lds(gp + cb * 128, (lds_void_t*)(ctile + (rb * NCB + cb) * 1024), 16,
                                         0, 0);
    }
  };
  // the wave finalises score registers v = wave*VPW + e: token 8*(v/4) + 4*g + v%4 of the tile
  auto issue_ke = [&](int64_t tile_t0) {
    if (TWO_R > 0) {
#pragma unroll
      for (int e = 0; e < VPW; ++e) {
        const int v = wave * VPW + e;
        const int64_t t = min(tile_t0 + 8 * (v >> 2) + 4 * g + (v & 3), t_end - 1);
        const uint4* kp = reinterpret_cast<const uint4*>(kbase + (row0 + t) * krow_bytes);
#pragma unroll
        for (int c = 0; c < KCH; ++c) kreg[e][c] = kp[c];
      }
    }
  };

  issue_tile(t0);
  issue_ke(t0);

  for (int64_t tile = t0; tile < t_end; tile += kTile) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // ---- scores over this wave's latent slice (two accumulators break the dependency chain)
    f32x16 sacc0 = (f32x16)(0.f), sacc1 = (f32x16)(0.f);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int inb = ((2 * (ks & 3) + g) ^ a_swz) << 4;
      const bf16x8 a = *reinterpret_cast<const bf16x8*>(a_row + (ks >> 2) * 1024 + inb);
      if (ks & 1) sacc1 = mfma32(a, Qb[ks], sacc1);
      else sacc0 = mfma32(a, Qb[ks], sacc0);
    }
    const f32x16 sacc = sacc0 + sacc1;
    // ---- stage 1: every wave publishes its partial scores, grouped by finalising wave
    {
      float* xw = x1 + (wave * NW) * (64 * VPW) + lane * VPW;
#pragma unroll
      for (int o = 0; o < NW; ++o) {
#pragma unroll
        for (int e = 0; e < VPW; ++e) xw[o * (64 * VPW) + e] = sacc[o * VPW + e];
      }
    }
    // elite term of the registers this wave finalises (overlaps the barrier)
    float fin[VPW];
#pragma unroll
    for (int e = 0; e < VPW; ++e) {
      float d = 0.f;
      if (TWO_R > 0) {
#pragma unroll
        for (int c = 0; c < KCH; ++c) {
          const uint32_t w[4] = {kreg[e][c].x, kreg[e][c].y, kreg[e][c].z, kreg[e][c].w};
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            d = fmaf(qe[8 * c + 2 * i], __uint_as_float(w[i] << 16), d);
            d = fmaf(qe[8 * c + 2 * i + 1], __uint_as_float(w[i] & 0xffff0000u), d);
          }
        }
      }
      fin[e] = d;
    }
    const int64_t next = tile + kTile;
    if (next < t_end) issue_ke(next);     // the elite-key registers are free again
    __syncthreads();
    // ---- stage 2: sum the NW partials of this wave's registers in a fixed order, publish
#pragma unroll
    for (int w2 = 0; w2 < NW; ++w2) {
      const float* xr = x1 + (w2 * NW + wave) * (64 * VPW) + lane * VPW;
#pragma unroll
      for (int e = 0; e < VPW; ++e) fin[e] += xr[e];
    }
    {
      float* xw = x2 + wave * (64 * VPW) + lane * VPW;
#pragma unroll
      for (int e = 0; e < VPW; ++e) xw[e] = fin[e];
    }
    __syncthreads();
    float s[16];
#pragma unroll
    for (int o = 0; o < NW; ++o) {
      const float* xr = x2 + o * (64 * VPW) + lane * VPW;
#pragma unroll
      for (int e = 0; e < VPW; ++e) s[o * VPW + e] = xr[e];
    }
    // ---- online softmax; lane = head n, half g; register v = token 8*(v/4) + 4*g + v%4
    float tmax = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int64_t t = tile + 8 * (v >> 2) + 4 * g + (v & 3);
      s[v] = (t < t_end) ? s[v] : -INFINITY;
      tmax = fmaxf(tmax, s[v]);
    }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, kWave));
    // the reference maximum is raised only when a score exceeds it by more than the slack
    const float m_new = (tmax > m_run + kRescaleSlack || m_run == -INFINITY) ? tmax : m_run;
    const float alpha = exp2f(m_run - m_new);
    float psum = 0.f;
    bf16x8 P[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float pv = exp2f(s[v] - m_new);
      psum += pv;
      P[v >> 3][v & 7] = (__bf16)pv;
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) uacc[ct] *= alpha;
    }

    // ---- latent accumulation: U^T += C^T P^T, the tile read transposed from LDS
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
      const char* trp = tr_row + (ct >> 1) * 1024 + ((ct & 1) ? tr_c1 : tr_c0);
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(trp + (2 * h2) * (NCB * 1024)));
        const s16x4 hi =
            __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(trp + (2 * h2 + 1) * (NCB * 1024)));
        const s16x8 a16 = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        uacc[ct] = mfma32(__builtin_bit_cast(bf16x8, a16), P[h2], uacc[ct]);
      }
    }
    // the tile slice is consumed: refill it with the next tile
    if (next < t_end) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      issue_tile(next);
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
  __syncthreads();                                          // every wave is done with its tile slice
  char* tt = smem + wave * (32 * TSTR);
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint2 pk;
      pk.x = (uint32_t)f32_to_bf16_bits(uacc[ct][4 * j]) | ((uint32_t)f32_to_bf16_bits(uacc[ct][4 * j + 1]) << 16);
      pk.y = (uint32_t)f32_to_bf16_bits(uacc[ct][4 * j + 2]) | ((uint32_t)f32_to_bf16_bits(uacc[ct][4 * j + 3]) << 16);
      *reinterpret_cast<uint2*>(tt + n * TSTR + (ct * 32 + 8 * j + 4 * g) * 2) = pk;
    }
  }
  constexpr int CPRW = DC_W * 2 / 16;                       // 16-byte chunks per head row
  char* ubase = reinterpret_cast<char*>(p.part_u) + (pidx * (int64_t)p.d_c + (int64_t)wave * DC_W) * 2;
#pragma unroll
  for (int i = 0; i < 32 * CPRW / 64; ++i) {
    const int idx = i * 64 + lane;
    const int row = idx / CPRW, ch = idx % CPRW;
    const uint4 v = *reinterpret_cast<const uint4*>(tt + row * TSTR + ch * 16);
    *reinterpret_cast<uint4*>(ubase + (int64_t)row * p.d_c * 2 + ch * 16) = v;
  }
}

// ---------------------------------------------------------------------------------------------
template <int NW, int DC_W, int TWO_R>
static hipError_t launch_attn(const AttnMfmaParams& prm, int64_t B, hipStream_t stream) {
  using L = AttnMfmaLayout<NW, DC_W>;
  static bool attr_done = false;   // raising the dynamic-LDS limit is idempotent
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_mfma_kernel<NW, DC_W, TWO_R>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, L::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  attn_mfma_kernel<NW, DC_W, TWO_R>
      <<<dim3(prm.n_splits, prm.head_groups, (unsigned)B), NW * 64, L::LDS_BYTES, stream>>>(prm);
  return hipGetLastError();
}

bool decode_mfma_supported(const elitekv_dims& d) {
  if (d.dtype != ELITEKV_BF16) return false;
  if ((d.head_dim != 128 && d.head_dim != 64) || (d.head_dim - 2 * d.r) % 8) return false;
  const int two_r = 2 * d.r;
  if (two_r != 8 && two_r != 16) return false;
  return d.d_c == 1536 || d.d_c == 768 || d.d_c == 256;
}

hipError_t launch_decode_mfma(const DecodeArgs& a, const DecodePlan& p, hipStream_t stream) {
  const elitekv_dims& d = a.dims;
  const int n_h = d.n_heads, d_h = d.head_dim, r = d.r, d_c = d.d_c;
  float* qe = (float*)(a.ws + p.off_qe);
  bf16_t* qt = (bf16_t*)(a.ws + p.off_qt);
  AttnMfmaParams prm;
  prm.ke_plane = (const bf16_t*)a.ke_plane; prm.c_plane = (const bf16_t*)a.c_plane;
  prm.qe = qe; prm.qt = qt; prm.seq_len = a.seq_len;
  prm.part_m = (float*)(a.ws + p.off_m); prm.part_l = (float*)(a.ws + p.off_l);
  prm.part_u = (bf16_t*)(a.ws + p.off_u);
  prm.n_h = n_h; prm.d_c = d_c; prm.n_splits = p.n_splits; prm.chunk = p.chunk;
  prm.head_groups = p.head_groups; prm.max_seq_len = a.max_seq_len;
  prm.batch_stride_rows = a.batch_stride_rows; prm.plane_rows = a.plane_rows;

  hipError_t e = launch_qprep_rows(a, qe, qt, (uint32_t*)(a.ws + p.off_cnt), stream);
  if (e != hipSuccess) return e;

  if (a.ev_before) (void)hipEventRecord(a.ev_before, stream);
  e = hipErrorInvalidValue;
  const int two_r = 2 * r;
#define EKV_CASE(DC, NWV, DCW)                                                        \
  if (d_c == DC) {                                                                    \
    e = two_r == 16 ? launch_attn<NWV, DCW, 16>(prm, a.B, stream)                     \
                    : launch_attn<NWV, DCW, 8>(prm, a.B, stream);                     \
  }
  EKV_CASE(1536, 8, 192)
  EKV_CASE(768, 4, 192)
  EKV_CASE(256, 4, 64)
#undef EKV_CASE
  if (e != hipSuccess) return e;
  if (a.ev_after) (void)hipEventRecord(a.ev_after, stream);

  return launch_merge_up(a, p, stream);
}

}  // namespace ekv
