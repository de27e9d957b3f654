// RoPElite search (Section 3.1, Algorithm 1): the greedy choice of every head's elite chunks from a
// sample of un-rotated queries and keys of one layer.
//
// With D_i[t, j] = q_{t,i} R((t - j) theta_i) k_{j,i}^T - q_{t,i} k_{j,i}^T (what rotating chunk i adds to
// the score of the causal pair j <= t; Section 3.1 score equation), the scores with elite set E
// differ from the scores of full RoPE by the residual R_E = sum_{i not in E} D_i, and trying chunk c
// as the one addition leaves R_E - D_c.  A round of the algorithm therefore is
//     distance[c] = sum over causal pairs of | R_E[t, j] - D_c[t, j] |   for every c not in E,
// followed by the arg-min (lowest index on ties).  D_i is recomputed from the fully rotated and
// the un-rotated vectors in every round (q^_i . k^_i - q_i . k_i, eq. 1a = 1b), never stored.
//
//   search_pack   : every token's chunks rotated at its position (angle reduced in double) and laid out as the
//                   operands of the round kernel: per (token, head) four rows of 64 chunk values,
//                   query side (q^.x, q^.y, -q.x, -q.y) / sqrt(d_h), key side (k^.x, k^.y, k.x, k.y),
//                   so that D_i[t, j] is the 4-term dot product of row-pairs: a rank-4 contraction per chunk
//   search_round  : per (head, block of 16 queries): the 64 distances over its causal pairs; D_i of a
//                   16 x 16 tile of pairs is one v_mfma_f32_16x16x4_f32 (fp32 in, fp32 out)
//   search_pick   : per head: fixed-order sum over the query blocks, arg-min, elite mask update
// All state (packed copies, partial distances, elite masks) lives in the caller's workspace; the
// r rounds are 2 r launches on the caller's stream with no host synchronisation in between.
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

constexpr int kSrTile = 16;      // queries (and keys) per tile
constexpr int kSrMaxChunks = 64; // head_dim <= 128; the packed rows always hold 64 chunks (zeros beyond d_h / 2)
constexpr int kSrRow = 4 * kSrMaxChunks;   // floats per (token, head) of a packed operand

typedef __attribute__((ext_vector_type(4))) float sr_f32x4;

// Operand order: the four rows x 64 chunks of the 16 tokens of a tile (tiles start at multiples of 16) lie as
// [quad of chunks c4 (16)][lane (64)][4 chunks], lane = 16 * row + token % 16: one 16-byte load per lane and
// instruction, 1 KiB contiguous per wave instruction, 16 instructions per operand.  Tokens beyond T are zeros.
__device__ __forceinline__ int64_t sr_packed_index(int64_t token, int n_h, int h, int row, int chunk) {
  const int64_t tile = token / kSrTile;
  const int lane = 16 * row + (int)(token % kSrTile);
  return (((tile * n_h + h) * (kSrMaxChunks / 4) + chunk / 4) * 64 + lane) * 4 + chunk % 4;
}

__global__ __launch_bounds__(256) void search_pack_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                          const int32_t* __restrict__ pos, float* __restrict__ qp,
                                                          float* __restrict__ kp, int64_t T, int64_t T_pad, int n_h,
                                                          int d_h, float scale, RopeTable rope) {
  const int half = d_h / 2;
  const int64_t total = T_pad * n_h * kSrMaxChunks;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int i = (int)(e % kSrMaxChunks);
    const int64_t th = e / kSrMaxChunks;          // t * n_h + h
    const int64_t t = th / n_h;
    const int h = (int)(th % n_h);
    float qu = 0.f, qv = 0.f, ku = 0.f, kv = 0.f, sn = 0.f, cs = 1.f;
    if (i < half && t < T) {
      rope_sincos(pos[t], rope.theta[i], &sn, &cs);
      const int64_t o = th * d_h + 2 * i;
      qu = q[o]; qv = q[o + 1]; ku = k[o]; kv = k[o + 1];
    }
    qp[sr_packed_index(t, n_h, h, 0, i)] = (qu * cs - qv * sn) * scale;
    qp[sr_packed_index(t, n_h, h, 1, i)] = (qu * sn + qv * cs) * scale;
    qp[sr_packed_index(t, n_h, h, 2, i)] = -qu * scale;
    qp[sr_packed_index(t, n_h, h, 3, i)] = -qv * scale;
    kp[sr_packed_index(t, n_h, h, 0, i)] = ku * cs - kv * sn;
    kp[sr_packed_index(t, n_h, h, 1, i)] = ku * sn + kv * cs;
    kp[sr_packed_index(t, n_h, h, 2, i)] = ku;
    kp[sr_packed_index(t, n_h, h, 3, i)] = kv;
  }
}

// One wave's operand of the 16-token tile `tile`: lane l holds row l / 16 (of the four) of token l % 16, all 64 chunks.
__device__ __forceinline__ void sr_load_operand(const float* __restrict__ packed, int64_t tile, int n_h, int h, int lane,
                                                float (&v)[kSrMaxChunks]) {
  const sr_f32x4* src = reinterpret_cast<const sr_f32x4*>(packed) + ((tile * n_h + h) * (kSrMaxChunks / 4)) * 64 + lane;
#pragma unroll
  for (int c4 = 0; c4 < kSrMaxChunks / 4; ++c4) {
    const sr_f32x4 x = src[c4 * 64];
    v[4 * c4] = x[0]; v[4 * c4 + 1] = x[1]; v[4 * c4 + 2] = x[2]; v[4 * c4 + 3] = x[3];
  }
}

// grid (query blocks, heads), four waves; the key tiles up to the diagonal are dealt to the waves round-robin.
// Per key tile a wave holds the query operand A (loaded once) and the key operand B in registers:
//   pass 1  R  = sum over the chunks outside E of A_c B_c   (the residual of the tile's 256 pairs, 4 per lane)
//   pass 2  for every chunk c: D_c = A_c B_c, distance[c] += sum over the lane's pairs of |R - D_c|
// (lane l of the result tile holds queries 4 (l / 16) + v, v < 4, against key l % 16; on the diagonal tile the
// pairs with key > query carry weight 0).  Chunks in E are computed like the others and ignored by search_pick.
__global__ __launch_bounds__(256, 2) void search_round_kernel(const float* __restrict__ qp, const float* __restrict__ kp,
                                                           const uint64_t* __restrict__ emask,
                                                           float* __restrict__ partial, int n_h) {
  __shared__ float red[4][kSrMaxChunks];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kk = lane >> 4;
  const int qb = gridDim.x - 1 - blockIdx.x, h = blockIdx.y;     // the blocks with the most key tiles start first
  const uint64_t elite = emask[h];

  // the query operand is the same for the four waves: it stays in LDS (operand order, each lane reads its own quads)
  // ... twice: as it is (pass 2) and with the chunks of E set to zero (pass 1: no branches, no masking in the loop)
  __shared__ sr_f32x4 As[kSrMaxChunks / 4][64];
  __shared__ sr_f32x4 Am[kSrMaxChunks / 4][64];
  {
    const sr_f32x4* src = reinterpret_cast<const sr_f32x4*>(qp) + (((int64_t)qb * n_h + h) * (kSrMaxChunks / 4)) * 64 + lane;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c4 = 4 * wave + u;
      sr_f32x4 x = src[c4 * 64];
      As[c4][lane] = x;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if ((elite >> (4 * c4 + e)) & 1ull) x[e] = 0.f;
      Am[c4][lane] = x;
    }
  }
  float B[kSrMaxChunks], acc[kSrMaxChunks];
#pragma unroll
  for (int c = 0; c < kSrMaxChunks; ++c) acc[c] = 0.f;
  __syncthreads();

  for (int jt = wave; jt <= qb; jt += 4) {
    asm volatile("" ::: "memory");     // the query quads are re-read from LDS for every tile, not kept in 64 more registers
    sr_load_operand(kp, jt, n_h, h, lane, B);
    // pass 1: four independent chains over the masked query operand
    sr_f32x4 Rc[4] = {(sr_f32x4)(0.f), (sr_f32x4)(0.f), (sr_f32x4)(0.f), (sr_f32x4)(0.f)};
#pragma unroll
    for (int c4 = 0; c4 < kSrMaxChunks / 4; ++c4) {
      const sr_f32x4 a4 = Am[c4][lane];
#pragma unroll
      for (int u = 0; u < 4; ++u) Rc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[u], B[4 * c4 + u], Rc[u], 0, 0, 0);
    }
    const sr_f32x4 R = (Rc[0] + Rc[1]) + (Rc[2] + Rc[3]);
    float w[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) w[v] = (jt < qb || i16 <= 4 * kk + v) ? 1.f : 0.f;
    // pass 2: four chunks' products in flight before the vector work on the first of them begins
#pragma unroll
    for (int c4 = 0; c4 < kSrMaxChunks / 4; ++c4) {
      const sr_f32x4 a4 = As[c4][lane];
      sr_f32x4 D[4];
#pragma unroll
      for (int u = 0; u < 4; ++u)
        D[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[u], B[4 * c4 + u], (sr_f32x4)(0.f), 0, 0, 0);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float a = acc[4 * c4 + u];
#pragma unroll
        for (int v = 0; v < 4; ++v) a = fmaf(w[v], fabsf(R[v] - D[u][v]), a);
        acc[4 * c4 + u] = a;
      }
    }
  }

  // sum over the 256 lanes in a fixed order: wave shuffles, then the four waves
#pragma unroll
  for (int c = 0; c < kSrMaxChunks; ++c) {
    const float v = wave_sum(acc[c]);
    if (lane == 0) red[wave][c] = v;
  }
  __syncthreads();
  if (tid < kSrMaxChunks)
    partial[((int64_t)h * gridDim.x + qb) * kSrMaxChunks + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
}

// grid (heads); one wave: lane <-> chunk
__global__ __launch_bounds__(64) void search_pick_kernel(const float* __restrict__ partial, uint64_t* __restrict__ emask,
                                                         int32_t* __restrict__ elite_out, float* __restrict__ dist_out,
                                                         int n_qb, int half, int r, int round) {
  const int h = blockIdx.x, c = threadIdx.x;
  float d = 0.f;
#pragma unroll 8
  for (int b = 0; b < n_qb; ++b) d += partial[((int64_t)h * n_qb + b) * kSrMaxChunks + c];
  const uint64_t elite = emask[h];
  const bool cand = c < half && !((elite >> c) & 1ull);
  float best = cand ? d : INFINITY;
  int arg = cand ? c : kSrMaxChunks;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {                 // arg-min, the lowest index wins a tie
    const float ob = __shfl_xor(best, o, kWave);
    const int oa = __shfl_xor(arg, o, kWave);
    if (ob < best || (ob == best && oa < arg)) { best = ob; arg = oa; }
  }
  if (c == 0) {
    elite_out[h * r + round] = arg;
    if (dist_out) dist_out[h * r + round] = best;
    emask[h] = elite | (1ull << arg);
  }
}

__global__ void search_init_kernel(uint64_t* emask, int n_h) {
  const int h = blockIdx.x * blockDim.x + threadIdx.x;
  if (h < n_h) emask[h] = 0ull;
}

size_t search_workspace_bytes(int64_t T, int n_h, int d_h) {
  const size_t n_qb = (size_t)((T + kSrTile - 1) / kSrTile);
  const size_t vec = n_qb * kSrTile * n_h * kSrRow * sizeof(float);      // one packed operand (whole tiles)
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  return up(vec) * 2 + up((size_t)n_h * n_qb * kSrMaxChunks * sizeof(float)) + up((size_t)n_h * sizeof(uint64_t));
}

hipError_t launch_ropelite_search(const float* q, const float* k, const int32_t* pos, int64_t T, int n_h, int d_h,
                                  int r, double rope_base, int32_t* elite_out, float* dist_out, char* ws,
                                  hipStream_t stream) {
  const int n_qb = (int)((T + kSrTile - 1) / kSrTile);
  const int64_t T_pad = (int64_t)n_qb * kSrTile;
  const size_t vec = ((size_t)T_pad * n_h * kSrRow * sizeof(float) + 255) / 256 * 256;
  float* qp = (float*)ws;
  float* kp = (float*)(ws + vec);
  float* partial = (float*)(ws + 2 * vec);
  uint64_t* emask = (uint64_t*)(ws + 2 * vec + ((size_t)n_h * n_qb * kSrMaxChunks * sizeof(float) + 255) / 256 * 256);
  const int half = d_h / 2;
  search_init_kernel<<<(n_h + 63) / 64, 64, 0, stream>>>(emask, n_h);
  const int64_t total = T_pad * n_h * kSrMaxChunks;
  const float scale = 1.f / sqrtf((float)d_h);
  search_pack_kernel<<<(unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096), 256, 0, stream>>>(
      q, k, pos, qp, kp, T, T_pad, n_h, d_h, scale, rope_table(rope_base, d_h));
  for (int round = 0; round < r; ++round) {
    search_round_kernel<<<dim3(n_qb, n_h), 256, 0, stream>>>(qp, kp, emask, partial, n_h);
    search_pick_kernel<<<n_h, 64, 0, stream>>>(partial, emask, elite_out, dist_out, n_qb, half, r, round);
  }
  return hipGetLastError();
}

}  // namespace ekv
