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
//   search_rotate : q^, k^ = every chunk rotated at the token's position (angle reduced in double)
//   search_round  : per (head, block of 16 queries): the 64 distances over its causal pairs
//   search_pick   : per head: fixed-order sum over the query blocks, arg-min, elite mask update
// All state (rotated copies, partial distances, elite masks) lives in the caller's workspace; the
// r rounds are 2 r launches on the caller's stream with no host synchronisation in between.
#include "common.hpp"
#include "launch.hpp"

namespace ekv {

constexpr int kSrTile = 16;      // queries (and keys) per tile; 16 x 16 pairs = one work-group of 256 threads
constexpr int kSrMaxChunks = 64; // head_dim <= 128

__global__ __launch_bounds__(256) void search_rotate_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                            const int32_t* __restrict__ pos, float* __restrict__ qr,
                                                            float* __restrict__ kr, int64_t T, int n_h, int d_h,
                                                            RopeTable rope) {
  const int half = d_h / 2;
  const int64_t total = T * n_h * half;
  for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < total; e += (int64_t)gridDim.x * 256) {
    const int i = (int)(e % half);
    const int64_t th = e / half;                  // t * n_h + h
    const int64_t t = th / n_h;
    float sn, cs;
    rope_sincos(pos[t], rope.theta[i], &sn, &cs);
    const int64_t o = th * d_h + 2 * i;
    const float qu = q[o], qv = q[o + 1], ku = k[o], kv = k[o + 1];
    qr[o] = qu * cs - qv * sn; qr[o + 1] = qu * sn + qv * cs;
    kr[o] = ku * cs - kv * sn; kr[o + 1] = ku * sn + kv * cs;
  }
}

// grid (query blocks, heads); thread <-> (query tq, key tk) of a 16 x 16 tile, looping over the key
// tiles up to the diagonal.  LDS: the tile's raw and rotated queries and keys.
__global__ __launch_bounds__(256) void search_round_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                           const float* __restrict__ qr, const float* __restrict__ kr,
                                                           const uint64_t* __restrict__ emask,
                                                           float* __restrict__ partial, int64_t T, int n_h, int d_h,
                                                           float scale) {
  __shared__ float2 qs[2][kSrTile][kSrMaxChunks];     // [raw | rotated][query][chunk]
  __shared__ float2 ks[2][kSrTile][kSrMaxChunks + 1]; // padded: 16 different keys are read at one chunk
  __shared__ float red[4][kSrMaxChunks];
  const int half = d_h / 2;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tq = tid >> 4, tk = tid & 15;
  const int qb = blockIdx.x, h = blockIdx.y;
  const int64_t t0 = (int64_t)qb * kSrTile;
  const uint64_t elite = emask[h];

  for (int e = tid; e < kSrTile * half; e += 256) {
    const int r = e / half, i = e % half;
    const int64_t t = t0 + r;
    float2 a = make_float2(0.f, 0.f), b = a;
    if (t < T) {
      const int64_t o = (t * n_h + h) * d_h + 2 * i;
      a = make_float2(q[o], q[o + 1]);
      b = make_float2(qr[o], qr[o + 1]);
    }
    qs[0][r][i] = a; qs[1][r][i] = b;
  }

  float acc[kSrMaxChunks];
#pragma unroll
  for (int c = 0; c < kSrMaxChunks; ++c) acc[c] = 0.f;

  for (int64_t j0 = 0; j0 <= t0; j0 += kSrTile) {
    __syncthreads();                                 // the previous key tile has been consumed (and qs is written)
    for (int e = tid; e < kSrTile * half; e += 256) {
      const int r = e / half, i = e % half;
      const int64_t j = j0 + r;
      float2 a = make_float2(0.f, 0.f), b = a;
      if (j < T) {
        const int64_t o = (j * n_h + h) * d_h + 2 * i;
        a = make_float2(k[o], k[o + 1]);
        b = make_float2(kr[o], kr[o + 1]);
      }
      ks[0][r][i] = a; ks[1][r][i] = b;
    }
    __syncthreads();
    const int64_t t = t0 + tq, j = j0 + tk;
    if (t < T && j <= t) {                           // causal pairs only
      float D[kSrMaxChunks];
      float resid = 0.f;
#pragma unroll
      for (int i = 0; i < kSrMaxChunks; ++i) {
        D[i] = 0.f;
        if (i < half) {
          const float2 a = qs[0][tq][i], ar = qs[1][tq][i], b = ks[0][tk][i], br = ks[1][tk][i];
          D[i] = ((ar.x * br.x + ar.y * br.y) - (a.x * b.x + a.y * b.y)) * scale;
          if (!((elite >> i) & 1ull)) resid += D[i];
        }
      }
#pragma unroll
      for (int c = 0; c < kSrMaxChunks; ++c) acc[c] += fabsf(resid - D[c]);
    }
  }

  // sum over the 256 threads in a fixed order: wave shuffles, then the four waves
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
  const size_t vec = (size_t)T * n_h * d_h * sizeof(float);
  const size_t n_qb = (size_t)((T + kSrTile - 1) / kSrTile);
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  return up(vec) * 2 + up((size_t)n_h * n_qb * kSrMaxChunks * sizeof(float)) + up((size_t)n_h * sizeof(uint64_t));
}

hipError_t launch_ropelite_search(const float* q, const float* k, const int32_t* pos, int64_t T, int n_h, int d_h,
                                  int r, double rope_base, int32_t* elite_out, float* dist_out, char* ws,
                                  hipStream_t stream) {
  const size_t vec = ((size_t)T * n_h * d_h * sizeof(float) + 255) / 256 * 256;
  const int n_qb = (int)((T + kSrTile - 1) / kSrTile);
  float* qr = (float*)ws;
  float* kr = (float*)(ws + vec);
  float* partial = (float*)(ws + 2 * vec);
  uint64_t* emask = (uint64_t*)(ws + 2 * vec + ((size_t)n_h * n_qb * kSrMaxChunks * sizeof(float) + 255) / 256 * 256);
  const int half = d_h / 2;
  search_init_kernel<<<(n_h + 63) / 64, 64, 0, stream>>>(emask, n_h);
  const int64_t total = T * n_h * half;
  search_rotate_kernel<<<(unsigned)((total + 255) / 256 < 4096 ? (total + 255) / 256 : 4096), 256, 0, stream>>>(
      q, k, pos, qr, kr, T, n_h, d_h, rope_table(rope_base, d_h));
  const float scale = 1.f / sqrtf((float)d_h);
  for (int round = 0; round < r; ++round) {
    search_round_kernel<<<dim3(n_qb, n_h), 256, 0, stream>>>(q, k, qr, kr, emask, partial, T, n_h, d_h, scale);
    search_pick_kernel<<<n_h, 64, 0, stream>>>(partial, emask, elite_out, dist_out, n_qb, half, r, round);
  }
  return hipGetLastError();
}

}  // namespace ekv
