// Last step of the merge kernels: out[b, h, :] = sum over the latent-column chunks of the chunk's
// up-projection partial (Section 3.2, o = ubar B^v_J, the contraction over the latent cut into chunks).
// The work-groups of one (batch-row tile, head) each leave their chunk's partial in global memory; the one
// that arrives last adds all of them in chunk order (so the sum does not depend on who is last) and writes
// the output rows.  No launch of its own and no cache-wide fence: the partials are written and read with
// device-scope accesses (they bypass the per-XCD L2s' non-coherent copies), a work-group's stores are
// complete before it counts itself in, and the counter is a device-scope atomic.  The counters start at
// zero (the attention kernel of the same call clears them) and the last arrival leaves them at zero.
#pragma once
#include "common.hpp"

namespace ekv {

__device__ __forceinline__ void store_partial_device_scope(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by every thread of the work-group after its partial stores.  opart: [B][n_h][n_chunks][DH] fp32;
// rows b0 .. b0 + rows - 1 of head `head` are this group's; `flag` is one int of LDS.
template <int DH>
__device__ __forceinline__ void sum_chunks_by_last_arrival(const float* opart, bf16_t* out, int* counter, int n_h,
                                                           int n_chunks, int head, int b0, int rows, int* flag) {
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this thread's partials have reached device scope
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int last = old == n_chunks - 1;
    if (last) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag = last;
  }
  __syncthreads();
  if (!*flag) return;
  for (int e = threadIdx.x; e < rows * DH; e += blockDim.x) {
    const int rl = e / DH, j = e % DH;
    const int64_t bh = (int64_t)(b0 + rl) * n_h + head;
    const float* p = opart + bh * n_chunks * DH + j;
    float a = 0.f;
#pragma unroll 4
    for (int c = 0; c < n_chunks; ++c)
      a += __hip_atomic_load(p + (int64_t)c * DH, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    st(out, bh * DH + j, a);
  }
}

}  // namespace ekv
