// Merging the sequence splits of a decode-attention launch inside the same kernel (the "sum reduction" that ends
// the V path in Section 3.3.2).  Every workgroup writes one partial (o[128], m, l) per query head; the workgroup
// that arrives last at a per-(batch, kv head) ticket counter merges all splits and writes the output.  The counter
// is left at zero for the next launch.
//
// gfx950 has one L2 per XCD, and the workgroups of one launch are spread over all XCDs.  A device-scope fence would
// write back / invalidate a whole L2 on every workgroup, which costs far more than the merge itself.  Instead the
// few words that cross workgroups -- the partials and the ticket -- are written and read with device-scope (agent)
// atomic accesses, which go through to the memory-side coherence point, and each wave waits for its own partial
// stores to complete before the workgroup takes its ticket.
#pragma once

#include "kvcomp_internal.h"

namespace kvc {

__device__ __forceinline__ void store_agent(float *p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_agent(const float *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by all threads of the workgroup after they have written this workgroup's partials with store_agent() to
// partials[(row0 + g) * kMaxSplits + split].  NT = threads per workgroup.
template <int G, int NT>
__device__ __forceinline__ void finish_splits(float *partials, uint32_t *counter, int row0, int n_splits, float *out,
                                              int tid) {
    __shared__ uint32_t s_last;
    // every wave: all of its (write-through) partial stores have completed before the barrier is passed
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);  // vmcnt(0) expcnt(0) lgkmcnt(0)
    __syncthreads();
    if (tid == 0) {
        const uint32_t ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = ticket == (uint32_t)(n_splits - 1);
    }
    __syncthreads();
    if (!s_last) return;
    for (int i = tid; i < G * kD; i += NT) {
        const int g = i / kD, c = i - g * kD;
        const float *p = partials + (size_t)(row0 + g) * kMaxSplits * kPartialStride;
        float M = -INFINITY;
        for (int s = 0; s < n_splits; s++) M = fmaxf(M, load_agent(p + s * kPartialStride + kD));
        float L = 0.f, O = 0.f;
#pragma unroll 4
        for (int s = 0; s < n_splits; s++) {
            const float ms = load_agent(p + s * kPartialStride + kD);
            const float l = load_agent(p + s * kPartialStride + kD + 1);
            const float o = load_agent(p + s * kPartialStride + c);
            const float f = ms == -INFINITY ? 0.f : __expf(ms - M);
            L = fmaf(l, f, L);
            O = fmaf(o, f, O);
        }
        out[(size_t)(row0 + g) * kD + c] = O / L;
    }
    if (tid == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace kvc
