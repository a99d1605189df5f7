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
// partials[(row0 + g) * split_stride + split].  nt = threads per workgroup.
template <int G>
__device__ __forceinline__ void finish_splits(float *partials, uint32_t *counter, int row0, int n_splits, float *out,
                                              int tid, int nt, int split_stride = kMaxSplits) {
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
    // One pass over the splits with a running maximum; the loads of a batch of splits are issued together so that
    // the merge costs a few memory round trips, not one per split.
    constexpr int kBatch = 16;
    for (int i = tid; i < G * kD; i += nt) {
        const int g = i / kD, c = i - g * kD;
        const float *p = partials + (size_t)(row0 + g) * split_stride * kPartialStride;
        float M = -INFINITY, L = 0.f, O = 0.f;
        for (int s0 = 0; s0 < n_splits; s0 += kBatch) {
            float ms[kBatch], ls[kBatch], os[kBatch];
#pragma unroll
            for (int k = 0; k < kBatch; k++) {
                const int s = min(s0 + k, n_splits - 1);  // clamped: every load is in bounds
                ms[k] = load_agent(p + s * kPartialStride + kD);
                ls[k] = load_agent(p + s * kPartialStride + kD + 1);
                os[k] = load_agent(p + s * kPartialStride + c);
            }
#pragma unroll
            for (int k = 0; k < kBatch; k++) {
                if (s0 + k < n_splits && ms[k] != -INFINITY) {
                    const float Mn = fmaxf(M, ms[k]);
                    const float fa = __expf(M - Mn), fb = __expf(ms[k] - Mn);
                    L = L * fa + ls[k] * fb;
                    O = O * fa + os[k] * fb;
                    M = Mn;
                }
            }
        }
        out[(size_t)(row0 + g) * kD + c] = O / L;
    }
    if (tid == 0) __hip_atomic_store(counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace kvc
