// In-kernel, deterministic combination of K-slice partial sums (no second kernel, no float atomics).
//
// Every block writes the fp32 partial sums of its (row tile, K slice) to the workspace, then
// bumps the tile's arrival counter.  The block that arrives last adds the partials of ALL slices
// in slice order - so the result does not depend on which block happened to be last - rounds to
// bf16 and stores y.  Counters live at the start of the workspace as 64-bit words
// (epoch << 8 | arrivals).  The epoch is a per-call number chosen on the host: a counter whose
// epoch differs from the current call's is stale (left-over or never-initialised memory) and
// counts as zero, so the workspace needs no initialisation.  The last block puts the counter back
// to (epoch, 0), which keeps a captured launch valid for any number of graph replays.
#pragma once
#include "any4_device.h"

namespace any4 {

constexpr int kMaxSplit = 64;

__host__ __device__ inline size_t splitk_counter_bytes(int64_t tiles) { return (size_t)((tiles * 8 + 255) / 256 * 256); }

// Partial sums and counters are exchanged between blocks that may run on different XCDs (each
// with its own L2).  Instead of device-wide fences - which write back and invalidate whole caches
// and were measured to cost tens of microseconds per launch here - every access to them is a
// relaxed agent-scope atomic (coherent by itself), and ordering comes from waiting for the
// stores' completion before the counter is bumped.
__device__ __forceinline__ void splitk_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float splitk_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Called by all threads of the block after their splitk_store()s.  Returns true (block-uniform)
// in the block that must finish the tile.  `flag` is one int of LDS.
__device__ __forceinline__ bool splitk_arrive(unsigned long long* counters, int tile, int ksplit,
                                              unsigned long long epoch, int* flag) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's partial sums have been written
    __syncthreads();                                   // ... and so have the whole block's
    if (threadIdx.x == 0) {
        unsigned long long* c = counters + tile;
        unsigned long long old = __hip_atomic_load(c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned long long cnt;
        for (;;) {
            cnt = ((old >> 8) == epoch) ? (old & 0xFFull) + 1ull : 1ull;
            const unsigned long long nv = (epoch << 8) | cnt;
            if (__hip_atomic_compare_exchange_strong(c, &old, nv, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT))
                break;
        }
        const bool last = cnt == (unsigned long long)ksplit;
        if (last) __hip_atomic_store(c, epoch << 8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *flag = last ? 1 : 0;
    }
    __syncthreads();
    return *flag != 0;
}

}  // namespace any4
