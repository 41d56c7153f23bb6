// In-kernel, deterministic combination of K-slab partial sums (no second kernel, no float atomics).
//
// Every block writes the fp32 partial sums of its (row tile, K slab) to the workspace and, when it
// has finished all its tiles, bumps each tile's arrival counter.  The block that arrives last at a
// tile adds the partials of ALL slabs in slab order - so the result does not depend on which
// block happened to be last - rounds to bf16 and stores y.  Counters live at the start of the
// workspace as 64-bit words (tag << 8 | arrivals) with a fixed 56-bit tag.  A word that does not
// carry the tag (never-initialised memory, or memory an earlier call used for something else)
// counts as zero arrivals, so the workspace needs no initialisation; the last block puts the
// counter back to (tag, 0), so every completed call leaves its counters clean - for the next call
// and for any number of replays of a captured launch.
#pragma once
#include "any4_device.h"

namespace any4 {

constexpr int kMaxSplit = 64;

__host__ __device__ inline size_t splitk_counter_bytes(int64_t tiles) { return (size_t)((tiles * 8 + 255) / 256 * 256); }

// Partial sums and counters are exchanged between blocks that may run on different XCDs (each
// with its own L2).  Instead of device-wide fences - which write back and invalidate whole caches
// and were measured to cost tens of microseconds per launch here - every access to them is a
// relaxed agent-scope atomic (coherent by itself: such accesses are served by the memory side of
// the cache hierarchy, never by a cache private to a compute unit or XCD), and ordering comes from
// waiting for the stores' completion (s_waitcnt vmcnt(0) plus a block barrier) before the counter
// is bumped: a store that has completed at that level is visible to every later agent-scope load,
// and the reader's loads are issued only after its own atomic on the counter has returned.
__device__ __forceinline__ void splitk_store(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float splitk_load(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// One arrival at a tile's counter by a single thread; true if this was the last of `ksplit`.
// The caller has made its partial sums visible (stores issued and waited for) beforehand.
// A counter word is (tag << 8 | arrivals).  The last arrival of a tile puts its counter back to
// "tag, 0", so a workspace that has served a call is clean for the next one and an arrival is ONE
// atomic add; a word without the tag (a workspace used for the first time, or memory that held
// something else) is claimed with a compare-and-swap instead.
constexpr unsigned long long kArriveTag = 0x00A4C0DE5EED17ull;          // 56 bits
__device__ __forceinline__ bool arrive_one(unsigned long long* c, int ksplit) {
    // a word is this call's own only if it carries the tag AND fewer than ksplit arrivals: a tagged word
    // with more (left by a launch that never finished, or by a call with another slab count that
    // shared the memory) is treated like memory that held something else
    auto own = [&](unsigned long long v) -> bool { return (v >> 8) == kArriveTag && (v & 0xFFull) < (unsigned long long)ksplit; };
    unsigned long long old = __hip_atomic_fetch_add(c, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    unsigned long long cnt;
    if (own(old)) {
        cnt = (old & 0xFFull) + 1ull;
    } else {
        // the add above went into a foreign word and is dropped with it
        old += 1ull;
        for (;;) {
            cnt = own(old) ? (old & 0xFFull) + 1ull : 1ull;
            const unsigned long long nv = (kArriveTag << 8) | cnt;
            if (__hip_atomic_compare_exchange_strong(c, &old, nv, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                     __HIP_MEMORY_SCOPE_AGENT))
                break;
        }
    }
    const bool last = cnt == (unsigned long long)ksplit;
    if (last) __hip_atomic_store(c, kArriveTag << 8, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return last;
}

}  // namespace any4
