// Host-side declarations shared between the C ABI (any4_api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <atomic>

namespace any4 {

// Work split of the persistent streaming decode kernel (any4_decode_stream.hip).
struct StreamPlan {
    int gw;               // groups per wavefront (0: the kernel cannot take this problem)
    int slabs;            // K slabs, each owned by `blocks_per_slab` blocks
    int slab_groups;      // groups per slab
    int blocks_per_slab;
    int64_t tiles;        // 16-row tiles
    bool aux;             // tables, scales and offsets are shared through LDS (K/128 multiple of 4)
    size_t workspace;     // bytes: tile counters + fp32 partial sums (several slabs only)
};
StreamPlan plan_stream(int64_t M, int64_t N, int64_t K, int cus);
int device_compute_units();

// Raises the dynamic-LDS limit of kernel `Kern` to `bytes` the first time it is asked for on a device
// (one bit per device ordinal; devices past 63 ask the runtime every time).  Launch functions call
// it before their first launch, so that a refusal leaves nothing enqueued.
template <auto Kern> hipError_t ensure_lds(int bytes) {
    static std::atomic<unsigned long long> done{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && ((done.load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) done.fetch_or(1ull << dev, std::memory_order_release);
    return e;
}

// Work split of the packed-activation kernel for M <= 4 (any4_decode_pack.hip): the whole K axis in one
// block, no workspace.
struct PackPlan {
    bool ok;              // the kernel takes this problem
    int mp;               // rows of x rounded up to 1, 2 or 4
    int passes;           // units of 4 groups per wavefront and tile
    int64_t tiles;        // 16-row tiles
    int nblocks;          // grid size
};
PackPlan plan_pack(int64_t M, int64_t N, int64_t K, int bits, bool one_table, int cus);
hipError_t launch_decode_pack(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                              const uint16_t* scale, const uint16_t* offset, int64_t M, int64_t N,
                              int64_t K, int bits, bool repacked, bool one_table, const PackPlan& pl, uint16_t* y,
                              hipStream_t stream);

// How any4_gemm runs a given problem; a pure function of (M, N, K, bits) so that
// any4_gemm_workspace_bytes() and any4_gemm() always agree.
struct GemmPlan {
    bool decode;          // true: memory-bound small-M kernel, false: matrix-core kernel
    bool stream;          // decode only: persistent streaming kernel; false: one wavefront per (row, K slice)
    StreamPlan sp;
    bool chunked;         // M just above the small-M range: the streaming kernel, 16 rows of x per launch
    StreamPlan sp_tail;   // chunked only: the plan of the last launch when M is not a multiple of 16
    int ksplit;           // number of K slices whose fp32 partials are reduced in a 2nd pass
    size_t workspace;     // bytes of scratch: K-slice partials (decode) or group sums of x (matrix-core path)
    size_t counter_offset, counter_bytes;   // where in the workspace the arrival counters sit (groups of 128)
};
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K, int bits);
// Validation, kernel choice and launches behind every any4_gemm* entry point; returns an ANY4_* code.
int gemm_dispatch(const uint16_t* x, const uint32_t* codes, bool repacked, const uint16_t* lut,
                  const uint16_t* scale, const uint16_t* offset, int64_t M, int64_t N, int64_t K,
                  int bits, int group, uint16_t* y, void* workspace, size_t workspace_bytes, void* stream,
                  bool f16, bool one_table);

hipError_t launch_pack(const uint8_t* codes_u8, int64_t N, int64_t K, int bits,
                       uint32_t* codes, hipStream_t stream);
hipError_t launch_dequant(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                          const uint16_t* offset, int64_t N, int64_t K, int bits, int lr, bool f16,
                          bool one_table, float* w, hipStream_t stream);
hipError_t launch_decode(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                         const uint16_t* scale, const uint16_t* offset,
                         int64_t M, int64_t N, int64_t K, int bits, const GemmPlan& plan, bool one_table,
                         uint16_t* y, float* partial, hipStream_t stream);
hipError_t launch_decode_stream(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                                const uint16_t* scale, const uint16_t* offset, int64_t M, int64_t N,
                                int64_t K, int bits, int lr, bool repacked, bool f16, bool one_table, const StreamPlan& sp, uint16_t* y,
                                void* workspace, hipStream_t stream);
hipError_t launch_reduce_slices(const float* partial, int ksplit, int64_t MN, uint16_t* y, hipStream_t stream);
hipError_t launch_prefill(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                          const uint16_t* scale, const uint16_t* offset,
                          int64_t M, int64_t N, int64_t K, int bits, int lr, bool repacked, bool f16, bool one_table, int cus,
                          uint16_t* y, void* workspace, hipStream_t stream);
// Tile-major re-layout of the packed codes (any4_repack).
hipError_t launch_repack(const uint32_t* codes, int64_t N, int64_t K, int bits, uint32_t* out, hipStream_t stream);

// Matrix-core path: padded length of the "group" dimension (two bf16 columns per group of 128 - of
// 64 with `fine` - rounded up to the MFMA K granularity of 16) and the scratch it needs for the group sums of x.
inline int prefill_kp(int64_t K, bool fine) { return (int)((2 * (K / (fine ? 64 : 128)) + 15) / 16 * 16); }
// its work split (tiles of 256 x 128 outputs; the tiles of a thin last round are cut along K) and scratch
struct PrefillPlan {
    int64_t gm, tiles, tail_tiles;
    int tail_s;
    size_t xsums_bytes, counter_bytes, partial_bytes;
};
PrefillPlan plan_prefill(int64_t M, int64_t N, int64_t K, int cus);
size_t prefill_workspace_bytes(int64_t M, int64_t N, int64_t K, int cus);

// Quantiser: one block per row, the row lives in LDS, which bounds K.  centre_gap < 0: every row by the
// per-weight method; otherwise rows of K <= 16384 are sorted once and a row falls back to the per-weight
// method when two unequal centres come closer than centre_gap * max|w_S|.
size_t quantize_max_k();
constexpr double kQuantizeCentreGap = 9.094947017729282e-13;      // 2^-40: ~2^12 roundings of a distance
hipError_t launch_quantize(const float* w, const float* act, const float* u, int64_t N, int64_t K, int bits,
                           int symmetric, int iters, double centre_gap, uint8_t* codes, uint16_t* lut, uint16_t* scale,
                           uint16_t* offset, int32_t* msteps, hipStream_t stream);

}  // namespace any4
