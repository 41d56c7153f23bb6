// any4_gemm_noalloc: any4_gemm for callers that cannot allocate device memory (code under HIP graph
// capture, tight serving loops, harnesses that forbid hipMalloc).  The scratch any4_gemm takes from
// its caller's workspace argument - arrival counters and fp32 partial sums of K slabs / K slices,
// bf16 group sums of the activations on the matrix-core path - lives here in a file-scope device
// array of fixed size instead, one copy per GPU, held until the process ends.
#include "any4.h"
#include "any4_internal.h"
#include <atomic>

namespace any4 {

constexpr size_t kScratchBytes = (size_t)ANY4_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// In host code `scratch` is only a handle for the runtime's symbol lookup, never an address: every use
// of the array's memory goes through the per-device pointer obtained here.
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_ptr[kMaxDevices];

static hipError_t scratch_of_current_device(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        // first call on this device (with it current): each GPU holds its own copy at its own address
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return hipSuccess;
}

// The array keeps whatever the previous call left.  Partial sums and group sums are always written
// before they are read; the arrival counters are the one thing that must start clean, and the
// words a call uses as counters may have held another call's partial sums, so they are reset to
// zero arrivals here (a fill kernel, not a memset: callers may be capturing a graph).
__global__ void clear_words_kernel(unsigned long long* p, int64_t n) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

}  // namespace any4

using namespace any4;

extern "C" int any4_gemm_noalloc(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                                 const uint16_t* scale, const uint16_t* offset,
                                 int64_t M, int64_t N, int64_t K, int bits, uint16_t* y, void* stream) {
    // the size first: it also rejects bad shapes / bits before anything else happens
    if (M < 1 || N < 1 || K < 1 || K % ANY4_GROUP != 0) return ANY4_ERR_SHAPE;
    if (bits != 4 && bits != 3 && bits != 2) return ANY4_ERR_BITS;
    const GemmPlan plan = plan_gemm(M, N, K, bits);
    if (plan.workspace > kScratchBytes) return ANY4_ERR_WORKSPACE;
    // the remaining argument checks of any4_gemm, so that nothing is looked up or launched for a call
    // that is going to be refused
    if (!x || !codes || !scale || !offset || !y) return ANY4_ERR_NULL;
    if (!lut && bits != 4) return ANY4_ERR_NULL;
    const uintptr_t bitsor = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(codes) |
                             reinterpret_cast<uintptr_t>(lut) | reinterpret_cast<uintptr_t>(scale) |
                             reinterpret_cast<uintptr_t>(offset) | reinterpret_cast<uintptr_t>(y);
    if (bitsor & 15u) return ANY4_ERR_ALIGN;
    void* ws = nullptr;
    if (scratch_of_current_device(&ws) != hipSuccess) return ANY4_ERR_HIP;
    if (plan.counter_bytes > 0) {
        const int64_t nclear = (int64_t)(plan.counter_bytes / 8);
        unsigned long long* base = reinterpret_cast<unsigned long long*>(static_cast<char*>(ws) + plan.counter_offset);
        hipLaunchKernelGGL(clear_words_kernel, dim3((unsigned)((nclear + 255) / 256)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), base, nclear);
        if (hipGetLastError() != hipSuccess) return ANY4_ERR_HIP;
    }
    return gemm_dispatch(x, codes, false, lut, scale, offset, M, N, K, bits, ANY4_GROUP, y, ws, kScratchBytes, stream, false, false);
}
