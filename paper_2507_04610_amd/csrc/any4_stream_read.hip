// Measurement helper: a kernel that only reads a buffer, used by the benchmark to find what
// a launch that streams the same bytes as a GEMM costs on this GPU when it does no arithmetic
// (launch, first-byte latency and the streaming rate a simple kernel reaches).  Not part of the
// any4 method.
#include "any4_device.h"
#include "any4_internal.h"

namespace any4 {

// 1024 persistent blocks of 512 threads; every thread keeps four 16-byte loads in flight and walks
// the buffer with a grid stride; the xor of everything read is stored only if it equals a value
// chosen by the caller (so the loads cannot be removed, and normally nothing is written).
__global__ __launch_bounds__(512) void stream_read_kernel(const uint4* __restrict__ p, int64_t n16,
                                                          uint32_t magic, uint32_t* __restrict__ sink) {
    const int64_t stride = (int64_t)gridDim.x * 512;
    uint32_t acc = 0;
    int64_t i = (int64_t)blockIdx.x * 512 + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = p[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == magic) sink[0] = acc;
}

hipError_t launch_stream_read(const void* p, size_t bytes, uint32_t magic, uint32_t* sink, hipStream_t stream) {
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t want = (n16 + 511) / 512;
    const unsigned blocks = (unsigned)(want < 1 ? 1 : (want > 1024 ? 1024 : want));
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(512), 0, stream,
                       static_cast<const uint4*>(p), n16, magic, sink);
    return hipGetLastError();
}

}  // namespace any4
