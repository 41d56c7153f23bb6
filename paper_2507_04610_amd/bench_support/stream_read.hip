// Measurement helper of bench.py, built as its own small library (libany4_bench.so): a kernel that
// only reads a buffer.  The benchmark times it on the same buffers as the GEMM to report what a
// launch that streams those bytes costs on this GPU when it does no arithmetic (launch, first-byte
// latency and the streaming rate a simple kernel reaches).  Not part of the any4 method and not
// part of libany4's C ABI.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

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

// Reads the first (bytes / 16) * 16 bytes at p (device memory, 16-byte aligned, at least 16 bytes) once
// on `stream`; sink is a device uint32[1] that is normally left untouched.  0 = launched, -1 = refused.
extern "C" int bench_stream_read(const void* p, size_t bytes, uint32_t magic, uint32_t* sink, void* stream) {
    if (!p || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(p) & 15u)) return -1;
    const int64_t n16 = (int64_t)(bytes / 16);
    const int64_t want = (n16 + 511) / 512;
    const unsigned blocks = (unsigned)(want < 1 ? 1 : (want > 1024 ? 1024 : want));
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(512), 0, static_cast<hipStream_t>(stream),
                       static_cast<const uint4*>(p), n16, magic, sink);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
