// any4_pack: one code per byte -> packed little-endian words (offline step).
// The any4 paper arranges weights offline too (section 4.2, second paragraph); the
// layout produced here is the plain row-major one of the problem statement.
#include "any4_device.h"
#include "any4_internal.h"

namespace any4 {

// One thread packs 32 consecutive codes (32 input bytes) into BITS output words.
// 32 codes * BITS bits is a whole number of words for BITS = 4, 3 and 2, and a row
// holds a whole number of such units because K is a multiple of 128.
template <int BITS>
__global__ __launch_bounds__(256) void pack_kernel(const uint4* __restrict__ in,
                                                   uint32_t* __restrict__ out, int64_t units) {
    const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= units) return;
    const uint4 a = in[2 * u], b = in[2 * u + 1];
    const uint32_t src[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
    constexpr uint32_t mask = (1u << BITS) - 1u;
    uint32_t w[BITS];
    uint64_t acc = 0;
    int fill = 0, ow = 0;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
        const uint32_t c = (src[j >> 2] >> (8 * (j & 3))) & mask;
        acc |= (uint64_t)c << fill;
        fill += BITS;
        if (fill >= 32) {
            w[ow++] = (uint32_t)acc;
            acc >>= 32;
            fill -= 32;
        }
    }
    uint32_t* o = out + u * BITS;
    if constexpr (BITS == 4) {
        *reinterpret_cast<uint4*>(o) = make_uint4(w[0], w[1], w[2], w[3]);
    } else if constexpr (BITS == 2) {
        *reinterpret_cast<uint2*>(o) = make_uint2(w[0], w[1]);
    } else {
        o[0] = w[0]; o[1] = w[1]; o[2] = w[2];
    }
}

hipError_t launch_pack(const uint8_t* codes_u8, int64_t N, int64_t K, int bits,
                       uint32_t* codes, hipStream_t stream) {
    const int64_t units = N * K / 32;
    const int64_t blocks = (units + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(256);
    const uint4* in = reinterpret_cast<const uint4*>(codes_u8);
    switch (bits) {
        case 4: hipLaunchKernelGGL(pack_kernel<4>, grid, block, 0, stream, in, codes, units); break;
        case 3: hipLaunchKernelGGL(pack_kernel<3>, grid, block, 0, stream, in, codes, units); break;
        default: hipLaunchKernelGGL(pack_kernel<2>, grid, block, 0, stream, in, codes, units); break;
    }
    return hipGetLastError();
}

}  // namespace any4
