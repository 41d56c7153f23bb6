// any4_dequant: materialise w[n][k] = fma(LUT[n][code], scale[n][k/128], offset[n][k/128]) in fp32
// (table, scale and offset stored as bf16, or as fp16 with F16)
// (any4 paper, section 2.4.1 for the per-row table, section 2.5.2 for alpha * w_Q + beta).
// The result is defined bit for bit: one fp32 fused multiply-add per weight.
//
// The kernel is bound by the fp32 store (4 B out per 0.5 B in), so the mapping is chosen for
// the store: one block per row, each thread produces 4 consecutive weights per step and the
// block writes 4 KB of contiguous fp32 with 16-byte stores.
#include "any4_device.h"
#include "any4_internal.h"

namespace any4 {

template <int BITS, bool F16>
__global__ __launch_bounds__(256) void dequant_kernel(const uint32_t* __restrict__ codes,
                                                      const uint16_t* __restrict__ lut,
                                                      const uint16_t* __restrict__ scale,
                                                      const uint16_t* __restrict__ offset,
                                                      int64_t K, int lr, int one_table, float* __restrict__ w) {
    constexpr int L = 1 << BITS;
    constexpr uint32_t mask = L - 1;
    __shared__ float table[L];
    const int64_t n = blockIdx.x;
    if (threadIdx.x < L) table[threadIdx.x] = lut ? h16_to_f32<F16>(lut[(one_table ? 0 : n * L) + threadIdx.x]) : (float)((int)threadIdx.x - L / 2);   // no table: the integer grid
    __syncthreads();

    const uint32_t* row = codes + n * row_words(K, BITS);
    const int gsh = 5 + lr;                             // log2(group size / 4), lr = -1 (groups of 64) .. 3
    const int64_t G = K >> (gsh + 2);                   // scales per row: one per 128 << lr weights
    const int quads = (int)(K / 4);                     // 4 weights = 4*BITS code bits
    float4* out = reinterpret_cast<float4*>(w + n * K);
    for (int q = threadIdx.x; q < quads; q += 256) {
        const int pos = q * 4 * BITS;                   // first bit of the quad inside the row
        const int word = pos >> 5, sh = pos & 31;
        uint64_t window = row[word];
        if (BITS == 3 && sh > 20) window |= (uint64_t)row[word + 1] << 32;   // 12 bits straddle
        const uint32_t c4 = (uint32_t)(window >> sh);
        const int g = q >> gsh;                         // (4q) / group size
        const float s = h16_to_f32<F16>(scale[n * G + g]);
        const float o = h16_to_f32<F16>(offset[n * G + g]);
        float4 r;
        r.x = __builtin_fmaf(table[(c4 >> (0 * BITS)) & mask], s, o);
        r.y = __builtin_fmaf(table[(c4 >> (1 * BITS)) & mask], s, o);
        r.z = __builtin_fmaf(table[(c4 >> (2 * BITS)) & mask], s, o);
        r.w = __builtin_fmaf(table[(c4 >> (3 * BITS)) & mask], s, o);
        out[q] = r;
    }
}

hipError_t launch_dequant(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                          const uint16_t* offset, int64_t N, int64_t K, int bits, int lr, bool f16,
                          bool one_table, float* w, hipStream_t stream) {
    if (N > 0x7FFFFFFF || K > (int64_t)1 << 28) return hipErrorInvalidValue;
    const dim3 grid((unsigned)N), block(256);
#define ANY4_DEQUANT(B)                                                                                   \
    do {                                                                                                  \
        if (f16) hipLaunchKernelGGL((dequant_kernel<B, true>), grid, block, 0, stream, codes, lut, scale, offset, K, lr, one_table ? 1 : 0, w);   \
        else hipLaunchKernelGGL((dequant_kernel<B, false>), grid, block, 0, stream, codes, lut, scale, offset, K, lr, one_table ? 1 : 0, w);      \
    } while (0)
    switch (bits) {
        case 4: ANY4_DEQUANT(4); break;
        case 3: ANY4_DEQUANT(3); break;
        default: ANY4_DEQUANT(2); break;
    }
#undef ANY4_DEQUANT
    return hipGetLastError();
}

}  // namespace any4
