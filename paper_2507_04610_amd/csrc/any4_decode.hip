// Memory-bound any-n GEMM for small M (token generation, M <= 16).
//
// y[m][n] = sum_k x[m][k] * (LUT[n][code[n][k]] * scale[n][k/128] + offset[n][k/128])
// (any4 paper, section 4.2 for y = x w^T and the on-the-fly dequantisation, sections 2.4.1
// and 2.5.2 for the per-row table and alpha * w_Q + beta).
//
// Mapping: one wavefront owns one (output row n, K slice).  Every lane streams the row's packed
// codes with 16-byte loads that are contiguous across the wave, so the row's table, scales and
// offsets are wave-uniform.  The table sits in LDS as 16 fp32 words (16 distinct banks: any mix
// of indices across the lanes is conflict free), weights are dequantised in fp32, multiplied
// into per-lane fp32 accumulators (one per m), and the 64 partial sums are combined with DPP
// row rotations + ds_swizzle.  With several K slices the fp32 partials go to the workspace and
// a second kernel adds them in slice order (no float atomics: bit-reproducible).
#include "any4_device.h"
#include "any4_internal.h"

namespace any4 {

// codes a lane takes per step, chosen so that a step is whole 16-byte loads and never spans
// two scale groups: 4-bit 32 codes (16 B), 2-bit 64 codes (16 B), 3-bit 128 codes (48 B).
template <int BITS> struct LaneUnit;
template <> struct LaneUnit<4> { static constexpr int codes = 32, words = 4; };
template <> struct LaneUnit<2> { static constexpr int codes = 64, words = 4; };
template <> struct LaneUnit<3> { static constexpr int codes = 128, words = 12; };

constexpr int kDecodeWaves = 4;   // wavefronts per block

template <int BITS, int MT>
__global__ __launch_bounds__(kDecodeWaves * 64) void decode_rows_kernel(
    const uint16_t* __restrict__ x, const uint32_t* __restrict__ codes,
    const uint16_t* __restrict__ lut, const uint16_t* __restrict__ scale,
    const uint16_t* __restrict__ offset, int M, int64_t N, int64_t K, int ksplit, int one_table,
    uint16_t* __restrict__ y, float* __restrict__ partial) {
    constexpr int L = 1 << BITS;
    constexpr uint32_t mask = L - 1;
    constexpr int UC = LaneUnit<BITS>::codes, UW = LaneUnit<BITS>::words;
    __shared__ float table[kDecodeWaves][16];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t task = (int64_t)blockIdx.x * kDecodeWaves + wave;   // (row, slice), slice fastest
    const int64_t n = task / ksplit;
    const int slice = (int)(task % ksplit);
    const bool active = n < N;                      // whole wave takes the same branch
    const int64_t nn = active ? n : 0;

    if (lane < L) table[wave][lane] = lut ? bf16_to_f32(lut[(one_table ? 0 : nn * L) + lane]) : (float)(lane - L / 2);   // no table: the integer grid
    __syncthreads();                                // one barrier, reached by every wave
    if (!active) return;

    const int units = (int)(K / UC);                // lane-units in a row
    const int per = (units + ksplit - 1) / ksplit;
    const int u_begin = slice * per;
    const int u_end = min(units, u_begin + per);
    const int64_t G = K / kGroup;
    const uint32_t* row = codes + nn * row_words(K, BITS);

    float acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) acc[m] = 0.f;

    for (int u = u_begin + lane; u < u_end; u += 64) {
        uint32_t q[UW];
#pragma unroll
        for (int i = 0; i < UW / 4; ++i) {
            const uint4 v = reinterpret_cast<const uint4*>(row + (int64_t)u * UW)[i];
            q[4 * i] = v.x; q[4 * i + 1] = v.y; q[4 * i + 2] = v.z; q[4 * i + 3] = v.w;
        }
        const int g = (int)(((int64_t)u * UC) / kGroup);
        const float s = bf16_to_f32(scale[nn * G + g]);
        const float o = bf16_to_f32(offset[nn * G + g]);
        const int64_t k0 = (int64_t)u * UC;
        // walk the unit in runs of 8 codes (= one 16-byte load of x per m)
#pragma unroll
        for (int r = 0; r < UC / 8; ++r) {
            float wv[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int bit = (r * 8 + j) * BITS;             // compile-time
                uint32_t c = q[bit >> 5] >> (bit & 31);
                if ((bit & 31) + BITS > 32) c |= q[(bit >> 5) + 1] << (32 - (bit & 31));
                wv[j] = __builtin_fmaf(table[wave][c & mask], s, o);
            }
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (m < M) {
                    const uint4 xv = *reinterpret_cast<const uint4*>(x + (int64_t)m * K + k0 + r * 8);
                    acc[m] = __builtin_fmaf(wv[0], bf16lo_to_f32(xv.x), acc[m]);
                    acc[m] = __builtin_fmaf(wv[1], bf16hi_to_f32(xv.x), acc[m]);
                    acc[m] = __builtin_fmaf(wv[2], bf16lo_to_f32(xv.y), acc[m]);
                    acc[m] = __builtin_fmaf(wv[3], bf16hi_to_f32(xv.y), acc[m]);
                    acc[m] = __builtin_fmaf(wv[4], bf16lo_to_f32(xv.z), acc[m]);
                    acc[m] = __builtin_fmaf(wv[5], bf16hi_to_f32(xv.z), acc[m]);
                    acc[m] = __builtin_fmaf(wv[6], bf16lo_to_f32(xv.w), acc[m]);
                    acc[m] = __builtin_fmaf(wv[7], bf16hi_to_f32(xv.w), acc[m]);
                }
            }
        }
    }

#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const float total = wave_sum(acc[m]);
        if (lane == 0 && m < M) {
            if (ksplit == 1) y[(int64_t)m * N + nn] = (uint16_t)f32_to_bf16(total);
            else partial[((int64_t)slice * M + m) * N + nn] = total;
        }
    }
}

// y[i] = bf16( sum over slices, in slice order, of partial[s][i] )
__global__ __launch_bounds__(256) void reduce_slices_kernel(const float* __restrict__ partial,
                                                            int ksplit, int64_t MN,
                                                            uint16_t* __restrict__ y) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= MN) return;
    float s = 0.f;
    for (int k = 0; k < ksplit; ++k) s += partial[(int64_t)k * MN + i];
    y[i] = (uint16_t)f32_to_bf16(s);
}

hipError_t launch_reduce_slices(const float* partial, int ksplit, int64_t MN, uint16_t* y, hipStream_t stream) {
    hipLaunchKernelGGL(reduce_slices_kernel, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, stream,
                       partial, ksplit, MN, y);
    return hipGetLastError();
}

template <int BITS>
static hipError_t launch_decode_bits(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                                     const uint16_t* scale, const uint16_t* offset, int M, int64_t N,
                                     int64_t K, const GemmPlan& plan, bool one_table, uint16_t* y, float* partial,
                                     hipStream_t stream) {
    const int64_t tasks = N * plan.ksplit;
    const int64_t blocks = (tasks + kDecodeWaves - 1) / kDecodeWaves;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(kDecodeWaves * 64);
#define ANY4_LAUNCH(MT)                                                                         \
    hipLaunchKernelGGL((decode_rows_kernel<BITS, MT>), grid, block, 0, stream, x, codes, lut,   \
                       scale, offset, M, N, K, plan.ksplit, one_table ? 1 : 0, y, partial)
    if (M == 1) ANY4_LAUNCH(1);
    else if (M == 2) ANY4_LAUNCH(2);
    else if (M <= 4) ANY4_LAUNCH(4);
    else if (M <= 8) ANY4_LAUNCH(8);
    else ANY4_LAUNCH(16);
#undef ANY4_LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || plan.ksplit == 1) return e;
    const int64_t MN = (int64_t)M * N;
    hipLaunchKernelGGL(reduce_slices_kernel, dim3((unsigned)((MN + 255) / 256)), dim3(256), 0, stream,
                       partial, plan.ksplit, MN, y);
    return hipGetLastError();
}

hipError_t launch_decode(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                         const uint16_t* scale, const uint16_t* offset,
                         int64_t M, int64_t N, int64_t K, int bits, const GemmPlan& plan, bool one_table,
                         uint16_t* y, float* partial, hipStream_t stream) {
    switch (bits) {
        case 4: return launch_decode_bits<4>(x, codes, lut, scale, offset, (int)M, N, K, plan, one_table, y, partial, stream);
        case 3: return launch_decode_bits<3>(x, codes, lut, scale, offset, (int)M, N, K, plan, one_table, y, partial, stream);
        default: return launch_decode_bits<2>(x, codes, lut, scale, offset, (int)M, N, K, plan, one_table, y, partial, stream);
    }
}

}  // namespace any4
