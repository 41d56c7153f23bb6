// Compute-bound any-n GEMM for large M (prompt processing): LDS-staged table lookup feeding
// bf16 matrix-core (MFMA) tiles with fp32 accumulation.
//
// y[m][n] = sum_k x[m][k] * w[n][k],  w[n][k] = LUT[n][code] * scale[n][k/128] + offset[n][k/128]
// (any4 paper, section 4.2: weights are dequantised on the fly before the matrix instruction;
// sections 2.4.1 / 2.5.2 define the table lookup and alpha * w_Q + beta).  The paper's own
// kernels stop at M = 16; this path is the large-M counterpart for CDNA4.
//
// Rounding a dequantised weight to bf16 would cost up to 2^-8 relative per weight, which is too
// much for the 1e-2 * rms output bound.  The kernel therefore never forms w.  Per group g of
// 128 weights it uses
//     sum_{k in g} x[m][k] w[n][k] = scale[n][g] * sum_{k in g} x[m][k] LUT[n][code[n][k]]
//                                  + offset[n][g] * X[m][g],      X[m][g] = sum_{k in g} x[m][k]
// The first sum multiplies two exact bf16 operands on the matrix cores (fp32 accumulate) and is
// scaled in fp32 on the vector ALU; the second term is a small extra GEMM over the "group"
// dimension whose left operand X is precomputed in fp32 and split into a bf16 high and low part
// (relative error 2^-16), and whose right operand is the bf16 offset itself.
//
// Block tile 256 (m) x 128 (n), K step 64, eight wavefronts in a 4 x 2 arrangement, each owning a
// 64 x 64 sub-tile as 2 x 2 v_mfma_f32_32x32x16_bf16 accumulators.  Two LDS buffers: while the
// matrix cores work on K step s, the activations and codes of step s+1 are already in registers
// (loaded before the MFMAs were issued) and are looked up / written to the other buffer behind
// them; one barrier per K step.
#include "any4_device.h"
#include "any4_internal.h"
#include <type_traits>

namespace any4 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PBM = 256, PBN = 128, PBK = 64;
constexpr int PTHREADS = 512;
constexpr int PLD = PBK + 8;          // LDS row stride in bf16 elements (144 B: keeps 16-byte reads spread over banks)

// X[m][g] = sum of the 128 activations of group g, in fp32, stored as two bf16 (high part,
// remainder) at xs[m][2g], xs[m][2g+1]; columns 2G .. KP-1 are zero.  16 lanes per (m, g).
__global__ __launch_bounds__(256) void group_sums_kernel(const uint16_t* __restrict__ x, int64_t M,
                                                         int64_t K, int KP, uint16_t* __restrict__ xs) {
    const int64_t G = K / kGroup;
    const int64_t unit = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;     // (m, g), g fastest
    const int sub = threadIdx.x & 15;
    const bool live = unit < M * G;
    const int64_t u = live ? unit : 0;
    const uint4 v = reinterpret_cast<const uint4*>(x + u * kGroup)[sub];     // x is [M][G][128]
    float s = ((bf16lo_to_f32(v.x) + bf16hi_to_f32(v.x)) + (bf16lo_to_f32(v.y) + bf16hi_to_f32(v.y))) +
              ((bf16lo_to_f32(v.z) + bf16hi_to_f32(v.z)) + (bf16lo_to_f32(v.w) + bf16hi_to_f32(v.w)));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x121, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x122, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x124, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x128, 0xF, 0xF, false));
    if (!live) return;
    const int64_t m = u / G, g = u % G;
    if (sub == 0) {
        const uint32_t hi = f32_to_bf16(s);
        const uint32_t lo = f32_to_bf16(s - bf16_to_f32(hi));
        *reinterpret_cast<uint32_t*>(xs + m * KP + 2 * g) = hi | (lo << 16);
    }
    // zero padding of the row tail, done by the lanes of the row's last group
    if (g == G - 1)
        for (int c = (int)(2 * G) + sub; c < KP; c += 16) xs[m * KP + c] = 0;
}

// LDS copy of the block's row tables, laid out so that the 32 lanes LDS serves together never share
// a bank: a half-wavefront holds 8 rows x 4 quarter-threads, and entry c of (row, quarter) lives at
// dword (row / 8) * (32 << BITS) + c * 32 + (row % 8) * 4 + quarter (every row is stored 4 times).
template <int BITS>
__global__ __launch_bounds__(PTHREADS, 1) void prefill_kernel(
    const uint16_t* __restrict__ x, const uint32_t* __restrict__ codes,
    const uint16_t* __restrict__ lut, const uint16_t* __restrict__ scale,
    const uint16_t* __restrict__ offset, const uint16_t* __restrict__ xsums, int KP,
    int64_t M, int64_t N, int64_t K, uint16_t* __restrict__ y) {
    constexpr int L = 1 << BITS;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint16_t* xs = reinterpret_cast<uint16_t*>(smem);                              // [2][PBM][PLD]
    uint16_t* ws = xs + 2 * PBM * PLD;                                             // [2][PBN][PLD]
    uint32_t* table = reinterpret_cast<uint32_t*>(ws + 2 * PBN * PLD);             // [PBN / 8][L][32], bf16 value in the low half

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * PBM, n0 = (int64_t)blockIdx.y * PBN;
    const int64_t G = K / kGroup, RW = row_words(K, BITS);

    // weight slab: thread -> (row, 16-code quarter of the K step)
    const int wrow = tid >> 2, wq = tid & 3;
    const int64_t wn_glob = min(n0 + wrow, N - 1);
    // word offset / bit shift of the thread's 16 codes inside the K step's (2 * BITS)-word chunk
    const int qword = BITS == 4 ? 2 * wq : (BITS == 2 ? wq : (6 * wq) >> 2);
    const int qshift = BITS == 3 ? ((6 * wq) & 3) * 8 : 0;
    const uint32_t* wsrc = codes + wn_glob * RW + qword;
    // LDS byte address of this thread's entry 0 (the kernel has no static LDS: dynamic LDS starts at 0)
    const uint32_t tbase = (uint32_t)((2 * PBM * PLD + 2 * PBN * PLD) * 2 + ((wrow >> 3) * (32 << BITS) + (wrow & 7) * 4 + wq) * 4);
    typedef const __attribute__((address_space(3))) uint32_t* lds_u32;
    // activation slab: thread -> 4 rows (256 rows / 64), one 16-byte column piece
    const int xr_row = tid >> 3, xc8 = tid & 7;
    int64_t xm[4];                                                          // rows past M are clamped, never stored
#pragma unroll
    for (int pi = 0; pi < 4; ++pi) xm[pi] = min(m0 + pi * 64 + xr_row, M - 1);
    // the two output columns this lane owns (one per 32-wide n tile of its wavefront)
    const uint16_t* scol[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) scol[j] = scale + min(n0 + wn * 64 + j * 32 + (lane & 31), N - 1) * G;

    f32x16 acc[2][2], part[2][2];
    f32x16 zero;
#pragma unroll
    for (int v = 0; v < 16; ++v) zero[v] = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) { acc[i][j] = zero; part[i][j] = zero; }

    // ---- registers of the K step being fetched
    uint4 xr[4];
    uint32_t qw[2];
    auto fetch_main = [&](int64_t k0) {
#pragma unroll
        for (int pi = 0; pi < 4; ++pi) xr[pi] = *reinterpret_cast<const uint4*>(x + xm[pi] * K + xc8 * 8 + k0);
        const int64_t wbase = (k0 >> 5) * BITS;              // the K step's codes start at word (k0 / 32) * BITS
        qw[0] = wsrc[wbase];
        qw[1] = BITS == 2 ? 0u : wsrc[wbase + 1];
    };
    auto stage_x = [&](int buf) {
        uint16_t* xb = xs + buf * PBM * PLD;
#pragma unroll
        for (int pi = 0; pi < 4; ++pi)
            *reinterpret_cast<uint4*>(&xb[(pi * 64 + xr_row) * PLD + xc8 * 8]) = xr[pi];
    };
    // code j (0..15) of the fetched quarter
    auto code_of = [&](uint32_t lo, uint32_t hi, int j) -> uint32_t {
        if constexpr (BITS == 4) return __builtin_amdgcn_ubfe(j < 8 ? lo : hi, 4 * (j & 7), 4);
        else if constexpr (BITS == 2) return __builtin_amdgcn_ubfe(lo, 2 * j, 2);
        else {
            const int bit = 3 * j;
            if (bit + 3 <= 32) return __builtin_amdgcn_ubfe(lo, bit, 3);
            if (bit >= 32) return __builtin_amdgcn_ubfe(hi, bit - 32, 3);
            return __builtin_amdgcn_alignbit(hi, lo, bit) & 7u;
        }
    };
    auto stage_w_main = [&](int buf) {
        uint16_t* wb = ws + buf * PBN * PLD;
        uint32_t lo = qw[0], hi = qw[1];
        if constexpr (BITS == 3) {
            const unsigned long long v = (((unsigned long long)hi << 32) | lo) >> qshift;
            lo = (uint32_t)v; hi = (uint32_t)(v >> 32);
        }
#pragma unroll
        for (int hlf = 0; hlf < 2; ++hlf) {
            uint32_t b[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) b[j] = *reinterpret_cast<lds_u32>(tbase + (code_of(lo, hi, hlf * 8 + j) << 7));
            *reinterpret_cast<uint4*>(&wb[wrow * PLD + wq * 16 + hlf * 8]) =
                make_uint4(b[0] | (b[1] << 16), b[2] | (b[3] << 16), b[4] | (b[5] << 16), b[6] | (b[7] << 16));
        }
    };
    // matrix cores on buffer `buf`; FIRST: the K step starts a group, its first MFMAs take a zero accumulator
    auto mma = [&](int buf, auto first) {
        constexpr bool FIRST = decltype(first)::value;
        const uint16_t* xb = xs + buf * PBM * PLD;
        const uint16_t* wb = ws + buf * PBN * PLD;
#pragma unroll
        for (int kk = 0; kk < PBK / 16; ++kk) {
            const int col = kk * 16 + (lane >> 5) * 8;
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&xb[(wm * 64 + i * 32 + (lane & 31)) * PLD + col]));
                b[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&wb[(wn * 64 + i * 32 + (lane & 31)) * PLD + col]));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    part[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], (FIRST && kk == 0) ? zero : part[i][j], 0, 0, 0);
        }
    };
    auto fold = [&](float s0, float s1) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                acc[i][0][v] = __builtin_fmaf(part[i][0][v], s0, acc[i][0][v]);
                acc[i][1][v] = __builtin_fmaf(part[i][1][v], s1, acc[i][1][v]);
            }
    };
    using T = std::true_type;
    using F = std::false_type;

    // ---- main loop over groups of 128 (two K steps each).  While the matrix cores work on one buffer,
    //      the next K step (fetched before the MFMAs were issued) is looked up and written to the other.
    fetch_main(0);                                             // in flight while the tables are filled
    // per-row tables of this block's weight rows (rows past N are clamped: they are never stored):
    // one thread fetches 8 bytes (4 entries) of a row and writes each entry's 4 adjacent copies at once
    {
        constexpr int PIECES = L / 4;                            // 8-byte pieces per row
        for (int i = tid; i < PBN * PIECES; i += PTHREADS) {
            const int row = i / PIECES, pc = i % PIECES;
            uint2 v;
            if (lut) v = *reinterpret_cast<const uint2*>(lut + min(n0 + row, N - 1) * L + pc * 4);
            else {                                             // no table: the integer grid, entries pc * 4 .. + 3
                const int c0 = pc * 4 - L / 2;
                v.x = f32_to_bf16((float)c0) | (f32_to_bf16((float)(c0 + 1)) << 16);
                v.y = f32_to_bf16((float)(c0 + 2)) | (f32_to_bf16((float)(c0 + 3)) << 16);
            }
            uint32_t* dst = table + (row >> 3) * (32 << BITS) + (pc * 4) * 32 + (row & 7) * 4;
            const uint32_t e0 = v.x & 0xFFFFu, e1 = v.x >> 16, e2 = v.y & 0xFFFFu, e3 = v.y >> 16;
            *reinterpret_cast<uint4*>(dst) = make_uint4(e0, e0, e0, e0);
            *reinterpret_cast<uint4*>(dst + 32) = make_uint4(e1, e1, e1, e1);
            *reinterpret_cast<uint4*>(dst + 64) = make_uint4(e2, e2, e2, e2);
            *reinterpret_cast<uint4*>(dst + 96) = make_uint4(e3, e3, e3, e3);
        }
    }

    __syncthreads();                                           // tables are written
    stage_x(0);
    stage_w_main(0);
    __syncthreads();
    for (int64_t g = 0; g < G; ++g) {
        const float s0 = bf16_to_f32(scol[0][g]), s1 = bf16_to_f32(scol[1][g]);
        const bool more = g + 1 < G;
        fetch_main(g * kGroup + PBK);
        mma(0, T{});
        stage_x(1);
        stage_w_main(1);
        __syncthreads();
        if (more) fetch_main((g + 1) * kGroup);
        mma(1, F{});
        if (more) { stage_x(0); stage_w_main(0); }
        fold(s0, s1);
        __syncthreads();
    }

    // ---- offset term: a few more K steps over the group dimension (activation group sums split into
    //      bf16 hi + lo in columns 2g, 2g+1; both columns meet offset[n][g]); unscaled
    for (int64_t k0 = 0; k0 < KP; k0 += PBK) {
#pragma unroll
        for (int pi = 0; pi < 4; ++pi)
            xr[pi] = k0 + xc8 * 8 < KP ? *reinterpret_cast<const uint4*>(xsums + xm[pi] * KP + xc8 * 8 + k0) : make_uint4(0, 0, 0, 0);
        uint32_t pk[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int64_t gg = (k0 + wq * 16 + 2 * j) >> 1;
            const uint32_t b = gg < G ? offset[wn_glob * G + gg] : 0u;
            pk[j] = b | (b << 16);
        }
        stage_x(0);
        *reinterpret_cast<uint4*>(&ws[wrow * PLD + wq * 16]) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        *reinterpret_cast<uint4*>(&ws[wrow * PLD + wq * 16 + 8]) = make_uint4(pk[4], pk[5], pk[6], pk[7]);
        __syncthreads();
        mma(0, T{});
        fold(1.f, 1.f);
        __syncthreads();
    }

    // ---- store: accumulator element v of a lane is row 8*(v/4) + 4*(lane/32) + v%4, column lane%32
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int64_t n = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t m = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
                if (m < M && n < N) y[m * N + n] = (uint16_t)f32_to_bf16(acc[i][j][v]);
            }
        }
}

constexpr size_t prefill_lds_bytes(int bits) {
    return (size_t)(2 * PBM * PLD + 2 * PBN * PLD) * 2 + (size_t)PBN * (1 << bits) * 4 * 4;
}

size_t prefill_workspace_bytes(int64_t M, int64_t K) {
    return (size_t)M * (size_t)prefill_kp(K) * sizeof(uint16_t);
}

hipError_t launch_prefill(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                          const uint16_t* scale, const uint16_t* offset,
                          int64_t M, int64_t N, int64_t K, int bits,
                          uint16_t* y, void* workspace, hipStream_t stream) {
    const int64_t gm = (M + PBM - 1) / PBM, gn = (N + PBN - 1) / PBN;
    const int64_t units = M * (K / kGroup);
    const int64_t sblocks = (units * 16 + 255) / 256;
    if (gm > 0x7FFFFFFF || gn > 65535 || sblocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const int KP = prefill_kp(K);
    uint16_t* xsums = static_cast<uint16_t*>(workspace);
    hipLaunchKernelGGL(group_sums_kernel, dim3((unsigned)sblocks), dim3(256), 0, stream, x, M, K, KP, xsums);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 grid((unsigned)gm, (unsigned)gn), block(PTHREADS);
#define ANY4_PREFILL(B)                                                                                           \
    do {                                                                                                          \
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_kernel<B>),                                 \
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)prefill_lds_bytes(B));           \
        if (e != hipSuccess) return e;                                                                            \
        hipLaunchKernelGGL(prefill_kernel<B>, grid, block, prefill_lds_bytes(B), stream, x, codes, lut, scale,    \
                           offset, xsums, KP, M, N, K, y);                                                        \
    } while (0)
    switch (bits) {
        case 4: ANY4_PREFILL(4); break;
        case 3: ANY4_PREFILL(3); break;
        default: ANY4_PREFILL(2); break;
    }
#undef ANY4_PREFILL
    return hipGetLastError();
}

}  // namespace any4
