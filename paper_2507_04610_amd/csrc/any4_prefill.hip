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
// Block tile 128 (m) x 128 (n), K step 64, four wavefronts in a 2 x 2 arrangement, each owning a
// 64 x 64 sub-tile as 2 x 2 v_mfma_f32_32x32x16_bf16 accumulators.
#include "any4_device.h"
#include "any4_internal.h"

namespace any4 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PBM = 128, PBN = 128, PBK = 64;
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

template <int BITS>
__global__ __launch_bounds__(256) void prefill_kernel(
    const uint16_t* __restrict__ x, const uint32_t* __restrict__ codes,
    const uint16_t* __restrict__ lut, const uint16_t* __restrict__ scale,
    const uint16_t* __restrict__ offset, const uint16_t* __restrict__ xsums, int KP,
    int64_t M, int64_t N, int64_t K, uint16_t* __restrict__ y) {
    constexpr int L = 1 << BITS;
    constexpr uint32_t mask = L - 1;
    __shared__ __attribute__((aligned(16))) uint16_t xs[PBM * PLD];
    __shared__ __attribute__((aligned(16))) uint16_t ws[PBN * PLD];
    __shared__ uint16_t table[PBN][L + 2];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.x * PBM, n0 = (int64_t)blockIdx.y * PBN;
    const int64_t G = K / kGroup, RW = row_words(K, BITS);

    // per-row tables of this block's weight rows (rows past N are clamped: they are never stored)
    for (int i = tid; i < PBN * L; i += 256) {
        const int r = i / L, c = i % L;
        table[r][c] = lut[min(n0 + r, N - 1) * L + c];
    }

    // weight slab: thread -> (row, 32-code half of the K step)
    const int wrow = tid >> 1, whalf = tid & 1;
    const int64_t wn_glob = min(n0 + wrow, N - 1);
    const uint32_t* wsrc = codes + wn_glob * RW;
    // the two output columns this lane owns (one per 32-wide n tile of its wavefront)
    int64_t ncol[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) ncol[j] = min(n0 + wn * 64 + j * 32 + (lane & 31), N - 1);

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int64_t main_steps = K / PBK, tail_steps = (KP + PBK - 1) / PBK;
    for (int64_t step = 0; step < main_steps + tail_steps; ++step) {
        const bool tail = step >= main_steps;            // block-uniform
        const int64_t k0 = (tail ? step - main_steps : step) * PBK;
        // ---- global loads into registers
        uint4 xr[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int idx = p * 256 + tid, r = idx >> 3, c8 = idx & 7;
            const int64_t m = m0 + r, c = k0 + c8 * 8;
            xr[p] = make_uint4(0, 0, 0, 0);
            if (m < M) {
                if (!tail) xr[p] = *reinterpret_cast<const uint4*>(x + m * K + c);
                else if (c < KP) xr[p] = *reinterpret_cast<const uint4*>(xsums + m * KP + c);
            }
        }
        uint32_t q[BITS];
        float sc[2] = {1.f, 1.f};
        if (!tail) {
            const int64_t wbase = ((k0 >> 5) + whalf) * BITS;  // word offset of this thread's 32 codes
#pragma unroll
            for (int i = 0; i < BITS; ++i) q[i] = wsrc[wbase + i];
#pragma unroll
            for (int j = 0; j < 2; ++j) sc[j] = bf16_to_f32(scale[ncol[j] * G + k0 / kGroup]);
        }

        __syncthreads();                                       // previous step's MFMA reads are done (and the tables are written)
        // ---- stage into LDS
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int idx = p * 256 + tid, r = idx >> 3, c8 = idx & 7;
            *reinterpret_cast<uint4*>(&xs[r * PLD + c8 * 8]) = xr[p];
        }
#pragma unroll
        for (int r8 = 0; r8 < 4; ++r8) {
            uint32_t pk[4];
            if (!tail) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int bit = (r8 * 8 + j) * BITS;
                    uint32_t c = q[bit >> 5] >> (bit & 31);
                    if ((bit & 31) + BITS > 32) c |= q[(bit >> 5) + 1] << (32 - (bit & 31));
                    const uint32_t b = table[wrow][c & mask];
                    if (j & 1) pk[j >> 1] |= b << 16; else pk[j >> 1] = b;
                }
            } else {
                // columns c, c+1 of the group dimension both carry offset[n][c/2]
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t g = (k0 + whalf * 32 + r8 * 8 + 2 * j) >> 1;
                    const uint32_t b = g < G ? offset[wn_glob * G + g] : 0u;
                    pk[j] = b | (b << 16);
                }
            }
            *reinterpret_cast<uint4*>(&ws[wrow * PLD + whalf * 32 + r8 * 8]) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
        }
        __syncthreads();
        // ---- matrix cores: partial products of this K step, then one fp32 scale per column
        f32x16 part[2][2];
#pragma unroll
        for (int kk = 0; kk < PBK / 16; ++kk) {
            const int col = kk * 16 + (lane >> 5) * 8;
            bf16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&xs[(wm * 64 + i * 32 + (lane & 31)) * PLD + col]));
                b[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(&ws[(wn * 64 + i * 32 + (lane & 31)) * PLD + col]));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    if (kk == 0) {
                        f32x16 zero;
#pragma unroll
                        for (int v = 0; v < 16; ++v) zero[v] = 0.f;
                        part[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], zero, 0, 0, 0);
                    } else {
                        part[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], part[i][j], 0, 0, 0);
                    }
                }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = __builtin_fmaf(part[i][j][v], sc[j], acc[i][j][v]);
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
    const dim3 grid((unsigned)gm, (unsigned)gn), block(256);
    switch (bits) {
        case 4: hipLaunchKernelGGL(prefill_kernel<4>, grid, block, 0, stream, x, codes, lut, scale, offset, xsums, KP, M, N, K, y); break;
        case 3: hipLaunchKernelGGL(prefill_kernel<3>, grid, block, 0, stream, x, codes, lut, scale, offset, xsums, KP, M, N, K, y); break;
        default: hipLaunchKernelGGL(prefill_kernel<2>, grid, block, 0, stream, x, codes, lut, scale, offset, xsums, KP, M, N, K, y); break;
    }
    return hipGetLastError();
}

}  // namespace any4
