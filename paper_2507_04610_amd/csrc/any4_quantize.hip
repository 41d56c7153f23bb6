// The any-n quantiser: from a weight matrix and per-channel activation statistics to codes,
// per-row lookup tables, group scales and group offsets (any4 paper, section 3.2 "any4
// Algorithm" and appendix, Algorithm 1; scaling equations of section 2.5.1).
//
// Rows are independent, so one block owns one row from start to end and the whole row lives in LDS.
//   1. group-wise scaling: one wavefront per group of 128 weights (two per lane), min / max by
//      wavefront shuffles; alpha, beta are rounded to bf16 first, then w_S = (w - beta) / alpha;
//   2. k-means++ start with the sample weights s = alpha * E|x|: every thread owns a contiguous
//      chunk of the row, chunk masses are scanned across the block, the thread whose chunk holds
//      the drawn point walks it (the uniform draws are an input, one per centre);
//   3. weighted Lloyd iterations in fp64 until a pass changes no code or `iters` centre updates
//      were made, by one of two methods:
//      sorted row (K <= 16384): the scaled row is sorted once (bitonic network, 16 elements per
//        thread in registers, LDS between rounds) and running sums of s and s * w_S are kept per 16
//        sorted elements.  A pass is then the work of 2^n lanes of one wavefront: order the centres,
//        find for each neighbouring pair the first sorted position the upper one wins - a binary
//        search that evaluates the very predicate of the E-step (squared fp64 distances, ties to the
//        lower index) - and take every cluster's sums as differences of running sums: O(2^n log K)
//        instead of O(K 2^n) per pass.  The E-step predicate is monotone along the sorted row as
//        long as unequal centres are further apart than the rounding of the distances; a row in
//        which two unequal centres come closer than `centre_gap * max|w_S|` is finished by the
//        other method from its starting centres;
//      per weight (larger K, and the rows just named): one pass assigns every weight to its nearest
//        centre and at the same time accumulates, per thread and per centre, sum(s * w_S) and
//        sum(s); the partial sums are combined in a fixed order (lanes, then wavefronts);
//      both are reproducible run to run; they differ from each other (and from a sequential sum)
//      only in the association of the fp64 sums;
//   4. the centres are sorted, the codes renumbered and written with 16-byte stores.
// The sample weights are never stored: s = alpha[group] * act[k] is one fp32 multiply.
#include "any4_device.h"
#include "any4_internal.h"
#include <type_traits>
#include <utility>

#pragma clang fp contract(off)

namespace any4 {

constexpr int QT = 256;                 // threads per block of the per-weight kernel (4 wavefronts; several blocks
                                        // share a compute unit: 512 or 1024 threads measured 1.2 - 2.2x slower)

__device__ __forceinline__ double shfl_xor_f64(double v, int mask) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_xor(lo, mask);
    hi = __shfl_xor(hi, mask);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double shfl_up_f64(double v, int delta) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl_up(lo, delta);
    hi = __shfl_up(hi, delta);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double shfl_f64(double v, int src) {
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __shfl(lo, src);
    hi = __shfl(hi, src);
    return __hiloint2double(hi, lo);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// Lane `src` (a constant) of a double, for every lane: two scalar reads, no trip through the LDS pipe.
template <int SRC>
__device__ __forceinline__ double lane_f64(double v) {
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), SRC), __builtin_amdgcn_readlane(__double2loint(v), SRC));
}
// The double `d` lanes down the same row of 16 lanes (0.0 where the row ends): a DPP move per half.
template <int D>
__device__ __forceinline__ double row_shr_f64(double v) {
    return __hiloint2double(__builtin_amdgcn_update_dpp(0, __double2hiint(v), 0x110 + D, 0xF, 0xF, false),
                            __builtin_amdgcn_update_dpp(0, __double2loint(v), 0x110 + D, 0xF, 0xF, false));
}
// Inclusive sum over the 64 lanes: along the rows of 16 by DPP moves, then the three row totals (scalars)
// onto the rows after them.  A fixed order of additions, like every sum here.
__device__ __forceinline__ double wave_inclusive_sum(double v, int lane) {
    v += row_shr_f64<1>(v);
    v += row_shr_f64<2>(v);
    v += row_shr_f64<4>(v);
    v += row_shr_f64<8>(v);
    const double t0 = lane_f64<15>(v), t1 = lane_f64<31>(v), t2 = lane_f64<47>(v);
    const double o2 = t0 + t1, o3 = o2 + t2;
    const int row = lane >> 4;
    const double off = row == 0 ? 0.0 : row == 1 ? t0 : row == 2 ? o2 : o3;
    return v + off;
}
// min / max over the 64 lanes (the same value in every lane): within rows of 16 by DPP, then four scalars
template <bool MAX>
__device__ __forceinline__ float wave_minmax(float v) {
    auto pick = [](float a, float b) { return MAX ? fmaxf(a, b) : fminf(a, b); };
    auto dpp = [](float x, auto ctrl) {
        return __uint_as_float(__builtin_amdgcn_update_dpp(__float_as_uint(x), __float_as_uint(x), decltype(ctrl)::value, 0xF, 0xF, false));
    };
    v = pick(v, dpp(v, std::integral_constant<int, 0xB1>{}));     // lanes 1 0 3 2 of each four
    v = pick(v, dpp(v, std::integral_constant<int, 0x4E>{}));     // lanes 2 3 0 1
    v = pick(v, dpp(v, std::integral_constant<int, 0x141>{}));    // the half row mirrored
    v = pick(v, dpp(v, std::integral_constant<int, 0x140>{}));    // the row mirrored
    const float a = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), 0));
    const float b = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), 16));
    const float c = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), 32));
    const float d = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(v), 48));
    return pick(pick(a, b), pick(c, d));
}

// ---- 1. group-wise scaling (section 2.5.1): scaled row to ws, group scales to alpha (both LDS)
template <int BITS, int T>
__device__ __forceinline__ void scale_row(const float* __restrict__ wrow, int64_t n, int G, int symmetric,
                                          uint16_t* __restrict__ scale, uint16_t* __restrict__ offset,
                                          float* ws, float* alpha, float* beta = nullptr) {
    constexpr int L = 1 << BITS;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const float qrange = symmetric ? (float)((1 << (BITS - 1)) - 1) : (float)(L - 1);
    for (int g = wv; g < G; g += T / kWave) {
        const float2 v = reinterpret_cast<const float2*>(wrow + (int64_t)g * kGroup)[lane];
        const float mn = wave_minmax<false>(fminf(v.x, v.y)), mx = wave_minmax<true>(fmaxf(v.x, v.y));
        const float am = fmaxf(fabsf(mn), fabsf(mx));             // the largest magnitude is at one of the two ends
        const float a32 = symmetric ? am / qrange : (mx - mn) / qrange;
        const float b32 = symmetric ? 0.0f : mn;
        uint32_t ab = f32_to_bf16(a32);
        const uint32_t bb = f32_to_bf16(b32);
        if (bf16_to_f32(ab) == 0.0f) ab = 0x3F80u;                 // constant group: alpha = 1
        const float a = bf16_to_f32(ab), b = bf16_to_f32(bb);
        if (lane == 0) {
            scale[n * G + g] = (uint16_t)ab;
            offset[n * G + g] = (uint16_t)bb;
            alpha[g] = a;
            if (beta) beta[g] = b;
        }
        const float d0 = v.x - b, d1 = v.y - b;
        reinterpret_cast<float2*>(ws + g * kGroup)[lane] = make_float2(d0 / a, d1 / a);
    }
    __syncthreads();
}

template <int BITS, int T>
__device__ __forceinline__ void emit_row_order(const unsigned char* codes, const double* cen, int* misc, int64_t K,
                                               int64_t n, uint8_t* __restrict__ codes_out, uint16_t* __restrict__ lut);

// ---- 3, per weight: Lloyd iterations (E-step: nearest centre; M-step: Eq. (B), weighted mean) over ws in row
// order, then 4: sorted centres, renumbered codes, stores.  cen holds the starting centres.
template <int BITS, int T>
__device__ __forceinline__ void lloyd_per_weight(const float* ws, unsigned char* codes, const float* alpha, double* red,
                                                 double* cen, int* misc, const float* __restrict__ act, int64_t K,
                                                 int iters, int64_t n, uint8_t* __restrict__ codes_out,
                                                 uint16_t* __restrict__ lut, int32_t* __restrict__ msteps) {
    constexpr int L = 1 << BITS;
    constexpr int W = T / kWave;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    auto sample_weight = [&](int j) -> float { return alpha[j >> 7] * (act ? act[j] : 1.0f); };
    for (int j = tid; j < K; j += T) codes[j] = 0xFF;
    int done = 0;
    for (;;) {
        double c[L];
#pragma unroll
        for (int p = 0; p < L; ++p) c[p] = cen[p];
        double num[L], den[L];
#pragma unroll
        for (int p = 0; p < L; ++p) { num[p] = 0.0; den[p] = 0.0; }
        int changed = 0;
#pragma unroll 2                                               // two independent chains of compare / select: 5 % faster
        for (int j = tid; j < K; j += T) {
            const double x = (double)ws[j];
            int best = 0;
            double bd = (x - c[0]) * (x - c[0]);
#pragma unroll
            for (int p = 1; p < L; ++p) {
                const double d = x - c[p];
                const double dd = d * d;
                if (dd < bd) { bd = dd; best = p; }
            }
            changed |= (codes[j] != (unsigned char)best);
            codes[j] = (unsigned char)best;
            const double s = (double)sample_weight(j);
            const double sx = s * x;
            // num[best] += sx, den[best] += s with the accumulators in registers: one fused multiply-add
            // per accumulator with a factor of exactly 1 or 0 (fma(v, 1, a) = a + v rounded once;
            // fma(v, 0, a) = a), cheaper than selecting v or 0 and adding
#pragma unroll
            for (int p = 0; p < L; ++p) {
                const double one = __hiloint2double(best == p ? 0x3FF00000 : 0, 0);
                num[p] = __builtin_fma(sx, one, num[p]);
                den[p] = __builtin_fma(s, one, den[p]);
            }
        }
        changed = __syncthreads_or(changed);
        if ((done > 0 && !changed) || done >= iters) break;
        // combine the partial sums: butterfly over the lanes, then the wavefronts in order
#pragma unroll
        for (int p = 0; p < L; ++p) {
#pragma unroll
            for (int m = 1; m < 64; m <<= 1) {
                num[p] += shfl_xor_f64(num[p], m);
                den[p] += shfl_xor_f64(den[p], m);
            }
        }
        if (lane == 0) {
#pragma unroll
            for (int p = 0; p < L; ++p) { red[(wv * 2 + 0) * L + p] = num[p]; red[(wv * 2 + 1) * L + p] = den[p]; }
        }
        __syncthreads();
        if (tid < L) {
            double a = 0.0, b = 0.0;
            for (int i = 0; i < W; ++i) { a += red[(i * 2 + 0) * L + tid]; b += red[(i * 2 + 1) * L + tid]; }
            if (b > 0.0) cen[tid] = a / b;
        }
        ++done;
        __syncthreads();
    }
    if (msteps && tid == 0) msteps[n] = done;
    emit_row_order<BITS, T>(codes, cen, misc, K, n, codes_out, lut);
}

// The same iterations for the rarely taken hand-over inside the sorted-row kernel, which has 128 registers
// per lane: the E-step and the M-step are separate passes and the M-step takes four centres at a time.
// Every accumulator still adds its weights in the same order, so the sums are the same bit for bit.
template <int BITS, int T>
__device__ __forceinline__ void lloyd_per_weight_lean(const float* ws, unsigned char* codes, const float* alpha, double* red,
                                                   double* cen, int* misc, const float* __restrict__ act, int64_t K,
                                                   int iters, int64_t n, uint8_t* __restrict__ codes_out,
                                                   uint16_t* __restrict__ lut, int32_t* __restrict__ msteps) {
    constexpr int L = 1 << BITS;
    constexpr int W = T / kWave;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    auto sample_weight = [&](int j) -> float { return alpha[j >> 7] * (act ? act[j] : 1.0f); };
    for (int j = tid; j < K; j += T) codes[j] = 0xFF;
    __syncthreads();
    int done = 0;
    for (;;) {
        int changed = 0;
        if (tid == 0) misc[40] = 0;                                // "some code changed in this pass"
        __syncthreads();
#pragma unroll 1
        for (int j = tid; j < K; j += T) {
            const double x = (double)ws[j];
            int best = 0;
            double bd = (x - cen[0]) * (x - cen[0]);
#pragma unroll 1
            for (int p = 1; p < L; ++p) {
                const double d = x - cen[p];
                const double dd = d * d;
                if (dd < bd) { bd = dd; best = p; }
            }
            changed |= (codes[j] != (unsigned char)best);
            codes[j] = (unsigned char)best;
        }
        if (changed) misc[40] = 1;
        __syncthreads();
        changed = misc[40];
        if ((done > 0 && !changed) || done >= iters) break;
#pragma unroll 1
        for (int p0 = 0; p0 < L; p0 += 4) {
            double num[4] = {0.0, 0.0, 0.0, 0.0}, den[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 1
            for (int j = tid; j < K; j += T) {
                const double x = (double)ws[j];
                const int best = (int)codes[j] - p0;
                const double s = (double)sample_weight(j);
                const double sx = s * x;
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const double one = __hiloint2double(best == p ? 0x3FF00000 : 0, 0);
                    num[p] = __builtin_fma(sx, one, num[p]);
                    den[p] = __builtin_fma(s, one, den[p]);
                }
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) {
#pragma unroll
                for (int m = 1; m < 64; m <<= 1) {
                    num[p] += shfl_xor_f64(num[p], m);
                    den[p] += shfl_xor_f64(den[p], m);
                }
            }
            if (lane == 0) {
#pragma unroll
                for (int p = 0; p < 4; ++p) { red[(wv * 2 + 0) * L + p0 + p] = num[p]; red[(wv * 2 + 1) * L + p0 + p] = den[p]; }
            }
        }
        __syncthreads();
        if (tid < L) {
            double a = 0.0, b = 0.0;
#pragma unroll 1
            for (int i = 0; i < W; ++i) { a += red[(i * 2 + 0) * L + tid]; b += red[(i * 2 + 1) * L + tid]; }
            if (b > 0.0) cen[tid] = a / b;
        }
        ++done;
        __syncthreads();
    }
    if (msteps && tid == 0) msteps[n] = done;
    emit_row_order<BITS, T>(codes, cen, misc, K, n, codes_out, lut);
}

// ---- 4, per weight: sort the centres (stable), renumber the codes (LDS, row order), store
template <int BITS, int T>
__device__ __forceinline__ void emit_row_order(const unsigned char* codes, const double* cen, int* misc, int64_t K,
                                               int64_t n, uint8_t* __restrict__ codes_out, uint16_t* __restrict__ lut) {
    constexpr int L = 1 << BITS;
    const int tid = threadIdx.x;
    __syncthreads();
    if (tid == 0) {
        int* order = misc + 1 + L;
        for (int p = 0; p < L; ++p) order[p] = p;
        for (int i = 1; i < L; ++i) {
            const int o = order[i];
            int p = i;
            while (p > 0 && cen[order[p - 1]] > cen[o]) { order[p] = order[p - 1]; --p; }
            order[p] = o;
        }
        for (int r = 0; r < L; ++r) {
            misc[1 + order[r]] = r;
            lut[n * L + r] = (uint16_t)f32_to_bf16((float)cen[order[r]]);
        }
    }
    __syncthreads();
    unsigned long long rank = 0;                                  // rank of centre p in nibble p
    for (int p = 0; p < L; ++p) rank |= (unsigned long long)misc[1 + p] << (4 * p);
    uint8_t* crow = codes_out + n * K;
    for (int j = tid * 16; j < K; j += T * 16) {
        uint4 v = *reinterpret_cast<const uint4*>(codes + j);
        uint32_t in[4] = {v.x, v.y, v.z, v.w}, out[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t o = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const uint32_t code = (in[i] >> (8 * b)) & 0xFFu;
                o |= (uint32_t)((rank >> (4 * code)) & 0xFull) << (8 * b);
            }
            out[i] = o;
        }
        *reinterpret_cast<uint4*>(crow + j) = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

// =====================================================================================================
// The per-weight kernel (any K up to the LDS limit).
// LDS of one block: ws [K] f32 | codes [K] u8 | alpha [K/128] f32 (padded to 16 B) | scan [W] f64 |
// red [W][2][L] f64 | cen [L] f64 | misc [64] i32
constexpr size_t quantize_small_offset(int64_t K) {
    return ((size_t)K * 5 + (size_t)(K / kGroup) * 4 + 15) & ~(size_t)15;
}
constexpr size_t quantize_lds_bytes(int64_t K, int bits) {
    return quantize_small_offset(K) + (size_t)(QT / kWave) * 8 + (size_t)(QT / kWave) * 2 * (1 << bits) * 8 +
           (size_t)(1 << bits) * 8 + 64 * 4;
}

template <int BITS>
__global__ __launch_bounds__(QT) void quantize_kernel(
    const float* __restrict__ w, const float* __restrict__ act, const float* __restrict__ u,
    int64_t K, int symmetric, int iters, uint8_t* __restrict__ codes_out, uint16_t* __restrict__ lut,
    uint16_t* __restrict__ scale, uint16_t* __restrict__ offset, int32_t* __restrict__ msteps) {
    constexpr int L = 1 << BITS;
    constexpr int QW = QT / kWave;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int G = (int)(K / kGroup);
    float* ws = reinterpret_cast<float*>(smem);
    unsigned char* codes = smem + (size_t)K * 4;
    float* alpha = reinterpret_cast<float*>(smem + (size_t)K * 5);
    double* scan = reinterpret_cast<double*>(smem + quantize_small_offset(K));     // [QW]
    double* red = scan + QW;                     // [QW][2][L]
    double* cen = red + QW * 2 * L;              // [L]
    int* misc = reinterpret_cast<int*>(cen + L); // [0] selected index, [1 .. L] rank of a centre, [1 + L .. 2L] sort order

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t n = blockIdx.x;
    scale_row<BITS, QT>(w + n * K, n, G, symmetric, scale, offset, ws, alpha);

    auto sample_weight = [&](int j) -> float { return alpha[j >> 7] * (act ? act[j] : 1.0f); };

    // ---- 2. k-means++ with sample weights; thread t owns the chunk [t * C, (t + 1) * C)
    const int C = (int)((K + QT - 1) / QT);
    const int j0 = min(tid * C, (int)K), j1 = min(j0 + C, (int)K);
    for (int q = 0; q < L; ++q) {
        // mass of a sample: s for the first centre, s * (squared distance to the nearest chosen centre) after
        auto mass = [&](int j) -> double {
            const double s = (double)sample_weight(j);
            if (q == 0) return s;
            const double x = (double)ws[j];
            double best = (x - cen[0]) * (x - cen[0]);
            for (int p = 1; p < q; ++p) {
                const double d = x - cen[p];
                const double dd = d * d;
                if (dd < best) best = dd;
            }
            return s * best;
        };
        double part = 0.0;
        for (int j = j0; j < j1; ++j) part += mass(j);
        // inclusive scan of the chunk masses over the block: lanes, then wavefronts
        double inc = part;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const double o = shfl_up_f64(inc, d);
            if (lane >= d) inc += o;
        }
        if (lane == 63) scan[wv] = inc;
        __syncthreads();
        double base = 0.0;
        for (int i = 0; i < wv; ++i) base += scan[i];
        double total = 0.0;
        for (int i = 0; i < QW; ++i) total += scan[i];
        inc += base;
        // running mass at the end of the previous chunk: the neighbour's own value, so that the
        // chunks' intervals [before, inc) tile [0, total) without gaps
        double before = shfl_up_f64(inc, 1);
        if (lane == 0) before = base;
        if (tid == 0) misc[0] = 0x7FFFFFFF;
        __syncthreads();
        if (total > 0.0) {
            const double t = (double)u[n * L + q] * total;
            // the first chunk whose running mass exceeds t holds the drawn sample
            if (before <= t && inc > t && j0 < j1) {
                double run = before;
                int pick = -1, lastpos = j0;
                for (int j = j0; j < j1; ++j) {
                    const double m = mass(j);
                    run += m;
                    if (m > 0.0) lastpos = j;
                    if (run > t) { pick = j; break; }
                }
                atomicMin(&misc[0], pick >= 0 ? pick : lastpos);
            }
        } else if (tid == 0) {
            int64_t j = (int64_t)((double)u[n * L + q] * (double)K);
            misc[0] = (int)min(j, K - 1);
        }
        __syncthreads();
        int sel = misc[0];
        if (sel >= K) sel = (int)K - 1;       // not reachable with finite, non-negative masses
        if (tid == 0) cen[q] = (double)ws[sel];
        __syncthreads();
    }

    lloyd_per_weight<BITS, QT>(ws, codes, alpha, red, cen, misc, act, K, iters, n, codes_out, lut, msteps);
}

// =====================================================================================================
// The sorted-row kernel.  T threads sort KP = 16 T elements (K <= KP; the tail is padding that sorts last).
//
// LDS of one block (PADW = KP + KP / 16 elements: one spare element after every 16 keeps all three access
// patterns of the sort - 16 neighbours per thread, strides of 16, strides of 256 - off each other's banks):
//   kv [PADW] u32 x 2   the row's scaled weights (fp32, row order, in the first 4 K bytes) until the sort; then
//                       the elements (order-preserving integer image of w_S, sample weight s as fp32 bits),
//                       ascending in w_S.  (The per-weight method keeps its codes behind the scaled weights.)
//   alpha, beta [KP/128] f32 | pre_s, pre_sx [T + 1] f64 (running sums before every 16th sorted element; the total)
//   scan [2 W] f64 | cen [L] f64 | cen0 [L] f64 | fin [L] u32 | misc [64] i32
//   (the per-weight method's partial sums red [W][2][L] f64 lie over pre_s: 2 W L <= 2 (T + 1))
constexpr int kSortedMaxK = 16384;
constexpr size_t sorted_padw(int T) { return (size_t)T * 17; }
constexpr size_t sorted_lds_bytes(int T, int bits) {
    const size_t W = (size_t)T / kWave, L = (size_t)1 << bits;
    return sorted_padw(T) * 8 + 2 * ((size_t)T / 8) * 4 + 2 * ((size_t)T + 1) * 8 + 2 * W * 8 + 2 * L * 8 + L * 4 + 64 * 4;
}

__device__ __forceinline__ int pad16(int p) { return p + (p >> 4); }
// fp32 -> u32 whose unsigned order is the order of the numbers (finite inputs), and back
__device__ __forceinline__ uint32_t f32_key(float f) {
    const uint32_t b = __float_as_uint(f);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}
__device__ __forceinline__ float key_f32(uint32_t k) {
    return __uint_as_float(k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu));
}
constexpr uint32_t kPadKey = 0xFFFFFFFFu;         // sorts after every number; its sample weight is 0

// Compare-exchange of two elements (key, sample weight): the smaller key goes to the first.
// (The empty asm statement keeps the two sample weights plain values: left alone, the compiler turns
// "one or the other element of the array" into an element picked by a computed index, which costs a
// chain of 16 selects per compare-exchange.)
__device__ __forceinline__ void compare_exchange(uint32_t& k1, uint32_t& s1, uint32_t& k2, uint32_t& s2) {
    uint32_t a = s1, b = s2;
    asm("" : "+v"(a), "+v"(b));
    const bool sw = k1 > k2;
    const uint32_t ka = min(k1, k2), kb = max(k1, k2);
    s1 = sw ? b : a;
    s2 = sw ? a : b;
    k1 = ka;
    k2 = kb;
}

// The first four merge sizes (2 .. 16) of the bitonic network stay inside the 16 neighbouring elements
// of a thread: one trip through LDS.  Up to size 8 the direction of a pair is a bit of its place among
// the 16 (known when compiling: descending = the roles swapped); for size 16 it is the thread's parity.
template <int T>
__device__ __forceinline__ void sort_first16(uint2* kv) {
    int base = threadIdx.x * 17;
    asm volatile("" : "+v"(base));
    uint32_t kk[16], ss[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uint2 v = kv[base + r];
        kk[r] = v.x;
        ss[r] = v.y;
    }
#pragma unroll
    for (int m = 1; m <= 4; ++m) {
        const uint32_t flip = m == 4 ? (uint32_t)(-(int)(threadIdx.x & 1)) : 0u;
        if (m == 4) {
#pragma unroll
            for (int r = 0; r < 16; ++r) kk[r] ^= flip;
        }
#pragma unroll
        for (int b = m - 1; b >= 0; --b) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if ((r & (1 << b)) != 0) continue;
                const int r2 = r | (1 << b);
                if (m < 4 && ((r >> m) & 1)) compare_exchange(kk[r2], ss[r2], kk[r], ss[r]);
                else compare_exchange(kk[r], ss[r], kk[r2], ss[r2]);
            }
        }
        if (m == 4) {
#pragma unroll
            for (int r = 0; r < 16; ++r) kk[r] ^= flip;
        }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) kv[base + r] = make_uint2(kk[r], ss[r]);
    __syncthreads();
}

// One round of the bitonic network on the 16 elements a thread holds: the elements differ in bits
// WB .. WB + NB - 1 of their position (16 / 2^NB independent groups per thread); the round runs the
// compare-exchange stages of merge size 2^m (m > top) for the strides 2^top .. 2^WB.  Pairs that sort
// descending (bit m of the position set) have their keys complemented on the way in and out, so that every
// compare-exchange is the same ascending one.  With the spare element after every 16, the 2^NB elements
// of a group lie a fixed distance apart.
template <int T, int WB, int NB>
__device__ __forceinline__ void sort_round(uint2* kv, int m, int top) {
    constexpr int E = 1 << NB, GROUPS = 16 / E;
    constexpr int STRIDE = WB >= 4 ? (1 << WB) + (1 << (WB >= 4 ? WB - 4 : 0)) : 1;
    // (the empty asm statement ties the addresses to this call: computed once for all calls, outside the
    // loop over the merge sizes, they would hold registers through the whole sort)
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const bool inside = m < WB + NB;                   // the direction bit is one of the bits the 2^NB elements differ in
    uint32_t kk[16], ss[16], flip[16];
    int base[GROUPS];
#pragma unroll
    for (int g = 0; g < GROUPS; ++g) {
        const int low = g * T + tid;
        const int pos0 = ((low >> WB) << (WB + NB)) | (low & ((1 << WB) - 1));
        base[g] = pos0 + (pos0 >> 4);
        const uint32_t gflip = inside ? 0u : (uint32_t)(-(int)(((uint32_t)low >> (m - NB)) & 1u));
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int r = g * E + e;
            const uint32_t eflip = inside ? (uint32_t)(-(int)(((uint32_t)e >> (m - WB)) & 1u)) : 0u;   // the same in all lanes
            flip[r] = gflip | eflip;
            const uint2 v = kv[base[g] + e * STRIDE];
            kk[r] = v.x ^ flip[r];
            ss[r] = v.y;
        }
    }
#pragma unroll
    for (int b = NB - 1; b >= 0; --b) {
        if (WB + b > top) continue;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            if ((r & (1 << b)) != 0) continue;
            const int r2 = r | (1 << b);
            compare_exchange(kk[r], ss[r], kk[r2], ss[r2]);
        }
    }
#pragma unroll
    for (int g = 0; g < GROUPS; ++g)
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const int r = g * E + e;
            kv[base[g] + e * STRIDE] = make_uint2(kk[r] ^ flip[r], ss[r]);
        }
    __syncthreads();
}

template <int BITS, int T>
__global__ __launch_bounds__(T, 4) void quantize_sorted_kernel(
    const float* __restrict__ w, const float* __restrict__ act, const float* __restrict__ u,
    int64_t K64, int symmetric, int iters, double centre_gap, uint8_t* __restrict__ codes_out,
    uint16_t* __restrict__ lut, uint16_t* __restrict__ scale, uint16_t* __restrict__ offset,
    int32_t* __restrict__ msteps) {
    constexpr int L = 1 << BITS;
    constexpr int W = T / kWave;
    constexpr int LOGKP = T == 256 ? 12 : T == 512 ? 13 : 14;
    static_assert(T == 256 || T == 512 || T == 1024, "16 elements per thread, 4096 to 16384 per block");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int K = (int)K64, G = K / kGroup;
    uint2* kv = reinterpret_cast<uint2*>(smem);
    float* ws = reinterpret_cast<float*>(smem);
    float* alpha = reinterpret_cast<float*>(smem + sorted_padw(T) * 8);
    float* beta = alpha + T / 8;
    double* pre_s = reinterpret_cast<double*>(beta + T / 8);   // [T + 1]
    double* pre_sx = pre_s + T + 1;             // [T + 1]
    double* scan = pre_sx + T + 1;              // [2 W]
    double* red = pre_s;                        // [W][2][L], per-weight method only: it has no running sums
    double* cen = scan + 2 * W;                 // [L]
    double* cen0 = cen + L;                     // [L]
    uint32_t* fin = reinterpret_cast<uint32_t*>(cen0 + L);   // [L] smallest key of the cluster of rank i (none: kPadKey)
    int* misc = reinterpret_cast<int*>(fin + L);// [0], [1] selected index (by turns); [2] method flag; [40] as below

    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t n = blockIdx.x;
    scale_row<BITS, T>(w + n * K64, n, G, symmetric, scale, offset, ws, alpha, beta);

    auto sample_weight = [&](int j) -> float { return alpha[j >> 7] * (act ? act[j] : 1.0f); };

    // ---- 2. k-means++ with sample weights; thread t owns the chunk [t * C, (t + 1) * C), C <= 16, in registers:
    // the scaled weight, the sample weight s and the sampling mass.  The mass is s for the first centre and
    // s * (squared distance to the nearest centre chosen so far) afterwards; as s >= 0, multiplying by s and
    // rounding is monotone, so s * min(d_old, d_new) is min(s * d_old, s * d_new) bit for bit and the
    // distances themselves need not be kept.
    {
        const int C = (K + T - 1) / T;
        const int j0 = min(tid * C, K), cnt = min(j0 + C, K) - j0;
        float xv[16], sv[16];
        double mass[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const bool in = e < cnt;
            xv[e] = in ? ws[j0 + e] : 0.0f;
            sv[e] = in ? sample_weight(j0 + e) : 0.0f;            // outside the chunk: mass +0, which changes no sum
            mass[e] = (double)sv[e];
        }
#pragma unroll 1
        for (int q = 0; q < L; ++q) {
            double part = 0.0;
#pragma unroll
            for (int e = 0; e < 16; ++e) part += mass[e];
            double inc = wave_inclusive_sum(part, lane);
            if (lane == 63) scan[(q & 1) * W + wv] = inc;          // (two sets of partial sums and of the selected
            if (tid == 0) misc[q & 1] = 0x7FFFFFFF;                // index, used by turns: one barrier less per centre)
            __syncthreads();
            double base = 0.0, total = 0.0;
#pragma unroll 1
            for (int i = 0; i < W; ++i) {
                if (i == wv) base = total;
                total += scan[(q & 1) * W + i];
            }
            inc += base;
            double before = shfl_up_f64(inc, 1);
            if (lane == 0) before = base;
            if (total > 0.0) {
                const double t = (double)u[n * L + q] * total;
                if (before <= t && inc > t && cnt > 0) {
                    double run = before;
                    int pick = -1, lastpos = j0;
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        run += mass[e];
                        if (e < cnt && pick < 0) {
                            if (mass[e] > 0.0) lastpos = j0 + e;
                            if (run > t) pick = j0 + e;
                        }
                    }
                    atomicMin(&misc[q & 1], pick >= 0 ? pick : lastpos);
                }
            } else if (tid == 0) {
                int64_t j = (int64_t)((double)u[n * L + q] * (double)K);
                misc[q & 1] = (int)min(j, (int64_t)K - 1);
            }
            __syncthreads();
            int sel = misc[q & 1];
            if (sel >= K) sel = K - 1;            // not reachable with finite, non-negative masses
            const double cq = (double)ws[sel];
            if (tid == 0) { cen[q] = cq; cen0[q] = cq; }
            // (the empty asm statements keep the fp32 -> fp64 conversions inside the loop over q: hoisted,
            // they would hold 64 more registers for the whole start)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float xe = xv[e], se = sv[e];
                asm volatile("" : "+v"(xe), "+v"(se));
                const double d = (double)xe - cq;
                const double sd = (double)se * (d * d);
                if (q == 0 || sd < mass[e]) mass[e] = sd;
            }
        }
    }

    // ---- sort the row: elements (order-preserving image of w_S, sample weight), ascending in w_S
    {
        uint32_t k0[16], s0[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int j = tid * 16 + e;
            k0[e] = j < K ? f32_key(ws[j]) : kPadKey;
            s0[e] = j < K ? __float_as_uint(sample_weight(j)) : 0u;
        }
        __syncthreads();                                           // every thread has read its part of ws
#pragma unroll
        for (int e = 0; e < 16; ++e) kv[pad16(tid * 16 + e)] = make_uint2(k0[e], s0[e]);
        __syncthreads();
        sort_first16<T>(kv);
        for (int m = 5; m <= LOGKP; ++m) {
            const int top = m - 1;
            if constexpr (LOGKP > 12) {
                if (top >= 12) sort_round<T, 12, LOGKP - 12>(kv, m, top);
            }
            if (top >= 8) sort_round<T, 8, 4>(kv, m, min(top, 11));
            if (top >= 4) sort_round<T, 4, 4>(kv, m, min(top, 7));
            sort_round<T, 0, 4>(kv, m, min(top, 3));
        }
    }

    // one sorted element: its scaled weight and sample weight in fp64 (the padding counts as nothing)
    auto element = [&](int p, double& x, double& sw) {
        const uint2 v = kv[pad16(p)];
        const bool real = v.x != kPadKey;
        x = real ? (double)key_f32(v.x) : 0.0;
        sw = real ? (double)__uint_as_float(v.y) : 0.0;
    };

    // ---- running sums of s and s * w_S along the sorted row, one entry per 16 elements
    {
        double cs = 0.0, csx = 0.0;
        int t16 = tid * 16;
        asm volatile("" : "+v"(t16));
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            double x, sw;
            element(t16 + e, x, sw);
            cs += sw;
            csx += sw * x;
        }
        double is = wave_inclusive_sum(cs, lane), isx = wave_inclusive_sum(csx, lane);
        if (lane == 63) { scan[2 * wv] = is; scan[2 * wv + 1] = isx; }
        __syncthreads();
        double bs = 0.0, bsx = 0.0;
#pragma unroll 1
        for (int i = 0; i < wv; ++i) { bs += scan[2 * i]; bsx += scan[2 * i + 1]; }
        is += bs;
        isx += bsx;
        double es = shfl_up_f64(is, 1), esx = shfl_up_f64(isx, 1);
        if (lane == 0) { es = bs; esx = bsx; }
        pre_s[tid] = es;
        pre_sx[tid] = esx;
        if (tid == T - 1) { pre_s[T] = is; pre_sx[T] = isx; }
        __syncthreads();
    }
    // ---- 3, sorted row: the Lloyd passes on wavefront 0, four lanes per centre (lane = 4 q + sub: the four
    // hold the same centre and split the searches and the partial sums).  Lanes 4 q .. 4 q + 3 hold centre q;
    // after ordering, lanes 4 i .. 4 i + 3 also hold the centre of rank i: value d, index own, range [start, end).
    if (wv == 0) {
        const int q4 = lane >> 2, sub = lane & 3, lane4 = lane & ~3;
        const bool live = q4 < L;
        double c = live ? cen[q4] : 0.0;
        const double maxabs = fmax(fabs((double)key_f32(kv[0].x)), fabs((double)key_f32(kv[pad16(K - 1)].x)));
        const double tol = centre_gap * maxabs;
        int prev_s = -2, prev_e = -2;                              // range of centre q in the previous pass
        int done = 0;
        bool fallback = false;
        double d = 0.0;
        int start = 0, end = 0;
        bool rep = false, ranked = false;
        int r = 0;
        // sum over the four lanes of a centre: two DPP moves inside the group of four per half
        auto quad_sum = [](double v) {
            v += __hiloint2double(__builtin_amdgcn_update_dpp(0, __double2hiint(v), 0xB1, 0xF, 0xF, false),
                                  __builtin_amdgcn_update_dpp(0, __double2loint(v), 0xB1, 0xF, 0xF, false));
            v += __hiloint2double(__builtin_amdgcn_update_dpp(0, __double2hiint(v), 0x4E, 0xF, 0xF, false),
                                  __builtin_amdgcn_update_dpp(0, __double2loint(v), 0x4E, 0xF, 0xF, false));
            return v;
        };
        for (;;) {
            // order the centres by (value, index): rank r of centre q; the lanes of rank i take that centre.
            // The order of the last pass is tried first (one permutation and a comparison of neighbours; the
            // centres of a one-dimensional k-means hardly ever overtake each other) and the ranks counted anew,
            // 2^n comparisons per centre, only if it no longer holds.
            int own = 0;
            for (int attempt = ranked ? 0 : 1; attempt < 2; ++attempt) {
                if (attempt == 1) {
                    r = 0;
                    static_for<L>([&](auto p_) {
                        constexpr int p = decltype(p_)::value;
                        const double cp = lane_f64<4 * p>(c);
                        r += (cp < c || (cp == c && p < q4)) ? 1 : 0;
                    });
                }
                const int to = ((live ? r : q4) * 4 + sub) * 4;    // the ranks are a permutation of the live centres
                d = __hiloint2double(__builtin_amdgcn_ds_permute(to, __double2hiint(c)),
                                     __builtin_amdgcn_ds_permute(to, __double2loint(c)));
                own = __builtin_amdgcn_ds_permute(to, q4);
                if (attempt == 1) break;
                const double below_d = shfl_up_f64(d, 4);
                const int below_own = __shfl_up(own, 4);
                const bool in_order = !live || q4 == 0 || below_d < d || (below_d == d && below_own < own);
                if (__ballot(!in_order) == 0ull) break;
            }
            ranked = true;
            // equal centres: only the lowest index ever wins a weight; it stands for the run
            const double dprev = shfl_up_f64(d, 4);
            rep = live && (q4 == 0 || dprev != d);
            const unsigned long long repmask = __ballot(rep && sub == 0);
            const unsigned long long below = repmask & ((1ull << lane4) - 1ull);
            const int prv = below ? 63 - __clzll(below) : 0;       // the previous run's first lane
            const int a_own = __shfl(own, prv);
            bool bad = rep && q4 > 0 && (d - dprev) <= tol;
            // first sorted position at which this centre beats the one below it (the E-step's own comparison, which
            // is false up to that position and true from it on): each round the four lanes probe the four
            // inner fifths of the open range
            int lo = 0, hi = (rep && q4 > 0) ? K : 0;              // the answer lies in [lo, hi]
            while (__ballot(lo < hi) != 0ull) {
                const int span = hi - lo;
                const int probe = lo + (span * (sub + 1)) / 5;     // lo <= probe < hi while the range is open
                const double x = (double)key_f32(kv[pad16(min(probe, K - 1))].x);
                const double da = x - dprev, db = x - d;
                const double dda = da * da, ddb = db * db;
                const bool win = ddb < dda || (ddb == dda && own < a_own);
                const int losses = __popc((unsigned)(__ballot(!win) >> lane4) & 15u);   // 0 .. 4, the first ones
                if (lo < hi) {
                    const int lo2 = losses > 0 ? lo + (span * losses) / 5 + 1 : lo;
                    const int hi2 = losses < 4 ? lo + (span * (losses + 1)) / 5 : hi;
                    lo = lo2;
                    hi = hi2;
                }
            }
            start = lo;
            // running sums before that position: the entry of its group of 16, then the group's first elements,
            // four apart per lane
            double ss = 0.0, sx = 0.0;
            {
                const int chunk = start >> 4, nrem = start & 15;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int e = sub + 4 * i;
                    double x, sw;
                    element(min(chunk * 16 + e, K - 1), x, sw);
                    if (e < nrem) { ss += sw; sx += sw * x; }
                }
                ss = quad_sum(ss) + pre_s[chunk];
                sx = quad_sum(sx) + pre_sx[chunk];
            }
            const unsigned long long above = lane4 >= 60 ? 0ull : (repmask & ~((1ull << (lane4 + 4)) - 1ull));
            const int nxt = above ? __ffsll((long long)above) - 1 : -1;
            const int s_nxt = __shfl(start, nxt < 0 ? 0 : nxt);
            end = nxt < 0 ? K : s_nxt;
            bad = bad || (rep && end < start);
            const double e_ss = shfl_f64(ss, nxt < 0 ? 0 : nxt), e_sx = shfl_f64(sx, nxt < 0 ? 0 : nxt);
            const double den = (nxt < 0 ? pre_s[K >> 4] : e_ss) - ss;   // K is a multiple of 16: the sums before position K
            const double num = (nxt < 0 ? pre_sx[K >> 4] : e_sx) - sx;
            double cn = d;
            if (rep && den > 0.0) cn = num / den;                   // M-step, Eq. (B); no weight: the centre stays
            // did any weight change its centre?  compare every centre's range with the previous pass
            const bool some = rep && start < end;
            const int rs = some ? start : -1, re = some ? end : -1;
            const int qs = __shfl(rs, r * 4), qe = __shfl(re, r * 4);
            const bool changed = __ballot(live && (qs != prev_s || qe != prev_e)) != 0ull;
            if (__ballot(bad) != 0ull) { fallback = true; break; }
            if ((done > 0 && !changed) || done >= iters) break;
            prev_s = qs;
            prev_e = qe;
            c = shfl_f64(cn, r * 4);
            ++done;
        }
        if (lane == 0) misc[2] = fallback ? 1 : 0;
        if (!fallback) {
            // ---- 4. lanes 4 i hold the centre of rank i: table entry i, and code i for every weight from the
            // first of its range up to the first of the next non-empty range
            if (live && sub == 0) {
                lut[n * L + q4] = (uint16_t)f32_to_bf16((float)d);
                fin[q4] = (rep && start < end) ? kv[pad16(start)].x : kPadKey;
            }
            if (msteps && lane == 0) msteps[n] = done;
        }
    }
    __syncthreads();
    if (misc[2] != 0) {
        // two unequal centres too close for the sorted search: the row again, per weight, from its starting centres
        __syncthreads();
        scale_row<BITS, T>(w + n * K64, n, G, symmetric, scale, offset, ws, alpha, beta);
        if (tid < L) cen[tid] = cen0[tid];
        __syncthreads();
        lloyd_per_weight_lean<BITS, T>(ws, smem + (size_t)K * 4, alpha, red, cen, misc, act, K64, iters, n, codes_out, lut,
                                       msteps);
        return;
    }
    // the codes in row order: scale the row again (the same arithmetic as in step 1) and place every weight
    // among the clusters' smallest members; a cluster never splits equal weights, so this is its range
    {
        uint32_t fk[L];
#pragma unroll
        for (int i = 0; i < L; ++i) fk[i] = fin[i];
        const float* wrow = w + n * K64;
        uint8_t* crow = codes_out + n * K64;
        for (int j = tid * 16; j < K; j += T * 16) {
            const float a = alpha[j >> 7], b = beta[j >> 7];
            uint32_t out[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float4 v = *reinterpret_cast<const float4*>(wrow + j + 4 * i);
                const float f[4] = {v.x, v.y, v.z, v.w};
                uint32_t o = 0;
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const float dlt = f[t] - b;
                    const uint32_t key = f32_key(dlt / a);
                    uint32_t code = 0;
#pragma unroll
                    for (int q = 1; q < L; ++q) code = key >= fk[q] ? q : code;
                    o |= code << (8 * t);
                }
                out[i] = o;
            }
            *reinterpret_cast<uint4*>(crow + j) = make_uint4(out[0], out[1], out[2], out[3]);
        }
    }
}

size_t quantize_max_k() {
    // the row, its codes and the scratch have to fit the 160 KB of LDS of one compute unit
    return 28672;
}

hipError_t launch_quantize(const float* w, const float* act, const float* u, int64_t N, int64_t K, int bits,
                           int symmetric, int iters, double centre_gap, uint8_t* codes, uint16_t* lut, uint16_t* scale,
                           uint16_t* offset, int32_t* msteps, hipStream_t stream) {
    if (N > 0x7FFFFFFF || K > (int64_t)quantize_max_k()) return hipErrorInvalidValue;
    hipError_t e = hipSuccess;
    if (centre_gap >= 0.0 && K <= kSortedMaxK) {
#define ANY4_QUANT_S(B, T)                                                                                        \
    do {                                                                                                          \
        e = ensure_lds<quantize_sorted_kernel<B, T>>((int)sorted_lds_bytes(T, B));                                \
        if (e != hipSuccess) return e;                                                                            \
        hipLaunchKernelGGL((quantize_sorted_kernel<B, T>), dim3((unsigned)N), dim3(T), sorted_lds_bytes(T, B), stream, w, \
                           act, u, K, symmetric, iters, centre_gap, codes, lut, scale, offset, msteps);           \
    } while (0)
#define ANY4_QUANT_ST(B)                                                                                          \
    do {                                                                                                          \
        if (K <= 4096) ANY4_QUANT_S(B, 256);                                                                      \
        else if (K <= 8192) ANY4_QUANT_S(B, 512);                                                                 \
        else ANY4_QUANT_S(B, 1024);                                                                               \
    } while (0)
        switch (bits) {
            case 4: ANY4_QUANT_ST(4); break;
            case 3: ANY4_QUANT_ST(3); break;
            default: ANY4_QUANT_ST(2); break;
        }
#undef ANY4_QUANT_ST
#undef ANY4_QUANT_S
        return hipGetLastError();
    }
    const size_t lds = quantize_lds_bytes(K, bits);
#define ANY4_QUANT(B)                                                                                             \
    do {                                                                                                          \
        e = ensure_lds<quantize_kernel<B>>((int)quantize_lds_bytes((int64_t)quantize_max_k(), B));                \
        if (e != hipSuccess) return e;                                                                            \
        hipLaunchKernelGGL(quantize_kernel<B>, dim3((unsigned)N), dim3(QT), lds, stream, w, act, u, K, symmetric, \
                           iters, codes, lut, scale, offset, msteps);                                             \
    } while (0)
    switch (bits) {
        case 4: ANY4_QUANT(4); break;
        case 3: ANY4_QUANT(3); break;
        default: ANY4_QUANT(2); break;
    }
#undef ANY4_QUANT
    return hipGetLastError();
}

}  // namespace any4
