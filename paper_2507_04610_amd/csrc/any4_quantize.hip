// The any-n quantiser: from a weight matrix and per-channel activation statistics to codes,
// per-row lookup tables, group scales and group offsets (any4 paper, section 3.2 "any4
// Algorithm" and appendix, Algorithm 1; scaling equations of section 2.5.1).
//
// Rows are independent, so one block of 256 threads owns one row from start to end and the whole
// row lives in LDS (fp32 scaled weights, one byte of code per weight, the group scales):
//   1. group-wise scaling: one wavefront per group of 128 weights (two per lane), min / max by
//      wavefront shuffles; alpha, beta are rounded to bf16 first, then w_S = (w - beta) / alpha;
//   2. k-means++ start with the sample weights s = alpha * E|x|: every thread owns a contiguous
//      chunk of the row, chunk masses are scanned across the block, the thread whose chunk holds
//      the drawn point walks it (the uniform draws are an input, one per centre);
//   3. weighted Lloyd iterations in fp64: one pass assigns every weight to its nearest centre and
//      at the same time accumulates, per thread and per centre, sum(s * w_S) and sum(s); the
//      partial sums are combined in a fixed order (lanes, then wavefronts), so a run is
//      reproducible; the loop ends when a pass changes no code or after `iters` centre updates;
//   4. the centres are sorted, the codes renumbered and written with 16-byte stores.
// The sample weights are never stored: s = alpha[group] * act[k] is one fp32 multiply.
#include "any4_device.h"
#include "any4_internal.h"

#pragma clang fp contract(off)

namespace any4 {

constexpr int QT = 256;                 // threads per block (4 wavefronts; several blocks share a compute unit:
                                        // blocks of 512 or 1024 threads measured 1.2 - 2.2x slower)
constexpr int QW = QT / kWave;

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

// LDS of one block: ws [K] f32 | codes [K] u8 | alpha [K/128] f32 (padded to 16 B) | scan [QW] f64 |
// red [QW][2][L] f64 | cen [L] f64 | misc [64] i32
constexpr size_t quantize_small_offset(int64_t K) {
    return ((size_t)K * 5 + (size_t)(K / kGroup) * 4 + 15) & ~(size_t)15;
}
constexpr size_t quantize_lds_bytes(int64_t K, int bits) {
    return quantize_small_offset(K) + (size_t)QW * 8 + (size_t)QW * 2 * (1 << bits) * 8 + (size_t)(1 << bits) * 8 + 64 * 4;
}

template <int BITS>
__global__ __launch_bounds__(QT) void quantize_kernel(
    const float* __restrict__ w, const float* __restrict__ act, const float* __restrict__ u,
    int64_t K, int symmetric, int iters, uint8_t* __restrict__ codes_out, uint16_t* __restrict__ lut,
    uint16_t* __restrict__ scale, uint16_t* __restrict__ offset, int32_t* __restrict__ msteps) {
    constexpr int L = 1 << BITS;
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
    const float* wrow = w + n * K;

    // ---- 1. group-wise scaling (section 2.5.1)
    const float qrange = symmetric ? (float)((1 << (BITS - 1)) - 1) : (float)(L - 1);
    for (int g = wv; g < G; g += QW) {
        const float2 v = reinterpret_cast<const float2*>(wrow + (int64_t)g * kGroup)[lane];
        float mn = fminf(v.x, v.y), mx = fmaxf(v.x, v.y), am = fmaxf(fabsf(v.x), fabsf(v.y));
#pragma unroll
        for (int m = 1; m < 64; m <<= 1) {
            mn = fminf(mn, __shfl_xor(mn, m));
            mx = fmaxf(mx, __shfl_xor(mx, m));
            am = fmaxf(am, __shfl_xor(am, m));
        }
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
        }
        const float d0 = v.x - b, d1 = v.y - b;
        reinterpret_cast<float2*>(ws + g * kGroup)[lane] = make_float2(d0 / a, d1 / a);
    }
    __syncthreads();

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

    // ---- 3. Lloyd iterations (E-step: nearest centre; M-step: Eq. (B), weighted mean)
    for (int j = tid; j < K; j += QT) codes[j] = 0xFF;
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
        for (int j = tid; j < K; j += QT) {
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
            for (int i = 0; i < QW; ++i) { a += red[(i * 2 + 0) * L + tid]; b += red[(i * 2 + 1) * L + tid]; }
            if (b > 0.0) cen[tid] = a / b;
        }
        ++done;
        __syncthreads();
    }
    if (msteps && tid == 0) msteps[n] = done;

    // ---- 4. sort the centres (stable), renumber the codes, store
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
    for (int j = tid * 16; j < K; j += QT * 16) {
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

size_t quantize_max_k() {
    // the row, its codes and the scratch have to fit the 160 KB of LDS of one compute unit
    return 28672;
}

hipError_t launch_quantize(const float* w, const float* act, const float* u, int64_t N, int64_t K, int bits,
                           int symmetric, int iters, uint8_t* codes, uint16_t* lut, uint16_t* scale,
                           uint16_t* offset, int32_t* msteps, hipStream_t stream) {
    if (N > 0x7FFFFFFF || K > (int64_t)quantize_max_k()) return hipErrorInvalidValue;
    const size_t lds = quantize_lds_bytes(K, bits);
    hipError_t e = hipSuccess;
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
