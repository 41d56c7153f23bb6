// Memory-bound any4 GEMV (M = 1, single-token generation): one lane per weight row.
//
// y[n] = sum_k x[k] * (LUT[n][code[n][k]] * scale[n][k/128] + offset[n][k/128])
// (any4 paper, section 4.2 for the on-the-fly dequantising GEMM, sections 2.4.1 and 2.5.2 for
// the per-row table and alpha * w_Q + beta).
//
// The paper keeps the 16-entry table in a register and looks codes up with a warp shuffle, and
// rejects a shared-memory table of all 256 value PAIRS because of bank conflicts (section 4.2,
// last paragraph).  Here the pair table is conflict free by construction: a block owns 64 rows,
// lane l of every wavefront works on row l, and entry e of row l lives at LDS byte address
// e * 256 + l * 4, so the lanes LDS serves together always hit distinct banks.  One v_perm_b32
// forms a lookup address (byte j of the code word -> address byte 1, lane offset -> byte 0), the
// lookup returns two bf16 table values, and one v_dot2 multiplies them with the matching pair of
// activations.  Because all lanes of a wavefront sit at the same k, the activations are
// wave-uniform and come from scalar loads; there is no cross-lane reduction at all.
//
// Scale and offset never touch individual weights.  With X[g] the sum of the 128 activations of
// group g,  y[n] = sum_g ( scale[n][g] * P[n][g] + offset[n][g] * X[g] ),
// P[n][g] = sum_{k in g} x[k] * LUT[n][code[n][k]].
//
// Work split: block = 64 rows x one K slice (<= gslice groups), wavefronts split the slice in
// interleaved chunks of 2 groups (128 B of codes per row: one cache line per lane and chunk,
// fetched by eight back-to-back 16-byte loads).  Two chunks per wavefront are kept in flight.
#include "any4_device.h"
#include "any4_internal.h"
#include "any4_splitk.h"
#include <type_traits>

namespace any4 {

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

#ifdef ANY4_STAMPS
__device__ long long* g_any4_dbg_m1 = nullptr;
#define M1_STAMP(i) do { if (g_any4_dbg_m1 && lane == 0) g_any4_dbg_m1[((int64_t)blockIdx.x * WAVES + wave) * 8 + (i)] = wall_clock64(); } while (0)
#else
#define M1_STAMP(i) do {} while (0)
#endif

constexpr int kM1Rows = 64;
constexpr int kM1TableBytes = 256 * kM1Rows * 4;       // 64 KB
constexpr int kM1ChunkGroups = 2;                       // 8 steps of 32 codes per lane
constexpr int kM1MaxSlice = 32;                         // most groups one block takes (K slice <= 4096)

template <int WAVES, int DEPTH, bool PIPE>
__global__ __launch_bounds__(WAVES * 64, (WAVES == 8 ? 4 : 2)) void decode_m1_kernel(
    const uint16_t* __restrict__ x, const uint32_t* __restrict__ codes,
    const uint16_t* __restrict__ lut, const uint16_t* __restrict__ scale,
    const uint16_t* __restrict__ offset, int64_t N, int64_t K, int gslice, int tiles,
    int ksplit, uint16_t* __restrict__ y, float* partial, unsigned long long* counters,
    unsigned long long epoch) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint32_t* table = reinterpret_cast<uint32_t*>(smem);
    float* xsum = reinterpret_cast<float*>(smem + kM1TableBytes);          // [kM1MaxSlice]
    uint16_t* sc_l = reinterpret_cast<uint16_t*>(smem + kM1TableBytes + kM1MaxSlice * 4);   // [g][64] bf16
    uint16_t* of_l = sc_l + kM1MaxSlice * kM1Rows;                                          // [g][64] bf16

    constexpr int THREADS = WAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // consecutive blocks take the K slices of one row tile, so that the blocks resident at any time
    // read whole rows between them (all DRAM channels busy), not one K slice of many rows
    const int tile = blockIdx.x / ksplit, slice = blockIdx.x % ksplit;
    const int64_t n0 = (int64_t)tile * kM1Rows;
    const int G = (int)(K / kGroup);
    const int g0 = slice * gslice, g1 = min(G, g0 + gslice), ng = g1 - g0;

    const int64_t n = min(n0 + lane, N - 1);            // rows past N are clamped, never stored
    const uint32_t r4 = (uint32_t)lane * 4u;
    const uint32_t* rowp = codes + n * (K / 8);
    const uint32_t* xw = reinterpret_cast<const uint32_t*>(x);            // activation pairs

    M1_STAMP(0);
    // ---- prologue loads, in the order their consumers need them (loads return in issue order)
    const uint4 la = reinterpret_cast<const uint4*>(lut + n * 16)[0];
    const uint4 lb = reinterpret_cast<const uint4*>(lut + n * 16)[1];
    uint16_t hraw[16 / WAVES];                          // LUT[hi] for the high nibbles this wavefront fills in
#pragma unroll
    for (int i = 0; i < 16 / WAVES; ++i) hraw[i] = lut[n * 16 + wave + i * WAVES];
    // scale / offset of the block's 64 rows x slice: 4 threads per row, 8 groups (16 B) each per pass;
    // staged through LDS so that the main loop issues no scattered small global loads
    constexpr int SP = (kM1Rows * (kM1MaxSlice / 8) + THREADS - 1) / THREADS;
    uint4 sv[SP], ov[SP];
#pragma unroll
    for (int i = 0; i < SP; ++i) {
        const int u = tid + i * THREADS, row = u >> 2, part = u & 3;
        sv[i] = make_uint4(0, 0, 0, 0);
        ov[i] = make_uint4(0, 0, 0, 0);
        if (row < kM1Rows && part * 8 < ng) {
            const int64_t nr = min(n0 + row, N - 1);
            sv[i] = *reinterpret_cast<const uint4*>(scale + nr * G + g0 + part * 8);
            ov[i] = *reinterpret_cast<const uint4*>(offset + nr * G + g0 + part * 8);
        }
    }
    constexpr int XP = (kM1MaxSlice * 16 + THREADS - 1) / THREADS;   // passes to cover the slice's activations
    uint4 xv[XP];                                       // 8 activations per thread and pass, for the group sums
#pragma unroll
    for (int i = 0; i < XP; ++i) {
        xv[i] = make_uint4(0, 0, 0, 0);
        if (tid + i * THREADS < ng * 16) xv[i] = reinterpret_cast<const uint4*>(x + (int64_t)g0 * kGroup)[tid + i * THREADS];
    }

    constexpr int cstep = WAVES * kM1ChunkGroups;
    int cg = g0 + wave * kM1ChunkGroups;                // first group of this wavefront's current chunk
    uint4 cw[DEPTH][8];
    auto load_chunk = [&](int buf, int c) {
        const uint32_t* p = rowp + (int64_t)c * 16;
#pragma unroll
        for (int s = 0; s < 8; ++s) cw[buf][s] = *reinterpret_cast<const uint4*>(p + s * 4);
    };
    if (cg < g1) load_chunk(0, cg);
    if (DEPTH > 1 && cg + cstep < g1) load_chunk(DEPTH - 1, cg + cstep);

    // ---- pair tables: entry (hi << 4 | lo) of row q = LUT[lo] | LUT[hi] << 16 at byte entry*256 + q*4
    {
        const uint32_t L[8] = {la.x, la.y, la.z, la.w, lb.x, lb.y, lb.z, lb.w};
#pragma unroll
        for (int i = 0; i < 16 / WAVES; ++i) {
            const int hi = wave + i * WAVES;            // wave-uniform
            const uint32_t hv = (uint32_t)hraw[i] << 16;
            uint32_t* dst = table + hi * 16 * kM1Rows + lane;
#pragma unroll
            for (int lo = 0; lo < 16; ++lo) {
                const uint32_t lv = (lo & 1) ? (L[lo >> 1] >> 16) : (L[lo >> 1] & 0xFFFFu);
                dst[lo * kM1Rows] = lv | hv;
            }
        }
    }
    M1_STAMP(1);
    // ---- group sums of the activations of this slice (16 lanes per group)
#pragma unroll
    for (int i = 0; i < XP; ++i) {
        const uint4 v = xv[i];
        float s = ((bf16lo_to_f32(v.x) + bf16hi_to_f32(v.x)) + (bf16lo_to_f32(v.y) + bf16hi_to_f32(v.y))) +
                  ((bf16lo_to_f32(v.z) + bf16hi_to_f32(v.z)) + (bf16lo_to_f32(v.w) + bf16hi_to_f32(v.w)));
        s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x121, 0xF, 0xF, false));
        s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x122, 0xF, 0xF, false));
        s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x124, 0xF, 0xF, false));
        s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x128, 0xF, 0xF, false));
        const int t = tid + i * THREADS;
        if ((t & 15) == 0 && t < ng * 16) xsum[t >> 4] = s;
    }
#pragma unroll
    for (int i = 0; i < SP; ++i) {
        const int u = tid + i * THREADS, row = u >> 2, part = u & 3;
        if (row < kM1Rows && part * 8 < ng) {
            const uint32_t a[4] = {sv[i].x, sv[i].y, sv[i].z, sv[i].w}, b[4] = {ov[i].x, ov[i].y, ov[i].z, ov[i].w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int g = part * 8 + 2 * j;
                sc_l[g * kM1Rows + row] = (uint16_t)(a[j] & 0xFFFFu);
                sc_l[(g + 1) * kM1Rows + row] = (uint16_t)(a[j] >> 16);
                of_l[g * kM1Rows + row] = (uint16_t)(b[j] & 0xFFFFu);
                of_l[(g + 1) * kM1Rows + row] = (uint16_t)(b[j] >> 16);
            }
        }
    }
    M1_STAMP(2);
    __syncthreads();
    M1_STAMP(3);

    const unsigned char* tb = reinterpret_cast<const unsigned char*>(table);
    float acc = 0.f;

    // one chunk = 2 groups = 8 steps; step s: lane's word group cw[s] holds codes s*32 .. s*32+31 of
    // the chunk, activations of the step are 16 wave-uniform dwords (scalar loads)
    auto chunk = [&](auto buf_tag, auto more_tag) {
        constexpr int B = decltype(buf_tag)::value;
        constexpr bool MORE = decltype(more_tag)::value;      // refill this buffer with chunk cg + DEPTH*cstep
        const int ccg = cg;
        const uint32_t* xc = xw + (int64_t)ccg * (kGroup / 2);
        const uint32_t* nextp = rowp + (int64_t)(ccg + DEPTH * cstep) * 16;
        uint32_t bb[2][16];
        auto lookups = [&](const uint4& c, uint32_t (&b)[16]) {
            const uint32_t w[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                b[4 * j + 0] = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w[j], r4, 0x0c0c0400u));
                b[4 * j + 1] = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w[j], r4, 0x0c0c0500u));
                b[4 * j + 2] = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w[j], r4, 0x0c0c0600u));
                b[4 * j + 3] = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w[j], r4, 0x0c0c0700u));
            }
        };
        // scale, offset and activation sum of the chunk's two groups, read ahead of their use
        const int gl = ccg - g0;
        const float sf[2] = {bf16_to_f32(sc_l[gl * kM1Rows + lane]), bf16_to_f32(sc_l[(gl + 1) * kM1Rows + lane])};
        const float of[2] = {bf16_to_f32(of_l[gl * kM1Rows + lane]), bf16_to_f32(of_l[(gl + 1) * kM1Rows + lane])};
        const float xg[2] = {xsum[gl], xsum[gl + 1]};
        // Per step: the scalar loads of the next step's activations and the lookups of the next
        // step's codes are issued first, then the 16 dot products of the current step run while
        // those are in flight.  (Scalar loads return out of order, so every wait on them is a
        // full lgkmcnt(0); issuing them a step ahead keeps that wait short.)
        float P = 0.f;
        if constexpr (PIPE) {
            uint32_t xs[2][16];
#pragma unroll
            for (int i = 0; i < 16; ++i) xs[0][i] = xc[i];
            lookups(cw[B][0], bb[0]);
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int cur = s & 1;
                if (s < 7) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) xs[cur ^ 1][i] = xc[(s + 1) * 16 + i];
                    lookups(cw[B][s + 1], bb[cur ^ 1]);
                    if (MORE && s == 6) {
                        // all lookup addresses of this buffer are formed: refill it with eight back-to-back
                        // loads, so that the 128-byte line of every lane is requested in one burst
#pragma unroll
                        for (int t = 0; t < 8; ++t) cw[B][t] = *reinterpret_cast<const uint4*>(nextp + t * 4);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    P = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, bb[cur][i]),
                                                        __builtin_bit_cast(bf16x2, xs[cur][i]), P, false);
                if ((s & 3) == 3) {
                    const int gi = s >> 2;
                    acc = __builtin_fmaf(P, sf[gi], acc);
                    acc = __builtin_fmaf(of[gi], xg[gi], acc);
                    P = 0.f;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            // no software pipelining: with four wavefronts per SIMD the other wavefronts cover the
            // lookup latency, and the smaller register footprint is what allows that occupancy
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                uint32_t xs1[16];
#pragma unroll
                for (int i = 0; i < 16; ++i) xs1[i] = xc[s * 16 + i];
                lookups(cw[B][s], bb[0]);
                if (MORE && s == 7) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) cw[B][t] = *reinterpret_cast<const uint4*>(nextp + t * 4);
                }
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    P = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, bb[0][i]),
                                                        __builtin_bit_cast(bf16x2, xs1[i]), P, false);
                if ((s & 3) == 3) {
                    const int gi = s >> 2;
                    acc = __builtin_fmaf(P, sf[gi], acc);
                    acc = __builtin_fmaf(of[gi], xg[gi], acc);
                    P = 0.f;
                }
            }
        }
        cg += cstep;
    };
    using T = std::true_type;
    using F = std::false_type;
    using B0 = std::integral_constant<int, 0>;
    // chunks alternate between the two register buffers; the last two are not refilled
    bool second = false;                               // wave-uniform
    while (cg < g1) {
        const bool more = cg + DEPTH * cstep < g1;
        if (DEPTH == 1 || !second) { if (more) chunk(B0{}, T{}); else chunk(B0{}, F{}); }
        else { if (more) chunk(std::integral_constant<int, DEPTH - 1>{}, T{}); else chunk(std::integral_constant<int, DEPTH - 1>{}, F{}); }
        second = !second;
    }

    // ---- combine the K parts of the block in a fixed order and store
    M1_STAMP(4);
    __syncthreads();
    M1_STAMP(5);                                   // all lookups done: the table space is reused
    float* red = reinterpret_cast<float*>(smem);       // [WAVES][64]
    red[wave * 64 + lane] = acc;
    __syncthreads();
    if (tid < kM1Rows) {
        float s = 0.f;
#pragma unroll
        for (int p = 0; p < WAVES; ++p) s += red[p * 64 + tid];
        const int64_t nn = n0 + tid;
        if (nn < N) {
            if (ksplit == 1) y[nn] = (uint16_t)f32_to_bf16(s);
            else splitk_store(partial + (int64_t)slice * N + nn, s);
        }
    }
    if (ksplit > 1) {
        int* flag = reinterpret_cast<int*>(smem + WAVES * 64 * 4);
        if (splitk_arrive(counters, tile, ksplit, epoch, flag) && tid < kM1Rows) {
            const int64_t nn = n0 + tid;
            if (nn < N) {
                float s = 0.f;
                for (int k = 0; k < ksplit; ++k) s += splitk_load(partial + (int64_t)k * N + nn);
                y[nn] = (uint16_t)f32_to_bf16(s);
            }
        }
    }
    M1_STAMP(6);
}

#ifdef ANY4_STAMPS
extern "C" int any4_debug_set_buffer_m1(void* p) {
    long long* q = static_cast<long long*>(p);
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_any4_dbg_m1), &q, sizeof(q));
}
#endif

int decode_m1_gslice_limit() { return kM1MaxSlice; }

size_t decode_m1_lds_bytes(int) { return (size_t)kM1TableBytes + kM1MaxSlice * 4 + 2 * kM1MaxSlice * kM1Rows * 2; }

hipError_t launch_decode_m1(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                            const uint16_t* scale, const uint16_t* offset, int64_t N, int64_t K,
                            const GemmPlan& plan, uint16_t* y, void* workspace, unsigned long long epoch,
                            hipStream_t stream) {
#ifndef ANY4_M1_WAVES
#define ANY4_M1_WAVES 4
#endif
#ifndef ANY4_M1_DEPTH
#define ANY4_M1_DEPTH 1
#endif
    constexpr int WAVES = ANY4_M1_WAVES;
    auto kern = decode_m1_kernel<WAVES, ANY4_M1_DEPTH, (WAVES == 4)>;
    const size_t lds = decode_m1_lds_bytes(plan.gslice);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int64_t tiles = (N + kM1Rows - 1) / kM1Rows;
    if (tiles * plan.ksplit > 0x7FFFFFFF) return hipErrorInvalidValue;
    unsigned long long* counters = static_cast<unsigned long long*>(workspace);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + splitk_counter_bytes(tiles));
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles * plan.ksplit)), dim3(WAVES * 64), lds, stream,
                       x, codes, lut, scale, offset, N, K, plan.gslice, (int)tiles, plan.ksplit, y, partial,
                       counters, epoch);
    return hipGetLastError();
}

}  // namespace any4
