// Memory-bound any4 GEMM for small M (token generation, M <= 16): row-tile kernel.
//
// y[m][n] = sum_k x[m][k] * (LUT[n][code[n][k]] * scale[n][k/128] + offset[n][k/128])
// (any4 paper, section 4.2 for y = x w^T with on-the-fly dequantisation, sections 2.4.1 and
// 2.5.2 for the per-row table and alpha * w_Q + beta).
//
// The paper's kernels look a code up with a register shuffle and note that a shared-memory
// table of all 16 x 16 value PAIRS (one lookup per packed byte) halves the lookups but suffers
// bank conflicts (section 4.2, last paragraph).  On CDNA4 the pair table can be made conflict
// free: a wavefront owns 32 weight rows, lane l works on row l % 32, and row r's 256 entries
// live at LDS byte address entry * 256 + r * 4, so the 32 lanes LDS serves per clock always hit
// 32 different banks.  The address of a lookup is one v_perm_b32 (byte j of the code word to
// address byte 1, the lane's row offset to byte 0), the lookup returns two bf16 table values
// already packed as a matrix-core operand, and v_mfma_f32_32x32x16_bf16 multiplies 32 rows x 16
// codes by the activations in one instruction (activations are the A operand, one row per m).
//
// The group scale and offset never touch individual weights.  With X[m][g] the sum of the 128
// activations of group g,
//     y[m][n] = sum_g ( scale[n][g] * P[m][n][g] + offset[n][g] * X[m][g] ),
//     P[m][n][g] = sum_{k in g} x[m][k] * LUT[n][code[n][k]]      (exact bf16 x bf16 products)
// so per group a lane does one fp32 fma per accumulator for the scale and one for the offset.
//
// Work split: a block owns 64 rows (two 32-row halves) and one K slice of at most `gslice`
// groups; its wavefronts are (row half) x (K part), K parts interleaved in chunks of 4 groups.
// Lane (r = l % 32, h = l / 32) streams 16-byte pieces of ITS row: step s of a chunk reads bytes
// [s*32 + h*16, +16) of the chunk, i.e. 32 codes; word j of that piece feeds MFMA (s, j), whose
// k-slot h therefore covers codes s*64 + h*32 + j*8 .. +8 of the chunk.
#include "any4_device.h"
#include "any4_internal.h"
#include "any4_splitk.h"
#include <type_traits>

namespace any4 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#ifdef ANY4_STAMPS
__device__ long long* g_any4_dbg = nullptr;
#define ANY4_STAMP(i) do { if (g_any4_dbg && lane == 0) g_any4_dbg[((int64_t)blockIdx.x * WAVES + wave) * 8 + (i)] = wall_clock64(); } while (0)
#else
#define ANY4_STAMP(i) do {} while (0)
#endif

constexpr int kTileRows = 64;
constexpr int kTableBytes = 256 * kTileRows * 4;      // 64 KB: 256 pair entries x 64 rows x 4 B
constexpr int kChunkGroups = 4;                        // groups per chunk (8 steps of 64 codes)

__device__ __forceinline__ float dpp_row_sum16(float s) {
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x121, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x122, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x124, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x128, 0xF, 0xF, false));
    return s;
}

// MT = number of accumulator registers a lane keeps: 1 (M == 1), 4 (M <= 8), 8 (M <= 16).
// FULL = every chunk of every slice has all 4 groups and scale rows are 8-byte aligned
//        (true when K/128 is a multiple of 4).
template <int MT, int WAVES, bool FULL>
__global__ __launch_bounds__(WAVES * 64, (MT == 1 && WAVES == 8 ? 4 : 2)) void decode_tile_kernel(
    const uint16_t* __restrict__ x, const uint32_t* __restrict__ codes,
    const uint16_t* __restrict__ lut, const uint16_t* __restrict__ scale,
    const uint16_t* __restrict__ offset, int M, int64_t N, int64_t K, int gslice, int tiles,
    int ksplit, uint16_t* __restrict__ y, float* partial, unsigned long long* counters,
    unsigned long long epoch) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint32_t* table = reinterpret_cast<uint32_t*>(smem);
    float* xsum = reinterpret_cast<float*>(smem + kTableBytes);                    // [gslice][16]
    const uint16_t* xl = reinterpret_cast<const uint16_t*>(smem + kTableBytes + gslice * 64);  // MT == 1: x slice

    constexpr int KPARTS = WAVES / 2;
    constexpr int THREADS = WAVES * 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // consecutive blocks take the K slices of one row tile, so that the blocks resident at any time
    // read whole rows between them (all DRAM channels busy), not one K slice of many rows
    const int tile = blockIdx.x / ksplit, slice = blockIdx.x % ksplit;
    const int64_t n0 = (int64_t)tile * kTileRows;
    const int G = (int)(K / kGroup);
    const int g0 = slice * gslice, g1 = min(G, g0 + gslice), ng = g1 - g0;

    const int rh = wave & 1, kp = wave >> 1;
    const int r = lane & 31, h = lane >> 5;
    const int rho = rh * 32 + r;
    const int64_t n = min(n0 + rho, N - 1);           // rows past N are clamped, never stored
    const uint32_t r4 = (uint32_t)rho * 4u;
    const uint32_t* rowp = codes + n * (K / 8) + h * 4;
    const uint16_t* srow = scale + n * G;
    const uint16_t* orow = offset + n * G;

    ANY4_STAMP(0);
    uint4 cw[8];
    uint32_t sc[kChunkGroups], of[kChunkGroups];
    auto load_chunk = [&](int cg) {
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (FULL || cg + (s >> 1) < g1) cw[s] = *reinterpret_cast<const uint4*>(rowp + ((int64_t)cg * 2 + s) * 8);
            else cw[s] = make_uint4(0, 0, 0, 0);
        }
        if (FULL) {
            const uint2 a = *reinterpret_cast<const uint2*>(srow + cg);
            const uint2 b = *reinterpret_cast<const uint2*>(orow + cg);
            sc[0] = a.x << 16; sc[1] = a.x & 0xFFFF0000u; sc[2] = a.y << 16; sc[3] = a.y & 0xFFFF0000u;
            of[0] = b.x << 16; of[1] = b.x & 0xFFFF0000u; of[2] = b.y << 16; of[3] = b.y & 0xFFFF0000u;
        } else {
#pragma unroll
            for (int i = 0; i < kChunkGroups; ++i) {
                const bool ok = cg + i < g1;
                sc[i] = ok ? (uint32_t)srow[cg + i] << 16 : 0u;
                of[i] = ok ? (uint32_t)orow[cg + i] << 16 : 0u;
            }
        }
    };

    // Order of the prologue loads matters: a wavefront's loads return in issue order, and the
    // table build needs the row's table first.  So: table values, then the first chunk of codes
    // (in flight while the block builds its tables).
    const int tq = tid & 63, tpart = tid >> 6;
    const int64_t nq = min(n0 + tq, N - 1);
    const uint4 la = reinterpret_cast<const uint4*>(lut + nq * 16)[0];
    const uint4 lb = reinterpret_cast<const uint4*>(lut + nq * 16)[1];
    constexpr int HIS = 16 / WAVES;                     // high nibbles handled per thread
    uint16_t hraw[HIS];
#pragma unroll
    for (int i = 0; i < HIS; ++i) hraw[i] = lut[nq * 16 + tpart + i * WAVES];

    int cg = g0 + kp * kChunkGroups;
    const int cstep = KPARTS * kChunkGroups;
    if (cg < g1) load_chunk(cg);

    // ---- pair tables: entry (hi << 4 | lo) of row q = LUT[lo] | LUT[hi] << 16 at byte entry*256 + q*4
    {
        const uint32_t L[8] = {la.x, la.y, la.z, la.w, lb.x, lb.y, lb.z, lb.w};
#pragma unroll
        for (int i = 0; i < HIS; ++i) {
            const int hi = tpart + i * WAVES;
            const uint32_t hv = (uint32_t)hraw[i] << 16;
            uint32_t* dst = table + hi * 16 * kTileRows + tq;
#pragma unroll
            for (int lo = 0; lo < 16; ++lo) {
                const uint32_t lv = (lo & 1) ? (L[lo >> 1] >> 16) : (L[lo >> 1] & 0xFFFFu);
                dst[lo * kTileRows] = lv | hv;
            }
        }
    }
    ANY4_STAMP(1);
    // ---- group sums of the activations of this K slice: xsum[g][m], 16 lanes per (g, m); for
    //      M == 1 the same registers also fill the block's LDS copy of the activation slice
    {
        const int sub = tid & 15;
        const int units = ng * M;                       // (g, m) pairs, m fastest
        auto sum8 = [](const uint4& v) {
            return ((bf16lo_to_f32(v.x) + bf16hi_to_f32(v.x)) + (bf16lo_to_f32(v.y) + bf16hi_to_f32(v.y))) +
                   ((bf16lo_to_f32(v.z) + bf16hi_to_f32(v.z)) + (bf16lo_to_f32(v.w) + bf16hi_to_f32(v.w)));
        };
        constexpr int UPB = THREADS / 16;               // units per pass of the block
        for (int u0 = tid >> 4; u0 < units; u0 += 4 * UPB) {
            uint4 v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {               // four independent loads in flight
                const int u = u0 + i * UPB;
                v[i] = make_uint4(0, 0, 0, 0);
                if (u < units) {
                    const int gl = u / M, m = u - gl * M;
                    v[i] = reinterpret_cast<const uint4*>(x + (int64_t)m * K + (int64_t)(g0 + gl) * kGroup)[sub];
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int u = u0 + i * UPB;
                const float t = dpp_row_sum16(sum8(v[i]));
                if (u < units) {
                    const int gl = u / M, m = u - gl * M;
                    if (sub == 0) xsum[gl * 16 + m] = t;
                    if (MT == 1) reinterpret_cast<uint4*>(smem + kTableBytes + gslice * 64)[gl * 16 + sub] = v[i];
                }
            }
        }
    }
    ANY4_STAMP(2);
    __syncthreads();
    ANY4_STAMP(3);

    float acc[MT];
#pragma unroll
    for (int v = 0; v < MT; ++v) acc[v] = 0.f;
    const unsigned char* tb = reinterpret_cast<const unsigned char*>(table);

    // four table lookups for the 8 codes of one word: the packed B operand of one MFMA
    auto lookup = [&](uint32_t w) {
        uint4 b;
#ifdef ANY4_EXP_NOLOOKUP
        b.x = w ^ r4; b.y = w + r4; b.z = w | r4; b.w = w & ~r4; return b;
#endif
        b.x = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w, r4, 0x0c0c0400u));
        b.y = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w, r4, 0x0c0c0500u));
        b.z = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w, r4, 0x0c0c0600u));
        b.w = *reinterpret_cast<const uint32_t*>(tb + __builtin_amdgcn_perm(w, r4, 0x0c0c0700u));
        return b;
    };
    auto mfma = [&](const uint4& a, const uint4& b, const f32x16& c) -> f32x16 {
#ifdef ANY4_EXP_NOMFMA
        f32x16 t = c; t[0] += __uint_as_float((a.x ^ b.x) + (a.y ^ b.y) + (a.z ^ b.z) + (a.w ^ b.w)); return t;
#endif
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    };
    f32x16 zero;
#pragma unroll
    for (int v = 0; v < 16; ++v) zero[v] = 0.f;

    if constexpr (MT == 1 && FULL) {
        // Software pipeline over the 8 steps of a chunk: the lookups of step s+1 are in flight
        // while the four MFMAs of step s run; the activation reads of step s+1 (only the two lanes
        // that own m = 0 take part) follow those MFMAs; and the code register of a step is
        // refilled from the wavefront's next chunk as soon as its lookup addresses have been
        // formed, so a full chunk of global loads is always in flight.
        uint4 bb[2][4], aa[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) aa[j] = make_uint4(0, 0, 0, 0);
        uint2 rs = *reinterpret_cast<const uint2*>(srow + min(cg, G - 4));   // raw scale / offset of the chunk
        uint2 ro = *reinterpret_cast<const uint2*>(orow + min(cg, G - 4));
        auto chunk = [&](auto more_tag) {
            constexpr bool MORE = decltype(more_tag)::value;
            const int ccg = cg;
            cg += cstep;
            const uint16_t* xc = xl + (ccg - g0) * kGroup + h * 32;
            const uint32_t* nextp = rowp + (int64_t)cg * 16;
            const uint2 cs = rs, co = ro;
            {
                const uint4 c = cw[0];
                bb[0][0] = lookup(c.x); bb[0][1] = lookup(c.y); bb[0][2] = lookup(c.z); bb[0][3] = lookup(c.w);
                if (r == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) aa[j] = *reinterpret_cast<const uint4*>(xc + j * 8);
                }
                if (MORE) cw[0] = *reinterpret_cast<const uint4*>(nextp);
            }
            f32x16 P;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int cur = s & 1, nxt = cur ^ 1;
                if (s < 7) {
                    const uint4 c = cw[s + 1];
                    bb[nxt][0] = lookup(c.x); bb[nxt][1] = lookup(c.y); bb[nxt][2] = lookup(c.z); bb[nxt][3] = lookup(c.w);
                    if (MORE) cw[s + 1] = *reinterpret_cast<const uint4*>(nextp + (s + 1) * 8);
                } else if (MORE) {
                    rs = *reinterpret_cast<const uint2*>(srow + cg);
                    ro = *reinterpret_cast<const uint2*>(orow + cg);
                }
                P = mfma(aa[0], bb[cur][0], (s & 1) ? P : zero);
                P = mfma(aa[1], bb[cur][1], P);
                P = mfma(aa[2], bb[cur][2], P);
                P = mfma(aa[3], bb[cur][3], P);
                if (s < 7 && r == 0) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) aa[j] = *reinterpret_cast<const uint4*>(xc + (s + 1) * 64 + j * 8);
                }
                if (s & 1) {
                    const int gi = s >> 1;
                    const uint32_t s2 = gi < 2 ? cs.x : cs.y, o2 = gi < 2 ? co.x : co.y;
                    const float sf = (gi & 1) ? bf16hi_to_f32(s2) : bf16lo_to_f32(s2);
                    const float ofs = (gi & 1) ? bf16hi_to_f32(o2) : bf16lo_to_f32(o2);
                    acc[0] = __builtin_fmaf(P[0], sf, acc[0]);
                    acc[0] = __builtin_fmaf(ofs, xsum[(ccg + gi - g0) * 16 + 4 * h], acc[0]);
                }
            }
        };
        if (cg < g1) {
            while (cg + cstep < g1) chunk(std::true_type{});
            chunk(std::false_type{});
        }
    } else {
        uint4 av = make_uint4(0, 0, 0, 0);            // A operand (activations); rows m >= M stay zero
        while (cg < g1) {
            // consume the loaded chunk, then prefetch the next one
            uint4 cur[8];
            uint32_t csc[kChunkGroups], cof[kChunkGroups];
#pragma unroll
            for (int s = 0; s < 8; ++s) cur[s] = cw[s];
#pragma unroll
            for (int i = 0; i < kChunkGroups; ++i) { csc[i] = sc[i]; cof[i] = of[i]; }
            const int ccg = cg;
            cg += cstep;
            if (cg < g1) load_chunk(cg);

#pragma unroll
            for (int gi = 0; gi < kChunkGroups; ++gi) {
                if (!FULL && ccg + gi >= g1) break;
                f32x16 P;
#pragma unroll
                for (int ss = 0; ss < 2; ++ss) {
                    const int s = gi * 2 + ss;
                    const uint32_t wj[4] = {cur[s].x, cur[s].y, cur[s].z, cur[s].w};
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const uint4 bv = lookup(wj[j]);
                        const int koff = s * 64 + h * 32 + j * 8;      // code offset inside the chunk
                        if (MT == 1) {
                            if (r == 0) av = *reinterpret_cast<const uint4*>(xl + (ccg - g0) * kGroup + koff);
                        } else {
                            if (r < M) av = *reinterpret_cast<const uint4*>(x + (int64_t)r * K + (int64_t)ccg * kGroup + koff);
                        }
                        P = mfma(av, bv, (ss == 0 && j == 0) ? zero : P);
                    }
                }
                // accumulator v of a lane is activation row m = 8*(v/4) + 4*h + v%4, weight row = the lane's
                const float sf = __uint_as_float(csc[gi]), off = __uint_as_float(cof[gi]);
                const float* xs = xsum + (ccg + gi - g0) * 16 + 4 * h;
#pragma unroll
                for (int v = 0; v < MT; ++v) {
                    acc[v] = __builtin_fmaf(P[v], sf, acc[v]);
                    acc[v] = __builtin_fmaf(off, xs[(v >> 2) * 8 + (v & 3)], acc[v]);
                }
            }
        }
    }

    // ---- combine the K parts of the block in a fixed order and store
    ANY4_STAMP(4);
    __syncthreads();
    ANY4_STAMP(5);                                   // all lookups done: the table space is reused
    float* red = reinterpret_cast<float*>(smem);       // [WAVES][MT][64]
#pragma unroll
    for (int v = 0; v < MT; ++v) red[(wave * MT + v) * 64 + lane] = acc[v];
    __syncthreads();
    for (int e = tid; e < M * kTileRows; e += THREADS) {
        const int m = e >> 6, q = e & 63;
        const int v = (m >> 3) * 4 + (m & 3), hh = (m >> 2) & 1;
        const int src_lane = hh * 32 + (q & 31), half = q >> 5;
        float s = 0.f;
#pragma unroll
        for (int p = 0; p < KPARTS; ++p) s += red[((p * 2 + half) * MT + v) * 64 + src_lane];
        const int64_t nn = n0 + q;
        if (nn < N) {
            if (ksplit == 1) y[(int64_t)m * N + nn] = (uint16_t)f32_to_bf16(s);
            else splitk_store(partial + ((int64_t)slice * M + m) * N + nn, s);
        }
    }
    if (ksplit > 1) {
        int* flag = reinterpret_cast<int*>(smem + WAVES * MT * 64 * 4);
        if (splitk_arrive(counters, tile, ksplit, epoch, flag)) {
            for (int e = tid; e < M * kTileRows; e += THREADS) {
                const int m = e >> 6, q = e & 63;
                const int64_t nn = n0 + q;
                if (nn < N) {
                    float s = 0.f;
                    for (int k = 0; k < ksplit; ++k)
                        s += splitk_load(partial + ((int64_t)k * M + m) * N + nn);
                    y[(int64_t)m * N + nn] = (uint16_t)f32_to_bf16(s);
                }
            }
        }
    }
    ANY4_STAMP(6);
}

#ifdef ANY4_STAMPS
extern "C" int any4_debug_set_buffer(void* p) {
    long long* q = static_cast<long long*>(p);
    return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_any4_dbg), &q, sizeof(q));
}
#endif

// ---------------------------------------------------------------------------------------------
int decode_tile_gslice_limit(int M) { return M == 1 ? 32 : 64; }

size_t decode_tile_lds_bytes(int M, int gslice) {
    return (size_t)kTableBytes + (size_t)gslice * 64 + (M == 1 ? (size_t)gslice * 256 : 0);
}

template <int MT, bool FULL>
static hipError_t launch_tile(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                              const uint16_t* scale, const uint16_t* offset, int M, int64_t N, int64_t K,
                              const GemmPlan& plan, uint16_t* y, void* workspace, unsigned long long epoch,
                              hipStream_t stream) {
#ifndef ANY4_TILE_WAVES
#define ANY4_TILE_WAVES 8
#endif
    constexpr int WAVES = ANY4_TILE_WAVES;
    auto kern = decode_tile_kernel<MT, WAVES, FULL>;
    const size_t lds = decode_tile_lds_bytes(M, plan.gslice);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const int64_t tiles = (N + kTileRows - 1) / kTileRows;
    if (tiles * plan.ksplit > 0x7FFFFFFF) return hipErrorInvalidValue;
    unsigned long long* counters = static_cast<unsigned long long*>(workspace);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + splitk_counter_bytes(tiles));
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles * plan.ksplit)), dim3(WAVES * 64), lds, stream,
                       x, codes, lut, scale, offset, M, N, K, plan.gslice, (int)tiles, plan.ksplit, y, partial,
                       counters, epoch);
    return hipGetLastError();
}

hipError_t launch_decode_tile(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                              const uint16_t* scale, const uint16_t* offset, int64_t M, int64_t N,
                              int64_t K, const GemmPlan& plan, uint16_t* y, void* workspace,
                              unsigned long long epoch, hipStream_t stream) {
    const bool full = (K / kGroup) % 4 == 0 && plan.gslice % 4 == 0;
    const int m = (int)M;
#define ANY4_TILE(MT)                                                                                   \
    (full ? launch_tile<MT, true>(x, codes, lut, scale, offset, m, N, K, plan, y, workspace, epoch, stream)      \
          : launch_tile<MT, false>(x, codes, lut, scale, offset, m, N, K, plan, y, workspace, epoch, stream))
    if (m == 1) return ANY4_TILE(1);
    if (m <= 8) return ANY4_TILE(4);
    return ANY4_TILE(8);
#undef ANY4_TILE
}

}  // namespace any4
