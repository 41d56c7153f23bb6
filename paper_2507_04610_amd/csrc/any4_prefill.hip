// Compute-bound any-n GEMM for large M (prompt processing): LDS-staged table lookup feeding
// bf16 matrix-core (MFMA) tiles with fp32 accumulation.
//
// y[m][n] = sum_k x[m][k] * w[n][k],  w[n][k] = LUT[n][code] * scale[n][k/128] + offset[n][k/128]
// (any4 paper, section 4.2: weights are dequantised on the fly before the matrix instruction;
// sections 2.4.1 / 2.5.2 define the table lookup and alpha * w_Q + beta).  The paper's own
// kernels stop at M = 16; this path is the large-M counterpart for CDNA4.
//
// Rounding a dequantised weight to bf16 costs up to 2^-8 relative per weight (1.7e-3 rms of the
// output, ~1e-2 * rms at the worst of a few million outputs), which is too much for the
// 1e-2 * rms output bound.  The kernel therefore never forms w.  Per group g of 128 weights it uses
//     sum_{k in g} x[m][k] w[n][k] = scale[n][g] * sum_{k in g} x[m][k] LUT[n][code[n][k]]
//                                  + offset[n][g] * X[m][g],      X[m][g] = sum_{k in g} x[m][k]
// The first sum multiplies two exact bf16 operands on the matrix cores (fp32 accumulate) and is
// scaled in fp32 on the vector ALU; the second term is a small extra GEMM over the "group"
// dimension whose left operand X is precomputed in fp32 and split into a bf16 high and low part
// (relative error 2^-16), and whose right operand is the bf16 offset itself.
//
// Block tile 256 (m) x 128 (n), K step 64, eight wavefronts in a 4 x 2 arrangement, each owning a
// 64 x 64 sub-tile as 2 x 2 v_mfma_f32_32x32x16_bf16 accumulators.  Two LDS buffers and one barrier
// per K step.  A K step is written as ONE software-pipelined instruction stream whose order is
// pinned (scheduling barriers): the 16 MFMAs of the step on buffer b are interleaved with
// everything that prepares the next step in buffer b^1 - operand reads one 16-wide slice ahead,
// the table lookups, packing and the LDS writes of the activation tile and of the looked-up tile,
// the per-group scale fold - while the global loads of later steps are in flight.  Left to
// itself the compiler emits "all MFMAs, then all staging", and the two wavefronts of a SIMD, which
// the barrier keeps in step, then leave the matrix cores idle while both stage.
#include "any4_device.h"
#include "any4_internal.h"
#include "any4_splitk.h"
#include <type_traits>

namespace any4 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) u32x4* lds_u4;
typedef const __attribute__((address_space(3))) uint32_t* lds_u32;

constexpr int PBM = 256, PBN = 128, PBK = 64;
constexpr int PTHREADS = 512;
constexpr int PLD = PBK + 8;          // LDS row stride in bf16 elements (144 B: keeps 16-byte reads spread over banks)
constexpr uint32_t kXBuf = PBM * PLD * 2, kWBuf = PBN * PLD * 2;   // bytes of one activation / weight buffer
constexpr uint32_t kTableOff = 2 * kXBuf + 2 * kWBuf;              // 110592 = 0x1B000: the low 12 bits are clear

__device__ __forceinline__ void lds_barrier() {                 // outstanding global loads stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}
#define ANY4_SB() __builtin_amdgcn_sched_barrier(0)

// X[m][g] = sum of the 128 activations of group g, in fp32, stored as two bf16 (high part,
// remainder) at xs[m][2g], xs[m][2g+1]; columns 2G .. KP-1 are zero.  16 lanes per (m, g).
// `fine`: groups of 64 activations, 8 lanes each.
template <bool F16>
__global__ __launch_bounds__(256) void group_sums_kernel(const uint16_t* __restrict__ x, int64_t M,
                                                         int64_t K, int KP, int fine, uint16_t* __restrict__ xs) {
    const int lanes = fine ? 8 : 16;
    const int64_t G = K / (8 * lanes);
    const int64_t unit = ((int64_t)blockIdx.x * 256 + threadIdx.x) / lanes;  // (m, g), g fastest
    const int sub = threadIdx.x & (lanes - 1);
    const bool live = unit < M * G;
    const int64_t u = live ? unit : 0;
    const uint4 v = reinterpret_cast<const uint4*>(x + u * (8 * lanes))[sub];    // x is [M][G][8 * lanes]
    float s = ((h16lo_to_f32<F16>(v.x) + h16hi_to_f32<F16>(v.x)) + (h16lo_to_f32<F16>(v.y) + h16hi_to_f32<F16>(v.y))) +
              ((h16lo_to_f32<F16>(v.z) + h16hi_to_f32<F16>(v.z)) + (h16lo_to_f32<F16>(v.w) + h16hi_to_f32<F16>(v.w)));
    // rotations inside rows of 16 lanes: after 1, 2, 4 a lane holds the sum of itself and the 7 lanes
    // before it (the last lane of a group of 8: its group); after 8, every lane holds the row's sum
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x121, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x122, 0xF, 0xF, false));
    s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x124, 0xF, 0xF, false));
    if (!fine) s += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(s), 0x128, 0xF, 0xF, false));
    if (!live) return;
    const int64_t m = u / G, g = u % G;
    if (sub == lanes - 1) {
        const uint32_t hi = f32_to_h16<F16>(s);
        const uint32_t lo = f32_to_h16<F16>(s - h16_to_f32<F16>(hi));
        *reinterpret_cast<uint32_t*>(xs + m * KP + 2 * g) = hi | (lo << 16);
    }
    // zero padding of the row tail, done by the lanes of the row's last group
    if (g == G - 1)
        for (int c = (int)(2 * G) + sub; c < KP; c += lanes) xs[m * KP + c] = 0;
}

// LDS copy of the block's row tables, laid out so that the 32 lanes LDS serves together never share
// a bank: a half-wavefront holds 8 rows x 4 quarter-threads, and entry c of (row, quarter) lives at
// dword (row / 8) * (32 << BITS) + c * 32 + (row % 8) * 4 + quarter (every row is stored 4 times;
// the bf16 value sits in the low half of the dword).
// FINE: groups of 64 weights - every K step is a group of its own (scale index 2g, 2g + 1 for the two
// steps of chunk g; the offset phase runs over 64-weight groups).  Otherwise groups of 128 << lr.
// F16: activations, table, scales, offsets and output are fp16 instead of bf16.
// NOLUT: 4-bit codes on the uniform grid (value = code - 8, the int4 format the paper compares with in
// section 4.2, last paragraph) without any table: a code c becomes the bf16 number 128 + c by OR-ing it
// into the mantissa of 128.0 (0x4300 | c) - two shifts and two and-or per pair of weights instead of
// two address computations, two LDS lookups and a pack - and the surplus 136 * scale * X (X = the
// group sum of the activations) is taken off in the offset phase by two more passes over the same
// group sums whose right operands are the exact bf16 numbers -128 * scale and -8 * scale.
template <int BITS, bool FINE, bool F16, bool NOLUT = false>
__global__ __launch_bounds__(PTHREADS, 1) void prefill_kernel(
    const uint16_t* __restrict__ x, const uint32_t* __restrict__ codes,
    const uint16_t* __restrict__ lut, const uint16_t* __restrict__ scale,
    const uint16_t* __restrict__ offset, const uint16_t* __restrict__ xsums, int KP,
    int64_t M, int64_t N, int64_t K, int lr, int flags, int gm, int tail_first, int tail_s,
    unsigned long long* __restrict__ counters, float* __restrict__ partial, uint16_t* __restrict__ y) {
    constexpr int L = 1 << BITS;
    const bool repacked = flags & 1, one_table = flags & 2;     // re-laid-out codes / one table for all rows
    static_assert(!(F16 && FINE), "fp16 comes with groups of 128 and more");
    static_assert(!NOLUT || (BITS == 4 && !F16 && !FINE), "the table-free path: 4-bit codes, bf16, groups of 128");
    using op16x8 = std::conditional_t<F16, f16x8, bf16x8>;
    auto mma = [](const op16x8& a, const op16x8& b, const f32x16& c) -> f32x16 {
        if constexpr (F16) return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
        else return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    };
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    uint32_t* table = reinterpret_cast<uint32_t*>(smem + kTableOff);      // [PBN / 8][L][32]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t G = K / kGroup, RW = row_words(K, BITS);
    // Blocks below tail_first own a whole output tile.  The tiles of the last, partly filled round
    // of blocks are cut along K into tail_s slices of whole groups, one block each, so that the
    // round keeps every compute unit busy for 1 / tail_s of a tile's time; the slices' fp32 results
    // meet in the workspace and the block that arrives last adds them in slice order.
    int tile = blockIdx.x, slice = -1;
    int g_lo = 0, g_hi = (int)G;
    if (tile >= tail_first) {
        const int idx = tile - tail_first;
        tile = tail_first + idx / tail_s;
        slice = idx % tail_s;
        g_lo = (int)(slice * G / tail_s);
        g_hi = (int)((slice + 1) * G / tail_s);
    }
    const int64_t m0 = (int64_t)(tile % gm) * PBM, n0 = (int64_t)(tile / gm) * PBN;   // m fastest: an XCD keeps its rows of x
    const int S0 = 2 * g_lo, T = 2 * g_hi;                                // this block's K steps

    // ---- staging roles.  Weights: thread -> (row, 16-code quarter of the K step); rows past N are
    //      clamped (computed, never stored).  Activations: thread -> 4 rows, one 16-byte piece each.
    const int wrow = tid >> 2, wq = tid & 3;
    const int64_t wn_glob = min(n0 + wrow, N - 1);
    // word offset / bit shift of the thread's 16 codes inside the K step's (2 * BITS)-word chunk
    const int qword = BITS == 4 ? 2 * wq : (BITS == 2 ? wq : (6 * wq) >> 2);
    const int qshift = BITS == 3 ? ((6 * wq) & 3) * 8 : 0;
    // plain layout: the K step's codes start at word tile * 2 * BITS of the row.  Tile-major layout
    // (any4_repack): the step is half of group tile / 2; the thread's 16 codes are one half of
    // piece 16 * q + n, q = 2 * (tile % 2) + wq / 2, of unit (row / 16, group): the word offset of
    // step `tile` is (tile / 2) * 64 * BITS + (tile % 2) * 32 * BITS past the thread's base.
    const int hword = (BITS == 4 ? 2 : 1) * (wq & 1);                     // first word of the thread's half inside its piece
    const uint32_t* const wsrc = repacked
        ? codes + (((wn_glob >> 4) * G * 64 + (wq >> 1) * 16 + (wn_glob & 15)) * BITS + hword)
        : codes + wn_glob * RW + qword;
    const int64_t qstep_even = repacked ? 64 * BITS : 4 * BITS, qstep_odd = repacked ? 32 * BITS : 2 * BITS;
    const int xr_row = tid >> 3, xc8 = tid & 7;
    const uint16_t* xsrc[4];                                              // rows past M are clamped, never stored
#pragma unroll
    for (int p = 0; p < 4; ++p) xsrc[p] = x + min(m0 + p * 64 + xr_row, M - 1) * K + xc8 * 8;
    // the two output columns this lane owns (one per 32-wide n tile of its wavefront)
    const uint16_t* scol[2];
    const int64_t GS = FINE ? 2 * G : G >> lr;                            // scales / offsets per row
#pragma unroll
    for (int j = 0; j < 2; ++j) scol[j] = scale + min(n0 + wn * 64 + j * 32 + (lane & 31), N - 1) * GS;
    // LDS byte addresses (the kernel has no static LDS: dynamic LDS starts at 0)
    const uint32_t tbase = kTableOff + (uint32_t)((wrow >> 3) * (32 << BITS) + (wrow & 7) * 4 + wq) * 4u;
    const uint32_t xwr = (uint32_t)(xr_row * PLD + xc8 * 8) * 2u;                         // + buf * kXBuf + p * 64 rows
    const uint32_t wwr = 2 * kXBuf + (uint32_t)(wrow * PLD + wq * 16) * 2u;               // + buf * kWBuf + chunk * 16
    const uint32_t ard = (uint32_t)((wm * 64 + (lane & 31)) * PLD + (lane >> 5) * 8) * 2u;
    const uint32_t brd = 2 * kXBuf + (uint32_t)((wn * 64 + (lane & 31)) * PLD + (lane >> 5) * 8) * 2u;

    f32x16 acc[2][2], part[2][2];
    f32x16 zero;
#pragma unroll
    for (int v = 0; v < 16; ++v) zero[v] = 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) { acc[i][j] = zero; part[i][j] = zero; }

    // ---- global fetches (tile indices are clamped by the callers: the loads are unconditional so
    //      that the compiler waits for them by count, not with vmcnt(0))
    u32x4 xr[4];
    auto fetch_x = [&](int tile) {
#pragma unroll
        for (int p = 0; p < 4; ++p) xr[p] = *reinterpret_cast<const u32x4*>(xsrc[p] + (int64_t)tile * PBK);
    };
    auto fetch_q = [&](uint32_t (&q)[2], int tile) {
        const int64_t wbase = (int64_t)(tile >> 1) * qstep_even + (tile & 1) * qstep_odd;
        q[0] = wsrc[wbase];
        q[1] = BITS == 2 ? 0u : wsrc[wbase + 1];
    };
    // LDS address of the table entry of code j (0..15) of the fetched quarter
    auto entry_addr = [&](uint32_t lo, uint32_t hi, int j) -> uint32_t {
        constexpr uint32_t mask = (uint32_t)(L - 1) << 7;
        const int bit = BITS * j;
        uint32_t v;
        if (bit + BITS <= 32) v = bit >= 7 ? lo >> (bit - 7) : lo << (7 - bit);
        else if (bit >= 32) v = bit - 32 >= 7 ? hi >> (bit - 32 - 7) : hi << (7 - (bit - 32));
        else v = __builtin_amdgcn_alignbit(hi, lo, bit) << 7;
        return (v & mask) | tbase;
    };
    // NOLUT: codes 2p, 2p + 1 of a word of eight as the bf16 pair (128 + c, 128 + c')
    auto grid_pair = [&](uint32_t w, int pi) -> uint32_t {
        const uint32_t t = w >> (8 * pi);
        return (t & 0xFu) | ((t << 12) & 0xF0000u) | 0x43004300u;
    };
    auto code_words = [&](const uint32_t (&q)[2], uint32_t& lo, uint32_t& hi) {
        lo = q[0]; hi = q[1];
        if constexpr (BITS == 3) {
            const unsigned long long v = (((unsigned long long)hi << 32) | lo) >> qshift;
            lo = (uint32_t)v; hi = (uint32_t)(v >> 32);
        }
    };

    // ---- one K step: matrix cores on buffer BUF, staging of the next step into buffer BUF ^ 1.
    //      FIRST: the step starts a group (its first MFMAs take a zero accumulator); FOLD: it ends
    //      one (acc += scale * part).  q: the codes of the step being staged; qn / tile_q: the set
    //      freed by this step's staging is refilled with the codes of step tile_q.
    auto step = [&](auto buf_, auto first_, auto fold_, uint32_t (&q)[2], int tile_q, int tile_x, uint32_t sraw0, uint32_t sraw1) {
        constexpr int BUF = decltype(buf_)::value;
        constexpr bool FIRST = decltype(first_)::value, FOLD = decltype(fold_)::value;
        op16x8 a[2][2], b[2][2];
        uint32_t lk[2][8], wpk[4];
        uint32_t lo, hi;
        auto read_ops = [&](int set, int kk) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[set][i] = __builtin_bit_cast(op16x8, *reinterpret_cast<lds_u4>(ard + BUF * kXBuf + i * (32 * PLD * 2) + kk * 32));
                b[set][i] = __builtin_bit_cast(op16x8, *reinterpret_cast<lds_u4>(brd + BUF * kWBuf + i * (32 * PLD * 2) + kk * 32));
            }
        };
        auto w_issue = [&](int c, int h) {                      // four of the eight lookups of chunk c
            if constexpr (NOLUT) return;
#pragma unroll
            for (int t = 0; t < 4; ++t) lk[c][h * 4 + t] = *reinterpret_cast<lds_u32>(entry_addr(lo, hi, c * 8 + h * 4 + t));
        };
        auto w_finish = [&](int c, int h) {                     // pack half of chunk c; then the 16-byte write
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                if constexpr (NOLUT) wpk[h * 2 + t] = grid_pair(c ? hi : lo, h * 2 + t);
                else wpk[h * 2 + t] = lk[c][h * 4 + 2 * t] | (lk[c][h * 4 + 2 * t + 1] << 16);
            }
            if (h == 1)
                *reinterpret_cast<lds_u4>(wwr + (BUF ^ 1) * kWBuf + c * 16) = u32x4{wpk[0], wpk[1], wpk[2], wpk[3]};
        };
        auto x_write = [&](int p) {
            *reinterpret_cast<lds_u4>(xwr + (BUF ^ 1) * kXBuf + p * (64 * PLD * 2)) = xr[p];
        };
        float s0 = 0.f, s1 = 0.f;
        auto fold = [&](int t) {
            const int i = t >> 1, j = t & 1;
            const float s = j ? s1 : s0;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = __builtin_fmaf(part[i][j][v], s, acc[i][j][v]);
        };

        read_ops(0, 0);
        code_words(q, lo, hi);
        w_issue(0, 0);
        w_issue(0, 1);
        ANY4_SB();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int cur = kk & 1;
            if (kk < 3) read_ops(cur ^ 1, kk + 1);
            ANY4_SB();
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int i = t >> 1, j = t & 1;
                part[i][j] = mma(a[cur][i], b[cur][j], (FIRST && kk == 0) ? zero : part[i][j]);
                if (kk == 0) {
                    if (t < 2) w_finish(0, t);
                    else w_issue(1, t - 2);
                } else if (kk == 1) {
                    if (t < 2) w_finish(1, t);
                    else if (t == 2) fetch_q(q, tile_q);        // the set is free: its codes are in lo / hi and used up
                } else if (kk == 2) {
                    x_write(t);
                    if (t == 3) fetch_x(tile_x);                // the registers are free again: a full K step of lead
                } else if (FOLD) {
                    // the scales were fetched two K steps ago; widening them here, not earlier,
                    // keeps the wait for that fetch away from the start of the group
                    if (t == 1) { s0 = h16_to_f32<F16>(sraw0); s1 = h16_to_f32<F16>(sraw1); }
                    if (t >= 2) fold(t - 2);
                }
                ANY4_SB();
            }
        }
        if constexpr (FOLD) { fold(2); fold(3); }
    };
    // matrix cores on buffer 0, accumulating straight into acc (the offset steps: nothing to scale)
    auto mma_plain = [&]() {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            op16x8 a[2], b[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                a[i] = __builtin_bit_cast(op16x8, *reinterpret_cast<lds_u4>(ard + i * (32 * PLD * 2) + kk * 32));
                b[i] = __builtin_bit_cast(op16x8, *reinterpret_cast<lds_u4>(brd + i * (32 * PLD * 2) + kk * 32));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = mma(a[i], b[j], acc[i][j]);
        }
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    using Yes = std::true_type;
    using No = std::false_type;

    uint32_t q0[2], q1[2];
    fetch_x(S0);                                               // in flight while the tables are filled
    fetch_q(q0, S0);
    fetch_q(q1, S0 + 1);
    // per-row tables of this block's weight rows (rows past N are clamped: they are never stored):
    // one thread fetches 8 bytes (4 entries) of a row and writes each entry's 4 adjacent copies at once
    if constexpr (!NOLUT) {
        constexpr int PIECES = L / 4;                            // 8-byte pieces per row
        for (int i = tid; i < PBN * PIECES; i += PTHREADS) {
            const int row = i / PIECES, pc = i % PIECES;
            uint2 v;
            if (lut) v = *reinterpret_cast<const uint2*>(lut + (one_table ? 0 : min(n0 + row, N - 1) * L) + pc * 4);
            else {                                             // no table: the integer grid, entries pc * 4 .. + 3
                const int c0 = pc * 4 - L / 2;
                v.x = f32_to_h16<F16>((float)c0) | (f32_to_h16<F16>((float)(c0 + 1)) << 16);
                v.y = f32_to_h16<F16>((float)(c0 + 2)) | (f32_to_h16<F16>((float)(c0 + 3)) << 16);
            }
            uint32_t* dst = table + (row >> 3) * (32 << BITS) + (pc * 4) * 32 + (row & 7) * 4;
            const uint32_t e0 = v.x & 0xFFFFu, e1 = v.x >> 16, e2 = v.y & 0xFFFFu, e3 = v.y >> 16;
            *reinterpret_cast<uint4*>(dst) = make_uint4(e0, e0, e0, e0);
            *reinterpret_cast<uint4*>(dst + 32) = make_uint4(e1, e1, e1, e1);
            *reinterpret_cast<uint4*>(dst + 64) = make_uint4(e2, e2, e2, e2);
            *reinterpret_cast<uint4*>(dst + 96) = make_uint4(e3, e3, e3, e3);
        }
    }
    lds_barrier();                                             // tables are written
    // K step 0 goes to buffer 0 with nothing to overlap with
    {
#pragma unroll
        for (int p = 0; p < 4; ++p) *reinterpret_cast<lds_u4>(xwr + p * (64 * PLD * 2)) = xr[p];
        uint32_t lo, hi;
        code_words(q0, lo, hi);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            if constexpr (NOLUT) {
                const uint32_t wd = c ? hi : lo;
                *reinterpret_cast<lds_u4>(wwr + c * 16) = u32x4{grid_pair(wd, 0), grid_pair(wd, 1), grid_pair(wd, 2), grid_pair(wd, 3)};
            } else {
                uint32_t v[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) v[t] = *reinterpret_cast<lds_u32>(entry_addr(lo, hi, c * 8 + t));
                *reinterpret_cast<lds_u4>(wwr + c * 16) =
                    u32x4{v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16)};
            }
        }
        fetch_q(q0, min(S0 + 2, T - 1));
        fetch_x(S0 + 1);
    }
    lds_barrier();

    // ---- main loop, one group of 128 (two K steps) per iteration.  Step s works on buffer s % 2 and
    //      stages step s + 1: activations fetched during step s - 1 (right after that step's LDS
    //      writes freed the registers), codes from set (s + 1) % 2, which it then refills with the
    //      codes of step s + 3.  The last step stages a repeat of step T - 1 into a buffer that is
    //      not read again.
    // FINE: both scales of a chunk in one aligned 4-byte load per column, fetched one chunk ahead (the
    // first fold comes three quarters of a K step after the top of the iteration: a load issued
    // there would be waited for together with everything issued since)
    uint32_t pn0 = 0, pn1 = 0;
    if constexpr (FINE) { pn0 = reinterpret_cast<const uint32_t*>(scol[0])[g_lo]; pn1 = reinterpret_cast<const uint32_t*>(scol[1])[g_lo]; }
    for (int g = g_lo; g < g_hi; ++g) {
        const int s = 2 * g;
        if constexpr (FINE) {
            const uint32_t p0 = pn0, p1 = pn1;
            const int gn = min(g + 1, g_hi - 1);
            pn0 = reinterpret_cast<const uint32_t*>(scol[0])[gn];
            pn1 = reinterpret_cast<const uint32_t*>(scol[1])[gn];
            step(B0{}, Yes{}, Yes{}, q1, min(s + 3, T - 1), min(s + 2, T - 1), p0 & 0xFFFFu, p1 & 0xFFFFu);
            lds_barrier();
            step(B1{}, Yes{}, Yes{}, q0, min(s + 4, T - 1), min(s + 3, T - 1), p0 >> 16, p1 >> 16);
            lds_barrier();
        } else {
            const uint32_t sraw0 = scol[0][g >> lr], sraw1 = scol[1][g >> lr];
            step(B0{}, Yes{}, No{}, q1, min(s + 3, T - 1), min(s + 2, T - 1), 0u, 0u);
            lds_barrier();
            step(B1{}, No{}, Yes{}, q0, min(s + 4, T - 1), min(s + 3, T - 1), sraw0, sraw1);
            lds_barrier();
        }
    }

    // ---- offset term: a few more K steps over the group dimension (activation group sums split into
    //      bf16 hi + lo in columns 2g, 2g+1; both columns meet offset[n][g]); unscaled
    const int og_lo = FINE ? 2 * g_lo : g_lo, og_hi = FINE ? 2 * g_hi : g_hi;      // this block's groups, in the units of xsums
    // NOLUT: three passes over the group sums - right operand offset, then -128 * scale and -8 * scale (the
    // bf16 scale with 7 / 3 added to its exponent and the sign flipped: exact)
    constexpr int kKinds = NOLUT ? 3 : 1;
#pragma unroll
    for (int kind = 0; kind < kKinds; ++kind)
    for (int k0 = 2 * og_lo / PBK * PBK; k0 < 2 * og_hi; k0 += PBK) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint16_t* src = xsums + min(m0 + p * 64 + xr_row, M - 1) * KP + xc8 * 8 + k0;
            xr[p] = k0 + xc8 * 8 < KP ? *reinterpret_cast<const u32x4*>(src) : u32x4{0, 0, 0, 0};
        }
        uint32_t pk[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int gg = (k0 + wq * 16 + 2 * j) >> 1;
            const bool in = gg >= og_lo && gg < og_hi;
            uint32_t b = in ? (kind == 0 ? offset : scale)[wn_glob * GS + (FINE ? gg : gg >> lr)] : 0u;
            if (kind == 1) b = in ? (b + 0x0380u) ^ 0x8000u : 0u;
            if (kind == 2) b = in ? (b + 0x0180u) ^ 0x8000u : 0u;
            pk[j] = b | (b << 16);
        }
#pragma unroll
        for (int p = 0; p < 4; ++p) *reinterpret_cast<lds_u4>(xwr + p * (64 * PLD * 2)) = xr[p];
        *reinterpret_cast<lds_u4>(wwr) = u32x4{pk[0], pk[1], pk[2], pk[3]};
        *reinterpret_cast<lds_u4>(wwr + 16) = u32x4{pk[4], pk[5], pk[6], pk[7]};
        lds_barrier();
        mma_plain();
        lds_barrier();
    }

    // ---- store (accumulator element v of a lane is row 8*(v/4) + 4*(lane/32) + v%4, column lane%32 of its
    //      32 x 32 tile)
    auto store_tile = [&](int i, int j, const f32x16& r) {
        const int64_t n = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int64_t m = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            if (m < M && n < N) y[m * N + n] = (uint16_t)f32_to_h16<F16>(r[v]);
        }
    };
    if (slice < 0) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) store_tile(i, j, acc[i][j]);
        return;
    }
    // ---- a K slice: its fp32 sums go to the workspace; the last slice of the tile to arrive adds them all
    float* mine = partial + ((int64_t)(tile - tail_first) * tail_s + slice) * (PBM * PBN);
    auto elem = [&](int i, int j, int v) -> int {
        return (wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3)) * PBN + wn * 64 + j * 32 + (lane & 31);
    };
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                // through an opaque copy: with the accumulator vector itself as the source of the atomic
                // stores the compiler copies all 64 accumulators inside the main loop on every iteration
                float t = acc[i][j][v];
                asm volatile("" : "+v"(t));
                splitk_store(mine + elem(i, j, v), t);
            }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // this thread's sums are out
    lds_barrier();                                             // ... and so are the whole block's
    int* flag = reinterpret_cast<int*>(smem);
    if (tid == 0) *flag = arrive_one(counters + (tile - tail_first), tail_s) ? 1 : 0;
    lds_barrier();
    if (*flag == 0) return;
    const float* all = partial + (int64_t)(tile - tail_first) * tail_s * (PBM * PBN);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            f32x16 sum;
#pragma unroll
            for (int v = 0; v < 16; ++v) sum[v] = 0.f;
            for (int sl = 0; sl < tail_s; sl += 2) {           // two slices' worth of loads in flight
                float a[16], b[16];
                const int sl1 = min(sl + 1, tail_s - 1);
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    a[v] = splitk_load(all + (int64_t)sl * (PBM * PBN) + elem(i, j, v));
                    b[v] = splitk_load(all + (int64_t)sl1 * (PBM * PBN) + elem(i, j, v));
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    sum[v] += a[v];
                    if (sl + 1 < tail_s) sum[v] += b[v];
                }
            }
            store_tile(i, j, sum);
        }
}

constexpr size_t prefill_lds_bytes(int bits) {
    return (size_t)kTableOff + (size_t)PBN * (1 << bits) * 4 * 4;
}

// Work split: whole tiles, and K slices for the tiles of a last round that would leave more than
// half of the compute units idle (also the only round of a small problem).
PrefillPlan plan_prefill(int64_t M, int64_t N, int64_t K, int cus) {
    PrefillPlan p{};
    const int64_t gm = (M + PBM - 1) / PBM, gn = (N + PBN - 1) / PBN, G = K / kGroup;
    p.gm = gm;
    p.tiles = gm * gn;
    p.tail_tiles = 0;
    p.tail_s = 1;
    const int64_t r = p.tiles % cus;
    if (r > 0) {
        int64_t sl = cus / r;
        if (sl > 8) sl = 8;
        if (sl > G / 4) sl = G / 4;                            // at least four groups (eight K steps) per slice
        if (sl >= 2) { p.tail_tiles = r; p.tail_s = (int)sl; }
    }
    // (sized for groups of 64, the largest case: the workspace does not depend on the group size)
    p.xsums_bytes = ((size_t)M * (size_t)prefill_kp(K, true) * sizeof(uint16_t) + 255) / 256 * 256;
    p.counter_bytes = p.tail_tiles ? splitk_counter_bytes(p.tail_tiles) : 0;
    p.partial_bytes = (size_t)p.tail_tiles * (size_t)p.tail_s * (PBM * PBN) * sizeof(float);
    return p;
}

size_t prefill_workspace_bytes(int64_t M, int64_t N, int64_t K, int cus) {
    const PrefillPlan p = plan_prefill(M, N, K, cus);
    return p.xsums_bytes + p.counter_bytes + p.partial_bytes;
}

hipError_t launch_prefill(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                          const uint16_t* scale, const uint16_t* offset,
                          int64_t M, int64_t N, int64_t K, int bits, int lr, bool repacked, bool f16, bool one_table, int cus,
                          uint16_t* y, void* workspace, hipStream_t stream) {
    const PrefillPlan pp = plan_prefill(M, N, K, cus);
    const bool fine = lr < 0;
    if (lr < -1 || (f16 && fine)) return hipErrorInvalidValue;
    const int64_t sblocks = (M * (K / 8) + 255) / 256;         // one lane per 8 activations
    const int64_t nblocks = pp.tiles - pp.tail_tiles + pp.tail_tiles * pp.tail_s;
    if (pp.gm > 0x7FFFFFFF || nblocks > 0x7FFFFFFF || sblocks > 0x7FFFFFFF || K / kGroup > 0x1FFFFFFF) return hipErrorInvalidValue;
    const int KP = prefill_kp(K, fine);
    uint16_t* xsums = static_cast<uint16_t*>(workspace);
    unsigned long long* counters = reinterpret_cast<unsigned long long*>(static_cast<char*>(workspace) + pp.xsums_bytes);
    float* partial = reinterpret_cast<float*>(static_cast<char*>(workspace) + pp.xsums_bytes + pp.counter_bytes);
    const dim3 grid((unsigned)nblocks), block(PTHREADS);
    const int gm = (int)pp.gm, tail_first = (int)(pp.tiles - pp.tail_tiles), tail_s = pp.tail_s;
    // the LDS limit first: whatever can be refused is refused before anything is enqueued
    hipError_t e = hipSuccess;
#define ANY4_PREFILL_F(B, F, H, NL)                                                                                 \
    do {                                                                                                          \
        e = ensure_lds<prefill_kernel<B, F, H, NL>>((int)prefill_lds_bytes(B));                                       \
        if (e != hipSuccess) return e;                                                                            \
        if (f16) hipLaunchKernelGGL(group_sums_kernel<true>, dim3((unsigned)sblocks), dim3(256), 0, stream, x, M, K, KP, 0, xsums); \
        else hipLaunchKernelGGL(group_sums_kernel<false>, dim3((unsigned)sblocks), dim3(256), 0, stream, x, M, K, KP, fine ? 1 : 0, xsums); \
        e = hipGetLastError();                                                                                    \
        if (e != hipSuccess) return e;                                                                            \
        hipLaunchKernelGGL((prefill_kernel<B, F, H, NL>), grid, block, prefill_lds_bytes(B), stream, x, codes, lut, scale, \
                           offset, xsums, KP, M, N, K, F ? 0 : lr, (repacked ? 1 : 0) | (one_table ? 2 : 0), gm, tail_first, tail_s, counters, partial, y); \
    } while (0)
#define ANY4_PREFILL(B)                                                                                           \
    do {                                                                                                          \
        if (B == 4 && !lut && !f16 && !fine && lr == 0) ANY4_PREFILL_F(4, false, false, true);                    \
        else if (f16) ANY4_PREFILL_F(B, false, true, false);                                                             \
        else if (fine) ANY4_PREFILL_F(B, true, false, false);                                                            \
        else ANY4_PREFILL_F(B, false, false, false);                                                                     \
    } while (0)
    switch (bits) {
        case 4: ANY4_PREFILL(4); break;
        case 3: ANY4_PREFILL(3); break;
        default: ANY4_PREFILL(2); break;
    }
#undef ANY4_PREFILL_F
#undef ANY4_PREFILL
    return hipGetLastError();
}

}  // namespace any4
