// Memory-bound any-n GEMM (n = 4, 3, 2) for very small M (1 <= M <= 4, token generation): the whole
// K axis inside one block, no K slabs, no workspace.
//
// y[m][n] = sum_k x[m][k] * (LUT[n][code[n][k]] * scale[n][k/128] + offset[n][k/128])
// (any4 paper, section 4.2 for y = x w^T with on-the-fly dequantisation, sections 2.4.1 and 2.5.2
// for the per-row table and alpha * w_Q + beta).
//
// Lookup and contraction are those of the streaming kernel for M <= 16 (any4_decode_stream.hip): a
// block works on 16 weight rows (a tile) at a time, lane l of every wavefront on row n = l % 16 and
// quarter q = l / 16 of a group of 128 codes; a conflict-free pair table in LDS turns a byte of
// codes into two bf16 weights that are already a matrix-core B operand; v_mfma_f32_16x16x32_bf16
// multiplies them by the activations; scale and offset are applied to group sums, never to weights.
//
// What differs is the A operand.  With M rows of x, 16 - M of the 16 operand rows of the matrix
// instruction are zero and so are their registers.  Here the operand rows hold DIFFERENT GROUPS
// instead: with MP = 1, 2 or 4 rows of x (M rounded up to a power of two), operand row r holds row
// r % MP of x restricted to group (r / MP) of a set of P = 16 / MP consecutive groups.  The four matrix
// instructions of group s of the set then leave the wanted partial sums in output rows
// s * MP .. s * MP + MP - 1 and unwanted products (other groups' activations with this group's
// weights) in the others; an accumulator lane holds output rows 4 q' .. 4 q' + 3, so the lanes of
// one quarter q' pick the wanted rows with their group's scale and everybody else adds zero.
// One register set (16 registers) so carries the activations of 16 / MP groups: a wavefront can
// own a sixteenth of a row of 64 K weights at M = 1 with 32 registers, which is what lets a block
// of 8 wavefronts walk over the WHOLE K axis: no slabs, no partial sums in global memory, no
// arrival counters, and the per-tile costs (table build, barrier) are paid once per 16 rows x K.
// The registers this saves also allow two blocks per compute unit, so that one block's barrier,
// table build and small reductions overlap with the other block's streaming.
//
// Work split.  Wavefront w owns the 4 * PASSES consecutive groups starting at 4 * PASSES * w
// (PASSES = ceil(K / 4096), at most 8: K <= 32768).  A tile is processed in PASSES units of 4
// groups per wavefront; the codes of a unit are 16 bytes per lane and group, held in a ring of two
// units that is refilled for unit u + 2 as soon as the lookup addresses of unit u are formed.  The
// ring runs across tile boundaries.
//
// Small per-tile inputs (the rows' tables, scales and offsets: 6 % of the bytes) are not read by every
// wavefront: a load instruction that picks 8 or 16 bytes out of each of 16 rows costs the memory
// pipeline as much as one that brings a kilobyte of codes.  They are fetched three tiles ahead with
// 2 * PASSES + 1 sixteen-byte-per-lane instructions per tile, dealt out over the wavefronts in turn,
// parked in registers for one tile and then written to one of three LDS slots; every wavefront reads
// what it needs from the slot just before it uses it (a lane needs the scales only of the groups whose
// wanted rows it holds: 8 bytes per 16 groups at M = 1, and 16 bytes of offsets per 16 groups).
// Block b takes tiles b, b + blocks, b + 2 blocks, ...
#pragma once
#include "any4_device.h"
#include "any4_internal.h"
#include <type_traits>
#include <utility>

namespace any4 {

namespace pack {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kTile = 16;                              // weight rows per tile
constexpr int kWaves = 8;                              // wavefronts per block
constexpr int kThreads = kWaves * 64;
constexpr int kSlots = 3;                              // LDS slots of small inputs (tiles t, t + 1, t + 2)
constexpr int kLdsPerCu = 160 * 1024;
// LDS bytes of the two table buffers: any4 256 pair entries x (2 buffers x 16 rows x 2 copies x 4 B), any3
// the same with 64 entries, any2 256 quad entries x (16 rows x 2 copies x 8 B) per buffer
constexpr int table_bytes(int bits) { return bits == 4 ? 256 * 256 : (bits == 3 ? 64 * 256 : 2 * 256 * 256); }
// partial sums [2][kWaves][MP][16] fp32; the same bytes hold the group sums of x [kWaves][MP][32] before the first tile
constexpr int red_bytes(int mp) { return 2 * kWaves * mp * 16 * 4; }
// A operands of the offset MFMAs: [kWaves][NOF][MP rows][4 quarters] of 16 bytes
constexpr int xo_bytes(int mp, int passes) { return kWaves * ((4 * passes + 15) / 16) * mp * 4 * 16; }
// one slot: scales [16 rows][G bf16 + 8 bytes of padding against bank conflicts], offsets the same, tables
// [16 rows][32 bytes]
constexpr int aux_row_bytes(int G) { return G * 2 + 8; }
constexpr int slot_bytes(int G) { return 2 * kTile * aux_row_bytes(G) + kTile * 32; }
constexpr int lds_bytes(int bits, int mp, int passes, int G) {
    return table_bytes(bits) + red_bytes(mp) + xo_bytes(mp, passes) + kSlots * slot_bytes(G);
}
// Two blocks per compute unit (4 wavefronts per SIMD, 128 registers each) where LDS holds two for every K
// the variant serves and the activations of a wavefront's groups are one register set; otherwise one
// block with up to 256 registers per lane.
constexpr bool two_blocks(int bits, int mp, int passes) {
    return (4 * passes + 16 / mp - 1) / (16 / mp) == 1 && (mp == 1 || passes == 1) && passes <= 3 &&
           2 * lds_bytes(bits, mp, passes, 32 * passes) <= kLdsPerCu;
}
constexpr int waves_per_eu(int bits, int mp, int passes) { return (two_blocks(bits, mp, passes) ? 2 : 1) * kWaves / 4; }

struct Params {
    const uint16_t* x;
    const uint32_t* codes;
    const uint16_t* lut;
    const uint16_t* scale;
    const uint16_t* offset;
    uint16_t* y;
    int64_t N, K;
    int M, G;                        // G = K / 128, a multiple of 8
    int tiles;                       // 16-row tiles
    int nblocks;                     // grid size
    int tpb, trem;                   // tiles = nblocks * tpb + trem: the first trem blocks get tpb + 1 tiles
    int codes_bytes, lut_bytes, so_bytes;    // sizes of the arrays (each below 2 GiB)
    int one_table;                   // lut holds ONE row that serves every row of the matrix (built once per block)
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant expression
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// LDS barrier that does not wait for outstanding global loads (the prefetched codes stay in flight)
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// fp32 -> bf16, round to nearest even, for finite values (the group sums of the activations)
__device__ __forceinline__ uint32_t bf16_rne_finite(float f) {
    const uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// BITS    code width: 4, 3 or 2
// MP      rows of x rounded up to a power of two: 1, 2 or 4
// PASSES  units of 4 groups a wavefront processes per tile: 8 wavefronts x 4 x PASSES groups cover K
// REPACK  codes in the tile-major layout of any4_repack
template <int BITS, int MP, int PASSES, bool REPACK>
__global__ __launch_bounds__(kThreads, waves_per_eu(BITS, MP, PASSES)) void decode_pack_kernel(const Params p) {
    static_assert(BITS == 4 || BITS == 3 || BITS == 2, "code width");
    static_assert(MP == 1 || MP == 2 || MP == 4, "rows of x, rounded up");
    constexpr int P = 16 / MP;                           // groups per register set of activations
    constexpr int GPW = 4 * PASSES;                      // groups per wavefront
    constexpr int NCH = (GPW + P - 1) / P;               // register sets of activations
    constexpr int NOF = (GPW + 15) / 16;                 // offset MFMAs per tile
    constexpr int NSC = 4 / MP;                          // scales a lane needs per register set
    constexpr int NG = 4 * PASSES;                       // groups per wavefront and tile, in processing order
    constexpr int QW = BITS;                             // 32-bit words of a lane's quarter group (32 codes)
    constexpr int QB = 4 * BITS, GB = 16 * BITS;         // bytes of a quarter group / of a group, per row
    constexpr int LUTB = 2 << BITS;                      // bytes of a row's table
    constexpr int NI = 2 * PASSES + 1;                   // load instructions that fetch a tile's small inputs
    constexpr int KI = (NI + kWaves - 1) / kWaves;       // ... of which a wavefront issues at most this many
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* const red = reinterpret_cast<float*>(smem + table_bytes(BITS));
    unsigned char* const xo_lds = smem + table_bytes(BITS) + red_bytes(MP);
    unsigned char* const slots = xo_lds + xo_bytes(MP, PASSES);

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, q = lane >> 4;

    // tiles of this block: tiles bid, bid + nblocks, bid + 2 nblocks, ... - tpb or tpb + 1 of them (no division
    // here: 64-bit divisions are hundreds of scalar instructions at the start of every block).  At any
    // moment the blocks so read one contiguous window of the matrix between them, which measured 3 %
    // faster on the row-major layout than a contiguous range of tiles per block and the same on the
    // re-laid-out one.  Tile number li of the block is tile_of(li); li >= ntiles is "past the end".
    const int bid = (int)blockIdx.x;
    const int ntiles = p.tpb + (bid < p.trem ? 1 : 0);
    if (ntiles < 1) return;
    auto tile_of = [&](int li) -> int { return bid + li * p.nblocks; };

    const int M = p.M, G = p.G;
    const int64_t N = p.N, K = p.K;
    const int aux_row = aux_row_bytes(G), slot_size = slot_bytes(G);
    // groups of this wavefront: G is a multiple of 4, so a unit of 4 groups exists entirely or not at all.
    // A wavefront (or unit) without groups reads the codes of a group that exists and multiplies them by
    // zero activations: every load stays unconditional and inside the arrays.
    const int ngw = max(0, min(GPW, G - w * GPW));
    const int gbase = ngw > 0 ? w * GPW : 0;
    const int gmaxl = max(ngw, 1) - 1;

    // Every array is read through a buffer descriptor: a load is "descriptor + scalar offset (tile, group) +
    // 32-bit lane offset", so the address arithmetic stays in scalar registers and a lane keeps one
    // offset register per array instead of a 64-bit address per load.  (The host side refuses arrays of
    // 2 GiB and more, so every offset fits 32 bits.)  In the problem's last tile the rows past N are
    // clamped to row N - 1 (read, never stored).
    constexpr int kRsrcFlags = 0x00020000;               // raw buffer, 32-bit data format
    const __amdgpu_buffer_rsrc_t codes_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p.codes), 0, p.codes_bytes, kRsrcFlags);
    const int last_tile = p.tiles - 1;
    const int rows_last = (int)(N - (int64_t)last_tile * kTile);             // rows of the problem's last tile
    const uint32_t row_bytes = (uint32_t)(K * BITS / 8);
    const uint32_t tile_code_bytes = (uint32_t)kTile * row_bytes;
    // row of this lane inside tile t (its own, or the tile's last row past the end of the matrix)
    auto row_in = [&](int t) -> uint32_t { return (uint32_t)min(n, (t == last_tile ? rows_last : kTile) - 1); };

    // ---- codes: a ring of two units; one lane holds the QW words of its quarter of each of the unit's 4 groups
    struct Quarter { uint32_t w[QW]; };
    Quarter cw[2][4];
    // (A unit of 4 groups exists entirely or not at all.  The scalar offset names the tile and the unit, the
    // group inside the unit is a constant that the load instruction carries itself.  A load that is not
    // wanted - a unit the wavefront does not have, a tile past the block's last - gets a lane offset
    // beyond the end of the descriptor: the hardware's range check then returns zeros without touching
    // memory, and the instruction stream stays free of branches.)
    constexpr uint32_t kGroupStride = REPACK ? 64 * QB : GB;
    constexpr uint32_t kOutOfRange = 0x80000000u;        // every array is shorter than this
    const int nunits = ngw / 4;
    auto load_codes = [&](Quarter& c, int li, int pp, int gi) {
        const int t = tile_of(li);
        const bool wanted = pp < nunits && li < ntiles;
        const uint32_t so = (uint32_t)t * tile_code_bytes + (uint32_t)(gbase + 4 * pp) * kGroupStride;
        const uint32_t lane_off = REPACK ? (uint32_t)lane * QB : row_in(t) * row_bytes + (uint32_t)q * QB;
        const uint32_t vo = (wanted ? lane_off : kOutOfRange) + (uint32_t)gi * kGroupStride;
        // the re-laid-out codes are read exactly once and whole cache lines per instruction: nontemporal
        constexpr int aux = REPACK ? 2 : 0;
        if constexpr (BITS == 4) {
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(codes_r, vo, so, aux);
            c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2]; c.w[3] = v[3];
        } else if constexpr (BITS == 3) {
            const auto v = __builtin_amdgcn_raw_buffer_load_b96(codes_r, vo, so, aux);
            c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2];
        } else {
            const auto v = __builtin_amdgcn_raw_buffer_load_b64(codes_r, vo, so, aux);
            c.w[0] = v[0]; c.w[1] = v[1];
        }
    };

    // ---- small inputs of a tile.  Instruction j of a tile's NI is issued by the wavefront with
    //      (w - t) % 8 == j % 8:  j < PASSES fetches pieces 4 j .. 4 j + 3 (16 bytes = 8 groups each) of the
    //      16 rows' scales, lane (n, sub) piece 4 j + sub of row n;  PASSES <= j < 2 PASSES the same of
    //      the offsets;  j = 2 PASSES the rows' tables (any4: lane (n, half) with half < 2; any3: 16 bytes
    //      a row; any2: the aligned 16 bytes that hold the row's 8).  A wavefront whose turn it is not, and
    //      lanes without a piece, issue the load with an out-of-range offset and write nothing.
    struct Stage { u32x4 v[KI]; };
    auto stage_load = [&](Stage& s, int li) {
        const int t = tile_of(li);
        const int r = (w - li) & (kWaves - 1);
#pragma unroll
        for (int k = 0; k < KI; ++k) {
            const int jr = r + kWaves * k;                                  // wave-uniform
            const int j = min(jr, NI - 1);
            const bool is_lut = j == 2 * PASSES;
            const bool is_off = !is_lut && j >= PASSES;
            const uint16_t* base = is_lut ? p.lut : (is_off ? p.offset : p.scale);
            const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(base), 0,
                                                                                is_lut ? p.lut_bytes : p.so_bytes, kRsrcFlags);
            const uint32_t row = (uint32_t)t * kTile + row_in(t);
            const uint32_t piece = (uint32_t)((j - (is_off ? PASSES : 0)) * 4 + q);
            uint32_t vo = row * (uint32_t)(G * 2) + piece * 16u;
            bool wanted = jr < NI && li < ntiles && piece < (uint32_t)(G / 8);
            if (is_lut) {
                wanted = jr < NI && li < ntiles && q < (BITS == 4 ? 2 : 1) && !p.one_table;
                if constexpr (BITS == 4) vo = row * 32u + (uint32_t)(q & 1) * 16u;
                else if constexpr (BITS == 3) vo = row * 16u;
                else vo = min((row * 8u) & ~15u, (uint32_t)p.lut_bytes - 16u);
            }
            s.v[k] = __builtin_amdgcn_raw_buffer_load_b128(rs, wanted ? vo : kOutOfRange, 0, 0);
        }
    };
    auto stage_write = [&](const Stage& s, int li, int slot) {
        if (li >= ntiles) return;
        const int t = tile_of(li);
        const int r = (w - li) & (kWaves - 1);
        unsigned char* const sb = slots + slot * slot_size;
#pragma unroll
        for (int k = 0; k < KI; ++k) {
            const int j = r + kWaves * k;
            if (j >= NI) continue;
            if (j == 2 * PASSES) {
                unsigned char* dst = sb + 2 * kTile * aux_row + n * 32;
                if constexpr (BITS == 4) { if (q < 2) *reinterpret_cast<u32x4*>(dst + q * 16) = s.v[k]; }
                else if constexpr (BITS == 3) { if (q < 1) *reinterpret_cast<u32x4*>(dst) = s.v[k]; }
                else {
                    // the row's 8 bytes are the lower or the upper half of the 16 that were fetched
                    const uint32_t rowb = ((uint32_t)t * kTile + row_in(t)) * 8u;
                    const bool upper = rowb - min(rowb & ~15u, (uint32_t)p.lut_bytes - 16u) != 0u;
                    if (q < 1) *reinterpret_cast<uint2*>(dst) = upper ? make_uint2(s.v[k][2], s.v[k][3]) : make_uint2(s.v[k][0], s.v[k][1]);
                }
            } else {
                const int jb = j >= PASSES ? j - PASSES : j;
                const int piece = jb * 4 + q;
                unsigned char* dst = sb + (j >= PASSES ? kTile * aux_row : 0) + n * aux_row + piece * 16;
                if (piece < G / 8) {                                // (rows are 8-byte aligned in the slot)
                    reinterpret_cast<uint2*>(dst)[0] = make_uint2(s.v[k][0], s.v[k][1]);
                    reinterpret_cast<uint2*>(dst)[1] = make_uint2(s.v[k][2], s.v[k][3]);
                }
            }
        }
    };

    // ---- table source of a tile.  The entries of a row are written by its 32 threads (w, q):
    //   any4: 256 pair entries (hi << 4 | lo): thread writes hi = 2w + q/2, lo = 8 (q % 2) .. + 8
    //   any3:  64 pair entries (hi << 3 | lo): thread writes hi = w,        lo = 2q, 2q + 1
    //   any2: 256 quad entries (c3 c2 c1 c0):  thread writes entries 8 (4w + q) .. + 8
    // LutSrc holds the part of the row's table a thread needs for that.
    struct LutSrc { uint32_t a[BITS == 4 ? 4 : (BITS == 3 ? 1 : 2)]; uint32_t h; };
    const uint32_t lut_lo_off = BITS == 4 ? (uint32_t)(q & 1) * 16u : (BITS == 3 ? (uint32_t)q * 4u : 0u);
    const uint32_t lut_hi_off = BITS == 4 ? (uint32_t)w * 4u : (uint32_t)(w >> 1) * 4u;
    // from a row of the table in an LDS slot
    auto read_lut = [&](LutSrc& l, int slot) {
        const unsigned char* row = slots + slot * slot_size + 2 * kTile * aux_row + n * 32;
        if constexpr (BITS == 4) {
            const uint4 v = *reinterpret_cast<const uint4*>(row + lut_lo_off);
            l.a[0] = v.x; l.a[1] = v.y; l.a[2] = v.z; l.a[3] = v.w;
            l.h = *reinterpret_cast<const uint32_t*>(row + lut_hi_off);
        } else if constexpr (BITS == 3) {
            l.a[0] = *reinterpret_cast<const uint32_t*>(row + lut_lo_off);
            l.h = *reinterpret_cast<const uint32_t*>(row + lut_hi_off);
        } else {
            const uint2 v = *reinterpret_cast<const uint2*>(row);
            l.a[0] = v.x; l.a[1] = v.y; l.h = 0;
        }
    };
    // straight from memory (the first tile of a block)
    auto load_lut = [&](LutSrc& l, int li) {
        const int t = tile_of(li);
        const __amdgpu_buffer_rsrc_t lut_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.lut), 0, p.lut_bytes, kRsrcFlags);
        const uint32_t vo = p.one_table ? 0u : ((uint32_t)t * kTile + row_in(t)) * LUTB;
        if constexpr (BITS == 4) {
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(lut_r, vo + lut_lo_off, 0, 0);
            l.a[0] = v[0]; l.a[1] = v[1]; l.a[2] = v[2]; l.a[3] = v[3];
            l.h = __builtin_amdgcn_raw_buffer_load_b32(lut_r, vo + lut_hi_off, 0, 0);
        } else if constexpr (BITS == 3) {
            l.a[0] = __builtin_amdgcn_raw_buffer_load_b32(lut_r, vo + lut_lo_off, 0, 0);
            l.h = __builtin_amdgcn_raw_buffer_load_b32(lut_r, vo + lut_hi_off, 0, 0);
        } else {
            const auto v = __builtin_amdgcn_raw_buffer_load_b64(lut_r, vo, 0, 0);
            l.a[0] = v[0]; l.a[1] = v[1]; l.h = 0;
        }
    };
    // table of a tile into buffer `par`
    auto build_table = [&](const LutSrc& l, int par) {
        uint32_t* const tab = reinterpret_cast<uint32_t*>(smem);
        if constexpr (BITS == 4) {
            // entry e of row n at dword e * 64 + par * 32 + n * 2, both copies
            const uint32_t hv = (q & 2) ? (l.h & 0xFFFF0000u) : (l.h << 16);
            uint32_t* dst = tab + ((2 * w + (q >> 1)) * 16 + 8 * (q & 1)) * 64 + par * 32 + n * 2;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t lv = (i & 1) ? (l.a[i >> 1] >> 16) : (l.a[i >> 1] & 0xFFFFu);
                *reinterpret_cast<uint2*>(dst + i * 64) = make_uint2(lv | hv, lv | hv);
            }
        } else if constexpr (BITS == 3) {
            const uint32_t hv = (w & 1) ? (l.h & 0xFFFF0000u) : (l.h << 16);
            uint32_t* dst = tab + (w * 8 + 2 * q) * 64 + par * 32 + n * 2;
            const uint32_t v0 = (l.a[0] & 0xFFFFu) | hv, v1 = (l.a[0] >> 16) | hv;
            *reinterpret_cast<uint2*>(dst) = make_uint2(v0, v0);
            *reinterpret_cast<uint2*>(dst + 64) = make_uint2(v1, v1);
        } else {
            // entry e of row n at dword e * 64 + par * 16384 + n * 4, both copies (16 bytes); the table words
            // are copied into scalars first: a choice between them by a lane-dependent index would
            // otherwise go through a copy of the struct in scratch memory
            const uint32_t a0 = l.a[0], a1 = l.a[1];
            auto val = [&](int c) -> uint32_t { return ((c & 2) ? a1 : a0) >> (16 * (c & 1)) & 0xFFFFu; };
            auto valv = [&](uint32_t c) -> uint32_t {
                const uint32_t d = (c & 2u) ? a1 : a0;
                return (c & 1u) ? (d >> 16) : (d & 0xFFFFu);
            };
            const uint32_t d1 = valv(((uint32_t)(w & 1) << 1) | (uint32_t)(q >> 1)) | (valv((uint32_t)(w >> 1)) << 16);
            uint32_t* dst = tab + ((4 * w + q) * 8) * 64 + par * 16384 + n * 4;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const uint32_t d0 = val(i & 3) | (valv(((uint32_t)(q & 1) << 1) | (uint32_t)(i >> 2)) << 16);
                *reinterpret_cast<uint4*>(dst + i * 64) = make_uint4(d0, d1, d0, d1);
            }
        }
    };

    // ---- scales from a slot: lane (n, q) holds the wanted output rows of the groups c * P + q * NSC .. + NSC
    //      of register set c, and needs only their scales: 2 * NSC contiguous bytes per set
    struct Scales { uint32_t v[NCH][NSC == 4 ? 2 : 1]; };
    const uint32_t sc_lane = (uint32_t)q * NSC;
    auto read_scales = [&](Scales& s, int slot) {
        const unsigned char* row = slots + slot * slot_size + n * aux_row;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const uint32_t gl = min((uint32_t)(c * P) + sc_lane, (uint32_t)(max(ngw, 4) - NSC));
            const unsigned char* a = row + ((uint32_t)gbase + gl) * 2u;
            if constexpr (NSC == 4) {
                const uint2 v = *reinterpret_cast<const uint2*>(a);
                s.v[c][0] = v.x; s.v[c][1] = v.y;
            } else if constexpr (NSC == 2) {
                s.v[c][0] = *reinterpret_cast<const uint32_t*>(a);
            } else {
                s.v[c][0] = *reinterpret_cast<const uint16_t*>(a);
            }
        }
    };
    // ---- offsets as the B operand of offset MFMA c: the hi parts of the group sums of local groups 16 c .. + 16
    //      sit in k-slots 0 .. 15 and their lo parts in k-slots 16 .. 31; lane (n, q) holds k-slots 8 q .. 8 q + 7,
    //      i.e. the offsets of groups 16 c + 8 (q % 2) .. + 8 of its row: two 8-byte reads, both clamped to
    //      groups the wavefront has (a clamped offset meets a zero group sum)
    auto read_offsets = [&](int c, int slot) -> uint4 {
        const unsigned char* row = slots + slot * slot_size + kTile * aux_row + n * aux_row;
        const uint32_t hi_grp = (uint32_t)(max(ngw, 4) - 4);
        const uint32_t g0 = min((uint32_t)(c * 16) + (uint32_t)(q & 1) * 8u, hi_grp);
        const uint32_t g1 = min((uint32_t)(c * 16) + (uint32_t)(q & 1) * 8u + 4u, hi_grp);
        const uint2 a = *reinterpret_cast<const uint2*>(row + ((uint32_t)gbase + g0) * 2u);
        const uint2 b = *reinterpret_cast<const uint2*>(row + ((uint32_t)gbase + g1) * 2u);
        return make_uint4(a.x, a.y, b.x, b.y);
    };

    // ---- prologue: everything the first tiles need is requested at once
    // activations as packed A operands: lane (r, q), set c, MFMA j holds x[r % MP][(group c * P + r / MP) * 128 +
    // q * 32 + j * 8 .. + 8]; rows >= M and groups the wavefront does not have are zero
    uint4 xa[NCH][4];
    {
        const int xm = n % MP, xs = n / MP;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int gl = c * P + xs;
            const bool valid = gl < ngw && xm < M;
            const uint16_t* src = p.x + (int64_t)min(xm, M - 1) * K + (int64_t)(gbase + min(gl, gmaxl)) * kGroup + q * 32;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint4 v = *reinterpret_cast<const uint4*>(src + j * 8);
                xa[c][j] = valid ? v : make_uint4(0, 0, 0, 0);
            }
        }
    }
    LutSrc lsrc;
    load_lut(lsrc, 0);                                   // the first table comes straight from memory
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) load_codes(cw[0][gi], 0, 0, gi);
    Stage st, st1, st2;
    stage_load(st, 0);
#pragma unroll
    for (int gi = 0; gi < 4; ++gi) {
        if constexpr (PASSES == 1) load_codes(cw[1][gi], 1, 0, gi);
        else load_codes(cw[1][gi], 0, 1, gi);
    }
    stage_load(st1, 1);
    stage_load(st2, 2);

    // group sums of the activations.  With an all-ones A operand and a register set as B operand the
    // matrix cores return, in every lane of column r, the sum of operand row r: the sum of row r % MP
    // of x over group c * P + r / MP.  They go through LDS (this wavefront's slice of the partial-sum
    // buffer, idle until the first tile ends) to the layout of the offset MFMAs' A operands: lane (m, q)
    // of MFMA c holds, for local groups 16 c + 8 (q % 2) .. + 8, the bf16 high parts (q < 2) or the bf16
    // low parts (q >= 2) of the sums of row m.  Only rows < M are non-zero, so the operands are kept in
    // LDS as [NOF][MP][4] pieces of 16 bytes per wavefront and re-read once per tile.
    unsigned char* const xo_w = xo_lds + w * (NOF * MP * 4 * 16);
    {
        float* const xsum = red + w * (MP * 32);                             // [MP][32], this wavefront only
        if (lane < MP * 32 / 2) reinterpret_cast<float2*>(xsum)[lane] = make_float2(0.f, 0.f);
        const uint4 ones = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
        const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            f32x4 gs = z4;
#pragma unroll
            for (int j = 0; j < 4; ++j) gs = mfma16(ones, xa[c][j], gs);
            if (q == 0) xsum[(n % MP) * 32 + c * P + n / MP] = gs[0];
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        if (n < MP) {
#pragma unroll
            for (int c = 0; c < NOF; ++c) {
                const float4 a = *reinterpret_cast<const float4*>(xsum + n * 32 + c * 16 + (q & 1) * 8);
                const float4 b = *reinterpret_cast<const float4*>(xsum + n * 32 + c * 16 + (q & 1) * 8 + 4);
                const float s8[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
                uint32_t h[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const uint32_t hi = bf16_rne_finite(s8[i]);
                    h[i] = (q & 2) ? bf16_rne_finite(s8[i] - bf16_to_f32(hi)) : hi;
                }
                uint4 v = make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
                if (n >= M) v = make_uint4(0, 0, 0, 0);
                *reinterpret_cast<uint4*>(xo_w + ((c * MP + n) * 4 + q) * 16) = v;
            }
        }
    }
    build_table(lsrc, 0);
    stage_write(st, 0, 0);
    stage_write(st1, 1, 1);
    stage_write(st2, 2, 2);
    lds_barrier();

    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    // the tables are the first thing in the block's LDS (the kernel has no static LDS), so a table
    // offset is an LDS address
    typedef const __attribute__((address_space(3))) uint32_t* lds_u32;
    typedef const __attribute__((address_space(3))) unsigned long long* lds_u64;
    // B operand of MFMA j (codes 8j .. 8j+7 of the lane's quarter) of one quarter group.
    // `low` = the lane's fixed part of a table address (row, copy and table buffer).
    auto lookup = [&](const Quarter& c, int j, uint32_t low) -> uint4 {
        uint4 b;
        if constexpr (BITS == 4) {
            const uint32_t wd = c.w[j];
            b.x = *reinterpret_cast<lds_u32>(__builtin_amdgcn_perm(wd, low, 0x0c0c0400u));
            b.y = *reinterpret_cast<lds_u32>(__builtin_amdgcn_perm(wd, low, 0x0c0c0500u));
            b.z = *reinterpret_cast<lds_u32>(__builtin_amdgcn_perm(wd, low, 0x0c0c0600u));
            b.w = *reinterpret_cast<lds_u32>(__builtin_amdgcn_perm(wd, low, 0x0c0c0700u));
        } else if constexpr (BITS == 3) {
            uint32_t r[4];
#pragma unroll
            for (int pi = 0; pi < 4; ++pi) {
                const int o = 24 * j + 6 * pi, wi = o >> 5, sh = o & 31;
                uint32_t idx;
                if (sh <= 26) idx = __builtin_amdgcn_ubfe(c.w[wi], sh, 6);
                else idx = __builtin_amdgcn_alignbit(c.w[wi + 1 < QW ? wi + 1 : wi], c.w[wi], sh) & 63u;
                r[pi] = *reinterpret_cast<lds_u32>((idx << 8) | low);
            }
            b = make_uint4(r[0], r[1], r[2], r[3]);
        } else {
            const uint32_t wd = c.w[j >> 1];
            const unsigned long long q0 = *reinterpret_cast<lds_u64>(__builtin_amdgcn_perm(wd, low, (j & 1) ? 0x0c020600u : 0x0c020400u));
            const unsigned long long q1 = *reinterpret_cast<lds_u64>(__builtin_amdgcn_perm(wd, low, (j & 1) ? 0x0c020700u : 0x0c020500u));
            b = make_uint4((uint32_t)q0, (uint32_t)(q0 >> 32), (uint32_t)q1, (uint32_t)(q1 >> 32));
        }
        return b;
    };
    // lane part of a table address for table buffer 0 / its increment for buffer 1
    const uint32_t low0 = BITS == 2 ? (uint32_t)(n * 16 + (q & 1) * 8) : (uint32_t)(n * 8 + (q & 1) * 4);
    constexpr uint32_t kLowPar = BITS == 2 ? 65536u : 128u;

    // sums the partial results of tile t (left in LDS before the barrier that ended its step) over the
    // wavefronts in a fixed order and stores them; the wavefronts take turns at this small job
    auto reduce_store = [&](int li, int par) {
        const int t = tile_of(li);
        const int rt = (tid - ((li & (kWaves - 1)) << 6)) & (kThreads - 1);
        if (rt < MP * kTile) {
            const int m = rt >> 4, nn = rt & 15;
            const float* src = red + (par * kWaves * MP + m) * 16 + nn;
            float s = 0.f;
#pragma unroll
            for (int ww = 0; ww < kWaves; ++ww) s += src[ww * MP * 16];
            const int64_t col = (int64_t)t * kTile + nn;
            if (m < M && col < N) p.y[(int64_t)m * N + col] = (uint16_t)f32_to_bf16(s);
        }
    };

    // ---- one tile.  `par` = i % 2 selects the table and partial-sum buffers (i: the tile's number in the block); `sl` = i % 3 is the
    //      LDS slot of the tile's small inputs; unit p of the tile sits in ring slot (SP + p) % 2, where
    //      SP = par for an odd number of units per tile and 0 for an even one (the ring position of a
    //      unit then does not depend on the tile, and one copy of the step serves every tile).
    auto tile_step = [&](auto sp_, int par, int i, int sl) {
        constexpr int SP = decltype(sp_)::value;
        // (one table for the whole matrix: built once, before the first tile, in buffer 0)
        const uint32_t low = low0 + (p.one_table ? 0u : (uint32_t)par) * kLowPar;
        const int sl1 = sl == kSlots - 1 ? 0 : sl + 1, sl2 = sl1 == kSlots - 1 ? 0 : sl1 + 1;
        // The tile is a sequence of NS = 16 * PASSES matrix instructions (4 per group).  The B operand of
        // instruction k is looked up kAhead instructions before it is used (ring of kAhead + 1 operands);
        // when the last word of a group's codes has been turned into addresses, the group's registers
        // are free and the same group of the unit two units on is requested.
        // (a shorter ring where two blocks share a compute unit: 128 registers a lane; measured, the depth
        // makes no difference between 2 and 11 - the kernel waits for memory, not for LDS)
        constexpr int NS = 4 * NG, kAhead = two_blocks(BITS, MP, PASSES) ? 2 : 3, NB = kAhead + 1;
        uint4 bq[NB];
        auto issue = [&](auto k_) {
            constexpr int k = decltype(k_)::value;
            constexpr int idx = k / 4, j = k % 4, pp = idx / 4, gi = idx % 4, slot = (SP + pp) & 1;
            bq[k % NB] = lookup(cw[slot][gi], j, low);
            if constexpr (j == 3) {
                constexpr int dt = PASSES == 1 ? 2 : (pp + 2 < PASSES ? 0 : 1);
                constexpr int np = PASSES == 1 ? 0 : (pp + 2 < PASSES ? pp + 2 : pp + 2 - PASSES);
                load_codes(cw[slot][gi], i + dt, np, gi);
            }
        };
        static_for<kAhead>(issue);
        __builtin_amdgcn_sched_barrier(0);
        if (i > 0) reduce_store(i - 1, par ^ 1);
        // small inputs: what was fetched during the previous tile (for tile t + 2) goes to its slot - the one
        // whose tile (t - 1) everybody finished with at the last barrier - and tile t + 3 is requested
        if (i > 0) stage_write(st, i + 2, sl2);
        stage_load(st, i + 3);
        // offset term of the whole tile: A = group sums of x (kept in LDS), B = this tile's offsets
        f32x4 doff = zero;
#pragma unroll
        for (int c = 0; c < NOF; ++c) {
            uint4 xo = make_uint4(0, 0, 0, 0);
            if (n < MP) xo = *reinterpret_cast<const uint4*>(xo_w + ((c * MP + n) * 4 + q) * 16);
            doff = mfma16(xo, read_offsets(c, sl), doff);
        }
        // the table of the next tile goes into the other buffer (everybody finished with it at the
        // barrier that ended the previous tile)
        if (i + 1 < ntiles && !p.one_table) {
            LutSrc l;
            read_lut(l, sl1);
            build_table(l, par ^ 1);
        }
        Scales sc;
        read_scales(sc, sl);
        float accm[MP];
#pragma unroll
        for (int m = 0; m < MP; ++m) accm[m] = q == 0 ? doff[m] : 0.f;
        f32x4 P0 = zero;
        auto step = [&](auto k_) {
            constexpr int k = decltype(k_)::value;
            if constexpr (k + kAhead < NS) issue(std::integral_constant<int, k + kAhead>{});
            __builtin_amdgcn_sched_barrier(0);
            constexpr int idx = k / 4, j = k % 4;
            constexpr int c = idx / P, s = idx % P;            // register set and slot of this group
            // one accumulation chain per group: the scale multiply then needs no extra adds
            P0 = mfma16(xa[c][j], bq[k % NB], j == 0 ? zero : P0);
            if constexpr (j == 3) {
                // wanted output rows: s * MP .. + MP, held by the lanes of quarter (s * MP) / 4
                constexpr int qsel = (s * MP) / 4, si = s % NSC;
                const uint32_t sw = sc.v[c][si >> 1];
                const float sf = (si & 1) ? bf16hi_to_f32(sw) : bf16lo_to_f32(sw);
                const float sfm = q == qsel ? sf : 0.f;
#pragma unroll
                for (int m = 0; m < MP; ++m) accm[m] = __builtin_fmaf(P0[(s * MP + m) % 4], sfm, accm[m]);
            }
        };
        static_for<NS>(step);
        // add the four quarters' parts (lanes n, n + 16, n + 32, n + 48) and leave the wavefront's partial sums in LDS
#pragma unroll
        for (int m = 0; m < MP; ++m) {
            float v = accm[m];
            v += __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(v), 0x401F /* lane ^ 16 */));
            v += __uint_as_float(__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __float_as_uint(v)));
            if (q == 0) red[((par * kWaves + w) * MP + m) * 16 + n] = v;
        }
        lds_barrier();
    };

    // One loop over the block's tiles with a single back edge (so that the compiler's count of outstanding
    // loads at the loop head is exact) and no copies of the step outside it: code that runs once per block
    // would be fetched from memory, not from the instruction cache, at the price of microseconds.
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    int li = 0, sl = 0, par = 0;
    auto next_slot = [&]() { sl = sl == kSlots - 1 ? 0 : sl + 1; };
    if constexpr (PASSES % 2 == 0) {
        for (;;) {
            tile_step(I0{}, par, li, sl);
            if (li + 1 >= ntiles) break;
            ++li; par ^= 1; next_slot();
        }
    } else {
        for (;;) {
            tile_step(I0{}, 0, li, sl);
            if (li + 1 >= ntiles) break;
            ++li; next_slot();
            tile_step(I1{}, 1, li, sl);
            par = 1;
            if (li + 1 >= ntiles) break;
            ++li; par = 0; next_slot();
        }
    }
    reduce_store(li, par);
}

}  // namespace pack

template <int BITS, int MP, int PASSES, bool REPACK>
inline hipError_t launch_pack_t(const pack::Params& p, hipStream_t stream) {
    constexpr auto kern = pack::decode_pack_kernel<BITS, MP, PASSES, REPACK>;
    // (the limit is raised once to all of a compute unit's LDS; what a launch asks for depends on K)
    const int lds = pack::lds_bytes(BITS, MP, PASSES, p.G);
    if (hipError_t e = ensure_lds<kern>(pack::kLdsPerCu); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)p.nblocks), dim3(pack::kThreads), lds, stream, p);
    return hipGetLastError();
}

template <int BITS, bool REPACK>
inline hipError_t launch_pack_b(const pack::Params& p, const PackPlan& pl, hipStream_t stream) {
#define ANY4_PACK(MP, PS) if (pl.mp == MP && pl.passes == PS) return launch_pack_t<BITS, MP, PS, REPACK>(p, stream)
    ANY4_PACK(1, 2); ANY4_PACK(1, 3); ANY4_PACK(1, 4);
    ANY4_PACK(1, 5); ANY4_PACK(1, 6); ANY4_PACK(1, 7); ANY4_PACK(1, 8);
    ANY4_PACK(2, 2); ANY4_PACK(2, 3); ANY4_PACK(2, 4);
    ANY4_PACK(4, 2);
#undef ANY4_PACK
    return hipErrorInvalidValue;
}


// one translation unit per code width instantiates these (any4_decode_pack_b4.hip, _b3, _b2)
hipError_t launch_pack_bits4(const pack::Params& p, const PackPlan& pl, bool repacked, hipStream_t stream);
hipError_t launch_pack_bits3(const pack::Params& p, const PackPlan& pl, bool repacked, hipStream_t stream);
hipError_t launch_pack_bits2(const pack::Params& p, const PackPlan& pl, bool repacked, hipStream_t stream);

}  // namespace any4
