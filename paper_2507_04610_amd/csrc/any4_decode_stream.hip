// Memory-bound any-n GEMM (n = 4, 3, 2) for small M (token generation, 1 <= M <= 16): persistent
// streaming kernel.
//
// y[m][n] = sum_k x[m][k] * (LUT[n][code[n][k]] * scale[n][k/128] + offset[n][k/128])
// (any4 paper, section 4.2 for y = x w^T with on-the-fly dequantisation, sections 2.4.1 and
// 2.5.2 for the per-row table and alpha * w_Q + beta).
//
// Lookup.  The paper keeps the 16-entry table in a register and looks codes up with a warp
// shuffle; it rejects a shared-memory table of all 16 x 16 value PAIRS (one lookup per packed
// byte) because of bank conflicts (section 4.2, last paragraph).  On CDNA4 the pair table is
// conflict free by construction.  A block works on 16 weight rows at a time; lane l of every
// wavefront works on row n = l % 16 and on quarter q = l / 16 of each group of 128 codes.  Entry
// e of row n is stored twice, at LDS bytes e * 256 + n * 8 and + 4 (and + 128 for the second of
// two table buffers); lane (n, q) reads copy q % 2, so the 32 lanes LDS serves together hit 32
// different banks.  One v_perm_b32 forms a lookup address (byte j of a code word -> address
// byte 1; buffer, row and copy -> byte 0); the lookup returns two bf16 table values, already
// packed as a matrix-core operand.
//
// Contraction.  v_mfma_f32_16x16x32_bf16 multiplies 16 rows x 32 codes by the activations
// (A operand: one row per m, rows >= M are zero).  Matrix-core throughput exceeds what the
// streamed codes need by a wide margin for every M <= 16, so the kernel costs nearly the same
// for M = 1 and M = 16: the time is that of reading the codes once.
//
// Scale and offset never touch individual weights.  With X[m][g] the sum of the 128
// activations of group g,
//     y[m][n] = sum_g ( scale[n][g] * P[m][n][g] + offset[n][g] * X[m][g] ),
//     P[m][n][g] = sum_{k in g} x[m][k] * LUT[n][code[n][k]]      (exact bf16 x bf16 products)
// P comes out of 4 MFMAs per group and is folded in with one fma per accumulator; the offset
// term of all groups of a wavefront is one more MFMA whose A operand is X split into a bf16
// high and low part (16 significant bits) and whose B operand is the offsets themselves.
//
// Work split ("K-stationary").  The K axis is cut into slabs of at most WAVES * GW groups.  A
// block belongs to one slab; wavefront w owns GW consecutive groups of it and keeps the
// activations of those groups in registers, as ready-made A operands, for its whole life.  The
// block then walks over its share of the 16-row tiles.  For every tile each wavefront streams
// the 64 * GW bytes per row that belong to its groups (the four lanes of a row read four
// consecutive 16-byte pieces), looks the codes up, multiplies, and leaves its partial sums in
// LDS; after one barrier per tile the partial sums of every output are added in a fixed order
// and stored.  The table of tile t+1 is built while tile t is being processed (two table
// buffers), and the code registers of a tile are refilled for tile t + kDepth as soon as their
// lookup addresses have been formed.  Loads in the steady state are unconditional (past the
// end of the block's share they re-read its last tile, which is cached), which lets the
// compiler count outstanding loads exactly.
//
// Small per-tile inputs (the rows' tables, scales and offsets: 2.5 KB per tile against 4 KB of
// codes per wavefront) are not read by every wavefront: for tile t one wavefront, taking turns,
// loads them four tiles ahead with five instructions and passes them on through LDS (AUX mode;
// it needs K/128 to be a multiple of 4 for the 8-byte alignment of its loads, otherwise every
// wavefront reads what it needs itself).
//
// 3- and 2-bit codes (the "anyn" variants of section 4.1) use the same kernel.  A lane's quarter of a
// group is 12 or 8 bytes instead of 16.  any3: a pair of codes is a 6-bit field of the lane's 96-bit
// chunk (v_bfe_u32, or v_alignbit_b32 for the two fields that straddle a word) indexing a
// 64-entry pair table of the same layout.  any2: a byte holds four codes and indexes a 256-entry
// table of QUADS (four bf16, one ds_read_b64, entry e of row n at LDS byte e * 256 + n * 16 and
// + 8, second buffer + 64 KB), so a lookup costs the same LDS slot as for any4 and yields four
// weights.
//
// With more than one slab the partial sums go to the workspace and the block that is last to
// finish a tile adds the slabs in slab order: results do not depend on the order in which
// blocks run.
#include "any4_device.h"
#include "any4_internal.h"
#include "any4_splitk.h"
#include <type_traits>

namespace any4 {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// D = A (16 x 32) * B (32 x 16) + C with eight 16-bit values per lane and operand
template <bool F16> __device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, const f32x4& c) {
    if constexpr (F16) return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

namespace stream {

constexpr int kTile = 16;                              // weight rows per tile
#ifndef ANY4_STREAM_DEPTH
#define ANY4_STREAM_DEPTH 2
#endif
constexpr int kDepth = ANY4_STREAM_DEPTH;              // tiles of code loads in flight per wavefront (2 or 4)
constexpr int kWaves = 8;                              // wavefronts per block: two per SIMD, up to 256 registers each
// LDS bytes of the two table buffers: any4 256 entries x (2 buffers x 16 rows x 2 copies x 4 B), any3 the
// same with 64 entries, any2 256 entries x (16 rows x 2 copies x 8 B) per buffer
constexpr int table_bytes(int bits) { return bits == 4 ? 256 * 256 : (bits == 3 ? 64 * 256 : 2 * 256 * 256); }
constexpr int kListTiles = 1024;                       // tiles whose slabs a block combines per round
constexpr int kAuxDist = 4;                            // tiles between the load of a tile's small inputs and their use
// LDS bytes per row of scales: 32 entries + 8 bytes of padding against bank conflicts; with groups of
// 64 weights (`fine`) 64 entries + 16 bytes
constexpr int aux_row(bool fine) { return fine ? 144 : 72; }
constexpr int aux_lut(bool fine) { return 2 * kTile * aux_row(fine); }
constexpr int aux_slot(bool fine) { return aux_lut(fine) + kTile * 32; }    // 2816 B (5120 B): scales, offsets and tables of one tile
constexpr int kRedBytes = 2 * kWaves * 4 * 64 * 4;     // [2][kWaves][4][64] fp32 partial sums
constexpr int aux_base(int bits) { return table_bytes(bits) + kRedBytes; }
constexpr int list_base(int bits, bool fine) { return aux_base(bits) + kAuxDist * aux_slot(fine); }
constexpr int lds_bytes(int bits, bool fine = false) { return list_base(bits, fine) + (1 + kListTiles) * 4; }

struct Params {
    const uint16_t* x;
    const uint32_t* codes;
    const uint16_t* lut;
    const uint16_t* scale;
    const uint16_t* offset;
    uint16_t* y;
    float* partial;                  // [slabs][M][N] fp32, slabs > 1 only
    unsigned long long* counters;    // [tiles], slabs > 1 only
    int64_t N, K;
    int M, G;                        // G = K / 128
    int lr;                          // log2(group size / 128): chunk g of 128 weights reads scale / offset g >> lr
                                     // of its row (rows of G >> lr entries)
    int slabs, slab_groups;          // groups per slab (the last slab may have fewer)
    int blocks_per_slab, tiles;      // grid = (blocks_per_slab, slabs)
    int tpb, trem;                   // tiles / blocks_per_slab and the remainder: block b of a slab owns tpb tiles, the
                                     // first trem blocks one more (computed by the host: two 64-bit divisions in the
                                     // kernel are ~300 instructions in front of the first load)
    int one_table;                   // lut holds ONE row that serves every row of the matrix (built once per block)
};

// LDS barrier that does not wait for outstanding global loads (the prefetched codes stay in flight)
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ float sum8(const uint4& v) {
    return ((bf16lo_to_f32(v.x) + bf16hi_to_f32(v.x)) + (bf16lo_to_f32(v.y) + bf16hi_to_f32(v.y))) +
           ((bf16lo_to_f32(v.z) + bf16hi_to_f32(v.z)) + (bf16lo_to_f32(v.w) + bf16hi_to_f32(v.w)));
}

// BITS    code width: 4, 3 or 2
// GW      groups (of 128 weights) a wavefront owns: 1, 2 or 4
// AUX     tables, scales and offsets of a tile are loaded by one wavefront and shared through LDS;
//         requires K/128 and the slab size to be multiples of 4 (8-byte aligned loads)
// NOLUT   4-bit codes on the uniform grid (value = code - 8, the int4 format): no table at all.
//         A code c becomes the bf16 number 128 + c by OR-ing it into the mantissa of 128.0
//         (0x4300 | c), and the surplus 136 * scale * (group sum of x) is taken off again by two more
//         exact bf16 terms (-128 * scale and -8 * scale) that ride in the offset MFMA.
// COARSE  groups of 256, 512 or 1024 weights: chunk g of 128 weights reads scale / offset g >> lr
// FINE    groups of 64 weights, M <= 8.  The codes, lookups and B operands are those of a chunk of 128;
//         the two halves of a chunk are told apart on the activation side.  Operand row r of the
//         matrix instructions holds activation row r % 8 with the quarters of the other half
//         zeroed (r < 8: quarters 0, 1 = the chunk's first 64 weights; r >= 8: quarters 2, 3), so
//         output rows m and m + 8 are the two halves' partial sums of activation row m.  An
//         accumulator lane holds rows 4q .. 4q + 3: lanes with q < 2 take the scale of the first
//         half, the others that of the second.  In the offset MFMA the group sums of the first
//         halves sit in the k-slots of quarter 0 (rows < 8) and those of the second halves in the
//         slots of quarter 1 (rows >= 8), facing the two offsets.  Rows m and m + 8 are added
//         when the wavefronts' partial sums are.
// F16     activations, table, scales, offsets and output are fp16 instead of bf16 (the f16 matrix
//         instruction; everything else moves 16-bit patterns and does not care)
template <int BITS, int GW, bool AUX, bool NOLUT, bool REPACK, bool COARSE, bool FINE, bool F16>
__global__ __launch_bounds__(kWaves * 64, 1) void decode_stream_kernel(const Params p) {
    static_assert(!F16 || (!NOLUT && !REPACK && !COARSE && !FINE), "fp16: table-based, plain layout, groups of 128");
    static_assert(!COARSE || (!NOLUT && !REPACK), "groups above 128 weights: table-based, plain layout");
    static_assert(!FINE || (!COARSE && !NOLUT && !REPACK), "groups of 64 weights: table-based, plain layout");
    static_assert(!(FINE && AUX && BITS == 2), "the larger slots of the shared small inputs do not fit beside the any2 tables");
    constexpr int kAuxRow = aux_row(FINE && AUX), kAuxScale = 0, kAuxOffset = kTile * kAuxRow, kAuxLut = aux_lut(FINE && AUX);
    constexpr int kAuxSlot = aux_slot(FINE && AUX);
    static_assert(!NOLUT || BITS == 4, "the table-free path is the 4-bit integer grid");
    static_assert(!(NOLUT && REPACK), "the table-free path reads the plain layout only");
    static_assert(BITS == 4 || BITS == 3 || BITS == 2, "code width");
    static_assert(kDepth == 4 || kDepth == 2, "the tile loop is unrolled by kDepth");
    constexpr int WAVES = kWaves, kThreads = WAVES * 64;
    constexpr int NP = (GW + 1) / 2;                     // packed bf16 pairs holding GW scales
    constexpr int QW = BITS;                             // 32-bit words of a lane's quarter group (32 codes)
    constexpr int QB = 4 * BITS, GB = 16 * BITS;         // bytes of a quarter group / of a group, per row
    constexpr int LUTB = 2 << BITS;                      // bytes of a row's table
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* red = reinterpret_cast<float*>(smem + table_bytes(BITS));    // [2][WAVES][4][64]
    unsigned char* const aux = smem + aux_base(BITS);                   // [kAuxDist] slots
    int* lastlist = reinterpret_cast<int*>(smem + list_base(BITS, FINE && AUX));     // [0] = count

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, q = lane >> 4;

    const int slab = blockIdx.y, bb = blockIdx.x;
    const int t0 = bb * p.tpb + min(bb, p.trem);
    const int ntiles = p.tpb + (bb < p.trem ? 1 : 0);
    const int t1 = t0 + ntiles;
    if (ntiles <= 0) return;

    const int M = p.M, G = p.G;
    const int64_t N = p.N, K = p.K;
    const int gs0 = slab * p.slab_groups;
    const int sg = min(p.slab_groups, G - gs0);          // groups of this slab
    const int ngw = max(0, min(GW, sg - w * GW));        // groups this wavefront really has (wave-uniform)
    // first group of this wavefront; a wavefront without groups points at the slab's first group and
    // keeps zero activations, scales and offsets, so whatever it reads contributes nothing
    const int gw0 = ngw > 0 ? gs0 + w * GW : gs0;
    auto group_of = [&](int gi) -> int { return gw0 + min(gi, max(ngw, 1) - 1); };        // clamped, wave-uniform

    // Addresses are a wave-uniform base (tile, group) plus a 32-bit per-lane byte offset (row, quarter),
    // so that the loads take their base from scalar registers.  In the problem's last tile the rows
    // past N are clamped to row N - 1 (they are read, never stored); only the lane offsets differ.
    const int last_tile = p.tiles - 1;
    const int nc = min(n, (int)(N - 1 - (int64_t)last_tile * kTile));        // this lane's row inside the last tile
    const uint32_t row_bytes = (uint32_t)(K * BITS / 8);
    const uint32_t vc_norm = (uint32_t)n * row_bytes + (uint32_t)q * QB, vc_last = (uint32_t)nc * row_bytes + (uint32_t)q * QB;
    const bool one_table = p.one_table != 0;
    const uint32_t vl_norm = one_table ? 0u : (uint32_t)n * LUTB, vl_last = one_table ? 0u : (uint32_t)nc * LUTB;
    const int64_t lut_tile_bytes = one_table ? 0 : kTile * LUTB;
    const int lr = COARSE ? p.lr : 0, GS = FINE ? 2 * G : G >> lr;      // scales / offsets per row
    const uint32_t vs_norm = (uint32_t)n * (uint32_t)GS * 2u, vs_last = (uint32_t)nc * (uint32_t)GS * 2u;
    const char* const codes_b = reinterpret_cast<const char*>(p.codes);
    const char* const lut_b = reinterpret_cast<const char*>(p.lut);
    const char* const scale_b = reinterpret_cast<const char*>(p.scale);
    const char* const offset_b = reinterpret_cast<const char*>(p.offset);

    // ---- codes: a ring of kDepth register sets indexed by (tile - t0) % kDepth; one lane holds the
    //      QW words of its quarter of each of the wavefront's groups
    struct Quarter { uint32_t w[QW]; };
    Quarter cw[kDepth][GW];
    // REPACK: the tile-major layout (any4_repack).  The 64 quarters of (tile, group) are 64 * QB
    // contiguous bytes in lane order, so one load instruction of a wavefront reads one contiguous
    // piece of memory (the plain layout gives it 16 pieces of 64 bytes, one per row); the last tile
    // is padded, no clamping.  These loads are nontemporal: every byte is read exactly once, and with
    // whole cache lines per instruction nothing is lost by not keeping them (with the plain layout,
    // where two instructions share each line, the same hint costs 5 %).
    auto load_codes = [&](Quarter& c, int t, int gi) {
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        typedef uint32_t u32x3 __attribute__((ext_vector_type(3), aligned(4)));
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        const char* base = codes_b + (int64_t)t * (kTile * (int64_t)row_bytes) + group_of(gi) * (REPACK ? 64 * QB : GB);
        const char* a = base + (REPACK ? (uint32_t)lane * QB : (t == last_tile ? vc_last : vc_norm));
        if constexpr (BITS == 4) {
            const u32x4 v = REPACK ? __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(a)) : *reinterpret_cast<const u32x4*>(a);
            c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2]; c.w[3] = v[3];
        } else if constexpr (BITS == 3) {
            const u32x3 v = REPACK ? __builtin_nontemporal_load(reinterpret_cast<const u32x3*>(a)) : *reinterpret_cast<const u32x3*>(a);
            c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2];
        } else {
            const u32x2 v = REPACK ? __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(a)) : *reinterpret_cast<const u32x2*>(a);
            c.w[0] = v[0]; c.w[1] = v[1];
        }
    };

    // ---- table source of a tile.  The entries of a row are written by its 32 threads (w, q):
    //   any4: 256 pair entries (hi << 4 | lo): thread writes hi = 2w + q/2, lo = 8 (q % 2) .. + 8
    //   any3:  64 pair entries (hi << 3 | lo): thread writes hi = w,        lo = 2q, 2q + 1
    //   any2: 256 quad entries (c3 c2 c1 c0):  thread writes entries 8 (4w + q) .. + 8
    // LutSrc holds the part of the row's table a thread needs for that: any4 its half row (4 words) and
    // the word with LUT[hi]; any3 word q and the word with LUT[w]; any2 the whole row (2 words).
    struct LutSrc { uint32_t a[BITS == 4 ? 4 : (BITS == 3 ? 1 : 2)]; uint32_t h; };
    const uint32_t lut_lo_off = BITS == 4 ? (uint32_t)(q & 1) * 16u : (BITS == 3 ? (uint32_t)q * 4u : 0u);
    const uint32_t lut_hi_off = BITS == 4 ? (uint32_t)w * 4u : (uint32_t)(w >> 1) * 4u;
    // reads a LutSrc from a row of the table, in memory or in an LDS slot (same code, any pointer)
    auto read_lut_row = [&](LutSrc& l, const char* row) {
        if constexpr (NOLUT) {
            (void)l; (void)row;
        } else if constexpr (BITS == 4) {
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
    auto load_lut = [&](LutSrc& l, int t) {          // straight from memory
        read_lut_row(l, lut_b + (int64_t)t * lut_tile_bytes + (t == last_tile ? vl_last : vl_norm));
    };
    // table of a tile into buffer `par`
    auto build_table = [&](const LutSrc& l, int par) {
        uint32_t* const tab = reinterpret_cast<uint32_t*>(smem);
        if constexpr (NOLUT) {
            (void)l; (void)par; (void)tab;
        } else if constexpr (BITS == 4) {
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
            // entry e of row n at dword e * 64 + par * 16384 + n * 4, both copies (16 bytes)
            // (copies first: a choice between l.a[0] and l.a[1] by a lane-dependent index is otherwise
            // compiled as an indexed load from a copy of the struct in scratch memory, once per tile)
            const uint32_t a0 = l.a[0], a1 = l.a[1];
            auto val = [&](int c) -> uint32_t { return ((c & 2) ? a1 : a0) >> (16 * (c & 1)) & 0xFFFFu; };
            auto valv = [&](uint32_t c) -> uint32_t {            // lane-dependent index
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

    // ---- AUX mode: the tile's scales, offsets and tables, loaded by one wavefront into registers
    //      (lane (n, j): scale / offset groups 4j .. 4j+3 and 16 + 4j .. 16 + 4j+3 of the slab; the
    //      row's table by lanes j < 2 (any4, 16 bytes each) or j = 0 (any3: 16 bytes, any2: 8)) and
    //      written to an LDS slot two tiles later.  Table rows keep a 32-byte stride in the slot.
    uint2 axs[2], axo[2];
    // FINE: twice the entries.  (Plain vector variables, not arrays of HIP's uint4: those the compiler
    // kept in scratch memory across the tile loop, with a store - and a full wait - right after each load.)
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    u32x4 fxs0 = {0, 0, 0, 0}, fxs1 = {0, 0, 0, 0}, fxo0 = {0, 0, 0, 0}, fxo1 = {0, 0, 0, 0};
    uint4 axl;
    auto aux_load = [&](int t) {
        if constexpr (FINE) {
            // two entries per chunk of 128: lane (n, j) loads those of chunks 4j .. 4j+3 and 16 + 4j .. + 3
            const int64_t tile_off = (int64_t)t * (kTile * 2) * GS + gs0 * 4;
            const uint32_t vs = t == last_tile ? vs_last : vs_norm;
            const uint32_t go0 = (uint32_t)min(q * 4, max(sg, 4) - 4) * 4u, go1 = (uint32_t)min((4 + q) * 4, max(sg, 4) - 4) * 4u;
            fxs0 = *reinterpret_cast<const u32x4*>(scale_b + tile_off + vs + go0);
            fxo0 = *reinterpret_cast<const u32x4*>(offset_b + tile_off + vs + go0);
            fxs1 = *reinterpret_cast<const u32x4*>(scale_b + tile_off + vs + go1);
            fxo1 = *reinterpret_cast<const u32x4*>(offset_b + tile_off + vs + go1);
        } else if constexpr (!COARSE) {
            // lanes past the slab's groups repeat its last four: the loads are unconditional
            const int64_t tile_off = (int64_t)t * (kTile * 2) * G + gs0 * 2;
            const uint32_t vs = t == last_tile ? vs_last : vs_norm;
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const uint32_t go = (uint32_t)min((c * 4 + q) * 4, max(sg, 4) - 4) * 2u;
                axs[c] = *reinterpret_cast<const uint2*>(scale_b + tile_off + vs + go);
                axo[c] = *reinterpret_cast<const uint2*>(offset_b + tile_off + vs + go);
            }
        } else {
            // groups of 256 weights and more: chunks 4j, 4j + 1 share a scale and so do 4j + 2, 4j + 3
            // (4j is a multiple of 4), so two 2-byte loads give the four entries the slot expects.
            // Lanes past the slab's groups repeat its last four chunks: all loads are unconditional.
            const int64_t tile_off = (int64_t)t * (kTile * 2) * GS;
            const uint32_t v = t == last_tile ? vs_last : vs_norm;
            // The registers keep the bare values; they are doubled up when the slot is written.
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const int g0 = gs0 + min((c * 4 + q) * 4, max(sg, 4) - 4);
                const uint32_t i0 = (uint32_t)(g0 >> lr) * 2u, i1 = (uint32_t)((g0 + 2) >> lr) * 2u;
                axs[c].x = *reinterpret_cast<const uint16_t*>(scale_b + tile_off + v + i0);
                axs[c].y = *reinterpret_cast<const uint16_t*>(scale_b + tile_off + v + i1);
                axo[c].x = *reinterpret_cast<const uint16_t*>(offset_b + tile_off + v + i0);
                axo[c].y = *reinterpret_cast<const uint16_t*>(offset_b + tile_off + v + i1);
            }
        }
        const char* lrow = lut_b + (int64_t)t * lut_tile_bytes + (t == last_tile ? vl_last : vl_norm);
        if constexpr (NOLUT) { (void)lrow; }
        // (every lane loads, also those whose copy is not written to the slot: a load under a per-lane
        // condition is waited for on the spot, together with all the code loads in flight)
        else if constexpr (BITS == 4) { axl = *reinterpret_cast<const uint4*>(lrow + (q & 1) * 16); }
        else if constexpr (BITS == 3) { axl = *reinterpret_cast<const uint4*>(lrow); }
        else { const uint2 v = *reinterpret_cast<const uint2*>(lrow); axl.x = v.x; axl.y = v.y; }
    };
    auto aux_write = [&](int slot) {
        unsigned char* s = aux + slot * kAuxSlot;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bool in_slab = (c * 4 + q) * 4 < sg;
            if constexpr (FINE) {
                if (in_slab) {
                    *reinterpret_cast<u32x4*>(s + kAuxScale + n * kAuxRow + (c * 4 + q) * 16) = c ? fxs1 : fxs0;
                    *reinterpret_cast<u32x4*>(s + kAuxOffset + n * kAuxRow + (c * 4 + q) * 16) = c ? fxo1 : fxo0;
                }
            } else {
                uint2 sv = axs[c], ov = axo[c];
                if constexpr (COARSE) {
                    sv = make_uint2(sv.x | (sv.x << 16), sv.y | (sv.y << 16));
                    ov = make_uint2(ov.x | (ov.x << 16), ov.y | (ov.y << 16));
                }
                if (in_slab) {
                    *reinterpret_cast<uint2*>(s + kAuxScale + n * kAuxRow + (c * 4 + q) * 8) = sv;
                    *reinterpret_cast<uint2*>(s + kAuxOffset + n * kAuxRow + (c * 4 + q) * 8) = ov;
                }
            }
        }
        if constexpr (NOLUT) { }
        else if constexpr (BITS == 4) { if (q < 2) *reinterpret_cast<uint4*>(s + kAuxLut + n * 32 + q * 16) = axl; }
        else if constexpr (BITS == 3) { if (q < 1) *reinterpret_cast<uint4*>(s + kAuxLut + n * 32) = axl; }
        else { if (q < 1) *reinterpret_cast<uint2*>(s + kAuxLut + n * 32) = make_uint2(axl.x, axl.y); }
    };
    auto aux_read_lut = [&](LutSrc& l, int slot) {
        read_lut_row(l, reinterpret_cast<const char*>(aux + slot * kAuxSlot + kAuxLut + n * 32));
    };

    // ---- scales and offsets of the wavefront's groups for one tile, as packed bf16 pairs
    //      (group gi in half gi % 2 of word gi / 2)
    auto aux_read_so = [&](uint32_t (&sp)[NP], uint32_t (&op)[NP], int slot) {
        const unsigned char* s = aux + slot * kAuxSlot + n * kAuxRow + (w * GW) * (FINE ? 4 : 2);
        if constexpr (FINE) {
            // a chunk's two entries are one word (first half | second half << 16); an accumulator lane
            // takes the scale of half q / 2, an offset-operand lane the offset of half q % 2
            const uint32_t ssel = (q >> 1) ? 0x07060302u : 0x05040100u, osel = (q & 1) ? 0x07060302u : 0x05040100u;
            if constexpr (GW == 4) {
                const uint4 a = *reinterpret_cast<const uint4*>(s + kAuxScale), b = *reinterpret_cast<const uint4*>(s + kAuxOffset);
                sp[0] = __builtin_amdgcn_perm(a.y, a.x, ssel); sp[1] = __builtin_amdgcn_perm(a.w, a.z, ssel);
                op[0] = __builtin_amdgcn_perm(b.y, b.x, osel); op[1] = __builtin_amdgcn_perm(b.w, b.z, osel);
            } else if constexpr (GW == 2) {
                const uint2 a = *reinterpret_cast<const uint2*>(s + kAuxScale), b = *reinterpret_cast<const uint2*>(s + kAuxOffset);
                sp[0] = __builtin_amdgcn_perm(a.y, a.x, ssel);
                op[0] = __builtin_amdgcn_perm(b.y, b.x, osel);
            } else {
                const uint32_t a = *reinterpret_cast<const uint32_t*>(s + kAuxScale), b = *reinterpret_cast<const uint32_t*>(s + kAuxOffset);
                sp[0] = __builtin_amdgcn_perm(0u, a, ssel) & 0xFFFFu;
                op[0] = __builtin_amdgcn_perm(0u, b, osel) & 0xFFFFu;
            }
        } else if constexpr (GW == 4) {
            const uint2 a = *reinterpret_cast<const uint2*>(s + kAuxScale), b = *reinterpret_cast<const uint2*>(s + kAuxOffset);
            sp[0] = a.x; sp[1] = a.y; op[0] = b.x; op[1] = b.y;
        } else if constexpr (GW == 2) {
            sp[0] = *reinterpret_cast<const uint32_t*>(s + kAuxScale);
            op[0] = *reinterpret_cast<const uint32_t*>(s + kAuxOffset);
        } else {
            sp[0] = *reinterpret_cast<const uint16_t*>(s + kAuxScale);
            op[0] = *reinterpret_cast<const uint16_t*>(s + kAuxOffset);
        }
        if (ngw == 0) {                                  // nothing was written for a wavefront without groups
#pragma unroll
            for (int i = 0; i < NP; ++i) { sp[i] = 0; op[i] = 0; }
        }
    };
    // without AUX: every wavefront reads its own scales, offsets (one bf16 per load) and table rows,
    // in rings like the codes
    uint32_t sraw[kDepth][GW], oraw[kDepth][GW];
    LutSrc lut_ring[kDepth];
    auto load_so = [&](uint32_t (&sr)[GW], uint32_t (&orw)[GW], int t) {
        const int64_t tile_off = (int64_t)t * (kTile * 2) * GS;
        const uint32_t v = t == last_tile ? vs_last : vs_norm;
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) {
            // FINE: accumulator lanes of quarters 0, 1 / 2, 3 scale the first / second half of the chunk;
            // offset-operand lanes of quarter 0 / 1 carry the first / second half's offset
            const uint32_t si = FINE ? (uint32_t)(2 * group_of(gi)) + (uint32_t)(q >> 1) : (uint32_t)(group_of(gi) >> lr);
            const uint32_t oi = FINE ? (uint32_t)(2 * group_of(gi)) + (uint32_t)(q & 1) : (uint32_t)(group_of(gi) >> lr);
            sr[gi] = *reinterpret_cast<const uint16_t*>(scale_b + tile_off + si * 2u + v);
            orw[gi] = *reinterpret_cast<const uint16_t*>(offset_b + tile_off + oi * 2u + v);
        }
    };
    auto pack_so = [&](uint32_t (&sp)[NP], uint32_t (&op)[NP], const uint32_t (&sr)[GW], const uint32_t (&orw)[GW]) {
#pragma unroll
        for (int i = 0; i < NP; ++i) { sp[i] = 0; op[i] = 0; }
#pragma unroll
        for (int gi = 0; gi < GW; ++gi)
            if (gi < ngw) { sp[gi >> 1] |= sr[gi] << (16 * (gi & 1)); op[gi >> 1] |= orw[gi] << (16 * (gi & 1)); }
    };
    auto scale_f = [&](const uint32_t (&sp)[NP], int gi) -> float {
        return (gi & 1) ? h16hi_to_f32<F16>(sp[gi >> 1]) : h16lo_to_f32<F16>(sp[gi >> 1]);
    };
    // offsets of the wavefront's groups as a B operand: k-slots 0..3 and 4..7 both hold o[g0..g3]
    // (slots of groups the wavefront does not have are zero and meet zero activation sums)
    auto offset_operand = [&](const uint32_t (&op)[NP]) -> uint4 {
        const uint32_t a = op[0], b = NP > 1 ? op[NP - 1] : 0u;
        return make_uint4(a, b, a, b);
    };
    // NOLUT: lanes of quarter 0 carry the offsets, quarter 1 carries -128 * scale and quarter 2
    // -8 * scale (exponent + 7 / + 3 and the sign flipped, on both bf16 halves of a word: exact);
    // all three meet the same group sums of x
    auto offset_operand_nolut = [&](const uint32_t (&sp)[NP], const uint32_t (&op)[NP]) -> uint4 {
        uint32_t a = op[0], b = NP > 1 ? op[NP - 1] : 0u;
        const uint32_t sa = sp[0], sb = NP > 1 ? sp[NP - 1] : 0u;
        if (q == 1) { a = (sa + 0x03800380u) ^ 0x80008000u; b = (sb + 0x03800380u) ^ 0x80008000u; }
        if (q == 2) { a = (sa + 0x01800180u) ^ 0x80008000u; b = (sb + 0x01800180u) ^ 0x80008000u; }
        return make_uint4(a, b, a, b);
    };

    // ---- prologue.  Activations first (small, and the first thing the matrix cores need), then the
    //      codes of the ring and the small inputs.
    // activations of the wavefront's groups as A operands: lane (m = n, q), MFMA j of group gi holds
    // x[m][(gw0 + gi) * 128 + q * 32 + j * 8 .. + 8]; rows m >= M and missing groups are zero.
    // The wavefront fetches each row's GW * 128 activations with ONE 16-byte load per lane (a
    // contiguous kilobyte per instruction) and re-distributes them to the operand layout through
    // LDS, instead of 4 * GW loads per lane that each pick 16-byte pieces out of 16 rows.  One or
    // two rows go through the partial-sum buffer (idle until the first tile; every wavefront has a
    // slice of its own, no barrier).  More rows are fetched 4, 8 or 16 at a time (rows past M repeat
    // row M - 1 so that the loads are unconditional) and go, kStageRows at a pass, through the table
    // buffers, which are idle until the first table is built - after a barrier in that case.
    constexpr int kStageRows = BITS == 4 ? 8 : (BITS == 2 ? 16 : 4);
    static_assert(2 * GW * 256 * kWaves <= kRedBytes, "one or two rows are staged in the partial-sum buffer");
    static_assert(kStageRows * GW * 256 * kWaves <= table_bytes(BITS) + kRedBytes, "more rows are staged in the table buffers");
    const bool compact = M <= 2;                          // the same for every thread
    const bool has = lane * 8 < ngw * kGroup;             // GW * 128 = up to 64 lanes x 8 elements
    uint4 xa[GW][4];
    uint4 xraw[kTile];
    if (compact) {
        // through a buffer descriptor over the M rows: a lane without a piece takes an offset beyond the
        // range and gets zeros without a memory access, so the load is unconditional.  (A load under a
        // per-lane condition is followed by a wait for ALL outstanding loads: here that wait stood in
        // front of the first code load, a whole trip to memory before the stream even started.)
        const __amdgpu_buffer_rsrc_t xr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), 0, (int)(M * K * 2), 0x00020000);
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const uint32_t vo = (m < M && has) ? (uint32_t)((m * K + (int64_t)gw0 * kGroup + lane * 8) * 2) : 0x80000000u;
            const auto v = __builtin_amdgcn_raw_buffer_load_b128(xr, vo, 0, 0);
            xraw[m] = make_uint4(v[0], v[1], v[2], v[3]);
        }
    } else {
        const uint16_t* xsrc = p.x + (int64_t)gw0 * kGroup + (has ? lane : 0) * 8;
        auto fetch_rows = [&](auto nr_) {
            constexpr int NR = decltype(nr_)::value;
#pragma unroll
            for (int m = 0; m < NR; ++m) {
                const uint4 v = *reinterpret_cast<const uint4*>(xsrc + (int64_t)min(m, M - 1) * K);
                xraw[m] = has ? v : make_uint4(0, 0, 0, 0);
            }
        };
        if (M <= 4) fetch_rows(std::integral_constant<int, 4>{});
        else if (M <= 8) fetch_rows(std::integral_constant<int, 8>{});
        else fetch_rows(std::integral_constant<int, kTile>{});
    }
    LutSrc lut0;
    if constexpr (AUX) {
        load_lut(lut0, t0);                              // the first tile's table comes straight from memory
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) load_codes(cw[0][gi], t0, gi);
        if (w < kAuxDist && w < ntiles) aux_load(t0 + w);
#pragma unroll
        for (int d = 1; d < kDepth; ++d)
#pragma unroll
            for (int gi = 0; gi < GW; ++gi) load_codes(cw[d][gi], min(t0 + d, t1 - 1), gi);
    } else {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int t = min(t0 + d, t1 - 1);
            load_lut(lut_ring[d], t);
#pragma unroll
            for (int gi = 0; gi < GW; ++gi) load_codes(cw[d][gi], t, gi);
            load_so(sraw[d], oraw[d], t);
        }
    }
#pragma unroll
    for (int gi = 0; gi < GW; ++gi)
#pragma unroll
        for (int j = 0; j < 4; ++j) xa[gi][j] = make_uint4(0, 0, 0, 0);
    {
        // row m of a pass at stage + m * (GW * 16) uint4 of the wavefront's slice; a lane's MFMA-j piece
        // of group gi is uint4 number gi * 16 + q * 4 + j of its row.  Lanes of groups the wavefront
        // does not have hold zeros.  The slice is written and read by this wavefront only.
        auto stage_pass = [&](uint4* stage, int r0, auto rows_) {
            constexpr int ROWS = decltype(rows_)::value;
#pragma unroll
            for (int m = 0; m < ROWS; ++m)
                if (lane < GW * 16 && r0 + m < M) stage[m * (GW * 16) + lane] = xraw[r0 + m];
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            // FINE: operand row n is activation row n % 8, restricted to the quarters of half n / 8
            const int xrow = FINE ? (n & 7) : n;
            const bool mine = FINE ? (n >> 3) == (q >> 1) : true;
            if (mine && xrow >= r0 && xrow < min(M, r0 + ROWS)) {
#pragma unroll
                for (int gi = 0; gi < GW; ++gi)
#pragma unroll
                    for (int j = 0; j < 4; ++j) xa[gi][j] = stage[(xrow - r0) * (GW * 16) + gi * 16 + q * 4 + j];
            }
        };
        if (compact) {
            stage_pass(reinterpret_cast<uint4*>(red) + w * (2 * GW * 16), 0, std::integral_constant<int, 2>{});
        } else {
            uint4* stage = reinterpret_cast<uint4*>(smem) + w * (kStageRows * GW * 16);
#pragma unroll
            for (int r0 = 0; r0 < kTile; r0 += kStageRows)
                if (r0 < M) stage_pass(stage, r0, std::integral_constant<int, kStageRows>{});
            lds_barrier();                                 // before anybody builds a table over a slice
        }
    }

    // group sums of the activations -> A operand of the offset MFMA (q == 0 lanes: hi parts in
    // k-slots 0..3, lo parts in k-slots 4..7; other lanes: zero); done as soon as the activations
    // are there, while the codes are still on their way.  The matrix cores add them up: with an
    // all-ones A operand and the activations as B operand, D[i][m] = sum_k x[m][k] for every i, and
    // the lanes of column m (the lanes that hold row m of x) receive exactly their own row's sum.
    uint4 xo;
    {
        constexpr uint32_t one2 = F16 ? 0x3C003C00u : 0x3F803F80u;      // 1.0 twice
        const uint4 ones = make_uint4(one2, one2, one2, one2);
        const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
        f32x4 gs[GW];
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) gs[gi] = z4;
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int gi = 0; gi < GW; ++gi)
                gs[gi] = mfma16<F16>(ones, xa[gi][j], gs[gi]);
        uint32_t hi[4] = {0, 0, 0, 0}, lo[4] = {0, 0, 0, 0};
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) {
            const float sgi = gs[gi][0];
            hi[gi] = f32_to_h16<F16>(sgi);
            lo[gi] = f32_to_h16<F16>(sgi - h16_to_f32<F16>(hi[gi]));
        }
        xo = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16));
        if (FINE ? q != (n >> 3) : (NOLUT ? q > 2 : q > 0)) xo = make_uint4(0, 0, 0, 0);
    }
    if constexpr (NOLUT) {
        // operand order of the table-free path: elements (0, 4), (1, 5), (2, 6), (3, 7) of every 8
#pragma unroll
        for (int gi = 0; gi < GW; ++gi)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint4 v = xa[gi][j];
                xa[gi][j] = make_uint4(__builtin_amdgcn_perm(v.z, v.x, 0x05040100u), __builtin_amdgcn_perm(v.z, v.x, 0x07060302u),
                                       __builtin_amdgcn_perm(v.w, v.y, 0x05040100u), __builtin_amdgcn_perm(v.w, v.y, 0x07060302u));
            }
    }
    if constexpr (AUX) {
        build_table(lut0, 0);
        if (w < kAuxDist && w < ntiles) aux_write(w);
    } else {
        build_table(lut_ring[0], 0);
        load_lut(lut_ring[0], min(t0 + kDepth, t1 - 1));
    }
    if (tid == 0) lastlist[0] = 0;
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
        if constexpr (NOLUT) {
            // nibbles n0..n7 of the word -> bf16 pairs (128 + n0, 128 + n4), (n1, n5), (n2, n6), (n3, n7);
            // the activations were put into the same order before the loop
            const uint32_t wd = c.w[j];
            b.x = (wd & 0x000F000Fu) | 0x43004300u;
            b.y = ((wd >> 4) & 0x000F000Fu) | 0x43004300u;
            b.z = ((wd >> 8) & 0x000F000Fu) | 0x43004300u;
            b.w = ((wd >> 12) & 0x000F000Fu) | 0x43004300u;
            (void)low;
        } else if constexpr (BITS == 4) {
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
    auto mfma = [&](const uint4& a, const uint4& b, const f32x4& c) -> f32x4 {
        return mfma16<F16>(a, b, c);
    };
    // lane part of a table address for table buffer 0 / its increment for buffer 1
    const uint32_t low0 = BITS == 2 ? (uint32_t)(n * 16 + (q & 1) * 8) : (uint32_t)(n * 8 + (q & 1) * 4);
    constexpr uint32_t kLowPar = BITS == 2 ? 65536u : 128u;

    // sums the partial results of tile t (left in LDS before the barrier that ended its step) over the
    // wavefronts in a fixed order and stores them; the wavefronts take turns at this small job
    auto reduce_store = [&](int t) {
        const int par = (t - t0) & 1;
        const int rt = (tid - ((t & (WAVES - 1)) << 6)) & (kThreads - 1);
        if (rt < M * kTile) {
            const int m = rt >> 4, nn = rt & 15;
            const float* src = red + (par * WAVES * 4 + (m & 3)) * 64 + (m >> 2) * 16 + nn;
            float s = 0.f;
#pragma unroll
            for (int ww = 0; ww < WAVES; ++ww) s += src[ww * 4 * 64];
            if constexpr (FINE) {                          // the second halves of the chunks: output row m + 8
                float s2 = 0.f;
#pragma unroll
                for (int ww = 0; ww < WAVES; ++ww) s2 += src[ww * 4 * 64 + 32];
                s += s2;
            }
            const int64_t col = (int64_t)t * kTile + nn;
            if (col < N) {
                if (p.slabs == 1) p.y[(int64_t)m * N + col] = (uint16_t)f32_to_h16<F16>(s);
                else splitk_store(p.partial + ((int64_t)slab * M + m) * N + col, s);
            }
        }
    };

    // ---- one tile.  B = (t - t0) % kDepth is the ring slot of its registers; (t - t0) & 1 selects the
    //      table and partial-sum buffers.  Order inside a step: the lookups of the first group are
    //      issued straight after the barrier that completed this tile's table; while they are in
    //      flight the previous tile's results are summed and stored, the small inputs move on and
    //      the next tile's table is written; then the groups follow, the lookups of group g+1 always
    //      issued before the matrix instructions of group g.
    auto tile_step = [&](auto slot, auto refill, int t) {
        constexpr int B = decltype(slot)::value, B1 = (B + 1) % kDepth;
        constexpr bool REFILL = decltype(refill)::value;    // false for the block's last tiles
        const int i = t - t0, par = i & 1;
        const int tn = min(t + kDepth, t1 - 1);
        // (one table for the whole matrix: built once, before the first tile, in buffer 0)
        const uint32_t low = low0 + (one_table ? 0 : par) * kLowPar;
        uint4 bq[2][4];
        auto lookups = [&](int gi, uint4 (&b)[4]) {
            const Quarter c = cw[B][gi];
            b[0] = lookup(c, 0, low); b[1] = lookup(c, 1, low); b[2] = lookup(c, 2, low); b[3] = lookup(c, 3, low);
            if constexpr (NOLUT) {
                // The table-free operands are plain arithmetic on the code words, which the compiler would
                // rather redo next to the matrix instructions: the code words then outlive the refill,
                // the refill lands in other registers and every round of the tile loop ends with copies
                // behind a wait for ALL outstanding loads.  Pin the operands here instead.
#pragma unroll
                for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(b[j].x), "+v"(b[j].y), "+v"(b[j].z), "+v"(b[j].w));
            }
            if constexpr (REFILL) load_codes(cw[B][gi], tn, gi);
        };
        lookups(0, bq[0]);
        __builtin_amdgcn_sched_barrier(0);
        if (i > 0) reduce_store(t - 1);
        uint32_t sp[NP], op[NP];
        if constexpr (AUX) {
            // small inputs: tile i + 2 goes to its LDS slot, tile i + 4 is requested, this tile's
            // scales and the next tile's table rows are read from their slots
            if (i + 2 >= kAuxDist && i + 2 < ntiles && w == ((i + 2) & 7)) aux_write((i + 2) & (kAuxDist - 1));
            if (i + kAuxDist < ntiles && w == ((i + kAuxDist) & 7)) aux_load(t + kAuxDist);
            aux_read_so(sp, op, i & (kAuxDist - 1));
            if (i + 1 < ntiles && !one_table) {
                LutSrc l;
                aux_read_lut(l, (i + 1) & (kAuxDist - 1));
                build_table(l, par ^ 1);
            }
        } else {
            pack_so(sp, op, sraw[B], oraw[B]);
            // the table of the next tile goes into the other buffer (everybody finished with it at the
            // barrier that ended the previous tile); its source registers are then refilled
            if (i + 1 < ntiles && !one_table) build_table(lut_ring[B1], par ^ 1);
            if constexpr (REFILL) load_lut(lut_ring[B1], min(t + 1 + kDepth, t1 - 1));
        }
        f32x4 acc = mfma(xo, NOLUT ? offset_operand_nolut(sp, op) : offset_operand(op), zero);
#pragma unroll
        for (int gi = 0; gi < GW; ++gi) {
            if (gi + 1 < GW) lookups(gi + 1, bq[(gi + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
            const uint4 (&b)[4] = bq[gi & 1];
            // one accumulation chain per group: the scale multiply then needs no extra adds
            f32x4 P0 = mfma(xa[gi][0], b[0], zero);
            P0 = mfma(xa[gi][1], b[1], P0);
            P0 = mfma(xa[gi][2], b[2], P0);
            P0 = mfma(xa[gi][3], b[3], P0);
            const float sf = scale_f(sp, gi);
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[v] = __builtin_fmaf(P0[v], sf, acc[v]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (!AUX && REFILL) load_so(sraw[B], oraw[B], tn);
        // partial sums of this wavefront: accumulator v of lane (n, q) is m = 4 q + v, row n
        float* rd = red + ((par * WAVES + w) * 4) * 64 + lane;
#pragma unroll
        for (int v = 0; v < 4; ++v) rd[v * 64] = acc[v];
        lds_barrier();
    };

    // full rounds of the ring in a loop with a single back edge (so that the compiler's count of
    // outstanding loads at the loop head is exact), then the remaining tiles
    const int rounds = ntiles / kDepth;
    int t = t0;
    using T = std::true_type;
    using F = std::false_type;
    for (int it = 0; it < rounds; ++it, t += kDepth) {
        tile_step(std::integral_constant<int, 0>{}, T{}, t);
        tile_step(std::integral_constant<int, 1>{}, T{}, t + 1);
        if constexpr (kDepth == 4) {
            tile_step(std::integral_constant<int, 2>{}, T{}, t + 2);
            tile_step(std::integral_constant<int, 3>{}, T{}, t + 3);
        }
    }
    if (t < t1) {
        tile_step(std::integral_constant<int, 0>{}, F{}, t);
        if constexpr (kDepth == 4) {
            if (t + 1 < t1) {
                tile_step(std::integral_constant<int, 1>{}, F{}, t + 1);
                if (t + 2 < t1) tile_step(std::integral_constant<int, 2>{}, F{}, t + 2);
            }
        }
    }
    reduce_store(t1 - 1);

    // ---- more than one slab: arrive at the counters of all tiles of this block, then finish the
    //      tiles for which this block was the last
    if (p.slabs > 1) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's partial sums have been written
        lds_barrier();                                     // ... and so have the whole block's
        for (int tb0 = t0; tb0 < t1; tb0 += kListTiles) {      // in rounds of what the list holds
            const int tb1 = min(t1, tb0 + kListTiles);
            for (int i = tb0 + tid; i < tb1; i += kThreads) {
                if (arrive_one(p.counters + i, p.slabs)) {
                    const int slot = atomicAdd(lastlist, 1);
                    lastlist[1 + slot] = i;
                }
            }
            lds_barrier();
            // All outputs of all listed tiles.  A thread takes UC outputs at a time and issues the
            // loads of KC slabs of all of them before it adds anything (one wait per KC * UC loads:
            // the partial sums come from other compute units, a load costs a trip to memory);
            // outputs past the end repeat the last one and slabs past the end repeat the last slab, so
            // that every load is unconditional, and are left out of the sum / not stored.  The sum runs
            // over the slabs in slab order whatever the batching.
            const int nlast = lastlist[0];
            const int nout = nlast * M * kTile;
            const int64_t slab_stride = (int64_t)M * N;
            auto combine = [&](auto kc_, auto uc_) {
                constexpr int KC = decltype(kc_)::value, UC = decltype(uc_)::value;
                for (int base = 0; base < nout; base += kThreads * UC) {
                    const float* src[UC];
                    int64_t dst[UC];
                    bool live[UC];
                    float s[UC];
#pragma unroll
                    for (int u = 0; u < UC; ++u) {
                        const int raw = base + u * kThreads + tid, idx = min(raw, nout - 1);
                        const int e = idx / (M * kTile), o = idx - e * (M * kTile);
                        const int m = o >> 4, nn = o & 15;
                        const int64_t col = (int64_t)lastlist[1 + e] * kTile + nn;
                        live[u] = raw < nout && col < N;
                        dst[u] = (int64_t)m * N + min(col, N - 1);
                        src[u] = p.partial + dst[u];
                        s[u] = 0.f;
                    }
                    for (int k0 = 0; k0 < p.slabs; k0 += KC) {
                        float v[KC][UC];
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk)
#pragma unroll
                            for (int u = 0; u < UC; ++u)
                                v[kk][u] = splitk_load(src[u] + (int64_t)min(k0 + kk, p.slabs - 1) * slab_stride);
#pragma unroll
                        for (int kk = 0; kk < KC; ++kk)
#pragma unroll
                            for (int u = 0; u < UC; ++u) s[u] += k0 + kk < p.slabs ? v[kk][u] : 0.f;
                    }
#pragma unroll
                    for (int u = 0; u < UC; ++u)
                        if (live[u]) p.y[dst[u]] = (uint16_t)f32_to_h16<F16>(s[u]);
                }
            };
            // few slabs: more outputs at a time instead (no repeated loads of the last slab)
            if (p.slabs <= 2) combine(std::integral_constant<int, 2>{}, std::integral_constant<int, 8>{});
            else combine(std::integral_constant<int, 4>{}, std::integral_constant<int, 4>{});
            lds_barrier();
            if (tid == 0) lastlist[0] = 0;
            lds_barrier();
        }
    }
}

}  // namespace stream

using stream::Params;

// Shape of the work split for a problem; a pure function of (M, N, K) and the number of compute units.
StreamPlan plan_stream(int64_t M, int64_t N, int64_t K, int cus) {
    StreamPlan best{};
    const int G = (int)(K / kGroup);
    const int64_t tiles = (N + stream::kTile - 1) / stream::kTile;
    if (M > stream::kTile || tiles > 0x7FFFFFFF) return best;
    double best_cost = 1e300;
    const bool aux = G % 4 == 0;
    for (int gw : {4, 2, 1}) {
        const int slab_max = stream::kWaves * gw;
        int slabs = (G + slab_max - 1) / slab_max;
        // equal slabs, each a multiple of gw groups (of 4 groups in AUX mode), except possibly the last
        const int unit = aux ? 4 : gw;
        const int sgroups = ((G + slabs - 1) / slabs + unit - 1) / unit * unit;
        if (sgroups > slab_max) continue;
        slabs = (G + sgroups - 1) / sgroups;
        if (slabs > kMaxSplit) continue;
        int bps = cus / slabs;                                 // one block per compute unit (two measured 25 - 30 % slower)
        if (bps < 1) bps = 1;
        if (bps > tiles) bps = (int)tiles;
        const int64_t tpb = (tiles + bps - 1) / bps;
        // microseconds: streaming of the block's bytes at ~22 GB/s per compute unit, per-tile
        // table build and barrier, and the end-of-kernel combination of slabs
        const double cost = (double)tpb * sgroups * 0.047 + (double)tpb * 0.15 + (slabs > 1 ? 3.0 : 0.0);
        if (cost < best_cost) {
            best_cost = cost;
            best.gw = gw;
            best.slabs = slabs;
            best.slab_groups = sgroups;
            best.blocks_per_slab = bps;
            best.tiles = tiles;
            best.aux = aux;
        }
    }
    best.workspace = best.slabs > 1
        ? splitk_counter_bytes(best.tiles) + (size_t)best.slabs * (size_t)M * (size_t)N * sizeof(float) : 0;
    return best;
}

template <int BITS, int GW, bool AUX, bool NOLUT = false, bool REPACK = false, bool COARSE = false, bool FINE = false,
          bool F16 = false>
static hipError_t launch_stream_t(const Params& p, int grid, hipStream_t stream) {
    constexpr auto kern = stream::decode_stream_kernel<BITS, GW, AUX, NOLUT, REPACK, COARSE, FINE, F16>;
    constexpr int lds = stream::lds_bytes(BITS, FINE && AUX);
    if (hipError_t e = ensure_lds<kern>(lds); e != hipSuccess) return e;
    if (grid != p.blocks_per_slab * p.slabs) return hipErrorInvalidValue;
    hipLaunchKernelGGL(kern, dim3((unsigned)p.blocks_per_slab, (unsigned)p.slabs), dim3(stream::kWaves * 64), lds, stream, p);
    return hipGetLastError();
}

template <int BITS, bool REPACK>
static hipError_t launch_stream_b(const Params& p, const StreamPlan& sp, int grid, hipStream_t stream) {
#define ANY4_STREAM(GW)                                                                    \
    (sp.aux ? launch_stream_t<BITS, GW, true, false, REPACK>(p, grid, stream)              \
            : launch_stream_t<BITS, GW, false, false, REPACK>(p, grid, stream))
    switch (sp.gw) {
        case 4: return ANY4_STREAM(4);
        case 2: return ANY4_STREAM(2);
        default: return ANY4_STREAM(1);
    }
#undef ANY4_STREAM
}

hipError_t launch_decode_stream(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                                const uint16_t* scale, const uint16_t* offset, int64_t M, int64_t N,
                                int64_t K, int bits, int lr, bool repacked, bool f16, bool one_table, const StreamPlan& sp_in, uint16_t* y,
                                void* workspace, hipStream_t stream) {
    const StreamPlan& sp = sp_in;
    Params p{};
    p.x = x; p.codes = codes; p.lut = lut; p.scale = scale; p.offset = offset; p.y = y;
    p.counters = static_cast<unsigned long long*>(workspace);
    p.partial = sp.slabs > 1
        ? reinterpret_cast<float*>(static_cast<char*>(workspace) + splitk_counter_bytes(sp.tiles)) : nullptr;
    p.N = N; p.K = K; p.M = (int)M; p.G = (int)(K / kGroup); p.lr = lr;
    p.slabs = sp.slabs; p.slab_groups = sp.slab_groups; p.blocks_per_slab = sp.blocks_per_slab;
    p.tiles = (int)sp.tiles;
    p.tpb = p.tiles / sp.blocks_per_slab;
    p.trem = p.tiles % sp.blocks_per_slab;
    p.one_table = one_table ? 1 : 0;
    const int grid = sp.slabs * sp.blocks_per_slab;
    if (f16) {
        // fp16: the table-based kernels on the plain layout with groups of 128
        if (lut == nullptr || repacked || lr != 0) return hipErrorInvalidValue;
#define ANY4_STREAM_H(B, GW)                                                               \
        return sp.aux ? launch_stream_t<B, GW, true, false, false, false, false, true>(p, grid, stream)   \
                      : launch_stream_t<B, GW, false, false, false, false, false, true>(p, grid, stream)
#define ANY4_STREAM_HB(B)                                                                  \
        switch (sp.gw) {                                                                   \
            case 4: ANY4_STREAM_H(B, 4);                                                   \
            case 2: ANY4_STREAM_H(B, 2);                                                   \
            default: ANY4_STREAM_H(B, 1);                                                  \
        }
        if (bits == 4) { ANY4_STREAM_HB(4) }
        if (bits == 3) { ANY4_STREAM_HB(3) }
        ANY4_STREAM_HB(2)
#undef ANY4_STREAM_HB
#undef ANY4_STREAM_H
    }
    if (bits == 4 && lut == nullptr) {                     // the integer grid: no table
        if (repacked || lr != 0) return hipErrorInvalidValue;
#define ANY4_STREAM_NL(GW)                                                                 \
    (sp.aux ? launch_stream_t<4, GW, true, true>(p, grid, stream) : launch_stream_t<4, GW, false, true>(p, grid, stream))
        switch (sp.gw) {
            case 4: return ANY4_STREAM_NL(4);
            case 2: return ANY4_STREAM_NL(2);
            default: return ANY4_STREAM_NL(1);
        }
#undef ANY4_STREAM_NL
    }
    if (lr < 0) {
        // groups of 64 weights: at most 8 rows a launch
        if (repacked || lr != -1 || M > stream::kTile / 2) return hipErrorInvalidValue;
        // (any2: every wavefront reads its own scales - no room for the shared slots beside its tables)
#define ANY4_STREAM_F(B, GW, SHARE)                                                        \
        return sp.aux && SHARE ? launch_stream_t<B, GW, SHARE, false, false, false, true>(p, grid, stream)   \
                               : launch_stream_t<B, GW, false, false, false, false, true>(p, grid, stream)
#define ANY4_STREAM_FB(B, SHARE)                                                           \
        switch (sp.gw) {                                                                   \
            case 4: ANY4_STREAM_F(B, 4, SHARE);                                            \
            case 2: ANY4_STREAM_F(B, 2, SHARE);                                            \
            default: ANY4_STREAM_F(B, 1, SHARE);                                           \
        }
        if (bits == 4) { ANY4_STREAM_FB(4, true) }
        if (bits == 3) { ANY4_STREAM_FB(3, true) }
        ANY4_STREAM_FB(2, false)
#undef ANY4_STREAM_FB
#undef ANY4_STREAM_F
    }
    if (lr > 0) {
        // groups of 256 weights and more: the variants that read one scale per group
        if (repacked) return hipErrorInvalidValue;
#define ANY4_STREAM_C(B, GW)                                                               \
        return sp.aux ? launch_stream_t<B, GW, true, false, false, true>(p, grid, stream)  \
                      : launch_stream_t<B, GW, false, false, false, true>(p, grid, stream)
#define ANY4_STREAM_CB(B)                                                                  \
        switch (sp.gw) {                                                                   \
            case 4: ANY4_STREAM_C(B, 4);                                                   \
            case 2: ANY4_STREAM_C(B, 2);                                                   \
            default: ANY4_STREAM_C(B, 1);                                                  \
        }
        if (bits == 4) { ANY4_STREAM_CB(4) }
        if (bits == 3) { ANY4_STREAM_CB(3) }
        ANY4_STREAM_CB(2)
#undef ANY4_STREAM_CB
#undef ANY4_STREAM_C
    }
    if (repacked) {
        if (bits == 4) return launch_stream_b<4, true>(p, sp, grid, stream);
        if (bits == 3) return launch_stream_b<3, true>(p, sp, grid, stream);
        return launch_stream_b<2, true>(p, sp, grid, stream);
    }
    if (bits == 4) return launch_stream_b<4, false>(p, sp, grid, stream);
    if (bits == 3) return launch_stream_b<3, false>(p, sp, grid, stream);
    return launch_stream_b<2, false>(p, sp, grid, stream);
}

}  // namespace any4
