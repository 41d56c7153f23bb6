// Host side of the packed-activation kernel for M <= 4 (any4_decode_pack.h): which problems it takes,
// its work split and the launch.
#include "any4_decode_pack.h"

namespace any4 {

// Whether and how the packed-activation kernel takes a problem; a pure function of its arguments.
PackPlan plan_pack(int64_t M, int64_t N, int64_t K, int bits, bool one_table, int cus) {
    PackPlan pl{};
    const int64_t G = K / kGroup;
    const int64_t tiles = (N + pack::kTile - 1) / pack::kTile;
    // (16-byte pieces of the rows of scales: K a multiple of 1024; any2 tables are fetched 16 bytes at a time)
    if (M < 1 || M > 4 || G % 8 != 0 || tiles > 0x7FFFFFFF || cus < 1 || N * (2 << bits) < 16) return pl;
    // the kernel addresses every array with 32-bit offsets (padded to whole tiles for the re-laid-out codes)
    if (tiles * pack::kTile * (K * bits / 8) >= ((int64_t)1 << 31)) return pl;
    const int mp = M == 1 ? 1 : (M == 2 ? 2 : 4);
    const int passes = (int)((G + 4 * pack::kWaves - 1) / (4 * pack::kWaves));
    // K = 4096 (one unit per wavefront and tile): nothing to gain over the streaming kernel, which needs no K
    // slabs there either and is 5 - 10 % faster on such shapes
    if (passes < 2) return pl;
    // the activations of a wavefront's groups must fit two register sets
    if (passes > 8 / mp) return pl;
    pl.mp = mp;
    pl.passes = passes;
    pl.tiles = tiles;
    if (pack::lds_bytes(bits, mp, passes, (int)G) > pack::kLdsPerCu) return pl;
    // as many blocks as the device holds at once (one or two per compute unit): more, started as others
    // finish, measured 5 - 25 % slower (every block pays for its first tile's latency)
    const int64_t slots = (int64_t)cus * (pack::two_blocks(bits, mp, passes) ? 2 : 1);
    pl.nblocks = (int)(tiles < slots ? tiles : slots);
    pl.ok = true;
    return pl;
}

hipError_t launch_decode_pack(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                              const uint16_t* scale, const uint16_t* offset, int64_t M, int64_t N,
                              int64_t K, int bits, bool repacked, bool one_table, const PackPlan& pl, uint16_t* y,
                              hipStream_t stream) {
    if (!pl.ok || !lut) return hipErrorInvalidValue;
    pack::Params p{};
    p.x = x; p.codes = codes; p.lut = lut; p.scale = scale; p.offset = offset; p.y = y;
    p.N = N; p.K = K; p.M = (int)M; p.G = (int)(K / kGroup);
    p.tiles = (int)pl.tiles;
    p.nblocks = pl.nblocks;
    p.tpb = (int)(pl.tiles / pl.nblocks); p.trem = (int)(pl.tiles % pl.nblocks);
    p.codes_bytes = (int)((repacked ? pl.tiles * pack::kTile : N) * (K * bits / 8));
    p.lut_bytes = (int)((one_table ? 1 : N) * (2 << bits));
    p.one_table = one_table ? 1 : 0;
    p.so_bytes = (int)(N * (K / kGroup) * 2);
    if (bits == 4) return launch_pack_bits4(p, pl, repacked, stream);
    if (bits == 3) return launch_pack_bits3(p, pl, repacked, stream);
    return launch_pack_bits2(p, pl, repacked, stream);
}

}  // namespace any4
