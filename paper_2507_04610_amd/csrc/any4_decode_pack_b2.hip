// The 2-bit variants of the packed-activation kernel (a translation unit per code width keeps the
// build parallel).
#include "any4_decode_pack.h"

namespace any4 {

hipError_t launch_pack_bits2(const pack::Params& p, const PackPlan& pl, bool repacked, hipStream_t stream) {
    return repacked ? launch_pack_b<2, true>(p, pl, stream) : launch_pack_b<2, false>(p, pl, stream);
}

}  // namespace any4
