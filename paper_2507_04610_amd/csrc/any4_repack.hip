// any4_repack: packed codes, row-major -> the tile-major layout the small-M kernel streams best.
// The any4 paper re-arranges the weights offline so that what a lane loads is already its operand
// of the matrix instruction (section 4.2, second paragraph).  With lane (n, q) of a wavefront on
// row n of a 16-row tile and quarter q of a 128-code group, the row-major layout already gives a
// lane its 32 codes as one contiguous load; what the re-layout adds on this GPU is that the 64
// loads of one wavefront instruction become one contiguous piece of memory (64 * 4 * bits bytes)
// instead of 16 pieces of 64 bytes from 16 rows.
//   unit (t, g)  = the codes of rows 16 t .. 16 t + 15, group g; units in order (t, g)
//   piece 16 q + n of a unit = codes 32 q .. 32 q + 31 of group g of row 16 t + n (bits words)
//   rows past N in the last tile are zero
#include "any4_device.h"
#include "any4_internal.h"

namespace any4 {

// One thread moves one piece.  Threads are ordered like the INPUT (row, then piece along the row),
// so a wavefront reads contiguous memory and scatters 4 * bits bytes per lane.
template <int BITS>
__global__ __launch_bounds__(256) void repack_kernel(const uint32_t* __restrict__ in, int64_t N, int64_t G,
                                                     uint32_t* __restrict__ out) {
    const int64_t rows = (N + 15) / 16 * 16;
    const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;          // (row, 4 g + q)
    if (id >= rows * G * 4) return;
    const int64_t r = id / (G * 4), gq = id % (G * 4), g = gq >> 2, q = gq & 3;
    uint32_t w[BITS];
#pragma unroll
    for (int j = 0; j < BITS; ++j) w[j] = r < N ? in[id * BITS + j] : 0u;   // row r, words (4 g + q) * BITS ..
    uint32_t* o = out + ((((r >> 4) * G + g) * 64) + 16 * q + (r & 15)) * BITS;
#pragma unroll
    for (int j = 0; j < BITS; ++j) o[j] = w[j];
}

hipError_t launch_repack(const uint32_t* codes, int64_t N, int64_t K, int bits, uint32_t* out, hipStream_t stream) {
    const int64_t G = K / kGroup, rows = (N + 15) / 16 * 16;
    const int64_t blocks = (rows * G * 4 + 255) / 256;
    if (blocks > 0x7FFFFFFF) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(256);
    switch (bits) {
        case 4: hipLaunchKernelGGL(repack_kernel<4>, grid, block, 0, stream, codes, N, G, out); break;
        case 3: hipLaunchKernelGGL(repack_kernel<3>, grid, block, 0, stream, codes, N, G, out); break;
        default: hipLaunchKernelGGL(repack_kernel<2>, grid, block, 0, stream, codes, N, G, out); break;
    }
    return hipGetLastError();
}

}  // namespace any4
