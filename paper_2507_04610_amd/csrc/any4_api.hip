// C ABI of libany4 (see include/any4.h): argument validation, kernel selection, launches.
#include "any4.h"
#include "any4_internal.h"
#include "any4_splitk.h"

namespace any4 {

static bool bits_ok(int bits) { return bits == 4 || bits == 3 || bits == 2; }
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static int shape_check(int64_t N, int64_t K, int bits) {
    if (!bits_ok(bits)) return ANY4_ERR_BITS;
    if (N < 1 || K < 1 || K % ANY4_GROUP != 0) return ANY4_ERR_SHAPE;
    return ANY4_OK;
}

// log2(group / 128) for the group sizes the kernels take (64 .. 1024, a divisor of K): -1 .. 3
static bool group_shift(int64_t K, int group, int* lr) {
    for (int l = -1; l <= 3; ++l)
        if (group == (l < 0 ? ANY4_GROUP / 2 : ANY4_GROUP << l)) { *lr = l; return K % group == 0; }
    return false;
}

constexpr int kDecodeMaxM = 16;
constexpr int kStreamMaxM = 16;
constexpr int kChunkedMaxM = 128;      // above this the matrix-core kernel is always taken
constexpr int kFineRows = 8;           // groups of 64 weights: rows of x per launch of the streaming kernel

// Compute units of the current device (256 on MI355X); only shapes the work split, never results.
// Asked of the runtime on every call (the current device may differ from call to call).
int device_compute_units() {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
        n = 256;
    return n;
}

GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K, int bits) {
    GemmPlan p{};
    if (M <= kStreamMaxM && N <= ((int64_t)1 << 35)) {
        p.sp = plan_stream(M, N, K, device_compute_units());
        if (p.sp.gw > 0) {
            p.decode = p.stream = true;
            p.ksplit = p.sp.slabs;
            p.workspace = p.sp.workspace;
            p.counter_bytes = p.sp.slabs > 1 ? splitk_counter_bytes(p.sp.tiles) : 0;
            return p;
        }
    }
    if (M > kStreamMaxM && M <= kChunkedMaxM && N <= ((int64_t)1 << 35)) {
        // A few dozen rows of x fill a fraction of one 256-row tile of the matrix-core kernel, whose
        // time does not depend on M below 256; streaming the weights once per 16 rows is faster while
        //   launches * (6.5 us + bytes of codes / 3.8 TB/s)
        // stays below the matrix-core kernel's time: per round of blocks 8 us + step * K / 64 with
        // step = 0.95 us (few blocks in flight) .. 1.3 us (every compute unit busy), the last round
        // divided by its number of K slices plus 3 + 2 * slices us for adding them up (all constants
        // measured on the two kernels).
        const int cus = device_compute_units();
        const double launches = (double)((M + kStreamMaxM - 1) / kStreamMaxM);
        const double t_stream = launches * (6.5 + (double)N * (double)K * bits / 8.0 / 3.8e6);
        const PrefillPlan pp = plan_prefill(M, N, K, cus);
        const double ksteps = (double)(K / 64);
        const int64_t last = pp.tiles % cus;
        double t_matrix = (double)(pp.tiles / cus) * (8.0 + 1.3 * ksteps);
        if (last > 0) {
            const double busy = (double)(last * pp.tail_s) / cus;
            t_matrix += 8.0 + (0.95 + 0.35 * (busy < 1.0 ? busy : 1.0)) * ksteps / pp.tail_s +
                        (pp.tail_s > 1 ? 3.0 + 2.0 * pp.tail_s : 0.0);
        }
        if (t_stream < t_matrix) {
            const int tail_rows = (int)(M % kStreamMaxM);
            const StreamPlan full = plan_stream(kStreamMaxM, N, K, cus);
            const StreamPlan tail = tail_rows ? plan_stream(tail_rows, N, K, cus) : full;
            if (full.gw > 0 && tail.gw > 0) {
                p.decode = p.stream = p.chunked = true;
                p.sp = full;
                p.sp_tail = tail;
                p.ksplit = full.slabs;
                p.workspace = full.workspace > tail.workspace ? full.workspace : tail.workspace;
                p.counter_bytes = full.slabs > 1 || tail.slabs > 1 ? splitk_counter_bytes(full.tiles) : 0;
                // (groups of 64 weights go to the matrix-core kernel for these M: room for either)
                const size_t wm = prefill_workspace_bytes(M, N, K, cus);
                if (wm > p.workspace) p.workspace = wm;
                return p;
            }
        }
    }
    p.decode = M <= kDecodeMaxM;
    p.ksplit = 1;
    if (p.decode) {
        // one wavefront per (row, K slice): aim for at least ~8K wavefronts in flight, but keep
        // every slice at least one full 64-lane step long
        const int unit_codes = bits == 4 ? 32 : (bits == 2 ? 64 : 128);
        const int64_t steps = (K / unit_codes + 63) / 64;
        int64_t want = (8192 + N - 1) / N;
        if (want > steps) want = steps;
        if (want > 64) want = 64;
        if (want < 1) want = 1;
        p.ksplit = (int)want;
    }
    if (p.decode) p.workspace = p.ksplit > 1 ? (size_t)p.ksplit * (size_t)M * (size_t)N * sizeof(float) : 0;
    else {
        const PrefillPlan pp = plan_prefill(M, N, K, device_compute_units());
        p.workspace = pp.xsums_bytes + pp.counter_bytes + pp.partial_bytes;
        p.counter_offset = pp.xsums_bytes;
        p.counter_bytes = pp.counter_bytes;
    }
    return p;
}

}  // namespace any4

using namespace any4;

namespace any4 {

int gemm_dispatch(const uint16_t* x, const uint32_t* codes, bool repacked, const uint16_t* lut,
                  const uint16_t* scale, const uint16_t* offset, int64_t M, int64_t N, int64_t K,
                  int bits, int group, uint16_t* y, void* workspace, size_t workspace_bytes, void* stream,
                  bool f16, bool one_table) {
    if (!x || !codes || !scale || !offset || !y) return ANY4_ERR_NULL;
    if ((f16 || one_table) && !lut) return ANY4_ERR_NULL;            // fp16 / one table for all rows: a table is required
    if (!lut && (bits != 4 || repacked)) return ANY4_ERR_NULL;       // no table = the 4-bit integer grid, plain layout only
    if (int rc = shape_check(N, K, bits)) return rc;
    if (M < 1) return ANY4_ERR_SHAPE;
    int lr;
    if (!group_shift(K, group, &lr)) return ANY4_ERR_SHAPE;
    if (!lut && lr != 0) return ANY4_ERR_NULL;                           // the table-free path has groups of 128
    if (!aligned16(x) || !aligned16(codes) || !aligned16(lut) || !aligned16(scale) ||
        !aligned16(offset) || !aligned16(y) || !aligned16(workspace))
        return ANY4_ERR_ALIGN;
    const GemmPlan plan = plan_gemm(M, N, K, bits);
    // K beyond the streaming kernel's range: only the plain layout with groups of 128
    if ((repacked || lr != 0 || f16) && plan.decode && !plan.stream) return ANY4_ERR_SHAPE;
    if (plan.workspace > 0 && (!workspace || workspace_bytes < plan.workspace)) return ANY4_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    // one to four rows of x, a table, groups of 128, bf16: the packed-activation kernel (whole K in one
    // block, no workspace) where it takes the shape
    const PackPlan pk = (M <= 4 && lut && lr == 0 && !f16) ? plan_pack(M, N, K, bits, one_table, device_compute_units()) : PackPlan{};
    if (pk.ok) {
        e = launch_decode_pack(x, codes, lut, scale, offset, M, N, K, bits, repacked, one_table, pk, y, s);
    } else if (lr < 0 && plan.stream && !plan.chunked) {
        // groups of 64 weights, M <= 16: the streaming kernel takes 8 rows of x a launch
        e = hipSuccess;
        for (int64_t m0 = 0; m0 < M && e == hipSuccess; m0 += kFineRows) {
            const int64_t rows = M - m0 < kFineRows ? M - m0 : kFineRows;
            e = launch_decode_stream(x + m0 * K, codes, lut, scale, offset, rows, N, K, bits, lr, false, false, one_table, plan.sp,
                                     y + m0 * N, workspace, s);
        }
    } else if (lr < 0) {
        e = launch_prefill(x, codes, lut, scale, offset, M, N, K, bits, lr, false, false, one_table, device_compute_units(), y, workspace, s);
    } else if (plan.chunked) {
        // launches run one after the other on the stream and leave the workspace's counters clean
        e = hipSuccess;
        for (int64_t m0 = 0; m0 < M && e == hipSuccess; m0 += kStreamMaxM) {
            const int64_t rows = M - m0 < kStreamMaxM ? M - m0 : kStreamMaxM;
            e = launch_decode_stream(x + m0 * K, codes, lut, scale, offset, rows, N, K, bits, lr, repacked, f16, one_table,
                                     rows == kStreamMaxM ? plan.sp : plan.sp_tail, y + m0 * N, workspace, s);
        }
    } else if (plan.stream) {
        e = launch_decode_stream(x, codes, lut, scale, offset, M, N, K, bits, lr, repacked, f16, one_table, plan.sp, y, workspace, s);
    } else if (plan.decode) {
        e = launch_decode(x, codes, lut, scale, offset, M, N, K, bits, plan, one_table, y, static_cast<float*>(workspace), s);
    } else {
        e = launch_prefill(x, codes, lut, scale, offset, M, N, K, bits, lr, repacked, f16, one_table, device_compute_units(), y, workspace, s);
    }
    return e == hipSuccess ? ANY4_OK : ANY4_ERR_HIP;
}

}  // namespace any4

extern "C" {

int any4_pack(const uint8_t* codes_u8, int64_t N, int64_t K, int bits, uint32_t* codes, void* stream) {
    if (!codes_u8 || !codes) return ANY4_ERR_NULL;
    if (int rc = shape_check(N, K, bits)) return rc;
    if (!aligned16(codes_u8) || !aligned16(codes)) return ANY4_ERR_ALIGN;
    return launch_pack(codes_u8, N, K, bits, codes, static_cast<hipStream_t>(stream)) == hipSuccess
               ? ANY4_OK : ANY4_ERR_HIP;
}

static int dequant_any(const uint32_t* codes, const uint16_t* lut, bool one_table, const uint16_t* scale,
                       const uint16_t* offset, int64_t N, int64_t K, int bits, int group, float* w,
                       void* stream) {
    if (!codes || !scale || !offset || !w) return ANY4_ERR_NULL;
    if (one_table && !lut) return ANY4_ERR_NULL;
    if (!lut && bits != 4) return ANY4_ERR_NULL;           // no table = the 4-bit integer grid only
    if (int rc = shape_check(N, K, bits)) return rc;
    int lr;
    if (!group_shift(K, group, &lr)) return ANY4_ERR_SHAPE;
    if (!aligned16(codes) || !aligned16(lut) || !aligned16(scale) || !aligned16(offset) || !aligned16(w))
        return ANY4_ERR_ALIGN;
    return launch_dequant(codes, lut, scale, offset, N, K, bits, lr, false, one_table, w, static_cast<hipStream_t>(stream)) == hipSuccess
               ? ANY4_OK : ANY4_ERR_HIP;
}

int any4_dequant_grouped(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                         const uint16_t* offset, int64_t N, int64_t K, int bits, int group, float* w,
                         void* stream) {
    return dequant_any(codes, lut, false, scale, offset, N, K, bits, group, w, stream);
}

int any4_dequant_single_table(const uint32_t* codes, const uint16_t* lut1, const uint16_t* scale,
                              const uint16_t* offset, int64_t N, int64_t K, int bits, float* w, void* stream) {
    return dequant_any(codes, lut1, true, scale, offset, N, K, bits, ANY4_GROUP, w, stream);
}

int any4_dequant_f16(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                     const uint16_t* offset, int64_t N, int64_t K, int bits, float* w, void* stream) {
    if (!codes || !lut || !scale || !offset || !w) return ANY4_ERR_NULL;
    if (int rc = shape_check(N, K, bits)) return rc;
    if (!aligned16(codes) || !aligned16(lut) || !aligned16(scale) || !aligned16(offset) || !aligned16(w))
        return ANY4_ERR_ALIGN;
    return launch_dequant(codes, lut, scale, offset, N, K, bits, 0, true, false, w, static_cast<hipStream_t>(stream)) == hipSuccess
               ? ANY4_OK : ANY4_ERR_HIP;
}

int any4_dequant(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                 const uint16_t* offset, int64_t N, int64_t K, int bits, float* w, void* stream) {
    return any4_dequant_grouped(codes, lut, scale, offset, N, K, bits, ANY4_GROUP, w, stream);
}

int64_t any4_quantize_max_k(void) { return (int64_t)quantize_max_k(); }

int any4_quantize_with_gap(const float* w, const float* act, const float* u, int64_t N, int64_t K, int bits,
                           int symmetric, int iters, double centre_gap, uint8_t* codes_u8, uint16_t* lut,
                           uint16_t* scale, uint16_t* offset, int32_t* msteps, void* stream) {
    if (!w || !u || !codes_u8 || !lut || !scale || !offset) return ANY4_ERR_NULL;
    if (int rc = shape_check(N, K, bits)) return rc;
    if (K > (int64_t)quantize_max_k() || iters < 0 || centre_gap != centre_gap) return ANY4_ERR_SHAPE;
    if (!aligned16(w) || !aligned16(u) || !aligned16(codes_u8) || !aligned16(lut) || !aligned16(scale) ||
        !aligned16(offset) || (act && !aligned16(act)) || (msteps && !aligned16(msteps)))
        return ANY4_ERR_ALIGN;
    return launch_quantize(w, act, u, N, K, bits, symmetric ? 1 : 0, iters, centre_gap, codes_u8, lut, scale, offset,
                           msteps, static_cast<hipStream_t>(stream)) == hipSuccess
               ? ANY4_OK : ANY4_ERR_HIP;
}

int any4_quantize(const float* w, const float* act, const float* u, int64_t N, int64_t K, int bits,
                  int symmetric, int iters, uint8_t* codes_u8, uint16_t* lut, uint16_t* scale,
                  uint16_t* offset, int32_t* msteps, void* stream) {
    return any4_quantize_with_gap(w, act, u, N, K, bits, symmetric, iters, kQuantizeCentreGap, codes_u8, lut, scale,
                                  offset, msteps, stream);
}

size_t any4_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits) {
    if (M < 1 || shape_check(N, K, bits) != ANY4_OK) return 0;
    return plan_gemm(M, N, K, bits).workspace;
}

int any4_gemm(const uint16_t* x, const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
              const uint16_t* offset, int64_t M, int64_t N, int64_t K, int bits, uint16_t* y,
              void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_dispatch(x, codes, false, lut, scale, offset, M, N, K, bits, ANY4_GROUP, y, workspace, workspace_bytes, stream, false, false);
}

int any4_gemm_f16(const uint16_t* x, const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                  const uint16_t* offset, int64_t M, int64_t N, int64_t K, int bits, uint16_t* y,
                  void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_dispatch(x, codes, false, lut, scale, offset, M, N, K, bits, ANY4_GROUP, y, workspace, workspace_bytes, stream, true, false);
}

int any4_gemm_grouped(const uint16_t* x, const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                      const uint16_t* offset, int64_t M, int64_t N, int64_t K, int bits, int group, uint16_t* y,
                      void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_dispatch(x, codes, false, lut, scale, offset, M, N, K, bits, group, y, workspace, workspace_bytes, stream, false, false);
}

int any4_gemm_repacked(const uint16_t* x, const uint32_t* rcodes, const uint16_t* lut, const uint16_t* scale,
                       const uint16_t* offset, int64_t M, int64_t N, int64_t K, int bits, uint16_t* y,
                       void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_dispatch(x, rcodes, true, lut, scale, offset, M, N, K, bits, ANY4_GROUP, y, workspace, workspace_bytes, stream, false, false);
}

int any4_gemm_single_table(const uint16_t* x, const uint32_t* codes, const uint16_t* lut1, const uint16_t* scale,
                           const uint16_t* offset, int64_t M, int64_t N, int64_t K, int bits, uint16_t* y,
                           void* workspace, size_t workspace_bytes, void* stream) {
    return gemm_dispatch(x, codes, false, lut1, scale, offset, M, N, K, bits, ANY4_GROUP, y, workspace, workspace_bytes, stream, false, true);
}

size_t any4_repack_bytes(int64_t N, int64_t K, int bits) {
    if (shape_check(N, K, bits) != ANY4_OK) return 0;
    return (size_t)((N + 15) / 16 * 16) * (size_t)row_words(K, bits) * sizeof(uint32_t);
}

int any4_repack(const uint32_t* codes, int64_t N, int64_t K, int bits, uint32_t* rcodes, void* stream) {
    if (!codes || !rcodes) return ANY4_ERR_NULL;
    if (int rc = shape_check(N, K, bits)) return rc;
    if (!aligned16(codes) || !aligned16(rcodes)) return ANY4_ERR_ALIGN;
    return launch_repack(codes, N, K, bits, rcodes, static_cast<hipStream_t>(stream)) == hipSuccess ? ANY4_OK : ANY4_ERR_HIP;
}

const char* any4_strerror(int code) {
    switch (code) {
        case ANY4_OK: return "ok";
        case ANY4_ERR_NULL: return "a required pointer is NULL";
        case ANY4_ERR_SHAPE: return "bad shape: M, N, K must be >= 1 and K a multiple of 128";
        case ANY4_ERR_BITS: return "bits must be 4, 3 or 2";
        case ANY4_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case ANY4_ERR_WORKSPACE: return "workspace is missing or smaller than any4_gemm_workspace_bytes()";
        case ANY4_ERR_HIP: return "the HIP runtime refused a kernel launch";
        default: return "unknown any4 error code";
    }
}

int any4_version(void) { return 100; }

}  // extern "C"
