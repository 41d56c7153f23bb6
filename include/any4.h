/*
 * any4.h - C ABI of libany4: the inference hot path of any4 (learned per-row 4-bit
 * numeric format; also 3- and 2-bit "anyn") on AMD MI355X (gfx950).
 *
 * The operation (any4 paper, section 4.2 "tinygemm Library", first paragraph):
 *     y = x w^T,   x: M x K activations,   w: N x K quantised weights,   y: M x N
 * where every weight is stored as an n-bit code that indexes the 2^n-entry lookup
 * table of its own output row (section 2.4.1) and is dequantised with the scale and
 * offset of its group of 128 consecutive weights along K (section 2.5.1 "Groupwise",
 * section 2.5.2: dequant(w_Q) = alpha * w_Q + beta):
 *     w[n][k] = LUT[n][code[n][k]] * scale[n][k/128] + offset[n][k/128].
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library never
 *     allocates, frees or keeps them.  All matrices are dense, row-major, no strides.
 *   - bf16 values travel as uint16_t bit patterns.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream) and the call returns without waiting for it.
 *   - Return value: ANY4_OK (0) or a negative error code.  Every argument check and every
 *     device-independent refusal happens before the first launch: on any error other than
 *     ANY4_ERR_HIP nothing was launched and no output byte was written.  ANY4_ERR_HIP means the
 *     HIP runtime refused a launch; calls that are served by several launches (any4_gemm with
 *     16 < M <= 128 or with groups of 64 and 8 < M <= 16, and the matrix-core path, whose
 *     group-sum pre-pass precedes the GEMM kernel) may then have written part of y or of the
 *     workspace: their contents are unspecified.  No exception or abort crosses the ABI.
 *   - K must be a positive multiple of 128 (the group size); M, N >= 1; bits is 4, 3
 *     or 2.  Every pointer must be 16-byte aligned.
 *   - The library keeps no state between calls that affects results: the only process-wide data
 *     are one-time, per-device set-up flags (the raised LDS limit of a kernel).  Calls on
 *     different streams may run concurrently as long as their outputs and workspaces do not
 *     overlap; two calls that share a workspace must not overlap in time.
 *
 * Packed code layout (codes[N][K*bits/32], uint32 words, per row, along K):
 *   bits = 4:  8 codes per word, code k in bits [4(k%8), 4(k%8)+4) of word k/8
 *   bits = 2: 16 codes per word, code k in bits [2(k%16), 2(k%16)+2) of word k/16
 *   bits = 3:  one contiguous little-endian bit stream per row: code k occupies bits
 *              [3k, 3k+3) of the row, counted from bit 0 of word 0 (a code may straddle
 *              two words); a row is 3K/32 words.
 */
#ifndef ANY4_H
#define ANY4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ANY4_OK             0
#define ANY4_ERR_NULL      -1   /* a required pointer is NULL */
#define ANY4_ERR_SHAPE     -2   /* M, N or K < 1, or K not a multiple of 128 */
#define ANY4_ERR_BITS      -3   /* bits is not 4, 3 or 2 */
#define ANY4_ERR_ALIGN     -4   /* a pointer is not 16-byte aligned */
#define ANY4_ERR_WORKSPACE -5   /* workspace smaller than any4_gemm_workspace_bytes() */
#define ANY4_ERR_HIP       -6   /* the HIP runtime refused a launch */

#define ANY4_GROUP 128          /* weights per scale/offset group along K */

/*
 * any4_pack - offline packing of codes (one per byte) into the layout above.
 * The paper pre-arranges weights offline as well (section 4.2, second paragraph);
 * its tile order is specific to its hardware, the layout here is the plain row-major one.
 *   codes_u8  in   uint8 [N][K], each value < 2^bits (higher bits are masked off)
 *   codes     out  uint32 [N][K*bits/32], fully overwritten
 */
int any4_pack(const uint8_t* codes_u8, int64_t N, int64_t K, int bits,
              uint32_t* codes, void* stream);

/*
 * any4_dequant - materialise the dequantised weights (sections 2.4.1 and 2.5.2):
 *     w[n][k] = fma(LUT[n][code], scale[n][k/128], offset[n][k/128])
 * evaluated in fp32 with a single rounding; the result is defined bit for bit.
 *   codes   in   uint32 [N][K*bits/32]
 *   lut     in   bf16   [N][2^bits]   the row's table; entry order carries no meaning.
 *                With bits = 4, lut may be NULL: the table of every row is then the integer
 *                grid -8 .. 7 (value = code - 8), the uniform int4 format the paper compares
 *                with (section 4.2, last paragraph); any4_gemm runs it without any table.
 *   scale   in   bf16   [N][K/128]
 *   offset  in   bf16   [N][K/128]
 *   w       out  fp32   [N][K], fully overwritten
 */
int any4_dequant(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                 const uint16_t* offset, int64_t N, int64_t K, int bits,
                 float* w, void* stream);

/*
 * any4_gemm - y[m][n] = sum_k x[m][k] * w[n][k] with w as defined above, never
 * materialised (section 4.2: weights are dequantised on the fly inside the GEMM).
 * Products are accumulated in fp32 (order unspecified but fixed for given shapes: the
 * result is reproducible run to run); y is rounded to bf16, round-to-nearest-even.
 * Small M (<= 16, token generation) takes a memory-bound kernel, large M a
 * matrix-core kernel, M up to 128 whichever of the two a cost model expects to be
 * faster (the memory-bound kernel then runs once per 16 rows of x); the choice depends
 * only on (M, N, K, bits) and the number of compute units of the device.
 *   x          in   bf16 [M][K]
 *   lut        as for any4_dequant, including NULL = int4 grid for bits = 4
 *   y          out  bf16 [M][N], fully overwritten
 *   workspace  scratch of at least any4_gemm_workspace_bytes(M, N, K, bits) bytes,
 *              16-byte aligned; may be NULL when that size is 0.  Contents on entry
 *              are ignored (no initialisation is needed), contents on exit are unspecified.
 *              A workspace must not serve two calls that overlap in time, and after a
 *              launch that did not run to its end (a device reset, an aborted process
 *              sharing the memory) it should be cleared or replaced: a half-finished
 *              call can leave arrival counters that look like its successor's own.
 */
int any4_gemm(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
              const uint16_t* scale, const uint16_t* offset,
              int64_t M, int64_t N, int64_t K, int bits,
              uint16_t* y, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace any4_gemm needs for this problem (0 for invalid arguments). */
size_t any4_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K, int bits);

/*
 * any4_dequant_f16 / any4_gemm_f16 - the same two operations with IEEE fp16 in place of bf16
 * (section 2.4.1 names bfloat16 and float16 as the types of the table entries): lut, scale, offset,
 * x and y are fp16 bit patterns; the products and sums are fp32 as before, w is fp32, y is
 * rounded to fp16 (nearest even).  Groups of 128, plain code layout, a table is required
 * (lut == NULL returns ANY4_ERR_NULL).  Shapes, alignment, workspace (any4_gemm_workspace_bytes)
 * and error behaviour are those of any4_dequant / any4_gemm; for M <= 16, K > 262144 returns
 * ANY4_ERR_SHAPE.  The sums of 128 consecutive activations must stay inside the fp16 range
 * (|sum| < 65504): they pass through fp16 pairs on their way to the matrix cores.
 */
int any4_dequant_f16(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                     const uint16_t* offset, int64_t N, int64_t K, int bits, float* w, void* stream);
int any4_gemm_f16(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                  const uint16_t* scale, const uint16_t* offset,
                  int64_t M, int64_t N, int64_t K, int bits,
                  uint16_t* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * any4_dequant_grouped / any4_gemm_grouped - the same two operations with a scale and an offset
 * shared by `group` consecutive weights along K instead of 128 (section 2.5.1, "Groupwise"; the
 * paper's Table 4 varies the group size): scale and offset are bf16 [N][K/group].
 *   group   64, 128, 256, 512 or 1024 (the range of Table 4), and a divisor of K; anything else
 *           returns ANY4_ERR_SHAPE.  With group = 64 and M <= 16 the weights are streamed once per
 *           8 rows of x (two launches for M > 8); for 16 < M the matrix-core kernel is used.
 * Every other argument, the workspace size (any4_gemm_workspace_bytes) and the error behaviour
 * are those of any4_dequant / any4_gemm; with group = 128 the calls are identical to them.
 * any4_gemm_grouped needs a table (lut != NULL) unless group = 128.
 * For M <= 16, K > 262144 is served for group = 128 only (ANY4_ERR_SHAPE otherwise).
 */
int any4_dequant_grouped(const uint32_t* codes, const uint16_t* lut, const uint16_t* scale,
                         const uint16_t* offset, int64_t N, int64_t K, int bits, int group,
                         float* w, void* stream);
int any4_gemm_grouped(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                      const uint16_t* scale, const uint16_t* offset,
                      int64_t M, int64_t N, int64_t K, int bits, int group,
                      uint16_t* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * any4_dequant_single_table / any4_gemm_single_table - the same two operations for formats that keep
 * ONE table for the whole matrix instead of one per row (the paper's nf4 and af4 comparisons: section
 * 2.4.1, last paragraph; section 5, "Speed Comparisons"): lut1 is bf16 [1][2^bits] and serves every
 * row, w[n][k] = lut1[code[n][k]] * scale[n][k/128] + offset[n][k/128].  The kernels build their lookup
 * structure from it once per block (not once per 16 rows) and read no per-row tables; everything else
 * - groups of 128, bf16, plain code layout, shapes, alignment, workspace (any4_gemm_workspace_bytes),
 * error behaviour - is that of any4_dequant / any4_gemm, and so is the result: the same bits as with lut1
 * repeated N times.  lut1 must not be NULL.
 */
int any4_dequant_single_table(const uint32_t* codes, const uint16_t* lut1, const uint16_t* scale,
                              const uint16_t* offset, int64_t N, int64_t K, int bits, float* w, void* stream);
int any4_gemm_single_table(const uint16_t* x, const uint32_t* codes, const uint16_t* lut1,
                           const uint16_t* scale, const uint16_t* offset,
                           int64_t M, int64_t N, int64_t K, int bits,
                           uint16_t* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * any4_repack - re-arrange packed codes offline into the order the kernels read them in.
 * The paper stores the weights in the operand order of the matrix instruction so that a lane's
 * load needs no shuffling (section 4.2, second paragraph).  On this GPU the row-major layout
 * already hands every lane its operand as one contiguous load; the tile-major layout produced
 * here additionally makes the 64 loads of one wavefront instruction one contiguous piece of
 * memory, which streams 6 - 9 % faster at small M:
 *   rows form tiles of 16; the codes of (tile t, group g of 128 codes) are one unit of 64 pieces,
 *   units in order (t, g); piece 16 * q + n of a unit holds codes 32 q .. 32 q + 31 of group g of
 *   row 16 t + n in `bits` words (same bit order as any4_pack); rows past N in the last tile are 0.
 * The layout is an implementation detail of this library version: treat rcodes as opaque.
 *   codes    in   uint32 [N][K*bits/32]          (output of any4_pack)
 *   rcodes   out  any4_repack_bytes(N, K, bits) bytes, fully overwritten; must not overlap codes
 */
int any4_repack(const uint32_t* codes, int64_t N, int64_t K, int bits, uint32_t* rcodes, void* stream);

/* Size of the re-arranged buffer in bytes (0 for invalid arguments). */
size_t any4_repack_bytes(int64_t N, int64_t K, int bits);

/*
 * any4_gemm_repacked - any4_gemm on codes re-arranged by any4_repack; every other argument, the
 * workspace size (any4_gemm_workspace_bytes) and the result, bit for bit, are those of any4_gemm.
 * lut must not be NULL.  For M <= 16, K beyond the streaming kernel's range (K > 262144 at
 * M <= 16) returns ANY4_ERR_SHAPE.
 */
int any4_gemm_repacked(const uint16_t* x, const uint32_t* rcodes, const uint16_t* lut,
                       const uint16_t* scale, const uint16_t* offset,
                       int64_t M, int64_t N, int64_t K, int bits,
                       uint16_t* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * any4_quantize - the step before the GEMM: learn the per-row tables (section 3.2 "any4
 * Algorithm"; appendix, Algorithm 1).  For every row independently:
 *   1. group-wise scaling of section 2.5.1 over groups of 128 weights along K,
 *        asymmetric (symmetric = 0): alpha = (max - min) / (2^bits - 1),      beta = min
 *        symmetric  (symmetric = 1): alpha = max|w| / (2^(bits-1) - 1),       beta = 0
 *      alpha and beta are rounded to bf16 (what the GEMM will read) and then
 *      w_S = (w - beta) / alpha in fp32; a constant group takes alpha = 1;
 *   2. weighted one-dimensional k-means with 2^bits centres on the scaled row, sample weight
 *      alpha * act[k] (scale of the weight's group times the mean absolute activation of its
 *      input channel): k-means++ start (appendix "K-Means Initialization") driven by the
 *      caller's uniform draws u, then the E-step (nearest centre) and the M-step (Eq. B: the
 *      weighted mean of a cluster) alternate in fp64 until no code changes or `iters` centre
 *      updates were made; a cluster without weight keeps its centre;
 *   3. the centres, sorted ascending, become the row's table (bf16), the codes are the indices
 *      of the nearest centres.
 * The outputs feed any4_pack / any4_gemm unchanged: alpha * lut[code] + beta reconstructs w.
 *   w          in   fp32 [N][K]
 *   act        in   fp32 [K], >= 0, mean |activation| per input channel; NULL = all ones
 *   u          in   fp32 [N][2^bits], each in [0, 1): draw q picks centre q of the row's start
 *   iters      in   >= 0, upper bound on the centre updates per row
 *   codes_u8   out  uint8 [N][K], one code per byte (the input format of any4_pack)
 *   lut        out  bf16 [N][2^bits], ascending
 *   scale      out  bf16 [N][K/128]
 *   offset     out  bf16 [N][K/128]
 *   msteps     out  int32 [N], centre updates actually made per row; may be NULL
 * K must not exceed any4_quantize_max_k() (a row is kept in on-chip memory); larger K returns
 * ANY4_ERR_SHAPE.  Needs no workspace.
 */
int any4_quantize(const float* w, const float* act, const float* u, int64_t N, int64_t K,
                  int bits, int symmetric, int iters, uint8_t* codes_u8, uint16_t* lut,
                  uint16_t* scale, uint16_t* offset, int32_t* msteps, void* stream);

/*
 * any4_quantize_with_gap - any4_quantize with its one tuning knob exposed.  Rows of K <= 16384 are
 * sorted once, after which a Lloyd pass (section 3.2, E-step and M-step) costs O(2^bits log K): the
 * clusters are runs of the sorted row, found by binary search with the E-step's own comparison, and
 * their sums are differences of running sums.  That search presumes that unequal centres are further
 * apart than the rounding of a distance; a row in which two unequal centres come closer than
 * centre_gap * max|w_S| is done again from its starting centres by the plain method (every weight
 * against every centre in every pass), which is also the method of longer rows.
 *   centre_gap  >= 0: as described (any4_quantize passes 2^-40); a huge value sends every row with two
 *               unequal centres through the hand-over; < 0: the plain method for all rows.
 * Both methods take every decision in fp64 on the same fp32 inputs and differ only in the
 * association of the fp64 sums.  All other arguments, errors and limits as any4_quantize; NaN for
 * centre_gap returns ANY4_ERR_SHAPE.
 */
int any4_quantize_with_gap(const float* w, const float* act, const float* u, int64_t N, int64_t K,
                           int bits, int symmetric, int iters, double centre_gap, uint8_t* codes_u8,
                           uint16_t* lut, uint16_t* scale, uint16_t* offset, int32_t* msteps,
                           void* stream);

/* Largest K any4_quantize accepts. */
int64_t any4_quantize_max_k(void);

/*
 * any4_gemm_noalloc - any4_gemm for callers that cannot allocate device memory or have no
 * workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same operation, arguments, result (bit for bit) and error codes as any4_gemm,
 * without the workspace arguments: the scratch lives in a device array inside the library,
 * ANY4_NOALLOC_SCRATCH_BYTES per GPU, held from the library's load until the process ends.  The
 * call allocates and frees nothing.
 *   - A problem whose any4_gemm_workspace_bytes() exceeds ANY4_NOALLOC_SCRATCH_BYTES returns
 *     ANY4_ERR_WORKSPACE (nothing launched): use any4_gemm with a workspace of your own.
 *   - All calls on one GPU share that GPU's array: two any4_gemm_noalloc calls that overlap in
 *     time on the same GPU (different streams, or graphs replayed concurrently) race on it and
 *     give undefined results.  Calls that follow each other on one stream are fine.
 *   - The first call on a GPU looks the array's address up (a host-side call into the HIP
 *     runtime); make one call outside any graph capture before capturing.
 */
#define ANY4_NOALLOC_SCRATCH_BYTES (48u << 20)
int any4_gemm_noalloc(const uint16_t* x, const uint32_t* codes, const uint16_t* lut,
                      const uint16_t* scale, const uint16_t* offset,
                      int64_t M, int64_t N, int64_t K, int bits, uint16_t* y, void* stream);

/* Static, human-readable text for a return code. */
const char* any4_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int any4_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ANY4_H */
