/*
 * CPU oracle for the any-n weight-only GEMM.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition the GPU library is checked against.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg may
 * call it; the product library never does and shares no code with it.
 *
 * What it computes (any4 paper):
 *   - every weight is stored as an n-bit code that is a direct, unsigned index
 *     into the 2^n-entry lookup table of ITS OWN ROW (section 2.4.1 "Arbitrary
 *     Non-uniform Quantization: any4"; section 4.2 "tinygemm Library", last
 *     paragraph: the codes are used as LUT indices);
 *   - dequant(w_Q) = alpha * w_Q + beta (section 2.5.2 "Rounding"), with w_Q the
 *     table entry, alpha/beta the scale/offset shared by a group of g = 128
 *     consecutive weights along the reduction dimension (section 2.5.1,
 *     "Groupwise", and the default g stated at the end of that section);
 *   - y = x w^T with x: M x K, w: N x K (section 4.2, first paragraph), i.e.
 *     y[m][n] = sum_k w[n][k] * x[m][k] (section 4.1, the per-element sum).
 *
 * Storage (fixed by the problem statement, not by the paper, whose own kernels
 * use an undisclosed tile order): codes are packed along K into little-endian
 * uint32 words, first code in the lowest bits; 4-bit: 8 per word, 2-bit: 16 per
 * word, 3-bit: one contiguous bit stream per row (a code may straddle two words).
 * Table, scale, offset and activations are bf16 bit patterns (uint16).
 *
 * Precision: the table value, scale and offset are widened to fp32 and combined
 * with ONE fp32 rounding (fmaf); the contraction runs in fp64, sequentially in k.
 *
 * Pins (tests/test_oracle_*.py): exact rational brute force on tiny inputs, the
 * int4 special case LUT = {-8..7}, code/LUT permutation invariance, shared-LUT
 * (nf4-style) equivalence, closed forms (one-hot table, constant codes, zero
 * table, unit-vector activations), reduction to a library fp64 matmul, pack /
 * unpack round trips, and the bits-per-weight figure printed in section 2.4.1.
 * Group sizes other than 128 (the *_g functions): expanding the scales to one per 128 weights
 * (or, for groups of 64, to one per 64) must give the finer-group result bit for bit, a single
 * group per row has a closed form, groups of 64 are checked block by block against numpy.
 * fp16 storage (the *_gd functions with f16 != 0): the widening is checked on all 65536 patterns
 * against numpy's float16, the GEMM against a library fp64 matmul of the widened arrays.
 * The tile-major re-layout (any4o_repack) is pinned by a word-level transpose written
 * with numpy, by reading single codes back out of it, by its zero padding and by the
 * multiset of its words.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ANY4O_GROUP 128

static float bf16_bits_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* IEEE binary16 bit pattern -> float, from the format's definition: 1 sign, 5 exponent (bias 15),
 * 10 fraction bits; exponent 0 = zero / subnormal (fraction * 2^-24), 31 = infinity / NaN */
float any4o_f16_bits_to_float(uint16_t h) {
    uint32_t sign = (h >> 15) & 1u, e = (h >> 10) & 31u, m = h & 1023u;
    float v;
    if (e == 0) v = ldexpf((float)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexpf((float)(m + 1024u), (int)e - 25);
    return sign ? -v : v;
}

/* 16-bit storage -> float: bf16, or fp16 (section 2.4.1 names both for the table) */
static float widen(uint16_t b, int f16) { return f16 ? any4o_f16_bits_to_float(b) : bf16_bits_to_float(b); }

static int bits_ok(int bits) { return bits == 2 || bits == 3 || bits == 4; }

/* number of uint32 words that hold one row of K codes */
int64_t any4o_row_words(int64_t K, int bits) { return K * bits / 32; }

/* code k of one packed row */
uint32_t any4o_code(const uint32_t *row, int64_t k, int bits) {
    int64_t b = k * bits;          /* bit position of the code inside the row */
    int64_t word = b / 32;
    int sh = (int)(b % 32);
    uint64_t window = row[word];
    if (sh + bits > 32)            /* only a 3-bit code can straddle two words */
        window |= (uint64_t)row[word + 1] << 32;
    return (uint32_t)((window >> sh) & ((1u << bits) - 1u));
}

/* one code per byte -> packed words.  Returns 0, or -1 on bad arguments,
 * or -2 if some code does not fit in `bits` bits. */
int any4o_pack(const uint8_t *codes_u8, int64_t N, int64_t K, int bits, uint32_t *packed) {
    if (!codes_u8 || !packed || N < 1 || K < 1 || K % ANY4O_GROUP || !bits_ok(bits)) return -1;
    int64_t W = any4o_row_words(K, bits);
    memset(packed, 0, (size_t)(N * W) * sizeof(uint32_t));
    for (int64_t n = 0; n < N; ++n) {
        uint32_t *row = packed + n * W;
        for (int64_t k = 0; k < K; ++k) {
            uint32_t c = codes_u8[n * K + k];
            if (c >> bits) return -2;
            for (int i = 0; i < bits; ++i) {          /* bit by bit: no cleverness */
                int64_t b = k * bits + i;
                if ((c >> i) & 1u) row[b / 32] |= 1u << (b % 32);
            }
        }
    }
    return 0;
}

/* Tile-major re-layout of the packed codes.  The paper re-arranges the weights offline so
 * that what one lane loads is already its operand of the matrix instruction (section 4.2,
 * second paragraph: the data is laid out in the order the tensor-core fragments want and
 * the kernel loads it without any shuffling).  The layout defined here is that idea for a
 * 64-lane wavefront whose lane (n, q) works on row n of a tile of 16 rows and on quarter q
 * of a group of 128 codes:
 *   rows form tiles of 16 (the last tile is padded with rows of zero codes);
 *   the codes of (tile t, group g) are one unit of 64 pieces, units in order (t, g);
 *   piece 16 * q + n of a unit holds codes 32 q .. 32 q + 31 of group g of row 16 t + n,
 *   as a little-endian bit stream of 32 * bits bits, first code in the lowest bits.
 * Written code by code, bit by bit.  Returns 0, or -1 on bad arguments. */
int64_t any4o_repack_words(int64_t N, int64_t K, int bits) {
    if (N < 1 || K < 1 || K % ANY4O_GROUP || !bits_ok(bits)) return -1;
    return (N + 15) / 16 * 16 * any4o_row_words(K, bits);
}

int any4o_repack(const uint32_t *packed, int64_t N, int64_t K, int bits, uint32_t *out) {
    int64_t total = any4o_repack_words(N, K, bits);
    if (!packed || !out || total < 0) return -1;
    int64_t W = any4o_row_words(K, bits), G = K / ANY4O_GROUP;
    memset(out, 0, (size_t)total * sizeof(uint32_t));
    for (int64_t r = 0; r < N; ++r) {
        int64_t t = r / 16, n = r % 16;
        for (int64_t k = 0; k < K; ++k) {
            uint32_t c = any4o_code(packed + r * W, k, bits);
            int64_t g = k / ANY4O_GROUP, q = (k % ANY4O_GROUP) / 32, e = k % 32;
            int64_t piece = (t * G + g) * 64 + 16 * q + n;
            int64_t b0 = piece * 32 * bits + e * bits;       /* bit position in the whole buffer */
            for (int i = 0; i < bits; ++i)
                if ((c >> i) & 1u) out[(b0 + i) / 32] |= 1u << ((b0 + i) % 32);
        }
    }
    return 0;
}

/* w[n][k] = fmaf(LUT[n][code(n,k)], scale[n][k/128], offset[n][k/128]) in fp32.
 * Returns the number of elements for which (v*s)+o, rounded after each step,
 * differs in bit pattern from the fused result (expected 0: a product of two bf16
 * numbers is exact in fp32), or -1 on bad arguments. */
static int group_ok(int64_t K, int64_t group) {
    return group >= 64 && group % 64 == 0 && K % group == 0;
}

/* the same with a group of `group` weights (a multiple of 64 that divides K; the paper's
 * Table 4 varies the group size from 64 to 1024): scale / offset are [N][K / group] */
/* f16 != 0: table, scale and offset (and the activations of the GEMM) are fp16 instead of bf16 */
int64_t any4o_dequant_gd(const uint32_t *packed, const uint16_t *lut, const uint16_t *scale,
                         const uint16_t *offset, int64_t N, int64_t K, int bits, int64_t group, int f16, float *w) {
    if (!packed || !lut || !scale || !offset || !w || N < 1 || K < 1 || K % ANY4O_GROUP || !bits_ok(bits) ||
        !group_ok(K, group))
        return -1;
    int64_t W = any4o_row_words(K, bits), G = K / group, L = 1 << bits;
    int64_t differ = 0;
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t k = 0; k < K; ++k) {
            uint32_t c = any4o_code(packed + n * W, k, bits);
            float v = widen(lut[n * L + c], f16);
            float s = widen(scale[n * G + k / group], f16);
            float o = widen(offset[n * G + k / group], f16);
            float fused = fmaf(v, s, o);
            volatile float prod = v * s;              /* force the intermediate rounding */
            volatile float two_step = prod + o;
            float ts = two_step;
            if (memcmp(&fused, &ts, sizeof fused) != 0) ++differ;
            w[n * K + k] = fused;
        }
    }
    return differ;
}

int64_t any4o_dequant_g(const uint32_t *packed, const uint16_t *lut, const uint16_t *scale,
                        const uint16_t *offset, int64_t N, int64_t K, int bits, int64_t group, float *w) {
    return any4o_dequant_gd(packed, lut, scale, offset, N, K, bits, group, 0, w);
}

int64_t any4o_dequant(const uint32_t *packed, const uint16_t *lut, const uint16_t *scale,
                      const uint16_t *offset, int64_t N, int64_t K, int bits, float *w) {
    return any4o_dequant_g(packed, lut, scale, offset, N, K, bits, ANY4O_GROUP, w);
}

/* y[m][n] = sum_{k=0..K-1} (double)w[n][k] * (double)x[m][k], k ascending, fp64.
 * `threads` > 1 only distributes whole output rows n over OpenMP threads; the
 * arithmetic of every output element is unchanged.  Returns 0 or -1. */
int any4o_gemm_gd(const uint16_t *x, const uint32_t *packed, const uint16_t *lut, const uint16_t *scale,
                  const uint16_t *offset, int64_t M, int64_t N, int64_t K, int bits, int64_t group, int f16,
                  double *y, int threads) {
    if (!x || !packed || !lut || !scale || !offset || !y || M < 1 || N < 1 || K < 1 ||
        K % ANY4O_GROUP || !bits_ok(bits) || !group_ok(K, group))
        return -1;
    int64_t W = any4o_row_words(K, bits), G = K / group, L = 1 << bits;
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
    {
        float *wrow = (float *)malloc((size_t)K * sizeof(float));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int64_t k = 0; k < K; ++k) {
                uint32_t c = any4o_code(packed + n * W, k, bits);
                float v = widen(lut[n * L + c], f16);
                float s = widen(scale[n * G + k / group], f16);
                float o = widen(offset[n * G + k / group], f16);
                wrow[k] = fmaf(v, s, o);
            }
            for (int64_t m = 0; m < M; ++m) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    acc += (double)wrow[k] * (double)widen(x[m * K + k], f16);
                y[m * N + n] = acc;
            }
        }
        free(wrow);
    }
    return 0;
}

int any4o_gemm_g(const uint16_t *x, const uint32_t *packed, const uint16_t *lut, const uint16_t *scale,
                 const uint16_t *offset, int64_t M, int64_t N, int64_t K, int bits, int64_t group,
                 double *y, int threads) {
    return any4o_gemm_gd(x, packed, lut, scale, offset, M, N, K, bits, group, 0, y, threads);
}

int any4o_gemm(const uint16_t *x, const uint32_t *packed, const uint16_t *lut, const uint16_t *scale,
               const uint16_t *offset, int64_t M, int64_t N, int64_t K, int bits, double *y, int threads) {
    return any4o_gemm_g(x, packed, lut, scale, offset, M, N, K, bits, ANY4O_GROUP, y, threads);
}

/* root mean square of n doubles */
double any4o_rms(const double *y, int64_t n) {
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s += y[i] * y[i];
    return n > 0 ? sqrt(s / (double)n) : 0.0;
}

/* Bits of storage per weight for an N x K matrix: codes + per-row table +
 * per-group scale and offset, all 16-bit metadata (section 2.4.1). */
double any4o_bits_per_weight(int64_t K, int bits) {
    double table = (double)(1 << bits) * 16.0 / (double)K;
    double groups = (double)(K / ANY4O_GROUP) * 2.0 * 16.0 / (double)K;
    return (double)bits + table + groups;
}
