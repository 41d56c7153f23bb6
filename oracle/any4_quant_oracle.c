/*
 * CPU oracle for the any-n quantiser (the step that produces codes, per-row lookup
 * tables, group scales and offsets for the GEMM).  TEST INFRASTRUCTURE ONLY: called
 * by the test-suite, the smoke check and the benchmark's cpu_baseline leg; the product
 * library never calls it and shares no code with it.
 *
 * What it computes (any4 paper), row by row, in the paper's order:
 *   1. Group-wise scaling, section 2.5.1 ("Scaling"): for every group of g = 128
 *      consecutive weights of a row, asymmetric
 *          alpha = (max - min) / (Qmax - Qmin),  beta = min,          Qmax - Qmin = 2^n - 1
 *      or symmetric
 *          alpha = max|w| / Qmax,  beta = 0,                           Qmax = 2^(n-1) - 1
 *      and the scaled weight w_S = (w - beta) / alpha.
 *   2. Per-row weighted one-dimensional k-means with 2^n centres on the scaled row
 *      (section 3.2 "any4 Algorithm"; appendix, Algorithm 1): sample j has weight
 *      alpha_j * E|x_j| (scale of its group times the mean absolute activation of its
 *      input channel).
 *        - initialisation: k-means++ (appendix "K-Means Initialization": the variant the
 *          paper finds best), D^2 sampling with the sample weights; the uniform random
 *          numbers it consumes are an INPUT (one per centre), so that any implementation
 *          can be fed the same draws;
 *        - E-step: every scaled weight takes the nearest centre (the last equation of
 *          the E-step: argmin of the squared difference);
 *        - M-step, Eq. (B) of section 3.2 (the last equation of the M-step): a centre is
 *          the weighted mean of the scaled weights assigned to it;
 *        - alternate until the assignment stops changing or `iters` M-steps were done.
 *   3. Emit codes (index of the centre), the centres as the row's table, alpha as scale
 *      and beta as offset, so that dequant = alpha * table[code] + beta (section 2.5.2).
 *
 * Readings where the paper is silent (it delegates to a library k-means):
 *   - scale and offset are stored as bf16, so they are rounded (nearest even) BEFORE the
 *     weights are scaled: w_S = (w - beta_bf16) / alpha_bf16, in fp32 (one rounding per
 *     operation); a constant group (alpha = 0, or alpha that rounds to 0) takes alpha = 1;
 *   - sample weight s = alpha_bf16 * E|x| in fp32; NULL activations mean E|x| = 1;
 *   - k-means arithmetic in fp64; nearest centre by strict '<' scanning centres in index
 *     order (ties go to the lowest index);
 *   - a centre that loses all its samples (or whose samples all have weight 0) keeps its
 *     value;
 *   - when every candidate has zero sampling mass the initialisation takes index
 *     floor(u * K);
 *   - the finished centres are sorted ascending (ties keep their order), the codes are
 *     renumbered accordingly, and the table is stored as bf16(fp32(centre)), both
 *     conversions round-to-nearest-even.
 *
 * Pins (tests/test_quant_oracle_pins.py): the scaling closed forms of section 2.5.1; Lloyd
 * iterations against scikit-learn's KMeans started from the same centres; hand-computed
 * k-means++ picks and their sampling frequencies; fixed-point conditions and a
 * non-increasing weighted error; rows with at most 2^n distinct values; the global optimum
 * by dynamic programming on tiny rows as a lower bound; unit weights reduce to plain k-means.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ANY4QO_GROUP 128
#define ANY4QO_MAXL 16

static float bf16_to_float(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

/* fp32 -> bf16, round to nearest even (finite inputs) */
static uint16_t float_to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    uint32_t bias = ((u >> 16) & 1u) + 0x7FFFu;
    return (uint16_t)((u + bias) >> 16);
}

static int bits_ok(int bits) { return bits == 2 || bits == 3 || bits == 4; }

/* Step 1 for one row: scale / offset of every group (bf16 bit patterns), scaled weights
 * and sample weights (fp32).  act may be NULL (all ones). */
int any4qo_scale_row(const float *w, const float *act, int64_t K, int bits, int symmetric,
                     uint16_t *scale, uint16_t *offset, float *ws, float *s) {
    if (!bits_ok(bits) || K < ANY4QO_GROUP || K % ANY4QO_GROUP) return -1;
    const float qrange = symmetric ? (float)((1 << (bits - 1)) - 1) : (float)((1 << bits) - 1);
    for (int64_t g = 0; g < K / ANY4QO_GROUP; ++g) {
        const float *wg = w + g * ANY4QO_GROUP;
        float mn = wg[0], mx = wg[0], amax = fabsf(wg[0]);
        for (int j = 1; j < ANY4QO_GROUP; ++j) {
            if (wg[j] < mn) mn = wg[j];
            if (wg[j] > mx) mx = wg[j];
            if (fabsf(wg[j]) > amax) amax = fabsf(wg[j]);
        }
        float alpha = symmetric ? amax / qrange : (mx - mn) / qrange;
        float beta = symmetric ? 0.0f : mn;
        uint16_t ab = float_to_bf16(alpha), bb = float_to_bf16(beta);
        if (bf16_to_float(ab) == 0.0f) ab = float_to_bf16(1.0f);
        scale[g] = ab;
        offset[g] = bb;
        const float a = bf16_to_float(ab), b = bf16_to_float(bb);
        for (int j = 0; j < ANY4QO_GROUP; ++j) {
            const int64_t k = g * ANY4QO_GROUP + j;
            const float d = wg[j] - b;
            ws[k] = d / a;
            s[k] = a * (act ? act[k] : 1.0f);
        }
    }
    return 0;
}

/* smallest index whose inclusive running sum of mass[] exceeds t (mass >= 0, total > 0);
 * the last index with positive mass if rounding lets none exceed it */
static int64_t pick(const double *mass, int64_t K, double t) {
    double run = 0.0;
    int64_t last = 0;
    for (int64_t j = 0; j < K; ++j) {
        run += mass[j];
        if (mass[j] > 0.0) last = j;
        if (run > t) return j;
    }
    return last;
}

/* k-means++ with sample weights: centre 0 is drawn with probability proportional to s,
 * centre q with probability proportional to s * (squared distance to the nearest centre
 * chosen so far); u[q] in [0, 1) is the draw for centre q. */
int any4qo_init(const float *ws, const float *s, int64_t K, int L, const float *u, double *c) {
    double *mass = (double *)malloc((size_t)K * sizeof(double));
    double *d2 = (double *)malloc((size_t)K * sizeof(double));
    if (!mass || !d2) { free(mass); free(d2); return -1; }
    for (int q = 0; q < L; ++q) {
        double total = 0.0;
        for (int64_t j = 0; j < K; ++j) {
            mass[j] = q == 0 ? (double)s[j] : (double)s[j] * d2[j];
            total += mass[j];
        }
        int64_t j;
        if (total > 0.0) j = pick(mass, K, (double)u[q] * total);
        else {
            j = (int64_t)((double)u[q] * (double)K);
            if (j > K - 1) j = K - 1;
        }
        c[q] = (double)ws[j];
        for (int64_t i = 0; i < K; ++i) {
            const double d = (double)ws[i] - c[q];
            const double dd = d * d;
            if (q == 0 || dd < d2[i]) d2[i] = dd;
        }
    }
    free(mass);
    free(d2);
    return 0;
}

/* E-step: nearest centre of every scaled weight; returns how many codes changed */
int64_t any4qo_assign(const float *ws, int64_t K, const double *c, int L, uint8_t *codes) {
    int64_t changed = 0;
    for (int64_t j = 0; j < K; ++j) {
        int best = 0;
        double bd = ((double)ws[j] - c[0]) * ((double)ws[j] - c[0]);
        for (int q = 1; q < L; ++q) {
            const double d = (double)ws[j] - c[q];
            const double dd = d * d;
            if (dd < bd) { bd = dd; best = q; }
        }
        if (codes[j] != (uint8_t)best) ++changed;
        codes[j] = (uint8_t)best;
    }
    return changed;
}

/* M-step: weighted mean of every cluster (Eq. B); empty or weightless clusters keep their centre */
void any4qo_update(const float *ws, const float *s, const uint8_t *codes, int64_t K, double *c, int L) {
    double num[ANY4QO_MAXL], den[ANY4QO_MAXL];
    for (int q = 0; q < L; ++q) num[q] = den[q] = 0.0;
    for (int64_t j = 0; j < K; ++j) {
        num[codes[j]] += (double)s[j] * (double)ws[j];
        den[codes[j]] += (double)s[j];
    }
    for (int q = 0; q < L; ++q)
        if (den[q] > 0.0) c[q] = num[q] / den[q];
}

/* weighted squared error of an assignment: sum_j s_j (ws_j - c[code_j])^2 */
double any4qo_objective(const float *ws, const float *s, const uint8_t *codes, int64_t K, const double *c) {
    double e = 0.0;
    for (int64_t j = 0; j < K; ++j) {
        const double d = (double)ws[j] - c[codes[j]];
        e += (double)s[j] * d * d;
    }
    return e;
}

/* Lloyd iterations from given centres: codes = E(c); up to `iters` times { c = M(codes);
 * codes' = E(c); stop when nothing changed }.  Returns the number of M-steps done. */
int any4qo_lloyd(const float *ws, const float *s, int64_t K, int L, int iters, double *c, uint8_t *codes) {
    memset(codes, 0xFF, (size_t)K);
    any4qo_assign(ws, K, c, L, codes);
    int done = 0;
    while (done < iters) {
        any4qo_update(ws, s, codes, K, c, L);
        ++done;
        if (any4qo_assign(ws, K, c, L, codes) == 0) break;
    }
    return done;
}

/* Step 3 for one row: sort the centres ascending (stable), renumber the codes, store bf16 table */
void any4qo_emit(const double *c, int L, uint8_t *codes, int64_t K, uint16_t *lut) {
    int order[ANY4QO_MAXL], rank[ANY4QO_MAXL];
    for (int q = 0; q < L; ++q) order[q] = q;
    for (int i = 1; i < L; ++i) {                 /* insertion sort: stable */
        const int o = order[i];
        int p = i;
        while (p > 0 && c[order[p - 1]] > c[o]) { order[p] = order[p - 1]; --p; }
        order[p] = o;
    }
    for (int r = 0; r < L; ++r) {
        rank[order[r]] = r;
        lut[r] = float_to_bf16((float)c[order[r]]);
    }
    for (int64_t j = 0; j < K; ++j) codes[j] = (uint8_t)rank[codes[j]];
}

/* The whole quantiser.  w fp32 [N][K]; act fp32 [K] or NULL; u fp32 [N][2^bits] in [0,1);
 * outputs: codes uint8 [N][K], lut bf16 [N][2^bits], scale / offset bf16 [N][K/128];
 * msteps (may be NULL) int32 [N]: M-steps done per row.  Rows are independent; `threads`
 * only spreads them over cores. */
int any4qo_quantize(const float *w, const float *act, const float *u, int64_t N, int64_t K, int bits,
                    int symmetric, int iters, uint8_t *codes, uint16_t *lut, uint16_t *scale,
                    uint16_t *offset, int32_t *msteps, int threads) {
    if (!bits_ok(bits) || N < 1 || K < ANY4QO_GROUP || K % ANY4QO_GROUP || iters < 0) return -1;
    const int L = 1 << bits;
    const int64_t G = K / ANY4QO_GROUP;
    int fail = 0;
    if (threads < 1) threads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (int64_t n = 0; n < N; ++n) {
        float *ws = (float *)malloc((size_t)K * sizeof(float));
        float *s = (float *)malloc((size_t)K * sizeof(float));
        double c[ANY4QO_MAXL];
        if (!ws || !s) { fail = 1; free(ws); free(s); continue; }
        any4qo_scale_row(w + n * K, act, K, bits, symmetric, scale + n * G, offset + n * G, ws, s);
        if (any4qo_init(ws, s, K, L, u + n * L, c) != 0) fail = 1;
        const int done = any4qo_lloyd(ws, s, K, L, iters, c, codes + n * K);
        if (msteps) msteps[n] = done;
        any4qo_emit(c, L, codes + n * K, K, lut + n * L);
        free(ws);
        free(s);
    }
    return fail ? -2 : 0;
}
