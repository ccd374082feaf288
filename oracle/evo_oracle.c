/*
 * evo_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, single-threaded CPU statement of what the fitness-and-validity
 * evaluation step of an LLM-driven kernel-evolution loop computes.  It exists only
 * so that the GPU library can be checked against it; nothing in the product path
 * may call, link or import it, and it shares no header, helper, table or constant
 * with the GPU code.
 *
 * What the paper fixes (EvoEngineer, arXiv 2510.03760):
 *   - Sec. 3.1, Eq. 1: kernel optimisation is  argmin f(p)  s.t.  g(p) = 0 ;
 *     g covers "compiles" and "output matches the reference implementation
 *     across test cases"; f is a performance objective.
 *   - Sec. 4.3 (modular system, two-stage evaluation): stage 2 runs test cases and
 *     compares candidate outputs against the reference outputs; execution time is
 *     then collected over 100 runs.
 *   - Sec. 5.1, "Evaluation Metric": speedup over the baseline kernel; a speedup of
 *     1.0 is assigned when nothing beats the baseline; validity is reported as the
 *     fraction of trials that give valid kernels (Pass@1).
 *   - Appendix, "Limitations and Threats to Validity": run-to-run timing noise is
 *     mitigated by taking the median of multiple runs (Sec. 4.3 and the
 *     reproducibility guidelines say "average": both are emitted here).
 *
 * What the paper does not fix (tolerance form, NaN/Inf rule, relative error at
 * r = 0, even-T median, fitness of an infeasible candidate) is a reading stated
 * next to the code that implements it.
 *
 * Parity status: every function here is pinned by tests that do not use this file
 * to produce their expected values (hand-written truth table and worked examples
 * under tests/golden/, numpy.isclose / numpy.median / math.fsum, an independent
 * element-at-a-time Python brute force, closed forms on the synthetic configs;
 * binary64 tensors: the same table and class fixtures, numpy.isclose in binary64,
 * agreement with the binary32 path where both are exact; integer tensors: Python
 * integers; mean-based speedup: closed forms on exactly summable samples; the
 * rounding order of the tolerance: hand-built examples in which a fused or a
 * wider product flips the verdict).
 *
 * Build:  gcc -O2 -std=c11 -ffp-contract=off -fPIC -shared
 * Every fp32 operation below is rounded on its own (no fused multiply-add, no
 * reassociation, subnormals kept).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum {
    ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F16 = 2,
    ORACLE_F64 = 3, /* IEEE-754 binary64, checked in binary64          */
    ORACLE_I32 = 4, /* two's complement, checked for exact equality    */
    ORACLE_I64 = 5
};

enum { ORACLE_REDUCE_MEDIAN = 0, ORACLE_REDUCE_MEAN = 1 };

enum {
    ORACLE_F_CAND_NAN      = 1u << 0, /* some candidate element is NaN          */
    ORACLE_F_CAND_INF      = 1u << 1, /* some candidate element is +-Inf        */
    ORACLE_F_REF_NAN       = 1u << 2, /* some reference element is NaN          */
    ORACLE_F_REF_INF       = 1u << 3, /* some reference element is +-Inf        */
    ORACLE_F_NAN_SITE_DIFF = 1u << 4, /* NaN on exactly one side at some index  */
    ORACLE_F_INF_DIFF      = 1u << 5, /* an Inf is involved, no NaN, c != r     */
    ORACLE_F_INTERNAL      = 1u << 31 /* an assertion of this file failed       */
};

/* Running per-candidate accumulator; a tensor may be fed in any number of
 * consecutive chunks (counts add, maxima max, sums continue in index order). */
typedef struct {
    uint64_t n_mismatch;
    uint64_t n_finite;
    double   sum_abs_err;
    double   sum_rel_err;
    float    max_abs_err;
    float    max_rel_err;
    uint32_t flags;
    uint32_t valid;
    uint64_t n_seen;
} oracle_check_acc;

typedef struct {
    uint32_t best_idx;     /* P when no candidate has fitness > 0 */
    uint32_t n_valid;
    float    best_speedup; /* floored at 1.0 */
    float    valid_rate;   /* n_valid / P    */
} oracle_pop;

void oracle_check_init(oracle_check_acc *a)
{
    memset(a, 0, sizeof *a);
    a->valid = 1u; /* an empty tensor has no mismatch */
}

/* IEEE-754 binary16 -> binary32, exact: 1 sign, 5 exponent (bias 15), 10 fraction bits.
 * Subnormal halves are normalised by hand; Inf/NaN keep their payload. */
static float half_to_float(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t exp = (h >> 10) & 0x1fu;
    uint32_t frac = h & 0x3ffu;
    uint32_t w;
    float f;
    if (exp == 0x1fu) {                 /* Inf or NaN */
        w = sign | 0x7f800000u | (frac << 13);
    } else if (exp != 0) {              /* normal: rebias 15 -> 127 */
        w = sign | ((exp + 112u) << 23) | (frac << 13);
    } else if (frac == 0) {             /* zero */
        w = sign;
    } else {                            /* subnormal: value = frac * 2^-24 */
        int shift = 0;
        while (!(frac & 0x400u)) {
            frac <<= 1;
            ++shift;
        }
        frac &= 0x3ffu;
        w = sign | ((uint32_t)(113 - shift) << 23) | (frac << 13);
    }
    memcpy(&f, &w, sizeof f);
    return f;
}

float oracle_half_to_float(uint16_t h) { return half_to_float(h); }

/* bf16 is the upper half of an IEEE-754 binary32: widening is exact. */
static float widen(const void *base, uint64_t i, int dtype)
{
    if (dtype == ORACLE_F16)
        return half_to_float(((const uint16_t *)base)[i]);
    if (dtype == ORACLE_BF16) {
        uint16_t h = ((const uint16_t *)base)[i];
        uint32_t w = (uint32_t)h << 16;
        float f;
        memcpy(&f, &w, sizeof f);
        return f;
    }
    return ((const float *)base)[i];
}

/*
 * binary64 tensors: the same rule and statistics with every operation in binary64
 * (the binary32 tolerances are widened exactly).  Reading: a tensor is checked in its
 * own precision.  The two maxima are reported in binary32, each element's value
 * rounded to nearest (rounding is monotone, so this is the rounded maximum; values
 * beyond the binary32 range become +Inf).  Relative error is 0 where |r| is below the
 * smallest normal binary64.
 */
static void check_chunk_f64(oracle_check_acc *a, const double *ref, const double *cand,
                            uint64_t n, float atol, float rtol)
{
    const double atol_d = (double)atol, rtol_d = (double)rtol;
    for (uint64_t i = 0; i < n; ++i) {
        const double rd = ref[i], cd = cand[i];
        const double ard = fabs(rd);
        const double scaled_d = rtol_d * ard;
        const double tol_d = atol_d + scaled_d;
        const int rd_nan = isnan(rd), cd_nan = isnan(cd);
        const int rd_inf = isinf(rd), cd_inf = isinf(cd);
        const int rd_fin = !rd_nan && !rd_inf;
        const int cd_fin = !cd_nan && !cd_inf;
        int match;

        if (cd == rd)
            match = 1;
        else if (rd_fin && cd_fin)
            match = (fabs(cd - rd) <= tol_d);
        else
            match = 0;
        if (!match)
            a->n_mismatch += 1;

        if (cd_nan) a->flags |= ORACLE_F_CAND_NAN;
        if (cd_inf) a->flags |= ORACLE_F_CAND_INF;
        if (rd_nan) a->flags |= ORACLE_F_REF_NAN;
        if (rd_inf) a->flags |= ORACLE_F_REF_INF;
        if (cd_nan != rd_nan) a->flags |= ORACLE_F_NAN_SITE_DIFF;
        if ((cd_inf || rd_inf) && !cd_nan && !rd_nan && cd != rd)
            a->flags |= ORACLE_F_INF_DIFF;

        if (rd_fin && cd_fin) {
            const double dd = fabs(cd - rd); /* may overflow to +Inf: kept */
            double inv_d = 0.0, qd;
            float d32, q32;
            if (ard >= 2.2250738585072014e-308) /* DBL_MIN, smallest normal */
                inv_d = 1.0 / ard;
            qd = dd * inv_d;
            if (isnan(qd))
                a->flags |= ORACLE_F_INTERNAL;
            d32 = (float)dd;
            q32 = (float)qd;
            a->n_finite += 1;
            if (d32 > a->max_abs_err) a->max_abs_err = d32;
            if (q32 > a->max_rel_err) a->max_rel_err = q32;
            a->sum_abs_err += dd;
            a->sum_rel_err += qd;
        }
    }
    a->n_seen += n;
    a->valid = (a->n_mismatch == 0) ? 1u : 0u;
}

/*
 * Integer tensors (index-valued outputs, e.g. of arg-reductions in the
 * "Normalization & Reduction" class of the kernel classification table): exact
 * equality, no tolerance.  d = |c - r| as an exact unsigned integer; its maximum is
 * reported rounded to binary32 (nearest even), its sum in binary64 (each term rounded
 * to binary64, added in index order).  Every element counts as finite; the relative
 * statistics and the flags stay 0.
 */
static void check_chunk_int(oracle_check_acc *a, const void *ref, const void *cand,
                            uint64_t n, int dtype)
{
    for (uint64_t i = 0; i < n; ++i) {
        int64_t r, c;
        uint64_t diff;
        float diff32;
        if (dtype == ORACLE_I32) {
            r = ((const int32_t *)ref)[i];
            c = ((const int32_t *)cand)[i];
        } else {
            r = ((const int64_t *)ref)[i];
            c = ((const int64_t *)cand)[i];
        }
        if (c != r)
            a->n_mismatch += 1;
        diff = (c > r) ? (uint64_t)c - (uint64_t)r : (uint64_t)r - (uint64_t)c;
        diff32 = (float)diff;
        a->n_finite += 1;
        if (diff32 > a->max_abs_err) a->max_abs_err = diff32;
        a->sum_abs_err += (double)diff;
    }
    a->n_seen += n;
    a->valid = (a->n_mismatch == 0) ? 1u : 0u;
}

/*
 * Functional-correctness constraint of Sec. 3.1 / functional testing of Sec. 4.3,
 * for one candidate over n elements, element by element in index order.
 *
 * Readings (the paper only says the outputs are compared):
 *   - "match" is the usual asymmetric all-close test  |c - r| <= atol + rtol*|r|
 *     in fp32, product rounded before the sum;
 *   - c == r always matches (same-sign Inf, +0 vs -0);
 *   - otherwise both sides must be finite: any NaN, Inf against finite, and
 *     +Inf against -Inf are mismatches (strict validity, motivated by the
 *     reward-hacking discussion in the AI-CUDA-Engineer replication appendix);
 *   - error statistics run over the elements where both sides are finite;
 *     relative error is d * (1/|r|) with the reciprocal rounded first, and is
 *     taken as 0 where |r| is below the smallest normal fp32.
 */
void oracle_check_chunk(oracle_check_acc *a, const void *ref, const void *cand,
                        uint64_t n, int dtype, float atol, float rtol)
{
    if (dtype == ORACLE_F64) {
        check_chunk_f64(a, (const double *)ref, (const double *)cand, n, atol, rtol);
        return;
    }
    if (dtype == ORACLE_I32 || dtype == ORACLE_I64) {
        check_chunk_int(a, ref, cand, n, dtype);
        return;
    }
    for (uint64_t i = 0; i < n; ++i) {
        const float r = widen(ref, i, dtype);
        const float c = widen(cand, i, dtype);
        const float ar = fabsf(r);
        const float scaled = rtol * ar;
        const float tol = atol + scaled;
        const int r_nan = isnan(r), c_nan = isnan(c);
        const int r_inf = isinf(r), c_inf = isinf(c);
        const int r_fin = !r_nan && !r_inf;
        const int c_fin = !c_nan && !c_inf;
        int match;

        if (c == r) {
            match = 1;
        } else if (r_fin && c_fin) {
            const float d = fabsf(c - r);
            match = (d <= tol);
        } else {
            match = 0;
        }
        if (!match)
            a->n_mismatch += 1;

        if (c_nan) a->flags |= ORACLE_F_CAND_NAN;
        if (c_inf) a->flags |= ORACLE_F_CAND_INF;
        if (r_nan) a->flags |= ORACLE_F_REF_NAN;
        if (r_inf) a->flags |= ORACLE_F_REF_INF;
        if (c_nan != r_nan) a->flags |= ORACLE_F_NAN_SITE_DIFF;
        if ((c_inf || r_inf) && !c_nan && !r_nan && c != r)
            a->flags |= ORACLE_F_INF_DIFF;

        if (r_fin && c_fin) {
            const float d = fabsf(c - r); /* may overflow to +Inf: kept */
            float inv = 0.0f;
            float q;
            if (ar >= 1.17549435e-38f) /* FLT_MIN, smallest normal */
                inv = 1.0f / ar;
            q = d * inv;
            if (isnan(q)) /* cannot happen: inv == 0 implies d finite */
                a->flags |= ORACLE_F_INTERNAL;
            a->n_finite += 1;
            if (d > a->max_abs_err) a->max_abs_err = d;
            if (q > a->max_rel_err) a->max_rel_err = q;
            a->sum_abs_err += (double)d;
            a->sum_rel_err += (double)q;
        }
    }
    a->n_seen += n;
    a->valid = (a->n_mismatch == 0) ? 1u : 0u;
}

static int cmp_float_asc(const void *pa, const void *pb)
{
    const float x = *(const float *)pa, y = *(const float *)pb;
    return (x > y) - (x < y);
}

/* A timing row is usable when every sample is finite and > 0. */
static int row_usable(const float *row, uint32_t T)
{
    for (uint32_t k = 0; k < T; ++k)
        if (!(row[k] > 0.0f) || isinf(row[k]))
            return 0;
    return 1;
}

static float quiet_nan(void)
{
    const uint32_t w = 0x7fc00000u;
    float f;
    memcpy(&f, &w, sizeof f);
    return f;
}

/* Median (even T: mean of the two middle order statistics, fp32 add then
 * multiply by one half) and mean (fp64 sum in sample order, one division, one
 * rounding to fp32) of one row.  Unusable row: both are the quiet NaN. */
static void row_reduce(const float *row, uint32_t T, float *scratch,
                       float *median, float *mean)
{
    double acc = 0.0;
    if (!row_usable(row, T)) {
        *median = quiet_nan();
        *mean = quiet_nan();
        return;
    }
    memcpy(scratch, row, (size_t)T * sizeof(float));
    qsort(scratch, T, sizeof(float), cmp_float_asc);
    if (T & 1u) {
        *median = scratch[T / 2];
    } else {
        const float s = scratch[T / 2 - 1] + scratch[T / 2];
        *median = 0.5f * s;
    }
    for (uint32_t k = 0; k < T; ++k)
        acc += (double)row[k];
    *mean = (float)(acc / (double)T);
}

/*
 * Objective of Sec. 3.1 with the metric of Sec. 5.1: per candidate, the time of
 * T runs is reduced to its median (and mean), speedup = baseline median /
 * candidate median (fp32 division; with reducer == ORACLE_REDUCE_MEAN, baseline mean /
 * candidate mean instead), fitness = speedup for a candidate that met
 * the constraint and 0 for one that did not.  Population: index of the largest
 * fitness (lowest index on ties, P when every fitness is 0), that fitness
 * floored at 1.0, the number of valid candidates and its ratio to P.
 * Returns 0, or -1 when scratch memory cannot be had.
 */
int oracle_fitness_ex(const float *timings, const float *baseline, uint32_t P,
                      uint32_t T, const uint32_t *valid, int reducer, float *median_ms,
                      float *mean_ms, float *speedup, float *fitness,
                      float *base_median_out, oracle_pop *pop)
{
    float *scratch = (float *)malloc((size_t)(T ? T : 1) * sizeof(float));
    float base_median, base_mean;
    uint32_t best = P, n_valid = 0;
    float best_fit = 0.0f;

    if (!scratch)
        return -1;
    row_reduce(baseline, T, scratch, &base_median, &base_mean);
    if (base_median_out)
        *base_median_out = base_median;

    for (uint32_t p = 0; p < P; ++p) {
        row_reduce(timings + (size_t)p * T, T, scratch, &median_ms[p], &mean_ms[p]);
        if (isnan(median_ms[p]) || isnan(base_median))
            speedup[p] = 0.0f;
        else if (reducer == ORACLE_REDUCE_MEAN) /* the "average over 100 runs" of Sec. 4.3 */
            speedup[p] = base_mean / mean_ms[p];
        else
            speedup[p] = base_median / median_ms[p];
        fitness[p] = valid[p] ? speedup[p] : 0.0f;
        if (valid[p])
            n_valid += 1;
        if (fitness[p] > best_fit) { /* strict: first of equal maxima wins */
            best_fit = fitness[p];
            best = p;
        }
    }
    free(scratch);
    if (pop) {
        pop->best_idx = best;
        pop->n_valid = n_valid;
        pop->best_speedup = (best_fit > 1.0f) ? best_fit : 1.0f;
        pop->valid_rate = (float)n_valid / (float)P;
    }
    return 0;
}

/* The default: timings reduced by their median (appendix on threats to validity). */
int oracle_fitness(const float *timings, const float *baseline, uint32_t P,
                   uint32_t T, const uint32_t *valid, float *median_ms,
                   float *mean_ms, float *speedup, float *fitness,
                   float *base_median_out, oracle_pop *pop)
{
    return oracle_fitness_ex(timings, baseline, P, T, valid, ORACLE_REDUCE_MEDIAN, median_ms,
                             mean_ms, speedup, fitness, base_median_out, pop);
}

/*
 * Elite preservation (population management, Sec. 3.2.2; the EoH-style baseline of the
 * parameter-settings appendix keeps the best 4 of parents plus offspring): the indices of
 * the k candidates with the largest fitness, best first, equal fitness in index order.
 * Only feasible candidates (fitness > 0) qualify; unused slots hold P.  Selection by
 * repeated scan -- O(P*k), no sort.  Returns the number of slots filled.
 */
uint32_t oracle_select_elite(const float *fitness, uint32_t P, uint32_t k, uint32_t *elite)
{
    uint32_t filled = 0;
    for (uint32_t r = 0; r < k; ++r)
        elite[r] = P;
    for (uint32_t r = 0; r < k; ++r) {
        uint32_t best = P;
        for (uint32_t i = 0; i < P; ++i) {
            int taken = 0;
            if (!(fitness[i] > 0.0f))
                continue;
            for (uint32_t q = 0; q < r; ++q)
                if (elite[q] == i)
                    taken = 1;
            if (taken)
                continue;
            if (best == P || fitness[i] > fitness[best])
                best = i; /* strict: the first of equal fitness wins */
        }
        if (best == P)
            break;
        elite[r] = best;
        filled = r + 1;
    }
    return filled;
}

/*
 * Elite preservation with diversity maintenance (the third population-management strategy
 * of Sec. 3.2.2): as oracle_select_elite, but no two selected candidates share a key.  The
 * key is the caller's notion of "the same solution" (a hash of the kernel source, say); of
 * the feasible candidates with one key only the best (lowest index on ties) can be
 * selected.  Repeated scan; returns the number of slots filled, unused slots hold P.
 */
uint32_t oracle_select_elite_diverse(const float *fit, const uint32_t *keys, uint32_t P,
                                     uint32_t k, uint32_t *elite)
{
    uint32_t filled = 0;
    for (uint32_t r = 0; r < k; ++r)
        elite[r] = P;
    for (uint32_t r = 0; r < k; ++r) {
        uint32_t top = P;
        for (uint32_t i = 0; i < P; ++i) {
            int key_taken = 0;
            if (!(fit[i] > 0.0f))
                continue;
            for (uint32_t q = 0; q < r; ++q)
                if (keys[elite[q]] == keys[i])
                    key_taken = 1;
            if (key_taken)
                continue;
            if (top == P || fit[i] > fit[top])
                top = i; /* strict: of equal fitness the first wins */
        }
        if (top == P)
            break;
        elite[r] = top;
        filled = r + 1;
    }
    return filled;
}

uint32_t oracle_acc_size(void) { return (uint32_t)sizeof(oracle_check_acc); }
