/*
 * Host-sanitizer driver for the CPU oracle (test infrastructure).
 *
 * Built by tests/test_host_sanitizers.py with gcc -fsanitize=address,undefined and run
 * on the CPU.  Every buffer is a heap allocation of exactly the size the call is told
 * about, so a read or write one element past the end, a misaligned access or signed
 * overflow inside the oracle ends the run with a sanitizer report.  The values
 * computed are not checked here (the pins do that); a few self-evident ones are.
 */
#include "../../oracle/evo_oracle.c"

#include <stdio.h>

static uint32_t rng_state = 0x2510u;
static uint32_t rng(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return rng_state;
}

static int fail(const char *what)
{
    printf("FAIL %s\n", what);
    return 1;
}

static int run_check(int dtype, uint64_t n)
{
    const size_t es = dtype == ORACLE_F32 ? 4 : 2;
    unsigned char *ref = (unsigned char *)malloc(n * es ? n * es : 1);
    unsigned char *cand = (unsigned char *)malloc(n * es ? n * es : 1);
    oracle_check_acc whole, parts;
    uint64_t done = 0;
    if (!ref || !cand) return fail("malloc");
    for (size_t i = 0; i < n * es; ++i) {   /* arbitrary bit patterns: NaN, Inf, subnormals */
        ref[i] = (unsigned char)(rng() >> 24);
        cand[i] = (rng() & 3u) ? ref[i] : (unsigned char)(rng() >> 24);
    }
    oracle_check_init(&whole);
    oracle_check_chunk(&whole, ref, cand, n, dtype, 1e-2f, 1e-2f);
    /* the same tensor in ragged chunks: exact fields must agree */
    oracle_check_init(&parts);
    while (done < n) {
        uint64_t step = 1 + rng() % 97u;
        if (step > n - done) step = n - done;
        oracle_check_chunk(&parts, ref + done * es, cand + done * es, step, dtype, 1e-2f, 1e-2f);
        done += step;
    }
    free(ref);
    free(cand);
    if (whole.n_seen != n || parts.n_seen != n) return fail("n_seen");
    if (whole.n_mismatch != parts.n_mismatch || whole.n_finite != parts.n_finite ||
        whole.flags != parts.flags || whole.valid != parts.valid ||
        memcmp(&whole.max_abs_err, &parts.max_abs_err, 4) ||
        memcmp(&whole.max_rel_err, &parts.max_rel_err, 4))
        return fail("chunked feeding changed an exact field");
    if (whole.flags & ORACLE_F_INTERNAL) return fail("internal assertion");
    if (whole.valid != (whole.n_mismatch == 0)) return fail("valid");
    return 0;
}

static int run_fitness(uint32_t P, uint32_t T)
{
    float *tim = (float *)malloc((size_t)P * T * sizeof(float));
    float *base = (float *)malloc((size_t)T * sizeof(float));
    uint32_t *valid = (uint32_t *)malloc(P * sizeof(uint32_t));
    float *med = (float *)malloc(P * sizeof(float)), *mean = (float *)malloc(P * sizeof(float));
    float *spd = (float *)malloc(P * sizeof(float)), *fit = (float *)malloc(P * sizeof(float));
    uint32_t *elite = NULL;
    float bm = 0.0f;
    oracle_pop pop;
    int rc = 0;
    if (!tim || !base || !valid || !med || !mean || !spd || !fit) return fail("malloc");
    for (uint32_t i = 0; i < P * T; ++i) tim[i] = 1.0f + (float)(rng() >> 8) * 0x1p-24f;
    for (uint32_t i = 0; i < T; ++i) base[i] = 2.0f + (float)(rng() >> 8) * 0x1p-24f;
    for (uint32_t p = 0; p < P; ++p) valid[p] = (rng() >> 16) & 1u;
    if (P > 2) tim[2 * T] = -1.0f;   /* an unusable row */
    if (oracle_fitness(tim, base, P, T, valid, med, mean, spd, fit, &bm, &pop) != 0)
        rc = fail("oracle_fitness status");
    if (!rc && (pop.best_idx > P || pop.n_valid > P || !(pop.best_speedup >= 1.0f)))
        rc = fail("population figures out of range");
    for (uint32_t k = 1; !rc && k <= P; ++k) {
        uint32_t feasible = 0, got;
        elite = (uint32_t *)malloc(k * sizeof(uint32_t));
        if (!elite) return fail("malloc");
        for (uint32_t p = 0; p < P; ++p) feasible += fit[p] > 0.0f;
        got = oracle_select_elite(fit, P, k, elite);
        if (got != (feasible < k ? feasible : k)) rc = fail("elite count");
        for (uint32_t i = 0; !rc && i < k; ++i)
            if ((i < got) != (elite[i] < P)) rc = fail("elite slot");
        free(elite);
    }
    free(tim); free(base); free(valid); free(med); free(mean); free(spd); free(fit);
    return rc;
}

int main(void)
{
    static const uint64_t sizes[] = {0, 1, 2, 7, 64, 1000, 4099};
    static const uint32_t Ts[] = {1, 2, 3, 5, 100, 101, 4096};
    int rc = 0;
    for (int dtype = ORACLE_F32; dtype <= ORACLE_F16; ++dtype)
        for (size_t i = 0; i < sizeof sizes / sizeof sizes[0]; ++i) rc |= run_check(dtype, sizes[i]);
    for (uint32_t h = 0; h < 65536u; h += 257u) (void)oracle_half_to_float((uint16_t)h);
    for (size_t i = 0; i < sizeof Ts / sizeof Ts[0]; ++i) {
        rc |= run_fitness(1, Ts[i]);
        rc |= run_fitness(5, Ts[i]);
    }
    if (oracle_acc_size() != sizeof(oracle_check_acc)) rc |= fail("acc size");
    puts(rc ? "san_oracle: FAILED" : "san_oracle: ok");
    return rc;
}
