/*
 * evo.h -- C ABI of the fitness-and-validity evaluation step of an LLM-driven
 * kernel-evolution loop, for AMD Instinct MI355X (gfx950).
 *
 * Background (EvoEngineer, arXiv 2510.03760).  Sec. 3.1, Eq. 1 states kernel
 * optimisation as  argmin f(p)  subject to  g(p) = 0 : g holds the validity
 * constraints (the code compiles; its output matches the reference implementation
 * across test cases) and f is the performance objective.  Sec. 4.3 describes the
 * evaluator: functional testing compares candidate outputs with reference outputs,
 * then execution time is collected over 100 runs.  Sec. 5.1 ("Evaluation Metric")
 * defines the reported figures: speedup over the baseline kernel, 1.0 when nothing
 * beats the baseline, and the ratio of valid kernels.  The appendix on threats to
 * validity reduces repeated timings by their median.
 *
 * This library evaluates a whole population at once on one GPU: P candidate output
 * tensors are checked against one reference output (evo_check_batch), ragged groups
 * of (reference, candidates) are checked in one launch (evo_check_segmented), and
 * per-candidate timing samples become a median, a speedup and a fitness
 * (evo_fitness).  The compiler stage of g and the program generator are not here.
 *
 * Conventions
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are ordinary process memory.  The library never frees, keeps or
 *     writes caller memory beyond what each call documents.
 *   - Tensors are contiguous and are read as flat arrays; their shape plays no
 *     part in a tolerance check.  EVO_BF16 elements are the upper 16 bits of an
 *     IEEE-754 binary32 and EVO_F16 elements are IEEE-754 binary16, both little
 *     endian; they are widened exactly and every operation is done in binary32.
 *     The other element types are listed with evo_dtype and evo_stats.
 *   - Every call that takes a stream enqueues its work on it and returns (the one
 *     exception is evo_time_candidates); results are defined once the caller has
 *     synchronised that stream.  `stream` is a hipStream_t passed as void* (NULL = the
 *     null stream).
 *   - A context owns scratch memory (partial results, counters, tables) that grows on
 *     demand: a call that needs more than the context holds frees and allocates device
 *     memory (which waits for the device), clears new counters and waits for that.  A
 *     call that repeats a shape the context has already run only enqueues kernels.
 *   - Graph capture.  A call may be recorded into a HIP graph when (a) the context has
 *     run the same call with the same shapes eagerly before, so that its scratch memory
 *     exists, and (b) its descriptors and candidate pointers travel inside the kernel
 *     arguments: at most 8 groups and 384 candidate pointers per call (after rounding
 *     the candidates beyond the last full group of 16 up to a power of two).  While the
 *     stream is capturing, a call that would have to allocate, free, clear or copy from
 *     staging memory returns EVO_ERR_CAPTURE and enqueues nothing.  evo_time_candidates
 *     cannot be captured.
 *   - A context must not be used from two streams or two host threads at once:
 *     consecutive calls reuse its scratch memory in stream order.
 *   - All functions return EVO_OK (0) or a negative evo_status.  Argument errors
 *     are detected on the host before anything is enqueued.  Nothing is printed,
 *     thrown or aborted.
 */
#ifndef EVO_H_
#define EVO_H_

#include <stdint.h>

#if defined(EVO_BUILDING)
#define EVO_API __attribute__((visibility("default")))
#else
#define EVO_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct evo_check evo_check_t; /* opaque, owned by the library */

typedef enum {
    EVO_F32  = 0, /* IEEE-754 binary32                                             */
    EVO_BF16 = 1, /* upper 16 bits of a binary32, checked in binary32               */
    EVO_F16  = 2, /* IEEE-754 binary16, checked in binary32                         */
    EVO_F64  = 3, /* IEEE-754 binary64, checked in binary64                         */
    EVO_I32  = 4, /* two's complement integers (index-valued outputs, e.g. of the   */
    EVO_I64  = 5  /* arg-reductions among the reduction operations of the kernel    */
                  /* classification table): exact equality, tolerances play no part */
} evo_dtype;

typedef enum {
    EVO_OK         = 0,
    EVO_ERR_NULL   = -1, /* a required pointer is NULL                          */
    EVO_ERR_DTYPE  = -2, /* unknown element type                                */
    EVO_ERR_SIZE   = -3, /* zero or out-of-range count (n, P, S, T, rows)       */
    EVO_ERR_TOL    = -4, /* tolerance negative, NaN or infinite; tolerance class */
                         /* out of range or never set                           */
    EVO_ERR_ALIGN  = -5, /* a tensor pointer is not aligned to its element size, or */
                         /* an output pointer not to its record (stats: 8 bytes) */
    EVO_ERR_DEVICE = -6, /* a HIP call failed (no device, launch error, ...)    */
    EVO_ERR_NOMEM  = -7, /* host or device allocation failed                    */
    EVO_ERR_HANDLE = -8, /* not a live context (never created, or destroyed)    */
    EVO_ERR_LIMIT  = -9, /* beyond the fixed capacity of evo_check_batch_static */
    EVO_ERR_CAPTURE = -10, /* the stream is capturing and the call would have to allocate, */
                         /* free, clear or stage (see "Graph capture" above)             */
    EVO_ERR_INTERNAL = -11 /* evo_check_destroy: a guard behind the library's scratch      */
                         /* memory was overwritten (a defect of the library, not a usage error) */
} evo_status;

/* Bits of evo_stats.flags */
enum {
    EVO_F_CAND_NAN      = 1u << 0, /* a candidate element is NaN                 */
    EVO_F_CAND_INF      = 1u << 1, /* a candidate element is +-Inf               */
    EVO_F_REF_NAN       = 1u << 2, /* a reference element is NaN                 */
    EVO_F_REF_INF       = 1u << 3, /* a reference element is +-Inf               */
    EVO_F_NAN_SITE_DIFF = 1u << 4, /* NaN on exactly one side at some index      */
    EVO_F_INF_DIFF      = 1u << 5  /* an Inf involved, no NaN, and c != r        */
};

/*
 * One row per candidate, 72 bytes, 8-byte aligned, in device memory.
 *
 * Element rule (reading of "output must match the reference", Sec. 3.1, with the
 * absolute/relative tolerance of the context; r = reference, c = candidate, all in
 * binary32 with each operation rounded on its own):
 *     match  <=>  c == r,  or  both finite and |c - r| <= atol + rtol*|r|
 * so any NaN, Inf against finite and +Inf against -Inf are mismatches.
 * Statistics run over elements where both sides are finite: d = |c - r| (kept when
 * it overflows to +Inf), q = d * (1/|r|) with the reciprocal rounded first and
 * q = 0 where |r| < FLT_MIN.
 *
 * EVO_F64: the same rule and statistics with every operation in binary64 (atol and rtol
 * widened exactly; q = 0 where |r| < DBL_MIN); the two maxima are reported rounded to
 * binary32 (to nearest; +Inf beyond its range).
 * EVO_I32 / EVO_I64: match <=> c == r.  d = |c - r| is an exact unsigned integer; every
 * element counts as finite; max_abs_err is the largest d rounded to binary32 (to nearest
 * even), sum_abs_err the sum of the d (each rounded to binary64); max_rel_err, sum_rel_err
 * and flags are 0.
 */
typedef struct evo_stats {
    uint64_t n_mismatch;  /* elements failing the rule (exact)                     */
    uint64_t n_finite;    /* elements with both sides finite (exact)               */
    double   sum_abs_err; /* sum of d; summation order is unspecified (1e-6 rel.)  */
    double   sum_rel_err; /* sum of q; summation order is unspecified (1e-6 rel.)  */
    float    max_abs_err; /* max d, 0 when the set is empty (exact)                */
    float    max_rel_err; /* max q, 0 when the set is empty (exact)                */
    uint32_t flags;       /* EVO_F_* bits (exact)                                  */
    uint32_t valid;       /* 1 iff n_mismatch == 0: the constraint g(p) = 0        */
    float    median_ms;   /* evo_fitness: median of the T samples                  */
    float    mean_ms;     /* evo_fitness: mean of the T samples                    */
    float    speedup;     /* evo_fitness: baseline median / candidate median       */
    float    fitness;     /* evo_fitness: valid ? speedup : 0                      */
    uint32_t n_elems_lo;  /* element count of the tensor this row was checked on   */
    uint32_t n_elems_hi;
} evo_stats;

/* One ragged group: a reference and the candidates checked against it. */
typedef struct evo_segment {
    const void        *ref;        /* device, n_elems elements of `dtype`            */
    const void *const *cand_ptrs;  /* HOST array of P_s device pointers              */
    uint64_t           n_elems;    /* > 0                                            */
    uint32_t           P_s;        /* > 0                                            */
    uint32_t           dtype;      /* evo_dtype                                      */
    uint32_t           stats_row0; /* first of the P_s rows this group writes        */
    uint32_t           tol_class;  /* 0: the context's tolerance for `dtype`; 1 ..   */
                                   /* EVO_TOL_CLASSES: that tolerance class          */
} evo_segment;

/* Population figures of Sec. 5.1, one per evo_fitness call, in device memory. */
typedef struct evo_pop_summary {
    uint32_t best_idx;     /* largest fitness, lowest index on ties; P if all are 0 */
    uint32_t n_valid;      /* candidates with valid == 1                            */
    float    best_speedup; /* max(1.0, fitness[best_idx]); 1.0 if none              */
    float    valid_rate;   /* n_valid / P  (Pass@1 of the functional stage)         */
} evo_pop_summary;

/*
 * Creates a context for tensors of `n_elems` elements of `dtype`, checked with the
 * tolerance |c - r| <= atol + rtol*|r| (Sec. 3.1 constraint; tolerance form is this
 * library's reading).  atol and rtol must be finite and >= 0; they are used as the
 * binary32 values given.  Only host work is done here; device scratch memory is
 * allocated by the first call that needs it, on the device current at that time.
 * Errors: EVO_ERR_NULL (out), EVO_ERR_DTYPE, EVO_ERR_SIZE (n_elems == 0),
 * EVO_ERR_TOL, EVO_ERR_NOMEM.  On error *out is set to NULL.
 */
EVO_API int evo_check_create(evo_check_t **out, evo_dtype dtype, uint64_t n_elems,
                     float atol, float rtol);

/*
 * Tolerance policy.  The functional test of Sec. 4.3 compares outputs of operations of
 * very different kinds and precisions (the kernel classification table of the appendix:
 * matrix products, reductions, losses, ...; half-precision and single-precision outputs),
 * and one absolute/relative pair does not fit them all.  A context therefore holds one
 * pair per element type -- all equal to the pair given to evo_check_create until changed
 * here -- and up to EVO_TOL_CLASSES caller-defined classes.  Every group of a call is
 * checked with the pair of its element type, unless its descriptor names a class
 * (evo_segment.tol_class; e.g. "loss outputs", "softmax rows").  The paper states no
 * tolerance values; none is built in.  Integer element types ignore tolerances.
 * Both calls are host-only and take effect for the calls made after them.
 * Errors: EVO_ERR_HANDLE, EVO_ERR_DTYPE (set_tolerance), EVO_ERR_SIZE (class 0 or beyond
 * EVO_TOL_CLASSES), EVO_ERR_TOL.
 */
#define EVO_TOL_CLASSES 15u
EVO_API int evo_check_set_tolerance(evo_check_t *c, evo_dtype dtype, float atol, float rtol);
EVO_API int evo_check_set_tolerance_class(evo_check_t *c, uint32_t tol_class, float atol, float rtol);

/*
 * Functional testing of Sec. 4.3 for a population: checks P candidate tensors
 * against `ref` (each of the context's n_elems elements and dtype) and overwrites
 * stats[0..P) completely (timing fields are set to 0).
 *   ref        device, read only
 *   cand_ptrs  HOST array of P device pointers, read during the call only
 *   stats      device, P rows, written by the enqueued work
 * Each reference element is fetched from memory once and compared with all P
 * candidates.  Tensor pointers must be aligned to the element size; 16-byte
 * alignment gives the fast path.  `stats` must be 8-byte aligned (here and in
 * every other call that writes evo_stats rows).
 * Errors: EVO_ERR_HANDLE, EVO_ERR_NULL (ref, cand_ptrs, any cand_ptrs[i], stats),
 * EVO_ERR_SIZE (P == 0 or P > 65535), EVO_ERR_ALIGN, EVO_ERR_NOMEM, EVO_ERR_DEVICE,
 * EVO_ERR_CAPTURE.
 */
EVO_API int evo_check_batch(evo_check_t *c, const void *ref, const void *const *cand_ptrs,
                    uint32_t P, void *stream, evo_stats *stats);

/*
 * evo_check_batch for callers that cannot allocate device memory: code that runs under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and, for the same arguments, the same stats rows as evo_check_batch; but
 * the partial rows and ticket counters live in a fixed array in the library's device image
 * (EVO_STATIC_SCRATCH_BYTES, about 6 MiB, held by every GPU the library is loaded on until
 * the process ends) instead of context-owned memory, and the call neither allocates nor
 * frees anything, on the device or on the host.  Its first call on a device looks the
 * array's address up (make that call outside a capture).
 * Capacity: P <= 384 after rounding the candidates beyond the last full group of 16 up to a
 * power of two, and at most EVO_STATIC_MAX_JOBS workgroups (a launch is planned for two
 * per compute unit, so on an MI355X only tensors of several GiB each come near it); beyond
 * it the call returns EVO_ERR_LIMIT and enqueues nothing.
 * All calls on one GPU share the one array: calls that overlap in time on one GPU (two
 * streams, two threads, two contexts) race, and the caller must serialise them.  The ticket
 * counters are cleared by a small kernel in front of the check, so the call is two launches.
 * Errors: as evo_check_batch, plus EVO_ERR_LIMIT.
 */
#define EVO_STATIC_MAX_JOBS 1024u
#define EVO_STATIC_SCRATCH_BYTES 6314048u
EVO_API int evo_check_batch_static(evo_check_t *c, const void *ref, const void *const *cand_ptrs,
                                   uint32_t P, void *stream, evo_stats *stats);

/*
 * The same check over S ragged groups in ONE launch (the test cases and output
 * shapes of an operation set differ in size, Sec. 4.3 / operation taxonomy in the
 * appendix).  Group s writes rows [stats_row0, stats_row0 + P_s); row ranges of
 * different groups must not overlap and must lie inside [0, n_rows).  Each group is
 * checked with the tolerance of its element type or of its tolerance class (see
 * evo_check_set_tolerance); the context's n_elems and dtype are ignored.
 *   segs   HOST array of S descriptors (and the host pointer arrays they name),
 *          read during the call only
 *   stats  device, n_rows rows; rows not named by any group are left untouched
 * Errors: as evo_check_batch, plus EVO_ERR_SIZE for S == 0, an empty group, a row
 * range outside n_rows or overlapping another, EVO_ERR_DTYPE per group, EVO_ERR_TOL for
 * a tolerance class that is out of range or was never set, EVO_ERR_CAPTURE.
 */
EVO_API int evo_check_segmented(evo_check_t *c, const evo_segment *segs, uint32_t S,
                        void *stream, evo_stats *stats, uint32_t n_rows);

/*
 * Functional testing over several test cases at once (Sec. 4.3 runs five test cases per
 * candidate; the AI-CUDA-Engineer replication appendix checks five random inputs): K
 * cases, each a reference and the SAME P candidates' outputs for that case, checked in
 * ONE launch.  Row p of stats describes candidate p over all cases together, exactly as
 * if the K tensors of a candidate were one tensor fed case after case: counts and
 * n_elems add, maxima are taken over all cases, the error sums add, flags are OR-ed, and
 * valid = 1 iff no element of any case mismatches.
 *   cases  HOST array of K descriptors with equal P_s (and the host pointer arrays they
 *          name); n_elems and dtype may differ per case; stats_row0 must be 0
 *   stats  device, P_s rows, completely overwritten
 * Errors: as evo_check_segmented, plus EVO_ERR_SIZE for K == 0, unequal P_s or a non-zero
 * stats_row0.
 */
EVO_API int evo_check_cases(evo_check_t *c, const evo_segment *cases, uint32_t K, void *stream,
                            evo_stats *stats);

/*
 * Performance objective of Sec. 3.1 with the metric of Sec. 5.1.  For each of the
 * P candidates: median of its T timing samples (even T: 0.5f*(lo+hi) of the two
 * middle order statistics), mean (binary64 sum in sample order, divided by T,
 * rounded once), speedup = median(baseline) / median(candidate) in binary32, and
 * fitness = stats[p].valid ? speedup : 0.  A row holding a sample that is not
 * finite and > 0 gets median_ms = mean_ms = quiet NaN (0x7fc00000) and speedup =
 * fitness = 0; an unusable baseline does that to every speedup.
 *   timings   device, P*T binary32 milliseconds, row major
 *   baseline  device, T samples of the baseline kernel
 *   stats     device, P rows: `valid` is read (as left by an evo_check_* call that
 *             precedes this one in stream order); median_ms, mean_ms, speedup and
 *             fitness are written; other fields are untouched
 *   summary   device, one record, or NULL
 * Errors: EVO_ERR_HANDLE, EVO_ERR_NULL, EVO_ERR_SIZE (P == 0, T == 0,
 * T > EVO_FITNESS_MAX_T, P > 1048576), EVO_ERR_ALIGN, EVO_ERR_DEVICE.
 */
#define EVO_FITNESS_MAX_T 4096u
EVO_API int evo_fitness(evo_check_t *c, const float *timings, const float *baseline,
                uint32_t P, uint32_t T, void *stream, evo_stats *stats,
                evo_pop_summary *summary);

/*
 * evo_fitness with the reduction of the T samples that feeds the speedup chosen by the
 * caller.  Sec. 4.3 and the reproducibility guidelines average the runs, the appendix on
 * threats to validity takes their median: EVO_REDUCE_MEDIAN (what evo_fitness does) gives
 * speedup = median(baseline) / median(candidate), EVO_REDUCE_MEAN gives
 * mean(baseline) / mean(candidate) with the means as defined above.  median_ms and mean_ms
 * are written either way; everything else is as in evo_fitness.
 * Errors: as evo_fitness, plus EVO_ERR_SIZE for an unknown reducer.
 */
typedef enum { EVO_REDUCE_MEDIAN = 0, EVO_REDUCE_MEAN = 1 } evo_reducer;
EVO_API int evo_fitness_ex(evo_check_t *c, const float *timings, const float *baseline,
                           uint32_t P, uint32_t T, int reducer /* evo_reducer */, void *stream,
                           evo_stats *stats, evo_pop_summary *summary);

/*
 * The whole evaluation of a population in one call: evo_check_cases (K >= 1 test cases of the
 * same P candidates; K = 1 is evo_check_batch on cases[0]) followed by evo_fitness_ex, with
 * the same results as those two calls in that order.  When the K descriptors and K*P
 * candidate pointers fit the kernel argument block (K <= 8, K*P' <= 384, P' being P rounded up
 * to whole groups of 16 plus one power of two; for K = 1 a population such as 17 or 33 counts
 * as two descriptors) it is ONE launch: the
 * timing rows are reduced by the last workgroups of the grid, which start when the first
 * check jobs end, and the last of them or of the check to finish computes speedup, fitness
 * and the population figures.  Larger tables run as two launches.
 * Arguments and errors: as evo_check_cases and evo_fitness_ex; P is cases[0].P_s.
 */
EVO_API int evo_evaluate(evo_check_t *c, const evo_segment *cases, uint32_t K,
                         const float *timings, const float *baseline, uint32_t T,
                         int reducer /* evo_reducer */, void *stream, evo_stats *stats,
                         evo_pop_summary *summary);

/*
 * The ragged counterpart: evo_check_segmented followed by evo_fitness_ex over the same n_rows
 * rows (timings holds one row of T samples per evo_stats row), with the same results as those
 * two calls in that order.  The groups must cover the rows [0, n_rows) exactly, since a row
 * without a group would have no valid flag.  One launch under the condition given for
 * evo_evaluate (S descriptors), else two.
 * Arguments and errors: as evo_check_segmented and evo_fitness_ex (P = n_rows), plus
 * EVO_ERR_SIZE when some row belongs to no group.
 */
EVO_API int evo_evaluate_segmented(evo_check_t *c, const evo_segment *segs, uint32_t S,
                           const float *timings, const float *baseline, uint32_t T, int reducer,
                           void *stream, evo_stats *stats, uint32_t n_rows,
                           evo_pop_summary *summary);

/*
 * Population management of Sec. 3.2.2 (elite preservation): the indices of the k
 * candidates with the largest fitness, best first, equal fitness in index order.  Only
 * feasible candidates (fitness > 0: valid, with usable timings) qualify; slots beyond
 * their number are set to P.
 *   stats     device, P rows; `fitness` is read (as left by an evo_fitness call that
 *             precedes this one in stream order)
 *   elite     device, k entries, all written
 *   n_elite   device, one entry: min(k, number of feasible candidates); may be NULL
 * Errors: EVO_ERR_HANDLE, EVO_ERR_NULL (stats, elite), EVO_ERR_SIZE (P == 0, k == 0,
 * k > P, P > 65535), EVO_ERR_ALIGN, EVO_ERR_DEVICE.
 */
EVO_API int evo_select_elite(evo_check_t *c, const evo_stats *stats, uint32_t P, uint32_t k,
                             void *stream, uint32_t *elite, uint32_t *n_elite);

/*
 * evo_select_elite with diversity maintenance (the third population-management strategy of
 * Sec. 3.2.2): keys[p] is the caller's notion of "the same solution" (a hash of the kernel
 * source, say), and no two selected candidates share a key -- of the feasible candidates with
 * one key only the best (lowest index on ties) competes.  n_elite is min(k, number of
 * distinct keys among the feasible candidates).
 *   keys   device, P entries
 * Errors: as evo_select_elite, plus EVO_ERR_NULL / EVO_ERR_ALIGN for keys, EVO_ERR_NOMEM.
 */
EVO_API int evo_select_elite_diverse(evo_check_t *c, const evo_stats *stats, const uint32_t *keys,
                                     uint32_t P, uint32_t k, void *stream, uint32_t *elite,
                                     uint32_t *n_elite);

/*
 * Timing stage of the evaluator (Sec. 4.3: the execution time of a candidate is collected
 * over 100 runs; the appendix on threats to validity names run-to-run noise): produces the
 * P x T table of milliseconds that evo_fitness consumes.  For every candidate p the library
 * calls launch[p](user[p], stream) `warmup` times untimed and then T times, each timed run
 * bracketed by two device events on `stream`; launch[p] must enqueue exactly one run of the
 * candidate on that stream and return (it must not synchronise the device).
 *   opts->flush_cache  non-zero: before every timed run a 512 MiB scratch buffer is
 *                      overwritten (outside the timed bracket), so that the run does not
 *                      find the previous run's data in the last-level cache
 *   timings            device, P*T binary32 milliseconds, row major, written in stream order
 *   clock_ratio        host, P entries, or NULL: a fixed chain of dependent FMAs is timed
 *                      before the first and after the last timed run of candidate p; entry
 *                      p is after/before (1.0 = the shader clock did not change; a caller
 *                      may discard rows far from 1)
 * Unlike the other calls this one BLOCKS: it returns when every run has completed and the
 * table has been copied.  It allocates events, pinned memory and (with flush_cache) the
 * scratch buffer on first use.
 * Errors: EVO_ERR_HANDLE, EVO_ERR_NULL (launch, any launch[p], timings, opts),
 * EVO_ERR_SIZE (P == 0, T == 0, T > EVO_FITNESS_MAX_T, P > 65535, warmup > 1000000),
 * EVO_ERR_ALIGN (timings, clock_ratio), EVO_ERR_NOMEM, EVO_ERR_DEVICE, EVO_ERR_CAPTURE
 * (the stream is capturing).
 */
typedef void (*evo_launch_fn)(void *user, void *stream);
typedef struct evo_timing_opts {
    uint32_t warmup;      /* untimed runs per candidate before the timed ones          */
    uint32_t flush_cache; /* 0 / 1                                                     */
    uint32_t reserved[2]; /* set to 0                                                  */
} evo_timing_opts;
EVO_API int evo_time_candidates(evo_check_t *c, const evo_launch_fn *launch, void *const *user,
                                uint32_t P, uint32_t T, const evo_timing_opts *opts,
                                void *stream, float *timings, float *clock_ratio);

/*
 * Destroys a context: waits for the device to go idle, checks the guard bytes behind the
 * scratch buffers its kernels wrote (EVO_ERR_INTERNAL if one was overwritten; the context is
 * destroyed all the same) and frees the library's scratch memory.  NULL, unknown and
 * already destroyed handles are ignored (evo_check_destroy returns EVO_ERR_HANDLE for them
 * and does nothing else).
 */
EVO_API int evo_check_destroy(evo_check_t *c);

/* Static, never NULL description of a status code. */
EVO_API const char *evo_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* EVO_H_ */
