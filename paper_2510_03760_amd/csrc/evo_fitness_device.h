// Device code of the timing reduction (median / mean per row, then speedup, fitness and the
// population figures), shared by the stand-alone fitness kernel and by the check kernel that
// carries the reduction in the same launch.  What is computed: see evo_fitness_kernel.hip
// and evo.h (evo_fitness).
#pragma once

#include "evo_internal.h"

namespace evo {
namespace {

constexpr uint32_t kQuietNan = 0x7fc00000u;
constexpr float kInfF = __builtin_huge_valf();

struct Best {
    float fitness;
    uint32_t idx;
    uint32_t n_valid;
};

__device__ __forceinline__ bool better(float fa, uint32_t ia, float fb, uint32_t ib) {
    return fa > fb || (fa == fb && ia < ib);
}

// Median and mean of the T samples at src, by one whole workgroup; the results are valid in
// thread 0.  The row is sorted in LDS by a bitonic network (padded with +Inf to a power of
// two); the mean is the binary64 sum in sample order -- taken by a tree when that is exact.
__device__ __forceinline__ void fitness_row(const float *__restrict__ src, uint32_t T, float &median,
                                            float &mean) {
    __shared__ float sorted[EVO_FITNESS_MAX_T];
    __shared__ double psum[kThreads];
    const uint32_t tid = threadIdx.x;

    uint32_t Tpad = 2;
    while (Tpad < T) Tpad <<= 1;

    // Row into LDS (+Inf padding); per-thread binary64 sum of its own samples; usable
    // iff every sample is finite and > 0.
    double mysum = 0.0;
    int bad = 0;
    for (uint32_t i = tid; i < Tpad; i += kThreads) {
        float x = kInfF;
        if (i < T) {
            x = src[i];
            mysum += (double)x;
            if (!(x > 0.0f) || x == kInfF) bad = 1;
        }
        sorted[i] = x;
    }
    psum[tid] = mysum;
    const int row_bad = __syncthreads_or(bad);

    // Bitonic sort, ascending.
    for (uint32_t k = 2; k <= Tpad; k <<= 1) {
        for (uint32_t j = k >> 1; j > 0; j >>= 1) {
            for (uint32_t i = tid; i < (Tpad >> 1); i += kThreads) {
                const uint32_t a = ((i & ~(j - 1)) << 1) | (i & (j - 1));
                const uint32_t b = a | j;
                const bool up = (a & k) == 0;
                const float x = sorted[a], y = sorted[b];
                if ((x > y) == up) {
                    sorted[a] = y;
                    sorted[b] = x;
                }
            }
            __syncthreads();
        }
    }

    // Tree sum of the per-thread sums (used only when it is exact, see evo_fitness_kernel.hip).
    for (uint32_t stride = kThreads / 2; stride >= 1; stride >>= 1) {
        if (tid < stride) psum[tid] += psum[tid + stride];
        __syncthreads();
    }

    if (tid == 0) {
        if (row_bad) {
            median = __builtin_bit_cast(float, kQuietNan);
            mean = median;
        } else {
            const float hi = sorted[T / 2];
            if (T & 1u) {
                median = hi;
            } else {
                const float s = sorted[T / 2 - 1] + hi;
                median = 0.5f * s;
            }
            double sum = psum[0];
            if (!(sorted[T - 1] < sorted[0] * 65536.0f)) {
                sum = 0.0;   // wide dynamic range: the defining order
                for (uint32_t i = 0; i < T; ++i) sum += (double)src[i];
            }
            mean = (float)(sum / (double)T);
        }
    }
    __syncthreads();   // the LDS arrays may be reused by the caller's next step
}

// Speedups, fitness and the population figures, by one whole workgroup, once every row's
// median and mean and every valid flag are in place (and visible: the caller has acquired).
// base: the baseline's median and mean.  rows: nullptr when the medians and means are already
// in the evo_stats rows, else P (median, mean) pairs that are copied there as well (the rows
// may have been rewritten since the pairs were computed).
__device__ __forceinline__ void fitness_finish(uint32_t P, uint32_t reducer, evo_stats *__restrict__ stats,
                                               evo_pop_summary *__restrict__ summary,
                                               const float *__restrict__ base,
                                               const float *__restrict__ rows) {
    __shared__ Best best_lds[kThreads];
    const uint32_t tid = threadIdx.x;
    // Numerator and denominator of the speedup: medians, or means when the caller asked for
    // the "average over the runs" of Sec. 4.3.  (A row is unusable for both or for neither.)
    const bool by_mean = reducer == EVO_REDUCE_MEAN;
    const float bm = __hip_atomic_load(base + (by_mean ? 1 : 0), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool base_ok = bm == bm;
    Best mine{0.0f, P, 0u};
    for (uint32_t p = tid; p < P; p += kThreads) {
        const float *pair = rows ? rows + 2 * (uint64_t)p : &stats[p].median_ms;   // adjacent fields
        const float row_median = __hip_atomic_load(pair, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float row_mean = __hip_atomic_load(pair + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (rows) {
            stats[p].median_ms = row_median;
            stats[p].mean_ms = row_mean;
        }
        const float med = by_mean ? row_mean : row_median;
        const uint32_t valid = __hip_atomic_load(&stats[p].valid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        float speedup = 0.0f;
        if (base_ok && med == med) speedup = bm / med;
        const float fit = valid ? speedup : 0.0f;
        stats[p].speedup = speedup;
        stats[p].fitness = fit;
        if (valid) mine.n_valid += 1;
        if (fit > mine.fitness) {            // ascending p: the first maximum is kept
            mine.fitness = fit;
            mine.idx = p;
        }
    }
    best_lds[tid] = mine;
    __syncthreads();
    for (uint32_t stride = kThreads / 2; stride >= 1; stride >>= 1) {
        if (tid < stride) {
            Best a = best_lds[tid];
            const Best b = best_lds[tid + stride];
            if (better(b.fitness, b.idx, a.fitness, a.idx)) {
                a.fitness = b.fitness;
                a.idx = b.idx;
            }
            a.n_valid += b.n_valid;
            best_lds[tid] = a;
        }
        __syncthreads();
    }
    if (tid == 0 && summary) {
        const Best b = best_lds[0];
        evo_pop_summary out;
        out.best_idx = b.fitness > 0.0f ? b.idx : P;
        out.n_valid = b.n_valid;
        out.best_speedup = b.fitness > 1.0f ? b.fitness : 1.0f;
        out.valid_rate = (float)b.n_valid / (float)P;
        *summary = out;
    }
}

// One timing row (row < P) or the baseline (row == P): reduce it, publish (median, mean) --
// in rows[2*row ..] when rows is given, else in the row's evo_stats record -- and take a
// ticket.  Returns true in every thread of the workgroup that drew ticket number `last`.
__device__ __forceinline__ bool fitness_row_and_ticket(const float *__restrict__ timings,
                                                       const float *__restrict__ baseline, uint32_t row,
                                                       uint32_t P, uint32_t T, evo_stats *__restrict__ stats,
                                                       float *__restrict__ rows,
                                                       float *__restrict__ base, uint32_t *__restrict__ ticket,
                                                       uint32_t last) {
    __shared__ uint32_t drew_last;
    float median = 0.0f, mean = 0.0f;
    fitness_row(row < P ? timings + (uint64_t)row * T : baseline, T, median, mean);
    if (threadIdx.x == 0) {
        if (row < P) {
            float *pair = rows ? rows + 2 * (uint64_t)row : &stats[row].median_ms;
            pair[0] = median;
            pair[1] = mean;
        } else {
            base[0] = median;
            base[1] = mean;
        }
        // the release of the ticket publishes the two stores above
        const uint32_t prev = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        drew_last = (prev == last) ? 1u : 0u;
    }
    __syncthreads();   // thread 0 acquired with the ticket; the barrier hands that on
    return drew_last != 0;
}

}  // namespace
}  // namespace evo
