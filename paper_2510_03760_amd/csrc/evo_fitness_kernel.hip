// Median-timing / speedup / fitness kernel for gfx950 (MI355X).
//
// Performance objective f(p) of EvoEngineer (arXiv 2510.03760, Sec. 3.1, Eq. 1) under
// the metric of Sec. 5.1 ("Evaluation Metric": speedup over the baseline kernel, 1.0
// when nothing beats it, ratio of valid kernels), with repeated timings reduced by
// their median as in the appendix on threats to validity and by their mean as in
// Sec. 4.3.  Exact definitions are in evo.h (evo_fitness).
//
// One launch.  Workgroup p < P reduces timing row p, workgroup P reduces the baseline
// row: the row is sorted in LDS by a bitonic network (padded with +Inf to a power of
// two; O(T log^2 T) compare-exchanges, no data-dependent control flow) and the middle
// order statistics are read off.  The last workgroup to finish turns medians into
// speedups and fitness and reduces the population figures.  The whole input is at
// most a few tens of KiB: this kernel is bound by launch and dependency latency, not
// by bandwidth.
//
// The mean is defined as the binary64 sum of the samples IN SAMPLE ORDER.  When the
// largest sample is below 2^16 times the smallest, every partial sum of at most 4096
// binary32 values is exactly representable in binary64 (24 + 12 + 17 = 53 bits), so
// the sum does not depend on the order and is taken by a parallel tree; otherwise one
// thread adds the row sequentially.

#include "evo_internal.h"

namespace evo {
namespace {

constexpr uint32_t kQuietNan = 0x7fc00000u;
constexpr float kInf = __builtin_huge_valf();

struct Best {
    float fitness;
    uint32_t idx;
    uint32_t n_valid;
};

__device__ __forceinline__ bool better(float fa, uint32_t ia, float fb, uint32_t ib) {
    return fa > fb || (fa == fb && ia < ib);
}

__global__ void __launch_bounds__(kThreads)
evo_fitness_kernel(const float *__restrict__ timings, const float *__restrict__ baseline,
                   uint32_t P, uint32_t T, uint32_t reducer, evo_stats *__restrict__ stats,
                   evo_pop_summary *__restrict__ summary, float *__restrict__ base_median,
                   uint32_t *__restrict__ ticket) {
    __shared__ float sorted[EVO_FITNESS_MAX_T];
    __shared__ double psum[kThreads];
    __shared__ uint32_t is_last;
    __shared__ Best best_lds[kThreads];

    const uint32_t row = blockIdx.x;
    const float *src = row < P ? timings + (uint64_t)row * T : baseline;
    const uint32_t tid = threadIdx.x;

    uint32_t Tpad = 2;
    while (Tpad < T) Tpad <<= 1;

    // Row into LDS (+Inf padding); per-thread binary64 sum of its own samples; usable
    // iff every sample is finite and > 0.
    double mysum = 0.0;
    int bad = 0;
    for (uint32_t i = tid; i < Tpad; i += kThreads) {
        float x = kInf;
        if (i < T) {
            x = src[i];
            mysum += (double)x;
            if (!(x > 0.0f) || x == kInf) bad = 1;
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

    // Tree sum of the per-thread sums (used only when it is exact, see the header).
    for (uint32_t stride = kThreads / 2; stride >= 1; stride >>= 1) {
        if (tid < stride) psum[tid] += psum[tid + stride];
        __syncthreads();
    }

    if (tid == 0) {
        float median, mean;
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
        if (row < P) {
            stats[row].median_ms = median;
            stats[row].mean_ms = mean;
        } else {
            base_median[0] = median;
            base_median[1] = mean;
        }
        // the release of the ticket publishes the two stores above
        const uint32_t prev = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        is_last = (prev == P) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;   // thread 0 acquired with the last ticket; the barrier hands that on

    // The last of the P+1 workgroups: speedups, fitness, population figures.
    // Numerator and denominator of the speedup: medians, or means when the caller asked for
    // the "average over the runs" of Sec. 4.3.  (A row is unusable for both or for neither.)
    const bool by_mean = reducer == EVO_REDUCE_MEAN;
    const float bm = __hip_atomic_load(base_median + (by_mean ? 1 : 0), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
    const bool base_ok = bm == bm;
    Best mine{0.0f, P, 0u};
    for (uint32_t p = tid; p < P; p += kThreads) {
        const float med = __hip_atomic_load(by_mean ? &stats[p].mean_ms : &stats[p].median_ms,
                                            __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t valid = stats[p].valid;
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
    if (tid == 0) {
        const Best b = best_lds[0];
        if (summary) {
            evo_pop_summary out;
            out.best_idx = b.fitness > 0.0f ? b.idx : P;
            out.n_valid = b.n_valid;
            out.best_speedup = b.fitness > 1.0f ? b.fitness : 1.0f;
            out.valid_rate = (float)b.n_valid / (float)P;
            *summary = out;
        }
        __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

}  // namespace

hipError_t launch_fitness(const float *timings, const float *baseline, uint32_t P, uint32_t T,
                          uint32_t reducer, evo_stats *stats, evo_pop_summary *summary,
                          float *base_median, uint32_t *ticket, hipStream_t stream) {
    hipLaunchKernelGGL(evo_fitness_kernel, dim3(P + 1), dim3(kThreads), 0, stream, timings,
                       baseline, P, T, reducer, stats, summary, base_median, ticket);
    return hipGetLastError();
}

}  // namespace evo
