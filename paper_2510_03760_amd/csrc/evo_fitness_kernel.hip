// Median-timing / speedup / fitness kernel for gfx950 (MI355X).
//
// Performance objective f(p) of EvoEngineer (arXiv 2510.03760, Sec. 3.1, Eq. 1) under
// the metric of Sec. 5.1 ("Evaluation Metric": speedup over the baseline kernel, 1.0
// when nothing beats it, ratio of valid kernels), with repeated timings reduced by
// their median as in the appendix on threats to validity and by their mean as in
// Sec. 4.3.  Exact definitions are in evo.h (evo_fitness).
//
// One launch.  Workgroup p < P reduces timing row p, workgroup P reduces the baseline
// row; each holds its row in LDS and finds the middle order statistics by rank
// counting (the rank of sample i is the number of samples that are smaller, or equal
// with a lower index -- unique per sample, so exactly one sample has each rank; no
// sort, no data-dependent control flow).  The last workgroup to finish turns medians
// into speedups and fitness and reduces the population figures.  The whole input is
// at most a few tens of KiB: this kernel is bound by launch and dependency latency,
// not by bandwidth.

#include "evo_internal.h"

namespace evo {
namespace {

constexpr int kMaxPerThread = EVO_FITNESS_MAX_T / kThreads;   // 16 samples per thread
constexpr uint32_t kQuietNan = 0x7fc00000u;

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
                   uint32_t P, uint32_t T, evo_stats *__restrict__ stats,
                   evo_pop_summary *__restrict__ summary, float *__restrict__ base_median,
                   uint32_t *__restrict__ ticket) {
    __shared__ float samples[EVO_FITNESS_MAX_T];
    __shared__ float mid[2];
    __shared__ uint32_t is_last;
    __shared__ Best best_lds[kThreads];

    const uint32_t row = blockIdx.x;
    const float *src = row < P ? timings + (uint64_t)row * T : baseline;
    const uint32_t tid = threadIdx.x;

    // Row into LDS and into registers; usable iff every sample is finite and > 0.
    float x[kMaxPerThread];
    int bad = 0;
#pragma unroll
    for (int e = 0; e < kMaxPerThread; ++e) {
        const uint32_t i = tid + (uint32_t)e * kThreads;
        x[e] = 0.0f;
        if (i < T) {
            x[e] = src[i];
            samples[i] = x[e];
            if (!(x[e] > 0.0f) || x[e] == __builtin_huge_valf()) bad = 1;
        }
    }
    const int row_bad = __syncthreads_or(bad);

    // Rank counting against every sample, and the row sum in sample order (each
    // thread carries the same sequential fp64 sum; thread 0 reports it).
    const uint32_t per_thread = (T + kThreads - 1) / kThreads;
    uint32_t rank[kMaxPerThread];
#pragma unroll
    for (int e = 0; e < kMaxPerThread; ++e) rank[e] = 0;
    double sum = 0.0;
    for (uint32_t j = 0; j < T; ++j) {
        const float sj = samples[j];
        sum += (double)sj;
#pragma unroll
        for (int e = 0; e < kMaxPerThread; ++e) {
            if ((uint32_t)e < per_thread) {
                const uint32_t i = tid + (uint32_t)e * kThreads;
                rank[e] += (sj < x[e] || (sj == x[e] && j < i)) ? 1u : 0u;
            }
        }
    }
    const uint32_t k_hi = T / 2;                         // middle (odd T) or upper middle
    const uint32_t k_lo = (T & 1u) ? k_hi : k_hi - 1;    // lower middle for even T
#pragma unroll
    for (int e = 0; e < kMaxPerThread; ++e) {
        const uint32_t i = tid + (uint32_t)e * kThreads;
        if (i < T) {
            if (rank[e] == k_hi) mid[1] = x[e];
            if (rank[e] == k_lo) mid[0] = x[e];
        }
    }
    __syncthreads();

    if (tid == 0) {
        float median, mean;
        if (row_bad) {
            median = __builtin_bit_cast(float, kQuietNan);
            mean = median;
        } else {
            if (T & 1u) {
                median = mid[1];
            } else {
                const float s = mid[0] + mid[1];
                median = 0.5f * s;
            }
            mean = (float)(sum / (double)T);
        }
        if (row < P) {
            stats[row].median_ms = median;
            stats[row].mean_ms = mean;
        } else {
            *base_median = median;
        }
    }

    // Ticket: the last of the P+1 workgroups finishes the population.
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_ACQ_REL,
                                                     __HIP_MEMORY_SCOPE_AGENT);
        is_last = (prev == P) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    __threadfence();

    const float bm = __hip_atomic_load(base_median, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool base_ok = bm == bm;
    Best mine{0.0f, P, 0u};
    for (uint32_t p = tid; p < P; p += kThreads) {
        const float med = __hip_atomic_load(&stats[p].median_ms, __ATOMIC_RELAXED,
                                            __HIP_MEMORY_SCOPE_AGENT);
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
                          evo_stats *stats, evo_pop_summary *summary, float *base_median,
                          uint32_t *ticket, hipStream_t stream) {
    hipLaunchKernelGGL(evo_fitness_kernel, dim3(P + 1), dim3(kThreads), 0, stream, timings,
                       baseline, P, T, stats, summary, base_median, ticket);
    return hipGetLastError();
}

}  // namespace evo
