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

#include "evo_fitness_device.h"

namespace evo {
namespace {

__global__ void __launch_bounds__(kThreads)
evo_fitness_kernel(const float *__restrict__ timings, const float *__restrict__ baseline,
                   uint32_t P, uint32_t T, uint32_t reducer, evo_stats *__restrict__ stats,
                   evo_pop_summary *__restrict__ summary, float *__restrict__ base_median,
                   uint32_t *__restrict__ ticket) {
    // the last of the P+1 workgroups to finish its row does the rest
    if (!fitness_row_and_ticket(timings, baseline, blockIdx.x, P, T, stats, nullptr, base_median, ticket, P)) return;
    fitness_finish(P, reducer, stats, summary, base_median, nullptr);
    if (threadIdx.x == 0) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
