// Elite selection for gfx950 (MI355X): population management of EvoEngineer (arXiv
// 2510.03760, Sec. 3.2.2 -- elite preservation keeps the best solutions; the EoH-style
// baseline in the parameter-settings appendix keeps the best 4 of parents plus
// offspring).  Consumes the fitness column that evo_fitness wrote into the evo_stats rows.
//
// Rank counting: the rank of candidate i is the number of candidates that beat it (larger
// fitness, or equal fitness and lower index).  Ranks are a permutation, feasible
// candidates (fitness > 0) occupy ranks 0 .. count-1, so candidate i simply writes its
// index to slot rank_i when that is below k; slots count .. k-1 are filled with P by the
// threads of the same number.  No sort, no atomics, every slot has exactly one writer.
// One thread per candidate; the fitness column is staged through LDS 256 values at a
// time.  Latency-bound: P*4 bytes of input.

#include "evo_internal.h"

namespace evo {
namespace {

__global__ void __launch_bounds__(kThreads)
evo_select_kernel(const evo_stats *__restrict__ stats, uint32_t P, uint32_t k,
                  uint32_t *__restrict__ elite, uint32_t *__restrict__ n_elite) {
    __shared__ float stage[kThreads];
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    const float fi = i < P ? stats[i].fitness : 0.0f;
    uint32_t rank = 0, count = 0;
    for (uint32_t j0 = 0; j0 < P; j0 += kThreads) {
        const uint32_t j = j0 + threadIdx.x;
        __syncthreads();
        stage[threadIdx.x] = j < P ? stats[j].fitness : 0.0f;
        __syncthreads();
        const uint32_t m = min((uint32_t)kThreads, P - j0);
        for (uint32_t t = 0; t < m; ++t) {
            const float fj = stage[t];
            rank += (fj > fi || (fj == fi && j0 + t < i)) ? 1u : 0u;
            count += fj > 0.0f ? 1u : 0u;
        }
    }
    if (i < P && fi > 0.0f && rank < k) elite[rank] = i;
    if (i < k && i >= count) elite[i] = P;      // k <= P, so thread i exists
    if (i == 0 && n_elite) *n_elite = min(count, k);
}

}  // namespace

hipError_t launch_select(const evo_stats *stats, uint32_t P, uint32_t k, uint32_t *elite,
                         uint32_t *n_elite, hipStream_t stream) {
    hipLaunchKernelGGL(evo_select_kernel, dim3((P + kThreads - 1) / kThreads), dim3(kThreads), 0,
                       stream, stats, P, k, elite, n_elite);
    return hipGetLastError();
}

}  // namespace evo
