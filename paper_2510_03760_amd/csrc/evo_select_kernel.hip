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
//
// Diversity maintenance (the third strategy of Sec. 3.2.2): with one caller-defined key per
// candidate, no two selected candidates may share a key.  A first kernel marks the
// representative of every key (its best feasible candidate, lowest index on ties); the
// second is the rank counting above restricted to representatives.

#include "evo_internal.h"

namespace evo {
namespace {

__device__ __forceinline__ bool beats(float fj, uint32_t j, float fi, uint32_t i) {
    return fj > fi || (fj == fi && j < i);
}

// rep[i] = 1 iff candidate i is feasible and no candidate with the same key beats it.
__global__ void __launch_bounds__(kThreads)
evo_key_representatives_kernel(const evo_stats *__restrict__ stats, const uint32_t *__restrict__ keys,
                               uint32_t P, uint32_t *__restrict__ rep) {
    __shared__ float stage_f[kThreads];
    __shared__ uint32_t stage_k[kThreads];
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    const float fi = i < P ? stats[i].fitness : 0.0f;
    const uint32_t ki = i < P ? keys[i] : 0u;
    uint32_t beaten = 0;
    for (uint32_t j0 = 0; j0 < P; j0 += kThreads) {
        const uint32_t j = j0 + threadIdx.x;
        __syncthreads();
        stage_f[threadIdx.x] = j < P ? stats[j].fitness : 0.0f;
        stage_k[threadIdx.x] = j < P ? keys[j] : 0u;
        __syncthreads();
        const uint32_t m = min((uint32_t)kThreads, P - j0);
        for (uint32_t t = 0; t < m; ++t)
            beaten |= (stage_k[t] == ki && beats(stage_f[t], j0 + t, fi, i)) ? 1u : 0u;
    }
    if (i < P) rep[i] = (fi > 0.0f && !beaten) ? 1u : 0u;
}

// rep == nullptr: every feasible candidate competes.
template <bool DIVERSE>
__global__ void __launch_bounds__(kThreads)
evo_select_kernel(const evo_stats *__restrict__ stats, const uint32_t *__restrict__ rep, uint32_t P,
                  uint32_t k, uint32_t *__restrict__ elite, uint32_t *__restrict__ n_elite) {
    __shared__ float stage[kThreads];
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    // a candidate that does not compete is given fitness 0, i.e. treated as infeasible
    const float fi = (i < P && (!DIVERSE || rep[i])) ? stats[i].fitness : 0.0f;
    uint32_t rank = 0, count = 0;
    for (uint32_t j0 = 0; j0 < P; j0 += kThreads) {
        const uint32_t j = j0 + threadIdx.x;
        __syncthreads();
        stage[threadIdx.x] = (j < P && (!DIVERSE || rep[j])) ? stats[j].fitness : 0.0f;
        __syncthreads();
        const uint32_t m = min((uint32_t)kThreads, P - j0);
        for (uint32_t t = 0; t < m; ++t) {
            const float fj = stage[t];
            rank += beats(fj, j0 + t, fi, i) ? 1u : 0u;
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
    hipLaunchKernelGGL(evo_select_kernel<false>, dim3((P + kThreads - 1) / kThreads), dim3(kThreads), 0,
                       stream, stats, (const uint32_t *)nullptr, P, k, elite, n_elite);
    return hipGetLastError();
}

hipError_t launch_select_diverse(const evo_stats *stats, const uint32_t *keys, uint32_t *rep, uint32_t P,
                                 uint32_t k, uint32_t *elite, uint32_t *n_elite, hipStream_t stream) {
    const dim3 grid((P + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(evo_key_representatives_kernel, grid, dim3(kThreads), 0, stream, stats, keys, P, rep);
    hipLaunchKernelGGL(evo_select_kernel<true>, grid, dim3(kThreads), 0, stream, stats,
                       (const uint32_t *)rep, P, k, elite, n_elite);
    return hipGetLastError();
}

}  // namespace evo
