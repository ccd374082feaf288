// Helper kernels of the timing stage (evo_time_candidates) for gfx950 (MI355X).
//
// The evaluator of EvoEngineer (arXiv 2510.03760, Sec. 4.3) collects the execution time of
// a candidate over 100 runs; the appendix on threats to validity names run-to-run noise,
// caching effects and clock behaviour as what such timings suffer from.  Two kernels serve
// the host loop that produces the timing table:
//   evo_flush_kernel  overwrites a buffer larger than the last-level cache (256 MiB of
//                     Infinity Cache on MI355X), so that a timed run does not find the
//                     previous run's data there;
//   evo_probe_kernel  a fixed chain of dependent fused multiply-adds in a single wavefront:
//                     its duration is a fixed number of shader clocks, so the ratio of two
//                     timings of it tells whether the clock changed in between.

#include "evo_internal.h"

namespace evo {
namespace {

__global__ void __launch_bounds__(kThreads)
evo_flush_kernel(uint32_t *__restrict__ buf, size_t n_words, uint32_t value) {
    const size_t stride = (size_t)gridDim.x * kThreads;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n_words; i += stride)
        buf[i] = value;
}

__global__ void __launch_bounds__(kLanes)
evo_probe_kernel(float *__restrict__ sink, uint32_t iterations, float seed) {
    float x = seed + (float)threadIdx.x;
    for (uint32_t i = 0; i < iterations; ++i) x = __builtin_fmaf(x, 0.999999f, 1e-7f);   // dependent chain
    if (x == 123456.0f) sink[0] = x;   // never true for the seeds used; keeps the chain alive
}

}  // namespace

hipError_t launch_flush(void *buf, size_t bytes, uint32_t value, hipStream_t stream) {
    const size_t n_words = bytes / sizeof(uint32_t);
    const size_t blocks = (n_words + kThreads - 1) / kThreads;   // small fills: no idle workgroups
    hipLaunchKernelGGL(evo_flush_kernel, dim3((unsigned)(blocks < 1 ? 1 : blocks > 2048 ? 2048 : blocks)),
                       dim3(kThreads), 0, stream, static_cast<uint32_t *>(buf), n_words, value);
    return hipGetLastError();
}

hipError_t launch_probe(float *sink, uint32_t iterations, hipStream_t stream) {
    hipLaunchKernelGGL(evo_probe_kernel, dim3(1), dim3(kLanes), 0, stream, sink, iterations, 0.5f);
    return hipGetLastError();
}

}  // namespace evo
