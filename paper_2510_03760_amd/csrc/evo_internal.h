// Internal layout shared by the host side of the C ABI and the gfx950 kernels.
// Nothing here is visible to callers of evo.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "evo.h"

namespace evo {

// Launch geometry of the check kernel.  A workgroup is 4 wavefronts of 64 lanes.
// Each wavefront owns one group of at most kG candidates and keeps that group's
// running statistics in registers for the whole job; the wavefronts of a
// workgroup either share a reference tile (different candidate groups) or take
// different tiles (same group), so that a reference tile never has to be fetched
// by more than one workgroup -- i.e. by more than one XCD's L2.
constexpr int kLanes = 64;
constexpr int kWaves = 4;
constexpr int kThreads = kLanes * kWaves;
constexpr int kG = 16;                     // candidates per wavefront group (max)
constexpr int kRowsPerJob = kWaves * kG;   // partial rows one job can produce

// Elements one wavefront consumes per tile and per tensor: 2 x 16 bytes per lane.
constexpr uint32_t kTileBytes = 2048;
__host__ __device__ constexpr uint32_t tile_elems(uint32_t dtype) {
    return dtype == EVO_BF16 ? kTileBytes / 2 : kTileBytes / 4;
}

// One ragged group as the kernel sees it (device memory, 64 bytes).
struct SegDesc {
    const void *ref;
    const void *const *cands;   // device array of P pointers
    uint64_t n;                 // elements per tensor
    uint32_t P;
    uint32_t dtype;
    uint32_t stats_row0;
    uint32_t job0;              // first workgroup index of this group
    uint32_t n_jobs;            // n_gblocks * n_chunks
    uint32_t n_chunks;          // tile chunks per candidate-group block
    uint32_t tiles_per_chunk;
    uint32_t n_groups;          // candidate groups
    uint32_t cpg;               // candidates per group (<= kG)
    uint32_t gpw;               // groups per workgroup: 1, 2 or 4
};
static_assert(sizeof(SegDesc) == 64, "SegDesc layout");

// What one job contributes to one candidate (device scratch, 48 bytes).
struct Partial {
    uint64_t n_mismatch;
    uint64_t n_excluded;        // elements with a non-finite side
    double sum_abs;
    double sum_rel;
    float max_abs;
    float max_rel;
    uint32_t flags;
    uint32_t pad;
};
static_assert(sizeof(Partial) == 48, "Partial layout");

hipError_t launch_check(const SegDesc *d_descs, uint32_t S, uint32_t total_jobs, float atol,
                        float rtol, Partial *partials, uint32_t *tickets, evo_stats *stats,
                        hipStream_t stream);

hipError_t launch_fitness(const float *timings, const float *baseline, uint32_t P, uint32_t T,
                          evo_stats *stats, evo_pop_summary *summary, float *base_median,
                          uint32_t *ticket, hipStream_t stream);

}  // namespace evo
