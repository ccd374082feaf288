// Internal layout shared by the host side of the C ABI and the gfx950 kernels.
// Nothing here is visible to callers of evo.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "evo.h"

namespace evo {

// Compile-time tunables (defaults are the measured best on MI355X).
#ifndef EVO_KG
#define EVO_KG 16            // candidates per wavefront group (max): 8 or 16
#endif
#ifndef EVO_DEPTH
#define EVO_DEPTH 2          // candidates whose tile loads a wavefront keeps in flight
#endif
#ifndef EVO_WAVES_PER_EU
#define EVO_WAVES_PER_EU 2   // occupancy the register allocator must allow
#endif
#ifndef EVO_NV_F32
#define EVO_NV_F32 2         // 16-byte vectors per lane per tile, fp32 tensors
#endif
#ifndef EVO_NV_BF16
#define EVO_NV_BF16 2        // 16-byte vectors per lane per tile, bf16 tensors
#endif
#ifndef EVO_NT_LOADS
#define EVO_NT_LOADS 1       // non-temporal loads for data that is read once
#endif
#ifndef EVO_ROTATE
#define EVO_ROTATE 61        // per-step rotation of the workgroup -> tile map (0 = fixed map)
#endif
#ifndef EVO_JOBS_PER_CU
#define EVO_JOBS_PER_CU 2    // workgroups the partitioner creates per compute unit
#endif
#ifndef EVO_XCD_BLOCKS
#define EVO_XCD_BLOCKS 1     // 1: the chunks of one XCD are neighbours in the window, 0: dealt round-robin
#endif
#ifndef EVO_GPW_MAX
#define EVO_GPW_MAX 4        // most candidate groups one workgroup takes side by side (1, 2 or 4)
#endif

// Launch geometry of the check kernel.  A workgroup is 4 wavefronts of 64 lanes.
// Each wavefront owns one group of candidates (a power of two, at most kG) and
// keeps that group's running statistics in registers for the whole job; the
// wavefronts of a workgroup either share a reference tile (different candidate
// groups) or take different tiles (same group).  With more than four groups the
// workgroups that take the same tiles for different groups have numbers that are
// congruent modulo 8 whenever the chunk count is a multiple of 8, i.e. they run on one
// XCD and meet the reference tile in one L2.
constexpr int kLanes = 64;
constexpr int kWaves = 4;
constexpr int kThreads = kLanes * kWaves;
constexpr int kG = EVO_KG;
constexpr int kRowsPerJob = kWaves * kG;   // partial rows one job can produce
constexpr uint32_t kMaxTilesPerWave = 2048; // per job: bounds the LDS redo list

// Bytes of one element, and elements one wavefront consumes per tile and per tensor (a tile
// is EVO_NV_* 16-byte vectors per lane: 2 KiB of every tensor with the default of 2).
__host__ __device__ constexpr uint32_t elem_bytes(uint32_t dtype) {
    return (dtype == EVO_BF16 || dtype == EVO_F16) ? 2u
         : (dtype == EVO_F64 || dtype == EVO_I64) ? 8u : 4u;
}
__host__ __device__ constexpr uint32_t tile_elems(uint32_t dtype) {
    return ((dtype == EVO_BF16 || dtype == EVO_F16) ? EVO_NV_BF16 : EVO_NV_F32) * 64u * 16u /
           elem_bytes(dtype);
}

// A population of P candidates is cut into groups whose sizes are powers of two:
// P / kG groups of kG, then one group per set bit of P % kG, largest first
// (P = 21, kG = 16: 16 + 4 + 1).  A wavefront then always works on a full group.
struct Group {
    uint32_t cand0;   // first candidate of the group
    uint32_t nc;      // its size: 1, 2, 4, ... kG
};

__host__ __device__ inline uint32_t group_count(uint32_t P) {
    uint32_t n = P / kG;
    for (uint32_t rem = P % kG; rem; rem &= rem - 1) ++n;
    return n;
}

__host__ __device__ inline Group group_of(uint32_t P, uint32_t g) {
    const uint32_t nfull = P / kG;
    if (g < nfull) return Group{g * kG, (uint32_t)kG};
    const uint32_t rem = P % kG;
    uint32_t base = nfull * kG, k = g - nfull;
    for (uint32_t b = kG >> 1; b; b >>= 1) {
        if (rem & b) {
            if (k == 0) return Group{base, b};
            base += b;
            --k;
        }
    }
    return Group{base, 0u};   // g >= group_count(P)
}

// Inverse: the group that holds candidate p and p's index inside it.
__host__ __device__ inline void locate(uint32_t P, uint32_t p, uint32_t *group, uint32_t *gi) {
    const uint32_t nfull = P / kG;
    if (p < nfull * kG) {
        *group = p / kG;
        *gi = p % kG;
        return;
    }
    const uint32_t rem = P % kG;
    uint32_t off = p - nfull * kG, k = nfull;
    for (uint32_t b = kG >> 1; b; b >>= 1) {
        if (rem & b) {
            if (off < b) break;
            off -= b;
            ++k;
        }
    }
    *group = k;
    *gi = off;
}

// How the jobs' partial rows become evo_stats rows.
//   kFoldLevels       per segment, by one or two levels of tickets; the cases of a case group
//                     are then merged behind a ticket of their own
//   kFoldCasesDirect  a small case group: every job of every case draws the group's ticket and
//                     the last one adds all rows, case by case, and merges the cases -- one
//                     ticket round trip and one fold less behind the last job
constexpr uint8_t kFoldLevels = 0, kFoldCasesDirect = 1;
constexpr uint32_t kDirectMaxCases = 8;      // most cases of a group folded directly
constexpr uint32_t kDirectRowsPerThread = 8; // most job rows one thread adds in that fold

// One ragged group as the kernel sees it (device memory, 64 bytes).
struct SegDesc {
    const void *ref;
    uint64_t n;                 // elements per tensor
    uint32_t ptr0;              // index of the segment's first candidate pointer in the table
    uint32_t P;                 // candidates the kernel walks: the caller's plus n_pad
    uint32_t stats_row0;
    uint32_t job0;              // first workgroup index of this segment
    uint32_t n_jobs;            // n_gblocks * n_chunks
    uint32_t n_chunks;          // workgroups that share the tiles of one group block
    uint32_t case0;             // first segment of the case group this segment belongs to
    uint32_t n_groups;          // candidate groups
    uint32_t n_cases;           // segments in that case group (1: the segment stands alone)
    float atol, rtol;           // the tolerance this segment is checked with
    uint8_t dtype;
    uint8_t fold_mode;          // kFoldLevels or kFoldCasesDirect (the same for all cases of a group)
    uint8_t gpw;                // groups per workgroup: 1, 2 or 4
    uint8_t n_pad;              // trailing candidates that are stand-ins (their pointer is the
                                // reference's); they get no evo_stats row
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

// Small launches carry their descriptors and candidate pointers in the kernel
// argument block itself (no staging copy precedes the kernel); larger ones read them
// from a device table.
constexpr uint32_t kInlineSegs = 8;
constexpr uint32_t kInlinePtrs = 384;
struct InlineTable {
    SegDesc descs[kInlineSegs];
    uint64_t ptrs[kInlinePtrs];
};
static_assert(sizeof(InlineTable) <= 3600, "kernel argument block must stay below 4 KiB");   // + other arguments

// Scratch layout of one launch (J = workgroups, S = segments, C = candidate pointers):
//   partials: J*kRowsPerJob first-level rows | J*kRowsPerJob second-level rows | C case rows
//   tickets:  J bundle tickets | S segment tickets | S case-group tickets
// dtype_set: OR of (1 << evo_dtype) over the segments of the launch.
// n_first: compute units of the device (workgroups numbered below it get a compute unit
// of their own when the launch starts).
hipError_t launch_check(uint32_t dtype_set, const SegDesc *d_descs, const uint64_t *d_ptrs,
                        uint32_t S, uint32_t total_jobs, uint32_t n_first,
                        Partial *partials, uint32_t *tickets, evo_stats *stats, hipStream_t stream);

hipError_t launch_check_inline(uint32_t dtype_set, const InlineTable &tab, uint32_t S,
                               uint32_t total_jobs, uint32_t n_first,
                               Partial *partials, uint32_t *tickets, evo_stats *stats,
                               hipStream_t stream);

// The check and the timing reduction in one launch (small launches only: the table travels
// in the kernel argument block; exactly one segment or one case group).
struct FitLaunch {
    const float *timings;
    const float *baseline;
    evo_pop_summary *summary;
    float *base;          // two floats of device scratch
    float *rows;          // 2 * P floats of device scratch
    uint32_t *ticket;     // device, zero between launches
    uint32_t P, T, reducer;
    uint32_t writers;     // workgroups that write evo_stats rows (one per segment or case group)
};
hipError_t launch_evaluate(uint32_t dtype_set, const InlineTable &tab, uint32_t S, uint32_t total_jobs,
                           uint32_t n_first, Partial *partials,
                           uint32_t *tickets, evo_stats *stats, const FitLaunch &fit,
                           hipStream_t stream);

// The same two launchers of one instantiation (DTS = its element-type set); each set is
// compiled in a translation unit of its own.
constexpr uint32_t kAllTypes = (1u << EVO_F32) | (1u << EVO_BF16) | (1u << EVO_F16) |
                               (1u << EVO_F64) | (1u << EVO_I32) | (1u << EVO_I64);
template <uint32_t DTS>
hipError_t launch_check_for(const SegDesc *d_descs, const uint64_t *d_ptrs, uint32_t S,
                            uint32_t total_jobs, uint32_t n_first,
                            Partial *partials, uint32_t *tickets, evo_stats *stats,
                            hipStream_t stream);
template <uint32_t DTS>
hipError_t launch_check_inline_for(const InlineTable &tab, uint32_t S, uint32_t total_jobs,
                                   uint32_t n_first, Partial *partials,
                                   uint32_t *tickets, evo_stats *stats, hipStream_t stream);
template <uint32_t DTS>
hipError_t launch_evaluate_for(const InlineTable &tab, uint32_t S, uint32_t total_jobs,
                               uint32_t n_first, Partial *partials, uint32_t *tickets,
                               evo_stats *stats, const FitLaunch &fit, hipStream_t stream);

// base_median: two floats of device scratch (the baseline's median and mean).
hipError_t launch_fitness(const float *timings, const float *baseline, uint32_t P, uint32_t T,
                          uint32_t reducer, evo_stats *stats, evo_pop_summary *summary,
                          float *base_median, uint32_t *ticket, hipStream_t stream);

hipError_t launch_select(const evo_stats *stats, uint32_t P, uint32_t k, uint32_t *elite,
                         uint32_t *n_elite, hipStream_t stream);

// The same with one key per candidate and no two selected candidates sharing a key.
// rep: P words of device scratch.
hipError_t launch_select_diverse(const evo_stats *stats, const uint32_t *keys, uint32_t *rep, uint32_t P,
                                 uint32_t k, uint32_t *elite, uint32_t *n_elite, hipStream_t stream);

// Timing stage helpers: overwrite `bytes` of `buf` (a multiple of 4) with `value`; run a
// fixed chain of `iterations` dependent FMAs in one wavefront (sink: 4 bytes of scratch).
hipError_t launch_flush(void *buf, size_t bytes, uint32_t value, hipStream_t stream);
hipError_t launch_probe(float *sink, uint32_t iterations, hipStream_t stream);

}  // namespace evo
