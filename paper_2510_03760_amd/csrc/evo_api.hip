// Host side of the C ABI declared in evo.h: argument validation, job partitioning,
// descriptor staging and launches.  Everything that is computed about tensors is
// computed by the kernels; nothing here touches tensor data.

#include <algorithm>
#include <cmath>
#include <cstring>
#include <mutex>
#include <new>
#include <set>
#include <utility>
#include <vector>

#include "evo_internal.h"

namespace {

using evo::Partial;
using evo::SegDesc;

constexpr uint32_t kJobsPerCu = EVO_JOBS_PER_CU;
#ifndef EVO_MIN_JOB_COST
#define EVO_MIN_JOB_COST 128   // tile loads a job should at least take ...
#endif
#ifndef EVO_MIN_JOBS
#define EVO_MIN_JOBS 256       // ... while this many jobs remain (128: slower at 2^21 x 16)
#endif
constexpr uint32_t kMinTilesPerWave = 4;
constexpr uint32_t kMaxP = 65535;
constexpr int kStageSlots = 8;
// Every scratch buffer the kernels write ends in a guard of this many bytes holding
// kGuardByte; evo_check_destroy checks that they still do.
constexpr size_t kGuardBytes = 256;
constexpr int kGuardByte = 0xC5;
constexpr size_t kFlushBytes = 512u << 20;      // twice the last-level cache of MI355X
constexpr uint32_t kProbeIterations = 20000;    // about 35 us at 2.4 GHz
constexpr int kProbeSpinUp = 100;

struct StageSlot {
    void *host = nullptr;      // pinned
    size_t bytes = 0;
    hipEvent_t done = nullptr; // recorded after the copy that reads `host`
    bool in_flight = false;
};

}  // namespace

// Scratch of evo_check_batch_static, the one call that allocates nothing: partial rows of
// at most kStaticMaxJobs jobs and of kInlinePtrs case rows, then the tickets.  Every device
// the library's code is loaded on holds its own copy until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress: kernels, copies and fills get
// the address that call returns for the current device (static_scratch()).
constexpr uint32_t kStaticMaxJobs = 1024;
constexpr size_t kStaticPartialRows = 2 * (size_t)kStaticMaxJobs * evo::kRowsPerJob + evo::kInlinePtrs;
constexpr size_t kStaticTicketWords = kStaticMaxJobs + 2 * evo::kInlineSegs;
constexpr size_t kStaticPartialBytes = kStaticPartialRows * sizeof(evo::Partial);
constexpr size_t kStaticScratchBytes = kStaticPartialBytes + kStaticTicketWords * sizeof(uint32_t);
static_assert(kStaticPartialBytes % 256 == 0, "the tickets start on a 256-byte boundary");
static_assert(kStaticMaxJobs == EVO_STATIC_MAX_JOBS && kStaticScratchBytes == EVO_STATIC_SCRATCH_BYTES,
              "evo.h states the capacity");
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr uint32_t kDtypes = 6;              // EVO_F32 .. EVO_I64
constexpr uint32_t kTolClasses = EVO_TOL_CLASSES;

struct Tolerance {
    float atol = 0.0f, rtol = 0.0f;
    bool set = false;
};

struct evo_check {
    evo_dtype dtype;
    uint64_t n_elems;
    Tolerance by_dtype[kDtypes];            // all start as the pair given to evo_check_create
    Tolerance by_class[kTolClasses + 1];    // [1 .. kTolClasses], set by the caller
    int device = -1;             // device the scratch lives on (-1: none yet)
    uint32_t n_cus = 0;          // compute units of that device
    // device scratch
    void *d_table = nullptr;     // SegDesc[S] followed by the candidate pointer table
    size_t table_bytes = 0;
    Partial *d_partials = nullptr;
    size_t partial_rows = 0;
    uint32_t *d_tickets = nullptr;   // per segment, self re-arming, + fitness ticket
    size_t n_tickets = 0;
    float *d_base_median = nullptr;
    uint32_t *d_fit_ticket = nullptr;
    float *d_fit_rows = nullptr;     // (median, mean) pairs of evo_evaluate
    size_t fit_rows_count = 0;
    uint32_t *d_rep = nullptr;       // key representatives of evo_select_elite_diverse
    size_t rep_count = 0;
    StageSlot slots[kStageSlots];
    int next_slot = 0;
    // timing stage (evo_time_candidates)
    std::vector<hipEvent_t> time_events;   // start/stop pairs, reused from candidate to candidate
    void *d_flush = nullptr;               // kFlushBytes of scratch
    float *h_times = nullptr;              // pinned staging of the timing table
    size_t h_times_count = 0;
    float *d_probe_sink = nullptr;
};

namespace {

std::mutex g_mu;
std::set<evo_check *> g_live;

// Device address of `scratch` on each device, looked up once per device.
constexpr int kMaxDevices = 64;
void *g_static_ptr[kMaxDevices];   // guarded by g_mu

int static_scratch(int device, unsigned char **out) {
    if (device < 0 || device >= kMaxDevices) return EVO_ERR_DEVICE;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_static_ptr[device]) {
        // `device` is the current device (bind_device): the address is this device's copy
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return EVO_ERR_DEVICE;
        g_static_ptr[device] = p;
    }
    *out = static_cast<unsigned char *>(g_static_ptr[device]);
    return EVO_OK;
}

bool is_live(evo_check *c) {
    std::lock_guard<std::mutex> lk(g_mu);
    return c != nullptr && g_live.count(c) != 0;
}

uint32_t elem_size(uint32_t dtype) { return evo::elem_bytes(dtype); }

bool dtype_ok(uint32_t dtype) { return dtype <= EVO_I64; }

int dev(hipError_t e) { return e == hipSuccess ? EVO_OK : (e == hipErrorOutOfMemory ? EVO_ERR_NOMEM : EVO_ERR_DEVICE); }

#define EVO_TRY(expr)                       \
    do {                                    \
        const int rc_ = dev(expr);          \
        if (rc_ != EVO_OK) return rc_;      \
    } while (0)

// True while `stream` records into a graph: nothing may be allocated, freed, cleared with a
// memset or copied from staging memory then (a replay would not repeat it).
bool capturing(hipStream_t stream) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    return st != hipStreamCaptureStatusNone;
}

// Scratch is tied to the device that is current when it is first needed.
int bind_device(evo_check *c) {
    int cur = -1;
    EVO_TRY(hipGetDevice(&cur));
    if (c->device == -1) c->device = cur;
    return c->device == cur ? EVO_OK : EVO_ERR_DEVICE;
}

// Scratch grows on demand.  Growing frees and allocates device memory and clears new
// counters, none of which may happen while `stream` records into a graph: then the call is
// refused (EVO_ERR_CAPTURE) before anything has been touched.  New counters are cleared and
// the clearing has completed before the call goes on, so that a later call on another stream
// is ordered after it.
int ensure_table(evo_check *c, size_t bytes, hipStream_t stream) {
    if (bytes <= c->table_bytes) return EVO_OK;
    if (capturing(stream)) return EVO_ERR_CAPTURE;
    if (c->d_table) EVO_TRY(hipFree(c->d_table));   // hipFree waits for the device
    c->d_table = nullptr;
    c->table_bytes = 0;
    const size_t cap = std::max<size_t>(bytes * 2, 4096);
    EVO_TRY(hipMalloc(&c->d_table, cap));
    c->table_bytes = cap;
    return EVO_OK;
}

int ensure_partials(evo_check *c, size_t rows, hipStream_t stream) {
    if (rows <= c->partial_rows) return EVO_OK;
    if (capturing(stream)) return EVO_ERR_CAPTURE;
    if (c->d_partials) EVO_TRY(hipFree(c->d_partials));
    c->d_partials = nullptr;
    c->partial_rows = 0;
    EVO_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_partials), rows * sizeof(Partial) + kGuardBytes));
    EVO_TRY(hipMemsetAsync(reinterpret_cast<char *>(c->d_partials) + rows * sizeof(Partial), kGuardByte,
                           kGuardBytes, stream));
    EVO_TRY(hipStreamSynchronize(stream));
    c->partial_rows = rows;
    return EVO_OK;
}

int ensure_tickets(evo_check *c, size_t n, hipStream_t stream) {
    if (n <= c->n_tickets) return EVO_OK;
    if (capturing(stream)) return EVO_ERR_CAPTURE;
    if (c->d_tickets) EVO_TRY(hipFree(c->d_tickets));
    c->d_tickets = nullptr;
    c->n_tickets = 0;
    const size_t cap = std::max<size_t>(n * 2, 64);
    EVO_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_tickets), cap * sizeof(uint32_t) + kGuardBytes));
    // counters start at zero and every launch leaves them at zero again
    EVO_TRY(hipMemsetAsync(c->d_tickets, 0, cap * sizeof(uint32_t), stream));
    EVO_TRY(hipMemsetAsync(c->d_tickets + cap, kGuardByte, kGuardBytes, stream));
    EVO_TRY(hipStreamSynchronize(stream));
    c->n_tickets = cap;
    return EVO_OK;
}

int ensure_fitness_scratch(evo_check *c, hipStream_t stream) {
    if (c->d_base_median) return EVO_OK;
    if (capturing(stream)) return EVO_ERR_CAPTURE;
    void *p = nullptr;
    EVO_TRY(hipMalloc(&p, 256));
    EVO_TRY(hipMemsetAsync(p, 0, 256, stream));
    EVO_TRY(hipStreamSynchronize(stream));
    c->d_base_median = static_cast<float *>(p);
    c->d_fit_ticket = reinterpret_cast<uint32_t *>(static_cast<char *>(p) + 128);
    return EVO_OK;
}

int ensure_fit_rows(evo_check *c, size_t P, hipStream_t stream) {
    if (P <= c->fit_rows_count) return EVO_OK;
    if (capturing(stream)) return EVO_ERR_CAPTURE;
    if (c->d_fit_rows) EVO_TRY(hipFree(c->d_fit_rows));
    c->d_fit_rows = nullptr;
    c->fit_rows_count = 0;
    const size_t cap = std::max<size_t>(2 * P, 256);
    EVO_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_fit_rows), cap * 2 * sizeof(float) + kGuardBytes));
    EVO_TRY(hipMemsetAsync(c->d_fit_rows + cap * 2, kGuardByte, kGuardBytes, stream));
    EVO_TRY(hipStreamSynchronize(stream));
    c->fit_rows_count = cap;
    return EVO_OK;
}

// A pinned staging buffer whose previous upload has completed.
int acquire_slot(evo_check *c, size_t bytes, StageSlot **out) {
    StageSlot &s = c->slots[c->next_slot];
    c->next_slot = (c->next_slot + 1) % kStageSlots;
    if (s.in_flight) {
        EVO_TRY(hipEventSynchronize(s.done));
        s.in_flight = false;
    }
    if (!s.done) EVO_TRY(hipEventCreateWithFlags(&s.done, hipEventDisableTiming));
    if (bytes > s.bytes) {
        if (s.host) EVO_TRY(hipHostFree(s.host));
        s.host = nullptr;
        s.bytes = 0;
        const size_t cap = std::max<size_t>(bytes * 2, 4096);
        EVO_TRY(hipHostMalloc(&s.host, cap, hipHostMallocDefault));
        s.bytes = cap;
    }
    *out = &s;
    return EVO_OK;
}

struct HostSeg {
    const void *ref;
    const void *const *cand_ptrs;
    uint64_t n;
    uint32_t P, dtype, row0;
    uint32_t case0 = 0, n_cases = 1;   // case group (evo_check_cases), else the segment alone
    float atol = 0.0f, rtol = 0.0f;    // filled in by resolve_tolerance
};

bool tolerance_ok(float atol, float rtol) {
    return atol >= 0.0f && rtol >= 0.0f && !std::isinf(atol) && !std::isinf(rtol);
}

// The tolerance a group is checked with: its class when it names one (1 .. kTolClasses, set
// beforehand), else the context's pair for its element type.
int resolve_tolerance(const evo_check *c, uint32_t tol_class, HostSeg &h) {
    if (tol_class > kTolClasses) return EVO_ERR_TOL;
    const Tolerance &t = tol_class ? c->by_class[tol_class] : c->by_dtype[h.dtype];
    if (!t.set) return EVO_ERR_TOL;
    h.atol = t.atol;
    h.rtol = t.rtol;
    return EVO_OK;
}


// Pure host validation of one group (no device call).
int validate_seg(const HostSeg &h) {
    if (!h.ref || !h.cand_ptrs) return EVO_ERR_NULL;
    if (!dtype_ok(h.dtype)) return EVO_ERR_DTYPE;
    if (h.n == 0 || h.P == 0 || h.P > kMaxP) return EVO_ERR_SIZE;
    const uintptr_t am = elem_size(h.dtype) - 1;
    if (reinterpret_cast<uintptr_t>(h.ref) & am) return EVO_ERR_ALIGN;
    for (uint32_t p = 0; p < h.P; ++p) {
        if (!h.cand_ptrs[p]) return EVO_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(h.cand_ptrs[p]) & am) return EVO_ERR_ALIGN;
    }
    return EVO_OK;
}

uint32_t pow2_ceil(uint32_t v) {
    uint32_t p = 1;
    while (p < v) p <<= 1;
    return p;
}

// What one step of a workgroup costs, in tile loads: its largest candidate group plus the
// reference.  A single candidate keeps one tile less in flight than the load pipeline
// holds, and its steps were measured 1.2x slower than their bytes: counted as 3.
uint32_t step_cost(uint32_t P) {
    uint32_t b = evo::kG;
    if (P < (uint32_t)evo::kG)
        for (b = 1; b * 2 <= P;) b *= 2;
    return std::max<uint32_t>(b + 1, 3u);
}

// The candidates beyond the last full group would be up to four groups of different sizes
// side by side, and the wavefronts of the small ones would idle while the largest works
// (7 bf16 candidates as 4 + 2 + 1: 0.47 of peak, 15 as 8 + 4 + 2 + 1: 0.54).  They are
// walked as ONE group of the next power of two instead, the missing candidates standing in
// as copies of the reference pointer: their loads hit the cache behind the reference's
// own, their statistics are computed and dropped.
uint32_t padded_population(uint32_t P) {
    const uint32_t rem = P % (uint32_t)evo::kG;
    return P - rem + (rem ? pow2_ceil(rem) : 0u);
}

// Share of a layout's wavefront slots that hold a group of at least half the full size.
double heavy_share(uint32_t n_heavy, uint32_t n_groups) {
    const uint32_t gpw = std::min<uint32_t>(pow2_ceil(n_groups), EVO_GPW_MAX);
    const uint32_t slots = (n_groups + gpw - 1) / gpw * gpw;
    return (double)n_heavy / slots;
}

// A small last group (1, 2 or 4 candidates) beside full groups leaves its wavefront idle
// most of the time.  Where that costs a quarter or more of the wavefront slots (17
// candidates: one full group beside a single candidate, 0.74 of the 16-candidate rate; 33
// bf16 candidates: 0.62), the segment is cut in two: the full groups, and the rest as a
// segment of its own whose jobs the partitioner sizes by their cost (33 candidates: 0.75).
// The price is a second read of the reference (1/(P+1) more bytes), so a segment stays
// whole where the small group rides in a slot that would be empty anyway (100 candidates =
// 6 full groups + 4: 0.83 whole, 0.74 cut), where it is short, and in case groups (one
// accumulator over several segments).
constexpr uint64_t kSplitMinTiles = 1024;

// out: room for two segments; returns how many were written (1 or 2).
size_t split_remainder(const HostSeg &h, HostSeg *out) {
    const uint32_t rem = h.P % (uint32_t)evo::kG, n_full = h.P / (uint32_t)evo::kG;
    const uint64_t tiles = (h.n + evo::tile_elems(h.dtype) - 1) / evo::tile_elems(h.dtype);
    const bool gains = n_full > 0 && rem != 0 && rem <= (uint32_t)evo::kG / 4 &&
                       heavy_share(n_full, n_full) - heavy_share(n_full, n_full + 1) >= 0.25;
    if (h.n_cases > 1 || !gains || tiles < kSplitMinTiles) {
        out[0] = h;
        return 1;
    }
    HostSeg full = h, rest = h;
    full.P = h.P - rem;
    rest.P = rem;
    rest.cand_ptrs = h.cand_ptrs + full.P;
    rest.row0 = h.row0 + full.P;
    out[0] = full;
    out[1] = rest;
    return 2;
}

void split_remainders(const std::vector<HostSeg> &in, std::vector<HostSeg> &out) {
    out.resize(in.size() * 2);
    size_t n = 0;
    for (const HostSeg &h : in) n += split_remainder(h, out.data() + n);
    out.resize(n);
}

// A case group is folded directly (kFoldCasesDirect) when one workgroup can hold all of it:
// a thread per (case, candidate, range of jobs) with at most kDirectRowsPerThread rows to add.
void choose_fold_modes(SegDesc *descs, size_t n_segs) {
    for (size_t s = 0; s < n_segs;) {
        const uint32_t K = descs[s].n_cases;
        if (K <= 1 || descs[s].case0 != s || s + K > n_segs) {
            ++s;
            continue;
        }
        const uint32_t Kp = pow2_ceil(K), pc = pow2_ceil(descs[s].P);
        bool ok = K <= evo::kDirectMaxCases && (uint64_t)Kp * pc <= (uint64_t)evo::kThreads;
        if (ok) {
            const uint32_t ranges = (uint32_t)evo::kThreads / (Kp * pc);
            for (uint32_t k = 0; k < K; ++k)
                ok = ok && descs[s + k].P == descs[s].P &&
                     (descs[s + k].n_chunks + ranges - 1) / ranges <= evo::kDirectRowsPerThread;
        }
        for (uint32_t k = 0; k < K; ++k) descs[s + k].fold_mode = ok ? evo::kFoldCasesDirect : evo::kFoldLevels;
        s += K;
    }
}

// Splits every segment into jobs (workgroups) of similar cost.  Cost unit: one tile load
// of one wavefront; a step of a workgroup costs its largest candidate group plus the
// reference.  The launch is sized to the machine (a fixed number of workgroups per
// compute unit, all resident at once), so that the per-job epilogue -- cross-lane
// reduction, partial rows, ticket -- is paid once per wavefront slot and not once per few
// tiles.
// descs: room for n_segs descriptors.  Allocates nothing.
void partition(const HostSeg *segs, size_t n_segs, uint32_t target_jobs, SegDesc *descs,
               uint32_t &total_jobs) {
    uint64_t cost = 0;   // summed over all jobs: steps x cost of a step
    for (size_t s = 0; s < n_segs; ++s) {
        const HostSeg &h = segs[s];
        SegDesc &d = descs[s];
        d.n = h.n;
        d.P = padded_population(h.P);
        d.n_pad = (uint8_t)(d.P - h.P);
        d.dtype = (uint8_t)h.dtype;
        d.fold_mode = evo::kFoldLevels;
        d.atol = h.atol;
        d.rtol = h.rtol;
        d.stats_row0 = h.row0;
        d.n_groups = evo::group_count(d.P);
        d.gpw = (uint8_t)std::min<uint32_t>(pow2_ceil(d.n_groups), EVO_GPW_MAX);
        d.case0 = h.n_cases > 1 ? h.case0 : (uint32_t)s;
        d.n_cases = h.n_cases;
        const uint64_t tiles = (h.n + evo::tile_elems(h.dtype) - 1) / evo::tile_elems(h.dtype);
        const uint32_t tpw = evo::kWaves / d.gpw;
        const uint32_t gblocks = (d.n_groups + d.gpw - 1) / d.gpw;
        cost += (tiles + tpw - 1) / tpw * gblocks * step_cost(d.P);
    }
    // cost one job should take
    uint64_t per_job = (cost + target_jobs - 1) / target_jobs;
    // A job should be worth its epilogue (reduction, rows, tickets, folds): in a launch too
    // small to give every slot such a job, jobs are made that long anyway as long as about
    // one per compute unit remains (fp32, one candidate of 2^22 elements: 40 -> 33 us; 16
    // candidates: 78 -> 70 us; nothing changes from 2^23 x 16 upwards or below 2^21 x 16).
    per_job = std::max<uint64_t>(per_job, std::min<uint64_t>(EVO_MIN_JOB_COST, cost / EVO_MIN_JOBS));
    if (per_job == 0) per_job = 1;
    // The rounding up per segment can push the total past the number of workgroups the
    // machine holds at once, and the surplus would run as a second round after everything
    // else: coarsen until the launch fits (it cannot when there are more segments than
    // slots; then every segment still gets its one workgroup).
    uint32_t job0 = 0;
    for (int attempt = 0; attempt < 64; ++attempt) {
        job0 = 0;
        bool any_free = false;   // some segment could still take longer jobs
        for (size_t s = 0; s < n_segs; ++s) {
            SegDesc &d = descs[s];
            const uint64_t tiles = (d.n + evo::tile_elems(d.dtype) - 1) / evo::tile_elems(d.dtype);
            const uint32_t tpw = evo::kWaves / d.gpw;
            const uint32_t per_step = step_cost(d.P);
            // tiles one wavefront takes per job
            uint64_t per_wave = (per_job + per_step - 1) / per_step;
            per_wave = std::max<uint64_t>(per_wave, kMinTilesPerWave);
            if (per_wave < evo::kMaxTilesPerWave) any_free = true;
            else per_wave = evo::kMaxTilesPerWave;
            const uint64_t per_chunk = per_wave * tpw;
            const uint64_t chunks = (tiles + per_chunk - 1) / per_chunk;
            d.n_chunks = (uint32_t)chunks;
            const uint32_t gblocks = (d.n_groups + d.gpw - 1) / d.gpw;
            d.n_jobs = gblocks * d.n_chunks;
            d.job0 = job0;
            job0 += d.n_jobs;
        }
        if (job0 <= target_jobs || !any_free) break;
        // next candidate: scale by the overshoot, at least one unit more
        per_job = std::max<uint64_t>(per_job + 1, per_job * job0 / target_jobs);
    }
    total_jobs = job0;
    choose_fold_modes(descs, n_segs);
}

// Upper bound on what partition() can produce for these segments (checked before any
// allocation): every count must stay inside 32 bits.
bool partition_fits(const HostSeg *segs, size_t n_segs) {
    uint64_t jobs = 0;
    for (size_t s = 0; s < n_segs; ++s) {
        const HostSeg &h = segs[s];
        const uint64_t tiles = (h.n + evo::tile_elems(h.dtype) - 1) / evo::tile_elems(h.dtype);
        const uint64_t groups = evo::group_count(h.P);
        jobs += (tiles / kMinTilesPerWave + 1) * groups;
        if (jobs > (1ull << 30)) return false;
    }
    return true;
}

// fit: when given, the timing reduction is part of the same work (evo_evaluate): one launch
// when the table fits the kernel argument block, else the check and then the fitness kernel.
int run_check(evo_check *c, const std::vector<HostSeg> &whole, hipStream_t stream,
              evo_stats *stats, const evo::FitLaunch *fit = nullptr) {
    int rc = bind_device(c);
    if (rc != EVO_OK) return rc;
    std::vector<HostSeg> segs;
    try {
        split_remainders(whole, segs);
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }

    if (c->n_cus == 0) {
        int cus = 0;
        EVO_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device));
        c->n_cus = cus > 0 ? (uint32_t)cus : 1u;
    }
    if (!partition_fits(segs.data(), segs.size())) return EVO_ERR_SIZE;

    std::vector<SegDesc> descs;
    uint32_t total_jobs = 0;
    size_t total_ptrs = 0;
    try {
        descs.resize(segs.size());
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }
    partition(segs.data(), segs.size(), c->n_cus * kJobsPerCu, descs.data(), total_jobs);
    uint32_t dtype_set = 0;
    for (size_t s = 0; s < segs.size(); ++s) {
        total_ptrs += descs[s].P;
        dtype_set |= 1u << segs[s].dtype;
    }

    const size_t S = segs.size();
    // first-level rows (one set per job) and second-level rows (at most one set per job);
    // bundle tickets (indexed like jobs) and segment tickets
    // (layout: see evo_internal.h)
    if ((rc = ensure_partials(c, 2 * (size_t)total_jobs * evo::kRowsPerJob + total_ptrs, stream)) != EVO_OK)
        return rc;
    if ((rc = ensure_tickets(c, (size_t)total_jobs + 2 * S, stream)) != EVO_OK) return rc;

    size_t off = 0;
    for (size_t s = 0; s < S; ++s) {
        descs[s].ref = segs[s].ref;
        descs[s].ptr0 = off;
        off += descs[s].P;
    }

    if (S <= evo::kInlineSegs && total_ptrs <= evo::kInlinePtrs) {
        // everything fits into the kernel argument block: no staging, no copy
        evo::InlineTable tab;
        std::memset(&tab, 0, sizeof tab);
        for (size_t s = 0; s < S; ++s) {
            tab.descs[s] = descs[s];
            for (uint32_t p = 0; p < descs[s].P; ++p)
                tab.ptrs[descs[s].ptr0 + p] =
                    reinterpret_cast<uint64_t>(p < segs[s].P ? segs[s].cand_ptrs[p] : segs[s].ref);
        }
        if (fit) {
            // one case group writes its rows once; independent segments write theirs each
            evo::FitLaunch f = *fit;
            f.writers = segs[0].n_cases > 1 ? 1u : (uint32_t)S;
            return dev(evo::launch_evaluate(dtype_set, tab, (uint32_t)S, total_jobs,
                                            c->n_cus, c->d_partials, c->d_tickets, stats, f, stream));
        }
        return dev(evo::launch_check_inline(dtype_set, tab, (uint32_t)S, total_jobs,
                                            c->n_cus, c->d_partials, c->d_tickets, stats, stream));
    }

    // blob = descriptors, then all candidate pointers, staged through pinned memory
    const size_t desc_bytes = S * sizeof(SegDesc);
    const size_t blob_bytes = desc_bytes + total_ptrs * sizeof(uint64_t);
    // a replay of a captured copy would read whatever the staging slot holds by then
    if (capturing(stream)) return EVO_ERR_CAPTURE;
    if ((rc = ensure_table(c, blob_bytes, stream)) != EVO_OK) return rc;
    StageSlot *slot = nullptr;
    if ((rc = acquire_slot(c, blob_bytes, &slot)) != EVO_OK) return rc;
    char *hb = static_cast<char *>(slot->host);
    uint64_t *hptrs = reinterpret_cast<uint64_t *>(hb + desc_bytes);
    for (size_t s = 0; s < S; ++s)
        for (uint32_t p = 0; p < descs[s].P; ++p)
            hptrs[descs[s].ptr0 + p] =
                reinterpret_cast<uint64_t>(p < segs[s].P ? segs[s].cand_ptrs[p] : segs[s].ref);
    std::memcpy(hb, descs.data(), desc_bytes);

    EVO_TRY(hipMemcpyAsync(c->d_table, hb, blob_bytes, hipMemcpyHostToDevice, stream));
    EVO_TRY(hipEventRecord(slot->done, stream));
    slot->in_flight = true;

    rc = dev(evo::launch_check(
        dtype_set, static_cast<const SegDesc *>(c->d_table),
        reinterpret_cast<const uint64_t *>(static_cast<char *>(c->d_table) + desc_bytes), (uint32_t)S,
        total_jobs, c->n_cus, c->d_partials, c->d_tickets, stats, stream));
    if (rc != EVO_OK || !fit) return rc;
    return dev(evo::launch_fitness(fit->timings, fit->baseline, fit->P, fit->T, fit->reducer, stats,
                                   fit->summary, fit->base, fit->ticket, stream));
}

// The groups of a segmented call: each valid on its own, rows inside [0, n_rows) and not
// shared between groups.  covered: rows that belong to some group.
int collect_segments(const evo_check *c, const evo_segment *segs, uint32_t S, uint32_t n_rows,
                     std::vector<HostSeg> &hs, uint64_t &covered) {
    hs.resize(S);
    std::vector<std::pair<uint64_t, uint64_t>> ranges(S);
    covered = 0;
    for (uint32_t s = 0; s < S; ++s) {
        hs[s] = HostSeg{segs[s].ref, segs[s].cand_ptrs, segs[s].n_elems, segs[s].P_s,
                        segs[s].dtype, segs[s].stats_row0, 0u, 1u};
        int rc = validate_seg(hs[s]);
        if (rc != EVO_OK) return rc;
        if ((rc = resolve_tolerance(c, segs[s].tol_class, hs[s])) != EVO_OK) return rc;
        const uint64_t lo = segs[s].stats_row0, hi = lo + segs[s].P_s;
        if (hi > n_rows) return EVO_ERR_SIZE;
        ranges[s] = {lo, hi};
        covered += segs[s].P_s;
    }
    std::sort(ranges.begin(), ranges.end());
    for (uint32_t s = 1; s < S; ++s)
        if (ranges[s].first < ranges[s - 1].second) return EVO_ERR_SIZE;
    return EVO_OK;
}

}  // namespace

extern "C" {

int evo_check_create(evo_check_t **out, evo_dtype dtype, uint64_t n_elems, float atol,
                     float rtol) {
    if (!out) return EVO_ERR_NULL;
    *out = nullptr;
    if (!dtype_ok((uint32_t)dtype)) return EVO_ERR_DTYPE;
    if (n_elems == 0) return EVO_ERR_SIZE;
    if (!tolerance_ok(atol, rtol)) return EVO_ERR_TOL;
    evo_check *c = new (std::nothrow) evo_check();
    if (!c) return EVO_ERR_NOMEM;
    c->dtype = dtype;
    c->n_elems = n_elems;
    for (Tolerance &t : c->by_dtype) t = Tolerance{atol, rtol, true};
    try {
        std::lock_guard<std::mutex> lk(g_mu);
        g_live.insert(c);
    } catch (const std::bad_alloc &) {
        delete c;
        return EVO_ERR_NOMEM;
    }
    *out = c;
    return EVO_OK;
}

int evo_check_set_tolerance(evo_check_t *c, evo_dtype dtype, float atol, float rtol) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!dtype_ok((uint32_t)dtype)) return EVO_ERR_DTYPE;
    if (!tolerance_ok(atol, rtol)) return EVO_ERR_TOL;
    c->by_dtype[(uint32_t)dtype] = Tolerance{atol, rtol, true};
    return EVO_OK;
}

int evo_check_set_tolerance_class(evo_check_t *c, uint32_t tol_class, float atol, float rtol) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (tol_class == 0 || tol_class > kTolClasses) return EVO_ERR_SIZE;
    if (!tolerance_ok(atol, rtol)) return EVO_ERR_TOL;
    c->by_class[tol_class] = Tolerance{atol, rtol, true};
    return EVO_OK;
}

int evo_check_batch(evo_check_t *c, const void *ref, const void *const *cand_ptrs, uint32_t P,
                    void *stream, evo_stats *stats) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!stats) return EVO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(stats) & 7u) return EVO_ERR_ALIGN;
    HostSeg h{ref, cand_ptrs, c->n_elems, P, (uint32_t)c->dtype, 0u, 0u, 1u};
    int rc = validate_seg(h);
    if (rc != EVO_OK) return rc;
    if ((rc = resolve_tolerance(c, 0u, h)) != EVO_OK) return rc;
    try {
        std::vector<HostSeg> segs(1, h);
        return run_check(c, segs, static_cast<hipStream_t>(stream), stats);
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }
}

int evo_check_batch_static(evo_check_t *c, const void *ref, const void *const *cand_ptrs, uint32_t P,
                           void *stream, evo_stats *stats) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!stats) return EVO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(stats) & 7u) return EVO_ERR_ALIGN;
    HostSeg h{ref, cand_ptrs, c->n_elems, P, (uint32_t)c->dtype, 0u, 0u, 1u};
    int rc = validate_seg(h);
    if (rc != EVO_OK) return rc;
    if ((rc = resolve_tolerance(c, 0u, h)) != EVO_OK) return rc;
    if (P > evo::kInlinePtrs) return EVO_ERR_LIMIT;
    if ((rc = bind_device(c)) != EVO_OK) return rc;
    if (c->n_cus == 0) {
        int cus = 0;
        EVO_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, c->device));
        c->n_cus = cus > 0 ? (uint32_t)cus : 1u;
    }
    unsigned char *base = nullptr;
    if ((rc = static_scratch(c->device, &base)) != EVO_OK) return rc;

    // the same plan as evo_check_batch, on the stack
    HostSeg segs[2];
    const size_t S = split_remainder(h, segs);
    if (!partition_fits(segs, S)) return EVO_ERR_SIZE;
    SegDesc descs[2];
    uint32_t total_jobs = 0;
    partition(segs, S, c->n_cus * kJobsPerCu, descs, total_jobs);
    size_t total_ptrs = 0;
    for (size_t s = 0; s < S; ++s) {
        descs[s].ref = segs[s].ref;
        descs[s].ptr0 = total_ptrs;
        total_ptrs += descs[s].P;
    }
    if (total_jobs > kStaticMaxJobs || total_ptrs > evo::kInlinePtrs) return EVO_ERR_LIMIT;

    evo::InlineTable tab;
    std::memset(&tab, 0, sizeof tab);
    for (size_t s = 0; s < S; ++s) {
        tab.descs[s] = descs[s];
        for (uint32_t p = 0; p < descs[s].P; ++p)
            tab.ptrs[descs[s].ptr0 + p] =
                reinterpret_cast<uint64_t>(p < segs[s].P ? segs[s].cand_ptrs[p] : segs[s].ref);
    }
    uint32_t dtype_set = 1u << (uint32_t)c->dtype;
    Partial *partials = reinterpret_cast<Partial *>(base);
    uint32_t *tickets = reinterpret_cast<uint32_t *>(base + kStaticPartialBytes);
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The tickets must be zero when the kernel starts.  Every launch leaves them at zero, but
    // the array is shared by all callers on this device and outlives a launch that failed: they
    // are cleared by a small fill kernel in front (not a memset node, so that the pair of
    // launches can be captured into a graph).
    EVO_TRY(evo::launch_flush(tickets, ((size_t)total_jobs + 2 * S) * sizeof(uint32_t), 0u, st));
    return dev(evo::launch_check_inline(dtype_set, tab, (uint32_t)S, total_jobs, c->n_cus,
                                        partials, tickets, stats, st));
}

int evo_check_segmented(evo_check_t *c, const evo_segment *segs, uint32_t S, void *stream,
                        evo_stats *stats, uint32_t n_rows) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!segs || !stats) return EVO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(stats) & 7u) return EVO_ERR_ALIGN;
    if (S == 0 || n_rows == 0) return EVO_ERR_SIZE;
    try {
        std::vector<HostSeg> hs;
        uint64_t covered = 0;
        const int rc = collect_segments(c, segs, S, n_rows, hs, covered);
        if (rc != EVO_OK) return rc;
        return run_check(c, hs, static_cast<hipStream_t>(stream), stats);
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }
}

int evo_check_cases(evo_check_t *c, const evo_segment *cases, uint32_t K, void *stream,
                    evo_stats *stats) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!cases || !stats) return EVO_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(stats) & 7u) return EVO_ERR_ALIGN;
    if (K == 0) return EVO_ERR_SIZE;
    try {
        std::vector<HostSeg> hs(K);
        for (uint32_t k = 0; k < K; ++k) {
            hs[k] = HostSeg{cases[k].ref, cases[k].cand_ptrs, cases[k].n_elems, cases[k].P_s,
                            cases[k].dtype, 0u, 0u, K};
            int rc = validate_seg(hs[k]);
            if (rc != EVO_OK) return rc;
            if ((rc = resolve_tolerance(c, cases[k].tol_class, hs[k])) != EVO_OK) return rc;
            if (cases[k].P_s != cases[0].P_s || cases[k].stats_row0 != 0) return EVO_ERR_SIZE;
        }
        return run_check(c, hs, static_cast<hipStream_t>(stream), stats);
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }
}

int evo_fitness(evo_check_t *c, const float *timings, const float *baseline, uint32_t P,
                uint32_t T, void *stream, evo_stats *stats, evo_pop_summary *summary) {
    return evo_fitness_ex(c, timings, baseline, P, T, EVO_REDUCE_MEDIAN, stream, stats, summary);
}

int evo_fitness_ex(evo_check_t *c, const float *timings, const float *baseline, uint32_t P,
                   uint32_t T, int reducer, void *stream, evo_stats *stats,
                   evo_pop_summary *summary) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!timings || !baseline || !stats) return EVO_ERR_NULL;
    if (reducer != EVO_REDUCE_MEDIAN && reducer != EVO_REDUCE_MEAN) return EVO_ERR_SIZE;
    if (P == 0 || T == 0 || T > EVO_FITNESS_MAX_T || P > (1u << 20)) return EVO_ERR_SIZE;
    if ((reinterpret_cast<uintptr_t>(timings) & 3u) || (reinterpret_cast<uintptr_t>(baseline) & 3u) ||
        (reinterpret_cast<uintptr_t>(stats) & 7u) || (reinterpret_cast<uintptr_t>(summary) & 3u))
        return EVO_ERR_ALIGN;
    int rc = bind_device(c);
    if (rc != EVO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if ((rc = ensure_fitness_scratch(c, st)) != EVO_OK) return rc;
    return dev(evo::launch_fitness(timings, baseline, P, T, (uint32_t)reducer, stats, summary,
                                   c->d_base_median, c->d_fit_ticket, st));
}

int evo_select_elite(evo_check_t *c, const evo_stats *stats, uint32_t P, uint32_t k, void *stream,
                     uint32_t *elite, uint32_t *n_elite) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!stats || !elite) return EVO_ERR_NULL;
    if (P == 0 || k == 0 || k > P || P > kMaxP) return EVO_ERR_SIZE;
    if ((reinterpret_cast<uintptr_t>(stats) & 7u) || (reinterpret_cast<uintptr_t>(elite) & 3u) ||
        (reinterpret_cast<uintptr_t>(n_elite) & 3u))
        return EVO_ERR_ALIGN;
    const int rc = bind_device(c);
    if (rc != EVO_OK) return rc;
    return dev(evo::launch_select(stats, P, k, elite, n_elite, static_cast<hipStream_t>(stream)));
}

int evo_select_elite_diverse(evo_check_t *c, const evo_stats *stats, const uint32_t *keys, uint32_t P,
                             uint32_t k, void *stream, uint32_t *elite, uint32_t *n_elite) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!stats || !keys || !elite) return EVO_ERR_NULL;
    if (P == 0 || k == 0 || k > P || P > kMaxP) return EVO_ERR_SIZE;
    if ((reinterpret_cast<uintptr_t>(stats) & 7u) || (reinterpret_cast<uintptr_t>(keys) & 3u) ||
        (reinterpret_cast<uintptr_t>(elite) & 3u) || (reinterpret_cast<uintptr_t>(n_elite) & 3u))
        return EVO_ERR_ALIGN;
    const int rc = bind_device(c);
    if (rc != EVO_OK) return rc;
    if (P > c->rep_count) {
        if (capturing(static_cast<hipStream_t>(stream))) return EVO_ERR_CAPTURE;
        if (c->d_rep) EVO_TRY(hipFree(c->d_rep));
        c->d_rep = nullptr;
        c->rep_count = 0;
        const size_t cap = std::max<size_t>(2 * (size_t)P, 1024);
        EVO_TRY(hipMalloc(reinterpret_cast<void **>(&c->d_rep), cap * sizeof(uint32_t)));
        c->rep_count = cap;
    }
    return dev(evo::launch_select_diverse(stats, keys, c->d_rep, P, k, elite, n_elite,
                                          static_cast<hipStream_t>(stream)));
}

int evo_evaluate(evo_check_t *c, const evo_segment *cases, uint32_t K, const float *timings,
                 const float *baseline, uint32_t T, int reducer, void *stream, evo_stats *stats,
                 evo_pop_summary *summary) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!cases || !stats || !timings || !baseline) return EVO_ERR_NULL;
    if (K == 0 || T == 0 || T > EVO_FITNESS_MAX_T) return EVO_ERR_SIZE;
    if (reducer != EVO_REDUCE_MEDIAN && reducer != EVO_REDUCE_MEAN) return EVO_ERR_SIZE;
    if ((reinterpret_cast<uintptr_t>(timings) & 3u) || (reinterpret_cast<uintptr_t>(baseline) & 3u) ||
        (reinterpret_cast<uintptr_t>(stats) & 7u) || (reinterpret_cast<uintptr_t>(summary) & 3u))
        return EVO_ERR_ALIGN;
    try {
        std::vector<HostSeg> hs(K);
        for (uint32_t k = 0; k < K; ++k) {
            hs[k] = HostSeg{cases[k].ref, cases[k].cand_ptrs, cases[k].n_elems, cases[k].P_s,
                            cases[k].dtype, 0u, 0u, K};
            int rc = validate_seg(hs[k]);
            if (rc != EVO_OK) return rc;
            if ((rc = resolve_tolerance(c, cases[k].tol_class, hs[k])) != EVO_OK) return rc;
            if (cases[k].P_s != cases[0].P_s || cases[k].stats_row0 != 0) return EVO_ERR_SIZE;
        }
        int rc = bind_device(c);
        if (rc != EVO_OK) return rc;
        hipStream_t st = static_cast<hipStream_t>(stream);
        if ((rc = ensure_fitness_scratch(c, st)) != EVO_OK) return rc;
        if ((rc = ensure_fit_rows(c, cases[0].P_s, st)) != EVO_OK) return rc;
        const evo::FitLaunch fit{timings, baseline, summary, c->d_base_median, c->d_fit_rows,
                                 c->d_fit_ticket, cases[0].P_s, T, (uint32_t)reducer, 1u};
        return run_check(c, hs, st, stats, &fit);
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }
}

int evo_evaluate_segmented(evo_check_t *c, const evo_segment *segs, uint32_t S, const float *timings,
                           const float *baseline, uint32_t T, int reducer, void *stream,
                           evo_stats *stats, uint32_t n_rows, evo_pop_summary *summary) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!segs || !stats || !timings || !baseline) return EVO_ERR_NULL;
    if (S == 0 || n_rows == 0 || n_rows > (1u << 20) || T == 0 || T > EVO_FITNESS_MAX_T)
        return EVO_ERR_SIZE;
    if (reducer != EVO_REDUCE_MEDIAN && reducer != EVO_REDUCE_MEAN) return EVO_ERR_SIZE;
    if ((reinterpret_cast<uintptr_t>(timings) & 3u) || (reinterpret_cast<uintptr_t>(baseline) & 3u) ||
        (reinterpret_cast<uintptr_t>(stats) & 7u) || (reinterpret_cast<uintptr_t>(summary) & 3u))
        return EVO_ERR_ALIGN;
    try {
        std::vector<HostSeg> hs;
        uint64_t covered = 0;
        int rc = collect_segments(c, segs, S, n_rows, hs, covered);
        if (rc != EVO_OK) return rc;
        if (covered != n_rows) return EVO_ERR_SIZE;   // a row without a group has no valid flag
        if ((rc = bind_device(c)) != EVO_OK) return rc;
        hipStream_t st = static_cast<hipStream_t>(stream);
        if ((rc = ensure_fitness_scratch(c, st)) != EVO_OK) return rc;
        if ((rc = ensure_fit_rows(c, n_rows, st)) != EVO_OK) return rc;
        const evo::FitLaunch fit{timings, baseline, summary, c->d_base_median, c->d_fit_rows,
                                 c->d_fit_ticket, n_rows, T, (uint32_t)reducer, 1u};
        return run_check(c, hs, st, stats, &fit);
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }
}

int evo_time_candidates(evo_check_t *c, const evo_launch_fn *launch, void *const *user, uint32_t P,
                        uint32_t T, const evo_timing_opts *opts, void *stream, float *timings,
                        float *clock_ratio) {
    if (!is_live(c)) return EVO_ERR_HANDLE;
    if (!launch || !timings || !opts) return EVO_ERR_NULL;
    if (P == 0 || T == 0 || T > EVO_FITNESS_MAX_T || P > kMaxP || opts->warmup > 1000000u)
        return EVO_ERR_SIZE;
    for (uint32_t p = 0; p < P; ++p)
        if (!launch[p]) return EVO_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(timings) & 3u) || (reinterpret_cast<uintptr_t>(clock_ratio) & 3u))
        return EVO_ERR_ALIGN;
    int rc = bind_device(c);
    if (rc != EVO_OK) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (capturing(st)) return EVO_ERR_CAPTURE;   // this call waits for its own runs

    // resources, on first use: two events per timed run plus two probe pairs, the pinned
    // staging table, the probe's sink, the flush buffer
    const size_t n_events = 2 * (size_t)T + 4;
    try {
        while (c->time_events.size() < n_events) {
            hipEvent_t e = nullptr;
            EVO_TRY(hipEventCreate(&e));
            c->time_events.push_back(e);
        }
    } catch (const std::bad_alloc &) {
        return EVO_ERR_NOMEM;
    }
    const size_t count = (size_t)P * T;
    if (count > c->h_times_count) {
        if (c->h_times) EVO_TRY(hipHostFree(c->h_times));
        c->h_times = nullptr;
        c->h_times_count = 0;
        void *h = nullptr;
        EVO_TRY(hipHostMalloc(&h, count * sizeof(float), hipHostMallocDefault));
        c->h_times = static_cast<float *>(h);
        c->h_times_count = count;
    }
    if (!c->d_probe_sink) {
        void *d = nullptr;
        EVO_TRY(hipMalloc(&d, 256));
        c->d_probe_sink = static_cast<float *>(d);
    }
    if (opts->flush_cache && !c->d_flush) EVO_TRY(hipMalloc(&c->d_flush, kFlushBytes));

    hipEvent_t *ev = c->time_events.data();
    hipEvent_t *probe = ev + 2 * (size_t)T;   // [0],[1] before, [2],[3] after
    // An idle device sits at a low clock and the first launch of a kernel also loads its
    // code: a few milliseconds of the probe before anything is timed.
    for (int i = 0; i < kProbeSpinUp; ++i)
        EVO_TRY(evo::launch_probe(c->d_probe_sink, kProbeIterations, st));
    for (uint32_t p = 0; p < P; ++p) {
        void *u = user ? user[p] : nullptr;
        for (uint32_t w = 0; w < opts->warmup; ++w) launch[p](u, stream);
        EVO_TRY(hipEventRecord(probe[0], st));
        EVO_TRY(evo::launch_probe(c->d_probe_sink, kProbeIterations, st));
        EVO_TRY(hipEventRecord(probe[1], st));
        for (uint32_t t = 0; t < T; ++t) {
            if (opts->flush_cache) EVO_TRY(evo::launch_flush(c->d_flush, kFlushBytes, p * T + t, st));
            EVO_TRY(hipEventRecord(ev[2 * t], st));
            launch[p](u, stream);
            EVO_TRY(hipEventRecord(ev[2 * t + 1], st));
        }
        EVO_TRY(hipEventRecord(probe[2], st));
        EVO_TRY(evo::launch_probe(c->d_probe_sink, kProbeIterations, st));
        EVO_TRY(hipEventRecord(probe[3], st));
        EVO_TRY(hipEventSynchronize(probe[3]));
        for (uint32_t t = 0; t < T; ++t) {
            float ms = 0.0f;
            EVO_TRY(hipEventElapsedTime(&ms, ev[2 * t], ev[2 * t + 1]));
            c->h_times[(size_t)p * T + t] = ms;
        }
        if (clock_ratio) {
            float before = 0.0f, after = 0.0f;
            EVO_TRY(hipEventElapsedTime(&before, probe[0], probe[1]));
            EVO_TRY(hipEventElapsedTime(&after, probe[2], probe[3]));
            clock_ratio[p] = before > 0.0f ? after / before : 0.0f;
        }
    }
    EVO_TRY(hipMemcpyAsync(timings, c->h_times, count * sizeof(float), hipMemcpyHostToDevice, st));
    EVO_TRY(hipStreamSynchronize(st));   // the staging table may be reused by the next call
    return EVO_OK;
}

int evo_check_destroy(evo_check_t *c) {
    {
        std::lock_guard<std::mutex> lk(g_mu);
        if (!c || g_live.erase(c) == 0) return EVO_ERR_HANDLE;
    }
    int rc = EVO_OK;
    if (c->device != -1) {
        int cur = -1;
        if (hipGetDevice(&cur) == hipSuccess && cur != c->device) (void)hipSetDevice(c->device);
        if (hipDeviceSynchronize() != hipSuccess) rc = EVO_ERR_DEVICE;
        // the guards behind the buffers the kernels write must be untouched
        const void *guards[3] = {
            c->d_partials ? reinterpret_cast<const char *>(c->d_partials) + c->partial_rows * sizeof(Partial) : nullptr,
            c->d_tickets ? reinterpret_cast<const char *>(c->d_tickets + c->n_tickets) : nullptr,
            c->d_fit_rows ? reinterpret_cast<const char *>(c->d_fit_rows + c->fit_rows_count * 2) : nullptr};
        for (const void *g : guards) {
            unsigned char host[kGuardBytes];
            if (!g || rc != EVO_OK) continue;
            if (hipMemcpy(host, g, kGuardBytes, hipMemcpyDeviceToHost) != hipSuccess) {
                rc = EVO_ERR_DEVICE;
                continue;
            }
            for (size_t i = 0; i < kGuardBytes; ++i)
                if (host[i] != kGuardByte) rc = EVO_ERR_INTERNAL;
        }
        if (c->d_table) (void)hipFree(c->d_table);
        if (c->d_partials) (void)hipFree(c->d_partials);
        if (c->d_tickets) (void)hipFree(c->d_tickets);
        if (c->d_base_median) (void)hipFree(c->d_base_median);
        if (c->d_fit_rows) (void)hipFree(c->d_fit_rows);
        if (c->d_rep) (void)hipFree(c->d_rep);
        for (StageSlot &s : c->slots) {
            if (s.host) (void)hipHostFree(s.host);
            if (s.done) (void)hipEventDestroy(s.done);
        }
        for (hipEvent_t e : c->time_events) (void)hipEventDestroy(e);
        if (c->d_flush) (void)hipFree(c->d_flush);
        if (c->h_times) (void)hipHostFree(c->h_times);
        if (c->d_probe_sink) (void)hipFree(c->d_probe_sink);
        if (cur != -1 && cur != c->device) (void)hipSetDevice(cur);
    }
    delete c;
    return rc;
}

const char *evo_strerror(int code) {
    switch (code) {
        case EVO_OK: return "ok";
        case EVO_ERR_NULL: return "a required pointer is NULL";
        case EVO_ERR_DTYPE: return "unknown element type";
        case EVO_ERR_SIZE: return "zero or out-of-range count";
        case EVO_ERR_TOL: return "tolerance is negative, NaN or infinite, or the tolerance class is not set";
        case EVO_ERR_ALIGN: return "pointer not aligned to its element size";
        case EVO_ERR_DEVICE: return "HIP call failed";
        case EVO_ERR_NOMEM: return "out of memory";
        case EVO_ERR_HANDLE: return "not a live context";
        case EVO_ERR_LIMIT: return "beyond the fixed capacity of the call that allocates nothing";
        case EVO_ERR_INTERNAL: return "a guard behind the library's scratch memory was overwritten";
        case EVO_ERR_CAPTURE: return "the stream is capturing and the call would have to allocate, clear or stage";
        default: return "unknown status";
    }
}

}  // extern "C"
