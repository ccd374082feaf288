// Host-sanitizer driver for the host side of the C ABI (include/evo.h).
//
// Built by tests/test_host_sanitizers.py with hipcc, the host pass under
// -fsanitize=address,undefined, and run on the CPU.  The translation unit of the
// library's host code is included textually so that its internal partitioner can be
// driven directly; the four kernel launchers are replaced by stubs that launch
// nothing, so no kernel runs even where a GPU is present.
//
// Covered: every argument check of every entry point, handle lifetime (double
// destroy, foreign pointers), behaviour when HIP has no device (a clean
// EVO_ERR_DEVICE, nothing leaked), and the partitioner on a few thousand seeded
// ragged populations, checked against the invariants the kernel's indexing relies
// on (the list of those is in check_partition below).
#include "../../paper_2510_03760_amd/csrc/evo_api.hip"

#include <cstdio>
#include <cstdlib>

namespace evo {
static int g_launches = 0;
hipError_t launch_check(uint32_t, const SegDesc *, const uint64_t *, uint32_t, uint32_t,
                        uint32_t, Partial *, uint32_t *, evo_stats *, hipStream_t) { ++g_launches; return hipSuccess; }
static float g_last_atol[8], g_last_rtol[8];   // tolerances of the last inline launch's descriptors
hipError_t launch_check_inline(uint32_t, const InlineTable &tab, uint32_t S, uint32_t, uint32_t,
                               Partial *, uint32_t *, evo_stats *, hipStream_t) {
    for (uint32_t s = 0; s < S && s < 8; ++s) {
        g_last_atol[s] = tab.descs[s].atol;
        g_last_rtol[s] = tab.descs[s].rtol;
    }
    ++g_launches;
    return hipSuccess;
}
hipError_t launch_fitness(const float *, const float *, uint32_t, uint32_t, uint32_t, evo_stats *,
                          evo_pop_summary *, float *, uint32_t *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_select(const evo_stats *, uint32_t, uint32_t, uint32_t *, uint32_t *, hipStream_t) {
    ++g_launches;
    return hipSuccess;
}
hipError_t launch_select_diverse(const evo_stats *, const uint32_t *, uint32_t *, uint32_t, uint32_t, uint32_t *,
                                 uint32_t *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_evaluate(uint32_t, const InlineTable &, uint32_t, uint32_t, uint32_t, Partial *,
                           uint32_t *, evo_stats *, const FitLaunch &, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_flush(void *, size_t, uint32_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_probe(float *, uint32_t, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace evo

static int g_fail = 0;
#define EXPECT(cond)                                                        \
    do {                                                                    \
        if (!(cond)) {                                                      \
            std::printf("FAIL %s:%d: %s\n", __FILE__, __LINE__, #cond);     \
            ++g_fail;                                                       \
        }                                                                   \
    } while (0)

static uint64_t g_rng = 0x2510037600000001ull;
static uint64_t rng() {
    g_rng = g_rng * 6364136223846793005ull + 1442695040888963407ull;
    return g_rng >> 17;
}

// Invariants of partition():
//  1. jobs of consecutive segments are consecutive, total_jobs is their sum;
//  2. n_jobs = ceil(n_groups / gpw) * n_chunks, gpw in {1, 2, 4}, gpw <= pow2_ceil(n_groups);
//     the groups are those of the population padded to full groups plus one power of two;
//  3. the tile slots of a segment's workgroups cover all its tiles;
//  4. no wavefront walks more than kMaxTilesPerWave tiles in one job (the size of the
//     kernel's per-wavefront redo list);
//  5. the launch fits the target when there is room for it (at most one job per segment
//     is forced, and the cap on tiles per wavefront can force more).
static void check_partition(const std::vector<HostSeg> &segs, uint32_t target) {
    std::vector<SegDesc> d(segs.size());
    uint32_t total = 0;
    partition(segs.data(), segs.size(), target, d.data(), total);
    uint64_t job = 0;
    bool capped = false;
    for (size_t s = 0; s < segs.size(); ++s) {
        const uint64_t te = evo::tile_elems(segs[s].dtype);
        const uint64_t tiles = (segs[s].n + te - 1) / te;
        EXPECT(d[s].job0 == job);
        EXPECT(d[s].n == segs[s].n && d[s].dtype == segs[s].dtype);
        {
            // the last group is filled up to a power of two with stand-ins: fewer of them
            // than it has real candidates
            const uint32_t rem = segs[s].P % 16, last = d[s].P % 16;
            EXPECT(d[s].P - d[s].n_pad == segs[s].P && d[s].P / 16 == segs[s].P / 16 + (rem > 8 && last == 0 ? 1 : 0));
            EXPECT((last & (last - 1)) == 0);
            EXPECT(rem == 0 ? d[s].n_pad == 0 : d[s].n_pad < rem);
            EXPECT(d[s].n_groups == segs[s].P / 16 + (rem ? 1u : 0u));
        }
        EXPECT(d[s].stats_row0 == segs[s].row0);
        EXPECT(d[s].n_groups == evo::group_count(d[s].P));
        EXPECT(d[s].gpw == 1 || d[s].gpw == 2 || d[s].gpw == 4);
        EXPECT(d[s].gpw <= pow2_ceil(d[s].n_groups));
        const uint32_t gblocks = (d[s].n_groups + d[s].gpw - 1) / d[s].gpw;
        EXPECT(d[s].n_chunks >= 1);
        EXPECT(d[s].n_jobs == gblocks * d[s].n_chunks);
        const uint64_t slots = (uint64_t)d[s].n_chunks * (evo::kWaves / d[s].gpw);
        const uint64_t steps = (tiles + slots - 1) / slots;   // tiles one wavefront walks
        EXPECT(steps >= 1 && steps <= evo::kMaxTilesPerWave);
        // the cap on tiles per wavefront decided this segment's chunk count
        const uint64_t cap_slots = (uint64_t)evo::kMaxTilesPerWave * (evo::kWaves / d[s].gpw);
        if (d[s].n_chunks > 1 && d[s].n_chunks == (tiles + cap_slots - 1) / cap_slots) capped = true;
        EXPECT(segs[s].n_cases > 1 ? d[s].case0 == segs[s].case0 : d[s].case0 == s);
        EXPECT(d[s].n_cases == segs[s].n_cases);
        job += d[s].n_jobs;
    }
    EXPECT(job == total);
    uint64_t forced = 0;   // group blocks: each needs a workgroup of its own
    for (const SegDesc &x : d) forced += (x.n_groups + x.gpw - 1) / x.gpw;
    if (!capped && forced <= target / 2) EXPECT(total <= target);
}

static void partition_cases() {
    const uint32_t targets[] = {1, 8, 64, 512, 608};
    for (int it = 0; it < 3000; ++it) {
        const uint32_t S = 1 + (uint32_t)(rng() % (it % 10 == 0 ? 700 : 9));
        std::vector<HostSeg> segs(S);
        uint32_t row0 = 0;
        for (HostSeg &h : segs) {
            const int lg = (int)(rng() % (S > 16 ? 22 : 34));
            h.n = 1 + rng() % (1ull << lg);
            const uint32_t pk = (uint32_t)(rng() % 8);
            h.P = pk == 0 ? 1 + (uint32_t)(rng() % kMaxP) : 1 + (uint32_t)(rng() % 70);
            h.dtype = (uint32_t)(rng() % 6);
            h.ref = nullptr;
            h.cand_ptrs = nullptr;
            h.row0 = row0;
            row0 += h.P;
            if (!partition_fits(&h, 1)) h.n = 1 + h.n % 4096;
        }
        if (!partition_fits(segs.data(), segs.size())) continue;
        check_partition(segs, targets[it % 5]);
    }
    // the shapes the benchmark runs: one dense tensor, one 2^30 one
    HostSeg h{};
    h.n = 1ull << 26; h.P = 16; h.dtype = EVO_F32; h.n_cases = 1;
    check_partition(std::vector<HostSeg>(1, h), 512);
    h.n = 1ull << 30; h.P = 8;
    check_partition(std::vector<HostSeg>(1, h), 512);
    h.n = 1ull << 40; h.P = kMaxP;          // too large: refused before partitioning
    EXPECT(!partition_fits(&h, 1));

    // Fold modes: a case group is folded directly only when one workgroup holds a thread per
    // (case, candidate, range) with at most kDirectRowsPerThread rows each; all cases of a
    // group get the same mode; segments outside a case group never get it.
    for (int it = 0; it < 2000; ++it) {
        const uint32_t K = 1 + (uint32_t)(rng() % 12);
        const uint32_t P = 1 + (uint32_t)(rng() % (it % 4 == 0 ? 300 : 40));
        std::vector<HostSeg> segs(K);
        for (HostSeg &c : segs) {
            c = HostSeg{};
            c.n = 1 + rng() % (1ull << (int)(rng() % 30));
            c.P = P; c.dtype = (uint32_t)(rng() % 6); c.row0 = 0; c.case0 = 0; c.n_cases = K;
        }
        if (!partition_fits(segs.data(), segs.size())) continue;
        std::vector<SegDesc> d(K);
        uint32_t total = 0;
        partition(segs.data(), K, targets[it % 5], d.data(), total);
        const uint32_t Kp = pow2_ceil(K), pc = pow2_ceil(d[0].P);
        bool fits = K > 1 && K <= evo::kDirectMaxCases && (uint64_t)Kp * pc <= (uint64_t)evo::kThreads;
        if (fits) {
            const uint32_t ranges = (uint32_t)evo::kThreads / (Kp * pc);
            for (const SegDesc &x : d) fits = fits && (x.n_chunks + ranges - 1) / ranges <= evo::kDirectRowsPerThread;
        }
        for (const SegDesc &x : d) EXPECT(x.fold_mode == (fits ? evo::kFoldCasesDirect : evo::kFoldLevels));
    }
    {
        std::vector<HostSeg> one(3);
        for (size_t i = 0; i < 3; ++i) { one[i] = HostSeg{}; one[i].n = 1000; one[i].P = 4; one[i].dtype = EVO_F32; one[i].row0 = 4 * (uint32_t)i; }
        std::vector<SegDesc> d(3);
        uint32_t total = 0;
        partition(one.data(), 3, 512, d.data(), total);
        for (const SegDesc &x : d) EXPECT(x.fold_mode == evo::kFoldLevels);
    }
}

// split_remainders(): a segment stays whole or is cut in two; the parts cover its
// candidates and rows once, in order; case groups, populations below one full group,
// multiples of the group size and short segments stay whole; 17, 33 and 65 candidates are
// cut, 100 are not.  And partition() sizes jobs by cost: of two equally long segments the
// one with 16 candidates gets 17/3 times the jobs of the one with a single candidate.
static void split_cases() {
    static const void *ptrs[70000];
    for (int it = 0; it < 2000; ++it) {
        const uint32_t S = 1 + (uint32_t)(rng() % 6);
        std::vector<HostSeg> segs(S), out;
        uint32_t row0 = 0;
        for (HostSeg &h : segs) {
            h.n = 1 + rng() % (1ull << (int)(rng() % 28));
            h.P = rng() % 4 == 0 ? 1 + (uint32_t)(rng() % kMaxP) : 1 + (uint32_t)(rng() % 70);
            h.dtype = (uint32_t)(rng() % 6);
            h.ref = ptrs;
            h.cand_ptrs = ptrs;
            h.row0 = row0;
            h.n_cases = rng() % 5 == 0 ? 3u : 1u;
            row0 += h.P;
        }
        split_remainders(segs, out);
        size_t o = 0;
        for (const HostSeg &h : segs) {
            const uint64_t te = evo::tile_elems(h.dtype);
            const bool must_stay = h.n_cases > 1 || h.P < 16 || h.P % 16 == 0 || (h.n + te - 1) / te < 1024;
            EXPECT(o < out.size());
            if (out[o].P == h.P) {
                EXPECT(out[o].row0 == h.row0 && out[o].cand_ptrs == h.cand_ptrs);
                EXPECT(out[o].n == h.n && out[o].dtype == h.dtype && out[o].n_cases == h.n_cases);
                o += 1;
            } else {
                EXPECT(!must_stay);
                EXPECT(o + 1 < out.size());
                if (o + 1 >= out.size()) break;
                const HostSeg &a = out[o], &b = out[o + 1];
                EXPECT(a.P % 16 == 0 && a.P > 0 && b.P > 0 && b.P < 16 && a.P + b.P == h.P);
                EXPECT(a.row0 == h.row0 && b.row0 == h.row0 + a.P);
                EXPECT(a.cand_ptrs == h.cand_ptrs && b.cand_ptrs == h.cand_ptrs + a.P);
                EXPECT(a.ref == h.ref && b.ref == h.ref && a.n == h.n && b.n == h.n);
                EXPECT(a.dtype == h.dtype && b.dtype == h.dtype && a.n_cases == 1 && b.n_cases == 1);
                o += 2;
            }
        }
        EXPECT(o == out.size());
    }
    {
        const uint32_t Ps[] = {17, 33, 65, 100, 49, 32, 12, 27, 20, 24};
        const size_t parts[] = {2, 2, 2, 1, 1, 1, 1, 1, 2, 1};
        for (int i = 0; i < 10; ++i) {
            HostSeg h{};
            h.n = 1ull << 24;
            h.P = Ps[i];
            h.dtype = EVO_F32;
            h.ref = ptrs;
            h.cand_ptrs = ptrs;
            h.n_cases = 1;
            std::vector<HostSeg> out;
            split_remainders(std::vector<HostSeg>(1, h), out);
            EXPECT(out.size() == parts[i]);
        }
    }
    HostSeg a{}, b{};
    a.n = b.n = 1ull << 26;
    a.dtype = b.dtype = EVO_F32;
    a.n_cases = b.n_cases = 1;
    a.P = 16;
    b.P = 1;
    b.row0 = 16;
    std::vector<HostSeg> two{a, b};
    std::vector<SegDesc> d(2);
    uint32_t total = 0;
    partition(two.data(), 2, 512, d.data(), total);
    EXPECT(total <= 512 && total >= 500);
    EXPECT(d[0].n_jobs > 5 * d[1].n_jobs && d[0].n_jobs < 6 * d[1].n_jobs);
}

static void group_cases() {
    for (uint32_t P = 1; P <= 300; ++P) {
        const uint32_t G = evo::group_count(P);
        uint32_t next = 0;
        for (uint32_t g = 0; g < G; ++g) {
            const evo::Group gr = evo::group_of(P, g);
            EXPECT(gr.cand0 == next);
            EXPECT(gr.nc >= 1 && gr.nc <= (uint32_t)evo::kG && (gr.nc & (gr.nc - 1)) == 0);
            for (uint32_t i = 0; i < gr.nc; ++i) {
                uint32_t gg = ~0u, gi = ~0u;
                evo::locate(P, gr.cand0 + i, &gg, &gi);
                EXPECT(gg == g && gi == i);
            }
            next += gr.nc;
        }
        EXPECT(next == P);
        EXPECT(evo::group_of(P, G).nc == 0);
    }
}

static void validation_cases() {
    evo_check_t *c = nullptr;
    EXPECT(evo_check_create(nullptr, EVO_F32, 16, 0.f, 0.f) == EVO_ERR_NULL);
    EXPECT(evo_check_create(&c, (evo_dtype)6, 16, 0.f, 0.f) == EVO_ERR_DTYPE && c == nullptr);
    EXPECT(evo_check_create(&c, EVO_F32, 0, 0.f, 0.f) == EVO_ERR_SIZE);
    EXPECT(evo_check_create(&c, EVO_F32, 16, -1.f, 0.f) == EVO_ERR_TOL);
    EXPECT(evo_check_create(&c, EVO_F32, 16, 0.f, __builtin_nanf("")) == EVO_ERR_TOL);
    EXPECT(evo_check_create(&c, EVO_F32, 16, __builtin_huge_valf(), 0.f) == EVO_ERR_TOL);
    EXPECT(evo_check_create(&c, EVO_F32, 1000, 1e-2f, 1e-2f) == EVO_OK && c != nullptr);

    // fake "device" addresses: validated, never dereferenced by host code
    alignas(16) static char arena[4096];
    const void *ref = arena;
    const void *cands[3] = {arena + 16, arena + 32, arena + 48};
    evo_stats *stats = reinterpret_cast<evo_stats *>(arena + 1024);
    int foreign = 0;

    EXPECT(evo_check_batch(nullptr, ref, cands, 3, nullptr, stats) == EVO_ERR_HANDLE);
    EXPECT(evo_check_batch(reinterpret_cast<evo_check_t *>(&foreign), ref, cands, 3, nullptr, stats) ==
           EVO_ERR_HANDLE);
    EXPECT(evo_check_batch(c, nullptr, cands, 3, nullptr, stats) == EVO_ERR_NULL);
    EXPECT(evo_check_batch(c, ref, nullptr, 3, nullptr, stats) == EVO_ERR_NULL);
    EXPECT(evo_check_batch(c, ref, cands, 3, nullptr, nullptr) == EVO_ERR_NULL);
    EXPECT(evo_check_batch(c, ref, cands, 0, nullptr, stats) == EVO_ERR_SIZE);
    EXPECT(evo_check_batch(c, ref, cands, 65536, nullptr, stats) == EVO_ERR_SIZE);
    EXPECT(evo_check_batch(c, arena + 2, cands, 3, nullptr, stats) == EVO_ERR_ALIGN);
    {
        evo_stats *odd = reinterpret_cast<evo_stats *>(reinterpret_cast<char *>(stats) + 4);
        evo_segment one = {ref, cands, 100, 3, EVO_F32, 0, 0};
        EXPECT(evo_check_batch(c, ref, cands, 3, nullptr, odd) == EVO_ERR_ALIGN);
        EXPECT(evo_check_segmented(c, &one, 1, nullptr, odd, 3) == EVO_ERR_ALIGN);
        EXPECT(evo_check_cases(c, &one, 1, nullptr, odd) == EVO_ERR_ALIGN);
    }
    {
        const void *bad[3] = {arena + 16, nullptr, arena + 48};
        EXPECT(evo_check_batch(c, ref, bad, 3, nullptr, stats) == EVO_ERR_NULL);
        bad[1] = arena + 33;
        EXPECT(evo_check_batch(c, ref, bad, 3, nullptr, stats) == EVO_ERR_ALIGN);
    }

    // the call that allocates nothing: the checks of evo_check_batch, plus its capacity
    EXPECT(evo_check_batch_static(nullptr, ref, cands, 3, nullptr, stats) == EVO_ERR_HANDLE);
    EXPECT(evo_check_batch_static(c, nullptr, cands, 3, nullptr, stats) == EVO_ERR_NULL);
    EXPECT(evo_check_batch_static(c, ref, cands, 3, nullptr, nullptr) == EVO_ERR_NULL);
    EXPECT(evo_check_batch_static(c, ref, cands, 0, nullptr, stats) == EVO_ERR_SIZE);
    EXPECT(evo_check_batch_static(c, arena + 2, cands, 3, nullptr, stats) == EVO_ERR_ALIGN);
    {
        std::vector<const void *> many(385, arena + 64);
        EXPECT(evo_check_batch_static(c, ref, many.data(), 385, nullptr, stats) == EVO_ERR_LIMIT);
    }

    // tolerance policy
    EXPECT(evo_check_set_tolerance(nullptr, EVO_F32, 0.f, 0.f) == EVO_ERR_HANDLE);
    EXPECT(evo_check_set_tolerance(c, (evo_dtype)6, 0.f, 0.f) == EVO_ERR_DTYPE);
    EXPECT(evo_check_set_tolerance(c, EVO_BF16, -1.f, 0.f) == EVO_ERR_TOL);
    EXPECT(evo_check_set_tolerance(c, EVO_BF16, 0.f, __builtin_huge_valf()) == EVO_ERR_TOL);
    EXPECT(evo_check_set_tolerance_class(nullptr, 1, 0.f, 0.f) == EVO_ERR_HANDLE);
    EXPECT(evo_check_set_tolerance_class(c, 0, 0.f, 0.f) == EVO_ERR_SIZE);
    EXPECT(evo_check_set_tolerance_class(c, EVO_TOL_CLASSES + 1, 0.f, 0.f) == EVO_ERR_SIZE);
    EXPECT(evo_check_set_tolerance_class(c, 2, __builtin_nanf(""), 0.f) == EVO_ERR_TOL);
    {
        evo_segment one = {ref, cands, 100, 3, EVO_F32, 0, 3};          // class 3 was never set
        EXPECT(evo_check_segmented(c, &one, 1, nullptr, stats, 3) == EVO_ERR_TOL);
        EXPECT(evo_check_cases(c, &one, 1, nullptr, stats) == EVO_ERR_TOL);
        one.tol_class = EVO_TOL_CLASSES + 1;
        EXPECT(evo_check_segmented(c, &one, 1, nullptr, stats, 3) == EVO_ERR_TOL);
    }

    evo_segment seg[2] = {{ref, cands, 100, 3, EVO_F32, 0, 0}, {ref, cands, 7, 2, EVO_BF16, 3, 0}};
    EXPECT(evo_check_segmented(nullptr, seg, 2, nullptr, stats, 5) == EVO_ERR_HANDLE);
    EXPECT(evo_check_segmented(c, nullptr, 2, nullptr, stats, 5) == EVO_ERR_NULL);
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, nullptr, 5) == EVO_ERR_NULL);
    EXPECT(evo_check_segmented(c, seg, 0, nullptr, stats, 5) == EVO_ERR_SIZE);
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 0) == EVO_ERR_SIZE);
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 4) == EVO_ERR_SIZE);   // rows past n_rows
    seg[1].stats_row0 = 2;                                                        // overlap
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 5) == EVO_ERR_SIZE);
    seg[1].stats_row0 = 3;
    seg[1].dtype = 9;
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 5) == EVO_ERR_DTYPE);
    seg[1].dtype = EVO_F16;
    seg[1].n_elems = 0;
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 5) == EVO_ERR_SIZE);
    seg[1].n_elems = 7;
    seg[1].P_s = 0;
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 5) == EVO_ERR_SIZE);
    seg[1].P_s = 2;
    seg[1].stats_row0 = 0xffffffffu;   // lo + P_s must not wrap
    EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 5) == EVO_ERR_SIZE);
    seg[1].stats_row0 = 3;

    evo_segment cs[2] = {{ref, cands, 100, 3, EVO_F32, 0, 0}, {ref, cands, 50, 3, EVO_F16, 0, 0}};
    EXPECT(evo_check_cases(nullptr, cs, 2, nullptr, stats) == EVO_ERR_HANDLE);
    EXPECT(evo_check_cases(c, nullptr, 2, nullptr, stats) == EVO_ERR_NULL);
    EXPECT(evo_check_cases(c, cs, 2, nullptr, nullptr) == EVO_ERR_NULL);
    EXPECT(evo_check_cases(c, cs, 0, nullptr, stats) == EVO_ERR_SIZE);
    cs[1].P_s = 2;
    EXPECT(evo_check_cases(c, cs, 2, nullptr, stats) == EVO_ERR_SIZE);
    cs[1].P_s = 3;
    cs[1].stats_row0 = 1;
    EXPECT(evo_check_cases(c, cs, 2, nullptr, stats) == EVO_ERR_SIZE);
    cs[1].stats_row0 = 0;

    const float *tim = reinterpret_cast<const float *>(arena + 2048);
    const float *base = reinterpret_cast<const float *>(arena + 3072);
    evo_pop_summary *pop = reinterpret_cast<evo_pop_summary *>(arena + 3584);
    EXPECT(evo_fitness(nullptr, tim, base, 3, 5, nullptr, stats, pop) == EVO_ERR_HANDLE);
    EXPECT(evo_fitness(c, nullptr, base, 3, 5, nullptr, stats, pop) == EVO_ERR_NULL);
    EXPECT(evo_fitness(c, tim, nullptr, 3, 5, nullptr, stats, pop) == EVO_ERR_NULL);
    EXPECT(evo_fitness(c, tim, base, 3, 5, nullptr, nullptr, pop) == EVO_ERR_NULL);
    EXPECT(evo_fitness(c, tim, base, 0, 5, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_fitness(c, tim, base, 3, 0, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_fitness(c, tim, base, 3, EVO_FITNESS_MAX_T + 1, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_fitness(c, tim, base, (1u << 20) + 1, 5, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_fitness(c, reinterpret_cast<const float *>(arena + 2050), base, 3, 5, nullptr, stats,
                       pop) == EVO_ERR_ALIGN);
    EXPECT(evo_fitness(c, tim, base, 3, 5, nullptr, reinterpret_cast<evo_stats *>(arena + 1028), pop) ==
           EVO_ERR_ALIGN);
    EXPECT(evo_fitness_ex(c, tim, base, 3, 5, 2, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_fitness_ex(nullptr, tim, base, 3, 5, EVO_REDUCE_MEAN, nullptr, stats, pop) == EVO_ERR_HANDLE);
    EXPECT(evo_fitness_ex(c, tim, nullptr, 3, 5, EVO_REDUCE_MEAN, nullptr, stats, pop) == EVO_ERR_NULL);
    {   // 8-byte element types need 8-byte aligned tensors
        evo_check_t *c64 = nullptr;
        EXPECT(evo_check_create(&c64, EVO_F64, 100, 0.f, 0.f) == EVO_OK);
        const void *c4[1] = {arena + 20};
        EXPECT(evo_check_batch(c64, ref, c4, 1, nullptr, stats) == EVO_ERR_ALIGN);
        EXPECT(evo_check_batch(c64, arena + 4, cands, 1, nullptr, stats) == EVO_ERR_ALIGN);
        EXPECT(evo_check_destroy(c64) == EVO_OK);
    }

    uint32_t *elite = reinterpret_cast<uint32_t *>(arena + 3600);
    EXPECT(evo_select_elite(nullptr, stats, 3, 2, nullptr, elite, nullptr) == EVO_ERR_HANDLE);
    EXPECT(evo_select_elite(c, nullptr, 3, 2, nullptr, elite, nullptr) == EVO_ERR_NULL);
    EXPECT(evo_select_elite(c, stats, 3, 2, nullptr, nullptr, nullptr) == EVO_ERR_NULL);
    EXPECT(evo_select_elite(c, stats, 0, 1, nullptr, elite, nullptr) == EVO_ERR_SIZE);
    EXPECT(evo_select_elite(c, stats, 3, 0, nullptr, elite, nullptr) == EVO_ERR_SIZE);
    EXPECT(evo_select_elite(c, stats, 3, 4, nullptr, elite, nullptr) == EVO_ERR_SIZE);
    EXPECT(evo_select_elite(c, stats, 65536, 4, nullptr, elite, nullptr) == EVO_ERR_SIZE);
    EXPECT(evo_select_elite(c, stats, 3, 2, nullptr, reinterpret_cast<uint32_t *>(arena + 3602),
                            nullptr) == EVO_ERR_ALIGN);

    {
        const uint32_t *keys = reinterpret_cast<const uint32_t *>(arena + 3700);
        EXPECT(evo_select_elite_diverse(nullptr, stats, keys, 3, 2, nullptr, elite, nullptr) == EVO_ERR_HANDLE);
        EXPECT(evo_select_elite_diverse(c, stats, nullptr, 3, 2, nullptr, elite, nullptr) == EVO_ERR_NULL);
        EXPECT(evo_select_elite_diverse(c, nullptr, keys, 3, 2, nullptr, elite, nullptr) == EVO_ERR_NULL);
        EXPECT(evo_select_elite_diverse(c, stats, keys, 3, 0, nullptr, elite, nullptr) == EVO_ERR_SIZE);
        EXPECT(evo_select_elite_diverse(c, stats, keys, 3, 4, nullptr, elite, nullptr) == EVO_ERR_SIZE);
        EXPECT(evo_select_elite_diverse(c, stats, reinterpret_cast<const uint32_t *>(arena + 3701), 3, 2,
                                        nullptr, elite, nullptr) == EVO_ERR_ALIGN);
    }

    // evaluation in one call
    EXPECT(evo_evaluate(nullptr, cs, 2, tim, base, 5, 0, nullptr, stats, pop) == EVO_ERR_HANDLE);
    EXPECT(evo_evaluate(c, nullptr, 2, tim, base, 5, 0, nullptr, stats, pop) == EVO_ERR_NULL);
    EXPECT(evo_evaluate(c, cs, 2, nullptr, base, 5, 0, nullptr, stats, pop) == EVO_ERR_NULL);
    EXPECT(evo_evaluate(c, cs, 2, tim, nullptr, 5, 0, nullptr, stats, pop) == EVO_ERR_NULL);
    EXPECT(evo_evaluate(c, cs, 2, tim, base, 5, 0, nullptr, nullptr, pop) == EVO_ERR_NULL);
    EXPECT(evo_evaluate(c, cs, 0, tim, base, 5, 0, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_evaluate(c, cs, 2, tim, base, 0, 0, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_evaluate(c, cs, 2, tim, base, EVO_FITNESS_MAX_T + 1, 0, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_evaluate(c, cs, 2, tim, base, 5, 7, nullptr, stats, pop) == EVO_ERR_SIZE);
    EXPECT(evo_evaluate(c, cs, 2, reinterpret_cast<const float *>(arena + 2050), base, 5, 0, nullptr, stats,
                        pop) == EVO_ERR_ALIGN);
    cs[1].P_s = 2;
    EXPECT(evo_evaluate(c, cs, 2, tim, base, 5, 0, nullptr, stats, pop) == EVO_ERR_SIZE);
    cs[1].P_s = 3;

    {   // ragged evaluation in one call
        evo_segment sg[2] = {{ref, cands, 100, 3, EVO_F32, 0, 0}, {ref, cands, 7, 2, EVO_BF16, 3, 0}};
        EXPECT(evo_evaluate_segmented(nullptr, sg, 2, tim, base, 5, 0, nullptr, stats, 5, pop) == EVO_ERR_HANDLE);
        EXPECT(evo_evaluate_segmented(c, nullptr, 2, tim, base, 5, 0, nullptr, stats, 5, pop) == EVO_ERR_NULL);
        EXPECT(evo_evaluate_segmented(c, sg, 2, nullptr, base, 5, 0, nullptr, stats, 5, pop) == EVO_ERR_NULL);
        EXPECT(evo_evaluate_segmented(c, sg, 2, tim, nullptr, 5, 0, nullptr, stats, 5, pop) == EVO_ERR_NULL);
        EXPECT(evo_evaluate_segmented(c, sg, 2, tim, base, 5, 0, nullptr, nullptr, 5, pop) == EVO_ERR_NULL);
        EXPECT(evo_evaluate_segmented(c, sg, 0, tim, base, 5, 0, nullptr, stats, 5, pop) == EVO_ERR_SIZE);
        EXPECT(evo_evaluate_segmented(c, sg, 2, tim, base, 0, 0, nullptr, stats, 5, pop) == EVO_ERR_SIZE);
        EXPECT(evo_evaluate_segmented(c, sg, 2, tim, base, 5, 3, nullptr, stats, 5, pop) == EVO_ERR_SIZE);
        EXPECT(evo_evaluate_segmented(c, sg, 2, tim, base, 5, 0, nullptr, stats, 4, pop) == EVO_ERR_SIZE);
        EXPECT(evo_evaluate_segmented(c, sg, 2, tim, base, 5, 0, nullptr, stats, 6, pop) ==
               EVO_ERR_SIZE);   // row 5 belongs to no group
        sg[1].stats_row0 = 2;   // overlap
        EXPECT(evo_evaluate_segmented(c, sg, 2, tim, base, 5, 0, nullptr, stats, 5, pop) == EVO_ERR_SIZE);
        sg[1].stats_row0 = 3;
        EXPECT(evo_evaluate_segmented(c, sg, 2, reinterpret_cast<const float *>(arena + 2050), base, 5, 0,
                                      nullptr, stats, 5, pop) == EVO_ERR_ALIGN);
        // valid arguments reach the device layer (absent where this test runs)
        const int rcv = evo_evaluate_segmented(c, sg, 2, tim, base, 5, 0, nullptr, stats, 5, pop);
        EXPECT(rcv == EVO_OK || rcv == EVO_ERR_DEVICE);
    }

    {   // timing stage
        static int calls = 0;
        const evo_launch_fn fns[2] = {[](void *, void *) { ++calls; }, [](void *, void *) { ++calls; }};
        const evo_launch_fn holes[2] = {fns[0], nullptr};
        const evo_timing_opts opts = {2, 0, {0, 0}};
        const evo_timing_opts silly = {2000000, 0, {0, 0}};
        float *tab = reinterpret_cast<float *>(arena + 2048);
        EXPECT(evo_time_candidates(nullptr, fns, nullptr, 2, 5, &opts, nullptr, tab, nullptr) == EVO_ERR_HANDLE);
        EXPECT(evo_time_candidates(c, nullptr, nullptr, 2, 5, &opts, nullptr, tab, nullptr) == EVO_ERR_NULL);
        EXPECT(evo_time_candidates(c, holes, nullptr, 2, 5, &opts, nullptr, tab, nullptr) == EVO_ERR_NULL);
        EXPECT(evo_time_candidates(c, fns, nullptr, 2, 5, nullptr, nullptr, tab, nullptr) == EVO_ERR_NULL);
        EXPECT(evo_time_candidates(c, fns, nullptr, 2, 5, &opts, nullptr, nullptr, nullptr) == EVO_ERR_NULL);
        EXPECT(evo_time_candidates(c, fns, nullptr, 0, 5, &opts, nullptr, tab, nullptr) == EVO_ERR_SIZE);
        EXPECT(evo_time_candidates(c, fns, nullptr, 2, 0, &opts, nullptr, tab, nullptr) == EVO_ERR_SIZE);
        EXPECT(evo_time_candidates(c, fns, nullptr, 2, EVO_FITNESS_MAX_T + 1, &opts, nullptr, tab, nullptr) ==
               EVO_ERR_SIZE);
        EXPECT(evo_time_candidates(c, fns, nullptr, 2, 5, &silly, nullptr, tab, nullptr) == EVO_ERR_SIZE);
        EXPECT(evo_time_candidates(c, fns, nullptr, 2, 5, &opts, nullptr,
                                   reinterpret_cast<float *>(arena + 2050), nullptr) == EVO_ERR_ALIGN);
        EXPECT(evo_time_candidates(c, fns, nullptr, 2, 5, &opts, nullptr, tab,
                                   reinterpret_cast<float *>(arena + 2050)) == EVO_ERR_ALIGN);
        EXPECT(calls == 0);
    }

    EXPECT(evo::g_launches == 0);   // nothing above got past validation

    // Valid arguments.  Without a device HIP refuses and the call reports it; with one,
    // scratch is allocated and the (stubbed) launcher is reached.  Either way nothing
    // may leak or be touched out of bounds.
    const int rc1 = evo_check_batch(c, ref, cands, 3, nullptr, stats);
    EXPECT(rc1 == EVO_OK || rc1 == EVO_ERR_DEVICE);
    const int rc2 = evo_check_segmented(c, seg, 2, nullptr, stats, 5);
    EXPECT(rc2 == rc1);
    if (rc1 == EVO_OK) {
        // every group is launched with the tolerance of its element type, or of its class
        EXPECT(evo::g_last_atol[0] == 1e-2f && evo::g_last_rtol[1] == 1e-2f);
        EXPECT(evo_check_set_tolerance(c, EVO_BF16, 0.5f, 0.25f) == EVO_OK);
        EXPECT(evo_check_set_tolerance_class(c, 7, 3.0f, 0.0f) == EVO_OK);
        EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 5) == EVO_OK);
        EXPECT(evo::g_last_atol[0] == 1e-2f && evo::g_last_rtol[0] == 1e-2f);
        EXPECT(evo::g_last_atol[1] == 0.5f && evo::g_last_rtol[1] == 0.25f);
        seg[0].tol_class = 7;
        EXPECT(evo_check_segmented(c, seg, 2, nullptr, stats, 5) == EVO_OK);
        EXPECT(evo::g_last_atol[0] == 3.0f && evo::g_last_rtol[0] == 0.0f && evo::g_last_atol[1] == 0.5f);
        seg[0].tol_class = 0;
    }
    const int rc3 = evo_check_cases(c, cs, 2, nullptr, stats);
    EXPECT(rc3 == rc1);
    if (rc1 == EVO_OK) {
        // more groups and pointers than the argument block holds: the staged-table path
        std::vector<const void *> many(400, arena + 64);
        std::vector<evo_segment> big(12);
        uint32_t row = 0;
        for (evo_segment &s : big) {
            s = evo_segment{ref, many.data(), 33, 400, EVO_F32, row, 0};
            row += 400;
        }
        EXPECT(evo_check_segmented(c, big.data(), 12, nullptr, stats, row) == EVO_OK);
        EXPECT(evo_check_segmented(c, big.data(), 12, nullptr, stats, row) == EVO_OK);
    }
    const int rc4 = evo_fitness(c, tim, base, 3, 5, nullptr, stats, pop);
    EXPECT(rc4 == rc1);
    const int rc5 = evo_select_elite(c, stats, 3, 2, nullptr, elite, nullptr);
    EXPECT(rc5 == rc1);
    std::printf("san_api: device calls %s\n", rc1 == EVO_OK ? "reached the launchers" : "refused (no device)");

    EXPECT(evo_check_destroy(c) == EVO_OK || rc1 != EVO_OK);
    EXPECT(evo_check_destroy(c) == EVO_ERR_HANDLE);        // already destroyed
    EXPECT(evo_check_destroy(nullptr) == EVO_ERR_HANDLE);
    EXPECT(evo_check_batch(c, ref, cands, 3, nullptr, stats) == EVO_ERR_HANDLE);

    for (int code = 1; code >= -12; --code) EXPECT(evo_strerror(code) != nullptr && evo_strerror(code)[0]);
}

int main() {
    group_cases();
    partition_cases();
    split_cases();
    validation_cases();
    std::puts(g_fail ? "san_api: FAILED" : "san_api: ok");
    return g_fail ? 1 : 0;
}
