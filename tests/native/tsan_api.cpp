// ThreadSanitizer driver for the host side of the C ABI: contexts are created, used (argument
// errors and, where HIP has no device, the device error path) and destroyed from several
// threads at once; the registry of live handles is the shared state.  Built by
// tests/test_host_sanitizers.py with the host pass under -fsanitize=thread; the kernel
// launchers are stubbed out as in san_api.cpp.
#include "../../paper_2510_03760_amd/csrc/evo_api.hip"

#include <atomic>
#include <cstdio>
#include <thread>

namespace evo {
hipError_t launch_check(uint32_t, const SegDesc *, const uint64_t *, uint32_t, uint32_t,
                        uint32_t, Partial *, uint32_t *, evo_stats *, hipStream_t) { return hipSuccess; }
hipError_t launch_check_inline(uint32_t, const InlineTable &, uint32_t, uint32_t, uint32_t,
                               Partial *, uint32_t *, evo_stats *, hipStream_t) { return hipSuccess; }
hipError_t launch_evaluate(uint32_t, const InlineTable &, uint32_t, uint32_t, uint32_t, Partial *,
                           uint32_t *, evo_stats *, const FitLaunch &, hipStream_t) { return hipSuccess; }
hipError_t launch_fitness(const float *, const float *, uint32_t, uint32_t, uint32_t, evo_stats *,
                          evo_pop_summary *, float *, uint32_t *, hipStream_t) { return hipSuccess; }
hipError_t launch_select(const evo_stats *, uint32_t, uint32_t, uint32_t *, uint32_t *, hipStream_t) { return hipSuccess; }
hipError_t launch_select_diverse(const evo_stats *, const uint32_t *, uint32_t *, uint32_t, uint32_t, uint32_t *,
                                 uint32_t *, hipStream_t) { return hipSuccess; }
hipError_t launch_flush(void *, size_t, uint32_t, hipStream_t) { return hipSuccess; }
hipError_t launch_probe(float *, uint32_t, hipStream_t) { return hipSuccess; }
}  // namespace evo

static std::atomic<int> g_fail{0};
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAIL line %d: %s\n", __LINE__, #cond); ++g_fail; } } while (0)

static void worker(int id, evo_check_t **shared_slot) {
    alignas(16) static char arena[256];
    const void *cands[2] = {arena + 16, arena + 32};
    evo_stats *stats = reinterpret_cast<evo_stats *>(arena + 64);
    for (int it = 0; it < 300; ++it) {
        evo_check_t *c = nullptr;
        EXPECT(evo_check_create(&c, (evo_dtype)(it % 6), 100 + id, 1e-2f, 1e-2f) == EVO_OK);
        EXPECT(evo_check_batch(c, nullptr, cands, 2, nullptr, stats) == EVO_ERR_NULL);
        EXPECT(evo_check_batch(c, arena, cands, 0, nullptr, stats) == EVO_ERR_SIZE);
        const int rc = evo_check_batch(c, arena, cands, 2, nullptr, stats);   // own context: allowed
        EXPECT(rc == EVO_OK || rc == EVO_ERR_DEVICE);
        // a handle that belongs to the main thread, looked up while the others change the registry
        evo_check_t *other = *shared_slot;
        const int ro = evo_check_batch(other, arena, cands, 0, nullptr, stats);
        EXPECT(ro == EVO_ERR_SIZE || ro == EVO_ERR_HANDLE);
        EXPECT(evo_check_destroy(c) == EVO_OK || rc == EVO_ERR_DEVICE);
        EXPECT(evo_check_destroy(c) == EVO_ERR_HANDLE);
    }
}

int main() {
    evo_check_t *shared = nullptr;
    EXPECT(evo_check_create(&shared, EVO_F32, 10, 0.f, 0.f) == EVO_OK);
    evo_check_t *slot = shared;
    std::thread th[4];
    for (int i = 0; i < 4; ++i) th[i] = std::thread(worker, i, &slot);
    for (auto &t : th) t.join();
    EXPECT(evo_check_destroy(shared) == EVO_OK);
    std::puts(g_fail ? "tsan_api: FAILED" : "tsan_api: ok");
    return g_fail ? 1 : 0;
}
