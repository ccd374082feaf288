"""The timing stage on a GPU: evo_time_candidates drives real kernels (here: matrix products
and a cache-sized copy enqueued by PyTorch on the stream it is handed), and its table is
checked for plausibility against PyTorch's own event timing, then fed to evo_fitness and
compared with the oracle.  A measurement has no oracle; what can be checked exactly is what
is done with it."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _say(msg):
    print(msg, flush=True)


def _torch_time_ms(fn, reps=20):
    for _ in range(3):
        fn()
    torch.cuda.synchronize()
    # all runs enqueued back to back, as the library does it: with a synchronisation per run
    # the bracket of a short kernel is mostly the launch latency of an empty queue
    pairs = []
    for _ in range(reps):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in pairs]))


def test_timing_table_is_plausible_and_feeds_fitness(gu):
    _say("timing stage")
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy
    sizes = [512, 1024, 2048, 1024]
    mats = [(torch.randn(s, s, device="cuda"), torch.randn(s, s, device="cuda"),
             torch.empty(s, s, device="cuda")) for s in sizes]
    calls = [0] * len(sizes)
    stream = torch.cuda.current_stream()

    def make(i):
        a, b, c = mats[i]

        def launch(stream_ptr):
            assert (stream_ptr or 0) == (stream.cuda_stream or 0)
            calls[i] += 1
            torch.mm(a, b, out=c)
        return launch

    launches = [make(i) for i in range(len(sizes))]
    P, T, W = len(sizes), 20, 3
    chk = evo.Checker(evo.EVO_F32, 16, 1e-2, 1e-2)
    timings = torch.full((P, T), -1.0, device="cuda")
    ratios = chk.time_candidates(launches, T, timings, warmup=W)
    torch.cuda.synchronize()
    t = timings.cpu().numpy()
    assert calls == [W + T] * P
    assert np.all(np.isfinite(t)) and np.all(t > 0)
    med = np.median(t, axis=1)
    _say("medians (ms): %s   clock ratios: %s" % (np.round(med, 4).tolist(), np.round(ratios, 3).tolist()))
    assert med[0] < med[1] < med[2]                        # 8x the work per step
    assert 0.5 < med[3] / med[1] < 2.0                      # the same kernel twice
    # against the same bracket taken with PyTorch's events: a bracket that counted a run twice,
    # or took the cache flush or a neighbouring run in, would be off by far more than this band
    for i, (lo, hi) in ((1, (0.7, 1.4)), (2, (0.7, 1.4))):
        a, b, c = mats[i]
        ref_ms = _torch_time_ms(lambda: torch.mm(a, b, out=c))
        assert lo < med[i] / ref_ms < hi, (i, med[i], ref_ms)
    assert len(ratios) == P and all(0.5 < r < 2.0 for r in ratios)

    # the table is the input of evo_fitness: candidate 1 is the baseline here
    stats = chk.new_stats(P)
    view = stats.view(P, 72)
    valid = np.array([1, 1, 0, 1], np.uint32)
    view[:, 44:48] = torch.from_numpy(valid.view(np.uint8).copy()).to("cuda").view(P, 4)
    summary = chk.new_summary()
    base = timings[1].clone()
    chk.fitness(timings, base, stats, summary)
    torch.cuda.synchronize()
    got = stats_to_numpy(stats)
    want = oracle.fitness(t, t[1], valid)
    for f in ("median_ms", "mean_ms", "speedup", "fitness"):
        assert got[f].tobytes() == want[f].tobytes(), f
    assert int(summary_to_numpy(summary)[0]["best_idx"]) == want["best_idx"] == 0
    assert float(got["speedup"][1]) == 1.0 and float(got["fitness"][2]) == 0.0
    chk.close()


def test_cache_flush_shows_in_the_timings(gu):
    """A kernel whose 64 MiB input fits the last-level cache: flushed runs must not be
    faster than unflushed ones (and are normally clearly slower)."""
    _say("timing stage, flush")
    import paper_2510_03760_amd as evo
    src = torch.randn(16 << 20, device="cuda")          # 64 MiB
    dst = torch.empty_like(src)
    launches = [lambda st: dst.copy_(src)]
    chk = evo.Checker(evo.EVO_F32, 16, 1e-2, 1e-2)
    tw = torch.zeros(1, 30, device="cuda")
    tc = torch.zeros(1, 30, device="cuda")
    chk.time_candidates(launches, 30, tw, warmup=3, flush_cache=False)
    chk.time_candidates(launches, 30, tc, warmup=3, flush_cache=True)
    chk.time_candidates(launches, 7, tw[:, :7].contiguous(), warmup=0, flush_cache=False)   # reuse, smaller
    torch.cuda.synchronize()
    warm, cold = float(tw.median()), float(tc.median())
    _say("64 MiB copy: %.4f ms warm, %.4f ms after a flush" % (warm, cold))
    assert warm > 0 and cold > 0.9 * warm
    chk.close()


def test_errors_on_live_device(gu):
    import ctypes
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import LAUNCH_FN, EvoTimingOpts
    chk = evo.Checker(evo.EVO_F32, 16, 1e-2, 1e-2)
    t = torch.zeros(2, 4, device="cuda")
    fn = LAUNCH_FN(lambda u, s: None)
    fns = (LAUNCH_FN * 2)(fn, fn)
    opts = EvoTimingOpts(0, 0)
    call = evo.lib.evo_time_candidates
    assert call(chk.ctx, fns, None, 2, 0, ctypes.byref(opts), None, t.data_ptr(), None) == -3
    assert call(chk.ctx, fns, None, 2, 4, None, None, t.data_ptr(), None) == -1
    assert call(chk.ctx, fns, None, 2, 4, ctypes.byref(opts), None, t.data_ptr() + 2, None) == -5
    assert call(chk.ctx, fns, None, 2, 4, ctypes.byref(opts), None, t.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert bool((t >= 0).all())
    chk.close()
