"""GPU parity at the full sizes of the five workloads, through the same entry points and
launch configuration that bench.py times.  Every row is compared with the CPU oracle
(large tensors are copied to the host and fed to the oracle in chunks)."""
import time

import pytest
import torch

pytestmark = pytest.mark.gpu

import synth  # noqa: E402


@pytest.fixture(scope="module")
def gu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def _say(msg):
    print(msg, flush=True)


def _full(gu, w, label):
    t0 = time.time()
    _say("%s: generated %s, checking on the GPU and on the CPU oracle" % (label, w.name))
    chk, stats, want = gu.check_parity(w, label=label)
    _say("%s: check rows agree (%.1f s), fitness" % (label, time.time() - t0))
    got, pop, fit = gu.fitness_parity(chk, stats, w.timings, w.baseline, label=label)
    if len(w.segments) == 1:
        # the entry point bench.py times for this workload: same bytes from one launch
        import paper_2510_03760_amd as evo
        seg = w.segments[0]
        one = chk.new_stats(w.P)
        one.fill_(0xAB)
        one_sum = chk.new_summary()
        chk.evaluate([{"ref": seg.ref, "cand_ptrs": seg.cands, "n_elems": seg.n, "dtype": gu.dtype_code(seg)}],
                     w.timings, w.baseline, one, one_sum)
        two_sum = chk.new_summary()
        chk.fitness(w.timings, w.baseline, stats, two_sum)
        torch.cuda.synchronize()
        assert torch.equal(one, stats) and torch.equal(one_sum, two_sum), label
        _say("%s: evo_evaluate gives the same bytes" % label)
    else:
        # likewise for the ragged workload: evo_evaluate_segmented
        row0, descs = 0, []
        for seg in w.segments:
            descs.append({"ref": seg.ref, "cand_ptrs": seg.cands, "n_elems": seg.n,
                          "dtype": gu.dtype_code(seg), "stats_row0": row0})
            row0 += len(seg.cands)
        one = chk.new_stats(w.P)
        one.fill_(0xAB)
        one_sum = chk.new_summary()
        chk.evaluate_segmented(descs, w.timings, w.baseline, one, w.P, one_sum)
        two_sum = chk.new_summary()
        chk.fitness(w.timings, w.baseline, stats, two_sum)
        torch.cuda.synchronize()
        assert torch.equal(one, stats) and torch.equal(one_sum, two_sum), label
        _say("%s: evo_evaluate_segmented gives the same bytes" % label)
    chk.close()
    return want, pop


def test_config2_full(gu):
    w = synth.dense_f32("cuda", side=8192, P=16, T=100)
    want, pop = _full(gu, w, "C2")
    seg = w.segments[0]
    for p, r in enumerate(want):
        if seg.corrupted[p]:
            k = seg.notes["replaced"][p]
            assert 0.98 * k <= r["n_mismatch"] <= k
        else:
            assert r["n_mismatch"] == 0
    assert int(pop["n_valid"]) == 12


def test_config3_full(gu):
    w = synth.softmax_bf16("cuda", B=32, R=128, C=4096, P=64, T=100)
    want, pop = _full(gu, w, "C3")
    assert [r["valid"] for r in want] == [0 if (p % 8) == 7 else 1 for p in range(64)]
    assert int(pop["n_valid"]) == 56


def test_config4_full(gu):
    w = synth.ragged_f32("cuda", P_s=32, T=100)
    want, pop = _full(gu, w, "C4")
    assert sum(r["valid"] for r in want) == 192 and int(pop["n_valid"]) == 192
    assert sorted(set(r["n_elems"] for r in want)) == sorted(
        [12845056, 16777216, 128, 1048576, 1204224, 262144, 2097152, 1000])


def test_config5_full(gu):
    w = synth.heavy_tail_f32("cuda", log2n=30, P=8, T=1000)
    want, pop = _full(gu, w, "C5")
    k = w.segments[0].notes["n_ref_nan"]
    assert k == 1024
    assert [r["n_mismatch"] for r in want] == [k, k, 2 * k, k, k, 2 * k, 3 * k, k]
    assert int(pop["n_valid"]) == 0 and int(pop["best_idx"]) == 8


@pytest.mark.parametrize("name", ["f64", "i32", "i64"])
def test_config7_full(gu, name):
    dt = {"f64": torch.float64, "i32": torch.int32, "i64": torch.int64}[name]
    w = synth.dense_typed("cuda", dt, n=(1 << 26) if name == "i32" else (1 << 25), P=16, T=100)
    want, pop = _full(gu, w, "C7-" + name)
    assert [r["valid"] for r in want] == [0 if (p % 4) == 3 else 1 for p in range(16)]
    assert int(pop["n_valid"]) == 12


@pytest.mark.timeout(600)
def test_more_than_two_to_the_32_elements(gu):
    """Element indices beyond 32 bits: 2^32 + 12345 bf16 elements per tensor (8.6 GB each), two
    candidates, with the differences that matter placed behind element 2^32 -- a far value, a
    NaN in the very last element, an Inf in the ragged last tile -- and one just before it.
    Every row against the CPU oracle, fed chunk by chunk; n_elems needs its high word."""
    free, _ = torch.cuda.mem_get_info()
    n = (1 << 32) + 12345
    if free < 4 * 2 * n:
        pytest.skip("needs 35 GB of free device memory")
    t0 = time.time()
    g = torch.Generator(device="cuda")
    g.manual_seed(0x5EED2032)
    ref = torch.empty(n, dtype=torch.bfloat16, device="cuda")
    step = 1 << 28
    for lo in range(0, n, step):                       # piecewise: no fp32 temporary of the whole tensor
        hi = min(n, lo + step)
        ref[lo:hi] = (torch.randn(hi - lo, generator=g, device="cuda") + 2).to(torch.bfloat16)
    near = ref.clone()
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        near[lo:hi] = (near[lo:hi].float() * 1.003).to(torch.bfloat16)
    edge = ref.clone()
    edge[(1 << 32) - 1] = 50.0
    edge[(1 << 32) + 5] = -50.0
    edge[n - 1] = float("nan")
    edge[n - 300] = float("inf")
    _say("2^32+: tensors generated (%.1f s)" % (time.time() - t0))
    seg = synth.Segment(ref, [near, edge], (n,), [True, False])
    w = synth.Workload("beyond-2^32-bf16-P2", [seg], 1e-2, 1e-2, 1 + torch.rand(2, 8, device="cuda"),
                       1 + torch.rand(8, device="cuda"))
    chk, stats, want = gu.check_parity(w, oracle_threads=2, label="2^32+")
    _say("2^32+: rows agree (%.1f s)" % (time.time() - t0))
    assert want[0]["valid"] == 1 and want[0]["n_finite"] == n
    assert want[1]["n_mismatch"] == 4 and want[1]["n_finite"] == n - 2
    from paper_2510_03760_amd.binding import stats_to_numpy
    got = stats_to_numpy(stats)
    assert int(got[0]["n_elems_hi"]) == 1 and int(got[0]["n_elems_lo"]) == 12345
    chk.close()
    del ref, near, edge, seg, w
    torch.cuda.empty_cache()
