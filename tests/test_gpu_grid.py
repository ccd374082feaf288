"""No result may depend on how a launch is cut into jobs.  The build links the same kernels a
second time behind host code that plans three workgroups per compute unit instead of two
(libevo_grid3.so: other chunk counts, other fold trees, more jobs than the GPU holds at once);
the same populations go through both libraries and the oracle: integers, flags and maxima are
the oracle's byte for byte under either plan, the two error sums within 1e-6."""
import ctypes

import numpy as np
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


@pytest.fixture(scope="module")
def alt():
    from paper_2510_03760_amd import binding, build
    return binding.load_library(build.GRID_VARIANT_PATH)


def _say(msg):
    print(msg, flush=True)


def _rows_with(lib, segs, atol, rtol, n_rows):
    """evo_check_segmented of `lib` on the segments; returns the rows as a structured array."""
    from paper_2510_03760_amd import binding
    import gpu_util
    out = ctypes.c_void_p()
    assert lib.evo_check_create(ctypes.byref(out), gpu_util.dtype_code(segs[0]), segs[0].n, atol, rtol) == 0
    stats = torch.full((n_rows * 72,), 0xAB, dtype=torch.uint8, device="cuda")
    row0, descs = 0, []
    for s in segs:
        descs.append({"ref": s.ref, "cand_ptrs": s.cands, "n_elems": s.n, "dtype": gpu_util.dtype_code(s),
                      "stats_row0": row0})
        row0 += len(s.cands)
    c_segs, keep = binding._segment_array(descs)
    rc = lib.evo_check_segmented(out.value, c_segs, len(descs), None, stats.data_ptr(), n_rows)
    assert rc == 0, rc
    torch.cuda.synchronize()
    del keep
    assert lib.evo_check_destroy(out.value) == 0      # also: the scratch guards are intact
    return binding.stats_to_numpy(stats)


def _population(n, P, seed, dtype):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    ref = 3 * torch.randn(n, generator=g, device="cuda", dtype=torch.float64)
    cands = []
    for p in range(P):
        c = ref * (1 + 0.02 * torch.randn(n, generator=g, device="cuda", dtype=torch.float64))
        far = torch.rand(n, generator=g, device="cuda") < 0.03
        c = torch.where(far, c + 5.0, c)
        cands.append(c)
    for t in [ref] + cands[::2]:
        idx = torch.randint(0, n, (max(1, n // 5000),), generator=g, device="cuda")
        t[idx] = torch.tensor([float("nan"), float("inf"), -float("inf"), 0.0, 1e-41],
                              device="cuda", dtype=torch.float64)[torch.randint(0, 5, (idx.numel(),), generator=g,
                                                                                  device="cuda")]
    return synth.Segment(ref.to(dtype).contiguous(), [c.to(dtype).contiguous() for c in cands], (n,), [True] * P)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float64], ids=["f32", "bf16", "f64"])
def test_rows_do_not_depend_on_the_job_plan(gu, alt, dtype):
    import paper_2510_03760_amd as evo
    shapes = [(1 << 22, 1), (3_000_017, 5), (1 << 21, 16), (700_001, 21), (1 << 19, 64), (40_001, 3)]
    for i, (n, P) in enumerate(shapes):
        _say("job plans %s n=%d P=%d" % (dtype, n, P))
        seg = _population(n, P, 600 + i, dtype)
        want = gu.oracle_rows(seg, 1e-2, 1e-2)
        for name, lib in (("two per compute unit", evo.lib), ("three per compute unit", alt)):
            got = _rows_with(lib, [seg], 1e-2, 1e-2, P)
            for p in range(P):
                gu.assert_rows_equal(got[p], want[p], "%s row %d" % (name, p))


def test_ragged_mix_under_both_job_plans(gu, alt):
    import paper_2510_03760_amd as evo
    _say("job plans, ragged mix")
    segs = [_population(n, P, 700 + i, dt) for i, (n, P, dt) in enumerate(
        [(1 << 20, 32, torch.float32), (333, 2, torch.float32), (2_000_003, 7, torch.bfloat16),
         (1 << 18, 17, torch.float16), (65_537, 4, torch.float64), (5, 1, torch.float32)])]
    n_rows = sum(len(s.cands) for s in segs)
    want = []
    for s in segs:
        want += gu.oracle_rows(s, 1e-2, 1e-2)
    rows = {}
    for name, lib in (("two", evo.lib), ("three", alt)):
        rows[name] = _rows_with(lib, segs, 1e-2, 1e-2, n_rows)
        for p in range(n_rows):
            gu.assert_rows_equal(rows[name][p], want[p], "%s per compute unit, row %d" % (name, p))
    for f in ("n_mismatch", "n_finite", "flags", "valid", "max_abs_err", "max_rel_err"):
        assert rows["two"][f].tobytes() == rows["three"][f].tobytes(), f
