"""evo_check_batch_static -- the entry point for callers that cannot allocate -- gives what
evo_check_batch gives, on two calls in a row through the C ABI, the second on a smaller
input; it allocates no device memory; it refuses what is beyond its fixed capacity."""
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


def _say(msg):
    print(msg, flush=True)


def _population(n, P, seed, dtype):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    ref = 2 * torch.randn(n, generator=g, device="cuda")
    cands = []
    for p in range(P):
        c = ref * (1 + 0.004 * torch.randn(n, generator=g, device="cuda"))
        if p % 3 == 1:
            far = torch.rand(n, generator=g, device="cuda") < 0.01
            c = torch.where(far, c + 1.0, c)
        if p % 5 == 2:
            c[int(torch.randint(0, n, (1,), generator=g, device="cuda"))] = float("nan")
        cands.append(c.to(dtype).contiguous())
    return ref.to(dtype).contiguous(), cands


def _rows(chk, call, ref, cands, gu):
    import paper_2510_03760_amd as evo
    stats = chk.new_stats(len(cands))
    stats.fill_(0xEE)
    call(ref, cands, stats)
    torch.cuda.synchronize()
    return evo.binding.stats_to_numpy(stats).copy()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_static_scratch_call_equals_check_batch(gu, dtype):
    import paper_2510_03760_amd as evo
    code = evo.EVO_F32 if dtype == torch.float32 else evo.EVO_BF16
    # first a large population (many jobs, two-level fold), then a smaller one (fewer jobs,
    # fewer candidates: whatever the first call left in the array must not show)
    shapes = [((1 << 22) + 12345, 21), (70001, 5), (300, 2)]
    before = None
    for i, (n, P) in enumerate(shapes):
        _say("static scratch %s n=%d P=%d" % (dtype, n, P))
        ref, cands = _population(n, P, 4100 + i, dtype)
        with evo.Checker(code, n, 1e-2, 1e-2) as plain, evo.Checker(code, n, 1e-2, 1e-2) as fixed:
            want = _rows(plain, plain.check_batch, ref, cands, gu)
            if i == 1:
                torch.cuda.synchronize()
                before = torch.cuda.mem_get_info()[0]
            got = _rows(fixed, fixed.check_batch_static, ref, cands, gu)
            if i == 1:
                assert torch.cuda.mem_get_info()[0] == before, "the call changed the free device memory"
            for p in range(P):
                gu.assert_rows_equal(got[p], dict(
                    {f: want[p][f] for f in want.dtype.names},
                    n_elems=int(want[p]["n_elems_lo"]) | (int(want[p]["n_elems_hi"]) << 32)), "row %d" % p)
            # same kernels, same launch geometry, same fold order: the bytes agree too
            assert got.tobytes() == want.tobytes()
            # and both agree with the oracle
            seg = synth.Segment(ref, cands, (n,), [False] * P)
            orows = gu.oracle_rows(seg, 1e-2, 1e-2)
            for p in range(P):
                gu.assert_rows_equal(got[p], orows[p], "oracle row %d" % p)


def test_static_scratch_call_refuses_what_exceeds_its_capacity(gu):
    import paper_2510_03760_amd as evo
    n = 256
    ref = torch.zeros(n, device="cuda")
    with evo.Checker(evo.EVO_F32, n, 0.0, 0.0) as chk:
        stats = chk.new_stats(400)
        stats.fill_(0x11)
        with pytest.raises(evo.EvoError) as err:
            chk.check_batch_static(ref, [ref] * 400, stats)
        assert err.value.code == -9
        torch.cuda.synchronize()
        assert int(stats.min()) == 0x11 and int(stats.max()) == 0x11   # nothing was enqueued
        chk.check_batch_static(ref, [ref] * 384, stats)                # the largest population
        torch.cuda.synchronize()
        got = evo.binding.stats_to_numpy(stats)
        assert int(got["valid"][:384].sum()) == 384
