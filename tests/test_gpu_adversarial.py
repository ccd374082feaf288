"""Candidates that try to pass without being right (the failure modes behind the inflated
success counts discussed in the paper's AI-CUDA-Engineer replication appendix): outputs
filled with NaN, Inf, zeros or a constant, outputs that are right except for a tail, outputs
that were never written.  Every one of them must come out invalid, for every element type,
and the rows must equal the oracle's.  Plus guard rows around the result buffer."""
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


FLOATS = [torch.float32, torch.bfloat16, torch.float16, torch.float64]


@pytest.mark.parametrize("dtype", FLOATS + [torch.int32, torch.int64], ids=lambda d: str(d).split(".")[-1])
def test_degenerate_candidates_are_invalid(gu, dtype):
    _say("degenerate candidates %s" % dtype)
    n = 300001
    g = torch.Generator(device="cuda")
    g.manual_seed(77)
    is_float = dtype in FLOATS
    if is_float:
        ref = (torch.randn(n, generator=g, device="cuda") * 2 + 3).to(dtype)      # few values near 0
    else:
        ref = torch.randint(1, 1000, (n,), generator=g, device="cuda", dtype=dtype)
    cands, names = [], []

    def add(name, c):
        names.append(name)
        cands.append(c.to(dtype).contiguous())

    add("copy", ref.clone())
    add("zeros", torch.zeros_like(ref))
    add("constant", torch.full_like(ref, 3))
    tail = ref.clone()
    tail[-7:] = 0                                   # right except for the last 7 elements
    add("wrong tail", tail)
    head = ref.clone()
    head[0] = head[0] + 1 if not is_float else head[0] * 2 + 1
    add("wrong first element", head)
    bits = torch.randint(-2 ** 31, 2 ** 31 - 1, (2 * n,), generator=g, device="cuda", dtype=torch.int32)
    raw = bits.view(torch.uint8)[: n * ref.element_size()].clone().view(dtype)
    add("never written (random bits)", raw)
    if is_float:
        add("NaN filled", torch.full_like(ref, float("nan")))
        add("Inf filled", torch.full_like(ref, float("inf")))
        one_nan = ref.clone()
        one_nan[n // 2] = float("nan")
        add("one NaN", one_nan)
        add("negated", -ref)
    P = len(cands)
    seg = synth.Segment(ref.contiguous(), cands, (n,), [True] * P)
    w = synth.Workload("degenerate", [seg], 1e-2, 1e-2, torch.ones(P, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, label="degenerate %s" % dtype)
    for name, row in zip(names, want):
        if name == "copy":
            assert row["valid"] == 1 and row["n_mismatch"] == 0, name
        else:
            assert row["valid"] == 0 and row["n_mismatch"] > 0, name
    assert want[names.index("wrong tail")]["n_mismatch"] == 7
    assert want[names.index("wrong first element")]["n_mismatch"] == 1
    # an invalid candidate gets fitness 0 however fast it is
    tim = torch.ones(P, 4, device="cuda")
    tim[1:] = 1e-3                                   # everything but the copy is "1000x faster"
    got, pop, fit = gu.fitness_parity(chk, stats, tim, torch.ones(4, device="cuda"), label="degenerate")
    assert int(pop["best_idx"]) == 0 and int(pop["n_valid"]) == 1
    assert float(pop["best_speedup"]) == 1.0 and np.all(got["fitness"][1:] == 0)
    chk.close()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16, torch.float64],
                         ids=lambda d: str(d).split(".")[-1])
def test_nan_filled_tiles_next_to_everything_else(gu, dtype):
    """Tiles that are NaN throughout are settled in the fast path by a closed form that only
    holds over a finite reference tile: NaN-filled candidates beside reference tiles that hold
    a NaN, an Inf or nothing special, NaN-filled except for one element, NaN in a single tile,
    Inf-filled, and a mixture of NaN and Inf."""
    _say("nan tiles %s" % dtype)
    n = 40 * 1024 + 333
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    ref = (torch.randn(n, generator=g, device="cuda") + 2).to(dtype)
    ref[3000] = float("nan")
    ref[9000] = float("inf")
    ref[9001] = float("-inf")
    ref[20000:20050] = float("nan")
    nan = torch.full_like(ref, float("nan"))
    cands = [nan.clone()]
    c = nan.clone(); c[12345] = 1.0; cands.append(c)                       # one number in one tile
    c = nan.clone(); c[::1024] = ref[::1024]; cands.append(c)              # one right element per tile
    c = ref.clone(); c[5 * 1024:6 * 1024] = float("nan"); cands.append(c)  # one tile (or two halves)
    c = ref.clone(); c[7 * 512:8 * 512] = float("nan"); cands.append(c)
    cands.append(torch.full_like(ref, float("inf")))
    c = nan.clone(); c[1::2] = float("inf"); cands.append(c)               # NaN and Inf alternate
    c = nan.clone(); c[9000] = float("inf"); c[9001] = float("inf"); cands.append(c)
    cands.append(ref.clone())
    P = len(cands)
    seg = synth.Segment(ref.contiguous(), [x.contiguous() for x in cands], (n,), [True] * P)
    w = synth.Workload("nan-tiles", [seg], 1e-2, 1e-2, torch.ones(P, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, label="nan tiles %s" % dtype)
    assert want[0]["n_mismatch"] == n and want[0]["n_finite"] == 0
    chk.close()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float64],
                         ids=lambda d: str(d).split(".")[-1])
def test_no_number_shortcut_stops_where_a_difference_can_overflow(gu, dtype):
    """A candidate tile whose differences are all NaN or Inf is settled without looking further
    only over reference elements small enough that a FINITE candidate element cannot overflow
    the difference (below 2^102 in binary32, 2^969 in binary64).  Here one difference per tile
    is infinite although both sides are finite: that element belongs to the statistics
    (n_finite, max and sum of the errors become Inf) and the shortcut must not take the tile.
    Beside it: the same tiles over a reference just below the bound, where the element's
    difference stays finite."""
    _say("overflowing difference in a NaN tile %s" % dtype)
    n = 12 * 4096 + 77
    big = {torch.float32: 2.0 ** 120, torch.bfloat16: 2.0 ** 120, torch.float64: 2.0 ** 970}[dtype]
    below = {torch.float32: 2.0 ** 101, torch.bfloat16: 2.0 ** 101, torch.float64: 2.0 ** 968}[dtype]
    lowest = torch.finfo(dtype).min
    g = torch.Generator(device="cuda")
    g.manual_seed(8)
    cands = []
    ref = (torch.randn(n, generator=g, device="cuda", dtype=torch.float64) + 2).to(dtype)
    sites = torch.arange(100, n, 1000, device="cuda")
    ref[sites[0::2]] = big                      # these can overflow against a finite candidate
    ref[sites[1::2]] = below                    # these cannot
    c = torch.full_like(ref, float("nan"))
    c[sites] = lowest                           # finite: |c - r| = Inf over `big`, finite over `below`
    cands.append(c)
    c = torch.full_like(ref, float("inf"))
    c[sites] = lowest
    cands.append(c)
    cands.append(torch.full_like(ref, float("nan")))
    cands.append(ref.clone())
    P = len(cands)
    seg = synth.Segment(ref.contiguous(), [x.contiguous() for x in cands], (n,), [True] * P)
    w = synth.Workload("overflow-tiles", [seg], 1e-2, 1e-2, torch.ones(P, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, label="overflow tiles %s" % dtype)
    assert want[0]["n_finite"] == sites.numel() and want[0]["n_mismatch"] == n
    assert np.isinf(want[0]["max_abs_err"]) and np.isinf(want[0]["sum_abs_err"])
    assert want[2]["n_finite"] == 0 and want[3]["valid"] == 1
    chk.close()


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16, torch.float64],
                         ids=lambda d: str(d).split(".")[-1])
def test_numbers_and_non_numbers_in_one_tile(gu, dtype):
    """NaN and Inf scattered among numbers (what a kernel with a data-dependent bug produces) are
    settled in the fast path, tile by tile: an element whose difference is not a number
    mismatches and is left out of the statistics, its neighbours count as usual.  Here: one NaN
    per tile, +Inf and -Inf, both kinds in one tile, non-numbers over reference elements that
    are 0 or subnormal (relative error defined as 0 there), next to finite mismatches and
    matches in the same tile, candidates whose numbers make a relative error overflow (those
    tiles go to the exact path), and the same over a reference tile that holds a huge value, a
    NaN or an Inf (never settled in the fast path)."""
    _say("mixed tiles %s" % dtype)
    n = 48 * 1024 + 421
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    ref = (torch.randn(n, generator=g, device="cuda", dtype=torch.float64) + 2).to(dtype)
    tiny = torch.finfo(dtype).tiny
    ref[5::97] = 0.0
    ref[6::197] = tiny / 4                       # subnormal
    ref[7::397] = -tiny / 2
    huge = {torch.float64: 2.0 ** 1000}.get(dtype, 2.0 ** 110 if dtype != torch.float16 else 60000.0)
    ref[30 * 1024 + 3] = huge                    # one tile with a huge reference element
    ref[33 * 1024 + 9] = float("nan")
    ref[36 * 1024 + 1] = float("-inf")
    ref[40 * 1024 + 5] = float("inf")            # each kind alone in a tile of otherwise plain values
    ref[42 * 1024 + 7] = float("-inf")
    ref[44 * 1024 + 9] = float("nan")
    near = (ref.double() * 1.001).to(dtype)      # inside the tolerance
    off = (ref.double() * 1.5 + 1).to(dtype)     # outside
    cands = []
    c = near.clone(); c[11::256] = float("nan"); cands.append(c)
    c = near.clone(); c[12::256] = float("inf"); c[140::256] = float("-inf"); cands.append(c)
    c = off.clone(); c[13::64] = float("nan"); c[14::128] = float("inf"); cands.append(c)
    c = near.clone(); c[5::97] = float("nan"); c[6::197] = float("inf"); c[7::397] = float("nan"); cands.append(c)
    c = near.clone(); c[::2] = float("nan"); c[1::512] = off[1::512]; cands.append(c)
    c = near.clone(); c[100::1000] = float("nan"); c[6::197] = 1.0; cands.append(c)   # 1 / subnormal: Inf
    c = torch.full_like(ref, float("nan")); c[3::64] = near[3::64]; cands.append(c)
    c = ref.clone(); c[777] = float("nan"); cands.append(c)                            # a single NaN
    c = ref.clone(); c[n - 1] = float("inf"); cands.append(c)                          # in the ragged tail
    c = near.clone(); c[40 * 1024 + 5] = float("-inf"); c[42 * 1024 + 7] = float("inf"); cands.append(c)   # wrong sign
    c = near.clone(); c[40 * 1024 + 5] = 1.0; c[42 * 1024 + 7] = float("nan"); c[44 * 1024 + 9] = 0.0; cands.append(c)
    cands.append(near.clone())
    P = len(cands)
    seg = synth.Segment(ref.contiguous(), [x.contiguous() for x in cands], (n,), [True] * P)
    w = synth.Workload("mixed-tiles", [seg], 1e-2, 1e-2, torch.ones(P, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, label="mixed tiles %s" % dtype)
    assert all(want[p]["valid"] == 0 for p in range(P))      # the reference's own NaN never matches
    assert want[7]["n_mismatch"] == 3 and want[0]["n_finite"] < n - n // 256
    chk.close()


def test_guard_rows_around_the_result_buffer(gu):
    """The calls write the rows they are given and not a byte more."""
    _say("guard rows")
    import paper_2510_03760_amd as evo
    P, n = 21, 100003
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    ref = torch.randn(n, generator=g, device="cuda")
    cands = [ref + 1e-3 * torch.randn(n, generator=g, device="cuda") for _ in range(P)]
    chk = evo.Checker(evo.EVO_F32, n, 1e-2, 1e-2)
    big = torch.full(((P + 4) * 72,), 0x5A, dtype=torch.uint8, device="cuda")
    rows = big[2 * 72:(P + 2) * 72]
    chk.check_batch(ref, cands, rows)
    tim = torch.rand(P, 10, device="cuda") + 0.5
    guard_sum = torch.full((16 * 3,), 0x5A, dtype=torch.uint8, device="cuda")
    chk.fitness(tim, tim[0].clone(), rows, guard_sum[16:32])
    elite = torch.full((4 + 8,), -1, dtype=torch.int32, device="cuda")
    chk.select_elite(rows, P, 4, elite[4:8])
    torch.cuda.synchronize()
    assert bool((big[: 2 * 72] == 0x5A).all()) and bool((big[(P + 2) * 72:] == 0x5A).all())
    assert bool((guard_sum[:16] == 0x5A).all()) and bool((guard_sum[32:] == 0x5A).all())
    assert bool((elite[:4] == -1).all()) and bool((elite[8:] == -1).all())
    assert bool((elite[4:8] >= 0).all())
    chk.close()


def _golden_example(name):
    import json
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "worked_examples.json")
    with open(path) as fh:
        for ex in json.load(fh)["check"]:
            if ex["name"] == name:
                return ex
    raise KeyError(name)


def _hexnum(x):
    return float.fromhex(x) if isinstance(x, str) and "0x" in x else float(x)


@pytest.mark.parametrize("kind", ["f32", "bf16", "f16", "f64"])
def test_tolerance_product_is_rounded_before_the_sum(gu, kind):
    """The hand-built inputs of tests/golden/worked_examples.json on which
    atol + fl(rtol*|r|) and a fused multiply-add differ by one unit in the last place, with
    |c - r| between the two: repeated over full tiles (fast path), over a ragged tail and on
    an unaligned view (exact path).  The mismatch count is known in closed form."""
    ex = _golden_example("product_rounds_before_sum_" + kind)
    atol, rtol = _hexnum(ex["atol"]), _hexnum(ex["rtol"])
    if kind in ("bf16", "f16"):
        tdt = torch.bfloat16 if kind == "bf16" else torch.float16
        r = torch.tensor(np.array(ex["ref_bits"], np.uint16).view(np.int16), device="cuda").view(tdt)
        c = torch.tensor(np.array(ex["cand_bits"], np.uint16).view(np.int16), device="cuda").view(tdt)
    else:
        tdt = torch.float32 if kind == "f32" else torch.float64
        r = torch.tensor([_hexnum(x) for x in ex["ref"]], dtype=torch.float64, device="cuda").to(tdt)
        c = torch.tensor([_hexnum(x) for x in ex["cand"]], dtype=torch.float64, device="cuda").to(tdt)
    k = r.numel()
    for reps, offset in ((1, 0), (3001, 0), (40000, 0), (40000, 1)):
        _say("fused-vs-unfused tolerance %s reps=%d offset=%d" % (kind, reps, offset))
        n = k * reps
        # offset 1: tensors that start one element past an aligned address (no 128-bit loads)
        ref = torch.zeros(n + offset, dtype=tdt, device="cuda")[offset:]
        cand = torch.zeros(n + offset, dtype=tdt, device="cuda")[offset:]
        ref.copy_(r.repeat(reps))
        cand.copy_(c.repeat(reps))
        seg = synth.Segment(ref, [cand, ref.clone()], (n,), [True, False])
        t = torch.ones(2, 4, device="cuda")
        w = synth.Workload("fma-" + kind, [seg], atol, rtol, t, torch.ones(4, device="cuda"))
        chk, stats, want = gu.check_parity(w, label="fma")
        assert want[0]["n_mismatch"] == ex["n_mismatch"] * reps     # the hand-computed count
        assert want[1]["n_mismatch"] == 0
        chk.close()
