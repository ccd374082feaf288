"""GPU parity on the awkward cases: ragged sizes, every special value, unaligned
tensors, odd population sizes, repeatability, argument errors on a live device."""
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


def _mixed(n, P, seed, dtype=torch.float32, special=True):
    """Reference and P candidates with near values, far values and (optionally) NaN,
    +-Inf, zeros, subnormals and huge values on both sides."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    ref = 3 * torch.randn(n, generator=g, device="cuda")
    cands = []
    for p in range(P):
        c = ref * (1 + 0.02 * torch.randn(n, generator=g, device="cuda"))
        far = torch.rand(n, generator=g, device="cuda") < 0.05
        c = torch.where(far, 20 * torch.rand(n, generator=g, device="cuda") - 10, c)
        same = torch.rand(n, generator=g, device="cuda") < 0.2
        c = torch.where(same, ref, c)
        cands.append(c)
    if special:
        vals = [float("nan"), float("inf"), float("-inf"), 0.0, -0.0, 1e-41, -1e-41, 3e38, -3e38,
                1.17549435e-38]
        for t in [ref] + cands:
            k = max(1, n // 40)
            idx = torch.randint(0, n, (k,), generator=g, device="cuda")
            v = torch.tensor(vals, device="cuda")[torch.randint(0, len(vals), (k,), generator=g,
                                                                 device="cuda")]
            t[idx] = v
    if dtype in (torch.bfloat16, torch.float16):
        # (3e38 etc. become Inf in binary16: more special sites, which is fine)
        ref = ref.to(dtype)
        cands = [c.to(dtype) for c in cands]
    seg = synth.Segment(ref.contiguous(), [c.contiguous() for c in cands], (n,), [True] * P)
    T = 8
    t = 1 + torch.rand(P, T, generator=g, device="cuda")
    b = 1 + torch.rand(T, generator=g, device="cuda")
    return synth.Workload("mixed-n%d-P%d" % (n, P), [seg], 1e-2, 1e-2, t, b)


SIZES = [1, 3, 4, 5, 63, 64, 65, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2047, 2049,
         4095, 4097, 65535, 65537, (1 << 20) + 1]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16],
                         ids=["f32", "bf16", "f16"])
def test_ragged_sizes_special_values(gu, dtype):
    for i, n in enumerate(SIZES):
        _say("mixed n=%d %s" % (n, dtype))
        w = _mixed(n, 3, 100 + i, dtype)
        chk, stats, want = gu.check_parity(w, label="sizes")
        chk.close()


@pytest.mark.parametrize("P", [1, 2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 33, 63, 64, 65, 130, 257])
def test_population_sizes(gu, P):
    _say("mixed P=%d" % P)
    w = _mixed(5000, P, 1000 + P, torch.float32)
    chk, stats, want = gu.check_parity(w, label="P")
    gu.fitness_parity(chk, stats, w.timings, w.baseline, label="P%d" % P)
    chk.close()
    w = _mixed(3000, P, 2000 + P, torch.bfloat16, special=False)
    chk, stats, want = gu.check_parity(w, label="P-bf16")
    chk.close()
    if P in (1, 5, 16, 33):
        w = _mixed(3000, P, 3000 + P, torch.float16, special=True)
        chk, stats, want = gu.check_parity(w, label="P-f16")
        chk.close()


@pytest.mark.parametrize("P", [3, 17, 40, 65])
def test_every_chunk_count_up_to_24(gu, P):
    """Sizes that give a segment 1, 2, ..., 24 chunks (so also counts that are not multiples
    of the number of XCDs), with one, two and four candidate groups per workgroup: every tile
    must be visited exactly once whatever the placement of chunks inside a window (a lost or
    doubled tile changes n_finite and the sums)."""
    groups = (P + 15) // 16 if P % 16 == 0 else P // 16 + bin(P % 16).count("1")
    gpw = min(4, 1 << (groups - 1).bit_length())
    tiles_per_chunk = 4 * (4 // gpw)        # smallest share of a wavefront x tile slots
    for chunks in range(1, 25):
        n = 512 * tiles_per_chunk * chunks - 300
        _say("P=%d chunks=%d n=%d" % (P, chunks, n))
        w = _mixed(n, P, 7000 + 31 * P + chunks, torch.float32, special=(chunks % 5 == 0))
        chk, stats, want = gu.check_parity(w, label="chunks%d" % chunks)
        chk.close()


def test_reciprocal_shortcut_is_exact_on_this_device(gu):
    """The kernel's 1/|r| shortcut (rcp + one FMA Newton step) equals the correctly rounded
    division for every binary32 input it is used on; checked exhaustively on the device."""
    _say("reciprocal shortcut")
    import os
    import subprocess
    import paper_2510_03760_amd as evo
    exe = os.path.join(os.path.dirname(evo.lib_path), "rcp_check")
    assert os.path.exists(exe), "build the package first (python -m paper_2510_03760_amd.build)"
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert res.returncode == 0, res.stdout
    assert " 0 mismatches" in res.stdout, res.stdout


def test_huge_reference_values(gu):
    """|r| at and above 2^126 (subnormal reciprocals) next to ordinary values."""
    _say("huge refs")
    n = 8192
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    ref = torch.randn(n, generator=g, device="cuda")
    big = torch.tensor([2.0 ** 126, -(2.0 ** 126), 2.0 ** 127, 3e38, 1.7e38, 2.0 ** 125, 8.5e37],
                       device="cuda")
    idx = torch.randint(0, n, (64,), generator=g, device="cuda")
    ref[idx] = big[torch.randint(0, 7, (64,), generator=g, device="cuda")]
    cands = [ref * (1 + 1e-3 * torch.randn(n, generator=g, device="cuda")) for _ in range(3)]
    cands = [torch.nan_to_num(c, posinf=3e38, neginf=-3e38) for c in cands]
    seg = synth.Segment(ref, cands, (n,), [False] * 3)
    w = synth.Workload("huge", [seg], 1e-2, 1e-2, torch.ones(3, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, label="huge")
    assert all(r["max_rel_err"] > 0 for r in want)
    chk.close()


def test_overflowing_differences(gu):
    """|c - r| and d/|r| overflow binary32 on finite inputs: the statistics keep +Inf."""
    _say("overflow")
    n = 4096
    ref = torch.full((n,), 3e38, device="cuda")
    ref[::3] = -3e38
    ref[5::7] = 1e-30
    c0 = -ref
    c1 = ref.clone()
    c1[100] = -3e38 if float(ref[100]) > 0 else 3e38
    seg = synth.Segment(ref, [c0, c1, ref.clone()], (n,), [True, True, False])
    w = synth.Workload("overflow", [seg], 1e-2, 1e-2, torch.ones(3, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, label="overflow")
    assert np.isinf(want[0]["max_abs_err"]) and np.isinf(want[0]["sum_abs_err"])
    assert want[2]["valid"] == 1
    chk.close()


def test_unaligned_tensors(gu):
    """Element-aligned but not 16-byte aligned views go through the exact path."""
    for dtype, offs in ((torch.float32, (1, 2, 3)), (torch.bfloat16, (1, 3, 7))):
        for k, off in enumerate(offs):
            _say("unaligned %s +%d" % (dtype, off))
            n = 3000 + k
            w = _mixed(n + 8, 4, 300 + k, dtype)
            seg = w.segments[0]
            ref = seg.ref[off:off + n] if k != 1 else seg.ref[:n]
            cands = [c[(off if i % 2 == 0 else 0):][:n] for i, c in enumerate(seg.cands)]
            assert any(t.data_ptr() % 16 for t in [ref] + cands)
            seg2 = synth.Segment(ref, cands, (n,), seg.corrupted)
            w2 = synth.Workload("unaligned", [seg2], w.atol, w.rtol, w.timings, w.baseline)
            chk, stats, want = gu.check_parity(w2, label="unaligned")
            chk.close()


def test_f16_every_bit_pattern(gu):
    """All 65536 binary16 patterns on both sides (subnormals, Inf, every NaN payload)."""
    _say("f16 all patterns")
    g = torch.Generator(device="cuda")
    g.manual_seed(16)
    allbits = torch.arange(65536, device="cuda", dtype=torch.int32)
    ref = allbits.repeat(8).to(torch.int16).view(torch.float16)
    n = ref.numel()
    cands = []
    for p in range(4):
        delta = torch.randint(-2, 3, (n,), generator=g, device="cuda", dtype=torch.int32)
        c = ((allbits.repeat(8) + delta) & 0xFFFF).to(torch.int16).view(torch.float16)
        cands.append(c.contiguous())
    cands.append(ref.clone())
    seg = synth.Segment(ref.contiguous(), cands, (n,), [True] * 5)
    w = synth.Workload("f16-all", [seg], 1e-2, 1e-2, torch.ones(5, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, label="f16-all")
    assert want[4]["n_mismatch"] == 8 * 2046   # the NaN patterns: 2 * (2^10 - 1) per copy
    chk.close()


def test_tolerance_extremes(gu):
    _say("tolerances")
    base = _mixed(10000, 4, 77, torch.float32)
    for atol, rtol in ((0.0, 0.0), (0.0, 1e-2), (1e-3, 0.0), (1e30, 0.0), (0.0, 3e38), (3e38, 3e38)):
        w = synth.Workload("tol", base.segments, atol, rtol, base.timings, base.baseline)
        chk, stats, want = gu.check_parity(w, label="tol %g %g" % (atol, rtol))
        chk.close()


def test_segmented_mixed_dtypes_and_row_layout(gu):
    """Groups of different dtype, size and population in one launch, rows scattered."""
    _say("segmented mixed")
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy
    ws = [_mixed(70000, 20, 1, torch.float32), _mixed(513, 3, 2, torch.float16),
          _mixed(1, 1, 3, torch.float32), _mixed(250000, 40, 4, torch.bfloat16, special=False),
          _mixed(4096, 16, 5, torch.float32, special=False)]
    order = [3, 0, 4, 1, 2]           # row ranges in a different order than the segments
    row0 = {}
    nxt = 2                           # leave rows 0-1 and a gap untouched
    for i in order:
        row0[i] = nxt
        nxt += ws[i].P + 1
    n_rows = nxt + 3
    chk = evo.Checker(evo.EVO_F32, 1, 1e-2, 1e-2)
    stats = chk.new_stats(n_rows)
    stats.fill_(0xEE)
    descs = [{"ref": w.segments[0].ref, "cand_ptrs": w.segments[0].cands, "n_elems": w.segments[0].n,
              "dtype": gu.dtype_code(w.segments[0]), "stats_row0": row0[i]} for i, w in enumerate(ws)]
    chk.check_segmented(descs, stats, n_rows)
    torch.cuda.synchronize()
    got = stats_to_numpy(stats)
    raw = stats.cpu().numpy().reshape(n_rows, 72)
    written = np.zeros(n_rows, bool)
    for i, w in enumerate(ws):
        want = gu.oracle_rows(w.segments[0], 1e-2, 1e-2)
        for p, o in enumerate(want):
            gu.assert_rows_equal(got[row0[i] + p], o, "seg %d row %d" % (i, p))
            written[row0[i] + p] = True
    assert np.all(raw[~written] == 0xEE), "rows outside every group must stay untouched"
    chk.close()


def test_check_cases_equals_one_accumulator_over_all_cases(gu):
    """K test cases of the same candidates in one launch: row p equals the oracle's single
    accumulator fed with candidate p's K (reference, output) pairs one after the other."""
    _say("cases")
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy
    for P, sizes, dts in ((16, (70001, 4096, 1, 300000, 513), [torch.float32] * 5),
                          (5, (1000, 65537), [torch.bfloat16, torch.float32]),
                          (40, (20000, 20000, 20000), [torch.float32, torch.bfloat16, torch.float32]),
                          (3, (12345,), [torch.float32])):
        ws = [_mixed(n, P, 7000 + 13 * i + P, dt, special=(i % 2 == 0))
              for i, (n, dt) in enumerate(zip(sizes, dts))]
        # make candidate 1 clean in every case, candidate 0 clean in all but the last
        for i, w in enumerate(ws):
            w.segments[0].cands[1] = w.segments[0].ref.clone() if not torch.isnan(
                w.segments[0].ref.float()).any() else w.segments[0].cands[1]
        chk = evo.Checker(evo.EVO_F32, 1, 1e-2, 1e-2)
        stats = chk.new_stats(P)
        stats.fill_(0x5A)
        cases = [{"ref": w.segments[0].ref, "cand_ptrs": w.segments[0].cands,
                  "n_elems": w.segments[0].n, "dtype": gu.dtype_code(w.segments[0])} for w in ws]
        chk.check_cases(cases, stats)
        torch.cuda.synchronize()
        got = stats_to_numpy(stats)
        for p in range(P):
            # fp32 and bf16 cases go through the same accumulator one after the other
            acc = None
            total = {"n_mismatch": 0, "n_finite": 0, "flags": 0, "n_elems": 0, "sum_abs_err": 0.0,
                     "sum_rel_err": 0.0, "max_abs_err": np.float32(0), "max_rel_err": np.float32(0)}
            for w in ws:
                seg = w.segments[0]
                r = oracle.check_one(synth.to_oracle_array(seg.ref), synth.to_oracle_array(seg.cands[p]),
                                     gu.oracle_dtype(seg), 1e-2, 1e-2)
                for f in ("n_mismatch", "n_finite", "n_elems", "sum_abs_err", "sum_rel_err"):
                    total[f] += r[f]
                total["flags"] |= r["flags"]
                total["max_abs_err"] = max(total["max_abs_err"], r["max_abs_err"])
                total["max_rel_err"] = max(total["max_rel_err"], r["max_rel_err"])
            total["valid"] = 1 if total["n_mismatch"] == 0 else 0
            gu.assert_rows_equal(got[p], total, "cases P=%d row %d" % (P, p))
        # same-dtype groups: also against ONE oracle accumulator fed case after case
        if len(set(dts)) == 1:
            for p in (0, P - 1):
                acc = oracle.CheckAccumulator(gu.oracle_dtype(ws[0].segments[0]), 1e-2, 1e-2)
                for w in ws:
                    acc.feed(synth.to_oracle_array(w.segments[0].ref),
                             synth.to_oracle_array(w.segments[0].cands[p]))
                gu.assert_rows_equal(got[p], acc.result(), "cases-acc P=%d row %d" % (P, p))
        chk.close()


@pytest.mark.parametrize("K,P,n", [(8, 32, 3000), (9, 4, 3000), (8, 4, 1 << 20), (5, 4, 1 << 20), (2, 128, 5000),
                                   (5, 8, 1 << 22), (3, 200, 40000), (8, 16, 70000)],
                         ids=lambda v: str(v))
def test_case_groups_on_both_sides_of_the_direct_fold(gu, K, P, n):
    """A small case group is folded by one workgroup in one go (at most 8 cases, a thread per
    case, candidate and range of jobs with at most 8 rows each); larger ones go through the
    per-segment levels and a merge.  Shapes on both sides of every one of those limits, against
    one oracle accumulator per candidate fed case after case; then the same cases through
    evo_evaluate, whose rows must be the same bytes."""
    _say("case group K=%d P=%d n=%d" % (K, P, n))
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy
    small = n <= 100000
    ws = [_mixed(n + 17 * i, P, 9100 + 7 * i + P + K, torch.float32, special=small and i % 2 == 0) for i in range(K)]
    chk = evo.Checker(evo.EVO_F32, 1, 1e-2, 1e-2)
    stats = chk.new_stats(P)
    stats.fill_(0x5A)
    cases = [{"ref": w.segments[0].ref, "cand_ptrs": w.segments[0].cands, "n_elems": w.segments[0].n,
              "dtype": evo.EVO_F32} for w in ws]
    chk.check_cases(cases, stats)
    torch.cuda.synchronize()
    got = stats_to_numpy(stats)
    picks = range(P) if small else (0, P // 2, P - 1)
    refs = [synth.to_oracle_array(w.segments[0].ref) for w in ws]
    for p in picks:
        acc = oracle.CheckAccumulator(oracle.F32, 1e-2, 1e-2)
        for w, r in zip(ws, refs):
            acc.feed(r, synth.to_oracle_array(w.segments[0].cands[p]))
        gu.assert_rows_equal(got[p], acc.result(), "case group K=%d P=%d n=%d row %d" % (K, P, n, p))
    if K <= 8 and K * P <= 384:
        timings, baseline = ws[0].timings, ws[0].baseline
        stats2, summary = chk.new_stats(P), chk.new_summary()
        chk.evaluate(cases, timings, baseline, stats2, summary)
        torch.cuda.synchronize()
        a, b = stats_to_numpy(stats2), got
        for f in ("n_mismatch", "n_finite", "sum_abs_err", "sum_rel_err", "max_abs_err", "max_rel_err", "flags", "valid"):
            assert a[f].tobytes() == b[f].tobytes(), f
    chk.close()


def test_large_tables_go_through_the_staged_path(gu):
    """More segments / candidate pointers than fit into the kernel-argument block: the
    descriptors are staged through pinned memory and a device table.  Also more segments
    than resident workgroup slots."""
    _say("staged table: 700 segments")
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    S = 700
    sizes = torch.randint(1, 3000, (S,), generator=g, device="cuda").tolist()
    segs, want_rows, row0 = [], [], 0
    keep = []
    for si, n in enumerate(sizes):
        dt = (torch.float32, torch.bfloat16, torch.float16)[si % 3]
        w = _mixed(n, 2, 5000 + si, dt, special=(si % 5 == 0))
        keep.append(w)
        seg = w.segments[0]
        segs.append({"ref": seg.ref, "cand_ptrs": seg.cands, "n_elems": seg.n,
                     "dtype": gu.dtype_code(seg), "stats_row0": row0})
        want_rows += gu.oracle_rows(seg, 1e-2, 1e-2, threads=1)
        row0 += 2
    chk = evo.Checker(evo.EVO_F32, 1, 1e-2, 1e-2)
    stats = chk.new_stats(row0)
    for rep in range(3):      # the staging slots rotate
        stats.fill_(0x11)
        chk.check_segmented(segs, stats, row0)
        torch.cuda.synchronize()
        got = stats_to_numpy(stats)
        for r, (gr, o) in enumerate(zip(got, want_rows)):
            gu.assert_rows_equal(gr, o, "staged rep %d row %d" % (rep, r))
    chk.close()
    _say("staged table: 1000 candidates")
    w = _mixed(2000, 1000, 4242, torch.float32, special=False)
    chk, stats, want = gu.check_parity(w, label="P1000")
    chk.close()


def test_repeatable_and_reusable_context(gu):
    """Same call twice gives byte-identical rows; a context can be reused for other
    populations (its counters re-arm themselves)."""
    _say("repeat")
    from paper_2510_03760_amd.binding import stats_to_numpy
    w = _mixed(300000, 16, 9, torch.float32)
    chk, stats, want = gu.check_parity(w, label="repeat")
    first = stats.clone()
    seg = w.segments[0]
    for _ in range(5):
        stats.fill_(0)
        chk.check_batch(seg.ref, seg.cands, stats)
        torch.cuda.synchronize()
        assert torch.equal(stats, first)
    # fewer candidates through the same context
    stats2 = chk.new_stats(5)
    chk.check_batch(seg.ref, seg.cands[:5], stats2)
    torch.cuda.synchronize()
    assert torch.equal(stats2, first[: 5 * 72])
    # back-to-back calls on one stream without synchronising in between
    outs = [chk.new_stats(16) for _ in range(12)]
    for o in outs:
        chk.check_batch(seg.ref, seg.cands, o)
    torch.cuda.synchronize()
    for o in outs:
        assert torch.equal(o, first)
    # on a side stream
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    o = chk.new_stats(16)
    with torch.cuda.stream(side):
        chk.check_batch(seg.ref, seg.cands, o, stream=side)
    side.synchronize()
    assert torch.equal(o, first)
    chk.close()


def test_alternating_populations_one_context(gu):
    """Two different populations of the same shape go through one context in turn, with
    no host synchronisation in between: every launch reuses the scratch rows of the
    previous one, so a stale read of those rows would show up as the other result."""
    _say("alternating")
    from paper_2510_03760_amd.binding import stats_to_numpy
    wa = _mixed(700001, 16, 21, torch.float32)
    wb = _mixed(700001, 16, 22, torch.float32)
    chk, stats_a, want_a = gu.check_parity(wa, label="alt-a")
    sa, sb = wa.segments[0], wb.segments[0]
    stats_b = chk.new_stats(16)
    chk.check_batch(sb.ref, sb.cands, stats_b)
    torch.cuda.synchronize()
    want_b = gu.oracle_rows(sb, wb.atol, wb.rtol)
    for p, (g, o) in enumerate(zip(stats_to_numpy(stats_b), want_b)):
        gu.assert_rows_equal(g, o, "alt-b row %d" % p)
    assert not torch.equal(stats_a, stats_b)
    outs = []
    for k in range(40):
        o = chk.new_stats(16)
        seg = sa if k % 2 == 0 else sb
        chk.check_batch(seg.ref, seg.cands, o)
        outs.append(o)
    torch.cuda.synchronize()
    for k, o in enumerate(outs):
        assert torch.equal(o, stats_a if k % 2 == 0 else stats_b), "launch %d" % k
    chk.close()


@pytest.mark.parametrize("T", [1, 2, 3, 5, 64, 100, 101, 255, 256, 257, 1000, 1001, 4095, 4096])
def test_fitness_T(gu, T):
    _say("fitness T=%d" % T)
    import paper_2510_03760_amd as evo
    g = torch.Generator(device="cuda")
    g.manual_seed(T)
    for P in (1, 9):
        t = torch.exp(0.1 * torch.randn(P, T, generator=g, device="cuda"))
        if P > 3 and T > 1:
            t[3] = t[2]
            t[4, : max(1, T // 2)] = float(t[4, 0])
        b = torch.exp(0.1 * torch.randn(T, generator=g, device="cuda"))
        chk = evo.Checker(evo.EVO_F32, 1, 0.0, 0.0)
        stats = chk.new_stats(P)
        view = stats.view(P, 72)
        valid = (torch.arange(P, device="cuda") % 3 != 1).to(torch.int32)
        view[:, 44:48] = valid.view(torch.uint8).view(P, 4)
        gu.fitness_parity(chk, stats, t, b, label="T%d" % T)
        chk.close()


def test_fitness_population_and_unusable_rows(gu):
    _say("fitness population")
    import paper_2510_03760_amd as evo
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    for P in (256, 1000, 3000):
        T = 100
        t = torch.exp(0.1 * torch.randn(P, T, generator=g, device="cuda"))
        b = torch.exp(0.1 * torch.randn(T, generator=g, device="cuda"))
        t[7, 3] = float("nan")
        t[8, 0] = float("inf")
        t[9, 99] = 0.0
        t[10, 50] = -1.0
        # dynamic range above 2^16: the mean has to be summed in sample order
        t[30, ::2] = 1e-20
        t[30, 1::2] = 3e20
        t[31, 0] = 1e-6
        t[32, 5] = 7e7
        t[35] = t[35] * 1e-42    # subnormal samples (candidate 35 is not valid below)
        t[20] = t[11]            # equal fitness: the lower index must win if it is the best
        t[11] *= 0.25
        t[20] *= 0.25
        chk = evo.Checker(evo.EVO_F32, 1, 0.0, 0.0)
        stats = chk.new_stats(P)
        view = stats.view(P, 72)
        valid = (torch.arange(P, device="cuda") % 5 != 0).to(torch.int32)
        view[:, 44:48] = valid.view(torch.uint8).view(P, 4)
        got, pop, want = gu.fitness_parity(chk, stats, t, b, label="pop%d" % P)
        assert int(pop["best_idx"]) == 11
        # nobody valid
        view[:, 44:48] = 0
        got, pop, want = gu.fitness_parity(chk, stats, t, b, label="none%d" % P)
        assert int(pop["best_idx"]) == P and float(pop["best_speedup"]) == 1.0
        # unusable baseline
        view[:, 44:48] = 1
        b2 = b.clone()
        b2[5] = float("nan")
        got, pop, want = gu.fitness_parity(chk, stats, t, b2, label="badbase%d" % P)
        assert np.all(got["speedup"] == 0)
        chk.close()


@pytest.mark.parametrize("P,k", [(1, 1), (5, 5), (8, 4), (256, 4), (300, 17), (1000, 1000),
                                 (4097, 64), (65535, 300)])
def test_select_elite(gu, P, k):
    """Top-k feasible candidates by fitness, ties in index order, against the oracle."""
    _say("elite P=%d k=%d" % (P, k))
    import oracle
    import paper_2510_03760_amd as evo
    g = torch.Generator(device="cuda")
    g.manual_seed(P * 31 + k)
    levels = torch.tensor([0.0, 0.0, 0.5, 0.75, 1.0, 1.25, 2.0, float("inf")], device="cuda")
    fit = levels[torch.randint(0, 8, (P,), generator=g, device="cuda")]
    some = torch.rand(P, generator=g, device="cuda") < 0.4
    fit = torch.where(some, torch.rand(P, generator=g, device="cuda") * 3, fit)
    for variant in range(3):
        if variant == 1:
            fit = torch.zeros(P, device="cuda")           # nobody feasible
        if variant == 2:
            fit = torch.full((P,), 1.5, device="cuda")    # everybody equal
        chk = evo.Checker(evo.EVO_F32, 1, 0.0, 0.0)
        stats = chk.new_stats(P)
        stats.view(P, 72)[:, 60:64] = fit.contiguous().view(torch.uint8).view(P, 4)
        elite = torch.full((k,), 0x7FFFFFFF, dtype=torch.int32, device="cuda")
        n_elite = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        chk.select_elite(stats, P, k, elite, n_elite)
        torch.cuda.synchronize()
        want = oracle.select_elite(fit.cpu().numpy(), k)
        assert elite.cpu().numpy().astype(np.uint32).tolist() == want["elite"].tolist()
        assert int(n_elite[0]) == want["n_elite"]
        chk.close()


@pytest.mark.parametrize("P,k,nkeys", [(1, 1, 1), (9, 4, 3), (256, 8, 30), (300, 300, 300), (1000, 64, 7),
                                       (4097, 100, 500), (65535, 300, 2000)])
def test_select_elite_diverse(gu, P, k, nkeys):
    _say("elite diverse P=%d k=%d keys=%d" % (P, k, nkeys))
    import oracle
    import paper_2510_03760_amd as evo
    rng = np.random.default_rng(P + k)
    f = rng.choice(np.array([0, 0.5, 0.75, 1, 1.25, 2, np.inf], np.float32), P)
    some = rng.random(P) < 0.4
    f[some] = rng.random(int(some.sum())).astype(np.float32)
    keys = (rng.integers(0, nkeys, P).astype(np.uint32) * np.uint32(2654435761))
    chk = evo.Checker(evo.EVO_F32, 1, 0.0, 0.0)
    stats = chk.new_stats(P)
    view = stats.view(P, 72)
    view[:, 60:64] = torch.from_numpy(f.view(np.uint8).copy()).to("cuda").view(P, 4)
    dkeys = torch.from_numpy(keys.view(np.int32).copy()).to("cuda")
    elite = torch.full((k + 2,), -7, dtype=torch.int32, device="cuda")
    n_elite = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    for _ in range(2):                                   # second call reuses the scratch
        chk.select_elite_diverse(stats, dkeys, P, k, elite[1:k + 1], n_elite)
    torch.cuda.synchronize()
    want = oracle.select_elite_diverse(f, keys, k)
    assert elite[1:k + 1].cpu().numpy().astype(np.uint32).tolist() == want["elite"].tolist()
    assert int(n_elite[0]) == want["n_elite"]
    assert int(elite[0]) == -7 and int(elite[k + 1]) == -7
    chosen = [int(i) for i in want["elite"] if i < P]
    assert len(set(int(keys[i]) for i in chosen)) == len(chosen)
    # all keys different: the plain selection
    uniq = torch.arange(P, dtype=torch.int32, device="cuda")
    plain = torch.zeros(k, dtype=torch.int32, device="cuda")
    div = torch.zeros(k, dtype=torch.int32, device="cuda")
    chk.select_elite(stats, P, k, plain)
    chk.select_elite_diverse(stats, uniq, P, k, div)
    torch.cuda.synchronize()
    assert torch.equal(plain, div)
    chk.close()


def test_errors_on_live_device(gu):
    """Argument errors are reported before anything is enqueued, also with a GPU."""
    _say("errors")
    import paper_2510_03760_amd as evo
    chk = evo.Checker(evo.EVO_F32, 1024, 1e-2, 1e-2)
    ref = torch.zeros(1024, device="cuda")
    stats = chk.new_stats(2)
    with pytest.raises(evo.EvoError) as e:
        evo.evo_check_batch(chk.ctx, ref, [ref, None], 2, None, stats)
    assert e.value.code == -1
    with pytest.raises(evo.EvoError) as e:
        evo.evo_check_batch(chk.ctx, ref.data_ptr() + 2, [ref], 1, None, stats)
    assert e.value.code == -5
    with pytest.raises(evo.EvoError) as e:
        evo.evo_fitness(chk.ctx, ref, ref, 1, 5000, None, stats, None)
    assert e.value.code == -3
    chk.check_batch(ref, [ref, ref], stats)   # still usable afterwards
    torch.cuda.synchronize()
    from paper_2510_03760_amd.binding import stats_to_numpy
    assert stats_to_numpy(stats)["valid"].tolist() == [1, 1]
    chk.close()
