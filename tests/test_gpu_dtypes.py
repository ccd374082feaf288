"""GPU parity for binary64 and integer tensors and for the mean-based speedup: the HIP
path through the C ABI against the CPU oracle, element types and sizes that span full
tiles, a ragged tail, unaligned tensors and every special value."""
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


def _workload(name, ref, cands, atol=1e-2, rtol=1e-2):
    P = len(cands)
    seg = synth.Segment(ref.contiguous(), [c.contiguous() for c in cands], tuple(ref.shape), [True] * P)
    return synth.Workload(name, [seg], atol, rtol, torch.ones(P, 4, device="cuda"),
                          torch.ones(4, device="cuda"))


def _mixed_f64(n, P, seed):
    """binary64 reference and candidates: close values, far values, values only binary64
    tells apart, values outside the binary32 range, NaN, Inf, zeros, subnormals."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    ref = torch.randn(n, generator=g, device="cuda", dtype=torch.float64) * 3
    k = max(1, n // 40)

    def sites():
        return torch.randint(0, n, (k,), generator=g, device="cuda")

    ref[sites()] = 0.0
    ref[sites()] = 1e-310
    ref[sites()] = 1e-40
    ref[sites()] = 1e300
    ref[sites()] = -1.7e308
    ref[sites()] = float("inf")
    ref[sites()] = float("-inf")
    ref[sites()] = float("nan")
    cands = []
    for p in range(P):
        c = ref * (1 + 1e-3 * torch.randn(n, generator=g, device="cuda", dtype=torch.float64))
        c[sites()] = ref[sites()] * (1 + 2.0 ** -40)          # below binary32 resolution
        far = sites()
        c[far] = torch.rand(k, generator=g, device="cuda", dtype=torch.float64) * 20 - 10
        c[sites()] = float("nan")
        c[sites()] = float("inf")
        c[sites()] = 1.7e308                                   # against -1.7e308: the difference overflows
        c[sites()] = -0.0
        same = sites()
        c[same] = ref[same]
        if p == 1:
            c = ref.clone()
        cands.append(c)
    return ref, cands


@pytest.mark.parametrize("n,P", [(1, 1), (255, 3), (256, 16), (257, 5), (70001, 21), ((1 << 20) + 3, 8),
                                 (70001, 11), (300001, 7), (150001, 3)])
def test_f64_special_values_and_ragged_sizes(gu, n, P):
    _say("f64 n=%d P=%d" % (n, P))
    ref, cands = _mixed_f64(n, P, 100 + n % 97)
    for atol, rtol in ((1e-2, 1e-2), (0.0, 0.0), (1e-9, 1e-9)):
        chk, stats, want = gu.check_parity(_workload("f64", ref, cands, atol, rtol), label="f64 %g" % atol)
        chk.close()
    if n > 1000:
        assert any(w["flags"] != 0 for w in want) and any(w["n_mismatch"] > 0 for w in want)


def test_f64_decides_what_f32_cannot(gu):
    _say("f64 resolution")
    n = 5000
    ref = torch.ones(n, device="cuda", dtype=torch.float64)
    cand = ref.clone()
    cand[::5] += 2.0 ** -40
    chk, stats, want = gu.check_parity(_workload("f64-res", ref, [cand, ref.clone()], 0.0, 0.0))
    assert want[0]["n_mismatch"] == 1000 and want[1]["n_mismatch"] == 0
    chk.close()


def test_f64_unaligned(gu):
    _say("f64 unaligned")
    ref, cands = _mixed_f64(30001, 4, 7)
    chk, stats, want = gu.check_parity(_workload("f64-unal", ref[1:], [c[1:] for c in cands]))
    chk.close()
    # only one candidate off the 16-byte grid
    c2 = [cands[0][:-1], cands[1][1:], cands[2][:-1]]
    chk, stats, want = gu.check_parity(_workload("f64-unal1", ref[:-1], c2))
    chk.close()


def _mixed_int(n, P, seed, dtype):
    info = torch.iinfo(dtype)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    ref = torch.randint(-1000, 1000, (n,), generator=g, device="cuda", dtype=dtype)
    k = max(1, n // 50)

    def sites():
        return torch.randint(0, n, (k,), generator=g, device="cuda")

    ref[sites()] = info.min
    ref[sites()] = info.max
    ref[sites()] = 0
    cands = []
    for p in range(P):
        c = ref.clone()
        s = sites()
        c[s] = c[s] + torch.randint(-3, 4, (k,), generator=g, device="cuda", dtype=dtype)   # wraps at the ends
        c[sites()] = info.max
        c[sites()] = info.min
        c[sites()] = 2 ** 30 + p
        if p == 1:
            c = ref.clone()
        cands.append(c)
    return ref, cands


@pytest.mark.parametrize("dtype", [torch.int32, torch.int64], ids=["i32", "i64"])
@pytest.mark.parametrize("n,P", [(1, 1), (511, 3), (512, 16), (513, 5), (70001, 21), ((1 << 20) + 3, 8),
                                 (70001, 11), (300001, 7), (150001, 3)])
def test_integer_tensors(gu, dtype, n, P):
    _say("%s n=%d P=%d" % (dtype, n, P))
    ref, cands = _mixed_int(n, P, 200 + n % 89, dtype)
    chk, stats, want = gu.check_parity(_workload("int", ref, cands, 5.0, 5.0))   # tolerances play no part
    chk.close()
    if P > 1:
        assert want[1]["n_mismatch"] == 0 and want[1]["valid"] == 1
    if n > 1000:
        assert want[0]["n_mismatch"] > 0
        # the largest difference needs one bit more than the type has
        assert float(want[0]["max_abs_err"]) == float(2 ** torch.iinfo(dtype).bits)
    for w in want:
        assert w["flags"] == 0 and w["max_rel_err"] == 0 and w["n_finite"] == n


@pytest.mark.parametrize("dtype", [torch.int32, torch.int64], ids=["i32", "i64"])
def test_integer_unaligned(gu, dtype):
    _say("unaligned %s" % dtype)
    ref, cands = _mixed_int(40001, 3, 11, dtype)
    chk, stats, want = gu.check_parity(_workload("int-unal", ref[1:], [c[1:] for c in cands]))
    chk.close()


def test_every_element_type_in_one_segmented_launch(gu):
    """Six groups, one per element type, different sizes and populations, one launch."""
    _say("all dtypes segmented")
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    groups = []
    f = torch.randn(50001, generator=g, device="cuda")
    groups.append((f, [f * 1.001, f.clone(), f + 1]))
    b = torch.randn(4099, generator=g, device="cuda").to(torch.bfloat16)
    groups.append((b, [b.clone(), (b.float() * 1.01).to(torch.bfloat16)]))
    h = torch.randn(9000, generator=g, device="cuda").to(torch.float16)
    groups.append((h, [(h.float() + 0.05).to(torch.float16)]))
    r64, c64 = _mixed_f64(33333, 5, 3)
    groups.append((r64, c64))
    r32, c32 = _mixed_int(20001, 17, 4, torch.int32)
    groups.append((r32, c32))
    rl, cl = _mixed_int(777, 2, 6, torch.int64)
    groups.append((rl, cl))
    segs = [synth.Segment(r.contiguous(), [c.contiguous() for c in cs], tuple(r.shape), [True] * len(cs))
            for r, cs in groups]
    P = sum(len(s.cands) for s in segs)
    w = synth.Workload("all-types", segs, 1e-2, 1e-2, torch.ones(P, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, segmented=True, label="all-types")
    chk.close()


def test_cases_mixing_float_and_integer_outputs(gu):
    """A candidate whose operation returns values (binary64) and indices (int64): two cases,
    one row per candidate."""
    _say("cases f64+i64")
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy
    P = 6
    rv, cv = _mixed_f64(20000, P, 21)
    ri, ci = _mixed_int(3000, P, 22, torch.int64)
    chk = evo.Checker(evo.EVO_F64, rv.numel(), 1e-2, 1e-2)
    stats = chk.new_stats(P)
    stats.fill_(0xAB)
    cases = [{"ref": rv, "cand_ptrs": cv, "n_elems": rv.numel(), "dtype": evo.EVO_F64},
             {"ref": ri, "cand_ptrs": ci, "n_elems": ri.numel(), "dtype": evo.EVO_I64}]
    chk.check_cases(cases, stats)
    torch.cuda.synchronize()
    got = stats_to_numpy(stats)
    for p in range(P):
        a = oracle.check_one(synth.to_oracle_array(rv), synth.to_oracle_array(cv[p]), oracle.F64, 1e-2, 1e-2)
        b = oracle.check_one(synth.to_oracle_array(ri), synth.to_oracle_array(ci[p]), oracle.I64, 1e-2, 1e-2)
        assert int(got[p]["n_mismatch"]) == a["n_mismatch"] + b["n_mismatch"]
        assert int(got[p]["n_finite"]) == a["n_finite"] + b["n_finite"]
        assert int(got[p]["flags"]) == a["flags"] | b["flags"]
        assert int(got[p]["valid"]) == (1 if a["valid"] and b["valid"] else 0)
        assert np.float32(got[p]["max_abs_err"]).tobytes() == max(a["max_abs_err"], b["max_abs_err"]).tobytes()
        assert np.float32(got[p]["max_rel_err"]).tobytes() == max(a["max_rel_err"], b["max_rel_err"]).tobytes()
        for f in ("sum_abs_err", "sum_rel_err"):
            want = a[f] + b[f]
            if np.isfinite(want):
                assert abs(float(got[p][f]) - want) <= gu.SUM_RTOL * abs(want), (p, f)
            else:
                assert float(got[p][f]) == want
    chk.close()


@pytest.mark.parametrize("T", [1, 2, 5, 100, 101, 1000, 4096])
def test_fitness_ratio_of_means(gu, T):
    _say("mean reducer T=%d" % T)
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy
    P = 9
    g = torch.Generator(device="cuda")
    g.manual_seed(T)
    tim = torch.exp(0.1 * torch.randn(P, T, generator=g, device="cuda")).float()
    base = torch.exp(0.1 * torch.randn(T, generator=g, device="cuda")).float()
    tim[4] *= 0.5
    if T > 2:
        tim[5, T // 2] = float("nan")            # unusable row
        tim[6, 0] *= 10.0 * T                    # an outlier moves the mean, not the median
    chk = evo.Checker(evo.EVO_F32, 16, 1e-2, 1e-2)
    stats = chk.new_stats(P)
    valid = np.array([1, 1, 0, 1, 1, 1, 1, 0, 1], np.uint32)
    view = stats.view(P, 72)
    view[:, 44:48] = torch.from_numpy(valid.view(np.uint8).copy()).to("cuda").view(P, 4)
    for reducer, code in ((evo.EVO_REDUCE_MEAN, oracle.REDUCE_MEAN), (evo.EVO_REDUCE_MEDIAN, oracle.REDUCE_MEDIAN)):
        summary = chk.new_summary()
        chk.fitness(tim, base, stats, summary, reducer=reducer)
        torch.cuda.synchronize()
        got = stats_to_numpy(stats)
        pop = summary_to_numpy(summary)[0]
        want = oracle.fitness(tim.cpu().numpy(), base.cpu().numpy(), valid, reducer=code)
        for f in ("median_ms", "mean_ms", "speedup", "fitness"):
            assert got[f].tobytes() == want[f].tobytes(), (reducer, f, got[f], want[f])
        assert int(pop["best_idx"]) == want["best_idx"] and int(pop["n_valid"]) == want["n_valid"]
        assert np.float32(pop["best_speedup"]).tobytes() == np.float32(want["best_speedup"]).tobytes()
    if T >= 100:
        mean_run = oracle.fitness(tim.cpu().numpy(), base.cpu().numpy(), valid, reducer=oracle.REDUCE_MEAN)
        med_run = oracle.fitness(tim.cpu().numpy(), base.cpu().numpy(), valid)
        assert mean_run["speedup"][6] < 0.5 * med_run["speedup"][6]
    chk.close()


def test_tolerance_policy_in_one_launch(gu):
    """Groups of different element types and tolerance classes in ONE launch, each checked with
    its own pair (functional testing over outputs of different precisions, Sec. 4.3): the
    ragged call, the fused ragged call and the test-case call against the oracle's policy."""
    _say("tolerance policy")
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy
    g = torch.Generator(device="cuda")
    g.manual_seed(91)

    def group(n, P, dtype, noise):
        r = torch.randn(n, generator=g, device="cuda", dtype=torch.float64)
        cs = [(r * (1 + noise * torch.randn(n, generator=g, device="cuda", dtype=torch.float64))).to(dtype).contiguous()
              for _ in range(P)]
        return r.to(dtype).contiguous(), cs

    P = 5
    spec = [   # (tensors, element type codes, tolerance class)
        (group(70001, P, torch.float32, 2e-4), evo.EVO_F32, oracle.F32, 0),
        (group(33000, P, torch.bfloat16, 6e-3), evo.EVO_BF16, oracle.BF16, 0),
        (group(12345, P, torch.float16, 8e-4), evo.EVO_F16, oracle.F16, 0),
        (group(50000, P, torch.float64, 2e-9), evo.EVO_F64, oracle.F64, 0),
        (group(4096, P, torch.float32, 2e-4), evo.EVO_F32, oracle.F32, 4),     # a stricter class
        (group(300, P, torch.bfloat16, 6e-3), evo.EVO_BF16, oracle.BF16, 9),   # a looser class
    ]
    pol = oracle.TolerancePolicy(1e-4, 3e-4)
    chk = evo.Checker(evo.EVO_F32, 1, 1e-4, 3e-4)
    for code, ocode, atol, rtol in ((evo.EVO_BF16, oracle.BF16, 1e-2, 8e-3), (evo.EVO_F16, oracle.F16, 1e-3, 1e-3),
                                    (evo.EVO_F64, oracle.F64, 1e-9, 3e-9)):
        chk.set_tolerance(code, atol, rtol)
        pol.set_dtype(ocode, atol, rtol)
    for cls, atol, rtol in ((4, 0.0, 1e-4), (9, 0.25, 0.0)):
        chk.set_tolerance_class(cls, atol, rtol)
        pol.set_class(cls, atol, rtol)

    descs, osegs, row0 = [], [], 0
    for (r, cs), code, ocode, cls in spec:
        descs.append({"ref": r, "cand_ptrs": cs, "n_elems": r.numel(), "dtype": code, "stats_row0": row0,
                      "tol_class": cls})
        osegs.append((synth.to_oracle_array(r), [synth.to_oracle_array(c) for c in cs], ocode, cls))
        row0 += len(cs)
    want = oracle.check_segments(osegs, pol, threads=8)
    # the tolerances differ enough to matter: some groups reject elements, some accept all
    per_group = [sum(w["n_mismatch"] for w in want[i * P:(i + 1) * P]) for i in range(len(spec))]
    assert all(m > 0 for m in per_group[:5]) and per_group[5] == 0, per_group

    stats = chk.new_stats(row0)
    stats.fill_(0xAB)
    chk.check_segmented(descs, stats, row0)
    torch.cuda.synchronize()
    got = stats_to_numpy(stats)
    for i, (gr, w) in enumerate(zip(got, want)):
        gu.assert_rows_equal(gr, w, "policy row %d" % i)

    # the fused ragged call uses the same pairs
    T = 6
    tim = 1 + torch.rand(row0, T, generator=g, device="cuda")
    base = 1 + torch.rand(T, generator=g, device="cuda")
    stats2, summary = chk.new_stats(row0), chk.new_summary()
    chk.evaluate_segmented(descs, tim, base, stats2, row0, summary)
    torch.cuda.synchronize()
    got2 = stats_to_numpy(stats2)
    for i, (gr, w) in enumerate(zip(got2, want)):
        gu.assert_rows_equal(gr, w, "policy (fused) row %d" % i)
    fit = oracle.fitness(tim.cpu().numpy(), base.cpu().numpy(), np.array([w["valid"] for w in want], np.uint32))
    for f in ("median_ms", "mean_ms", "speedup", "fitness"):
        assert got2[f].tobytes() == fit[f].tobytes(), f
    assert int(summary_to_numpy(summary)[0]["n_valid"]) == fit["n_valid"]

    # as test cases of the same P candidates: one row per candidate, each case with its pair
    cases = [{k: v for k, v in d.items() if k != "stats_row0"} for d in descs]
    stats3 = chk.new_stats(P)
    stats3.fill_(0xAB)
    chk.check_cases(cases, stats3)
    torch.cuda.synchronize()
    got3 = stats_to_numpy(stats3)
    want3 = oracle.check_cases(osegs, pol)
    for p in range(P):
        gu.assert_rows_equal(got3[p], want3[p], "policy case row %d" % p)

    # a class that was never set is refused before anything is enqueued
    bad = dict(descs[0], tol_class=7)
    stats.fill_(0x5A)
    with pytest.raises(evo.EvoError) as err:
        chk.check_segmented([bad], stats, row0)
    assert err.value.code == -4
    torch.cuda.synchronize()
    assert int(stats.min()) == 0x5A and int(stats.max()) == 0x5A
    chk.close()
