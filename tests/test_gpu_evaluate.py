"""evo_evaluate (check of K test cases plus the timing reduction, one launch when the table
fits the kernel argument block) against the two calls it stands for and against the oracle."""
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


def _cases(K, n, P, dtype, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    out = []
    for k in range(K):
        nk = n + 37 * k
        ref = (torch.randn(nk, generator=g, device="cuda") * 2).to(dtype)
        cands = []
        for p in range(P):
            c = (ref.float() * (1 + 1e-3 * torch.randn(nk, generator=g, device="cuda"))).to(dtype)
            if p % 4 == 3 and k == (p // 4) % K:
                c[nk // 3] = 50.0                       # one case of this candidate fails
            if p == 5 and k == 0:
                c[7] = float("nan")
            cands.append(c)
        out.append((ref, cands))
    return out


@pytest.mark.parametrize("K,n,P,dtype,T,reducer", [
    (1, 4096, 4, torch.float32, 5, 0),            # a single job: rows written directly
    (1, 3000001, 16, torch.float32, 100, 0),
    (5, 700001, 16, torch.float32, 100, 1),
    (5, 400001, 64, torch.bfloat16, 101, 0),      # 320 pointers: still one launch
    (3, 200001, 21, torch.float16, 7, 1),
    (5, 60001, 100, torch.float32, 100, 0),       # 500 pointers: two launches, same results
    (9, 30001, 8, torch.float32, 64, 0),          # 9 cases: two launches
    (1, 700001, 33, torch.float32, 100, 0),       # cut into 32 + 1 candidates: two writers of rows
    (1, 1200001, 37, torch.bfloat16, 9, 1),       # 32 + 5
])
def test_evaluate_equals_check_then_fitness(gu, K, n, P, dtype, T, reducer):
    _say("evaluate K=%d n=%d P=%d %s T=%d reducer=%d" % (K, n, P, dtype, T, reducer))
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy
    code = {torch.float32: evo.EVO_F32, torch.bfloat16: evo.EVO_BF16, torch.float16: evo.EVO_F16}[dtype]
    ocode = {torch.float32: oracle.F32, torch.bfloat16: oracle.BF16, torch.float16: oracle.F16}[dtype]
    data = _cases(K, n, P, dtype, 1000 + K * 7 + P)
    cases = [{"ref": r, "cand_ptrs": cs, "n_elems": r.numel(), "dtype": code} for r, cs in data]
    g = torch.Generator(device="cuda")
    g.manual_seed(T)
    tim = torch.exp(0.1 * torch.randn(P, T, generator=g, device="cuda")).float()
    base = torch.exp(0.1 * torch.randn(T, generator=g, device="cuda")).float()
    if T > 2 and P > 2:
        tim[2, 1] = float("inf")
    chk = evo.Checker(code, data[0][0].numel(), 1e-2, 1e-2)

    # the two calls
    want_stats = chk.new_stats(P)
    want_sum = chk.new_summary()
    chk.check_cases(cases, want_stats)
    chk.fitness(tim, base, want_stats, want_sum, reducer=reducer)
    torch.cuda.synchronize()

    # the one call, several times (its ticket re-arms itself), rows poisoned in between
    for rep in range(3):
        stats = chk.new_stats(P)
        stats.fill_(0xAB)
        summary = chk.new_summary()
        summary.fill_(0xCD)
        chk.evaluate(cases, tim, base, stats, summary, reducer=reducer)
        torch.cuda.synchronize()
        assert torch.equal(stats, want_stats), rep
        assert torch.equal(summary, want_sum), rep

    # and the oracle
    got = stats_to_numpy(stats)
    accs = [oracle.CheckAccumulator(ocode, 1e-2, 1e-2) for _ in range(P)]
    for r, cs in data:
        ra = synth.to_oracle_array(r)
        for p in range(P):
            accs[p].feed(ra, synth.to_oracle_array(cs[p]))
    rows = [a.result() for a in accs]
    for p in range(P):
        gu.assert_rows_equal(got[p], rows[p], "evaluate row %d" % p)
    valid = np.array([r["valid"] for r in rows], np.uint32)
    fit = oracle.fitness(tim.cpu().numpy(), base.cpu().numpy(), valid, reducer=reducer)
    for f in ("median_ms", "mean_ms", "speedup", "fitness"):
        assert got[f].tobytes() == fit[f].tobytes(), f
    pop = summary_to_numpy(summary)[0]
    assert int(pop["best_idx"]) == fit["best_idx"] and int(pop["n_valid"]) == fit["n_valid"]
    assert np.float32(pop["best_speedup"]).tobytes() == np.float32(fit["best_speedup"]).tobytes()
    assert 0 < fit["n_valid"] < P or P < 4
    chk.close()


@pytest.mark.parametrize("shapes,T,reducer", [
    ([(4096, 4, torch.float32)], 5, 0),                                   # one group: as evo_check_batch
    ([(700001, 16, torch.float32), (30001, 16, torch.float32)], 100, 0),
    ([(300001, 32, torch.float32), (128, 32, torch.float32), (1000, 32, torch.float32),
      (262144, 32, torch.float32)], 100, 1),                              # the ragged workload in small
    ([(600001, 17, torch.float32), (90001, 5, torch.bfloat16), (200001, 33, torch.float16)], 64, 0),
    ([(20001, 60, torch.float32)] * 9, 7, 0),                             # 9 groups, 540 pointers: two launches
])
def test_evaluate_segmented_equals_check_then_fitness(gu, shapes, T, reducer):
    _say("evaluate_segmented %s T=%d reducer=%d" % ([(n, P, str(d)) for n, P, d in shapes], T, reducer))
    import oracle
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy
    code = {torch.float32: evo.EVO_F32, torch.bfloat16: evo.EVO_BF16, torch.float16: evo.EVO_F16}
    ocode = {torch.float32: oracle.F32, torch.bfloat16: oracle.BF16, torch.float16: oracle.F16}
    segs, row0 = [], 0
    data = []
    for i, (n, P, dtype) in enumerate(shapes):
        (ref, cands), = _cases(1, n, P, dtype, 3000 + 17 * i + P)
        data.append((ref, cands, dtype))
        segs.append({"ref": ref, "cand_ptrs": cands, "n_elems": n, "dtype": code[dtype], "stats_row0": row0})
        row0 += P
    rows = row0
    g = torch.Generator(device="cuda")
    g.manual_seed(T + rows)
    tim = torch.exp(0.1 * torch.randn(rows, T, generator=g, device="cuda")).float()
    base = torch.exp(0.1 * torch.randn(T, generator=g, device="cuda")).float()
    chk = evo.Checker(evo.EVO_F32, shapes[0][0], 1e-2, 1e-2)

    want_stats = chk.new_stats(rows)
    want_sum = chk.new_summary()
    chk.check_segmented(segs, want_stats, rows)
    chk.fitness(tim, base, want_stats, want_sum, reducer=reducer)
    torch.cuda.synchronize()

    for rep in range(3):
        stats = chk.new_stats(rows)
        stats.fill_(0xAB)
        summary = chk.new_summary()
        summary.fill_(0xCD)
        chk.evaluate_segmented(segs, tim, base, stats, rows, summary, reducer=reducer)
        torch.cuda.synchronize()
        assert torch.equal(stats, want_stats), rep
        assert torch.equal(summary, want_sum), rep

    got = stats_to_numpy(stats)
    want_rows = []
    for ref, cands, dtype in data:
        want_rows += oracle.check_batch(synth.to_oracle_array(ref), [synth.to_oracle_array(c) for c in cands],
                                        ocode[dtype], 1e-2, 1e-2, threads=16)
    for p in range(rows):
        gu.assert_rows_equal(got[p], want_rows[p], "evaluate_segmented row %d" % p)
    valid = np.array([r["valid"] for r in want_rows], np.uint32)
    fit = oracle.fitness(tim.cpu().numpy(), base.cpu().numpy(), valid, reducer=reducer)
    for f in ("median_ms", "mean_ms", "speedup", "fitness"):
        assert got[f].tobytes() == fit[f].tobytes(), f
    pop = summary_to_numpy(summary)[0]
    assert int(pop["best_idx"]) == fit["best_idx"] and int(pop["n_valid"]) == fit["n_valid"]
    chk.close()
