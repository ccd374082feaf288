"""Helpers for the GPU parity tests: run a synthetic workload through the C ABI
(via the binding) and through the CPU oracle, and compare row by row."""
import math

import numpy as np
import torch

import oracle
import synth
import paper_2510_03760_amd as evo
from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy

# Relative tolerance of the two error sums (everything else is compared exactly).
# The kernel adds fp32 pairwise trees of a tile's 8 (fp32) or 16 (bf16) non-negative terms
# (<= 4 roundings, 4*2^-24 = 2.4e-7 relative) into fp64; the oracle adds every term in fp64.
SUM_RTOL = 1e-6

EXACT_INT_FIELDS = ("n_mismatch", "n_finite", "flags", "valid")
EXACT_F32_FIELDS = ("max_abs_err", "max_rel_err")
SUM_FIELDS = ("sum_abs_err", "sum_rel_err")


def dtype_code(seg):
    return {"bf16": evo.EVO_BF16, "f16": evo.EVO_F16, "f64": evo.EVO_F64, "i32": evo.EVO_I32,
            "i64": evo.EVO_I64}.get(seg.dtype_name, evo.EVO_F32)


def oracle_dtype(seg):
    return {"bf16": oracle.BF16, "f16": oracle.F16, "f64": oracle.F64, "i32": oracle.I32,
            "i64": oracle.I64}.get(seg.dtype_name, oracle.F32)


def oracle_rows(seg, atol, rtol, threads=16, chunk=1 << 24):
    """Oracle statistics for one segment; large tensors are copied to the host and
    fed chunk by chunk (the accumulator continues in index order)."""
    dt = oracle_dtype(seg)
    if seg.n <= chunk:
        ref = synth.to_oracle_array(seg.ref)
        return oracle.check_batch(ref, [synth.to_oracle_array(c) for c in seg.cands], dt, atol,
                                  rtol, threads=threads)
    from concurrent.futures import ThreadPoolExecutor
    accs = [oracle.CheckAccumulator(dt, atol, rtol) for _ in seg.cands]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        for lo in range(0, seg.n, chunk):
            hi = min(seg.n, lo + chunk)
            r = synth.to_oracle_array(seg.ref[lo:hi])
            list(ex.map(lambda pc: pc[0].feed(r, synth.to_oracle_array(pc[1][lo:hi])),
                        zip(accs, seg.cands)))
    return [a.result() for a in accs]


def assert_rows_equal(got_row, want, where=""):
    for f in EXACT_INT_FIELDS:
        assert int(got_row[f]) == int(want[f]), (where, f, int(got_row[f]), int(want[f]))
    for f in EXACT_F32_FIELDS:
        a, b = np.float32(got_row[f]), np.float32(want[f])
        assert a.tobytes() == b.tobytes(), (where, f, a, b)
    for f in SUM_FIELDS:
        a, b = float(got_row[f]), float(want[f])
        if math.isinf(b) or math.isnan(b):
            assert a == b, (where, f, a, b)
        else:
            assert abs(a - b) <= SUM_RTOL * abs(b), (where, f, a, b)
    n = int(got_row["n_elems_lo"]) | (int(got_row["n_elems_hi"]) << 32)
    assert n == int(want["n_elems"]), (where, "n_elems", n, want["n_elems"])


def run_check(w, segmented=None, stream=None):
    """Runs the check of every segment of workload `w` on the GPU.  One segment goes
    through evo_check_batch unless `segmented` is True; several always through
    evo_check_segmented.  Returns (Checker, stats tensor)."""
    segs = w.segments
    use_seg = segmented if segmented is not None else len(segs) > 1
    P = w.P
    chk = evo.Checker(dtype_code(segs[0]), segs[0].n, w.atol, w.rtol)
    stats = chk.new_stats(P)
    stats.fill_(0xAB)   # the call must overwrite every byte it owns
    if use_seg:
        row0, descs = 0, []
        for s in segs:
            descs.append({"ref": s.ref, "cand_ptrs": s.cands, "n_elems": s.n,
                          "dtype": dtype_code(s), "stats_row0": row0})
            row0 += len(s.cands)
        chk.check_segmented(descs, stats, P, stream=stream)
    else:
        assert len(segs) == 1
        chk.check_batch(segs[0].ref, segs[0].cands, stats, stream=stream)
    return chk, stats


def check_parity(w, segmented=None, oracle_threads=16, label=""):
    """GPU check vs oracle on every row of the workload; returns (chk, stats, oracle rows)."""
    chk, stats = run_check(w, segmented)
    torch.cuda.synchronize()
    got = stats_to_numpy(stats)
    want = []
    for s in w.segments:
        want += oracle_rows(s, w.atol, w.rtol, threads=oracle_threads)
    assert len(got) == len(want)
    for p, (g, o) in enumerate(zip(got, want)):
        assert_rows_equal(g, o, "%s %s row %d" % (label, w.name, p))
        for f in ("median_ms", "mean_ms", "speedup", "fitness"):
            assert float(g[f]) == 0.0
    return chk, stats, want


def fitness_parity(chk, stats, timings, baseline, want_rows=None, label=""):
    """evo_fitness on the GPU vs the oracle, bit for bit (uses the valid flags that
    are in `stats`)."""
    summary = chk.new_summary()
    summary.fill_(0xCD)
    before = stats_to_numpy(stats).copy()
    chk.fitness(timings, baseline, stats, summary)
    torch.cuda.synchronize()
    got = stats_to_numpy(stats)
    pop = summary_to_numpy(summary)[0]
    valid = before["valid"].astype(np.uint32)
    want = oracle.fitness(timings.cpu().numpy(), baseline.cpu().numpy(), valid)
    for f in ("median_ms", "mean_ms", "speedup", "fitness"):
        assert got[f].tobytes() == want[f].tobytes(), (label, f, got[f], want[f])
    for f in ("n_mismatch", "n_finite", "sum_abs_err", "sum_rel_err", "max_abs_err",
              "max_rel_err", "flags", "valid", "n_elems_lo", "n_elems_hi"):
        assert got[f].tobytes() == before[f].tobytes(), (label, f, "must be left untouched")
    assert int(pop["best_idx"]) == want["best_idx"], (label, pop, want)
    assert int(pop["n_valid"]) == want["n_valid"], (label, pop, want)
    assert np.float32(pop["best_speedup"]).tobytes() == np.float32(want["best_speedup"]).tobytes()
    assert np.float32(pop["valid_rate"]).tobytes() == np.float32(want["valid_rate"]).tobytes()
    return got, pop, want
