"""Closed forms the synthetic populations fix by construction, checked on the CPU oracle
(reduced sizes except the tiny config).  No GPU, no GPU library."""
import numpy as np
import pytest
import torch

import oracle
import synth


def _rows(seg, atol, rtol):
    dt = oracle.BF16 if seg.dtype_name == "bf16" else oracle.F32
    ref = synth.to_oracle_array(seg.ref)
    return oracle.check_batch(ref, [synth.to_oracle_array(c) for c in seg.cands], dt, atol, rtol,
                              threads=4)


def _fitness(w, rows):
    valid = np.array([r["valid"] for r in rows], np.uint32)
    return oracle.fitness(w.timings.numpy(), w.baseline.numpy(), valid)


def test_config1_tiny_closed_form():
    w = synth.tiny("cpu")
    rows = _rows(w.segments[0], w.atol, w.rtol)
    assert [r["n_mismatch"] for r in rows] == [0, 0, 10, 1]
    assert [r["valid"] for r in rows] == [1, 1, 0, 0]
    assert [r["n_finite"] for r in rows] == [4096, 4096, 4096, 4095]
    assert [r["flags"] for r in rows] == [0, 0, 0, oracle.F_CAND_NAN | oracle.F_NAN_SITE_DIFF]
    assert rows[1]["max_abs_err"] == 0 and rows[1]["sum_abs_err"] == 0
    assert 1 - 1e-4 < rows[2]["max_abs_err"] < 1 + 1e-4
    assert 0 < rows[0]["max_abs_err"] < 1e-4
    f = _fitness(w, rows)
    assert f["n_valid"] == 2 and f["fitness"][2] == 0 and f["fitness"][3] == 0
    assert f["best_idx"] in (0, 1) and f["best_speedup"] >= 1.0
    assert np.all((f["median_ms"] >= 1) & (f["median_ms"] <= 2))


def test_config2_reduced():
    w = synth.dense_f32("cpu", side=256, P=8, T=100, corrupt_frac=1e-2)
    seg = w.segments[0]
    rows = _rows(seg, w.atol, w.rtol)
    for p, r in enumerate(rows):
        if seg.corrupted[p]:
            k = seg.notes["replaced"][p]
            assert 0.9 * k <= r["n_mismatch"] <= k and r["valid"] == 0
        else:
            assert r["n_mismatch"] == 0 and r["valid"] == 1
            assert r["max_rel_err"] < 1e-3
        assert r["flags"] == 0 and r["n_finite"] == seg.n
    f = _fitness(w, rows)
    assert f["n_valid"] == 6 and f["valid_rate"] == np.float32(0.75)
    assert not seg.corrupted[f["best_idx"]]


def test_config3_reduced_bf16():
    w = synth.softmax_bf16("cpu", B=4, R=16, C=512, P=16, T=100)
    seg = w.segments[0]
    ref = seg.ref.view(4, 16, 512).float()
    assert float(ref.min()) >= 0 and float(ref.max()) <= 1
    assert torch.allclose(ref.sum(-1), torch.ones(4, 16), atol=0.05)
    rows = _rows(seg, w.atol, w.rtol)
    assert seg.corrupted == [(p % 8) == 7 for p in range(16)]
    for p, r in enumerate(rows):
        assert r["valid"] == (0 if seg.corrupted[p] else 1), (p, r)
        assert r["flags"] == 0 and r["n_finite"] == seg.n
        if seg.corrupted[p]:
            assert r["n_mismatch"] <= 16 * 512
    assert any(r["max_abs_err"] > 0 for r in rows)


def test_config4_reduced_ragged():
    shapes = ((2, 8, 14, 14), (96, 96), (128, 1, 1), (4096,), (2, 3, 28, 28), (64, 64),
              (8, 16, 32), (1, 1000))
    w = synth.ragged_f32("cpu", shapes=shapes, P_s=8, T=100)
    assert w.P == 64
    all_rows = []
    for seg in w.segments:
        rows = _rows(seg, w.atol, w.rtol)
        for p, r in enumerate(rows):
            if seg.corrupted[p]:
                assert r["n_mismatch"] == seg.notes["bumped"][p] >= 1 and r["valid"] == 0
                assert 1 - 1e-3 < r["max_abs_err"] < 1 + 1e-3
            else:
                assert r["n_mismatch"] == 0 and r["valid"] == 1
            assert r["n_finite"] == seg.n
        all_rows += rows
    f = _fitness(w, all_rows)
    assert f["n_valid"] == 48 and f["valid_rate"] == np.float32(0.75)


def test_config5_reduced_heavy_tail():
    w = synth.heavy_tail_f32("cpu", log2n=16, P=8, T=1000)
    seg = w.segments[0]
    k = seg.notes["n_ref_nan"]
    assert k == 1024
    rows = _rows(seg, w.atol, w.rtol)
    base = oracle.F_CAND_NAN | oracle.F_CAND_INF | oracle.F_REF_NAN | oracle.F_REF_INF
    for p, r in enumerate(rows):
        assert r["valid"] == 0
        want = k
        flags = base
        if p in (2, 5):
            want += k
            flags |= oracle.F_NAN_SITE_DIFF
        if p == 6:
            want += 2 * k
            flags |= oracle.F_INF_DIFF
        assert r["n_mismatch"] == want, (p, r)
        assert r["flags"] == flags, (p, r)
        non_finite_sites = 3 * k + (k if p in (2, 5) else 0)
        assert r["n_finite"] == seg.n - non_finite_sites
        assert r["max_rel_err"] < 1e-4
    f = _fitness(w, rows)
    assert f["n_valid"] == 0 and f["best_idx"] == 8 and f["best_speedup"] == 1.0
    assert np.all(f["fitness"] == 0) and np.all(f["speedup"] > 0.5)
