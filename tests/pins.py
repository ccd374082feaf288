"""Pins for the CPU oracle: checks whose expected values come from hand-written
fixtures, library routines or mathematics, never from the oracle itself.

Every function takes the oracle as an argument (a module-like object with
``check_one``, ``check_batch``, ``fitness`` and the flag constants), so that the same
pins can be pointed at deliberately broken copies of it (test_oracle_mutants.py).
Each raises AssertionError on a violated pin.
"""
import json
import math
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")

_F = np.float32
SPECIAL = {
    "+0": _F(0.0), "-0": _F(-0.0), "1": _F(1.0), "1+ulp": np.nextafter(_F(1), _F(2)),
    "-1": _F(-1.0), "FLT_MIN": _F(1.17549435e-38), "DENORM_MIN": _F(1e-45),
    "FLT_MAX": _F(3.4028234663852886e38), "+Inf": _F(np.inf), "-Inf": _F(-np.inf),
    "NaN": _F(np.nan),
}


def _num(x):
    """A JSON number, "inf"/"nan", or a C99 hexadecimal literal ("0x1.8p-3": exact)."""
    if isinstance(x, str) and "0x" in x:
        return float.fromhex(x)
    return float(x)


def _arr(xs):
    return np.array([_num(x) for x in xs], dtype=np.float32)


def _same_f32(a, b):
    a, b = np.float32(a), np.float32(b)
    return a.tobytes() == b.tobytes()


def pin_truth_table(orc):
    """121 special-value pairs against the hand-written match matrix."""
    rows = []
    with open(os.path.join(GOLDEN, "match_truth_table.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rows.append(line.split())
    assert rows[0][0] == "values:"
    names = rows[0][1:]
    assert len(names) == 11 and len(rows) == 12
    for row in rows[1:]:
        rname, cells = row[0], row[1:]
        assert len(cells) == 11
        for cname, cell in zip(names, cells):
            r = np.array([SPECIAL[rname]], np.float32)
            c = np.array([SPECIAL[cname]], np.float32)
            got = orc.check_one(r, c, orc.F32, 0.25, 0.25)
            want_mismatch = 0 if cell == "M" else 1
            assert got["n_mismatch"] == want_mismatch, (rname, cname, got)
            assert got["valid"] == 1 - want_mismatch, (rname, cname, got)


def pin_flag_classes(orc):
    """Flag bits and statistics membership for each pair of value classes."""
    bit = {"CN": orc.F_CAND_NAN, "CI": orc.F_CAND_INF, "RN": orc.F_REF_NAN,
           "RI": orc.F_REF_INF, "ND": orc.F_NAN_SITE_DIFF, "ID": orc.F_INF_DIFF}
    val = {"fin": 2.0, "+inf": np.inf, "-inf": -np.inf, "nan": np.nan}
    seen = 0
    with open(os.path.join(GOLDEN, "flag_classes.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            rcls, ccls, flags, in_stats = line.split()
            want = 0
            if flags != "-":
                for name in flags.split(","):
                    want |= bit[name]
            cv = 2.5 if ccls == "fin" else val[ccls]
            for code, npdt in ((orc.F32, np.float32), (orc.F64, np.float64)):   # same classes in binary64
                got = orc.check_one(np.array([val[rcls]], npdt), np.array([cv], npdt), code, 1.0, 1.0)
                assert got["flags"] == want, (rcls, ccls, npdt, got)
                assert got["n_finite"] == int(in_stats), (rcls, ccls, npdt, got)
            seen += 1
    assert seen == 16


def _load_examples():
    with open(os.path.join(GOLDEN, "worked_examples.json")) as fh:
        return json.load(fh)


def pin_worked_check_examples(orc):
    for ex in _load_examples()["check"]:
        if ex["dtype"] in ("bf16", "f16"):
            r = np.array(ex["ref_bits"], dtype=np.uint16)
            c = np.array(ex["cand_bits"], dtype=np.uint16)
            dt = orc.BF16 if ex["dtype"] == "bf16" else orc.F16
        elif ex["dtype"] == "f64":
            r = np.array([_num(x) for x in ex["ref"]], dtype=np.float64)
            c = np.array([_num(x) for x in ex["cand"]], dtype=np.float64)
            dt = orc.F64
        else:
            r, c, dt = _arr(ex["ref"]), _arr(ex["cand"]), orc.F32
            if ex["name"].startswith("product_rounds"):   # these inputs must be exact in binary32
                assert [float(v) for v in r] == [_num(x) for x in ex["ref"]], ex["name"]
                assert [float(v) for v in c] == [_num(x) for x in ex["cand"]], ex["name"]
        atol, rtol = _num(ex["atol"]), _num(ex["rtol"])
        assert float(np.float32(atol)) == atol and float(np.float32(rtol)) == rtol, ex["name"]
        got = orc.check_one(r, c, dt, atol, rtol)
        for key in ("n_mismatch", "n_finite", "valid", "flags"):
            assert got[key] == ex[key], (ex["name"], key, got)
        for key in ("max_abs_err", "max_rel_err"):
            assert _same_f32(got[key], _num(ex[key])), (ex["name"], key, got)
        for key in ("sum_abs_err", "sum_rel_err"):
            assert got[key] == _num(ex[key]), (ex["name"], key, got)


def pin_worked_fitness_examples(orc):
    for ex in _load_examples()["fitness"]:
        got = orc.fitness(np.array(ex["timings"], np.float32),
                          np.array(ex["baseline"], np.float32),
                          np.array(ex["valid"], np.uint32))
        for key in ("median_ms", "mean_ms", "speedup", "fitness"):
            want = np.array(ex[key], np.float32)
            assert got[key].tobytes() == want.tobytes(), (ex["name"], key, got[key], want)
        assert got["best_idx"] == ex["best_idx"], (ex["name"], got)
        assert got["n_valid"] == ex["n_valid"], (ex["name"], got)
        assert _same_f32(got["best_speedup"], ex["best_speedup"]), (ex["name"], got)
        assert _same_f32(got["valid_rate"], ex["valid_rate"]), (ex["name"], got)


def _mixed_pair(rng, n):
    """Reference/candidate pair with close values, far values and special sites."""
    r = rng.standard_normal(n).astype(np.float32) * np.float32(3)
    c = (r * (1 + 0.02 * rng.standard_normal(n))).astype(np.float32)
    far = rng.random(n) < 0.1
    c[far] = rng.uniform(-10, 10, far.sum()).astype(np.float32)
    for arr in (r, c):
        k = max(1, n // 50)
        arr[rng.integers(0, n, k)] = np.inf
        arr[rng.integers(0, n, k)] = -np.inf
        arr[rng.integers(0, n, k)] = np.nan
        arr[rng.integers(0, n, k)] = 0.0
        arr[rng.integers(0, n, k)] = np.float32(1e-41)
    same = rng.random(n) < 0.2
    c[same] = r[same]
    return r, c


def pin_numpy_isclose(orc):
    """The mismatch count is the complement of numpy.isclose in binary32."""
    rng = np.random.default_rng(1234)
    for n, atol, rtol in ((1, 1e-2, 1e-2), (257, 1e-2, 1e-2), (4099, 0.0, 3e-2),
                          (4099, 5e-2, 0.0), (1000, 0.0, 0.0)):
        r, c = _mixed_pair(rng, n)
        with np.errstate(all="ignore"):
            close = np.isclose(c, r, rtol=np.float32(rtol), atol=np.float32(atol), equal_nan=False)
        got = orc.check_one(r, c, orc.F32, atol, rtol)
        assert got["n_mismatch"] == int((~close).sum()), (n, atol, rtol, got)
        both = np.isfinite(r) & np.isfinite(c)
        assert got["n_finite"] == int(both.sum())
        assert got["n_elems"] == n


def pin_sums_and_maxima(orc):
    """Sums against exact summation (math.fsum), maxima against an element scan
    written with Python scalars (no shared code path with the C loop)."""
    rng = np.random.default_rng(99)
    r, c = _mixed_pair(rng, 3001)
    got = orc.check_one(r, c, orc.F32, 1e-2, 1e-2)
    ds, qs = [], []
    for ri, ci in zip(r, c):
        if not (np.isfinite(ri) and np.isfinite(ci)):
            continue
        d = np.float32(abs(np.float32(ci - ri)))
        ar = np.float32(abs(ri))
        q = np.float32(d * np.float32(np.float32(1) / ar)) if ar >= np.float32(1.17549435e-38) else np.float32(0)
        ds.append(float(d))
        qs.append(float(q))
    assert _same_f32(got["max_abs_err"], max(ds))
    assert _same_f32(got["max_rel_err"], max(qs))
    for key, terms in (("sum_abs_err", ds), ("sum_rel_err", qs)):
        exact = math.fsum(terms)
        assert abs(got[key] - exact) <= 1e-12 * exact, (key, got[key], exact)


def pin_invariants(orc):
    rng = np.random.default_rng(7)
    r = rng.standard_normal(5000).astype(np.float32)
    # identical candidate: nothing differs
    got = orc.check_one(r, r.copy(), orc.F32, 0.0, 0.0)
    assert got["n_mismatch"] == 0 and got["valid"] == 1 and got["flags"] == 0
    assert got["max_abs_err"] == 0 and got["max_rel_err"] == 0
    assert got["sum_abs_err"] == 0 and got["sum_rel_err"] == 0 and got["n_finite"] == 5000
    # one NaN anywhere makes the candidate invalid, whatever the tolerance
    c = r.copy()
    c[1234] = np.nan
    got = orc.check_one(r, c, orc.F32, 1e30, 1e30)
    assert got["valid"] == 0 and got["n_mismatch"] == 1
    assert got["flags"] == orc.F_CAND_NAN | orc.F_NAN_SITE_DIFF
    # NaN in the reference at the same site does not excuse it
    r2 = r.copy()
    r2[1234] = np.nan
    got = orc.check_one(r2, c, orc.F32, 1e30, 1e30)
    assert got["valid"] == 0 and got["n_mismatch"] == 1
    assert got["flags"] == orc.F_CAND_NAN | orc.F_REF_NAN
    # monotone in each tolerance
    c = (r + 0.05 * rng.standard_normal(5000)).astype(np.float32)
    grid = [0.0, 1e-3, 1e-2, 3e-2, 1e-1, 1.0]
    for fixed in (0.0, 1e-2):
        prev_a = prev_r = None
        for t in grid:
            ma = orc.check_one(r, c, orc.F32, t, fixed)["n_mismatch"]
            mr = orc.check_one(r, c, orc.F32, fixed, t)["n_mismatch"]
            assert prev_a is None or ma <= prev_a
            assert prev_r is None or mr <= prev_r
            prev_a, prev_r = ma, mr
    assert orc.check_one(r, c, orc.F32, 0.0, 0.0)["n_mismatch"] > 0
    assert orc.check_one(r, c, orc.F32, 1.0, 0.0)["n_mismatch"] == 0
    # candidate order only permutes rows
    cands = [(r + s * rng.standard_normal(5000)).astype(np.float32) for s in (0, 1e-3, 1e-1)]
    rows = orc.check_batch(r, cands, orc.F32, 1e-2, 1e-2)
    rows_rev = orc.check_batch(r, cands[::-1], orc.F32, 1e-2, 1e-2)
    assert rows == rows_rev[::-1]
    # chunked feeding equals one pass (sums continue in index order: bit-identical)
    rr, cc = _mixed_pair(rng, 4001)
    whole = orc.check_one(rr, cc, orc.F32, 1e-2, 1e-2)
    acc = orc.CheckAccumulator(orc.F32, 1e-2, 1e-2)
    for lo, hi in ((0, 1), (1, 1000), (1000, 1000), (1000, 4001)):
        acc.feed(rr[lo:hi], cc[lo:hi])
    assert acc.result() == whole
    # every element is either in the statistics set or has a non-finite side
    nonfinite = int((~(np.isfinite(rr) & np.isfinite(cc))).sum())
    assert whole["n_finite"] + nonfinite == 4001
    # empty tensor
    e = orc.check_one(np.zeros(0, np.float32), np.zeros(0, np.float32), orc.F32, 0.0, 0.0)
    assert e["valid"] == 1 and e["n_mismatch"] == 0 and e["n_finite"] == 0


def pin_bf16_widening(orc):
    """bf16 inputs give exactly what the same values give as binary32."""
    rng = np.random.default_rng(5)
    bits_r = rng.integers(0, 1 << 16, 20000).astype(np.uint16)
    bits_c = bits_r.copy()
    move = rng.random(20000) < 0.5
    bits_c[move] = (bits_c[move].astype(np.int32) + rng.integers(-3, 4, move.sum())).clip(0, 65535).astype(np.uint16)
    r32 = (bits_r.astype(np.uint32) << 16).view(np.float32)
    c32 = (bits_c.astype(np.uint32) << 16).view(np.float32)
    a = orc.check_one(bits_r, bits_c, orc.BF16, 1e-2, 1e-2)
    b = orc.check_one(r32, c32, orc.F32, 1e-2, 1e-2)
    assert a == b and a["flags"] != 0  # random bits include Inf and NaN patterns


def pin_f16_widening(orc):
    """binary16 inputs: every one of the 65536 bit patterns widens as numpy's float16 does,
    and a check on halves equals the check on the same values as binary32."""
    all_bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = all_bits.view(np.float16).astype(np.float32)
    for b in range(0, 65536, 1):
        got = orc.half_to_float(b)
        w = want[b]
        assert (np.isnan(got) and np.isnan(w)) or got.tobytes() == w.tobytes(), hex(b)
    rng = np.random.default_rng(8)
    bits_r = rng.integers(0, 1 << 16, 20000).astype(np.uint16)
    bits_c = bits_r.copy()
    move = rng.random(20000) < 0.5
    bits_c[move] = (bits_c[move].astype(np.int32) + rng.integers(-3, 4, move.sum())).clip(0, 65535).astype(np.uint16)
    a = orc.check_one(bits_r, bits_c, orc.F16, 1e-2, 1e-2)
    b = orc.check_one(bits_r.view(np.float16).astype(np.float32),
                      bits_c.view(np.float16).astype(np.float32), orc.F32, 1e-2, 1e-2)
    assert a == b and a["flags"] != 0


def _rank_select(row, k):
    """k-th smallest by counting, O(T^2): no sort involved."""
    T = len(row)
    for i in range(T):
        rank = sum(1 for j in range(T) if row[j] < row[i] or (row[j] == row[i] and j < i))
        if rank == k:
            return row[i]
    raise AssertionError("no element of rank %d" % k)


def pin_median_and_speedup(orc):
    rng = np.random.default_rng(11)
    for T in (1, 2, 5, 100, 101, 1000):
        P = 7
        t = np.exp(0.1 * rng.standard_normal((P, T))).astype(np.float32)
        t[3] = t[2]                      # duplicate row
        t[4, : max(1, T // 3)] = t[4, 0]  # many equal samples
        b = np.exp(0.1 * rng.standard_normal(T)).astype(np.float32)
        valid = np.array([1, 0, 1, 1, 1, 1, 0], np.uint32)
        got = orc.fitness(t, b, valid)
        for p in range(P):
            row = [np.float32(x) for x in t[p]]
            if T % 2:
                want = _rank_select(row, T // 2)
            else:
                want = np.float32(0.5) * np.float32(_rank_select(row, T // 2 - 1) + _rank_select(row, T // 2))
            assert _same_f32(got["median_ms"][p], want), (T, p)
            assert _same_f32(got["median_ms"][p], np.median(t[p])), (T, p)
            exact_mean = math.fsum(float(x) for x in t[p]) / T
            assert abs(float(got["mean_ms"][p]) - exact_mean) <= 2.0 ** -23 * exact_mean
        bm = np.median(b)
        assert _same_f32(got["base_median_ms"], bm)
        for p in range(P):
            assert _same_f32(got["speedup"][p], np.float32(bm) / got["median_ms"][p])
            assert _same_f32(got["fitness"][p], got["speedup"][p] if valid[p] else 0.0)
        assert got["n_valid"] == 5 and _same_f32(got["valid_rate"], np.float32(5) / np.float32(7))
        fit = got["fitness"]
        assert got["best_idx"] == int(np.argmax(fit))  # argmax returns the first maximum
        assert _same_f32(got["best_speedup"], max(np.float32(1), fit.max()))
    # closed forms: identical rows -> speedup exactly 1; doubling a row halves it
    row = np.exp(0.1 * rng.standard_normal(100)).astype(np.float32)
    got = orc.fitness(np.stack([row, row * 2, row[::-1].copy()]), row, np.ones(3, np.uint32))
    assert got["speedup"].tolist() == [1.0, 0.5, 1.0]
    assert got["best_idx"] == 0
    # one huge outlier (the largest sample made 1000x larger) moves the mean, not the median
    row2 = row.copy()
    row2[int(np.argmax(row))] *= 1000
    g1 = orc.fitness(row[None, :], row, np.ones(1, np.uint32))
    g2 = orc.fitness(row2[None, :], row, np.ones(1, np.uint32))
    assert _same_f32(g1["median_ms"][0], g2["median_ms"][0])
    assert g2["mean_ms"][0] > 2 * g1["mean_ms"][0]


def pin_unusable_timing_rows(orc):
    """A row with a NaN, an Inf, a zero or a negative sample has no median."""
    base = np.array([1, 2, 3, 4], np.float32)
    rows = np.array([[1, 2, 3, 4], [1, np.nan, 3, 4], [1, 2, np.inf, 4], [0, 2, 3, 4],
                     [1, 2, 3, -4]], np.float32)
    got = orc.fitness(rows, base, np.ones(5, np.uint32))
    qnan = np.array([0x7FC00000], np.uint32).view(np.float32)[0]
    for p in range(1, 5):
        assert _same_f32(got["median_ms"][p], qnan) and _same_f32(got["mean_ms"][p], qnan)
        assert got["speedup"][p] == 0 and got["fitness"][p] == 0
    assert got["speedup"][0] == 1.0 and got["best_idx"] == 0 and got["n_valid"] == 5
    bad_base = orc.fitness(rows[:1], np.array([1, 2, 3, np.nan], np.float32), np.ones(1, np.uint32))
    assert bad_base["speedup"][0] == 0 and bad_base["fitness"][0] == 0 and bad_base["best_idx"] == 1
    assert bad_base["median_ms"][0] == 2.5


def pin_select_elite(orc):
    """Elite selection against a stable library sort and a hand-made case."""
    f = np.array([0.5, 2.0, 0.0, 2.0, 1.5, 0.0, 3.0, 2.0], np.float32)
    got = orc.select_elite(f, 4)
    assert got["elite"].tolist() == [6, 1, 3, 7] and got["n_elite"] == 4   # ties in index order
    got = orc.select_elite(f, 8)
    assert got["elite"].tolist() == [6, 1, 3, 7, 4, 0, 8, 8] and got["n_elite"] == 6
    got = orc.select_elite(np.zeros(5, np.float32), 3)
    assert got["elite"].tolist() == [5, 5, 5] and got["n_elite"] == 0
    got = orc.select_elite(np.array([1.0], np.float32), 1)
    assert got["elite"].tolist() == [0] and got["n_elite"] == 1
    rng = np.random.default_rng(3)
    for P, k in ((1, 1), (17, 4), (256, 8), (1000, 1000), (333, 50)):
        f = rng.choice(np.array([0, 0.5, 0.75, 1, 1.25, 2, np.inf], np.float32), P)
        some = rng.random(P) < 0.3
        f[some] = rng.random(int(some.sum())).astype(np.float32)
        order = np.lexsort((np.arange(P), -f.astype(np.float64)))   # stable: fitness desc, index asc
        order = [int(i) for i in order if f[i] > 0][:k]
        got = orc.select_elite(f, k)
        assert got["n_elite"] == len(order)
        assert got["elite"].tolist() == order + [P] * (k - len(order)), (P, k)


_D = np.float64
SPECIAL64 = {   # the binary64 analogues of SPECIAL, under the same names
    "+0": _D(0.0), "-0": _D(-0.0), "1": _D(1.0), "1+ulp": np.nextafter(_D(1), _D(2)),
    "-1": _D(-1.0), "FLT_MIN": _D(2.2250738585072014e-308), "DENORM_MIN": _D(5e-324),
    "FLT_MAX": _D(1.7976931348623157e308), "+Inf": _D(np.inf), "-Inf": _D(-np.inf),
    "NaN": _D(np.nan),
}


def pin_f64_truth_table(orc):
    """The hand-written match matrix holds for the binary64 analogues of its values too
    (the worked tolerances of the fixture carry over: 0.25 + fl(0.25*(1+2^-52)) rounds
    to 0.5, and 0.25*DBL_MAX is far below DBL_MAX - 1)."""
    rows = []
    with open(os.path.join(GOLDEN, "match_truth_table.txt")) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    names = rows[0][1:]
    for row in rows[1:]:
        for cname, cell in zip(names, row[1:]):
            r = np.array([SPECIAL64[row[0]]], np.float64)
            c = np.array([SPECIAL64[cname]], np.float64)
            got = orc.check_one(r, c, orc.F64, 0.25, 0.25)
            assert got["n_mismatch"] == (0 if cell == "M" else 1), (row[0], cname, got)


def _mixed_pair64(rng, n):
    r = rng.standard_normal(n) * 3.0
    c = r * (1 + 0.02 * rng.standard_normal(n))
    far = rng.random(n) < 0.1
    c[far] = rng.uniform(-10, 10, far.sum())
    for arr in (r, c):
        k = max(1, n // 50)
        arr[rng.integers(0, n, k)] = np.inf
        arr[rng.integers(0, n, k)] = -np.inf
        arr[rng.integers(0, n, k)] = np.nan
        arr[rng.integers(0, n, k)] = 0.0
        arr[rng.integers(0, n, k)] = 1e-310            # subnormal
        arr[rng.integers(0, n, k)] = 1e-40             # below the binary32 range, normal here
    same = rng.random(n) < 0.2
    c[same] = r[same]
    return r, c


def pin_f64_numpy_isclose_sums_maxima(orc):
    """binary64 tensors: mismatches against numpy.isclose in binary64 (tolerances are the
    binary32 values, widened), sums against math.fsum, maxima against a scan with Python
    floats, rounded to binary32 at the end."""
    rng = np.random.default_rng(4321)
    for n, atol, rtol in ((1, 1e-2, 1e-2), (4099, 1e-2, 1e-2), (4099, 0.0, 3e-2), (2000, 5e-2, 0.0),
                          (1000, 0.0, 0.0), (3000, 1e-9, 1e-9)):
        r, c = _mixed_pair64(rng, n)
        a64, r64 = float(np.float32(atol)), float(np.float32(rtol))
        with np.errstate(all="ignore"):
            close = np.isclose(c, r, rtol=r64, atol=a64, equal_nan=False)
        got = orc.check_one(r, c, orc.F64, atol, rtol)
        assert got["n_mismatch"] == int((~close).sum()), (n, atol, rtol, got)
        both = np.isfinite(r) & np.isfinite(c)
        assert got["n_finite"] == int(both.sum()) and got["n_elems"] == n
        ds, qs = [], []
        for ri, ci in zip(r.tolist(), c.tolist()):
            if not (math.isfinite(ri) and math.isfinite(ci)):
                continue
            d = abs(ci - ri)
            q = d * (1.0 / abs(ri)) if abs(ri) >= 2.2250738585072014e-308 else 0.0
            ds.append(d)
            qs.append(q)
        if ds:
            with np.errstate(over="ignore"):     # beyond the binary32 range: +Inf, as intended
                assert _same_f32(got["max_abs_err"], np.float32(max(ds))), (n, got)
                assert _same_f32(got["max_rel_err"], np.float32(max(qs))), (n, got)
            for key, terms in (("sum_abs_err", ds), ("sum_rel_err", qs)):
                exact = math.fsum(terms)
                assert abs(got[key] - exact) <= 1e-12 * exact, (key, got[key], exact)
    # the relative error is d * (1/|r|), two roundings -- not d / |r| (one element: the sum
    # is the term itself, in binary64)
    pairs = [(float(a), float(d)) for a in range(3, 60) for d in range(1, 60)
             if d * (1.0 / a) != d / a]
    assert len(pairs) > 20
    for a, d in pairs[:20]:
        got = orc.check_one(np.array([a]), np.array([a + d]), orc.F64, 0.0, 0.0)
        assert got["sum_rel_err"] == d * (1.0 / a) and got["sum_abs_err"] == d
    # a difference binary32 cannot tell apart decides here
    r = np.array([1.0], np.float64)
    c = np.array([1.0 + 2.0 ** -40], np.float64)
    assert orc.check_one(r, c, orc.F64, 0.0, 0.0)["n_mismatch"] == 1
    assert orc.check_one(r, c, orc.F64, 0.0, 1e-6)["n_mismatch"] == 0
    # a maximum beyond the binary32 range is reported as +Inf, the sum stays finite
    got = orc.check_one(np.array([0.0, 1.0]), np.array([1e300, 1.0]), orc.F64, 0.0, 0.0)
    assert np.isposinf(got["max_abs_err"]) and got["sum_abs_err"] == 1e300 and got["n_finite"] == 2
    # relative error is dropped below DBL_MIN, kept at DBL_MIN
    got = orc.check_one(np.array([2.0e-308]), np.array([0.0]), orc.F64, 1.0, 0.0)
    assert got["max_rel_err"] == 0 and got["sum_rel_err"] == 0
    got = orc.check_one(np.array([2.2250738585072014e-308]), np.array([0.0]), orc.F64, 1.0, 0.0)
    assert got["max_rel_err"] == 1.0
    # chunked feeding equals one pass
    rr, cc = _mixed_pair64(rng, 3001)
    whole = orc.check_one(rr, cc, orc.F64, 1e-2, 1e-2)
    acc = orc.CheckAccumulator(orc.F64, 1e-2, 1e-2)
    for lo, hi in ((0, 7), (7, 7), (7, 2000), (2000, 3001)):
        acc.feed(rr[lo:hi], cc[lo:hi])
    assert acc.result() == whole


def pin_f64_agrees_with_f32_where_both_are_exact(orc):
    """On a dyadic grid (multiples of 2^-6 in [-8, 8], tolerances 2^-2) every operation of the
    match rule and of the absolute statistics is exact in both precisions, so checking the
    same values as binary64 and as binary32 tensors must give the same numbers."""
    rng = np.random.default_rng(64)
    r = rng.integers(-512, 513, 5000) / 64.0
    c = r + rng.integers(-200, 201, 5000) / 64.0
    g64 = orc.check_one(r, c, orc.F64, 0.25, 0.25)
    g32 = orc.check_one(r.astype(np.float32), c.astype(np.float32), orc.F32, 0.25, 0.25)
    for key in ("n_mismatch", "n_finite", "sum_abs_err", "flags", "valid"):
        assert g64[key] == g32[key], key
    assert _same_f32(g64["max_abs_err"], g32["max_abs_err"])
    want = int((np.abs(c - r) > 0.25 + 0.25 * np.abs(r)).sum())
    assert g64["n_mismatch"] == want and want > 0


def pin_integer_equality(orc):
    """Integer tensors: exact equality; |c - r| as an exact integer (Python ints), its
    maximum rounded to binary32 by numpy, its sum exact while it fits 2^53."""
    rng = np.random.default_rng(5)
    for code, npdt, lo, hi in ((orc.I32, np.int32, -2 ** 31, 2 ** 31 - 1), (orc.I64, np.int64, -2 ** 63, 2 ** 63 - 1)):
        for n in (1, 63, 4099):
            r = rng.integers(-1000, 1000, n).astype(npdt)
            c = r.copy()
            sites = rng.random(n) < 0.3
            c[sites] += rng.integers(-5, 6, int(sites.sum())).astype(npdt)   # some of these are +0
            got = orc.check_one(r, c, code, 123.0, 456.0)                      # tolerances play no part
            diffs = [abs(int(ci) - int(ri)) for ri, ci in zip(r, c)]
            assert got["n_mismatch"] == sum(1 for d in diffs if d) == int(np.count_nonzero(c != r))
            assert got["n_finite"] == n and got["n_elems"] == n and got["flags"] == 0
            assert got["valid"] == (1 if not any(diffs) else 0)
            assert _same_f32(got["max_abs_err"], np.float32(max(diffs)))
            assert got["sum_abs_err"] == float(sum(diffs))
            assert got["max_rel_err"] == 0 and got["sum_rel_err"] == 0
        # extremes: the magnitude needs one bit more than the type has
        r = np.array([lo, hi, lo, 0, -1], npdt)
        c = np.array([hi, lo, lo, hi, hi], npdt)
        got = orc.check_one(r, c, code, 0.0, 0.0)
        diffs = [abs(int(ci) - int(ri)) for ri, ci in zip(r, c)]
        assert diffs[0] == hi - lo
        assert got["n_mismatch"] == 4
        assert _same_f32(got["max_abs_err"], np.float32(float(max(diffs))))   # 2^32 and 2^64
        assert abs(got["sum_abs_err"] - float(sum(diffs))) <= 4 * 2.0 ** -53 * float(sum(diffs))
        # values that differ only beyond 24 or 53 bits are still different
        r = np.array([2 ** 30], npdt)
        c = np.array([2 ** 30 + 1], npdt)
        assert orc.check_one(r, c, code, 1e30, 1e30)["n_mismatch"] == 1
        # identical, empty, chunked
        r = rng.integers(lo // 2, hi // 2, 1000).astype(npdt)
        got = orc.check_one(r, r.copy(), code, 0.0, 0.0)
        assert got["valid"] == 1 and got["max_abs_err"] == 0 and got["sum_abs_err"] == 0
        e = orc.check_one(np.zeros(0, npdt), np.zeros(0, npdt), code, 0.0, 0.0)
        assert e["valid"] == 1 and e["n_finite"] == 0
        c = r.copy()
        c[::7] -= 3
        whole = orc.check_one(r, c, code, 0.0, 0.0)
        acc = orc.CheckAccumulator(code, 0.0, 0.0)
        for a, b in ((0, 1), (1, 500), (500, 1000)):
            acc.feed(r[a:b], c[a:b])
        assert acc.result() == whole and whole["n_mismatch"] == len(range(0, 1000, 7))
    # 2^40 + 1 needs int64: as int32 data it cannot even be written, as int64 it is one mismatch
    got = orc.check_one(np.array([2 ** 40], np.int64), np.array([2 ** 40 + 1], np.int64), orc.I64, 0.0, 0.0)
    assert got["n_mismatch"] == 1 and got["max_abs_err"] == 1.0


def pin_mean_reducer(orc):
    """Speedup as a ratio of means (the "average" reading of Sec. 4.3) on samples whose sums
    are exact in any order, so the expected values are closed forms."""
    t = np.array([[1, 2, 9], [2, 2, 2], [4, 4, 4], [1, 1, np.nan]], np.float32)
    b = np.array([2, 4, 6], np.float32)
    valid = np.array([1, 1, 0, 1], np.uint32)
    got = orc.fitness(t, b, valid, reducer=orc.REDUCE_MEAN)
    assert got["mean_ms"][:3].tolist() == [4.0, 2.0, 4.0] and got["median_ms"][:3].tolist() == [2.0, 2.0, 4.0]
    assert got["speedup"].tolist() == [1.0, 2.0, 1.0, 0.0]          # 4/4, 4/2, 4/4, unusable row
    assert got["fitness"].tolist() == [1.0, 2.0, 0.0, 0.0]
    assert got["best_idx"] == 1 and got["best_speedup"] == 2.0 and got["n_valid"] == 3
    med = orc.fitness(t, b, valid)                                   # default: ratio of medians
    assert med["speedup"].tolist() == [2.0, 2.0, 1.0, 0.0]
    assert orc.fitness(t, b, valid, reducer=orc.REDUCE_MEDIAN)["speedup"].tolist() == med["speedup"].tolist()
    # random dyadic samples: every partial sum is exact, so the mean is fl32(sum / T) exactly
    rng = np.random.default_rng(17)
    T = 100
    t = (rng.integers(1, 4096, (5, T)) / 1024.0).astype(np.float32)
    b = (rng.integers(1, 4096, T) / 1024.0).astype(np.float32)
    got = orc.fitness(t, b, np.ones(5, np.uint32), reducer=orc.REDUCE_MEAN)
    bm = np.float32(float(b.astype(np.float64).sum()) / T)
    for p in range(5):
        m = np.float32(float(t[p].astype(np.float64).sum()) / T)
        assert _same_f32(got["mean_ms"][p], m)
        assert _same_f32(got["speedup"][p], bm / m)


def pin_select_elite_diverse(orc):
    """Diversity-keeping elite selection against a stable library sort with first-occurrence
    filtering, and a hand-made case."""
    f = np.array([0.5, 2.0, 0.0, 2.0, 1.5, 0.0, 3.0, 2.0, 3.0], np.float32)
    keys = np.array([7, 1, 1, 1, 2, 9, 3, 4, 3], np.uint32)
    got = orc.select_elite_diverse(f, keys, 4)
    # 6 (3.0, key 3) ; 8 has key 3 again ; 1 (2.0, key 1) ; 3 has key 1 again ; 7 (2.0, key 4) ; 4
    assert got["elite"].tolist() == [6, 1, 7, 4] and got["n_elite"] == 4
    got = orc.select_elite_diverse(f, keys, 9)
    assert got["elite"].tolist() == [6, 1, 7, 4, 0, 9, 9, 9, 9] and got["n_elite"] == 5
    # all keys different: the plain selection; all keys equal: only the best
    assert orc.select_elite_diverse(f, np.arange(9, dtype=np.uint32), 4)["elite"].tolist() == \
        orc.select_elite(f, 4)["elite"].tolist()
    got = orc.select_elite_diverse(f, np.zeros(9, np.uint32), 3)
    assert got["elite"].tolist() == [6, 9, 9] and got["n_elite"] == 1
    # an infeasible candidate does not block its key
    got = orc.select_elite_diverse(np.array([0.0, 1.0], np.float32), np.array([5, 5], np.uint32), 2)
    assert got["elite"].tolist() == [1, 2] and got["n_elite"] == 1
    rng = np.random.default_rng(8)
    for P, k, nkeys in ((1, 1, 1), (17, 4, 5), (256, 8, 30), (1000, 1000, 400), (333, 50, 10)):
        f = rng.choice(np.array([0, 0.5, 0.75, 1, 1.25, 2, np.inf], np.float32), P)
        some = rng.random(P) < 0.3
        f[some] = rng.random(int(some.sum())).astype(np.float32)
        keys = rng.integers(0, nkeys, P).astype(np.uint32) * np.uint32(2654435761)
        order = np.lexsort((np.arange(P), -f.astype(np.float64)))
        want, seen = [], set()
        for i in order:
            if f[i] > 0 and int(keys[i]) not in seen:
                seen.add(int(keys[i]))
                want.append(int(i))
        want = want[:k]
        got = orc.select_elite_diverse(f, keys, k)
        assert got["n_elite"] == len(want)
        assert got["elite"].tolist() == want + [P] * (k - len(want)), (P, k)


def pin_tolerance_policy(orc):
    """Every group of a launch is checked with the pair of its element type, or of the class it
    names: the hand-built example, groups against single checks with the pair written out,
    and an unset class is an error."""
    dt = {"f32": (orc.F32, np.float32), "bf16": (orc.BF16, None)}
    for ex in _load_examples()["policy"]:
        pol = orc.TolerancePolicy(ex["default"]["atol"], ex["default"]["rtol"])
        for name, pr in ex["by_dtype"].items():
            pol.set_dtype(dt[name][0], pr["atol"], pr["rtol"])
        for cls, pr in ex["by_class"].items():
            pol.set_class(int(cls), pr["atol"], pr["rtol"])
        r32, c32 = _arr(ex["ref"]), _arr(ex["cand"])
        as_bf16 = lambda a: (a.view(np.uint32) >> 16).astype(np.uint16)   # exact for these values
        assert np.array_equal((as_bf16(c32).astype(np.uint32) << 16).view(np.float32), c32)
        segs = []
        for g in ex["groups"]:
            code = dt[g["dtype"]][0]
            r, c = (r32, c32) if g["dtype"] == "f32" else (as_bf16(r32), as_bf16(c32))
            segs.append((r, [c], code, g["tol_class"]))
        rows = orc.check_segments(segs, pol)
        assert len(rows) == len(ex["groups"])
        for row, g in zip(rows, ex["groups"]):
            assert row["n_mismatch"] == g["n_mismatch"] and row["valid"] == g["valid"], (ex["name"], g, row)
            assert row["n_finite"] == len(ex["ref"]) and row["flags"] == 0
            assert _same_f32(row["max_abs_err"], ex["max_abs_err"]) and _same_f32(row["max_rel_err"], ex["max_rel_err"])
            assert row["sum_abs_err"] == ex["sum_abs_err"] and row["sum_rel_err"] == ex["sum_rel_err"]
        one = orc.check_cases(segs, pol)
        assert len(one) == 1
        for key, want in ex["as_cases"].items():
            assert one[0][key] == want, (ex["name"], key, one[0])
        assert one[0]["n_elems"] == len(ex["ref"]) * len(ex["groups"])
    # groups against single checks with the pair written out
    rng = np.random.default_rng(77)
    pol = orc.TolerancePolicy(1e-3, 1e-3)
    pol.set_dtype(orc.F64, 1e-9, 1e-9)
    pol.set_class(5, 0.5, 0.0)
    r32 = rng.standard_normal(300).astype(np.float32)
    c32 = (r32 * (1 + 2e-3 * rng.standard_normal(300))).astype(np.float32)
    r64 = rng.standard_normal(200)
    c64 = r64 * (1 + 2e-9 * rng.standard_normal(200))
    rows = orc.check_segments([(r32, [c32], orc.F32, 0), (r64, [c64], orc.F64, 0), (r32, [c32], orc.F32, 5)], pol)
    assert rows[0] == orc.check_one(r32, c32, orc.F32, 1e-3, 1e-3)
    assert rows[1] == orc.check_one(r64, c64, orc.F64, 1e-9, 1e-9)
    assert rows[2] == orc.check_one(r32, c32, orc.F32, 0.5, 0.0)
    assert 0 < rows[0]["n_mismatch"] < 300 and 0 < rows[1]["n_mismatch"] < 200 and rows[2]["n_mismatch"] == 0
    try:
        orc.check_segments([(r32, [c32], orc.F32, 6)], pol)
    except KeyError:
        pass
    else:
        raise AssertionError("a tolerance class that was never set must be refused")


ALL_PINS = [
    pin_truth_table, pin_flag_classes, pin_worked_check_examples, pin_worked_fitness_examples,
    pin_numpy_isclose, pin_sums_and_maxima, pin_invariants, pin_bf16_widening, pin_f16_widening,
    pin_median_and_speedup, pin_unusable_timing_rows, pin_select_elite,
    pin_f64_truth_table, pin_f64_numpy_isclose_sums_maxima, pin_f64_agrees_with_f32_where_both_are_exact,
    pin_integer_equality, pin_mean_reducer, pin_select_elite_diverse, pin_tolerance_policy,
]
