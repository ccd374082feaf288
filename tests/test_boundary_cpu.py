"""The C-ABI library without a GPU: it loads, exports every symbol the header declares,
its records have the documented layout, and every argument error is reported from pure
host code (no kernel is launched by anything here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "evo.h")


@pytest.fixture(scope="module")
def evo():
    from paper_2510_03760_amd import build as hip_build
    if hip_build.is_stale():
        hip_build.build()
    import paper_2510_03760_amd as evo
    return evo


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"EVO_API\s+[\w\s\*]+?\b(evo_\w+)\s*\(", text)))


def test_header_declares_the_documented_entry_points():
    assert declared_functions() == ["evo_check_batch", "evo_check_batch_static", "evo_check_cases", "evo_check_create",
                                    "evo_check_destroy", "evo_check_segmented", "evo_check_set_tolerance",
                                    "evo_check_set_tolerance_class", "evo_evaluate",
                                    "evo_evaluate_segmented",
                                    "evo_fitness",
                                    "evo_fitness_ex", "evo_select_elite", "evo_select_elite_diverse",
                                    "evo_strerror",
                                    "evo_time_candidates"]


def test_library_exports_every_declared_symbol(evo):
    lib = ctypes.CDLL(evo.lib_path)
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_record_layouts_match_the_header(evo):
    text = open(HEADER).read()
    assert "72 bytes" in text
    assert ctypes.sizeof(evo.EvoStats) == 72
    assert evo.EvoStats.valid.offset == 44 and evo.EvoStats.median_ms.offset == 48
    assert evo.EvoStats.n_elems_lo.offset == 64
    assert ctypes.sizeof(evo.EvoSegment) == 40
    assert ctypes.sizeof(evo.EvoPopSummary) == 16
    for name, val in (("EVO_F_CAND_NAN", 0), ("EVO_F_CAND_INF", 1), ("EVO_F_REF_NAN", 2),
                      ("EVO_F_REF_INF", 3), ("EVO_F_NAN_SITE_DIFF", 4), ("EVO_F_INF_DIFF", 5)):
        assert re.search(r"%s\s*=\s*1u << %d" % (name, val), text), name


def _create(evo, *args):
    out = ctypes.c_void_p()
    rc = evo.lib.evo_check_create(ctypes.byref(out), *args)
    return rc, out.value


def test_create_validates(evo):
    assert evo.lib.evo_check_create(None, 0, 10, 0.0, 0.0) == -1
    assert _create(evo, 7, 10, 0.0, 0.0) == (-2, None)
    for code in range(6):                    # f32, bf16, f16, f64, i32, i64
        rc, hx = _create(evo, code, 10, 0.0, 0.0)
        assert rc == 0 and evo.lib.evo_check_destroy(hx) == 0
    assert _create(evo, 6, 10, 0.0, 0.0) == (-2, None)
    assert _create(evo, 0, 0, 0.0, 0.0) == (-3, None)
    for atol, rtol in ((-1e-3, 0.0), (0.0, -1.0), (float("nan"), 0.0), (0.0, float("nan")),
                       (float("inf"), 0.0), (0.0, float("inf"))):
        assert _create(evo, 0, 10, atol, rtol) == (-4, None), (atol, rtol)
    rc, h = _create(evo, 1, 1 << 40, 0.0, 0.0)
    assert rc == 0 and h
    assert evo.lib.evo_check_destroy(h) == 0


def test_handle_lifetime(evo):
    rc, h = _create(evo, 0, 10, 1e-2, 1e-2)
    assert rc == 0
    assert evo.lib.evo_check_destroy(h) == 0
    assert evo.lib.evo_check_destroy(h) == -8          # double destroy
    assert evo.lib.evo_check_destroy(None) == -8
    arr = (ctypes.c_void_p * 1)(16)
    assert evo.lib.evo_check_batch(h, 16, arr, 1, None, 16) == -8        # use after destroy
    assert evo.lib.evo_fitness(h, 16, 16, 1, 1, None, 16, None) == -8
    assert evo.lib.evo_check_batch(0x1234, 16, arr, 1, None, 16) == -8   # never created


def test_check_batch_validates_before_any_launch(evo):
    rc, h = _create(evo, 0, 1000, 1e-2, 1e-2)
    assert rc == 0
    ok = (ctypes.c_void_p * 3)(64, 128, 256)
    call = evo.lib.evo_check_batch
    assert call(h, None, ok, 3, None, 512) == -1
    assert call(h, 64, None, 3, None, 512) == -1
    assert call(h, 64, ok, 3, None, None) == -1
    assert call(h, 64, (ctypes.c_void_p * 3)(64, None, 256), 3, None, 512) == -1
    assert call(h, 64, ok, 0, None, 512) == -3
    assert call(h, 64, ok, 70000, None, 512) == -3
    assert call(h, 66, ok, 3, None, 512) == -5                      # fp32 needs 4-byte alignment
    assert call(h, 64, (ctypes.c_void_p * 3)(64, 130, 256), 3, None, 512) == -5
    assert evo.lib.evo_check_destroy(h) == 0
    rc, h = _create(evo, 1, 1000, 1e-2, 1e-2)                       # bf16: 2-byte alignment
    assert call(h, 65, ok, 3, None, 512) == -5
    assert evo.lib.evo_check_destroy(h) == 0


def test_check_segmented_validates_before_any_launch(evo):
    rc, h = _create(evo, 0, 1, 1e-2, 1e-2)
    ptrs = (ctypes.c_void_p * 2)(64, 128)
    pp = ctypes.cast(ptrs, ctypes.POINTER(ctypes.c_void_p))

    def seg(ref=64, cand=pp, n=100, P=2, dtype=0, row0=0):
        s = evo.EvoSegment()
        s.ref, s.cand_ptrs, s.n_elems, s.P_s, s.dtype, s.stats_row0 = ref, cand, n, P, dtype, row0
        return s

    def call(segs, n_rows=8, stats=512):
        arr = (evo.EvoSegment * len(segs))(*segs)
        return evo.lib.evo_check_segmented(h, arr, len(segs), None, stats, n_rows)

    assert evo.lib.evo_check_segmented(h, None, 1, None, 512, 8) == -1
    assert call([seg()], stats=None) == -1
    assert evo.lib.evo_check_segmented(h, (evo.EvoSegment * 1)(seg()), 0, None, 512, 8) == -3
    assert call([seg(ref=None)]) == -1
    assert call([seg(cand=None)]) == -1
    assert call([seg(n=0)]) == -3
    assert call([seg(P=0)]) == -3
    assert call([seg(dtype=6)]) == -2
    assert call([seg(ref=66)]) == -5
    assert call([seg(row0=7)]) == -3                                   # rows 7,8 exceed n_rows
    assert call([seg(row0=0), seg(row0=1)]) == -3                      # overlapping rows
    assert call([seg(row0=2), seg(row0=0), seg(row0=3)]) == -3         # overlap, unsorted
    assert evo.lib.evo_check_destroy(h) == 0


def test_check_cases_validates_before_any_launch(evo):
    rc, h = _create(evo, 0, 1, 1e-2, 1e-2)
    ptrs = (ctypes.c_void_p * 2)(64, 128)
    pp = ctypes.cast(ptrs, ctypes.POINTER(ctypes.c_void_p))

    def case(P=2, row0=0, ref=64, n=10, dtype=0):
        s = evo.EvoSegment()
        s.ref, s.cand_ptrs, s.n_elems, s.P_s, s.dtype, s.stats_row0 = ref, pp, n, P, dtype, row0
        return s

    def call(cases, stats=512):
        arr = (evo.EvoSegment * len(cases))(*cases)
        return evo.lib.evo_check_cases(h, arr, len(cases), None, stats)

    assert evo.lib.evo_check_cases(h, None, 1, None, 512) == -1
    assert call([case()], stats=None) == -1
    assert evo.lib.evo_check_cases(h, (evo.EvoSegment * 1)(case()), 0, None, 512) == -3
    assert call([case(), case(P=1)]) == -3           # unequal populations
    assert call([case(), case(row0=2)]) == -3        # rows must start at 0
    assert call([case(), case(n=0)]) == -3
    assert call([case(), case(dtype=9)]) == -2
    assert call([case(), case(ref=None)]) == -1
    assert evo.lib.evo_check_destroy(h) == 0


def test_fitness_validates_before_any_launch(evo):
    rc, h = _create(evo, 0, 1, 0.0, 0.0)
    call = evo.lib.evo_fitness
    assert call(h, None, 64, 4, 10, None, 512, None) == -1
    assert call(h, 64, None, 4, 10, None, 512, None) == -1
    assert call(h, 64, 64, 4, 10, None, None, None) == -1
    assert call(h, 64, 64, 0, 10, None, 512, None) == -3
    assert call(h, 64, 64, 4, 0, None, 512, None) == -3
    assert call(h, 64, 64, 4, 4097, None, 512, None) == -3
    assert call(h, 66, 64, 4, 10, None, 512, None) == -5
    assert call(h, 64, 64, 4, 10, None, 516, None) == -5
    ex = evo.lib.evo_fitness_ex
    assert ex(h, 64, 64, 4, 10, 2, None, 512, None) == -3      # unknown reducer
    assert ex(h, 64, 64, 4, 10, -1, None, 512, None) == -3
    assert ex(h, None, 64, 4, 10, 1, None, 512, None) == -1
    assert ex(h, 64, 64, 4, 4097, 1, None, 512, None) == -3
    assert ex(None, 64, 64, 4, 10, 1, None, 512, None) == -8
    assert evo.lib.evo_check_destroy(h) == 0


def test_select_elite_validates_before_any_launch(evo):
    rc, h = _create(evo, 0, 1, 0.0, 0.0)
    call = evo.lib.evo_select_elite
    assert call(h, None, 4, 2, None, 64, None) == -1
    assert call(h, 64, 4, 2, None, None, None) == -1
    assert call(h, 64, 0, 1, None, 64, None) == -3
    assert call(h, 64, 4, 0, None, 64, None) == -3
    assert call(h, 64, 4, 5, None, 64, None) == -3
    assert call(h, 64, 70000, 5, None, 64, None) == -3
    assert call(h, 68, 4, 2, None, 64, None) == -5
    assert call(h, 64, 4, 2, None, 66, None) == -5
    assert evo.lib.evo_check_destroy(h) == 0


def test_strerror(evo):
    seen = set()
    for code in range(0, -9, -1):
        msg = evo.evo_strerror(code)
        assert msg and msg != "unknown status"
        seen.add(msg)
    assert len(seen) == 9
    assert evo.evo_strerror(-99) == "unknown status"


def test_group_decomposition_matches_its_inverse():
    """Host logic mirrored from the kernel's candidate grouping: sizes are powers of two,
    cover 0..P-1 once, in order (checked here against a direct Python statement)."""
    kG = 16
    for P in list(range(1, 70)) + [255, 256, 257, 1000]:
        sizes = [kG] * (P // kG) + [b for b in (8, 4, 2, 1) if (P % kG) & b]
        assert sum(sizes) == P and all(s & (s - 1) == 0 for s in sizes)


def test_no_product_code_touches_the_oracle():
    """The package and the benchmark's GPU path never import the CPU oracle."""
    pkg = os.path.join(ROOT, "paper_2510_03760_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
