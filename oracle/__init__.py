"""CPU oracle for the fitness-and-validity evaluation step -- TEST INFRASTRUCTURE.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It loads ``evo_oracle.c`` (plain C, one
thread, one element at a time; see the header of that file for what it follows in
EvoEngineer, arXiv 2510.03760, Sec. 3.1 / 4.3 / 5.1) through ctypes and exposes it
on numpy arrays.  It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "evo_oracle.c")
_LIB = os.path.join(_HERE, "libevo_oracle.so")

F32 = 0
BF16 = 1
F16 = 2
F64 = 3
I32 = 4
I64 = 5

REDUCE_MEDIAN = 0
REDUCE_MEAN = 1

F_CAND_NAN = 1 << 0
F_CAND_INF = 1 << 1
F_REF_NAN = 1 << 2
F_REF_INF = 1 << 3
F_NAN_SITE_DIFF = 1 << 4
F_INF_DIFF = 1 << 5

CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fPIC", "-shared"]


def build(force: bool = False) -> str:
    """Compile evo_oracle.c with gcc when the library is absent or stale."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Acc(ctypes.Structure):
    _fields_ = [
        ("n_mismatch", ctypes.c_uint64),
        ("n_finite", ctypes.c_uint64),
        ("sum_abs_err", ctypes.c_double),
        ("sum_rel_err", ctypes.c_double),
        ("max_abs_err", ctypes.c_float),
        ("max_rel_err", ctypes.c_float),
        ("flags", ctypes.c_uint32),
        ("valid", ctypes.c_uint32),
        ("n_seen", ctypes.c_uint64),
    ]


class _Pop(ctypes.Structure):
    _fields_ = [
        ("best_idx", ctypes.c_uint32),
        ("n_valid", ctypes.c_uint32),
        ("best_speedup", ctypes.c_float),
        ("valid_rate", ctypes.c_float),
    ]


_libs = {}
_load_lock = threading.Lock()


def _load(path: str = None):
    """ctypes handle of the oracle library (default: built from evo_oracle.c here)."""
    key = path or _LIB
    if key in _libs:
        return _libs[key]
    with _load_lock:   # one thread compiles and binds; check_batch may get here from several
        return _load_locked(path, key)


def _load_locked(path, key):
    if key not in _libs:
        lib = ctypes.CDLL(path or build())
        lib.oracle_check_init.argtypes = [ctypes.POINTER(_Acc)]
        lib.oracle_check_init.restype = None
        lib.oracle_check_chunk.argtypes = [
            ctypes.POINTER(_Acc), ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_uint64, ctypes.c_int, ctypes.c_float, ctypes.c_float,
        ]
        lib.oracle_check_chunk.restype = None
        lib.oracle_fitness.argtypes = [ctypes.c_void_p] * 2 + [ctypes.c_uint32] * 2 + [ctypes.c_void_p] * 7
        lib.oracle_fitness.restype = ctypes.c_int
        lib.oracle_fitness_ex.argtypes = ([ctypes.c_void_p] * 2 + [ctypes.c_uint32] * 2 + [ctypes.c_void_p]
                                          + [ctypes.c_int] + [ctypes.c_void_p] * 6)
        lib.oracle_fitness_ex.restype = ctypes.c_int
        lib.oracle_select_elite.argtypes = [ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint32,
                                            ctypes.c_void_p]
        lib.oracle_select_elite.restype = ctypes.c_uint32
        lib.oracle_select_elite_diverse.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                                    ctypes.c_uint32, ctypes.c_void_p]
        lib.oracle_select_elite_diverse.restype = ctypes.c_uint32
        lib.oracle_half_to_float.argtypes = [ctypes.c_uint16]
        lib.oracle_half_to_float.restype = ctypes.c_float
        lib.oracle_acc_size.restype = ctypes.c_uint32
        assert lib.oracle_acc_size() == ctypes.sizeof(_Acc)
        _libs[key] = lib
    return _libs[key]


def _as_elems(x, dtype: int) -> np.ndarray:
    """Flat contiguous view: float32 / float64 / int32 / int64 for those types, uint16 bit
    patterns for BF16 and F16."""
    a = np.ascontiguousarray(x).reshape(-1)
    if dtype == F16 and a.dtype == np.float16:
        a = a.view(np.uint16)
    want = {F32: np.float32, F64: np.float64, I32: np.int32, I64: np.int64}.get(dtype, np.uint16)
    if a.dtype != want:
        raise TypeError("oracle expects %s elements, got %s" % (np.dtype(want), a.dtype))
    return a


class CheckAccumulator:
    """One candidate's running statistics; feed consecutive chunks in order."""

    def __init__(self, dtype: int, atol: float, rtol: float, lib_path: str = None):
        self._lib = _load(lib_path)
        self.dtype = dtype
        self.atol = float(np.float32(atol))
        self.rtol = float(np.float32(rtol))
        self._acc = _Acc()
        self._lib.oracle_check_init(ctypes.byref(self._acc))

    def feed(self, ref_chunk, cand_chunk, dtype: int = None, atol: float = None,
             rtol: float = None) -> None:
        """The next chunk; a chunk that is another test case of the same candidate may have
        its own element type and tolerance."""
        dt = self.dtype if dtype is None else dtype
        a = self.atol if atol is None else float(np.float32(atol))
        t = self.rtol if rtol is None else float(np.float32(rtol))
        r = _as_elems(ref_chunk, dt)
        c = _as_elems(cand_chunk, dt)
        if r.size != c.size:
            raise ValueError("chunk sizes differ")
        self._lib.oracle_check_chunk(
            ctypes.byref(self._acc), r.ctypes.data, c.ctypes.data, r.size, dt, a, t)

    def result(self) -> dict:
        a = self._acc
        return {
            "n_mismatch": int(a.n_mismatch),
            "n_finite": int(a.n_finite),
            "sum_abs_err": float(a.sum_abs_err),
            "sum_rel_err": float(a.sum_rel_err),
            "max_abs_err": np.float32(a.max_abs_err),
            "max_rel_err": np.float32(a.max_rel_err),
            "flags": int(a.flags),
            "valid": int(a.valid),
            "n_elems": int(a.n_seen),
        }


def check_one(ref, cand, dtype: int, atol: float, rtol: float, lib_path: str = None) -> dict:
    acc = CheckAccumulator(dtype, atol, rtol, lib_path)
    acc.feed(ref, cand)
    return acc.result()


def check_batch(ref, cands, dtype: int, atol: float, rtol: float, threads: int = 1,
                lib_path: str = None) -> list:
    """Statistics rows for a list of candidates against one reference.

    ``threads`` > 1 runs whole candidates side by side (each candidate is still
    reduced sequentially by one thread, so the rows do not depend on it).
    """
    if threads <= 1 or len(cands) <= 1:
        return [check_one(ref, c, dtype, atol, rtol, lib_path) for c in cands]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(lambda c: check_one(ref, c, dtype, atol, rtol, lib_path), cands))


class TolerancePolicy:
    """Which absolute/relative pair a group of tensors is checked with (functional testing
    of Sec. 4.3 over outputs of different kinds and precisions, cf. the kernel
    classification table of the appendix; the paper gives no values): one pair per element
    type, all equal to the pair given here until set_dtype changes one, and caller-defined
    classes 1..15; a group that names a class takes the class's pair, any other group the
    pair of its element type."""

    N_CLASSES = 15

    def __init__(self, atol: float, rtol: float):
        self.by_dtype = {d: (atol, rtol) for d in (F32, BF16, F16, F64, I32, I64)}
        self.by_class = {}

    def set_dtype(self, dtype: int, atol: float, rtol: float) -> None:
        if dtype not in self.by_dtype:
            raise ValueError("unknown element type")
        self.by_dtype[dtype] = (atol, rtol)

    def set_class(self, tol_class: int, atol: float, rtol: float) -> None:
        if not 1 <= tol_class <= self.N_CLASSES:
            raise ValueError("tolerance classes are 1..%d" % self.N_CLASSES)
        self.by_class[tol_class] = (atol, rtol)

    def lookup(self, dtype: int, tol_class: int = 0):
        if tol_class == 0:
            return self.by_dtype[dtype]
        return self.by_class[tol_class]   # KeyError: the class was never set


def check_segments(segments, policy: TolerancePolicy, threads: int = 1, lib_path: str = None) -> list:
    """Rows of a ragged launch: ``segments`` is a list of (ref, cands, dtype, tol_class);
    every group is checked on its own with the pair the policy gives it.  Returns the rows
    of all groups, in group order."""
    rows = []
    for ref, cands, dtype, tol_class in segments:
        atol, rtol = policy.lookup(dtype, tol_class)
        rows += check_batch(ref, cands, dtype, atol, rtol, threads, lib_path)
    return rows


def check_cases(cases, policy: TolerancePolicy, lib_path: str = None) -> list:
    """One row per candidate over K test cases: ``cases`` is a list of (ref, cands, dtype,
    tol_class) with the same number of candidates each; candidate p's accumulator is fed
    case after case, each case with its own element type and the pair the policy gives it."""
    P = len(cases[0][1])
    accs = None
    for ref, cands, dtype, tol_class in cases:
        if len(cands) != P:
            raise ValueError("every case has the same candidates")
        atol, rtol = policy.lookup(dtype, tol_class)
        if accs is None:
            accs = [CheckAccumulator(dtype, atol, rtol, lib_path) for _ in range(P)]
        for acc, cand in zip(accs, cands):
            acc.feed(ref, cand, dtype, atol, rtol)
    return [a.result() for a in accs]


def fitness(timings, baseline, valid, lib_path: str = None, reducer: int = REDUCE_MEDIAN) -> dict:
    """Median/mean time, speedup, fitness per candidate and the population summary.
    ``reducer`` picks what the speedup is the ratio of: medians (default) or means."""
    lib = _load(lib_path)
    t = np.ascontiguousarray(timings, dtype=np.float32)
    if t.ndim != 2:
        raise ValueError("timings must be [P, T]")
    P, T = t.shape
    b = np.ascontiguousarray(baseline, dtype=np.float32).reshape(-1)
    if b.size != T:
        raise ValueError("baseline must hold T samples")
    v = np.ascontiguousarray(valid, dtype=np.uint32).reshape(-1)
    if v.size != P:
        raise ValueError("valid must hold P flags")
    med = np.empty(P, np.float32)
    mean = np.empty(P, np.float32)
    spd = np.empty(P, np.float32)
    fit = np.empty(P, np.float32)
    base = ctypes.c_float()
    pop = _Pop()
    rc = lib.oracle_fitness_ex(
        t.ctypes.data, b.ctypes.data, P, T, v.ctypes.data, int(reducer), med.ctypes.data,
        mean.ctypes.data, spd.ctypes.data, fit.ctypes.data,
        ctypes.addressof(base), ctypes.addressof(pop))
    if rc != 0:
        raise MemoryError("oracle_fitness")
    return {
        "median_ms": med, "mean_ms": mean, "speedup": spd, "fitness": fit,
        "base_median_ms": np.float32(base.value),
        "best_idx": int(pop.best_idx), "n_valid": int(pop.n_valid),
        "best_speedup": np.float32(pop.best_speedup),
        "valid_rate": np.float32(pop.valid_rate),
    }


def half_to_float(bits: int, lib_path: str = None) -> np.float32:
    return np.float32(_load(lib_path).oracle_half_to_float(int(bits)))


def select_elite(fitness_values, k: int, lib_path: str = None) -> dict:
    """Indices of the k best feasible candidates (fitness > 0), best first."""
    lib = _load(lib_path)
    f = np.ascontiguousarray(fitness_values, dtype=np.float32).reshape(-1)
    out = np.empty(max(1, k), np.uint32)
    n = lib.oracle_select_elite(f.ctypes.data, f.size, k, out.ctypes.data)
    return {"elite": out[:k].copy(), "n_elite": int(n)}


def select_elite_diverse(fitness_values, keys, k: int, lib_path: str = None) -> dict:
    """Indices of the k best feasible candidates with pairwise different keys, best first."""
    lib = _load(lib_path)
    f = np.ascontiguousarray(fitness_values, dtype=np.float32).reshape(-1)
    ky = np.ascontiguousarray(keys, dtype=np.uint32).reshape(-1)
    if ky.size != f.size:
        raise ValueError("one key per candidate")
    out = np.empty(max(1, k), np.uint32)
    n = lib.oracle_select_elite_diverse(f.ctypes.data, ky.ctypes.data, f.size, k, out.ctypes.data)
    return {"elite": out[:k].copy(), "n_elite": int(n)}


class Variant:
    """The same interface bound to another build of the C file (used by the tests
    that check the pins catch planted mistakes)."""

    F32, BF16, F16, F64, I32, I64 = F32, BF16, F16, F64, I32, I64
    REDUCE_MEDIAN, REDUCE_MEAN = REDUCE_MEDIAN, REDUCE_MEAN
    F_CAND_NAN, F_CAND_INF, F_REF_NAN, F_REF_INF = F_CAND_NAN, F_CAND_INF, F_REF_NAN, F_REF_INF
    F_NAN_SITE_DIFF, F_INF_DIFF = F_NAN_SITE_DIFF, F_INF_DIFF

    def __init__(self, lib_path: str):
        self.lib_path = lib_path

    def CheckAccumulator(self, dtype, atol, rtol):
        return CheckAccumulator(dtype, atol, rtol, self.lib_path)

    def check_one(self, ref, cand, dtype, atol, rtol):
        return check_one(ref, cand, dtype, atol, rtol, self.lib_path)

    def check_batch(self, ref, cands, dtype, atol, rtol, threads=1):
        return check_batch(ref, cands, dtype, atol, rtol, threads, self.lib_path)

    TolerancePolicy = TolerancePolicy

    def check_segments(self, segments, policy, threads=1):
        return check_segments(segments, policy, threads, self.lib_path)

    def check_cases(self, cases, policy):
        return check_cases(cases, policy, self.lib_path)

    def fitness(self, timings, baseline, valid, reducer=REDUCE_MEDIAN):
        return fitness(timings, baseline, valid, self.lib_path, reducer)

    def select_elite(self, fitness_values, k):
        return select_elite(fitness_values, k, self.lib_path)

    def select_elite_diverse(self, fitness_values, keys, k):
        return select_elite_diverse(fitness_values, keys, k, self.lib_path)

    def half_to_float(self, bits):
        return half_to_float(bits, self.lib_path)
