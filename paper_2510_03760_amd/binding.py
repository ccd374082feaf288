"""ctypes binding of include/evo.h: argument marshalling only.

Every function here has the name and the argument order of its C counterpart and
does nothing but convert Python objects to pointers and sizes.  Device memory and
streams come from PyTorch (``tensor.data_ptr()``, ``torch.cuda.current_stream()``);
all computing is done by the kernels behind the C ABI.  There is no fallback: if the
shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import numpy as np
import torch  # loads the HIP runtime that the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
lib_path = os.path.join(_HERE, "libevo.so")

EVO_F32 = 0
EVO_BF16 = 1
EVO_F16 = 2
EVO_F64 = 3
EVO_I32 = 4
EVO_I64 = 5

EVO_REDUCE_MEDIAN = 0
EVO_REDUCE_MEAN = 1


class EvoError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, evo_strerror(code), code))


class EvoStats(ctypes.Structure):
    _fields_ = [
        ("n_mismatch", ctypes.c_uint64), ("n_finite", ctypes.c_uint64),
        ("sum_abs_err", ctypes.c_double), ("sum_rel_err", ctypes.c_double),
        ("max_abs_err", ctypes.c_float), ("max_rel_err", ctypes.c_float),
        ("flags", ctypes.c_uint32), ("valid", ctypes.c_uint32),
        ("median_ms", ctypes.c_float), ("mean_ms", ctypes.c_float),
        ("speedup", ctypes.c_float), ("fitness", ctypes.c_float),
        ("n_elems_lo", ctypes.c_uint32), ("n_elems_hi", ctypes.c_uint32),
    ]


class EvoSegment(ctypes.Structure):
    _fields_ = [
        ("ref", ctypes.c_void_p), ("cand_ptrs", ctypes.POINTER(ctypes.c_void_p)),
        ("n_elems", ctypes.c_uint64), ("P_s", ctypes.c_uint32), ("dtype", ctypes.c_uint32),
        ("stats_row0", ctypes.c_uint32), ("tol_class", ctypes.c_uint32),
    ]


class EvoPopSummary(ctypes.Structure):
    _fields_ = [
        ("best_idx", ctypes.c_uint32), ("n_valid", ctypes.c_uint32),
        ("best_speedup", ctypes.c_float), ("valid_rate", ctypes.c_float),
    ]


# numpy views of the two records, for reading results copied back to the host
LAUNCH_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)   # evo_launch_fn


class EvoTimingOpts(ctypes.Structure):
    _fields_ = [("warmup", ctypes.c_uint32), ("flush_cache", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32 * 2)]


STATS_DTYPE = np.dtype([
    ("n_mismatch", "<u8"), ("n_finite", "<u8"), ("sum_abs_err", "<f8"), ("sum_rel_err", "<f8"),
    ("max_abs_err", "<f4"), ("max_rel_err", "<f4"), ("flags", "<u4"), ("valid", "<u4"),
    ("median_ms", "<f4"), ("mean_ms", "<f4"), ("speedup", "<f4"), ("fitness", "<f4"),
    ("n_elems_lo", "<u4"), ("n_elems_hi", "<u4"),
])
SUMMARY_DTYPE = np.dtype([("best_idx", "<u4"), ("n_valid", "<u4"), ("best_speedup", "<f4"),
                          ("valid_rate", "<f4")])
assert STATS_DTYPE.itemsize == ctypes.sizeof(EvoStats) == 72
assert SUMMARY_DTYPE.itemsize == ctypes.sizeof(EvoPopSummary) == 16


def load_library(path: str = None) -> ctypes.CDLL:
    """The C ABI of the library at `path` (default: the package's libevo.so) with its argument
    types declared.  The package itself binds the default; tests use this for other builds of
    the same sources."""
    path = path or lib_path
    if not os.path.exists(path):
        raise ImportError(
            "%s is missing: build it with `python paper_2510_03760_amd/build.py` "
            "(there is no fallback implementation)" % path)
    h = ctypes.CDLL(path)
    vp, u32, u64, f32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float
    h.evo_check_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, u64, f32, f32]
    h.evo_check_set_tolerance.argtypes = [vp, ctypes.c_int, f32, f32]
    h.evo_check_set_tolerance_class.argtypes = [vp, u32, f32, f32]
    h.evo_check_batch.argtypes = [vp, vp, ctypes.POINTER(vp), u32, vp, vp]
    h.evo_check_batch_static.argtypes = [vp, vp, ctypes.POINTER(vp), u32, vp, vp]
    h.evo_check_segmented.argtypes = [vp, ctypes.POINTER(EvoSegment), u32, vp, vp, u32]
    h.evo_check_cases.argtypes = [vp, ctypes.POINTER(EvoSegment), u32, vp, vp]
    h.evo_fitness.argtypes = [vp, vp, vp, u32, u32, vp, vp, vp]
    h.evo_fitness_ex.argtypes = [vp, vp, vp, u32, u32, ctypes.c_int, vp, vp, vp]
    h.evo_select_elite.argtypes = [vp, vp, u32, u32, vp, vp, vp]
    h.evo_select_elite_diverse.argtypes = [vp, vp, vp, u32, u32, vp, vp, vp]
    h.evo_evaluate.argtypes = [vp, ctypes.POINTER(EvoSegment), u32, vp, vp, u32, ctypes.c_int, vp, vp, vp]
    h.evo_evaluate_segmented.argtypes = [vp, ctypes.POINTER(EvoSegment), u32, vp, vp, u32, ctypes.c_int, vp,
                                         vp, u32, vp]
    h.evo_time_candidates.argtypes = [vp, ctypes.POINTER(LAUNCH_FN), ctypes.POINTER(vp), u32, u32,
                                      ctypes.POINTER(EvoTimingOpts), vp, vp, ctypes.POINTER(f32)]
    h.evo_check_destroy.argtypes = [vp]
    h.evo_strerror.argtypes = [ctypes.c_int]
    h.evo_strerror.restype = ctypes.c_char_p
    for name in ("evo_check_create", "evo_check_set_tolerance", "evo_check_set_tolerance_class", "evo_check_batch", "evo_check_batch_static", "evo_check_segmented", "evo_check_cases",
                 "evo_fitness", "evo_fitness_ex", "evo_select_elite", "evo_time_candidates", "evo_evaluate", "evo_evaluate_segmented", "evo_select_elite_diverse",
                 "evo_check_destroy"):
        getattr(h, name).restype = ctypes.c_int
    return h


lib = load_library()


def evo_strerror(code: int) -> str:
    return lib.evo_strerror(int(code)).decode()


def _ptr(x) -> Optional[int]:
    """Device or host address of a tensor / raw integer address / None."""
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        return x.data_ptr()
    return int(x)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def evo_check_create(dtype: int, n_elems: int, atol: float, rtol: float) -> int:
    """Returns the context handle (an integer address); raises EvoError on failure."""
    out = ctypes.c_void_p()
    rc = lib.evo_check_create(ctypes.byref(out), int(dtype), int(n_elems), float(atol), float(rtol))
    if rc != 0:
        raise EvoError(rc, "evo_check_create")
    return out.value


def evo_check_set_tolerance(ctx: int, dtype: int, atol: float, rtol: float) -> None:
    rc = lib.evo_check_set_tolerance(ctx, int(dtype), float(atol), float(rtol))
    if rc != 0:
        raise EvoError(rc, "evo_check_set_tolerance")


def evo_check_set_tolerance_class(ctx: int, tol_class: int, atol: float, rtol: float) -> None:
    rc = lib.evo_check_set_tolerance_class(ctx, int(tol_class), float(atol), float(rtol))
    if rc != 0:
        raise EvoError(rc, "evo_check_set_tolerance_class")


def evo_check_batch(ctx: int, ref, cand_ptrs: Sequence, P: int, stream, stats) -> None:
    arr = (ctypes.c_void_p * max(1, len(cand_ptrs)))(*[_ptr(c) for c in cand_ptrs])
    rc = lib.evo_check_batch(ctx, _ptr(ref), arr if cand_ptrs is not None else None, int(P),
                             _stream(stream), _ptr(stats))
    if rc != 0:
        raise EvoError(rc, "evo_check_batch")


def evo_check_batch_static(ctx: int, ref, cand_ptrs: Sequence, P: int, stream, stats) -> None:
    arr = (ctypes.c_void_p * max(1, len(cand_ptrs)))(*[_ptr(c) for c in cand_ptrs])
    rc = lib.evo_check_batch_static(ctx, _ptr(ref), arr, int(P), _stream(stream), _ptr(stats))
    if rc != 0:
        raise EvoError(rc, "evo_check_batch_static")


def _segment_array(segs: Sequence[dict]):
    """ctypes evo_segment array for dicts with keys ref, cand_ptrs, n_elems, dtype and
    (optionally) stats_row0, P_s, tol_class; also returns the objects that must stay alive."""
    keep: List[object] = []
    c_segs = (EvoSegment * max(1, len(segs)))()
    for i, sg in enumerate(segs):
        ptrs = sg["cand_ptrs"]
        arr = (ctypes.c_void_p * max(1, len(ptrs)))(*[_ptr(c) for c in ptrs])
        keep.append(arr)
        c_segs[i].ref = _ptr(sg["ref"])
        c_segs[i].cand_ptrs = ctypes.cast(arr, ctypes.POINTER(ctypes.c_void_p))
        c_segs[i].n_elems = int(sg["n_elems"])
        c_segs[i].P_s = int(sg.get("P_s", len(ptrs)))
        c_segs[i].dtype = int(sg["dtype"])
        c_segs[i].stats_row0 = int(sg.get("stats_row0", 0))
        c_segs[i].tol_class = int(sg.get("tol_class", 0))
    return c_segs, keep


def evo_check_segmented(ctx: int, segs: Sequence[dict], S: int, stream, stats, n_rows: int) -> None:
    """``segs``: dicts with keys ref, cand_ptrs, n_elems, dtype, stats_row0."""
    c_segs, keep = _segment_array(segs)
    rc = lib.evo_check_segmented(ctx, c_segs, int(S), _stream(stream), _ptr(stats), int(n_rows))
    del keep
    if rc != 0:
        raise EvoError(rc, "evo_check_segmented")


def evo_check_cases(ctx: int, cases: Sequence[dict], K: int, stream, stats) -> None:
    """``cases``: dicts with keys ref, cand_ptrs, n_elems, dtype (same candidates, one
    dict per test case)."""
    c_segs, keep = _segment_array(cases)
    rc = lib.evo_check_cases(ctx, c_segs, int(K), _stream(stream), _ptr(stats))
    del keep
    if rc != 0:
        raise EvoError(rc, "evo_check_cases")


def evo_fitness(ctx: int, timings, baseline, P: int, T: int, stream, stats, summary=None) -> None:
    rc = lib.evo_fitness(ctx, _ptr(timings), _ptr(baseline), int(P), int(T), _stream(stream),
                         _ptr(stats), _ptr(summary))
    if rc != 0:
        raise EvoError(rc, "evo_fitness")


def evo_fitness_ex(ctx: int, timings, baseline, P: int, T: int, reducer: int, stream, stats,
                   summary=None) -> None:
    rc = lib.evo_fitness_ex(ctx, _ptr(timings), _ptr(baseline), int(P), int(T), int(reducer),
                            _stream(stream), _ptr(stats), _ptr(summary))
    if rc != 0:
        raise EvoError(rc, "evo_fitness_ex")


def evo_select_elite_diverse(ctx: int, stats, keys, P: int, k: int, stream, elite, n_elite=None) -> None:
    rc = lib.evo_select_elite_diverse(ctx, _ptr(stats), _ptr(keys), int(P), int(k), _stream(stream),
                                      _ptr(elite), _ptr(n_elite))
    if rc != 0:
        raise EvoError(rc, "evo_select_elite_diverse")


def evo_evaluate(ctx: int, cases: Sequence[dict], K: int, timings, baseline, T: int, reducer: int,
                 stream, stats, summary=None) -> None:
    """``cases`` as for evo_check_cases."""
    c_segs, keep = _segment_array(cases)
    rc = lib.evo_evaluate(ctx, c_segs, int(K), _ptr(timings), _ptr(baseline), int(T), int(reducer),
                          _stream(stream), _ptr(stats), _ptr(summary))
    del keep
    if rc != 0:
        raise EvoError(rc, "evo_evaluate")


def evo_evaluate_segmented(ctx: int, segs: Sequence[dict], S: int, timings, baseline, T: int, reducer: int,
                           stream, stats, n_rows: int, summary=None) -> None:
    """``segs`` as for evo_check_segmented."""
    c_segs, keep = _segment_array(segs)
    rc = lib.evo_evaluate_segmented(ctx, c_segs, int(S), _ptr(timings), _ptr(baseline), int(T), int(reducer),
                                    _stream(stream), _ptr(stats), int(n_rows), _ptr(summary))
    del keep
    if rc != 0:
        raise EvoError(rc, "evo_evaluate_segmented")


def evo_time_candidates(ctx: int, launches, T: int, stream, timings, warmup: int = 3,
                        flush_cache: bool = False, want_clock_ratio: bool = True):
    """``launches``: one Python callable per candidate, called as f(stream_pointer); each must
    enqueue one run of its candidate on that stream.  Returns the clock ratios (or None)."""
    P = len(launches)
    keep = [LAUNCH_FN(lambda user, st, f=f: f(st)) for f in launches]   # keep the thunks alive
    fns = (LAUNCH_FN * P)(*keep)
    opts = EvoTimingOpts(int(warmup), 1 if flush_cache else 0)
    ratios = (ctypes.c_float * P)() if want_clock_ratio else None
    rc = lib.evo_time_candidates(ctx, fns, None, P, int(T), ctypes.byref(opts), _stream(stream),
                                 _ptr(timings), ratios)
    del keep
    if rc != 0:
        raise EvoError(rc, "evo_time_candidates")
    return list(ratios) if ratios is not None else None


def evo_select_elite(ctx: int, stats, P: int, k: int, stream, elite, n_elite=None) -> None:
    rc = lib.evo_select_elite(ctx, _ptr(stats), int(P), int(k), _stream(stream), _ptr(elite),
                              _ptr(n_elite))
    if rc != 0:
        raise EvoError(rc, "evo_select_elite")


def evo_check_destroy(ctx: int) -> int:
    return lib.evo_check_destroy(ctx)


class Checker:
    """Owns one context and the device buffers for its results (convenience only;
    each method is one C call)."""

    def __init__(self, dtype: int, n_elems: int, atol: float, rtol: float):
        self.ctx = evo_check_create(dtype, n_elems, atol, rtol)
        self.dtype, self.n_elems = dtype, n_elems

    def close(self) -> None:
        if self.ctx:
            ctx, self.ctx = self.ctx, None
            rc = evo_check_destroy(ctx)
            if rc != 0:
                raise EvoError(rc, "evo_check_destroy")

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_tolerance(self, dtype: int, atol: float, rtol: float) -> None:
        evo_check_set_tolerance(self.ctx, dtype, atol, rtol)

    def set_tolerance_class(self, tol_class: int, atol: float, rtol: float) -> None:
        evo_check_set_tolerance_class(self.ctx, tol_class, atol, rtol)

    @staticmethod
    def new_stats(rows: int, device="cuda") -> torch.Tensor:
        return torch.zeros(rows * 72, dtype=torch.uint8, device=device)

    @staticmethod
    def new_summary(device="cuda") -> torch.Tensor:
        return torch.zeros(16, dtype=torch.uint8, device=device)

    def check_batch(self, ref: torch.Tensor, cands: Sequence[torch.Tensor], stats: torch.Tensor,
                    stream=None) -> None:
        evo_check_batch(self.ctx, ref, list(cands), len(cands),
                        stream if stream is not None else torch.cuda.current_stream(), stats)

    def check_batch_static(self, ref: torch.Tensor, cands: Sequence[torch.Tensor], stats: torch.Tensor,
                           stream=None) -> None:
        evo_check_batch_static(self.ctx, ref, list(cands), len(cands),
                               stream if stream is not None else torch.cuda.current_stream(), stats)

    def check_segmented(self, segs: Sequence[dict], stats: torch.Tensor, n_rows: int,
                        stream=None) -> None:
        evo_check_segmented(self.ctx, segs, len(segs),
                            stream if stream is not None else torch.cuda.current_stream(),
                            stats, n_rows)

    def check_cases(self, cases: Sequence[dict], stats: torch.Tensor, stream=None) -> None:
        evo_check_cases(self.ctx, cases, len(cases),
                        stream if stream is not None else torch.cuda.current_stream(), stats)

    def fitness(self, timings: torch.Tensor, baseline: torch.Tensor, stats: torch.Tensor,
                summary: Optional[torch.Tensor] = None, stream=None,
                reducer: Optional[int] = None) -> None:
        P, T = timings.shape
        st = stream if stream is not None else torch.cuda.current_stream()
        if reducer is None:
            evo_fitness(self.ctx, timings, baseline, P, T, st, stats, summary)
        else:
            evo_fitness_ex(self.ctx, timings, baseline, P, T, reducer, st, stats, summary)


    def select_elite_diverse(self, stats: torch.Tensor, keys: torch.Tensor, P: int, k: int,
                             elite: torch.Tensor, n_elite: Optional[torch.Tensor] = None,
                             stream=None) -> None:
        evo_select_elite_diverse(self.ctx, stats, keys, P, k,
                                 stream if stream is not None else torch.cuda.current_stream(), elite,
                                 n_elite)

    def evaluate(self, cases: Sequence[dict], timings: torch.Tensor, baseline: torch.Tensor,
                 stats: torch.Tensor, summary: Optional[torch.Tensor] = None, stream=None,
                 reducer: int = EVO_REDUCE_MEDIAN) -> None:
        evo_evaluate(self.ctx, cases, len(cases), timings, baseline, timings.shape[1], reducer,
                     stream if stream is not None else torch.cuda.current_stream(), stats, summary)

    def evaluate_segmented(self, segs: Sequence[dict], timings: torch.Tensor, baseline: torch.Tensor,
                           stats: torch.Tensor, n_rows: int, summary: Optional[torch.Tensor] = None,
                           stream=None, reducer: int = EVO_REDUCE_MEDIAN) -> None:
        evo_evaluate_segmented(self.ctx, segs, len(segs), timings, baseline, timings.shape[1], reducer,
                               stream if stream is not None else torch.cuda.current_stream(), stats,
                               n_rows, summary)

    def time_candidates(self, launches, T: int, timings: torch.Tensor, warmup: int = 3,
                        flush_cache: bool = False, stream=None):
        return evo_time_candidates(self.ctx, launches, T,
                                   stream if stream is not None else torch.cuda.current_stream(),
                                   timings, warmup, flush_cache)

    def select_elite(self, stats: torch.Tensor, P: int, k: int, elite: torch.Tensor,
                     n_elite: Optional[torch.Tensor] = None, stream=None) -> None:
        evo_select_elite(self.ctx, stats, P, k,
                         stream if stream is not None else torch.cuda.current_stream(), elite,
                         n_elite)


def stats_to_numpy(stats: torch.Tensor) -> np.ndarray:
    """Copies a device stats buffer to the host as a structured array."""
    return stats.detach().cpu().numpy().view(STATS_DTYPE)


def summary_to_numpy(summary: torch.Tensor) -> np.ndarray:
    return summary.detach().cpu().numpy().view(SUMMARY_DTYPE)
