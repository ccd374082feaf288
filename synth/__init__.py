"""Seeded synthetic populations for the fitness-and-validity evaluation step.

Generators only: this module draws tensors and timing samples and records how
they were built (which candidates were corrupted, how many special sites were
planted).  It contains none of the evaluation arithmetic and is used by the tests,
the smoke check and the benchmark to feed the SAME tensors to the CPU oracle and
to the GPU library.  Inputs are always generated once, on one device, and copied.

The five workloads stand in for the candidate-kernel outputs of the paper's
KernelBench-derived operation set (EvoEngineer, arXiv 2510.03760, Sec. 5.1
"Dataset" and the operation taxonomy table in the appendix): feature maps, square
matrices, class logits, tiny loss outputs, softmax rows.  None of that dataset is
reproduced here; shapes and value distributions only.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import torch

SEED_BASE = 0x5EED0000


def _gen(device, config_no: int, stream: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(SEED_BASE + config_no * 100003 + stream)
    return g


@dataclass
class Segment:
    """One reference tensor and the candidates that are checked against it."""
    ref: torch.Tensor                 # flat, contiguous
    cands: List[torch.Tensor]         # flat, contiguous, same dtype and length
    shape: Tuple[int, ...]
    corrupted: List[bool]             # per candidate: built to violate the tolerance
    notes: Dict[str, object] = field(default_factory=dict)

    @property
    def dtype_name(self) -> str:
        return {torch.bfloat16: "bf16", torch.float16: "f16", torch.float64: "f64",
                torch.int32: "i32", torch.int64: "i64"}.get(self.ref.dtype, "f32")

    @property
    def n(self) -> int:
        return self.ref.numel()


@dataclass
class Workload:
    name: str
    segments: List[Segment]
    atol: float
    rtol: float
    timings: torch.Tensor             # [P_total, T] fp32, milliseconds
    baseline: torch.Tensor            # [T] fp32, milliseconds
    notes: Dict[str, object] = field(default_factory=dict)

    @property
    def P(self) -> int:
        """Rows of results: every segment has its own candidates, unless the segments
        are test cases of the same candidates (notes["cases"])."""
        if self.notes.get("cases"):
            return len(self.segments[0].cands)
        return sum(len(s.cands) for s in self.segments)

    @property
    def cand_elems(self) -> int:
        return sum(s.n * len(s.cands) for s in self.segments)

    @property
    def algorithmic_bytes(self) -> int:
        """Reference read once plus every candidate read once."""
        return sum(s.n * s.ref.element_size() * (len(s.cands) + 1) for s in self.segments)


def _timings(device, config_no: int, P: int, T: int, kind: str):
    gt = _gen(device, config_no, 2000)
    gb = _gen(device, config_no, 1999)
    if kind == "uniform":
        t = 1.0 + torch.rand(P, T, generator=gt, device=device, dtype=torch.float32)
        b = 1.0 + torch.rand(T, generator=gb, device=device, dtype=torch.float32)
    elif kind == "lognormal":
        t = torch.exp(0.1 * torch.randn(P, T, generator=gt, device=device, dtype=torch.float32))
        b = torch.exp(0.1 * torch.randn(T, generator=gb, device=device, dtype=torch.float32))
    else:
        raise ValueError(kind)
    return t.contiguous(), b.contiguous()


def _distinct_sites(n: int, k: int, g: torch.Generator, device) -> torch.Tensor:
    """k distinct indices in [0, n), in a seeded random order."""
    if k > n:
        raise ValueError("more sites than elements")
    if n <= (1 << 22):
        return torch.randperm(n, generator=g, device=device)[:k]
    idx = torch.randint(0, n, (4 * k + 64,), generator=g, device=device, dtype=torch.int64)
    idx = torch.unique(idx)
    if idx.numel() < k:
        raise RuntimeError("site draw collided too often")
    order = torch.randperm(idx.numel(), generator=g, device=device)
    return idx[order][:k]


def tiny(device="cpu", side: int = 64) -> Workload:
    """Config 1: fp32 side x side reference ~N(0,1); P=4; T=5 samples ~U(1,2) ms.

    cand0 = ref + N(0, sd 1e-5); cand1 = exact copy; cand2 = noise and +1.0 at 10
    distinct seeded sites; cand3 = noise and one NaN at a seeded site.
    """
    cfg = 1
    n = side * side
    ref = torch.randn(n, generator=_gen(device, cfg, 0), device=device, dtype=torch.float32)
    cands = []
    for p in range(4):
        z = torch.randn(n, generator=_gen(device, cfg, 1 + p), device=device, dtype=torch.float32)
        cands.append(ref + 1e-5 * z)
    cands[1] = ref.clone()
    sites2 = _distinct_sites(n, 10, _gen(device, cfg, 1000 + 2), device)
    cands[2][sites2] += 1.0
    site3 = _distinct_sites(n, 1, _gen(device, cfg, 1000 + 3), device)
    cands[3][site3] = float("nan")
    t, b = _timings(device, cfg, 4, 5, "uniform")
    seg = Segment(ref, cands, (side, side), [False, False, True, True],
                  {"plus_one_sites": sites2.tolist(), "nan_site": int(site3[0])})
    return Workload("C1-tiny-f32-%dx%d-P4" % (side, side), [seg], 1e-2, 1e-2, t, b)


def dense_f32(device="cpu", side: int = 8192, P: int = 16, T: int = 100,
              corrupt_frac: float = 1e-3) -> Workload:
    """Config 2: fp32 side x side ~N(0,1); cand = ref*(1 + N(0, sd 1e-4)); every
    fourth candidate (3, 7, 11, ...) has a Bernoulli(corrupt_frac) set of elements
    replaced by U(-10, 10).  T lognormal(0, 0.1) ms samples per candidate."""
    cfg = 2
    n = side * side
    ref = torch.randn(n, generator=_gen(device, cfg, 0), device=device, dtype=torch.float32)
    cands, corrupted, replaced = [], [], []
    for p in range(P):
        z = torch.randn(n, generator=_gen(device, cfg, 1 + p), device=device, dtype=torch.float32)
        c = ref * (1.0 + 1e-4 * z)
        del z
        bad = (p % 4) == 3
        k = 0
        if bad:
            gs = _gen(device, cfg, 1000 + p)
            mask = torch.rand(n, generator=gs, device=device) < corrupt_frac
            if not bool(mask.any()):
                mask[int(torch.randint(0, n, (1,), generator=gs, device=device))] = True
            u = torch.rand(n, generator=gs, device=device, dtype=torch.float32) * 20.0 - 10.0
            c = torch.where(mask, u, c)
            k = int(mask.sum())
            del mask, u
        cands.append(c.contiguous())
        corrupted.append(bad)
        replaced.append(k)
    t, b = _timings(device, cfg, P, T, "lognormal")
    seg = Segment(ref, cands, (side, side), corrupted, {"replaced": replaced})
    return Workload("C2-f32-%dx%d-P%d" % (side, side, P), [seg], 1e-2, 1e-2, t, b)


def dense_typed(device="cpu", dtype=torch.float64, n: int = 1 << 25, P: int = 16, T: int = 100,
                corrupt_frac: float = 1e-3) -> Workload:
    """The dense recipe of config 2 for the other element types (config number 7).
    binary64: ref ~N(0,1), cand = ref*(1 + N(0, sd 1e-4)), every fourth candidate with a
    Bernoulli(corrupt_frac) set of elements replaced by U(-10, 10).  Integers (the index
    output of an arg-reduction over 4096 positions): ref ~U{0..4095}, candidates equal to
    it, every fourth one with a Bernoulli(corrupt_frac) set of elements redrawn."""
    cfg = 7
    is_int = dtype in (torch.int32, torch.int64)
    if is_int:
        ref = torch.randint(0, 4096, (n,), generator=_gen(device, cfg, 0), device=device, dtype=dtype)
    else:
        ref = torch.randn(n, generator=_gen(device, cfg, 0), device=device, dtype=dtype)
    cands, corrupted = [], []
    for p in range(P):
        if is_int:
            c = ref.clone()
        else:
            z = torch.randn(n, generator=_gen(device, cfg, 1 + p), device=device, dtype=dtype)
            c = ref * (1.0 + 1e-4 * z)
            del z
        bad = (p % 4) == 3
        if bad:
            gs = _gen(device, cfg, 1000 + p)
            mask = torch.rand(n, generator=gs, device=device) < corrupt_frac
            if not bool(mask.any()):
                mask[int(torch.randint(0, n, (1,), generator=gs, device=device))] = True
            if is_int:
                u = torch.randint(0, 4096, (n,), generator=gs, device=device, dtype=dtype)
            else:
                u = torch.rand(n, generator=gs, device=device, dtype=dtype) * 20.0 - 10.0
            c = torch.where(mask, u, c)
            del mask, u
        cands.append(c.contiguous())
        corrupted.append(bad)
    t, b = _timings(device, cfg, P, T, "lognormal")
    name = {torch.float64: "f64", torch.int32: "i32", torch.int64: "i64"}[dtype]
    seg = Segment(ref, cands, (n,), corrupted)
    return Workload("C7-%s-2^%d-P%d" % (name, n.bit_length() - 1, P), [seg], 1e-2, 1e-2, t, b)


def softmax_bf16(device="cpu", B: int = 32, R: int = 128, C: int = 4096, P: int = 64,
                 T: int = 100, dtype=torch.bfloat16) -> Workload:
    """Config 3: bf16 [B, R, C] with softmax rows (fp64 softmax of N(0, sd 3) logits,
    rounded to bf16); each candidate element is moved by +-1 or +-2 bf16 ulp with
    probability one half (clamped to [0, 1]); candidates 7, 15, 23, ... also have the
    R rows of one seeded batch slab rotated by one row.  With dtype=torch.float16 the same
    recipe in binary16 (the half-precision variant of the workload)."""
    cfg = 3
    logits = 3.0 * torch.randn(B, R, C, generator=_gen(device, cfg, 0), device=device,
                               dtype=torch.float64)
    ref = torch.softmax(logits, dim=-1).to(dtype).contiguous()
    del logits
    ref_bits = ref.view(torch.int16).to(torch.int32)
    one_bits = 0x3F80 if dtype == torch.bfloat16 else 0x3C00  # 1.0
    cands, corrupted, slabs = [], [], []
    for p in range(P):
        g = _gen(device, cfg, 1 + p)
        move = torch.rand(B, R, C, generator=g, device=device) < 0.5
        delta = torch.randint(1, 3, (B, R, C), generator=g, device=device, dtype=torch.int32)
        sign = torch.randint(0, 2, (B, R, C), generator=g, device=device, dtype=torch.int32) * 2 - 1
        bits = ref_bits + torch.where(move, delta * sign, torch.zeros_like(delta))
        bits = bits.clamp_(0, one_bits).to(torch.int16)
        c = bits.view(dtype)
        bad = (p % 8) == 7
        slab = -1
        if bad:
            slab = int(torch.randint(0, B, (1,), generator=_gen(device, cfg, 1000 + p),
                                     device=device))
            c = c.clone()
            c[slab] = torch.roll(c[slab], shifts=1, dims=0)
        cands.append(c.contiguous().view(-1))
        corrupted.append(bad)
        slabs.append(slab)
        del move, delta, sign, bits
    t, b = _timings(device, cfg, P, T, "lognormal")
    seg = Segment(ref.view(-1), cands, (B, R, C), corrupted, {"rotated_slab": slabs})
    tag = "C3-bf16" if dtype == torch.bfloat16 else "C3h-f16"
    return Workload("%s-%dx%dx%d-P%d" % (tag, B, R, C, P), [seg], 1e-2, 1e-2, t, b)


RAGGED_SHAPES: Tuple[Tuple[int, ...], ...] = (
    (16, 64, 112, 112), (4096, 4096), (128, 1, 1), (2 ** 20,),
    (8, 3, 224, 224), (512, 512), (64, 128, 256), (1, 1000),
)


def ragged_f32(device="cpu", shapes: Sequence[Tuple[int, ...]] = RAGGED_SHAPES,
               P_s: int = 32, T: int = 100, corrupt_frac: float = 1e-3) -> Workload:
    """Config 4: one fp32 reference ~N(0,1) per shape, P_s candidates each =
    ref + N(0, sd 1e-5); candidates with (p mod 4) == 3 get +1.0 at a
    Bernoulli(corrupt_frac) set of elements (at least one)."""
    cfg = 4
    segs = []
    for s, shape in enumerate(shapes):
        n = 1
        for d in shape:
            n *= d
        ref = torch.randn(n, generator=_gen(device, cfg, 10000 * s), device=device,
                          dtype=torch.float32)
        cands, corrupted, bumped = [], [], []
        for p in range(P_s):
            z = torch.randn(n, generator=_gen(device, cfg, 10000 * s + 1 + p), device=device,
                            dtype=torch.float32)
            c = ref + 1e-5 * z
            del z
            bad = (p % 4) == 3
            k = 0
            if bad:
                gs = _gen(device, cfg, 10000 * s + 1000 + p)
                mask = torch.rand(n, generator=gs, device=device) < corrupt_frac
                if not bool(mask.any()):
                    mask[int(torch.randint(0, n, (1,), generator=gs, device=device))] = True
                c = torch.where(mask, c + 1.0, c)
                k = int(mask.sum())
                del mask
            cands.append(c.contiguous())
            corrupted.append(bad)
            bumped.append(k)
        segs.append(Segment(ref, cands, tuple(shape), corrupted, {"bumped": bumped}))
    P = P_s * len(shapes)
    t, b = _timings(device, cfg, P, T, "lognormal")
    return Workload("C4-ragged-f32-%dshapes-P%d" % (len(shapes), P), segs, 1e-2, 1e-2, t, b)


def heavy_tail_f32(device="cpu", log2n: int = 30, P: int = 8, T: int = 1000,
                   sites_each: int = 1024) -> Workload:
    """Config 5: fp32 2**log2n elements ~Cauchy(0,1) (ratio of two normals) with
    disjoint seeded site sets of subnormals, +Inf, -Inf and NaN written identically
    into the reference and every candidate; cand = ref + 1e-6*|ref|*N(0,1);
    candidates 2 and 5 get extra NaNs at fresh sites, candidate 6 has the sign of
    every Inf site flipped."""
    cfg = 5
    n = 1 << log2n
    k = max(2, min(sites_each, n // 64))
    g0 = _gen(device, cfg, 0)
    ref = torch.randn(n, generator=g0, device=device, dtype=torch.float32)
    den = torch.randn(n, generator=g0, device=device, dtype=torch.float32)
    ref.div_(den)
    del den
    # a Cauchy draw can itself be non-finite (0/0, x/0): make the base finite
    ref = torch.nan_to_num(ref, nan=0.0, posinf=1.0e30, neginf=-1.0e30)
    sites = _distinct_sites(n, 6 * k, _gen(device, cfg, 999), device)
    s_sub, s_pinf, s_ninf, s_nan = (sites[i * k:(i + 1) * k] for i in range(4))
    extra = {2: sites[4 * k:5 * k], 5: sites[5 * k:6 * k]}
    gsub = _gen(device, cfg, 998)
    sub_bits = torch.randint(1, 0x800000, (k,), generator=gsub, device=device, dtype=torch.int32)
    sub_sign = torch.randint(0, 2, (k,), generator=gsub, device=device, dtype=torch.int32) << 31
    sub_vals = (sub_bits | sub_sign).view(torch.float32)

    def plant(x: torch.Tensor, flip_inf: bool) -> None:
        x[s_sub] = sub_vals
        x[s_pinf] = float("-inf") if flip_inf else float("inf")
        x[s_ninf] = float("inf") if flip_inf else float("-inf")
        x[s_nan] = float("nan")

    absref = ref.abs()
    cands, corrupted = [], []
    for p in range(P):
        z = torch.randn(n, generator=_gen(device, cfg, 1 + p), device=device, dtype=torch.float32)
        z.mul_(absref).mul_(1e-6).add_(ref)
        plant(z, flip_inf=(p == 6))
        if p in extra:
            z[extra[p]] = float("nan")
        cands.append(z)
        corrupted.append(True)  # the reference itself holds NaN: nobody is valid
    del absref
    plant(ref, flip_inf=False)
    t, b = _timings(device, cfg, P, T, "lognormal")
    seg = Segment(ref, cands, (n,), corrupted,
                  {"n_ref_nan": k, "n_inf_sites": 2 * k, "n_subnormal": k,
                   "extra_nan": {p: k for p in extra if p < P},
                   "inf_flipped": [p for p in range(P) if p == 6]})
    return Workload("C5-heavy-f32-2^%d-P%d" % (log2n, P), [seg], 1e-4, 1e-4, t, b)


def multi_case_f32(device="cpu", K: int = 5, side: int = 4096, P: int = 16, T: int = 100) -> Workload:
    """Five-test-case workload (the paper's functional testing runs five cases per
    candidate): K independent fp32 side x side references ~N(0,1); candidate p's output for
    case k = ref_k*(1 + N(0, sd 1e-4)); candidates with (p mod 4) == 3 fail exactly one case
    (case p mod K) through a Bernoulli(1e-3) set of elements replaced by U(-10, 10)."""
    cfg = 6
    n = side * side
    segs = []
    for k in range(K):
        ref = torch.randn(n, generator=_gen(device, cfg, 10000 * k), device=device, dtype=torch.float32)
        cands, corrupted = [], []
        for p in range(P):
            z = torch.randn(n, generator=_gen(device, cfg, 10000 * k + 1 + p), device=device,
                            dtype=torch.float32)
            c = ref * (1.0 + 1e-4 * z)
            del z
            bad = (p % 4) == 3 and (p % K) == k
            if bad:
                gs = _gen(device, cfg, 10000 * k + 1000 + p)
                mask = torch.rand(n, generator=gs, device=device) < 1e-3
                if not bool(mask.any()):
                    mask[int(torch.randint(0, n, (1,), generator=gs, device=device))] = True
                u = torch.rand(n, generator=gs, device=device, dtype=torch.float32) * 20.0 - 10.0
                c = torch.where(mask, u, c)
                del mask, u
            cands.append(c.contiguous())
            corrupted.append(bad)
        segs.append(Segment(ref, cands, (side, side), corrupted))
    t, b = _timings(device, cfg, P, T, "lognormal")
    w = Workload("C6-cases-f32-%dx%dx%d-P%d" % (K, side, side, P), segs, 1e-2, 1e-2, t, b,
                 {"cases": True})
    return w


def to_oracle_array(x: torch.Tensor):
    """Host numpy view the CPU oracle accepts (uint16 bits for the 16-bit types, the
    tensor's own element type otherwise)."""
    import numpy as np
    x = x.detach().cpu().contiguous()
    if x.dtype in (torch.bfloat16, torch.float16):
        return x.view(torch.int16).numpy().view(np.uint16)
    return x.numpy()
