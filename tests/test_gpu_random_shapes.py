"""GPU parity on seeded random launches: sizes, populations, element types, alignment and
kinds of candidates drawn at random, one segment or several, every row against the oracle.
The fixed cases elsewhere aim at known edges; this one walks the combinations in between
(population sizes that pad or split, tiles that are NaN or Inf throughout next to tiles
that are not, unaligned tensors in a launch with aligned ones)."""
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


DTYPES = [torch.float32, torch.bfloat16, torch.float16, torch.float64]
SPECIALS = [float("nan"), float("inf"), float("-inf"), 0.0, -0.0, 1e-41, 3e38, -3e38, 6e-5]


def _candidate(kind, ref32, rs, g):
    n = ref32.numel()
    if kind == "near":
        return ref32 * (1 + 0.004 * torch.randn(n, generator=g, device="cuda"))
    if kind == "copy":
        return ref32.clone()
    if kind == "far":
        return 20 * torch.rand(n, generator=g, device="cuda") - 10
    if kind == "nan":
        return torch.full_like(ref32, float("nan"))
    if kind == "inf":
        c = torch.full_like(ref32, float("inf"))
        c[::3] = float("-inf")
        return c
    if kind == "nan_inf":
        c = torch.full_like(ref32, float("nan"))
        c[1::2] = float("inf")
        return c
    if kind == "nan_block":                        # NaN over a random stretch, right elsewhere
        c = ref32.clone()
        lo = int(rs.integers(0, n))
        hi = min(n, lo + int(rs.integers(1, 6000)))
        c[lo:hi] = float("nan")
        return c
    if kind == "nan_but_one":                      # NaN except one element per kilo-element
        c = torch.full_like(ref32, float("nan"))
        c[int(rs.integers(0, min(n, 1000)))::1000] = 1.0
        return c
    if kind == "sprinkled":
        c = ref32 * (1 + 0.004 * torch.randn(n, generator=g, device="cuda"))
        k = max(1, n // 500)
        idx = torch.randint(0, n, (k,), generator=g, device="cuda")
        c[idx] = torch.tensor(SPECIALS, device="cuda")[torch.randint(0, len(SPECIALS), (k,), generator=g,
                                                                     device="cuda")]
        return c
    raise AssertionError(kind)


KINDS = ["near", "near", "near", "copy", "far", "nan", "inf", "nan_inf", "nan_block", "nan_but_one", "sprinkled"]


def _segment(rs, g, dtype, n, P, unaligned):
    ref32 = 3 * torch.randn(n + 1, generator=g, device="cuda")
    if rs.random() < 0.5:                          # special values in the reference too
        k = max(1, n // 2000)
        idx = torch.randint(0, n, (k,), generator=g, device="cuda")
        ref32[idx] = torch.tensor(SPECIALS, device="cuda")[torch.randint(0, len(SPECIALS), (k,), generator=g,
                                                                         device="cuda")]
    if rs.random() < 0.2:
        ref32 = ref32 * 1e33                       # beyond the range where the NaN/Inf shortcut may apply
    off = 1 if unaligned else 0
    ref = ref32.to(dtype)[off:off + n]
    cands = []
    for _ in range(P):
        kind = KINDS[int(rs.integers(0, len(KINDS)))]
        c = _candidate(kind, ref32[:n + 1].clone(), rs, g).to(dtype)
        o = 1 if (unaligned and rs.random() < 0.5) else 0
        cands.append(c[o:o + n] if o else c[:n].clone())
    return synth.Segment(ref, cands, (n,), [True] * P)


@pytest.mark.parametrize("seed", list(range(100)))
def test_random_launch(gu, seed):
    rs = np.random.default_rng(1000 + seed)
    g = torch.Generator(device="cuda")
    g.manual_seed(5000 + seed)
    S = 1 if seed % 3 else int(rs.integers(2, 6))
    segs = []
    for s in range(S):
        dtype = DTYPES[int(rs.integers(0, 4)) if seed >= 60 else int(rs.integers(0, 3))]
        tile = {torch.float32: 512, torch.float64: 256}.get(dtype, 1024)
        big = rs.random() < 0.35
        n = int(rs.integers(1, 40 * tile)) if not big else int(rs.integers(1024 * tile, 1400 * tile))
        P = int(rs.choice([1, 2, 3, 5, 6, 7, 9, 11, 12, 13, 15, 16, 17, 20, 27, 33, 37, 48, 65]))
        if big:
            P = min(P, 37)
        segs.append(_segment(rs, g, dtype, n, P, unaligned=rs.random() < 0.15))
    _say("seed %d: %s" % (seed, [(s.dtype_name, s.n, len(s.cands)) for s in segs]))
    Ptot = sum(len(s.cands) for s in segs)
    w = synth.Workload("random-%d" % seed, segs, 1e-2, 1e-2, torch.ones(Ptot, 4, device="cuda"),
                       torch.ones(4, device="cuda"))
    chk, stats, want = gu.check_parity(w, segmented=(S > 1) or bool(seed % 2), label="random %d" % seed)
    chk.close()
