"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element-exact
on integers and maxima, 1e-6 relative on the two error sums."""
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


def test_config1_tiny(gu):
    _say("C1 tiny")
    w = synth.tiny("cuda")
    chk, stats, want = gu.check_parity(w)
    assert [r["n_mismatch"] for r in want] == [0, 0, 10, 1]
    gu.fitness_parity(chk, stats, w.timings, w.baseline, label="C1")
    chk.close()


@pytest.mark.parametrize("side,P", [(256, 16), (1000, 16), (1024, 5), (777, 16)])
def test_config2_reduced(gu, side, P):
    _say("C2 reduced side=%d P=%d" % (side, P))
    w = synth.dense_f32("cuda", side=side, P=P, T=100, corrupt_frac=1e-3)
    chk, stats, want = gu.check_parity(w)
    gu.fitness_parity(chk, stats, w.timings, w.baseline, label="C2r")
    chk.close()


def test_config3_reduced_bf16(gu):
    _say("C3 reduced")
    w = synth.softmax_bf16("cuda", B=4, R=32, C=1000, P=64, T=100)
    chk, stats, want = gu.check_parity(w)
    assert sum(r["valid"] for r in want) == 56
    gu.fitness_parity(chk, stats, w.timings, w.baseline, label="C3r")
    chk.close()


def test_config3_reduced_f16(gu):
    _say("C3 reduced, binary16")
    w = synth.softmax_bf16("cuda", B=4, R=32, C=1000, P=64, T=100, dtype=torch.float16)
    chk, stats, want = gu.check_parity(w)
    assert sum(r["valid"] for r in want) == 56
    gu.fitness_parity(chk, stats, w.timings, w.baseline, label="C3h")
    chk.close()


def test_config4_reduced_ragged(gu):
    _say("C4 reduced")
    shapes = ((4, 16, 28, 28), (512, 512), (128, 1, 1), (2 ** 16,), (8, 3, 56, 56), (128, 128),
              (16, 32, 64), (1, 1000))
    w = synth.ragged_f32("cuda", shapes=shapes, P_s=32, T=100)
    chk, stats, want = gu.check_parity(w)
    assert sum(r["valid"] for r in want) == 192
    gu.fitness_parity(chk, stats, w.timings, w.baseline, label="C4r")
    chk.close()


def test_config5_reduced_heavy_tail(gu):
    _say("C5 reduced")
    w = synth.heavy_tail_f32("cuda", log2n=22, P=8, T=1000)
    chk, stats, want = gu.check_parity(w)
    assert all(r["valid"] == 0 for r in want)
    gu.fitness_parity(chk, stats, w.timings, w.baseline, label="C5r")
    chk.close()
