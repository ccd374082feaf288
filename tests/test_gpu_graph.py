"""The calls only enqueue kernels on the caller's stream, so once a context has its scratch
memory they can be captured into a HIP graph: replays (with eager work and synchronisations
in between, and with new tensor contents behind the same pointers) must give what the eager
calls give."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_util
    return gpu_util


def test_evaluate_and_select_in_a_graph(gu):
    print("graph capture", flush=True)
    import paper_2510_03760_amd as evo
    P, n, T = 16, 1 << 20, 50
    g = torch.Generator(device="cuda")
    g.manual_seed(11)
    ref = torch.randn(n, generator=g, device="cuda")
    cands = [ref * (1 + 1e-3 * torch.randn(n, generator=g, device="cuda")) for _ in range(P)]
    cands[3][12345] = 9.0
    tim = torch.exp(0.1 * torch.randn(P, T, generator=g, device="cuda")).float()
    base = torch.exp(0.1 * torch.randn(T, generator=g, device="cuda")).float()
    cases = [{"ref": ref, "cand_ptrs": cands, "n_elems": n, "dtype": evo.EVO_F32}]
    chk = evo.Checker(evo.EVO_F32, n, 1e-2, 1e-2)
    stats, summary = chk.new_stats(P), chk.new_summary()
    elite = torch.zeros(4, dtype=torch.int32, device="cuda")
    n_elite = torch.zeros(1, dtype=torch.int32, device="cuda")

    def eager():
        s, m = chk.new_stats(P), chk.new_summary()
        e, ne = torch.zeros_like(elite), torch.zeros_like(n_elite)
        chk.evaluate(cases, tim, base, s, m)
        chk.select_elite(s, P, 4, e, ne)
        torch.cuda.synchronize()
        return s, m, e, ne

    want = eager()                       # also allocates the context's scratch memory
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        chk.evaluate(cases, tim, base, stats, summary)          # on the capture stream
        chk.select_elite(stats, P, 4, elite, n_elite)
    for rep in range(4):
        stats.fill_(0xAB)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(stats, want[0]) and torch.equal(summary, want[1]), rep
        assert torch.equal(elite, want[2]) and torch.equal(n_elite, want[3]), rep
        if rep == 1:
            # new contents behind the same pointers: the graph must follow them
            cands[5][777] = float("nan")
            tim[2] *= 0.25
            want = eager()
        else:
            eager()                      # eager work between replays
    assert int(want[3][0]) == 4
    chk.close()
