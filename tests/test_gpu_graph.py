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


def test_capture_is_refused_when_the_call_would_allocate_or_stage(gu):
    """Under stream capture a call may only enqueue kernels.  A context that has never run the
    shape (its scratch memory would have to be allocated and cleared) and a launch whose
    table does not fit the kernel arguments (it would be copied from a staging buffer that
    later calls overwrite) are refused with EVO_ERR_CAPTURE before anything is enqueued; the
    same calls work eagerly, and after the eager run the first one can be captured."""
    print("graph capture: refused cases", flush=True)
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy
    n, T = 50000, 8
    g = torch.Generator(device="cuda")
    g.manual_seed(12)
    ref = torch.randn(n, generator=g, device="cuda")
    cands = [ref + 1e-3 * torch.randn(n, generator=g, device="cuda") for _ in range(6)]
    cands[2][17] = 5.0
    tim = 1 + torch.rand(6, T, generator=g, device="cuda")
    base = 1 + torch.rand(T, generator=g, device="cuda")
    cases = [{"ref": ref, "cand_ptrs": cands, "n_elems": n, "dtype": evo.EVO_F32}]
    scratch = torch.zeros(16, device="cuda")

    fresh = evo.Checker(evo.EVO_F32, n, 1e-2, 1e-2)
    stats, summary = fresh.new_stats(6), fresh.new_summary()
    stats.fill_(0x33)
    codes = []
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        scratch.add_(1.0)                     # the graph is not empty
        for call in (lambda: fresh.check_batch(ref, cands, stats),
                     lambda: fresh.evaluate(cases, tim, base, stats, summary),
                     lambda: fresh.fitness(tim, base, stats, summary)):
            try:
                call()
                codes.append(0)
            except evo.EvoError as e:
                codes.append(e.code)
    assert codes == [-10, -10, -10], codes
    graph.replay()
    torch.cuda.synchronize()
    assert int(stats.min()) == 0x33 and int(stats.max()) == 0x33    # nothing was recorded

    # eager run of the same shape, then the capture goes through and replays give its result
    want_stats, want_summary = fresh.new_stats(6), fresh.new_summary()
    fresh.evaluate(cases, tim, base, want_stats, want_summary)
    torch.cuda.synchronize()
    graph2 = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph2):
        fresh.evaluate(cases, tim, base, stats, summary)
    for rep in range(3):
        stats.fill_(0x44)
        graph2.replay()
        torch.cuda.synchronize()
        assert torch.equal(stats, want_stats) and torch.equal(summary, want_summary), rep
        fresh.check_batch(ref, cands, fresh.new_stats(6))          # eager work between replays
        torch.cuda.synchronize()

    # 400 candidate pointers do not fit the kernel arguments: staged path, eager only
    many = [ref] * 399 + [cands[2]]
    big = fresh.new_stats(400)
    fresh.check_batch(ref, many, big)                               # eager: allocates, stages, runs
    torch.cuda.synchronize()
    rows = stats_to_numpy(big)
    assert int(rows["valid"][:399].sum()) == 399 and int(rows["n_mismatch"][399]) == 1
    graph3 = torch.cuda.CUDAGraph()
    code = 0
    with torch.cuda.graph(graph3):
        scratch.add_(1.0)
        try:
            fresh.check_batch(ref, many, big)
        except evo.EvoError as e:
            code = e.code
    assert code == -10
    fresh.close()
