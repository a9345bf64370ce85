"""fo_step_dev_round captured into a HIP graph (through torch.cuda.CUDAGraph) and replayed: every replay must give
exactly what the eager fo_step gives for that round.  Between replays the program does eager work and
synchronises, and every replay is checked, not just the first."""
import time

import pytest

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,d,M,blk", [("c1_two_pass", 1 << 16, 4, 0), ("single_tile", 20_000, 3, 0),
                                          ("blocked", 100_000, 2, 10)])
def test_graph_replays_match_eager_rounds(oracle, name, d, M, blk):
    import torch
    from paper_2405_11095_amd import binding as B, inputs
    dev = torch.device("cuda:0")
    gs = [torch.from_numpy(inputs.gaussian(d, m)).to(dev) for m in range(M)]
    delta, rounds = 0.01, 8

    plan_e = B.Plan(d=d, M=M, block_log2=blk, seed=91)
    x_e = torch.zeros(d, dtype=torch.float32, device=dev)
    want = []
    for r in range(rounds):
        plan_e.fo_step(gs, x_e, delta, r)
        want.append(x_e.clone())
    torch.cuda.synchronize()

    plan_g = B.Plan(d=d, M=M, block_log2=blk, seed=91)
    x_g = torch.zeros(d, dtype=torch.float32, device=dev)
    rnd = torch.zeros(1, dtype=torch.int64, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                     # warm-up outside the capture, as torch asks
        plan_g.fo_step_dev_round(gs, x_g, delta, rnd)
        rnd.add_(1)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    assert torch.equal(x_g, want[0])                  # the eager call with a device-side round is the same step
    x_g.zero_()
    rnd.zero_()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        plan_g.fo_step_dev_round(gs, x_g, delta, rnd)
        rnd.add_(1)                                   # an increment kernel, captured with the step
    scratch = torch.zeros(1 << 20, device=dev)
    for r in range(rounds):
        graph.replay()
        scratch.add_(1.0)                             # eager work of the program between replays
        torch.cuda.synchronize()
        assert torch.equal(x_g, want[r]), f"replay {r}"
    assert int(rnd.item()) == rounds

    # launch-bound sizes are what graphs are for: time both ways
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for r in range(50):
        plan_e.fo_step(gs, x_e, delta, rounds + r)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for r in range(50):
        graph.replay()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    print(f"{name}: eager {(t1 - t0) / 50 * 1e3:.3f} ms per step, graph replay {(t2 - t1) / 50 * 1e3:.3f} ms per step")
    plan_e.close()
    plan_g.close()
