"""The sweeps inside a HIP graph: the library allocates nothing, clears nothing with memsets and never
waits for the stream, so a caller may capture forward + backward once and replay them (the launch-bound
small shapes are where that pays).  Every replay is checked bit for bit against the same calls made
eagerly on the same inputs, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from mrf_inputs import DIRS8, make_config, random_problem

pytestmark = pytest.mark.gpu

CASES = [
    ("config 1 isgmr", lambda: make_config(1, algo="isgmr"), False),
    ("config 1 trwp", lambda: make_config(1, algo="trwp"), False),
    ("8 directions, dense table, all gradients", lambda: random_problem(811, "isgmr", 1, 9, 11, 21, DIRS8, 3), True),
    ("config 2 crop trwp", lambda: make_config(2, crop=(24, 40), algo="trwp"), False),
]


def _outputs(g, want_V):
    outs = [g.cost, g.labels, g.p, g.q, g.grad_unary, g.grad_edge_weight]
    if want_V:
        outs.append(g.grad_pairwise)
    return [o.clone() for o in outs]


@pytest.mark.parametrize("name,make,want_V", CASES, ids=[c[0] for c in CASES])
def test_forward_and_backward_replayed_from_a_graph(name, make, want_V):
    from gpu_harness import GpuProblem
    print("case graph", name, flush=True)
    pr = make()
    g = GpuProblem(pr, want_messages=False)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        g.forward()
        g.backward(want_V=want_V)          # (first calls outside the capture: attribute calls of big-LDS kernels)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        g.forward()
        g.backward(want_V=want_V)
    rng = np.random.default_rng(5)
    for replay in range(3):
        # new inputs in place, eager reference first, then poison and replay
        g.unary.add_(torch.from_numpy(rng.random(g.unary.shape, dtype=np.float32) * 0.25).to(g.unary.device))
        g.grad_cost.mul_(-1.25)
        g.forward()
        g.backward(want_V=want_V)
        torch.cuda.synchronize()
        ref = _outputs(g, want_V)
        g.poison_outputs()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = _outputs(g, want_V)
        for a, b in zip(ref, got):
            assert torch.equal(a, b), "replay %d differs from the eager calls" % replay
