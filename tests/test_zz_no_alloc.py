"""The entry point that allocates nothing: mrf_energy_noalloc keeps its partial sums in a device
array of the library's own.  Checked through the C ABI against mrf_energy (same kernels, caller's
workspace), which the other tests check against the fp64 oracle; two calls in a row, the second on
a smaller input, so that what the first call left in the shared array cannot leak into the second."""
import numpy as np
import pytest

from mrf_inputs import DIRS4, DIRS8, random_problem

pytestmark = pytest.mark.gpu


def _energies(pr, lab):
    import torch
    import paper_1910_10892_amd as mrf
    from gpu_harness import GpuProblem
    g = GpuProblem(pr, want_messages=False)
    B = pr.shape[0]
    labels = torch.from_numpy(lab).cuda()
    ws = torch.empty(mrf.mrf_energy_workspace_bytes(g.prob), dtype=torch.uint8, device="cuda:0")
    ref = torch.full((B,), float("nan"), dtype=torch.float64, device="cuda:0")
    mrf.mrf_energy(g.prob, labels, ref, ws)
    out = torch.full((B,), float("nan"), dtype=torch.float64, device="cuda:0")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    mrf.mrf_energy_noalloc(g.prob, labels, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return out.cpu().numpy(), ref.cpu().numpy()


def test_energy_noalloc_equals_energy_on_two_calls_in_a_row():
    from oracle import mrf_heads_oracle as ho
    # first a batch of large images (every partial-sum slot of four images is written) ...
    big = random_problem(401, "isgmr", 4, 96, 130, 21, DIRS8, 1, symmetric=False)
    rng = np.random.default_rng(402)
    lab_big = rng.integers(0, 21, (4, 96, 130)).astype(np.uint8)
    print("case no-alloc energy, first call", big.shape, flush=True)
    got, ref = _energies(big, lab_big)
    np.testing.assert_array_equal(got, ref)          # same kernels, same order of the sums
    # ... then a small one, whose sums use a few slots of the same array
    small = random_problem(403, "isgmr", 2, 5, 7, 9, DIRS4, 1, symmetric=False)
    lab_small = rng.integers(0, 9, (2, 5, 7)).astype(np.uint8)
    print("case no-alloc energy, second call", small.shape, flush=True)
    got, ref = _energies(small, lab_small)
    np.testing.assert_array_equal(got, ref)
    want = ho.energy(small.unary, small.pairwise, small.dirs, lab_small, edge_weight=small.edge_weight,
                     edge_weight_scalar=small.edge_weight_scalar)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-9)


def test_energy_noalloc_rejects_batches_beyond_its_scratch():
    import torch
    import paper_1910_10892_amd as mrf
    from gpu_harness import GpuProblem
    pr = random_problem(404, "isgmr", 65, 2, 2, 3, DIRS4, 1)
    g = GpuProblem(pr, want_messages=False)
    out = torch.zeros((65,), dtype=torch.float64, device="cuda:0")
    with pytest.raises(mrf.MrfError) as ei:
        mrf.mrf_energy_noalloc(g.prob, torch.zeros((65, 2, 2), dtype=torch.uint8, device="cuda:0"), out)
    assert ei.value.status == -10
    assert "scratch" in str(ei.value)
