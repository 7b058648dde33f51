"""GPU parity of the two heads (energy of a labelling, SoftMin regression + L1) with their fp64
oracle, through the C ABI."""
import numpy as np
import pytest

from mrf_inputs import DIRS4, DIRS8, make_config, random_problem

pytestmark = pytest.mark.gpu


def _gpu_problem(pr):
    from gpu_harness import GpuProblem
    return GpuProblem(pr, want_messages=False)


@pytest.mark.parametrize("case", [
    (1, 1, 5, 7, 9, DIRS4, True), (2, 3, 6, 5, 33, DIRS8, True), (3, 1, 1, 9, 4, DIRS4, False),
    (4, 2, 40, 70, 96, DIRS4, True), (5, 1, 7, 1, 256, [(0, 1), (1, 0), (-1, 0)], True),
], ids=lambda c: "seed%d" % c[0])
def test_energy_matches_oracle(case):
    import torch
    import paper_1910_10892_amd as mrf
    from oracle import mrf_heads_oracle as ho
    seed, B, H, W, L, dirs, per_edge = case
    print("case energy", case[:5], flush=True)
    pr = random_problem(seed, "isgmr", B, H, W, L, dirs, 1, per_edge=per_edge, symmetric=False)
    rng = np.random.default_rng(seed + 500)
    lab = rng.integers(0, L, (B, H, W)).astype(np.uint8)
    g = _gpu_problem(pr)
    ws = torch.empty(mrf.mrf_energy_workspace_bytes(g.prob), dtype=torch.uint8, device="cuda:0")
    out = torch.full((B,), float("nan"), dtype=torch.float64, device="cuda:0")
    mrf.mrf_energy(g.prob, torch.from_numpy(lab).cuda(), out, ws)
    ref = ho.energy(pr.unary, pr.pairwise, pr.dirs, lab, edge_weight=pr.edge_weight,
                    edge_weight_scalar=pr.edge_weight_scalar)
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-12, atol=1e-9)


@pytest.mark.parametrize("case", [(11, 2, 5, 7, 9, DIRS4), (12, 1, 6, 4, 21, DIRS8), (13, 1, 3, 5, 64, [(0, 1), (1, 0), (-1, 0)])],
                         ids=lambda c: "seed%d" % c[0])
def test_energy_with_pairwise_potentials_per_edge(case):
    """Problems that give one table per edge (and no V): the energy reads theta_{i-r,i}(x_{i-r}, x_i)
    from the edge's table."""
    import torch
    import paper_1910_10892_amd as mrf
    from oracle import mrf_heads_oracle as ho
    seed, B, H, W, L, dirs = case
    print("case energy, per-edge tables", case[:5], flush=True)
    pr = random_problem(seed, "isgmr", B, H, W, L, dirs, 1, per_edge=False)
    rng = np.random.default_rng(seed + 600)
    pr.pairwise_edge = rng.random((len(dirs), B, H, W, L, L)).astype(np.float32)
    lab = rng.integers(0, L, (B, H, W)).astype(np.uint8)
    g = _gpu_problem(pr)
    assert g.prob.pairwise is None
    ws = torch.empty(mrf.mrf_energy_workspace_bytes(g.prob), dtype=torch.uint8, device="cuda:0")
    out = torch.full((B,), float("nan"), dtype=torch.float64, device="cuda:0")
    mrf.mrf_energy(g.prob, torch.from_numpy(lab).cuda(), out, ws)
    ref = ho.energy(pr.unary, None, pr.dirs, lab, pairwise_edge=pr.pairwise_edge)
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-12, atol=1e-9)


def test_energy_of_the_labelling_the_sweeps_return():
    """Forward pass, then the energy of its labels, on the stereo recipe (cropped)."""
    import torch
    import paper_1910_10892_amd as mrf
    from oracle import mrf_heads_oracle as ho
    print("case energy of forward labels", flush=True)
    pr = make_config(2, crop=(24, 40))
    g = _gpu_problem(pr)
    g.forward()
    ws = torch.empty(mrf.mrf_energy_workspace_bytes(g.prob), dtype=torch.uint8, device="cuda:0")
    out = torch.empty((1,), dtype=torch.float64, device="cuda:0")
    mrf.mrf_energy(g.prob, g.labels, out, ws)
    ref = ho.energy(pr.unary, pr.pairwise, pr.dirs, g.labels.cpu().numpy(), edge_weight=pr.edge_weight,
                    edge_weight_scalar=pr.edge_weight_scalar)
    np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-12, atol=1e-9)


@pytest.mark.parametrize("index,crop", [(2, (24, 40)), (4, (10, 12))])
@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_energy_minimisation_protocol_on_crops(oracle, index, crop, algo):
    """The protocol of the energy tables of Sec. 5.1 on synthetic stand-ins: run K = 1 and K = 50
    iterations, take the labelling, evaluate its energy.  Labels against the oracle's forward pass,
    the energy of those labels against the fp64 definition (the tables' own numbers need the
    paper's datasets: parity with them is unpinned)."""
    import torch
    import paper_1910_10892_amd as mrf
    from oracle import mrf_heads_oracle as ho
    energies = {}
    for K in (1, 50):
        print("case energy protocol", index, crop, algo, K, flush=True)
        pr = make_config(index, crop=crop, algo=algo, K=K)
        g = _gpu_problem(pr)
        g.forward()
        f = oracle.forward(pr.algo, pr.unary, pr.pairwise, pr.dirs, pr.K, edge_weight=pr.edge_weight,
                           edge_weight_scalar=pr.edge_weight_scalar, rho=pr.rho, threads=True)
        labels = g.labels.cpu().numpy()
        np.testing.assert_array_equal(labels, f.labels)
        ws = torch.empty(mrf.mrf_energy_workspace_bytes(g.prob), dtype=torch.uint8, device="cuda:0")
        out = torch.empty((pr.shape[0],), dtype=torch.float64, device="cuda:0")
        mrf.mrf_energy(g.prob, g.labels, out, ws)
        ref = ho.energy(pr.unary, pr.pairwise, pr.dirs, f.labels, edge_weight=pr.edge_weight,
                        edge_weight_scalar=pr.edge_weight_scalar)
        np.testing.assert_allclose(out.cpu().numpy(), ref, rtol=1e-12, atol=1e-9)
        energies[K] = float(ref.sum())
    print("  energies", energies, flush=True)
    assert np.isfinite(list(energies.values())).all()


@pytest.mark.parametrize("n,L,masked", [(1, 1, False), (37, 2, False), (1000, 96, True), (513, 200, True),
                                        (4099, 21, False), (64, 256, True)])
def test_softmin_l1_matches_oracle(n, L, masked):
    import torch
    import paper_1910_10892_amd as mrf
    from oracle import mrf_heads_oracle as ho
    print("case softmin", n, L, masked, flush=True)
    rng = np.random.default_rng(900 + n + L)
    cost = rng.normal(0.0, 3.0, (n, L)).astype(np.float32)
    target = rng.uniform(0.0, max(L - 1, 1), n).astype(np.float32)
    mask = (rng.random(n) > 0.25).astype(np.uint8) if masked else None
    ws = torch.empty(mrf.mrf_softmin_l1_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
    disp = torch.full((n,), float("nan"), device="cuda:0")
    grad = torch.full((n, L), float("nan"), device="cuda:0")
    loss = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
    for _ in range(2):      # twice: the workspace keeps nothing that matters from call to call
        mrf.mrf_softmin_l1(torch.from_numpy(cost).cuda(), torch.from_numpy(target).cuda(),
                           None if mask is None else torch.from_numpy(mask).cuda(), disp, loss, grad, ws)
    d, l, gr = ho.softmin_l1(cost, target, mask)
    np.testing.assert_allclose(disp.cpu().numpy(), d, rtol=1e-5, atol=1e-4)
    np.testing.assert_allclose(loss.cpu().numpy()[0], l, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(grad.cpu().numpy(), gr, rtol=1e-5, atol=1e-7 / max(n, 1) + 1e-12)


@pytest.mark.parametrize("n,L,masked,beta", [(1000, 96, True, 1.0), (513, 21, False, 0.25), (64, 256, True, 3.0)])
def test_softmin_smooth_l1_matches_oracle(n, L, masked, beta):
    import torch
    import paper_1910_10892_amd as mrf
    from oracle import mrf_heads_oracle as ho
    print("case softmin smooth l1", n, L, masked, beta, flush=True)
    rng = np.random.default_rng(950 + n + L)
    cost = rng.normal(0.0, 3.0, (n, L)).astype(np.float32)
    d0, _, _ = ho.softmin_l1(cost, np.zeros(n))
    # targets on both sides of the threshold |d - g| = beta
    target = (d0 + rng.uniform(-3.0 * beta, 3.0 * beta, n)).astype(np.float32)
    mask = (rng.random(n) > 0.25).astype(np.uint8) if masked else None
    ws = torch.empty(mrf.mrf_softmin_l1_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
    disp = torch.full((n,), float("nan"), device="cuda:0")
    grad = torch.full((n, L), float("nan"), device="cuda:0")
    loss = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda:0")
    mrf.mrf_softmin_smooth_l1(torch.from_numpy(cost).cuda(), torch.from_numpy(target).cuda(),
                              None if mask is None else torch.from_numpy(mask).cuda(), beta, disp, loss, grad, ws)
    d, l, gr = ho.softmin_l1(cost, target, mask, beta=beta)
    np.testing.assert_allclose(disp.cpu().numpy(), d, rtol=1e-5, atol=1e-4)
    # (the regressed disparity carries the single-precision exponential: about 1e-6 relative)
    np.testing.assert_allclose(loss.cpu().numpy()[0], l, rtol=1e-5, atol=1e-7)
    # (inside the threshold the slope (d - g) / beta inherits the absolute error of d, about 1e-7 L)
    np.testing.assert_allclose(grad.cpu().numpy(), gr, rtol=1e-4, atol=2e-4 / max(n, 1))
    with pytest.raises(mrf.MrfError):
        mrf.mrf_softmin_smooth_l1(torch.from_numpy(cost).cuda(), torch.from_numpy(target).cuda(), None, 0.0, disp, loss,
                                  grad, ws)


def test_heads_reject_bad_arguments():
    import torch
    import paper_1910_10892_amd as mrf
    ws = torch.empty(16, dtype=torch.uint8, device="cuda:0")
    c = torch.zeros((4, 3), device="cuda:0")
    t = torch.zeros((4,), device="cuda:0")
    loss = torch.zeros((1,), dtype=torch.float64, device="cuda:0")
    with pytest.raises(mrf.MrfError) as ei:
        mrf.mrf_softmin_l1(c, t, None, None, loss, None, ws)
    assert ei.value.status == -6


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_autograd_wrapper_returns_the_library_gradients(algo):
    """cost -> SoftMin + L1 head -> backward through torch.autograd equals the oracle's gradients of
    the same composite (oracle backward fed with the oracle head's grad_cost)."""
    import torch
    from oracle import mrf_oracle, mrf_heads_oracle as ho
    from paper_1910_10892_amd.autograd import message_passing
    import paper_1910_10892_amd as mrf
    print("case autograd", algo, flush=True)
    pr = random_problem(33, algo, 1, 6, 7, 12, DIRS4, 2, rho=np.linspace(0.4, 0.8, 4))
    rng = np.random.default_rng(77)
    target = rng.uniform(0, 11, (1, 6, 7)).astype(np.float32)
    unary = torch.from_numpy(pr.unary).cuda().requires_grad_(True)
    V = torch.from_numpy(pr.pairwise).cuda().requires_grad_(True)
    w = torch.from_numpy(pr.edge_weight).cuda().requires_grad_(True)
    cost, labels = message_passing(unary, V, w, algo=algo, dirs=pr.dirs, K=pr.K, rho=pr.rho)
    ws = torch.empty(mrf.mrf_softmin_l1_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
    loss = torch.empty((1,), dtype=torch.float64, device="cuda:0")
    gcost = torch.empty_like(cost)
    mrf.mrf_softmin_l1(cost.detach(), torch.from_numpy(target).cuda(), None, None, loss, gcost, ws)
    cost.backward(gcost)
    f = mrf_oracle.forward(pr.algo, pr.unary, pr.pairwise, pr.dirs, pr.K, edge_weight=pr.edge_weight,
                           edge_weight_scalar=pr.edge_weight_scalar, rho=pr.rho)
    assert (labels.cpu().numpy() == f.labels).all()
    _, l_ref, g_ref = ho.softmin_l1(f.cost, target)
    b = mrf_oracle.backward(pr.algo, pr.shape, pr.pairwise, pr.dirs, pr.K, g_ref.astype(np.float32), f.p, f.q,
                            edge_weight=pr.edge_weight, edge_weight_scalar=pr.edge_weight_scalar, rho=pr.rho,
                            dtype=np.float64)
    assert loss.cpu().numpy()[0] == pytest.approx(l_ref, rel=1e-6)
    np.testing.assert_allclose(unary.grad.cpu().numpy(), b.grad_unary, rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(w.grad.cpu().numpy(), b.grad_edge_weight, rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(V.grad.cpu().numpy(), b.grad_pairwise, rtol=1e-4, atol=1e-6)


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_autograd_wrapper_for_per_edge_tables(algo):
    """The same composite with pairwise potentials given per edge: gradients of unary and of the
    tables equal the oracle's."""
    import torch
    from oracle import mrf_oracle, mrf_heads_oracle as ho
    from paper_1910_10892_amd.autograd import message_passing_edge_tables
    import paper_1910_10892_amd as mrf
    print("case autograd, per-edge tables", algo, flush=True)
    pr = random_problem(34, algo, 1, 5, 6, 9, DIRS4, 2, rho=np.linspace(0.4, 0.8, 4))
    rng = np.random.default_rng(78)
    Te = rng.random((4, 1, 5, 6, 9, 9)).astype(np.float32)
    target = rng.uniform(0, 8, (1, 5, 6)).astype(np.float32)
    unary = torch.from_numpy(pr.unary).cuda().requires_grad_(True)
    tab = torch.from_numpy(Te).cuda().requires_grad_(True)
    cost, labels = message_passing_edge_tables(unary, tab, algo=algo, dirs=pr.dirs, K=pr.K, rho=pr.rho)
    ws = torch.empty(mrf.mrf_softmin_l1_workspace_bytes(), dtype=torch.uint8, device="cuda:0")
    loss = torch.empty((1,), dtype=torch.float64, device="cuda:0")
    gcost = torch.empty_like(cost)
    mrf.mrf_softmin_l1(cost.detach(), torch.from_numpy(target).cuda(), None, None, loss, gcost, ws)
    cost.backward(gcost)
    f = mrf_oracle.forward(pr.algo, pr.unary, None, pr.dirs, pr.K, rho=pr.rho, pairwise_edge=Te)
    assert (labels.cpu().numpy() == f.labels).all()
    _, l_ref, g_ref = ho.softmin_l1(f.cost, target)
    b = mrf_oracle.backward(pr.algo, pr.shape, None, pr.dirs, pr.K, g_ref.astype(np.float32), f.p, f.q, rho=pr.rho,
                            dtype=np.float64, per_edge_pairwise=True)
    assert loss.cpu().numpy()[0] == pytest.approx(l_ref, rel=1e-6)
    np.testing.assert_allclose(unary.grad.cpu().numpy(), b.grad_unary, rtol=1e-4, atol=1e-6)
    np.testing.assert_allclose(tab.grad.cpu().numpy(), b.grad_pairwise_edge, rtol=1e-4, atol=1e-6)
