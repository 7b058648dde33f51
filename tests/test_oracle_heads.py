"""Pins of the heads oracle (energy of a labelling, SoftMin regression + L1) against things it
does not compute itself: explicit edge lists fed to the brute-force energy routine, closed
forms, finite differences, invariants."""
import numpy as np
import pytest

from bruteforce import all_labelings, energies
from oracle import mrf_heads_oracle as ho

DIRS4 = [(0, 1), (0, -1), (1, 0), (-1, 0)]
DIRS8 = DIRS4 + [(1, 1), (-1, -1), (1, -1), (-1, 1)]


def explicit_edges(H, W, dirs, w, V):
    """One entry per undirected neighbour pair, written from the grid alone: for every
    unordered pair of opposite directions the copy that appears first in dirs."""
    dirs = [tuple(d) for d in dirs]
    edges = []
    seen = set()
    for r, (dh, dw) in enumerate(dirs):
        if (-dh, -dw) in seen:
            continue
        seen.add((dh, dw))
        for y in range(H):
            for x in range(W):
                ys, xs = y - dh, x - dw
                if 0 <= ys < H and 0 <= xs < W:
                    edges.append((ys * W + xs, y * W + x, float(w[r, 0, y, x]), V))
    return edges


@pytest.mark.parametrize("H,W,L,dirs", [(2, 3, 3, DIRS4), (2, 2, 3, DIRS8), (1, 4, 4, DIRS4), (3, 2, 2, [(0, 1), (1, 0), (-1, 0)])])
def test_energy_matches_enumeration_over_explicit_edges(H, W, L, dirs):
    rng = np.random.default_rng(7 + H * 10 + W)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L))                       # asymmetric: pins the orientation V[x_src][x_dst]
    w = rng.uniform(0.5, 1.5, (len(dirs), 1, H, W))
    X = all_labelings(H * W, L)
    E = energies(X, unary.reshape(H * W, L), explicit_edges(H, W, dirs, w, V))
    for k in range(0, X.shape[0], max(1, X.shape[0] // 50)):
        lab = X[k].reshape(1, H, W)
        got = ho.energy(unary, V, np.array(dirs), lab, edge_weight=w)
        assert got.shape == (1,)
        np.testing.assert_allclose(got[0], E[k], rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("H,W,L,dirs", [(2, 3, 3, DIRS4), (2, 2, 2, DIRS8), (3, 1, 3, [(1, 0), (0, 1)])])
def test_energy_with_one_table_per_edge_matches_enumeration(H, W, L, dirs):
    """Pairwise potentials given per edge: every edge of the explicit list carries its own table."""
    rng = np.random.default_rng(70 + H * 10 + W)
    unary = rng.random((1, H, W, L))
    Te = rng.random((len(dirs), 1, H, W, L, L))
    ones = np.ones((len(dirs), 1, H, W))
    edges = [(a, b) for a, b, _, _ in explicit_edges(H, W, dirs, ones, None)]
    # the table of edge (a, b) lives at the destination node b, under the direction that produced the edge
    d = [tuple(v) for v in dirs]
    table = {}
    seen = set()
    for r, (dh, dw) in enumerate(d):
        if (-dh, -dw) in seen:
            continue
        seen.add((dh, dw))
        for y in range(H):
            for x in range(W):
                ys, xs = y - dh, x - dw
                if 0 <= ys < H and 0 <= xs < W:
                    table[(ys * W + xs, y * W + x)] = Te[r, 0, y, x]
    assert sorted(table) == sorted(edges)
    X = all_labelings(H * W, L)
    E = energies(X, unary.reshape(H * W, L), [(a, b, 1.0, table[(a, b)]) for a, b in edges])
    for k in range(0, X.shape[0], max(1, X.shape[0] // 40)):
        got = ho.energy(unary, None, np.array(dirs), X[k].reshape(1, H, W), pairwise_edge=Te)
        np.testing.assert_allclose(got[0], E[k], rtol=1e-13, atol=1e-13)
    # tables that repeat weight times V give the energy of the weighted form
    V = rng.random((L, L))
    w = rng.uniform(0.5, 1.5, (len(dirs), 1, H, W))
    lab = X[X.shape[0] // 3].reshape(1, H, W)
    np.testing.assert_allclose(ho.energy(unary, None, np.array(dirs), lab, pairwise_edge=w[..., None, None] * V),
                               ho.energy(unary, V, np.array(dirs), lab, edge_weight=w), rtol=1e-13)


def test_energy_scalar_weight_and_batch_independence():
    rng = np.random.default_rng(3)
    unary = rng.random((2, 3, 3, 4))
    V = rng.random((4, 4))
    lab = rng.integers(0, 4, (2, 3, 3))
    both = ho.energy(unary, V, np.array(DIRS4), lab, edge_weight_scalar=0.7)
    one = ho.energy(unary[1:], V, np.array(DIRS4), lab[1:], edge_weight_scalar=0.7)
    np.testing.assert_allclose(both[1], one[0], rtol=0, atol=0)
    w = np.full((4, 2, 3, 3), 0.7)
    np.testing.assert_allclose(ho.energy(unary, V, np.array(DIRS4), lab, edge_weight=w), both, rtol=1e-15)


def test_energy_of_map_labelling_is_the_minimum_on_a_chain():
    rng = np.random.default_rng(11)
    H, W, L = 1, 5, 3
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L)); V = (V + V.T) / 2
    dirs = [(0, 1), (0, -1)]
    w = np.ones((2, 1, H, W))
    X = all_labelings(W, L)
    E = energies(X, unary.reshape(W, L), explicit_edges(H, W, dirs, w, V))
    best = X[np.argmin(E)].reshape(1, H, W)
    assert ho.energy(unary, V, np.array(dirs), best, edge_weight=w)[0] == pytest.approx(E.min(), abs=1e-13)


def test_softmin_two_labels_is_the_logistic_function():
    c = np.array([[0.3, 1.1], [2.0, -1.0]])
    d, _, _ = ho.softmin_l1(c, np.zeros(2))
    np.testing.assert_allclose(d, 1.0 / (1.0 + np.exp(c[:, 1] - c[:, 0])), rtol=1e-14)


def test_softmin_uniform_costs_and_shift_invariance():
    L = 9
    d, loss, g = ho.softmin_l1(np.full((4, L), 3.25), np.full(4, 1.0))
    np.testing.assert_allclose(d, (L - 1) / 2.0, rtol=1e-14)
    assert loss == pytest.approx((L - 1) / 2.0 - 1.0)
    rng = np.random.default_rng(5)
    c = rng.normal(0, 2, (6, L))
    d0, l0, g0 = ho.softmin_l1(c, rng.uniform(0, L - 1, 6))
    d1, _, g1 = ho.softmin_l1(c + rng.normal(0, 5, (6, 1)), rng.uniform(0, L - 1, 6))
    np.testing.assert_allclose(d0, d1, rtol=1e-12)
    np.testing.assert_allclose(g0.sum(-1), 0.0, atol=1e-15)      # a common shift of the costs changes nothing


def test_softmin_sharp_costs_pick_the_argmin():
    c = np.full((1, 7), 50.0); c[0, 4] = 0.0
    d, _, _ = ho.softmin_l1(c, np.zeros(1))
    assert d[0] == pytest.approx(4.0, abs=1e-15)


@pytest.mark.parametrize("masked", [False, True])
def test_softmin_l1_gradient_by_finite_differences(masked):
    rng = np.random.default_rng(21)
    n, L = 7, 6
    c = rng.normal(0, 1.5, (n, L))
    g = rng.uniform(0, L - 1, n)
    mask = (rng.random(n) > 0.3).astype(np.uint8) if masked else None
    _, _, grad = ho.softmin_l1(c, g, mask)
    h = 1e-6
    fd = np.zeros_like(c)
    for i in range(n):
        for l in range(L):
            cp, cm = c.copy(), c.copy()
            cp[i, l] += h; cm[i, l] -= h
            fd[i, l] = (ho.softmin_l1(cp, g, mask)[1] - ho.softmin_l1(cm, g, mask)[1]) / (2 * h)
    np.testing.assert_allclose(grad, fd, rtol=1e-6, atol=1e-9)
    if masked:
        assert np.all(grad[mask == 0] == 0.0)


@pytest.mark.parametrize("beta", [1.0, 0.25])
def test_smooth_l1_closed_forms_and_gradient(beta):
    """Smooth L1 against its two closed-form branches, its limits, and finite differences."""
    rng = np.random.default_rng(41)
    n, L = 9, 5
    c = rng.normal(0, 1.5, (n, L))
    d, _, _ = ho.softmin_l1(c, np.zeros(n))
    # targets placed so that some pixels fall on either side of |d - g| = beta
    g = d + np.array([0.0, 0.1, -0.2, 0.9, -0.99, 1.01, -3.0, 0.5, 2.0]) * beta
    _, l1, _ = ho.softmin_l1(c, g)
    _, ls, grad = ho.softmin_l1(c, g, beta=beta)
    x = np.abs(d - g)
    want = np.where(x < beta, x * x / (2 * beta), x - beta / 2).mean()
    assert ls == pytest.approx(want, rel=1e-13)
    assert ls <= l1 + 1e-15                                  # smooth L1 never exceeds L1
    far = ho.softmin_l1(c, d + 5.0 * beta, beta=beta)[1]
    assert far == pytest.approx(5.0 * beta - beta / 2, rel=1e-12)
    h = 1e-6
    fd = np.zeros_like(c)
    for i in range(n):
        for l in range(L):
            cp, cm = c.copy(), c.copy()
            cp[i, l] += h; cm[i, l] -= h
            fd[i, l] = (ho.softmin_l1(cp, g, beta=beta)[1] - ho.softmin_l1(cm, g, beta=beta)[1]) / (2 * h)
    np.testing.assert_allclose(grad, fd, rtol=2e-5, atol=1e-9)
    # beta -> 0 recovers the plain L1 loss and its gradient away from d = g
    _, l0, g0 = ho.softmin_l1(c, g, beta=1e-12)
    _, _, g1 = ho.softmin_l1(c, g)
    assert l0 == pytest.approx(l1, abs=1e-11)
    np.testing.assert_allclose(g0[1:], g1[1:], atol=1e-12)
