"""Pins of the oracle's per-edge pairwise potentials theta_{i-r,i}(mu,lambda) (the form in
which Eq. isgmr / Eq. trwp are written, before the decomposition into edge weight times V) and
of their gradient (Eq. supp-gradient-pairwise): exhaustive min-marginals on chains whose edges
all have different random tables, reduction to the decomposed form with the chain-rule
identities that tie the three pairwise gradients together, and central finite differences."""
import numpy as np
import pytest

from bruteforce import min_marginals
from mrf_inputs import DIRS4, DIRS8

F64 = np.float64
EPS = 1e-6


def rel(c):
    return c - c.min(axis=-1, keepdims=True)


@pytest.mark.parametrize("algo,K", [("isgmr", 1), ("isgmr", 3), ("trwp", 1), ("trwp", 2)])
@pytest.mark.parametrize("vertical", [False, True])
def test_chain_min_marginals_with_one_table_per_edge(oracle, algo, K, vertical):
    n, L = 5, 3
    rng = np.random.default_rng(31)
    th = rng.random((n, L))
    E = rng.random((n - 1, L, L))            # E[t][x_t][x_{t+1}], not symmetric
    H, W = (n, 1) if vertical else (1, n)
    dirs = [(1, 0), (-1, 0)] if vertical else [(0, 1), (0, -1)]
    Te = np.zeros((2, 1, H, W, L, L))
    Tv = Te.reshape(2, n, L, L)
    for t in range(n - 1):
        Tv[0, t + 1] = E[t]                  # edge arriving at t+1 from t: [mu at t][lambda at t+1]
        Tv[1, t] = E[t].T                    # edge arriving at t from t+1: [mu at t+1][lambda at t]
    f = oracle.forward(algo, th.reshape(1, H, W, L), None, dirs, K, rho=[1.0, 1.0], dtype=F64, pairwise_edge=Te)
    edges = [(t, t + 1, 1.0, E[t]) for t in range(n - 1)]
    mm, xmap, _ = min_marginals(th, edges, L)
    np.testing.assert_allclose(rel(f.cost.reshape(-1, L)), rel(mm), atol=1e-12)
    assert (f.labels.reshape(-1) == xmap).all()


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_tables_built_from_weight_times_v_give_the_decomposed_results(oracle, algo):
    """theta_e = w V reproduces the decomposed problem, and the three pairwise gradients are tied
    by the chain rule: grad w = sum_{mu,lambda} grad theta_e V, grad V = sum_{r,i} w grad theta_e."""
    rng = np.random.default_rng(32)
    B, H, W, L, K = 2, 3, 4, 3, 2
    R = len(DIRS8)
    unary = rng.random((B, H, W, L))
    V = rng.random((L, L))
    w = rng.uniform(0.5, 1.5, (R, B, H, W))
    rho = rng.uniform(0.3, 0.9, R)
    gc = rng.normal(0, 1, (B, H, W, L))
    Te = w[..., None, None] * V
    a = oracle.forward(algo, unary, V, DIRS8, K, edge_weight=w, rho=rho, dtype=F64)
    b = oracle.forward(algo, unary, None, DIRS8, K, rho=rho, dtype=F64, pairwise_edge=Te)
    np.testing.assert_array_equal(a.p, b.p)
    np.testing.assert_array_equal(a.q, b.q)
    np.testing.assert_allclose(a.cost, b.cost, atol=1e-12)
    ga = oracle.backward(algo, unary.shape, V, DIRS8, K, gc, a.p, a.q, edge_weight=w, rho=rho, dtype=F64)
    gb = oracle.backward(algo, unary.shape, None, DIRS8, K, gc, a.p, a.q, rho=rho, dtype=F64, per_edge_pairwise=True)
    np.testing.assert_allclose(gb.grad_unary, ga.grad_unary, atol=1e-12)
    np.testing.assert_allclose((gb.grad_pairwise_edge * V).sum(axis=(-1, -2)), ga.grad_edge_weight, atol=1e-10)
    np.testing.assert_allclose((gb.grad_pairwise_edge * w[..., None, None]).sum(axis=(0, 1, 2, 3)), ga.grad_pairwise, atol=1e-10)


@pytest.mark.parametrize("algo,dirs,K", [("isgmr", DIRS4, 2), ("trwp", DIRS4, 2), ("trwp", [(0, 1), (1, 0), (-1, 0)], 3),
                                         ("isgmr", DIRS8, 2)])
def test_gradient_of_per_edge_tables_by_finite_differences(oracle, algo, dirs, K):
    rng = np.random.default_rng(40 + K + len(dirs))
    H, W, L = 3, 3, 2
    R = len(dirs)
    unary = rng.random((1, H, W, L))
    Te = rng.random((R, 1, H, W, L, L))
    rho = rng.uniform(0.3, 0.9, R)
    gc = rng.normal(0, 1, (1, H, W, L))

    def loss():
        f = oracle.forward(algo, unary, None, dirs, K, rho=rho, dtype=F64, pairwise_edge=Te)
        return float((f.cost * gc).sum())

    f = oracle.forward(algo, unary, None, dirs, K, rho=rho, dtype=F64, pairwise_edge=Te)
    b = oracle.backward(algo, unary.shape, None, dirs, K, gc, f.p, f.q, rho=rho, dtype=F64, per_edge_pairwise=True)

    def fd(arr, idx):
        old = arr[idx]
        arr[idx] = old + EPS
        up = loss()
        arr[idx] = old - EPS
        dn = loss()
        arr[idx] = old
        return (up - dn) / (2 * EPS)

    for idx in np.ndindex(unary.shape):
        assert abs(fd(unary, idx) - b.grad_unary[idx]) < 1e-6, ("unary", idx)
    for idx in np.ndindex(Te.shape):
        r, _, y, x = idx[:4]
        inside = 0 <= y - dirs[r][0] < H and 0 <= x - dirs[r][1] < W
        want = fd(Te, idx) if inside else 0.0          # tables of first nodes are never read
        assert abs(want - b.grad_pairwise_edge[idx]) < 1e-6, ("theta_e", idx)
