"""Pins of the CPU oracle's backward passes (Alg. 3, Alg. 4) by central finite differences
of its own double-precision forward passes -- which are themselves pinned by brute force in
test_oracle_bruteforce.py -- and by invariants that follow from Eq. supp-isgmr-back-norm.

The map parameters -> costs is piecewise linear (min-sum), so central differences are
exact up to rounding whenever no argmin flips inside the step; inputs are continuous
random numbers, for which a flip inside +-1e-6 has negligible probability.
"""
import numpy as np
import pytest

from mrf_inputs import DIRS4, DIRS8, DIRS16, mirrored_edge_weights

F64 = np.float64
EPS = 1e-6


def make(seed, H, W, L, dirs, B=1):
    rng = np.random.default_rng(seed)
    unary = rng.random((B, H, W, L))
    V = rng.random((L, L))                      # asymmetric on purpose
    w = rng.uniform(0.5, 1.5, (len(dirs), B, H, W))   # directed copies independent on purpose
    gc = rng.normal(0.0, 1.0, (B, H, W, L))
    rho = rng.uniform(0.2, 0.9, len(dirs))
    return unary, V, w, gc, rho


def loss(oracle, algo, unary, V, w, dirs, K, rho, gc):
    f = oracle.forward(algo, unary, V, dirs, K, edge_weight=w, rho=rho, dtype=F64)
    return float((f.cost * gc).sum())


def fd(fun, arr, idx):
    old = arr[idx]
    arr[idx] = old + EPS
    up = fun()
    arr[idx] = old - EPS
    dn = fun()
    arr[idx] = old
    return (up - dn) / (2 * EPS)


CASES = [
    ("isgmr", DIRS4, 3, (3, 4, 3)),
    ("isgmr", DIRS8, 2, (3, 3, 3)),
    ("isgmr", [(0, 1), (1, 0)], 3, (3, 3, 3)),          # no opposite directions in the set
    ("isgmr", DIRS16, 2, (4, 4, 2)),
    ("trwp", DIRS4, 3, (3, 4, 3)),
    ("trwp", DIRS8, 2, (3, 3, 3)),
    ("trwp", [(0, 1), (1, 0), (-1, 0)], 3, (3, 3, 3)),  # r- present for some directions only
    ("trwp", DIRS16, 2, (4, 4, 2)),
]


@pytest.mark.parametrize("algo,dirs,K,dims", CASES)
def test_backward_matches_finite_differences(oracle, algo, dirs, K, dims):
    H, W, L = dims
    unary, V, w, gc, rho = make(101 + K + len(dirs), H, W, L, dirs)
    f = oracle.forward(algo, unary, V, dirs, K, edge_weight=w, rho=rho, dtype=F64)
    b = oracle.backward(algo, unary.shape, V, dirs, K, gc, f.p, f.q, edge_weight=w, rho=rho, dtype=F64)
    fun = lambda: loss(oracle, algo, unary, V, w, dirs, K, rho, gc)

    num = np.zeros_like(unary)
    for idx in np.ndindex(*unary.shape):
        num[idx] = fd(fun, unary, idx)
    np.testing.assert_allclose(b.grad_unary, num, rtol=1e-6, atol=1e-6)

    numV = np.zeros_like(V)
    for idx in np.ndindex(*V.shape):
        numV[idx] = fd(fun, V, idx)
    np.testing.assert_allclose(b.grad_pairwise, numV, rtol=1e-6, atol=1e-6)

    numw = np.zeros_like(w)
    for idx in np.ndindex(*w.shape):
        numw[idx] = fd(fun, w, idx)
    np.testing.assert_allclose(b.grad_edge_weight, numw, rtol=1e-6, atol=1e-6)
    # weights of first nodes are never read
    for r, (dh, dw) in enumerate(dirs):
        for y in range(H):
            for x in range(W):
                if not (0 <= y - dh < H and 0 <= x - dw < W):
                    assert b.grad_edge_weight[r, 0, y, x] == 0.0


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_batch_entries_are_independent(oracle, algo):
    H, W, L, K = 3, 3, 3, 2
    unary, V, w, gc, rho = make(9, H, W, L, DIRS4, B=2)
    f = oracle.forward(algo, unary, V, DIRS4, K, edge_weight=w, rho=rho, dtype=F64)
    b = oracle.backward(algo, unary.shape, V, DIRS4, K, gc, f.p, f.q, edge_weight=w, rho=rho, dtype=F64)
    gV = np.zeros_like(V)
    for n in range(2):
        f1 = oracle.forward(algo, unary[n:n + 1], V, DIRS4, K, edge_weight=w[:, n:n + 1], rho=rho, dtype=F64)
        b1 = oracle.backward(algo, (1, H, W, L), V, DIRS4, K, gc[n:n + 1], f1.p, f1.q,
                             edge_weight=w[:, n:n + 1], rho=rho, dtype=F64)
        np.testing.assert_array_equal(f1.cost[0], f.cost[n])
        np.testing.assert_allclose(b1.grad_unary[0], b.grad_unary[n], atol=1e-13)
        gV += b1.grad_pairwise
    np.testing.assert_allclose(gV, b.grad_pairwise, atol=1e-12)


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_scalar_weight_equals_constant_array(oracle, algo):
    H, W, L, K = 3, 4, 3, 2
    unary, V, w, gc, rho = make(4, H, W, L, DIRS4)
    w[:] = 0.7
    fa = oracle.forward(algo, unary, V, DIRS4, K, edge_weight=w, rho=rho, dtype=F64)
    fb = oracle.forward(algo, unary, V, DIRS4, K, edge_weight=None, edge_weight_scalar=0.7, rho=rho, dtype=F64)
    np.testing.assert_array_equal(fa.cost, fb.cost)
    np.testing.assert_array_equal(fa.p, fb.p)
    ba = oracle.backward(algo, unary.shape, V, DIRS4, K, gc, fa.p, fa.q, edge_weight=w, rho=rho, dtype=F64)
    bb = oracle.backward(algo, unary.shape, V, DIRS4, K, gc, fa.p, fa.q, edge_weight=None,
                         edge_weight_scalar=0.7, rho=rho, dtype=F64)
    np.testing.assert_array_equal(ba.grad_unary, bb.grad_unary)
    np.testing.assert_array_equal(ba.grad_pairwise, bb.grad_pairwise)


def test_isgmr_unary_gradient_mass_is_conserved(oracle):
    """Every reparametrised message gradient sums to 0 over labels (Eq. supp-isgmr-back-norm),
    and each label's gradient is moved, not scaled, to one label of the previous node; so
    per node sum_lambda grad theta_i = sum_lambda grad c_i in ISGMR."""
    H, W, L, K = 4, 5, 4, 3
    unary, V, w, gc, rho = make(12, H, W, L, DIRS8)
    f = oracle.forward("isgmr", unary, V, DIRS8, K, edge_weight=w, dtype=F64)
    b = oracle.backward("isgmr", unary.shape, V, DIRS8, K, gc, f.p, f.q, edge_weight=w, dtype=F64)
    np.testing.assert_allclose(b.grad_unary.sum(-1), gc.sum(-1), atol=1e-9)


def test_f32_backward_close_to_f64(oracle):
    """The float instantiation follows the same steps; on the same indices it differs from
    the double one by rounding only."""
    H, W, L, K = 6, 7, 5, 3
    unary, V, w, gc, rho = make(31, H, W, L, DIRS4)
    for algo in ("isgmr", "trwp"):
        f = oracle.forward(algo, unary, V, DIRS4, K, edge_weight=w, rho=rho, dtype=np.float32)
        b32 = oracle.backward(algo, unary.shape, V, DIRS4, K, gc, f.p, f.q, edge_weight=w, rho=rho,
                              dtype=np.float32)
        b64 = oracle.backward(algo, unary.shape, V, DIRS4, K, gc, f.p, f.q, edge_weight=w, rho=rho, dtype=F64)
        scale = np.abs(b64.grad_unary).max()
        np.testing.assert_allclose(b32.grad_unary, b64.grad_unary, atol=2e-5 * scale)
        np.testing.assert_allclose(b32.grad_pairwise, b64.grad_pairwise,
                                   atol=2e-5 * np.abs(b64.grad_pairwise).max())
