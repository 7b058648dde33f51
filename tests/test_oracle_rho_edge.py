"""Pins of the oracle's per-edge TRW coefficients rho_{i-r,i} (Eq. trwp writes rho per edge; the
experiments of the paper use one constant): reduction to the per-direction path, a brute-force
discounted minimisation on a chain in which every edge has its own rho, and central finite
differences of the double forward for the backward pass."""
import itertools

import numpy as np
import pytest

from mrf_inputs import DIRS4, DIRS8

F64 = np.float64
EPS = 1e-6


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_constant_array_equals_per_direction_rho(oracle, dtype):
    rng = np.random.default_rng(5)
    B, H, W, L, K = 2, 4, 5, 4, 2
    unary = rng.random((B, H, W, L)).astype(dtype)
    V = rng.random((L, L)).astype(dtype)
    w = rng.uniform(0.5, 1.5, (8, B, H, W)).astype(dtype)
    gc = rng.normal(0, 1, (B, H, W, L)).astype(dtype)
    rho = rng.uniform(0.2, 0.9, 8).astype(dtype)
    rho_e = np.broadcast_to(rho[:, None, None, None], (8, B, H, W)).copy()
    a = oracle.forward("trwp", unary, V, DIRS8, K, edge_weight=w, rho=rho, dtype=dtype)
    b = oracle.forward("trwp", unary, V, DIRS8, K, edge_weight=w, rho=[0.0] * 8, rho_edge=rho_e, dtype=dtype)
    for name in ("cost", "labels", "p", "q", "messages"):
        np.testing.assert_array_equal(getattr(a, name), getattr(b, name), err_msg=name)
    ga = oracle.backward("trwp", unary.shape, V, DIRS8, K, gc, a.p, a.q, edge_weight=w, rho=rho, dtype=dtype)
    gb = oracle.backward("trwp", unary.shape, V, DIRS8, K, gc, a.p, a.q, edge_weight=w, rho=[0.0] * 8,
                         rho_edge=rho_e, dtype=dtype)
    for name in ("grad_unary", "grad_edge_weight", "grad_pairwise"):
        np.testing.assert_array_equal(getattr(ga, name), getattr(gb, name), err_msg=name)


def test_chain_discounted_bruteforce_with_one_rho_per_edge(oracle):
    """1 x W chain, K = 1, directions (->, <-).  Unrolling Eq. trwp, the terms of node t reach
    node i multiplied by the rho of every edge crossed on the way, each edge having its own:
    that minimisation is enumerated.  Pins that the rho of edge (i-r, i) is the entry stored at
    node i and that it multiplies the unary and all messages at i-r, but not m^{r-}."""
    W, L = 4, 3
    rng = np.random.default_rng(78)
    unary = rng.random((1, 1, W, L))
    V = rng.random((L, L))
    dirs = [(0, 1), (0, -1)]
    w = rng.uniform(0.5, 1.5, (2, 1, 1, W))
    rho_e = rng.uniform(0.2, 0.9, (2, 1, 1, W))
    f = oracle.forward("trwp", unary, V, dirs, 1, edge_weight=w, rho=[9.0, 9.0], rho_edge=rho_e, dtype=F64)
    th = unary[0, 0]
    rf = rho_e[0, 0, 0]        # rf[s] = rho of edge (s-1 -> s)
    rb = rho_e[1, 0, 0]        # rb[s] = rho of edge (s+1 -> s)

    def prod(a, lo, hi):       # product of a[lo..hi], 1 when empty
        return float(np.prod(a[lo:hi + 1])) if hi >= lo else 1.0

    # forward sweep: node t's unary crosses edges t+1..i, the pairwise term of edge t+1 crosses t+2..i
    mf = np.zeros((W, L))
    for i in range(1, W):
        for lam in range(L):
            best = np.inf
            for xs in itertools.product(range(L), repeat=i):
                seq = list(xs) + [lam]
                e = sum(prod(rf, t + 1, i) * th[t][seq[t]] for t in range(i))
                e += sum(prod(rf, t + 2, i) * w[0, 0, 0, t + 1] * V[seq[t]][seq[t + 1]] for t in range(i))
                best = min(best, e)
            mf[i, lam] = best
        mf[i] -= mf[i].min()
    np.testing.assert_allclose(f.messages[0, 0, 0], mf, atol=1e-12)

    # backward sweep (<-): the potential of node t as seen over edge (t -> t-1) is
    # rb[t-1] th_t + (rb[t-1] - 1) mf_t; further edges towards i multiply it by their own rho
    mb = np.zeros((W, L))
    for i in range(W - 2, -1, -1):
        n = W - 1 - i
        for lam in range(L):
            best = np.inf
            for xs in itertools.product(range(L), repeat=n):
                seq = [lam] + list(xs)          # labels of nodes i, i+1, ..., W-1
                e = 0.0
                for t in range(1, n + 1):       # node i+t, first edge it crosses arrives at i+t-1
                    node = i + t
                    phi = rb[node - 1] * th[node][seq[t]] + (rb[node - 1] - 1.0) * mf[node][seq[t]]
                    e += prod(rb, i, node - 2) * phi
                for t in range(n):              # edge (i+t+1 -> i+t), weight stored at i+t
                    e += prod(rb, i, i + t - 1) * w[1, 0, 0, i + t] * V[seq[t + 1]][seq[t]]
                best = min(best, e)
            mb[i, lam] = best
        mb[i] -= mb[i].min()
    np.testing.assert_allclose(f.messages[1, 0, 0], mb, atol=1e-12)
    np.testing.assert_allclose(f.cost[0, 0], th + mf + mb, atol=1e-12)


@pytest.mark.parametrize("dirs,K,dims", [(DIRS4, 3, (3, 4, 3)), (DIRS8, 2, (3, 3, 3)),
                                         ([(0, 1), (1, 0), (-1, 0)], 3, (3, 3, 3))])
def test_backward_matches_finite_differences_with_per_edge_rho(oracle, dirs, K, dims):
    H, W, L = dims
    rng = np.random.default_rng(300 + K + len(dirs))
    R = len(dirs)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L))
    w = rng.uniform(0.5, 1.5, (R, 1, H, W))
    rho_e = rng.uniform(0.2, 0.9, (R, 1, H, W))
    gc = rng.normal(0.0, 1.0, (1, H, W, L))

    def loss():
        f = oracle.forward("trwp", unary, V, dirs, K, edge_weight=w, rho_edge=rho_e, dtype=F64)
        return float((f.cost * gc).sum())

    f = oracle.forward("trwp", unary, V, dirs, K, edge_weight=w, rho_edge=rho_e, dtype=F64)
    b = oracle.backward("trwp", unary.shape, V, dirs, K, gc, f.p, f.q, edge_weight=w, rho_edge=rho_e, dtype=F64)

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
    for idx in np.ndindex(V.shape):
        assert abs(fd(V, idx) - b.grad_pairwise[idx]) < 1e-6, ("V", idx)
    for idx in np.ndindex(w.shape):
        assert abs(fd(w, idx) - b.grad_edge_weight[idx]) < 1e-6, ("w", idx)
