"""Pins of the oracle's standard single-pass SGM (Sec. 3.2, Eq. sgm_old, Eq. isgmr-aggregation-old)
against things it does not compute itself: enumeration along scanlines with the node's own unary
inside the minimum, and the relations to the revised update that Sec. 3.2 states."""
import itertools

import numpy as np
import pytest

from mrf_inputs import DIRS4, DIRS8, sgm_penalties

F64 = np.float64


def scanlines(H, W, dh, dw):
    out = []
    for y0 in range(H):
        for x0 in range(W):
            if 0 <= y0 - dh < H and 0 <= x0 - dw < W:
                continue
            line, y, x = [], y0, x0
            while 0 <= y < H and 0 <= x < W:
                line.append((y, x)); y += dh; x += dw
            out.append(line)
    return out


def aggregated_cost_along(unary_line, w_line, V):
    """Eq. sgm_old unrolled: for node n and label lam, the minimum over the labels of nodes 0..n-1 of
    all unaries up to and INCLUDING node n's own plus the pairwise terms up to node n."""
    n_nodes, L = unary_line.shape
    out = np.zeros((n_nodes, L))
    out[0] = unary_line[0]
    for n in range(1, n_nodes):
        for lam in range(L):
            best = np.inf
            for xs in itertools.product(range(L), repeat=n):
                seq = list(xs) + [lam]
                e = sum(unary_line[t][seq[t]] for t in range(n + 1))
                e += sum(w_line[t + 1] * V[seq[t]][seq[t + 1]] for t in range(n))
                best = min(best, e)
            out[n, lam] = best
    return out


@pytest.mark.parametrize("dirs", [DIRS4, DIRS8])
def test_standard_sgm_is_scanline_enumeration_with_own_unary(oracle, dirs):
    H, W, L = 3, 4, 2
    rng = np.random.default_rng(31)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L))                      # asymmetric: pins V[mu at i-r][lambda at i]
    w = rng.uniform(0.5, 1.5, (len(dirs), 1, H, W))
    f = oracle.sgm_standard_forward(unary, V, dirs, edge_weight=w, dtype=F64)
    total = np.zeros((H, W, L))
    for r, (dh, dw) in enumerate(dirs):
        for line in scanlines(H, W, dh, dw):
            ul = np.array([unary[0, y, x] for y, x in line])
            wl = np.array([w[r, 0, y, x] for y, x in line])
            ref = aggregated_cost_along(ul, wl, V)
            for n, (y, x) in enumerate(line):
                got = f.messages[r, 0, y, x]
                if n == 0:
                    np.testing.assert_allclose(got, ref[0], atol=1e-12)            # the unary itself
                else:
                    np.testing.assert_allclose(got, ref[n] - ref[n].min(), atol=1e-12)
                    assert got.min() == 0.0 and f.q[0, r, 0, y, x] == int(np.argmin(ref[n]))
                total[y, x] += got
    np.testing.assert_allclose(f.cost[0], total, atol=1e-12)                     # Eq. isgmr-aggregation-old
    assert (f.labels[0] == total.argmin(-1)).all()


def test_standard_and_revised_sgm_differ_by_the_overcounted_unaries(oracle):
    """Sec. 3.2: the standard messages are the revised ones plus the node's unary (up to the constant
    the reparametrisation removes), so the standard cost counts every unary |R| - 1 times more."""
    H, W, L = 5, 6, 4
    rng = np.random.default_rng(32)
    unary = rng.random((1, H, W, L))
    V = sgm_penalties(L, 0.3, 1.1).astype(F64)
    w = rng.uniform(0.5, 1.5, (8, 1, H, W))
    std = oracle.sgm_standard_forward(unary, V, DIRS8, edge_weight=w, dtype=F64)
    rev = oracle.forward("isgmr", unary, V, DIRS8, 1, edge_weight=w, dtype=F64)
    np.testing.assert_array_equal(std.p, rev.p)         # same minimisers over mu (real arithmetic, no ties here)
    rel = lambda a: a - a.min(-1, keepdims=True)
    for r in range(8):
        np.testing.assert_allclose(rel(std.messages[r]), rel(rev.messages[r] + unary), atol=1e-12)
    np.testing.assert_allclose(rel(std.cost), rel(rev.cost + 7.0 * unary), atol=1e-11)


def test_standard_sgm_float_and_double_agree(oracle):
    rng = np.random.default_rng(33)
    unary = rng.random((2, 4, 5, 6)).astype(np.float32)
    V = sgm_penalties(6, 0.5, 2.0)
    a = oracle.sgm_standard_forward(unary, V, DIRS4, edge_weight_scalar=0.7, dtype=np.float32)
    b = oracle.sgm_standard_forward(unary, V, DIRS4, edge_weight_scalar=0.7, dtype=F64)
    np.testing.assert_allclose(a.cost, b.cost, rtol=1e-5, atol=1e-5)
    assert a.p.shape == (1, 4, 2, 4, 5, 6) and a.q.shape == (1, 4, 2, 4, 5)
