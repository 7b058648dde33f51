"""Invariants of the CPU oracle in the precision of record (float32), no GPU:
normalised messages (Eq. isgmr-norm), first nodes, index ranges, aggregation
(Eq. isgmr-aggregation), labelling (Eq. disp), tie-breaking, scanline counts
(Eq. supp-wide), and bit-identity of the threaded build."""
import numpy as np
import pytest

from mrf_inputs import DIRS4, DIRS8, DIRS16, make_config, random_problem


def has_pred(H, W, dh, dw):
    yy, xx = np.meshgrid(np.arange(H), np.arange(W), indexing="ij")
    return (yy - dh >= 0) & (yy - dh < H) & (xx - dw >= 0) & (xx - dw < W)


def run_forward(oracle, pr, **kw):
    return oracle.forward(pr.algo, pr.unary, pr.pairwise, pr.dirs, pr.K, edge_weight=pr.edge_weight,
                          edge_weight_scalar=pr.edge_weight_scalar, rho=pr.rho, **kw)


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
@pytest.mark.parametrize("dirs", [DIRS4, DIRS8, DIRS16])
def test_message_invariants(oracle, algo, dirs):
    B, H, W, L, K = 2, 6, 7, 5, 3
    pr = random_problem(1, algo, B, H, W, L, dirs, K)
    f = run_forward(oracle, pr)
    assert f.p.max() < L and f.q.max() < L
    for r, (dh, dw) in enumerate(dirs):
        hp = has_pred(H, W, dh, dw)
        m = f.messages[r]
        # first nodes: message 0 for ever, p = q = 0
        assert (m[:, ~hp] == 0).all()
        assert (f.p[:, r][:, :, ~hp] == 0).all() and (f.q[:, r][:, :, ~hp] == 0).all()
        # every other message has minimum exactly +0 and it sits at index q of the last iteration
        mm = m[:, hp]
        assert (mm.min(-1) == 0).all()
        qlast = f.q[K - 1, r][:, hp]
        assert (np.take_along_axis(mm, qlast[..., None].astype(np.int64), -1) == 0).all()
        assert (mm.argmin(-1) == qlast).all()          # numpy argmin = lowest index
    # aggregation in direction-index order, float32 adds
    c = pr.unary.copy()
    for r in range(len(dirs)):
        c = c + f.messages[r]
    np.testing.assert_array_equal(c, f.cost)
    np.testing.assert_array_equal(f.cost.argmin(-1), f.labels)


def test_ties_go_to_lowest_label(oracle):
    L = 6
    dirs = DIRS4
    unary = np.zeros((1, 4, 5, L), np.float32)
    zeroV = np.zeros((L, L), np.float32)
    potts = (1 - np.eye(L)).astype(np.float32)
    for algo in ("isgmr", "trwp"):
        f = oracle.forward(algo, unary, zeroV, dirs, 2, edge_weight_scalar=1.0, rho=[0.5] * 4)
        assert (f.p == 0).all() and (f.q == 0).all() and (f.labels == 0).all()
        # Potts, flat unaries: delta(lambda, mu) = [mu != lambda], so p(lambda) = lambda, q = 0
        f = oracle.forward(algo, unary, potts, dirs, 1, edge_weight_scalar=1.0, rho=[0.5] * 4)
        hp = has_pred(4, 5, 0, 1)
        assert (f.p[0, 0, 0][hp] == np.arange(L)).all()
        assert (f.q == 0).all()


def test_integer_valued_ties_lowest_index(oracle):
    """Integer data makes ties frequent; the stored p must be the lowest minimiser, which a
    direct evaluation of Eq. sgm for the first direction of the first iteration shows."""
    pr = random_problem(6, "isgmr", 1, 3, 6, 4, [(0, 1)], 1, integer_valued=True)
    f = run_forward(oracle, pr)
    L = 4
    for y in range(3):
        m_prev = np.zeros(L, np.float32)
        for x in range(1, 6):
            h = pr.unary[0, y, x - 1] + m_prev
            delta = h[:, None] + pr.edge_weight[0, 0, y, x] * pr.pairwise   # [mu, lambda], exact in float
            np.testing.assert_array_equal(f.p[0, 0, 0, y, x], delta.argmin(0))
            t = delta.min(0)
            assert f.q[0, 0, 0, y, x] == t.argmin()
            m_prev = t - t.min()


@pytest.mark.parametrize("H,W", [(5, 9), (9, 5), (1, 7), (7, 1)])
def test_scanline_counts(oracle, H, W):
    assert oracle.count_scanlines(H, W, 0, 1) == H
    assert oracle.count_scanlines(H, W, 1, 0) == W
    for sw in (1, -1, 2, -2):
        for sh in (1, -1):
            # Eq. supp-wide: N = W + (H - 1) |S_w| trees for symmetric / asymmetric wide steps
            if abs(sw) <= W:
                assert oracle.count_scanlines(H, W, sh, sw) == W + (H - 1) * abs(sw)


def test_unary_shift_moves_only_that_cost(oracle):
    """Messages are normalised and depend on the previous node's values only through
    differences... a constant added to one node's unary vector shifts that node's cost and
    nothing else (Eq. isgmr-norm)."""
    for algo in ("isgmr", "trwp"):
        pr = random_problem(2, algo, 1, 4, 5, 4, DIRS4, 3)
        f0 = run_forward(oracle, pr, dtype=np.float64)
        pr.unary = pr.unary.astype(np.float64)
        pr.unary[0, 2, 3] += 0.625
        f1 = run_forward(oracle, pr, dtype=np.float64)
        d = f1.cost - f0.cost
        assert abs(d[0, 2, 3] - 0.625).max() < 1e-12
        d[0, 2, 3] = 0
        assert np.abs(d).max() < 1e-12
        np.testing.assert_array_equal(f0.p, f1.p)


def test_threaded_build_is_bit_identical(oracle):
    assert oracle.openmp_enabled(True) and not oracle.openmp_enabled(False)
    for idx, crop in ((1, None), (2, (24, 40)), (5, (16, 24))):
        for algo in ("isgmr", "trwp"):
            pr = make_config(idx, crop=crop, algo=algo, K=2)
            a = run_forward(oracle, pr, threads=False)
            b = run_forward(oracle, pr, threads=True)
            for name in ("cost", "labels", "p", "q", "messages"):
                np.testing.assert_array_equal(getattr(a, name), getattr(b, name))


def test_rejects_bad_problems(oracle):
    u = np.zeros((1, 2, 2, 2), np.float32)
    V = np.zeros((2, 2), np.float32)
    with pytest.raises(ValueError):
        oracle.forward("isgmr", u, V, [(0, 0)], 1)
    with pytest.raises(ValueError):
        oracle.forward("isgmr", u, V, [(0, 1), (0, 1)], 1)
    with pytest.raises(ValueError):
        oracle.forward("isgmr", u, V, [(0, 1)], 0)
