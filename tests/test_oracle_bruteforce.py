"""Pins of the CPU oracle's forward passes against exhaustive enumeration (no GPU).

Min-sum message passing is exact on chains and trees, so the final costs of ISGMR
(Alg. 1) and of TRWP with rho = 1 (= loopy belief propagation, Sec. 3.3) must equal the
brute-force min-marginals of the energy (Eq. 1) up to one additive constant per node.
TRWP with rho != 1 on a chain is pinned by a brute-force "discounted" minimisation
derived from Eq. trwp.  All comparisons use the double instantiation of the oracle.
"""
import itertools

import numpy as np
import pytest

from bruteforce import all_labelings, energies, min_marginals
from mrf_inputs import DIRS4, DIRS8, DIRS16, mirrored_edge_weights

F64 = np.float64


def grid_edges(H, W, dirs, w, V, only=None):
    """Directed message edges (pred -> node) of each direction, as the oracle's layout
    defines them: weight stored at the destination node, V[x_pred][x_node]."""
    out = []
    for r, (dh, dw) in enumerate(dirs):
        if only is not None and r not in only:
            continue
        for y in range(H):
            for x in range(W):
                yp, xp = y - dh, x - dw
                if 0 <= yp < H and 0 <= xp < W:
                    out.append((yp * W + xp, y * W + x, float(w[r, 0, y, x]), V))
    return out


def rel(c):
    return c - c.min(axis=-1, keepdims=True)


def rand_problem(seed, H, W, L, dirs, symmetric=True):
    rng = np.random.default_rng(seed)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L))
    if symmetric:
        V = (V + V.T) / 2
    w = mirrored_edge_weights(rng, 1, H, W, dirs, lambda g, s: g.uniform(0.5, 1.5, s)).astype(F64)
    return unary, V, w


@pytest.mark.parametrize("algo,K", [("isgmr", 1), ("isgmr", 3), ("trwp", 1), ("trwp", 2)])
@pytest.mark.parametrize("shape,dirs", [((1, 5), [(0, 1), (0, -1)]), ((5, 1), [(1, 0), (-1, 0)])])
def test_chain_min_marginals(oracle, algo, K, shape, dirs):
    H, W = shape
    L = 3
    unary, V, w = rand_problem(11, H, W, L, dirs)
    f = oracle.forward(algo, unary, V, dirs, K, edge_weight=w, rho=[1.0, 1.0], dtype=F64)
    mm, xmap, _ = min_marginals(unary.reshape(-1, L), grid_edges(H, W, dirs, w, V, only=[0]), L)
    np.testing.assert_allclose(rel(f.cost.reshape(-1, L)), rel(mm), atol=1e-12)
    assert (f.labels.reshape(-1) == xmap).all()


@pytest.mark.parametrize("dirs", [[(1, 1), (-1, -1)], [(1, -1), (-1, 1)]])
@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_diagonal_chains_min_marginals(oracle, algo, dirs):
    """With only one diagonal pair of directions a 3x3 grid is a set of disjoint chains."""
    H, W, L = 3, 3, 3
    unary, V, w = rand_problem(5, H, W, L, dirs)
    f = oracle.forward(algo, unary, V, dirs, 2, edge_weight=w, rho=[1.0, 1.0], dtype=F64)
    mm, xmap, _ = min_marginals(unary.reshape(-1, L), grid_edges(H, W, dirs, w, V, only=[0]), L)
    np.testing.assert_allclose(rel(f.cost.reshape(-1, L)), rel(mm), atol=1e-12)
    assert (f.labels.reshape(-1) == xmap).all()


def comb_tree_weights(rng, H, W, dirs):
    """4-connected grid turned into a spanning tree: all vertical edges plus the horizontal
    edges of row 0; every other edge gets weight 0 (a zero-weight edge carries a constant
    message, which normalises to exactly 0, so the edge vanishes)."""
    w = mirrored_edge_weights(rng, 1, H, W, dirs, lambda g, s: g.uniform(0.5, 1.5, s)).astype(F64)
    for r, (dh, dw) in enumerate(dirs):
        if dh == 0:
            w[r, :, 1:, :] = 0.0
    return w


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_comb_tree_min_marginals(oracle, algo):
    H, W, L = 3, 3, 3
    rng = np.random.default_rng(23)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L)); V = (V + V.T) / 2
    w = comb_tree_weights(rng, H, W, DIRS4)
    f = oracle.forward(algo, unary, V, DIRS4, 8, edge_weight=w, rho=[1.0] * 4, dtype=F64)
    mm, xmap, _ = min_marginals(unary.reshape(-1, L), grid_edges(H, W, DIRS4, w, V, only=[0, 2]), L)
    np.testing.assert_allclose(rel(f.cost.reshape(-1, L)), rel(mm), atol=1e-12)
    assert (f.labels.reshape(-1) == xmap).all()


def test_wrong_exclusion_would_break_tree(oracle):
    """Sanity of the pin above: on the comb tree one ISGMR iteration is NOT yet exact
    (messages must turn a corner), so the test can tell converged from unconverged."""
    H, W, L = 3, 3, 3
    rng = np.random.default_rng(23)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L)); V = (V + V.T) / 2
    w = comb_tree_weights(rng, H, W, DIRS4)
    f = oracle.forward("isgmr", unary, V, DIRS4, 1, edge_weight=w, dtype=F64)
    mm, _, _ = min_marginals(unary.reshape(-1, L), grid_edges(H, W, DIRS4, w, V, only=[0, 2]), L)
    assert np.abs(rel(f.cost.reshape(-1, L)) - rel(mm)).max() > 1e-3


def scanline_prefix_min(unary_line, w_line, V):
    """Brute force of Eq. sgm along one scanline: for node n and label lam, the minimum over
    labels of nodes 0..n-1 of their unaries plus the pairwise terms up to node n."""
    n_nodes, L = unary_line.shape
    out = np.zeros((n_nodes, L))
    for n in range(1, n_nodes):
        for lam in range(L):
            best = np.inf
            for xs in itertools.product(range(L), repeat=n):
                seq = list(xs) + [lam]
                e = sum(unary_line[t][seq[t]] for t in range(n))
                e += sum(w_line[t + 1] * V[seq[t]][seq[t + 1]] for t in range(n))
                best = min(best, e)
            out[n, lam] = best
        out[n] -= out[n].min()
    return out


@pytest.mark.parametrize("dirs", [DIRS8, DIRS16])
def test_single_iteration_is_scanline_dp_all_directions(oracle, dirs):
    """ISGMR with K = 1 is the revised SGM (Eq. sgm): every direction's messages are an
    independent 1-D dynamic programme along its scanlines.  Asymmetric V pins the index
    order V[mu at i-r][lambda at i]; per-edge weights pin where theta_{i-r,i} is stored."""
    H, W, L = 4, 5, 2
    rng = np.random.default_rng(3)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L))
    w = rng.uniform(0.5, 1.5, (len(dirs), 1, H, W))
    f = oracle.forward("isgmr", unary, V, dirs, 1, edge_weight=w, dtype=F64)
    for r, (dh, dw) in enumerate(dirs):
        seen = np.zeros((H, W), bool)
        for y0 in range(H):
            for x0 in range(W):
                if 0 <= y0 - dh < H and 0 <= x0 - dw < W:
                    continue
                line = []
                y, x = y0, x0
                while 0 <= y < H and 0 <= x < W:
                    line.append((y, x)); y += dh; x += dw
                ul = np.array([unary[0, yy, xx] for yy, xx in line])
                wl = np.array([w[r, 0, yy, xx] for yy, xx in line])
                ref = scanline_prefix_min(ul, wl, V)
                got = np.array([f.messages[r, 0, yy, xx] for yy, xx in line])
                np.testing.assert_allclose(got, ref, atol=1e-12)
                for yy, xx in line:
                    assert not seen[yy, xx]
                    seen[yy, xx] = True
        assert seen.all()  # every node lies on exactly one scanline of each direction


def _scanlines(H, W, dh, dw):
    """Maximal in-grid chains of direction (dh, dw), written from the grid alone."""
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


@pytest.mark.parametrize("H,W,L", [(3, 3, 3), (3, 4, 2)])
def test_isgmr_second_iteration_reads_last_iterations_messages(oracle, H, W, L):
    """The schedule of Alg. 1 on a loopy grid: in iteration 2, direction r reads the messages that
    iteration 1 left in the other directions d (not the ones iteration 2 is producing), and neither
    its own old message nor that of r- (Eq. isgmr).  Then the iteration-2 messages of direction r are
    the scanline minimisation of Eq. sgm over the unaries theta + sum_{d not in {r, r-}} m^{d,1}.
    Both the iteration-1 messages and the iteration-2 reference are enumerated here."""
    rng = np.random.default_rng(100 + H * W)
    unary = rng.random((1, H, W, L))
    V = rng.random((L, L))                 # asymmetric
    w = rng.uniform(0.5, 1.5, (4, 1, H, W))
    opp = {0: 1, 1: 0, 2: 3, 3: 2}
    m1 = np.zeros((4, H, W, L))
    for r, (dh, dw) in enumerate(DIRS4):
        for line in _scanlines(H, W, dh, dw):
            ul = np.array([unary[0, y, x] for y, x in line])
            wl = np.array([w[r, 0, y, x] for y, x in line])
            ref = scanline_prefix_min(ul, wl, V)
            for n, (y, x) in enumerate(line):
                m1[r, y, x] = ref[n]
    f1 = oracle.forward("isgmr", unary, V, DIRS4, 1, edge_weight=w, dtype=F64)
    np.testing.assert_allclose(f1.messages[:, 0], m1, atol=1e-12)
    f2 = oracle.forward("isgmr", unary, V, DIRS4, 2, edge_weight=w, dtype=F64)
    for r, (dh, dw) in enumerate(DIRS4):
        others = [d for d in range(4) if d != r and d != opp[r]]
        theta = unary[0] + sum(m1[d] for d in others)
        for line in _scanlines(H, W, dh, dw):
            ul = np.array([theta[y, x] for y, x in line])
            wl = np.array([w[r, 0, y, x] for y, x in line])
            ref = scanline_prefix_min(ul, wl, V)
            got = np.array([f2.messages[r, 0, y, x] for y, x in line])
            np.testing.assert_allclose(got, ref, atol=1e-12)
    # and the final costs are the aggregation of exactly those messages
    np.testing.assert_allclose(f2.cost[0], unary[0] + f2.messages[:, 0].sum(0), atol=1e-12)


def test_trwp_single_direction_equals_isgmr(oracle):
    """First direction of the first iteration: all messages are 0, so Eq. trwp with rho = 1
    and Eq. isgmr coincide."""
    H, W, L = 3, 4, 3
    unary, V, w = rand_problem(8, H, W, L, [(0, 1)], symmetric=False)
    a = oracle.forward("isgmr", unary, V, [(0, 1)], 1, edge_weight=w, dtype=F64)
    b = oracle.forward("trwp", unary, V, [(0, 1)], 1, edge_weight=w, rho=[1.0], dtype=F64)
    np.testing.assert_array_equal(a.p, b.p)
    np.testing.assert_allclose(a.cost, b.cost, atol=1e-12)


def test_trwp_rho_chain_discounted_bruteforce(oracle):
    """Eq. trwp on a 1 x W chain, K = 1, directions (->, <-) with rho_-> != rho_<- != 1.
    Unrolling the update gives a minimisation over the labels of the nodes behind node i in
    which node t's terms are discounted by powers of rho; that minimisation is enumerated
    here.  Pins: rho multiplies the unary AND every message at i-r (own direction
    included), and m^{r-} is subtracted undiscounted."""
    W, L = 4, 3
    rho_f, rho_b = 0.6, 0.3
    rng = np.random.default_rng(77)
    unary = rng.random((1, 1, W, L))
    V = rng.random((L, L))
    dirs = [(0, 1), (0, -1)]
    w = rng.uniform(0.5, 1.5, (2, 1, 1, W))
    f = oracle.forward("trwp", unary, V, dirs, 1, edge_weight=w, rho=[rho_f, rho_b], dtype=F64)
    th = unary[0, 0]

    # forward sweep: m_i(lam) = min_{x_0..x_{i-1}} sum_t rho^(i-t) th_t(x_t) + rho^(i-1-t) w_{t+1} V(x_t,x_{t+1})
    mf = np.zeros((W, L))
    for i in range(1, W):
        for lam in range(L):
            best = np.inf
            for xs in itertools.product(range(L), repeat=i):
                seq = list(xs) + [lam]
                e = sum(rho_f ** (i - t) * th[t][seq[t]] for t in range(i))
                e += sum(rho_f ** (i - 1 - t) * w[0, 0, 0, t + 1] * V[seq[t]][seq[t + 1]] for t in range(i))
                best = min(best, e)
            mf[i, lam] = best
        mf[i] -= mf[i].min()
    np.testing.assert_allclose(f.messages[0, 0, 0], mf, atol=1e-12)

    # backward sweep sees the fresh forward messages: node potential
    # phi_t = rho_b th_t + (rho_b - 1) mf_t ; V is indexed [x_{t+1}][x_t] (source = t+1)
    phi = rho_b * th + (rho_b - 1.0) * mf
    mb = np.zeros((W, L))
    for i in range(W - 2, -1, -1):
        n = W - 1 - i
        for lam in range(L):
            best = np.inf
            for xs in itertools.product(range(L), repeat=n):
                seq = [lam] + list(xs)          # labels of nodes i, i+1, ..., W-1
                e = sum(rho_b ** (t - 1) * phi[i + t][seq[t]] for t in range(1, n + 1))
                e += sum(rho_b ** t * w[1, 0, 0, i + t] * V[seq[t + 1]][seq[t]] for t in range(n))
                best = min(best, e)
            mb[i, lam] = best
        mb[i] -= mb[i].min()
    np.testing.assert_allclose(f.messages[1, 0, 0], mb, atol=1e-12)
    np.testing.assert_allclose(f.cost[0, 0], th + mf + mb, atol=1e-12)


def test_loopy_grid_energy_not_below_optimum(oracle):
    """On a loopy 3x3 grid the labelling need not be optimal but its energy (Eq. 1) can
    never be below the brute-force minimum, and on this easy instance (strong unaries)
    both algorithms find the optimum."""
    H, W, L = 3, 3, 3
    rng = np.random.default_rng(5)
    unary = rng.random((1, H, W, L)) * 4.0
    V = np.abs(np.subtract.outer(np.arange(L), np.arange(L))).astype(F64)
    w = mirrored_edge_weights(rng, 1, H, W, DIRS4, lambda g, s: g.uniform(0.1, 0.3, s)).astype(F64)
    edges = grid_edges(H, W, DIRS4, w, V, only=[0, 2])
    _, xmap, emin = min_marginals(unary.reshape(-1, L), edges, L)
    for algo in ("isgmr", "trwp"):
        f = oracle.forward(algo, unary, V, DIRS4, 10, edge_weight=w, rho=[0.5] * 4, dtype=F64)
        e = energies(f.labels.reshape(1, -1).astype(np.int64), unary.reshape(-1, L), edges)[0]
        assert e >= emin - 1e-12
        assert (f.labels.reshape(-1) == xmap).all()
