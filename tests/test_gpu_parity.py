"""GPU parity: the HIP path (through the C-ABI library) against the CPU oracle, element by
element, on the same seeded inputs.

Bar: p, q, labels bit-exact (the argmins are decided in float32 on both sides, lowest
index on ties); costs and messages within 1e-5 relative / 1e-4 absolute (they are in fact
expected to be identical: same operations in the same order); gradients within the same
tolerance of the oracle's double instantiation replaying the same indices (the library
carries its sums in double and rounds once on store; the float32 instantiation of the
oracle rounds after every addition and is itself up to about one tolerance away from the
double one on the larger problems -- its distance is printed, not asserted).
"""
import os

import numpy as np
import pytest

from mrf_inputs import DIRS4, DIRS8, DIRS16, make_config, random_problem

pytestmark = pytest.mark.gpu

RTOL, ATOL = 1e-5, 1e-4


def oracle_forward(oracle, pr, threads=False):
    return oracle.forward(pr.algo, pr.unary, pr.pairwise, pr.dirs, pr.K, edge_weight=pr.edge_weight,
                          edge_weight_scalar=pr.edge_weight_scalar, rho=pr.rho, threads=threads,
                          rho_edge=pr.rho_edge)


def oracle_backward(oracle, pr, p, q, dtype=np.float32):
    c = lambda a: None if a is None else a.astype(dtype)
    return oracle.backward(pr.algo, pr.shape, c(pr.pairwise), pr.dirs, pr.K, c(pr.grad_cost), p, q,
                           edge_weight=c(pr.edge_weight), edge_weight_scalar=pr.edge_weight_scalar,
                           rho=pr.rho, dtype=dtype, rho_edge=c(pr.rho_edge))


def check_forward(g, f):
    np.testing.assert_array_equal(g.p, f.p)
    np.testing.assert_array_equal(g.q, f.q)
    np.testing.assert_array_equal(g.labels, f.labels)
    np.testing.assert_allclose(g.messages, f.messages, rtol=RTOL, atol=ATOL)
    np.testing.assert_allclose(g.cost, f.cost, rtol=RTOL, atol=ATOL)


def check_grad(name, got, ref32, ref64):
    """Asserts against the double replay alone; ref32 (the float32 oracle, may be None) only
    adds its own distance to the message."""
    assert np.isfinite(got).all(), name
    e64 = np.abs(got.astype(np.float64) - ref64) / (ATOL + RTOL * np.abs(ref64))
    worst = e64.max() if e64.size else 0.0
    if worst > 1.0:
        e32 = -1.0 if ref32 is None else (np.abs(got.astype(np.float64) - ref32) / (ATOL + RTOL * np.abs(ref32))).max()
        raise AssertionError("%s: worst error/tolerance vs double replay %.3f (vs f32 oracle %.3f)" % (name, worst, e32))


def check_backward(g, b32, b64, want_V=True):
    f = lambda name: None if b32 is None else getattr(b32, name)
    check_grad("grad_unary", g.grad_unary, f("grad_unary"), b64.grad_unary)
    check_grad("grad_edge_weight", g.grad_edge_weight, f("grad_edge_weight"), b64.grad_edge_weight)
    if want_V:
        check_grad("grad_pairwise", g.grad_pairwise, f("grad_pairwise"), b64.grad_pairwise)


def full_check(oracle, pr, threads=False, want_V=True):
    """want_V=False: the caller passes no grad_pairwise buffer (a model whose V has no free
    parameters); the library may then pick other backward kernels."""
    from gpu_harness import run_gpu
    g = run_gpu(pr, want_V=want_V)
    f = oracle_forward(oracle, pr, threads=threads)
    check_forward(g, f)
    b32 = oracle_backward(oracle, pr, f.p, f.q, np.float32)
    b64 = oracle_backward(oracle, pr, f.p, f.q, np.float64)
    check_backward(g, b32, b64, want_V)
    return g


CONFIG_CASES = [
    (1, None, "isgmr", None), (1, None, "trwp", None),
    (2, (24, 40), "trwp", None), (2, (24, 40), "isgmr", None),
    (3, (12, 20), "isgmr", None), (3, (12, 20), "trwp", None),
    (4, (10, 12), "trwp", 3), (4, (10, 12), "isgmr", 2),
    (5, (24, 32), "isgmr", None), (5, (24, 32), "trwp", None),
]


@pytest.mark.parametrize("index,crop,algo,K", CONFIG_CASES)
def test_benchmark_configs_cropped(oracle, index, crop, algo, K):
    print("case config", index, crop, algo, K, flush=True)
    pr = make_config(index, crop=crop, algo=algo, K=K)
    full_check(oracle, pr)


RANDOM_CASES = [
    # seed, algo, B, H, W, L, dirs, K, integer_valued, per_edge
    (1, "isgmr", 1, 5, 7, 1, DIRS4, 2, False, True),
    (2, "trwp", 1, 5, 7, 2, DIRS4, 2, False, True),
    (3, "isgmr", 2, 6, 5, 33, DIRS8, 2, False, True),
    (4, "trwp", 2, 6, 5, 65, DIRS8, 2, False, False),
    (5, "isgmr", 1, 7, 6, 100, DIRS16, 2, False, True),
    (6, "trwp", 1, 7, 6, 129, DIRS16, 2, False, True),
    (7, "isgmr", 1, 4, 9, 200, DIRS4, 3, False, False),
    (8, "trwp", 1, 9, 4, 255, DIRS4, 2, False, True),
    (9, "isgmr", 1, 8, 8, 7, DIRS8, 3, True, True),      # integer data: many ties
    (10, "trwp", 1, 8, 8, 70, DIRS4, 3, True, True),
    (11, "isgmr", 1, 1, 12, 12, DIRS8, 2, False, True),   # one row: vertical/diagonal scanlines have one node
    (12, "trwp", 1, 12, 1, 12, DIRS8, 2, False, True),    # one column
    (13, "isgmr", 1, 6, 6, 16, [(0, 1), (1, 0)], 3, False, True),        # no opposite directions
    (14, "trwp", 1, 6, 6, 16, [(0, 1), (1, 0), (-1, 0)], 3, False, True),
    (15, "trwp", 3, 5, 5, 64, DIRS4, 2, False, True),
    (16, "isgmr", 1, 1, 1, 5, DIRS4, 2, False, True),     # single node: nothing to pass
]


@pytest.mark.parametrize("case", RANDOM_CASES, ids=lambda c: "seed%d" % c[0])
def test_random_shapes(oracle, case):
    print("case random", case[:8], flush=True)
    seed, algo, B, H, W, L, dirs, K, iv, pe = case
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=pe,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    full_check(oracle, pr)


@pytest.mark.parametrize("algo", ["isgmr", "trwp"])
def test_asymmetric_pairwise(oracle, algo):
    print("case asymmetric", algo, flush=True)
    pr = random_problem(21, algo, 1, 6, 7, 40, DIRS8, 2, symmetric=False)
    full_check(oracle, pr)


@pytest.mark.parametrize("mch", [8, 16, 32])
def test_wavefront_split_does_not_change_results(oracle, mch):
    """The number of source labels per wavefront is a tuning knob; p, q and messages must not
    depend on it."""
    import paper_1910_10892_amd as mrf
    print("case tune", mch, flush=True)
    try:
        assert mrf.mrf_tune(0, mch) == 0
        for L in (48, 96, 130):
            pr = random_problem(30 + L, "trwp", 1, 5, 6, L, DIRS4, 2)
            full_check(oracle, pr)
    finally:
        mrf.mrf_tune(0, 0)


@pytest.mark.parametrize("case", [
    (601, "trwp", 1, 5, 9, 65, DIRS4, 2, False), (602, "isgmr", 2, 4, 7, 96, DIRS8, 2, True),
    (603, "trwp", 1, 6, 5, 130, DIRS8, 2, False), (604, "isgmr", 1, 3, 11, 192, DIRS16, 2, False),
    (605, "trwp", 1, 7, 6, 255, DIRS4, 3, True), (606, "isgmr", 1, 4, 8, 256, DIRS4, 2, False),
    (607, "trwp", 1, 3, 40, 100, [(0, 1), (1, 0), (-1, 0)], 2, False),
], ids=lambda c: "seed%d" % c[0])
def test_dense_sweep_with_a_slice_of_labels_per_wavefront(oracle, case):
    """More than 64 labels, general dense table: the sweep in which every wavefront owns 32 labels
    against the oracle, and bit for bit against the sweep in which every wavefront does the O(L) work
    of the whole node."""
    import paper_1910_10892_amd as mrf
    print("case dense sliced", case[:8], flush=True)
    seed, algo, B, H, W, L, dirs, K, iv = case
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, symmetric=False,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    try:
        assert mrf.mrf_tune(16, 2) == 0
        a = full_check(oracle, pr, want_V=False)
        assert mrf.mrf_last_sweep_kernel(False) == "mrf_fwd_sweep_sliced"
        assert mrf.mrf_tune(16, 1) == 0
        b = full_check(oracle, pr, want_V=False)
        assert mrf.mrf_last_sweep_kernel(False) == "mrf_fwd_sweep"
    finally:
        mrf.mrf_tune(16, 0)
    for name in ("p", "q", "labels", "cost", "messages"):
        np.testing.assert_array_equal(getattr(a, name), getattr(b, name), err_msg=name)


PRESUM_CASES = [
    # seed, B, H, W, L, dirs, K, integer_valued, truncated
    (701, 1, 6, 7, 40, DIRS8, 3, False, False), (702, 2, 5, 6, 21, DIRS8, 3, True, False),
    (703, 1, 5, 5, 33, DIRS16, 3, False, False), (704, 1, 7, 9, 96, DIRS8, 3, False, True),
    (705, 1, 6, 8, 192, DIRS16, 2, True, True), (706, 1, 9, 5, 70, DIRS4, 4, False, True),
    (707, 1, 5, 7, 13, ((0, 1), (1, 0), (1, 1)), 3, False, False),      # no direction has its opposite in the set
    (708, 1, 3, 5, 7, ((0, 1), (0, -1), (1, 0)), 3, True, False),       # one pair and a single direction; N L odd
    (709, 1, 12, 11, 130, DIRS8, 2, False, False),
]


@pytest.mark.gpu
@pytest.mark.parametrize("case", PRESUM_CASES, ids=lambda c: "seed%d" % c[0])
def test_isgmr_sums_of_the_previous_iteration_formed_once(oracle, case):
    """ISGMR forward where a streaming pass per iteration sums the unary and the previous iteration's
    messages once per pair of opposite directions and the sweeps read that one array (Eq. isgmr):
    against the oracle, and bit for bit against the sweeps that read every array themselves."""
    import paper_1910_10892_amd as mrf
    print("case presum", case[:5], len(case[5]), case[6:], flush=True)
    seed, B, H, W, L, dirs, K, iv, trunc = case
    if trunc:
        pr = truncated_problem(seed, "isgmr", H, W, L, dirs, K, 1, 3.0, iv, "pos")
    else:
        pr = random_problem(seed, "isgmr", B, H, W, L, dirs, K, integer_valued=iv, symmetric=False)
    try:
        assert mrf.mrf_tune(17, 2) == 0
        a = full_check(oracle, pr, want_V=False)
        assert mrf.mrf_tune(17, 1) == 0
        b = full_check(oracle, pr, want_V=False)
    finally:
        mrf.mrf_tune(17, 0)
    for name in ("p", "q", "labels", "cost", "messages"):
        np.testing.assert_array_equal(getattr(a, name), getattr(b, name), err_msg=name)


@pytest.mark.gpu
def test_knobs_and_reports_are_kept_per_thread(oracle):
    """The kernel-choice knobs and the launch reports are the library's only state and belong to the calling
    thread: another thread neither sees this thread's knob nor disturbs its report."""
    import threading
    import paper_1910_10892_amd as mrf
    from gpu_harness import GpuProblem
    pr = make_config(1, algo="isgmr")
    g = GpuProblem(pr)
    seen = {}
    try:
        assert mrf.mrf_tune(3, 1) == 0                    # this thread: never the packed sweep
        g.forward()
        torch_sync = __import__("torch").cuda.synchronize
        torch_sync()
        mine = mrf.mrf_last_sweep_kernel(False)
        assert mine != "mrf_fwd_sweep_packed"

        def other():
            seen["before"] = mrf.mrf_last_sweep_kernel(False)
            g2 = GpuProblem(pr)
            g2.forward()
            torch_sync()
            seen["after"] = mrf.mrf_last_sweep_kernel(False)
        t = threading.Thread(target=other)
        t.start()
        t.join()
        assert seen["before"] == ""                       # nothing launched from that thread yet
        assert seen["after"] == "mrf_fwd_sweep_packed"    # its own default rules, not this thread's knob
        assert mrf.mrf_last_sweep_kernel(False) == mine
    finally:
        mrf.mrf_tune(3, 0)


CHAIN_PK_CASES = [
    # seed, B, H, W, L, dirs, K, integer_valued, per_edge, want_V
    (771, 1, 6, 9, 21, DIRS4, 3, False, True, True), (772, 3, 5, 7, 32, DIRS8, 2, True, True, False),
    (773, 1, 7, 5, 5, ((0, 1), (1, 0), (1, 1)), 2, False, False, True), (774, 1, 1, 13, 17, DIRS4, 2, False, True, True),
    (775, 2, 9, 4, 1, DIRS4, 2, False, True, True), (776, 1, 23, 31, 16, DIRS8, 2, True, True, True),
    (777, 1, 40, 37, 21, DIRS4, 2, False, True, True),
]


@pytest.mark.gpu
@pytest.mark.parametrize("case", CHAIN_PK_CASES, ids=lambda c: "seed%d" % c[0])
def test_chain_backward_with_two_scanlines_per_workgroup(oracle, case):
    """TRWP with up to 32 labels: the chain layout with two scanlines per workgroup (odd scanline counts,
    diagonal scanlines of unequal length, one-node scanlines, with and without grad_pairwise) against the oracle
    and against the layout the rules would pick."""
    import paper_1910_10892_amd as mrf
    print("case chain pk", case[:5], len(case[5]), case[6:], flush=True)
    seed, B, H, W, L, dirs, K, iv, per_edge, want_V = case
    pr = random_problem(seed, "trwp", B, H, W, L, dirs, K, integer_valued=iv, per_edge=per_edge, symmetric=False,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    pr.grad_cost = (pr.grad_cost * 0.2).astype(np.float32)
    try:
        for ni in (2, 4, 8):
            assert mrf.mrf_tune(20, 2) == 0 and mrf.mrf_tune(7, ni) == 0
            a = full_check(oracle, pr, want_V=want_V)
            assert mrf.mrf_last_sweep_kernel(True) == "mrf_bwd_sweep_chain_pk", mrf.mrf_last_sweep_launch(True)
        assert mrf.mrf_tune(20, 1) == 0 and mrf.mrf_tune(7, 0) == 0
        b = full_check(oracle, pr, want_V=want_V)
        assert mrf.mrf_last_sweep_kernel(True) != "mrf_bwd_sweep_chain_pk"
    finally:
        mrf.mrf_tune(20, 0)
        mrf.mrf_tune(7, 0)
    for name in ("grad_unary", "grad_edge_weight") + (("grad_pairwise",) if want_V else ()):
        check_grad(name + " (two layouts)", getattr(a, name), None, getattr(b, name).astype(np.float64))


GV_APART_CASES = [
    # seed, B, H, W, L, dirs, K, integer_valued, per_edge
    (751, 1, 6, 9, 96, DIRS4, 3, False, True), (752, 2, 5, 7, 128, DIRS8, 2, True, True),
    (753, 1, 7, 5, 65, ((0, 1), (1, 0), (1, 1)), 2, False, False), (754, 1, 4, 33, 100, DIRS4, 2, False, True),
]


@pytest.mark.gpu
@pytest.mark.parametrize("case", GV_APART_CASES, ids=lambda c: "seed%d" % c[0])
def test_pairwise_gradient_added_up_behind_the_chain_sweep(oracle, case):
    """TRWP with 65..128 labels and grad_pairwise: the chain sweep stores the node gradients and a streaming
    pass forms the table (Eq. supp-gradient-smoothness); against the oracle, and against the sweep that
    accumulates the table itself."""
    import paper_1910_10892_amd as mrf
    print("case grad V apart", case[:5], len(case[5]), case[6:], flush=True)
    seed, B, H, W, L, dirs, K, iv, per_edge = case
    pr = random_problem(seed, "trwp", B, H, W, L, dirs, K, integer_valued=iv, per_edge=per_edge, symmetric=False,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    pr.grad_cost = (pr.grad_cost * 0.2).astype(np.float32)
    try:
        a = full_check(oracle, pr, want_V=True)
        assert mrf.mrf_last_sweep_kernel(True) == "mrf_bwd_sweep_chain", mrf.mrf_last_sweep_launch(True)
        assert mrf.mrf_tune(19, 1) == 0
        b = full_check(oracle, pr, want_V=True)
        assert mrf.mrf_last_sweep_kernel(True) != "mrf_bwd_sweep_chain"
    finally:
        mrf.mrf_tune(19, 0)
    check_grad("grad_pairwise (two layouts)", a.grad_pairwise, None, b.grad_pairwise.astype(np.float64))


def truncated_problem(seed, algo, H, W, L, dirs, K, kind, trunc, integer_valued, weights):
    """Truncated linear (kind 1) / quadratic (kind 2) pairwise with the kind announced, so the
    library may take its window path.  weights: 'pos' | 'zero_mix' | 'neg_mix'."""
    from mrf_inputs import truncated_linear, truncated_quadratic
    pr = random_problem(seed, algo, 1, H, W, L, dirs, K, integer_valued=integer_valued,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    scale = 1.0 if integer_valued else 0.37
    pr.pairwise = truncated_linear(L, trunc, scale) if kind == 1 else truncated_quadratic(L, trunc, scale)
    pr.pairwise_kind, pr.trunc, pr.scale = kind, float(trunc), float(scale)
    rng = np.random.default_rng(seed + 1000)
    if weights == "zero_mix":
        pr.edge_weight = pr.edge_weight * (rng.random(pr.edge_weight.shape) > 0.3)
    elif weights == "neg_mix":
        pr.edge_weight = pr.edge_weight * np.where(rng.random(pr.edge_weight.shape) > 0.2, 1.0, -0.5)
    pr.edge_weight = pr.edge_weight.astype(np.float32)
    return pr


WINDOW_CASES = [
    # seed, algo, H, W, L, dirs, K, kind, trunc, integer_valued, weights
    (41, "trwp", 6, 9, 96, DIRS4, 3, 1, 8.0, False, "pos"),
    (42, "isgmr", 6, 9, 96, DIRS8, 2, 1, 8.0, True, "pos"),        # integer data: ties between window and far field
    (43, "trwp", 5, 7, 40, DIRS4, 3, 1, 2.0, True, "zero_mix"),    # zero weights: every candidate ties
    (44, "isgmr", 5, 7, 70, DIRS4, 2, 2, 200.0, False, "pos"),     # quadratic, window 15
    (45, "trwp", 5, 7, 130, DIRS8, 2, 2, 30.0, True, "neg_mix"),   # negative weights take the full loop
    (46, "isgmr", 4, 6, 200, DIRS4, 2, 1, 1.0, True, "pos"),       # Potts
    (47, "trwp", 4, 6, 17, DIRS4, 2, 1, 16.0, False, "pos"),       # window almost as wide as the label range
    (48, "trwp", 4, 6, 12, DIRS4, 2, 1, 20.0, False, "pos"),       # no truncation inside the range: dense kernel
    (49, "isgmr", 5, 5, 256, DIRS4, 2, 2, 200.0, True, "zero_mix"),
    # scanlines several times longer than the ring between the value and index wavefronts
    (50, "trwp", 3, 41, 96, DIRS4, 2, 1, 8.0, False, "pos"),
    (54, "trwp", 5, 9, 70, DIRS4, 3, 1, 4.0, False, "pos"),          # window 4
    (57, "trwp", 4, 7, 96, DIRS4, 2, 1, 11.0, False, "pos"),         # window 12
    (58, "isgmr", 5, 6, 256, DIRS8, 2, 2, 100.0, True, "zero_mix"),  # quadratic, window 10 -> 12; the 64-label layouts take 16
    (55, "isgmr", 6, 7, 130, DIRS8, 2, 1, 3.0, True, "zero_mix"),
    (56, "trwp", 4, 6, 200, DIRS4, 2, 2, 10.0, True, "pos"),         # quadratic, sqrt(10) -> window 4
    (51, "trwp", 6, 8, 40, DIRS16, 2, 1, 3.0, False, "pos"),       # sixteen directions: fifteen message arrays per update
    (52, "trwp", 5, 9, 200, DIRS16, 2, 2, 60.0, True, "zero_mix"),
    (53, "isgmr", 6, 7, 130, DIRS16, 3, 1, 8.0, True, "pos"),
    (51, "isgmr", 2, 37, 40, DIRS8, 2, 1, 2.0, True, "zero_mix"),
    (52, "trwp", 2, 33, 70, DIRS4, 2, 2, 30.0, True, "neg_mix"),
    (53, "trwp", 1, 12, 40, DIRS8, 2, 1, 2.0, False, "pos"),       # one row: vertical and diagonal scanlines of one node
    (54, "trwp", 5, 6, 96, [(0, 1), (1, 0), (-1, 0)], 3, 1, 8.0, False, "pos"),   # a direction without its opposite
    (55, "isgmr", 6, 1, 33, DIRS4, 2, 1, 4.0, True, "zero_mix"),   # one column
    # 65 .. 128 labels, TRWP: the loader-fed value wavefront holds two adjacent labels per lane
    (56, "trwp", 4, 19, 65, DIRS4, 2, 1, 8.0, False, "pos"),       # one label in the second half of a pair
    (57, "trwp", 5, 13, 75, DIRS4, 3, 1, 2.0, True, "zero_mix"),   # odd label count, narrowest window
    (58, "trwp", 3, 21, 127, DIRS4, 2, 2, 200.0, False, "pos"),    # widest window, last lane half used
    (59, "trwp", 4, 11, 128, DIRS4, 2, 1, 8.0, True, "neg_mix"),   # every lane full; negative weights
    (60, "trwp", 6, 10, 100, [(0, 1), (0, -1), (1, 0)], 3, 2, 30.0, False, "pos"),
    (61, "trwp", 2, 40, 97, DIRS4, 2, 1, 16.0, True, "pos"),
]


@pytest.mark.parametrize("case", WINDOW_CASES, ids=lambda c: "seed%d" % c[0])
def test_window_path_is_exact(oracle, case):
    """Truncated models run through the window kernel; its results must equal the oracle's
    and, bit for bit, those of the dense kernel on the same problem."""
    import paper_1910_10892_amd as mrf
    from gpu_harness import run_gpu
    print("case window", case[:5], case[7:], flush=True)
    pr = truncated_problem(*case)
    if len(pr.dirs) > 8:
        # (the backward pass amplifies grad c with every direction and iteration: keep the gradients in the
        # range where the absolute part of the tolerance means something in fp32)
        pr.grad_cost = (pr.grad_cost * 0.05).astype(np.float32)
    got = {}
    try:
        assert mrf.mrf_tune(2, 1) == 0 and mrf.mrf_tune(4, 1) == 0      # one wavefront per scanline
        got["single"] = full_check(oracle, pr)
        if case[0] in (51, 52, 53):     # sixteen directions take the window sweep too
            assert mrf.mrf_last_sweep_kernel(False) == "mrf_fwd_sweep_window", mrf.mrf_last_sweep_launch(False)
        assert mrf.mrf_tune(4, 2) == 0 and mrf.mrf_tune(5, 1) == 0      # value + one index wavefront
        got["pair"] = full_check(oracle, pr)
        assert mrf.mrf_tune(5, 2) == 0 and mrf.mrf_tune(8, 1) == 0      # value + two index wavefronts
        got["trio"] = full_check(oracle, pr)
        assert mrf.mrf_tune(8, 2) == 0                                  # and a loader wavefront (TRWP)
        got["quad"] = full_check(oracle, pr)
        assert mrf.mrf_tune(2, 2) == 0 and mrf.mrf_tune(9, 1) == 0      # one wavefront per 64 labels
        got["split"] = full_check(oracle, pr)
        assert mrf.mrf_tune(9, 2) == 0 and mrf.mrf_tune(10, 4) == 0     # ... for the values, 4 index wavefronts
        got["squad4"] = full_check(oracle, pr)
        assert mrf.mrf_tune(10, 8) == 0
        got["squad8"] = full_check(oracle, pr)
        assert mrf.mrf_tune(1, 1) == 0                                  # dense sweep
        d = run_gpu(pr)
    finally:
        for knob in (1, 2, 4, 5, 8, 9, 10):
            mrf.mrf_tune(knob, 0)
    for layout, g in got.items():
        for name in ("p", "q", "labels", "cost", "messages"):
            np.testing.assert_array_equal(getattr(g, name), getattr(d, name), err_msg="%s %s" % (layout, name))


CHAIN_CASES = [
    # seed, algo, B, H, W, L, dirs, K, integer_valued, per_edge
    (81, "trwp", 1, 3, 70, 96, DIRS4, 2, False, True),      # scanlines many times the ring
    (82, "isgmr", 1, 2, 45, 40, DIRS8, 2, True, True),
    (83, "trwp", 2, 5, 6, 128, DIRS8, 2, False, False),
    (84, "isgmr", 1, 7, 9, 1, DIRS4, 2, False, True),
    (85, "trwp", 1, 1, 11, 20, DIRS16, 2, True, True),      # one row: most scanlines have one node
    (86, "trwp", 1, 9, 2, 65, [(0, 1), (1, 0), (-1, 0)], 3, False, True),
    (87, "trwp", 1, 4, 30, 200, DIRS4, 2, False, True),     # three and four labels per lane
    (88, "isgmr", 1, 3, 20, 256, DIRS8, 2, True, False),
]


@pytest.mark.parametrize("case", CHAIN_CASES, ids=lambda c: "seed%d" % c[0])
def test_chain_wavefront_backward_layout(oracle, case):
    """Backward sweeps that keep only the node-to-node chain on one wavefront and give the rest
    of a node to 2, 4, 6 or 8 helper wavefronts (chosen for launches with few scanlines when no
    grad_pairwise is asked for): each against the oracle, and against the one-wavefront sweep."""
    import paper_1910_10892_amd as mrf
    print("case chain backward", case[:8], flush=True)
    seed, algo, B, H, W, L, dirs, K, iv, pe = case
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=pe,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    got = {}
    try:
        assert mrf.mrf_tune(6, 1) == 0
        got[0] = full_check(oracle, pr, want_V=False)
        assert mrf.mrf_tune(6, 2) == 0
        for ni in (2, 4, 6, 8, 12):
            assert mrf.mrf_tune(7, ni) == 0
            got[ni] = full_check(oracle, pr, want_V=False)
    finally:
        mrf.mrf_tune(6, 0)
        mrf.mrf_tune(7, 0)
    for ni in (2, 4, 6, 8, 12):
        for name in ("grad_unary", "grad_edge_weight"):
            np.testing.assert_allclose(getattr(got[ni], name), getattr(got[0], name), rtol=1e-5, atol=1e-4,
                                       err_msg="%d helpers, %s" % (ni, name))


CHAIN_HOT_CASES = [
    # seed, algo, B, H, W, L, dirs, K, kind, trunc, integer_valued
    (101, "trwp", 1, 4, 60, 96, DIRS4, 2, 1, 8.0, False),
    (102, "isgmr", 2, 3, 25, 40, DIRS8, 2, 1, 2.0, True),
    (103, "trwp", 1, 6, 9, 130, DIRS8, 2, 2, 30.0, False),
    (104, "isgmr", 1, 2, 31, 256, DIRS4, 3, 2, 200.0, False),
    (105, "trwp", 1, 5, 5, 2, DIRS4, 2, 1, 1.0, True),
    (106, "trwp", 1, 3, 40, 64, [(0, 1), (0, -1), (1, 1)], 2, 3, 2.0, False),
]


@pytest.mark.parametrize("case", CHAIN_HOT_CASES, ids=lambda c: "seed%d" % c[0])
def test_chain_wavefront_backward_hot_label(oracle, case):
    """The chain layout on truncated models, where most labels scatter to one source label: with
    and without the register sum of that label's lanes, 2 and 8 helpers, against the oracle and
    against each other."""
    import paper_1910_10892_amd as mrf
    from mrf_inputs import truncated_linear, truncated_quadratic, sgm_penalties
    print("case chain backward, hot label", case, flush=True)
    seed, algo, B, H, W, L, dirs, K, kind, trunc, iv = case
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=True,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    scale = 1.0 if iv else 0.37
    pr.pairwise = (truncated_linear(L, trunc, scale) if kind == 1 else
                   truncated_quadratic(L, trunc, scale) if kind == 2 else sgm_penalties(L, 0.5, 2.0))
    pr.pairwise_kind, pr.trunc, pr.scale = kind, trunc, scale
    got = {}
    try:
        assert mrf.mrf_tune(6, 2) == 0
        for hot in (1, 2):
            for ni in (2, 8, 12):
                assert mrf.mrf_tune(12, hot) == 0 and mrf.mrf_tune(7, ni) == 0
                got[hot, ni] = full_check(oracle, pr, want_V=False)
                assert mrf.mrf_last_sweep_kernel(1) == "mrf_bwd_sweep_chain"
    finally:
        mrf.mrf_tune(6, 0)
        mrf.mrf_tune(7, 0)
        mrf.mrf_tune(12, 0)
    for key in got:
        for name in ("grad_unary", "grad_edge_weight"):
            np.testing.assert_allclose(getattr(got[key], name), getattr(got[1, 2], name), rtol=1e-5, atol=1e-4,
                                       err_msg="%s, %s" % (key, name))


CHAIN_GV_CASES = [
    # seed, algo, B, H, W, L, dirs, K, integer_valued, per_edge
    (91, "trwp", 2, 6, 40, 21, DIRS4, 2, False, True),
    (92, "isgmr", 1, 5, 33, 32, DIRS8, 2, True, True),
    (93, "trwp", 1, 9, 4, 2, DIRS4, 3, False, False),
    (94, "trwp", 1, 1, 13, 17, DIRS8, 2, True, True),       # one row: most scanlines have one node
    (95, "isgmr", 3, 4, 7, 1, DIRS4, 2, False, True),
    (96, "trwp", 1, 5, 30, 48, DIRS4, 2, False, True),      # more than 32 labels: fewer helpers fit
    (97, "isgmr", 1, 4, 21, 64, DIRS4, 2, True, True),
]


@pytest.mark.parametrize("case", CHAIN_GV_CASES, ids=lambda c: "seed%d" % c[0])
def test_chain_wavefront_backward_with_pairwise_gradient(oracle, case):
    """The chain layout when grad_pairwise is asked for (L <= 32: every helper wavefront keeps a
    V-gradient accumulator of its own): 2, 4, 6, 8 helpers against the oracle and against the
    one-wavefront sweep."""
    import paper_1910_10892_amd as mrf
    print("case chain backward with grad V", case[:8], flush=True)
    seed, algo, B, H, W, L, dirs, K, iv, pe = case
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=pe,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    got = {}
    try:
        assert mrf.mrf_tune(3, 1) == 0
        assert mrf.mrf_tune(6, 1) == 0
        got[0] = full_check(oracle, pr, want_V=True)
        assert mrf.mrf_last_sweep_kernel(1) == "mrf_bwd_sweep"
        assert mrf.mrf_tune(6, 2) == 0
        for ni in (2, 4, 6, 8, 12):
            assert mrf.mrf_tune(7, ni) == 0
            got[ni] = full_check(oracle, pr, want_V=True)
            assert mrf.mrf_last_sweep_kernel(1) == "mrf_bwd_sweep_chain"
    finally:
        mrf.mrf_tune(3, 0)
        mrf.mrf_tune(6, 0)
        mrf.mrf_tune(7, 0)
    for ni in (2, 4, 6, 8, 12):
        for name in ("grad_unary", "grad_edge_weight", "grad_pairwise"):
            np.testing.assert_allclose(getattr(got[ni], name), getattr(got[0], name), rtol=1e-5, atol=1e-4,
                                       err_msg="%d helpers, %s" % (ni, name))


@pytest.mark.parametrize("index,crop,algo,K", [c for c in CONFIG_CASES if c[0] != 5])
def test_benchmark_configs_cropped_without_pairwise_gradient(oracle, index, crop, algo, K):
    """The truncated models have no free parameters in V: run them the way bench.py does."""
    print("case config, no grad_pairwise", index, crop, algo, K, flush=True)
    pr = make_config(index, crop=crop, algo=algo, K=K)
    full_check(oracle, pr, want_V=False)


@pytest.mark.parametrize("algo,K,L,p1,p2", [("isgmr", 1, 64, 0.3, 1.7), ("isgmr", 3, 96, 1.0, 1.0),
                                           ("trwp", 2, 130, 0.5, 2.0)])
def test_sgm_penalties_through_the_window_path(oracle, algo, K, L, p1, p2):
    """The three SGM penalties (Eq. vsgm) announced as a distance function that is constant from
    distance 2 on; K = 1 with ISGMR is the revised single-pass SGM (Eq. sgm).  Window sweep against
    the oracle and, bit for bit, against the dense sweep."""
    import paper_1910_10892_amd as mrf
    from gpu_harness import run_gpu
    from mrf_inputs import sgm_penalties
    print("case sgm penalties", algo, K, L, flush=True)
    pr = random_problem(71, algo, 1, 6, 8, L, DIRS8, K, rho=np.linspace(0.3, 0.9, 8))
    pr.pairwise = sgm_penalties(L, p1, p2)
    pr.pairwise_kind, pr.trunc, pr.scale = 3, 2.0, 1.0
    g = full_check(oracle, pr)
    try:
        assert mrf.mrf_tune(1, 1) == 0
        d = run_gpu(pr)
    finally:
        mrf.mrf_tune(1, 0)
    for name in ("p", "q", "labels", "cost", "messages"):
        np.testing.assert_array_equal(getattr(g, name), getattr(d, name), err_msg=name)


@pytest.mark.parametrize("case", [
    (61, "trwp", 1, 6, 7, 200, DIRS4, 3, False, True),
    (62, "isgmr", 1, 5, 6, 256, DIRS8, 2, True, True),
    (63, "trwp", 2, 4, 5, 130, DIRS8, 2, False, False),
    (64, "isgmr", 1, 7, 5, 192, DIRS4, 2, False, True),
], ids=lambda c: "seed%d" % c[0])
def test_multi_wavefront_backward_layout(oracle, case):
    """Backward sweeps with one wavefront per 64 labels (chosen for launches with few scanlines
    and many labels) against the oracle, and identical to the one-wavefront layout."""
    import paper_1910_10892_amd as mrf
    print("case split backward", case[:8], flush=True)
    seed, algo, B, H, W, L, dirs, K, iv, pe = case
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=pe,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    try:
        assert mrf.mrf_tune(2, 1) == 0
        a = full_check(oracle, pr)
        assert mrf.mrf_tune(2, 2) == 0
        b = full_check(oracle, pr)
    finally:
        mrf.mrf_tune(2, 0)
    for name in ("grad_unary", "grad_edge_weight", "grad_pairwise"):
        np.testing.assert_allclose(getattr(a, name), getattr(b, name), rtol=1e-5, atol=1e-4, err_msg=name)


PACK_CASES = [
    (71, "isgmr", 2, 9, 11, 21, DIRS4, 3, False, True),
    (72, "trwp", 1, 7, 13, 16, DIRS8, 2, True, True),
    (73, "isgmr", 1, 6, 10, 5, DIRS16, 2, False, True),     # 16 directions: scanlines of very different length
    (74, "trwp", 3, 5, 6, 32, DIRS4, 2, False, False),
    (75, "isgmr", 1, 8, 3, 17, DIRS8, 2, True, True),
    (76, "trwp", 1, 3, 9, 1, DIRS4, 2, False, True),
    (77, "isgmr", 2, 13, 17, 21, DIRS8, 2, False, True),    # 21 labels, scanlines of many lengths: packs of three
    (78, "trwp", 1, 10, 7, 20, DIRS4, 3, True, True),
    (79, "isgmr", 1, 5, 64, 18, DIRS4, 2, True, False),
]


@pytest.mark.parametrize("case", PACK_CASES, ids=lambda c: "seed%d" % c[0])
def test_packed_scanlines_layout(oracle, case):
    """For L <= 32 several scanlines share a wavefront; results must not depend on it."""
    import paper_1910_10892_amd as mrf
    print("case packed", case[:8], flush=True)
    seed, algo, B, H, W, L, dirs, K, iv, pe = case
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=pe,
                        rho=np.linspace(0.3, 0.9, len(dirs)))
    try:
        assert mrf.mrf_tune(3, 1) == 0
        a = full_check(oracle, pr)
        assert mrf.mrf_tune(3, 2) == 0 and mrf.mrf_tune(11, 1) == 0      # packed, one wavefront does all
        b = full_check(oracle, pr)
        assert mrf.mrf_tune(11, 2) == 0                                  # packed, value + index wavefront
        c = full_check(oracle, pr)
        more = []
        if 16 < L <= 21:
            # three scanlines per wavefront (segments of 21 lanes), with and without index wavefronts
            assert mrf.mrf_tune(13, 2) == 0
            more.append(full_check(oracle, pr))
            assert "mrf_fwd_sweep_packed<21," in mrf.mrf_last_sweep_launch(False)
            assert "mrf_bwd_sweep_packed<21," in mrf.mrf_last_sweep_launch(True)
            assert mrf.mrf_tune(11, 1) == 0
            more.append(full_check(oracle, pr))
            more.append(full_check(oracle, pr, want_V=False))
    finally:
        mrf.mrf_tune(3, 0)
        mrf.mrf_tune(11, 0)
        mrf.mrf_tune(13, 0)
    for name in ("p", "q", "labels", "cost", "messages"):
        np.testing.assert_array_equal(getattr(a, name), getattr(b, name), err_msg=name)
        np.testing.assert_array_equal(getattr(a, name), getattr(c, name), err_msg=name)
        for m in more:
            np.testing.assert_array_equal(getattr(a, name), getattr(m, name), err_msg=name)


def test_optional_outputs_may_be_null(oracle):
    from gpu_harness import GpuProblem
    import torch
    print("case optional outputs", flush=True)
    for algo in ("isgmr", "trwp"):
        pr = make_config(1, algo=algo, K=2)
        full = GpuProblem(pr)
        full.forward(); full.backward()
        ref = full.results()
        g = GpuProblem(pr, want_messages=False)
        fn = __import__("paper_1910_10892_amd").mrf_isgmr_forward if algo == "isgmr" else \
            __import__("paper_1910_10892_amd").mrf_trwp_forward
        fn(g.prob, g.cost, None, g.p, g.q, None, g.workspace)
        g.backward(want_w=False, want_V=False)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(g.cost.cpu().numpy(), ref.cost)
        np.testing.assert_array_equal(g.p.cpu().numpy(), ref.p)
        # (without grad_pairwise the library may run other backward kernels: same sums, other order)
        np.testing.assert_allclose(g.grad_unary.cpu().numpy(), ref.grad_unary, rtol=1e-5, atol=1e-5)


def test_backward_is_reproducible_run_to_run():
    from gpu_harness import GpuProblem
    print("case reproducible", flush=True)
    for idx, crop, algo in ((2, (24, 40), "trwp"), (5, (24, 32), "isgmr")):
        pr = make_config(idx, crop=crop, algo=algo)
        g = GpuProblem(pr)
        g.forward(); g.backward()
        a = g.results()
        g.poison_outputs()
        g.forward(); g.backward()
        b = g.results()
        for name in ("cost", "p", "q", "grad_unary", "grad_edge_weight", "grad_pairwise"):
            np.testing.assert_array_equal(getattr(a, name), getattr(b, name), err_msg=name)


def test_waits_between_wavefronts_are_bounded(oracle):
    """The layouts that spread a scanline over several wavefronts give every wait a budget.  With a
    budget of one turn (set from the host) their first unmet wait gives up: every kernel still ends
    normally, and mrf_workspace_fault reports it.  With the default budget the same calls complete
    and report nothing."""
    import torch
    import paper_1910_10892_amd as mrf
    from gpu_harness import GpuProblem
    print("case bounded waits", flush=True)
    cases = [(make_config(2, crop=(24, 40), algo="trwp"), {}),       # value / loader / index wavefronts, chain backward
             (make_config(4, crop=(10, 12), algo="trwp", K=2), {}),  # value wavefronts that meet through LDS, index wavefronts
             (make_config(5, crop=(24, 32), algo="trwp"), {}),       # packed scanlines with index wavefronts
             (make_config(5, crop=(24, 32), algo="trwp"), {20: 2})]  # chain backward with two scanlines per workgroup
    for pr, knobs in cases:
        g = GpuProblem(pr)
        for k, v in knobs.items():
            assert mrf.mrf_tune(k, v) == 0
        try:
            assert mrf.mrf_tune(14, 1) == 0
            g.forward()
            fwd = mrf.mrf_workspace_fault(g.workspace)
            g.backward(want_V=False)
            bwd = mrf.mrf_workspace_fault(g.workspace)
            if knobs:
                assert mrf.mrf_last_sweep_kernel(True) == "mrf_bwd_sweep_chain_pk" and bwd == -11
        finally:
            mrf.mrf_tune(14, 0)
        print("  ", pr.name, mrf.mrf_last_sweep_launch(False), fwd, mrf.mrf_last_sweep_launch(True), bwd, flush=True)
        assert fwd in (0, -11) and bwd in (0, -11)
        assert fwd == -11 or bwd == -11          # these shapes take multi-wavefront layouts: some wait is unmet at first
        # default budget: complete, correct, nothing reported
        g.poison_outputs()
        g.forward()
        assert mrf.mrf_workspace_fault(g.workspace) == 0
        g.backward(want_V=False)
        assert mrf.mrf_workspace_fault(g.workspace) == 0
        got = g.results()
        f = oracle_forward(oracle, pr)
        check_forward(got, f)
        b64 = oracle_backward(oracle, pr, f.p, f.q, np.float64)
        check_grad("grad_unary", got.grad_unary, None, b64.grad_unary)
        for k in knobs:
            mrf.mrf_tune(k, 0)


def test_workspace_too_small_is_an_error_not_a_fault():
    from gpu_harness import GpuProblem
    import paper_1910_10892_amd as mrf
    print("case small workspace", flush=True)
    pr = make_config(1)
    g = GpuProblem(pr)
    small = g.workspace[: 256]
    with pytest.raises(mrf.MrfError) as ei:
        mrf.mrf_isgmr_forward(g.prob, g.cost, g.labels, g.p, g.q, g.messages, small)
    assert ei.value.status == -6


@pytest.mark.parametrize("index,crop,algo", [
    (2, None, "isgmr"),            # stereo shape, all four directions in one launch
    (3, (96, 312), "isgmr"),       # driving-stereo recipe, 1/16 of the area, L = 192, 8 directions
    (4, (64, 64), "trwp"),         # denoising recipe, 1/16 of the area, L = 256
    (5, None, "isgmr"),            # segmentation shape at full size (batch 4, 512 x 512, L = 21)
    (5, None, "trwp"),
])
def test_large_configs(oracle, index, crop, algo):
    """The other benchmark shapes at full size where the oracle finishes in seconds on all host
    threads, else on a centred fraction of the grid with every other parameter unchanged."""
    print("case large config", index, crop, algo, flush=True)
    pr = make_config(index, crop=crop, algo=algo)
    full_check(oracle, pr, threads=True)


def test_full_size_stereo_config_trwp(oracle):
    """The configuration the bench times (TRWP, 256x512, L = 96, K = 5), whole grid, in the
    launch configuration the bench uses (no grad_pairwise buffer: truncated linear V), and once
    more with that buffer; oracle forward on all host threads (bit-identical to one thread,
    asserted in the CPU suite)."""
    from gpu_harness import run_gpu
    print("case full config 2", flush=True)
    pr = make_config(2)
    f = oracle_forward(oracle, pr, threads=True)
    b32 = oracle_backward(oracle, pr, f.p, f.q, np.float32)
    b64 = oracle_backward(oracle, pr, f.p, f.q, np.float64)
    for want_V in (False, True):
        print("  grad_pairwise buffer:", want_V, flush=True)
        g = run_gpu(pr, want_V=want_V)
        check_forward(g, f)
        check_backward(g, b32, b64, want_V)


SGM_STD_CASES = [
    # seed, B, H, W, L, dirs, integer_valued, per_edge, kind (0 dense table, 3 SGM penalties)
    (501, 1, 6, 9, 16, DIRS8, False, True, 3),
    (502, 2, 5, 7, 70, DIRS4, True, True, 3),        # integer data: ties in both argmins
    (503, 1, 4, 6, 130, DIRS16, False, False, 3),
    (504, 1, 7, 5, 21, DIRS8, False, True, 0),       # general dense table
    (505, 1, 1, 9, 200, DIRS4, True, True, 3),       # one row
    (506, 1, 3, 3, 256, DIRS8, False, True, 0),
    (507, 1, 5, 5, 1, DIRS4, False, True, 0),
]


@pytest.mark.parametrize("case", SGM_STD_CASES, ids=lambda c: "seed%d" % c[0])
def test_standard_single_pass_sgm(oracle, case):
    """The standard SGM update (Eq. sgm_old: the message carries the node's own unary) and its
    aggregation (Eq. isgmr-aggregation-old) as a problem flag: forward outputs against the oracle;
    the backward entry points refuse the flag."""
    import torch
    import paper_1910_10892_amd as mrf
    from gpu_harness import GpuProblem
    from mrf_inputs import sgm_penalties
    print("case standard sgm", case, flush=True)
    seed, B, H, W, L, dirs, iv, pe, kind = case
    pr = random_problem(seed, "isgmr", B, H, W, L, dirs, 1, integer_valued=iv, per_edge=pe, symmetric=False)
    if kind == 3:
        pr.pairwise = sgm_penalties(L, 1.0 if iv else 0.3, 2.0 if iv else 1.7)
        pr.pairwise_kind, pr.trunc, pr.scale = 3, 2.0, 1.0
    pr.sgm_standard = True
    g = GpuProblem(pr)
    g.poison_outputs()
    g.forward()
    got = g.results(backward=False)
    f = oracle.sgm_standard_forward(pr.unary, pr.pairwise, pr.dirs, edge_weight=pr.edge_weight,
                                    edge_weight_scalar=pr.edge_weight_scalar)
    check_forward(got, f)
    np.testing.assert_array_equal(got.messages, f.messages)
    np.testing.assert_array_equal(got.cost, f.cost)
    with pytest.raises(mrf.MrfError) as ei:
        g.backward()
    assert ei.value.status == -8
    # more than one iteration has no meaning for a single-pass method
    g.prob.K = 2
    assert mrf.mrf_validate(g.prob, mrf.MRF_ISGMR) == -8


def _progress(msg):
    """Long tests say where they are: on stdout and, where a GPU job's output folder exists, in
    a file there (a run that is silent for minutes is taken for hung)."""
    import os, time
    print(msg, flush=True)
    d = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    if os.path.isdir(d):
        with open(os.path.join(d, "test_progress.log"), "a") as fh:
            fh.write("%s %s\n" % (time.strftime("%H:%M:%S"), msg))


def _full_size_check(oracle, pr, want_V, fwd_launch, bwd_launch):
    """Whole-grid parity in the launch configuration bench.py times: forward element by element
    (oracle forward on all host threads, bit-identical to one thread), gradients against the
    double replay, and the kernel instantiations the launch rules picked."""
    import gc
    import torch
    import paper_1910_10892_amd as mrf
    from gpu_harness import GpuProblem
    g = GpuProblem(pr)
    g.poison_outputs()
    g.forward()
    g.backward(want_V=want_V)
    assert mrf.mrf_workspace_fault(g.workspace) == 0
    assert mrf.mrf_last_sweep_launch(False) == fwd_launch, mrf.mrf_last_sweep_launch(False)
    assert mrf.mrf_last_sweep_launch(True) == bwd_launch, mrf.mrf_last_sweep_launch(True)
    _progress("  GPU done; oracle forward (all host threads)")
    f = oracle_forward(oracle, pr, threads=True)
    _progress("  oracle forward done; comparing")
    for name in ("p", "q", "labels"):
        got = getattr(g, name).cpu().numpy()
        assert np.array_equal(got, getattr(f, name)), name
        del got
    for name in ("messages", "cost"):
        got = getattr(g, name).cpu().numpy()
        ref = getattr(f, name)
        # (identical in fact: same operations in the same order)
        bad = np.abs(got - ref) > ATOL + RTOL * np.abs(ref)
        assert not bad.any(), "%s: %d entries off" % (name, int(bad.sum()))
        del got, bad
    p, q = f.p, f.q
    del f
    gc.collect()
    _progress("  oracle backward (double)")
    b64 = oracle_backward(oracle, pr, p, q, np.float64)
    _progress("  oracle backward done; comparing")
    check_grad("grad_unary", g.grad_unary.cpu().numpy(), None, b64.grad_unary)
    check_grad("grad_edge_weight", g.grad_edge_weight.cpu().numpy(), None, b64.grad_edge_weight)
    if want_V:
        check_grad("grad_pairwise", g.grad_pairwise.cpu().numpy(), None, b64.grad_pairwise)


def test_full_size_driving_stereo_config_isgmr(oracle):
    """The largest benchmark shape whole, as bench.py times it: ISGMR, 384 x 1248, L = 192, 8
    directions, K = 3 -- 9,788 scanlines per launch, message and index arrays beyond 2^31 bytes.
    The first iteration runs the launch with zero messages, the later ones the same launch on the
    per-pair sums that a streaming pass forms from the previous iteration's messages.  (The oracle's share of the test is about 35 s per iteration on 16 host
    threads.)"""
    _progress("case full config 3")
    pr = make_config(3)
    _full_size_check(oracle, pr, False,
                     "mrf_fwd_sweep_window<3,1,4,false,2> grid=9788 block=64 after mrf_isgmr_presum<8,4>",
                     "mrf_bwd_sweep<3,1,2,false,true,false,false> grid=2447 block=256")


def test_full_size_denoising_config_trwp(oracle):
    """The denoising shape whole: TRWP, 256 x 256, L = 256, truncated quadratic, rho = 0.5, in the
    launch configuration of the bench (no grad_pairwise buffer), all K = 10 iterations."""
    _progress("case full config 4")
    pr = make_config(4)
    _full_size_check(oracle, pr, False,
                     "mrf_fwd_sweep_window_squad<4,4,true,16,8> grid=256 block=768",
                     "mrf_bwd_sweep_chain<4,4,1,8,false,false,true> grid=256 block=576")


def test_full_size_denoising_config_dense_sweep(oracle):
    """The same shape through the dense O(L^2) sweep (the launch bench.py times as the dense
    variant of this configuration): K = 2, forward outputs only."""
    import torch
    import paper_1910_10892_amd as mrf
    from gpu_harness import GpuProblem
    _progress("case full config 4, dense sweep (K = 2)")
    pr = make_config(4, K=2)
    pr.pairwise_kind = 0
    g = GpuProblem(pr)
    g.poison_outputs()
    g.forward()
    torch.cuda.synchronize()
    assert mrf.mrf_last_sweep_launch(False) == "mrf_fwd_sweep_sliced<4,4,4,true> grid=256 block=512"
    f = oracle_forward(oracle, pr, threads=True)
    for name in ("p", "q", "labels", "messages", "cost"):
        assert np.array_equal(getattr(g, name).cpu().numpy(), getattr(f, name)), name


def _drawn_problem(seed):
    """A small problem with everything drawn at random: shape, label count (biased towards the
    borders of the kernels' layouts), direction set, iteration count, model and weights."""
    from mrf_inputs import truncated_linear, truncated_quadratic, sgm_penalties
    rng = np.random.default_rng(5000 + seed)
    algo = ("isgmr", "trwp")[int(rng.integers(0, 2))]
    B = int(rng.integers(1, 3))
    H, W = int(rng.integers(1, 11)), int(rng.integers(1, 14))
    L = int(rng.choice([1, 2, 3, 15, 16, 17, 21, 31, 32, 33, 63, 64, 65, 96, 127, 128, 129, 191, 192, 193, 255, 256]))
    sets = [DIRS4, DIRS8, DIRS16, [(0, 1)], [(1, 0), (-1, 0)], [(0, 1), (0, -1), (1, 1)], [(1, 2), (-1, -2), (0, 1), (2, -1)]]
    dirs = sets[int(rng.integers(0, len(sets)))]
    K = int(rng.integers(1, 4))
    iv = bool(rng.integers(0, 2))
    pe = bool(rng.integers(0, 4) > 0)
    pr = random_problem(6000 + seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=pe,
                        rho=rng.uniform(0.2, 1.0, len(dirs)))
    kind = int(rng.integers(0, 4))
    if kind and L >= 2:
        scale = 1.0 if iv else 0.41
        if kind == 1:
            trunc = float(rng.choice([1.0, 2.0, 3.0, 8.0, 11.0, 16.0, 40.0]))
            pr.pairwise = truncated_linear(L, trunc, scale)
        elif kind == 2:
            trunc = float(rng.choice([1.0, 4.0, 30.0, 200.0]))
            pr.pairwise = truncated_quadratic(L, trunc, scale)
        else:
            trunc = 2.0
            pr.pairwise = sgm_penalties(L, 0.5 if not iv else 1.0, 2.0)
        pr.pairwise_kind, pr.trunc, pr.scale = kind, trunc, scale
        if pr.edge_weight is not None and rng.integers(0, 3) == 0:
            pr.edge_weight = (pr.edge_weight * np.where(rng.random(pr.edge_weight.shape) > 0.15, 1.0, -0.5)).astype(np.float32)
    return pr, bool(rng.integers(0, 2))


# MRF_TEST_EXTRA_SEEDS=n adds n further seeds to each of the three drawn-problem tests (a longer soak)
EXTRA_SEEDS = int(os.environ.get("MRF_TEST_EXTRA_SEEDS", "0"))


@pytest.mark.parametrize("seed", range(150 + EXTRA_SEEDS))
def test_drawn_problems_default_dispatch(oracle, seed):
    """Whatever kernels the launch rules pick for a randomly drawn small problem, with and without
    a grad_pairwise buffer."""
    pr, want_V = _drawn_problem(seed)
    print("case drawn", seed, pr.algo, pr.shape, len(pr.dirs), pr.K, pr.pairwise_kind, pr.trunc, want_V, flush=True)
    # The backward pass is linear in grad c, and with many directions and iterations it amplifies
    # it by orders of magnitude (ISGMR re-injects every message into R - 2 others per iteration).
    # The absolute tolerance only means something for fp32 tensors of moderate size, so grad c is
    # scaled to keep the largest gradient entry near 10.
    f = oracle_forward(oracle, pr)
    b = oracle_backward(oracle, pr, f.p, f.q, np.float64)
    big = max(float(np.abs(b.grad_unary).max()), float(np.abs(b.grad_pairwise).max()),
              float(np.abs(b.grad_edge_weight).max()) if b.grad_edge_weight is not None else 0.0)
    if big > 10.0:
        pr.grad_cost = (pr.grad_cost * np.float32(10.0 / big)).astype(np.float32)
    full_check(oracle, pr, want_V=want_V)


@pytest.mark.parametrize("seed", range(120 + EXTRA_SEEDS))
def test_drawn_problems_forced_layouts(oracle, seed):
    """The same kind of random problems with the kernel-choice knobs drawn at random too, so that
    layouts meet shapes they would not be picked for (the results may not depend on the knobs)."""
    import paper_1910_10892_amd as mrf
    pr, want_V = _drawn_problem(1000 + seed)
    rng = np.random.default_rng(9000 + seed)
    knobs = {2: int(rng.integers(0, 3)), 3: int(rng.integers(0, 3)), 4: int(rng.integers(0, 3)),
             5: int(rng.integers(0, 3)), 6: int(rng.integers(0, 3)), 7: int(rng.choice([0, 2, 4, 6, 8, 12])),
             8: int(rng.integers(0, 3)), 9: int(rng.integers(0, 3)), 10: int(rng.choice([0, 4, 8])),
             11: int(rng.integers(0, 3)), 12: int(rng.integers(0, 3)), 13: int(rng.integers(0, 3)), 15: int(rng.integers(0, 3)), 16: int(rng.integers(0, 3)), 17: int(rng.integers(0, 3)), 18: int(rng.integers(0, 2)), 19: int(rng.integers(0, 2)), 20: int(rng.integers(0, 3))}
    print("case drawn+knobs", seed, pr.algo, pr.shape, len(pr.dirs), pr.K, pr.pairwise_kind, pr.trunc, want_V, knobs,
          flush=True)
    f = oracle_forward(oracle, pr)
    b = oracle_backward(oracle, pr, f.p, f.q, np.float64)
    big = max(float(np.abs(b.grad_unary).max()), float(np.abs(b.grad_pairwise).max()),
              float(np.abs(b.grad_edge_weight).max()) if b.grad_edge_weight is not None else 0.0)
    if big > 10.0:
        pr.grad_cost = (pr.grad_cost * np.float32(10.0 / big)).astype(np.float32)
    try:
        for k, v in knobs.items():
            assert mrf.mrf_tune(k, v) == 0
        full_check(oracle, pr, want_V=want_V)
    finally:
        for k in knobs:
            mrf.mrf_tune(k, 0)


RHO_EDGE_CASES = [
    # seed, B, H, W, L, dirs, K, kind, trunc, integer_valued, per_edge weights
    (201, 2, 6, 9, 21, DIRS4, 2, 0, 0.0, False, True),
    (202, 1, 5, 11, 96, DIRS8, 2, 1, 8.0, False, True),
    (203, 1, 4, 7, 130, DIRS4, 3, 0, 0.0, True, False),
    (204, 1, 3, 9, 200, DIRS4, 2, 2, 30.0, False, True),
    (205, 1, 6, 6, 3, DIRS16, 2, 0, 0.0, False, True),
    (206, 1, 1, 12, 40, [(0, 1), (0, -1), (1, 1)], 2, 3, 2.0, False, True),
    (207, 1, 8, 3, 256, DIRS4, 1, 1, 2.0, True, True),
]


@pytest.mark.parametrize("case", RHO_EDGE_CASES, ids=lambda c: "seed%d" % c[0])
def test_trwp_with_one_rho_per_edge(oracle, case):
    """TRWP with the TRW coefficient of Eq. trwp given per directed edge (an [R,B,H,W] array like
    the edge weights) instead of per direction: forward and backward against the oracle, with and
    without grad_pairwise; and an array that repeats one value per direction gives the forward
    results of the per-direction path bit for bit."""
    from mrf_inputs import truncated_linear, truncated_quadratic, sgm_penalties
    print("case per-edge rho", case, flush=True)
    seed, B, H, W, L, dirs, K, kind, trunc, iv, pe = case
    R = len(dirs)
    pr = random_problem(seed, "trwp", B, H, W, L, dirs, K, integer_valued=iv, per_edge=pe,
                        rho=np.linspace(0.3, 0.9, R))
    if kind:
        scale = 1.0 if iv else 0.37
        pr.pairwise = (truncated_linear(L, trunc, scale) if kind == 1 else
                       truncated_quadratic(L, trunc, scale) if kind == 2 else sgm_penalties(L, 0.5, 2.0))
        pr.pairwise_kind, pr.trunc, pr.scale = kind, trunc, scale
    rng = np.random.default_rng(7000 + seed)
    base = full_check(oracle, pr, want_V=False)
    pr.rho_edge = np.broadcast_to(pr.rho[:, None, None, None], (R, B, H, W)).astype(np.float32).copy()
    same = full_check(oracle, pr, want_V=False)
    for name in ("p", "q", "labels", "cost", "messages"):
        np.testing.assert_array_equal(getattr(base, name), getattr(same, name), err_msg=name)
    np.testing.assert_allclose(same.grad_unary, base.grad_unary, rtol=1e-5, atol=1e-4)
    pr.rho_edge = (rng.integers(1, 4, (R, B, H, W)) / 4.0 if iv else rng.uniform(0.2, 0.9, (R, B, H, W))).astype(np.float32)
    pr.rho = None
    full_check(oracle, pr, want_V=False)
    full_check(oracle, pr, want_V=True)


EDGE_TABLE_CASES = [
    # seed, algo, B, H, W, L, dirs, K, integer_valued
    (301, "isgmr", 2, 5, 7, 21, DIRS4, 2, False),
    (302, "trwp", 1, 6, 5, 21, DIRS4, 3, False),
    (303, "isgmr", 1, 4, 6, 64, DIRS8, 2, False),
    (304, "trwp", 1, 3, 9, 33, DIRS8, 2, True),
    (305, "isgmr", 1, 4, 4, 5, DIRS16, 2, True),
    (306, "trwp", 1, 7, 1, 9, [(1, 0), (-1, 0), (0, 1)], 2, False),
    (307, "trwp", 1, 2, 8, 1, DIRS4, 2, False),
    (308, "isgmr", 1, 3, 5, 16, DIRS4, 1, False),
    (309, "trwp", 1, 3, 5, 17, DIRS4, 2, False),
]


@pytest.mark.parametrize("case", EDGE_TABLE_CASES, ids=lambda c: "seed%d" % c[0])
def test_pairwise_potentials_given_per_edge(oracle, case):
    """Pairwise potentials as one L x L table per directed edge (Eq. isgmr / Eq. trwp as written)
    and the gradient of those tables (Eq. supp-gradient-pairwise): forward and backward against the
    oracle, with and without the table gradient; for TRWP also with one rho per edge."""
    print("case per-edge tables", case, flush=True)
    seed, algo, B, H, W, L, dirs, K, iv = case
    R = len(dirs)
    pr = random_problem(seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=False,
                        rho=np.linspace(0.3, 0.9, R))
    rng = np.random.default_rng(8000 + seed)
    Te = rng.integers(0, 3, (R, B, H, W, L, L)) if iv else rng.random((R, B, H, W, L, L))
    pr.pairwise_edge = Te.astype(np.float32)

    def check(want_V):
        from gpu_harness import run_gpu
        g = run_gpu(pr, want_V=want_V)
        f = oracle.forward(pr.algo, pr.unary, None, pr.dirs, pr.K, rho=pr.rho, rho_edge=pr.rho_edge,
                           pairwise_edge=pr.pairwise_edge)
        check_forward(g, f)
        b = {}
        for dt in (np.float32, np.float64):
            b[dt] = oracle.backward(pr.algo, pr.shape, None, pr.dirs, pr.K, pr.grad_cost.astype(dt), f.p, f.q,
                                    rho=pr.rho, dtype=dt, per_edge_pairwise=True,
                                    rho_edge=None if pr.rho_edge is None else pr.rho_edge.astype(dt))
        check_grad("grad_unary", g.grad_unary, b[np.float32].grad_unary, b[np.float64].grad_unary)
        if want_V:
            check_grad("grad_pairwise_edge", g.grad_pairwise, b[np.float32].grad_pairwise_edge,
                       b[np.float64].grad_pairwise_edge)
        return g

    a = check(True)
    c = check(False)
    np.testing.assert_allclose(c.grad_unary, a.grad_unary, rtol=1e-5, atol=1e-4)
    if algo == "trwp":
        pr.rho_edge = rng.uniform(0.2, 0.9, (R, B, H, W)).astype(np.float32)
        pr.rho = None
        check(True)


def test_per_edge_tables_argument_errors():
    import torch
    import paper_1910_10892_amd as mrf
    dev = torch.device("cuda:0")
    L = 70
    z = lambda *s: torch.zeros(s, dtype=torch.float32, device=dev)
    prob = mrf.MrfProblem(z(1, 2, 2, L), None, DIRS4, 1, pairwise_edge=z(4, 1, 2, 2, L, L))
    assert mrf.mrf_workspace_bytes(prob, mrf.MRF_ISGMR, False) == 0          # more than 64 labels
    L = 4
    prob = mrf.MrfProblem(z(1, 2, 2, L), None, DIRS4, 1, pairwise_edge=z(4, 1, 2, 2, L, L))
    ws = torch.empty(max(mrf.mrf_workspace_bytes(prob, mrf.MRF_ISGMR, True), 256), dtype=torch.uint8, device=dev)
    p = torch.zeros((1, 4, 1, 2, 2, L), dtype=torch.uint8, device=dev)
    q = torch.zeros((1, 4, 1, 2, 2), dtype=torch.uint8, device=dev)
    with pytest.raises(mrf.MrfError):      # there are no edge weights to differentiate
        mrf.mrf_isgmr_backward(prob, z(1, 2, 2, L), p, q, z(1, 2, 2, L), z(4, 1, 2, 2), None, ws)


@pytest.mark.parametrize("seed", range(30 + EXTRA_SEEDS))
def test_drawn_medium_problems_forced_layouts(oracle, seed):
    """Random problems whose scanlines are several times longer than the LDS rings of the
    taken-apart layouts (20..69 nodes), with the kernel-choice knobs drawn at random."""
    import paper_1910_10892_amd as mrf
    from mrf_inputs import truncated_linear, truncated_quadratic, sgm_penalties
    rng = np.random.default_rng(77000 + seed)
    algo = ("isgmr", "trwp")[int(rng.integers(0, 2))]
    B, H, W = int(rng.integers(1, 3)), int(rng.integers(20, 70)), int(rng.integers(20, 70))
    L = int(rng.choice([5, 16, 21, 32, 40, 64, 96, 130, 192, 256]))
    dirs = [DIRS4, DIRS8][int(rng.integers(0, 2))]
    K = int(rng.integers(1, 3))
    iv = bool(rng.integers(0, 2))
    pr = random_problem(88000 + seed, algo, B, H, W, L, dirs, K, integer_valued=iv, per_edge=bool(rng.integers(0, 2)),
                        rho=rng.uniform(0.2, 1.0, len(dirs)))
    kind = int(rng.integers(0, 4))
    if kind:
        scale = 1.0 if iv else 0.41
        if kind == 1:
            trunc = float(rng.choice([2.0, 3.0, 8.0, 11.0, 16.0]))
            pr.pairwise = truncated_linear(L, trunc, scale)
        elif kind == 2:
            trunc = float(rng.choice([4.0, 12.0, 30.0, 110.0, 200.0]))
            pr.pairwise = truncated_quadratic(L, trunc, scale)
        else:
            trunc = 2.0
            pr.pairwise = sgm_penalties(L, 0.5 if not iv else 1.0, 2.0)
        pr.pairwise_kind, pr.trunc, pr.scale = kind, trunc, scale
    want_V = bool(rng.integers(0, 2))
    knobs = {2: int(rng.integers(0, 3)), 3: int(rng.integers(0, 3)), 4: int(rng.integers(0, 3)),
             5: int(rng.integers(0, 3)), 6: int(rng.integers(0, 3)), 7: int(rng.choice([0, 2, 4, 6, 8, 12])),
             8: int(rng.integers(0, 3)), 9: int(rng.integers(0, 3)), 10: int(rng.choice([0, 4, 8])),
             11: int(rng.integers(0, 3)), 12: int(rng.integers(0, 3)), 13: int(rng.integers(0, 3)), 15: int(rng.integers(0, 3)), 16: int(rng.integers(0, 3)), 17: int(rng.integers(0, 3)), 18: int(rng.integers(0, 2)), 19: int(rng.integers(0, 2)), 20: int(rng.integers(0, 3))}
    print("case drawn medium", seed, algo, (B, H, W, L), len(dirs), K, kind, want_V, knobs, flush=True)
    f = oracle_forward(oracle, pr, threads=True)
    b = oracle_backward(oracle, pr, f.p, f.q, np.float64)
    big = max(float(np.abs(b.grad_unary).max()), float(np.abs(b.grad_pairwise).max()),
              float(np.abs(b.grad_edge_weight).max()) if b.grad_edge_weight is not None else 0.0)
    if big > 10.0:
        pr.grad_cost = (pr.grad_cost * np.float32(10.0 / big)).astype(np.float32)
    try:
        for k, v in knobs.items():
            assert mrf.mrf_tune(k, v) == 0
        full_check(oracle, pr, threads=True, want_V=want_V)
    finally:
        for k in knobs:
            mrf.mrf_tune(k, 0)
