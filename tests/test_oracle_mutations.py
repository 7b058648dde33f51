"""Do the pins of the oracle bite?  Each case plants one plausible mistake in a temporary copy of
the oracle's C source (a dropped exclusion, a transposed table, a wrong order, a wrong tie-break
...), builds that copy and runs the pin tests against it in a child process: at least one pin has
to fail.  A mistake that survives means the pins leave that part of the algorithm unchecked.
CPU only; the repository's own oracle files are never touched."""
import concurrent.futures
import os
import shutil
import subprocess
import sys
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["test_oracle_bruteforce.py", "test_oracle_gradients.py", "test_oracle_invariants.py",
             "test_oracle_rho_edge.py", "test_oracle_pairwise_edge.py", "test_oracle_sgm.py"]

# name, file, text as it stands, text with the mistake
MUTATIONS = [
    ("isgmr_forward_keeps_opposite_direction", "mrf_oracle_impl.h",
     "if (d != r && d != rm) a = a + m[((size_t)d * N + j) * L + mu];",
     "if (d != r) a = a + m[((size_t)d * N + j) * L + mu];"),
    ("isgmr_forward_reads_fresh_messages", "mrf_oracle_impl.h",
     "if (d != r && d != rm) a = a + m[((size_t)d * N + j) * L + mu];",
     "if (d != r && d != rm) a = a + mhat[((size_t)d * N + j) * L + mu];"),
    ("isgmr_forward_own_message_from_last_iteration", "mrf_oracle_impl.h",
     "a = a + mhat[((size_t)r * N + j) * L + mu];",
     "a = a + m[((size_t)r * N + j) * L + mu];"),
    ("trwp_rho_also_on_opposite_message", "mrf_oracle_impl.h",
     "if (rm >= 0) a = a - m[((size_t)rm * N + j) * L + mu];",
     "if (rm >= 0) a = a - rho[r] * m[((size_t)rm * N + j) * L + mu];"),
    ("trwp_sum_skips_own_direction", "mrf_oracle_impl.h",
     "for (int d = 0; d < R; ++d) s = s + m[((size_t)d * N + j) * L + mu];",
     "for (int d = 0; d < R; ++d) if (d != r) s = s + m[((size_t)d * N + j) * L + mu];"),
    ("pairwise_table_transposed", "mrf_oracle_impl.h",
     ": REAL_FMA(wgt, V[(size_t)mu * L + lam], h[mu]);",
     ": REAL_FMA(wgt, V[(size_t)lam * L + mu], h[mu]);"),
    ("argmin_over_mu_takes_highest_on_ties", "mrf_oracle_impl.h",
     "if (delta < best) { best = delta; arg = mu; }",
     "if (delta <= best) { best = delta; arg = mu; }"),
    ("argmin_over_lambda_takes_highest_on_ties", "mrf_oracle_impl.h",
     "if (out[lam] < out[q]) q = lam;",
     "if (out[lam] <= out[q]) q = lam;"),
    ("no_reparametrisation", "mrf_oracle_impl.h",
     "for (int lam = 0; lam < L; ++lam) out[lam] = out[lam] - mn;",
     "(void)mn;"),
    ("aggregation_without_unary", "mrf_oracle_impl.h",
     "REAL c = unary[i * L + lam];\n            for (int d = 0; d < g->R; ++d) c = c + m[((size_t)d * N + i) * L + lam];",
     "REAL c = (REAL)0;\n            for (int d = 0; d < g->R; ++d) c = c + m[((size_t)d * N + i) * L + lam];"),
    ("backward_without_norm_step", "mrf_oracle_impl.h",
     "g[qstar] = g[qstar] - tot;", ";"),
    ("isgmr_backward_accumulates_instead_of_handing_over", "mrf_oracle_impl.h",
     "memcpy(Ghat, G, sizeof(REAL) * (size_t)R * NL);",
     "for (size_t z = 0; z < (size_t)R * NL; ++z) Ghat[z] += G[z];"),
    ("isgmr_backward_feeds_opposite_direction", "mrf_oracle_impl.h",
     "if (d != r && d != rm)\n                                G[((size_t)d * N + j) * L + mu]",
     "if (d != r)\n                                G[((size_t)d * N + j) * L + mu]"),
    ("trwp_backward_in_forward_direction_order", "mrf_oracle_impl.h",
     "for (int r = R - 1; r >= 0; --r) {       /* reverse of the forward direction order */",
     "for (int r = 0; r < R; ++r) {"),
    ("trwp_backward_opposite_term_scaled_by_rho", "mrf_oracle_impl.h",
     "G[((size_t)rm * N + j) * L + mu] = G[((size_t)rm * N + j) * L + mu] - gl[lam];",
     "G[((size_t)rm * N + j) * L + mu] = G[((size_t)rm * N + j) * L + mu] - sg;"),
    ("trwp_backward_keeps_consumed_gradient", "mrf_oracle_impl.h",
     "memset(G + (size_t)r * NL, 0, sizeof(REAL) * NL);            /* zero-out */", ";"),
    ("edge_weight_gradient_offset", "mrf_oracle_impl.h",
     "REAL acc = (REAL)0;\n        for (int lam = 0; lam < L; ++lam) acc = acc + g[lam] * V[(size_t)pidx[lam] * L + lam];",
     "REAL acc = (REAL)0;\n        for (int lam = 0; lam < L; ++lam) acc = acc + g[lam] * V[(size_t)lam * L + pidx[lam]];"),
    ("pairwise_gradient_without_edge_weight", "mrf_oracle_impl.h",
     "gV[(size_t)pidx[lam] * L + lam] = gV[(size_t)pidx[lam] * L + lam] + wgt * g[lam];",
     "gV[(size_t)pidx[lam] * L + lam] = gV[(size_t)pidx[lam] * L + lam] + g[lam];"),
    ("standard_sgm_adds_the_previous_nodes_unary", "mrf_oracle_impl.h",
     "for (int lam = 0; lam < L; ++lam) t[lam] = unary[i * L + lam] + t[lam];",
     "for (int lam = 0; lam < L; ++lam) t[lam] = unary[j * L + lam] + t[lam];"),
    ("standard_sgm_first_node_without_unary", "mrf_oracle_impl.h",
     "for (int lam = 0; lam < L; ++lam) m[((size_t)r * N + j) * L + lam] = unary[j * L + lam];",
     "for (int lam = 0; lam < L; ++lam) m[((size_t)r * N + j) * L + lam] = (REAL)0;"),
    ("standard_sgm_cost_with_extra_unary", "mrf_oracle_impl.h",
     "REAL c = (REAL)0;\n            for (int d = 0; d < R; ++d) c = c + m[((size_t)d * N + i) * L + lam];\n            cost[i * L + lam] = c;",
     "REAL c = unary[i * L + lam];\n            for (int d = 0; d < R; ++d) c = c + m[((size_t)d * N + i) * L + lam];\n            cost[i * L + lam] = c;"),
    ("first_nodes_by_wrong_neighbour", "mrf_oracle.c",
     "if (!in_grid(g, y - g->dh[r], x - g->dw[r])) {",
     "if (!in_grid(g, y - g->dw[r], x - g->dh[r])) {"),
]


def _run_pins_on(name, fname, old, new):
    tmp = tempfile.mkdtemp(prefix="mrf_mut_%s_" % name)
    try:
        odir = os.path.join(tmp, "oracle")
        os.makedirs(odir)
        for f in os.listdir(os.path.join(ROOT, "oracle")):
            if f.endswith((".c", ".h", ".py")):
                shutil.copy(os.path.join(ROOT, "oracle", f), odir)
        path = os.path.join(odir, fname)
        text = open(path).read()
        if text.count(old) < 1:
            return name, "pattern not found"
        open(path, "w").write(text.replace(old, new))
        chk = subprocess.run(["gcc", "-std=c11", "-fsyntax-only", os.path.join(odir, "mrf_oracle.c")],
                             capture_output=True, text=True)
        if chk.returncode != 0:
            return name, "patched source does not compile:\n" + chk.stderr[-400:]
        env = dict(os.environ, MRF_ORACLE_UNDER_TEST=tmp, OMP_NUM_THREADS="1")
        files = [os.path.join(ROOT, "tests", f) for f in PIN_FILES if os.path.exists(os.path.join(ROOT, "tests", f))]
        res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files],
                             cwd=ROOT, env=env, capture_output=True, text=True, timeout=600)
        return name, ("caught" if res.returncode == 1 else
                      ("survived" if res.returncode == 0 else "pytest error:\n" + (res.stdout + res.stderr)[-800:]))
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def test_every_planted_mistake_is_caught_by_a_pin():
    with concurrent.futures.ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda m: _run_pins_on(*m), MUTATIONS))
    bad = [(n, r) for n, r in results if r != "caught"]
    assert not bad, "planted mistakes that no pin caught (or that could not be planted): %s" % bad


def test_the_unpatched_copy_passes():
    """The harness itself: an unchanged copy must pass the pins (so 'caught' means the mistake,
    not the copying)."""
    name, res = _run_pins_on("identity", "mrf_oracle.c", "static size_t grid_nodes", "static size_t grid_nodes")
    assert res == "survived", res
