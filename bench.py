#!/usr/bin/env python3
"""Throughput of the hot path on one MI355X.

Headline ("step"): one forward + one backward pass of ISGMR (Alg. 1 + Alg. 3) on the largest
benchmark shape, the driving-stereo one: 1 x 384 x 1248 grid, L = 192 labels, 8 directions,
K = 3, truncated-linear pairwise with a scalar weight.  Inputs are seeded and synthetic and
already resident in HBM when the timed region starts.

Prints ONE JSON line.  value = message updates per second of the headline step, where one
message update is one (node with a predecessor, direction, label, iteration): sum_r E_r * L * K
per pass, divided by the time of forward + backward.  The "configs" array holds the same
measurement for every benchmark shape and both algorithms (ISGMR and TRWP), each with the
kernels the library launched and a roofline object for its forward and its backward sweep.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

METRIC = "message updates/sec (node*label*dir*iter), ISGMR+TRWP fwd+bwd; % VALU/HBM peak"
# Peak of plain fp32 VALU issue: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions/s.
VALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9
# Dense sweep: one (lambda, mu) candidate costs the kernel INSTR_PER_PAIR vector instructions
# (1 FMA + 1 compare + 2 selects in the straight loop), counted as 5 flops (FMA = 2).  None of
# them has a packed form that applies, so the ceiling of this instruction mix is
# FLOPS_PER_PAIR / INSTR_PER_PAIR flop per lane-instruction.
FLOPS_PER_PAIR, INSTR_PER_PAIR = 5.0, 4.0
ALU_PEAK_TFLOPS = VALU_LANE_OPS_PER_S * FLOPS_PER_PAIR / INSTR_PER_PAIR / 1e12
HBM_PEAK_GBS = 8000.0
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.md")

HEADLINE = (3, "isgmr", False)
# every benchmark shape, both algorithms where the shape names both (5) or is the paper's timing
# shape (2), and the dense-table variant of the denoising shape (forward only)
ALL_RUNS = [(1, "isgmr", False), (1, "trwp", False), (2, "trwp", False), (2, "isgmr", False),
            (3, "isgmr", False), (4, "trwp", False), (4, "trwp", True), (5, "isgmr", False), (5, "trwp", False)]


def edges_per_direction(pr):
    B, H, W, L = pr.shape
    return [B * max(H - abs(dh), 0) * max(W - abs(dw), 0) for dh, dw in pr.dirs.tolist()]


def measured_traffic(version):
    """HBM bytes per launch from rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE, scaled by what the
    same counters read for a copy of known size), as tabulated in profiles/hbm_traffic.md:
    | library version | workload | kernel | bytes per launch |.  Only rows of this library
    version count: a kernel that changed since has no figure until it is measured again."""
    out = {}
    if not os.path.exists(TRAFFIC_TABLE):
        return out
    for line in open(TRAFFIC_TABLE):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) >= 4 and cells[0] == version:
            try:
                out[(cells[1], cells[2])] = float(cells[3])
            except ValueError:
                pass
    return out


def cpu_baseline(index, algo, crop):
    """The oracle as it stands, single thread, on a crop of the same recipe."""
    from mrf_inputs import make_config
    from oracle import mrf_oracle
    pr = make_config(index, crop=crop, algo=algo)
    mrf_oracle.build()
    t0 = time.perf_counter()
    f = mrf_oracle.forward(pr.algo, pr.unary, pr.pairwise, pr.dirs, pr.K, edge_weight=pr.edge_weight,
                           edge_weight_scalar=pr.edge_weight_scalar, rho=pr.rho, threads=False)
    t1 = time.perf_counter()
    mrf_oracle.backward(pr.algo, pr.shape, pr.pairwise, pr.dirs, pr.K, pr.grad_cost, f.p, f.q,
                        edge_weight=pr.edge_weight, edge_weight_scalar=pr.edge_weight_scalar, rho=pr.rho)
    t2 = time.perf_counter()
    return {
        "value": pr.message_updates() / (t2 - t0), "unit": "message updates/s", "cores": 1, "kind": "oracle",
        "sample": "same recipe (configuration %d, %s) cropped to %dx%d (L, R, K unchanged), forward %.2f s + backward %.2f s"
                  % (index, algo, crop[0], crop[1], t1 - t0, t2 - t1),
    }


def measure(index, algo, dense, steps, warmup, traffic, tune=()):
    """One benchmark shape with one algorithm: ms per forward + backward, the sweeps alone (HIP
    events the library records on its stream around its sweep launches), kernels, rooflines."""
    from mrf_inputs import make_config
    pr = make_config(index, algo=algo)
    if dense:
        # the same potentials announced as a general dense table: the O(L^2) sweep runs
        pr.pairwise_kind = 0
        pr.name += "_dense"
    return measure_problem(pr, dense, steps, warmup, traffic)


GRAPH = False      # --graph: also time the same step replayed from a captured HIP graph


def measure_problem(pr, dense, steps, warmup, traffic):
    import torch
    from gpu_harness import GpuProblem
    import paper_1910_10892_amd as mrf

    g = GpuProblem(pr, want_messages=False)
    updates = pr.message_updates()
    E = edges_per_direction(pr)
    B, H, W, L = pr.shape
    R, K = pr.R, pr.K
    # grad_pairwise is asked for only where V is a free (dense) table, as in the segmentation
    # configuration; truncated linear / quadratic V has no per-entry parameters to learn.
    # The dense variant of the denoising shape times the forward pass only.
    want_V = pr.pairwise_kind == 0 and not dense
    backward = not dense

    def step():
        g.forward()
        if backward:
            g.backward(want_V=want_V)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    ms_per_step_graph = None
    if GRAPH:
        # the library allocates nothing and never waits for the stream: the step can be captured once
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_per_step_graph = (time.perf_counter() - t0) * 1e3 / steps
        del graph

    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    mrf.mrf_set_sweep_events(ev[0], ev[1])
    fwd_ms, bwd_ms = [], []
    for _ in range(max(2, min(steps, 5))):
        g.forward()
        torch.cuda.synchronize()
        fwd_ms.append(ev[0].elapsed_time(ev[1]))
        if backward:
            g.backward(want_V=want_V)
            torch.cuda.synchronize()
            bwd_ms.append(ev[0].elapsed_time(ev[1]))
    mrf.mrf_set_sweep_events(None, None)
    fwd_sweeps_ms = sum(fwd_ms) / len(fwd_ms)
    bwd_sweeps_ms = sum(bwd_ms) / len(bwd_ms) if bwd_ms else None
    n_launch = K * (R if pr.algo == "trwp" else 1)

    # Algorithmic work.  Forward: per message update (node, direction, label, iteration) the
    # sweep reads the unary and the other directions' messages (4 B each), writes the message
    # (4 B) and p (1 B), plus q and the edge weight once per node.  Backward: p (1 B), incoming
    # gradient (4 B) and outgoing share (4 B) per label, grad theta read-modify-write once per node
    # and iteration (8 B / R per direction), q + weight + weight gradient (9 B) per node.
    window = mrf.mrf_forward_window(g.prob, g.algo)
    dirs = pr.dirs.tolist()
    opp = sum(1 for d in dirs if [-d[0], -d[1]] in dirs)
    n_in = R if pr.algo == "trwp" else (R - 1 if opp == R else R)   # label vectors read per update (iterations >= 2)
    node_dirs = sum(E) * K                                          # node-direction-iterations per pass
    # Message arrays that are still zero are part of the algorithm's initialisation, not of its
    # traffic: in the first iteration ISGMR reads the unary only, and TRWP's sweep of direction r the
    # unary and the r directions swept before it.
    def vectors_read(k, r):
        has_opp = [-dirs[r][0], -dirs[r][1]] in dirs
        if pr.algo == "trwp":
            return 1 + (r if k == 0 else R - 1)
        return 1 + (0 if k == 0 else R - 1 - (1 if has_opp else 0))
    fwd_bytes_direct = sum(E[r] * (L * (4 * vectors_read(k, r) + 5) + 5) for k in range(K) for r in range(R))
    fwd_launch, bwd_launch = mrf.mrf_last_sweep_launch(False), mrf.mrf_last_sweep_launch(True)
    presum = "mrf_isgmr_presum" in fwd_launch
    if presum:
        # ISGMR with many directions: a streaming pass per later iteration reads the unary and the R message
        # arrays once and writes one sum per pair of opposite directions; every sweep then reads one vector
        pairs_of_dirs = sum(1 for r in range(R) if [-dirs[r][0], -dirs[r][1]] not in dirs[:r])
        fwd_bytes = (sum(E[r] * (L * (4 * 1 + 5) + 5) for k in range(K) for r in range(R)) +
                     (K - 1) * 4 * B * H * W * L * (1 + R + pairs_of_dirs))
    else:
        fwd_bytes = fwd_bytes_direct
    bwd_bytes = node_dirs * (9 * L + 8 * L / R + 9)
    fwd_kernel, bwd_kernel = mrf.mrf_last_sweep_kernel(False), mrf.mrf_last_sweep_kernel(True)
    if window > 0:
        # the window sweeps evaluate 2*window-1 candidates per label instead of L: bytes, not pairs, are
        # the resource a faster machine would have to supply
        gbs = fwd_bytes / (fwd_sweeps_ms * 1e-3) / 1e9
        roof_fwd = {"kernel": fwd_kernel, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": traffic.get((pr.name, fwd_kernel)),
                    "algorithmic_bytes_per_launch": fwd_bytes / n_launch, "bytes_per_node_direction_later_iterations": L * (4 * n_in + 5) + 5,
                    "bytes_per_launch_if_every_sweep_read_all_its_sources": fwd_bytes_direct / n_launch,
                    "launches_per_pass": n_launch, "avg_launch_ms": fwd_sweeps_ms / n_launch, "window": window}
    else:
        pairs = node_dirs * L * L                       # (lambda, mu) candidates of one forward pass
        tflops = pairs * FLOPS_PER_PAIR / (fwd_sweeps_ms * 1e-3) / 1e12
        roof_fwd = {"kernel": fwd_kernel, "bound": "alu", "achieved": tflops, "peak": ALU_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": tflops / ALU_PEAK_TFLOPS, "traffic": traffic.get((pr.name, fwd_kernel)),
                    "pairs_per_launch": pairs / n_launch, "valu_instructions_per_pair": INSTR_PER_PAIR,
                    "launches_per_pass": n_launch, "avg_launch_ms": fwd_sweeps_ms / n_launch}
    roof_bwd = None
    if backward:
        gbs = bwd_bytes / (bwd_sweeps_ms * 1e-3) / 1e9
        roof_bwd = {"kernel": bwd_kernel, "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": gbs / HBM_PEAK_GBS, "traffic": traffic.get((pr.name, bwd_kernel)),
                    "algorithmic_bytes_per_launch": bwd_bytes / n_launch, "bytes_per_node_direction": 9 * L + 8 * L / R + 9,
                    "launches_per_pass": n_launch, "avg_launch_ms": bwd_sweeps_ms / n_launch}
    out = {
        "workload": pr.name, "algorithm": pr.algo, "grid": [B, H, W], "labels": L, "directions": R, "iterations": K,
        "pairwise": "dense" if pr.pairwise_kind == 0 else ["", "truncated_linear", "truncated_quadratic", "distance"][pr.pairwise_kind],
        "message_updates_per_pass": updates,
        "passes": "forward+backward" if backward else "forward",
        "gradients": (["unary", "edge_weight"] + (["pairwise"] if want_V else [])) if backward else [],
        "ms_per_step": ms_per_step, "updates_per_s": updates / (ms_per_step * 1e-3),
        "forward_sweeps_ms": fwd_sweeps_ms, "backward_sweeps_ms": bwd_sweeps_ms, "ms_per_step_graph_replay": ms_per_step_graph,
        "forward_updates_per_s": updates / (fwd_sweeps_ms * 1e-3),
        "backward_updates_per_s": updates / (bwd_sweeps_ms * 1e-3) if backward else None,
        "kernels": {"forward": fwd_launch, "backward": bwd_launch if backward else None},
        "roofline_forward": roof_fwd, "roofline_backward": roof_bwd,
    }
    del g
    torch.cuda.empty_cache()
    return out


def heads(index, algo):
    """The two heads around the path on one workload's final costs and labels: streaming kernels,
    priced against HBM with their algorithmic bytes."""
    import torch
    from mrf_inputs import make_config
    from gpu_harness import GpuProblem
    import paper_1910_10892_amd as mrf
    pr = make_config(index, algo=algo)
    g = GpuProblem(pr, want_messages=False)
    g.forward()
    B, H, W, L = pr.shape
    R = pr.R
    E = edges_per_direction(pr)
    N = B * H * W
    ws = torch.empty(max(mrf.mrf_energy_workspace_bytes(g.prob), mrf.mrf_softmin_l1_workspace_bytes()),
                     dtype=torch.uint8, device="cuda:0")
    energy = torch.empty((B,), dtype=torch.float64, device="cuda:0")
    target = torch.rand((B, H, W), device="cuda:0") * (L - 1)
    disp = torch.empty((B, H, W), device="cuda:0")
    loss = torch.empty((1,), dtype=torch.float64, device="cuda:0")
    gcost = torch.empty_like(g.cost)

    def timed(fn, reps=20):
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    t_e = timed(lambda: mrf.mrf_energy(g.prob, g.labels, energy, ws))
    t_l = timed(lambda: mrf.mrf_softmin_l1(g.cost, target, None, disp, loss, gcost, ws))
    dirs = pr.dirs.tolist()
    n_edge_dirs = sum(1 for i, d in enumerate(dirs) if [-d[0], -d[1]] not in dirs or dirs.index([-d[0], -d[1]]) > i)
    e_bytes = N * (1 + 4) + sum(E) // R * n_edge_dirs * (4 + 4)   # label, theta(x); per edge: weight, V entry
    l_bytes = N * (L * 4 * 2 + 4 * 2)
    rf = lambda b, t: {"ms": t, "bound": "hbm", "achieved": b / (t * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                       "frac": b / (t * 1e-3) / 1e9 / HBM_PEAK_GBS}
    return {"workload": pr.name, "energy": rf(e_bytes, t_e), "softmin_l1": rf(l_bytes, t_l)}


def speed_table(steps):
    """The shape of the paper's speed table (Sec. 5.3): one 256 x 512 image, 32 or 96 labels, 4, 8 or 16
    directions, both algorithms, a general (dense) pairwise table with per-edge weights, forward and
    backward with every gradient.  The paper does not state the iteration count of its timings: K = 5
    here, and the times are given per iteration."""
    from mrf_inputs import DIRS4, DIRS8, DIRS16, random_problem
    rows = []
    for L in (32, 96):
        for dirs in (DIRS4, DIRS8, DIRS16):
            for algo in ("isgmr", "trwp"):
                pr = random_problem(19101089 + L + len(dirs), algo, 1, 256, 512, L, dirs, 5)
                pr.name = "speed_table_256x512_L%d_R%d_%s" % (L, len(dirs), algo)
                m = measure_problem(pr, False, steps, 1, {})
                rows.append({"workload": pr.name, "algorithm": algo, "labels": L, "directions": len(dirs), "iterations": pr.K,
                             "forward_ms_per_iteration": m["forward_sweeps_ms"] / pr.K,
                             "backward_ms_per_iteration": m["backward_sweeps_ms"] / pr.K,
                             "updates_per_s": m["updates_per_s"], "kernels": m["kernels"],
                             "forward_frac": m["roofline_forward"]["frac"], "forward_bound": m["roofline_forward"]["bound"],
                             "backward_frac": m["roofline_backward"]["frac"]})
    return rows


def energy_protocol():
    """The protocol of the paper's energy tables (Sec. 5.1) on the synthetic stereo and denoising
    shapes: K = 1 and K = 50 iterations of both algorithms, the energy of the labelling each returns
    (Eq. energy-function, mrf_energy) and the time of the forward pass.  The tables' own numbers need
    the paper's datasets; these are the stand-ins' energies."""
    import torch
    from mrf_inputs import make_config
    from gpu_harness import GpuProblem
    import paper_1910_10892_amd as mrf
    rows = []
    for index in (2, 4):
        for algo in ("isgmr", "trwp"):
            for K in (1, 50):
                pr = make_config(index, algo=algo, K=K)
                g = GpuProblem(pr, want_messages=False)
                ws = torch.empty(mrf.mrf_energy_workspace_bytes(g.prob), dtype=torch.uint8, device="cuda:0")
                e = torch.empty((pr.shape[0],), dtype=torch.float64, device="cuda:0")
                g.forward()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                g.forward()
                torch.cuda.synchronize()
                t1 = time.perf_counter()
                mrf.mrf_energy(g.prob, g.labels, e, ws)
                rows.append({"workload": pr.name, "algorithm": algo, "iterations": K,
                             "energy": float(e.sum().item()), "forward_ms": (t1 - t0) * 1e3})
                del g
                torch.cuda.empty_cache()
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=0,
                    help="time only this benchmark configuration 1..5 (default: the headline, configuration 3, "
                         "plus every configuration in the \"configs\" array)")
    ap.add_argument("--algo", default=None, help="with --config: isgmr | trwp (default: the configuration's)")
    ap.add_argument("--dense", action="store_true",
                    help="with --config: announce the pairwise table as dense (the O(L^2) sweep runs), forward only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a 1 GiB device-to-device copy (calibration of HBM byte counters)")
    ap.add_argument("--heads", action="store_true",
                    help="also time the energy and SoftMin + L1 heads (extra \"heads\" object)")
    ap.add_argument("--energy-protocol", action="store_true",
                    help="also run K = 1 and K = 50 iterations of both algorithms on configurations 2 and 4 and "
                         "report the energy of each labelling (extra \"energy_protocol\" array)")
    ap.add_argument("--speed-table", action="store_true",
                    help="also time the shape of the paper's speed table: 256 x 512, 32 / 96 labels, 4 / 8 / 16 "
                         "directions, dense pairwise table, both algorithms (extra \"speed_table\" array)")
    ap.add_argument("--shape", default=None, metavar="ALGO:BxHxW:L:R:K[:TRUNC]",
                    help="time a shape of your own instead of a benchmark configuration: isgmr|trwp, grid, labels, 4|8|16 "
                         "directions, iterations, truncated-linear pairwise with that truncation (0 or absent: a general "
                         "dense table with all gradients); seeded random unaries and per-edge weights")
    ap.add_argument("--graph", action="store_true",
                    help="also capture each step (forward + backward) into a HIP graph and time its replay "
                         "(\"ms_per_step_graph_replay\" of every entry of \"configs\")")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE",
                    help="experiment: set a kernel-choice knob of mrf_tune (results never depend on them)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_1910_10892_amd as mrf

    global GRAPH
    GRAPH = args.graph
    mrf.load_library()      # no fallback: raises if libmrfmp.so is missing
    for kv in args.tune:
        knob, value = kv.split("=")
        mrf.mrf_tune(int(knob), int(value))
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    traffic = measured_traffic(mrf.mrf_version())

    if args.copy_probe:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        a.fill_(1.0)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            b.copy_(a)
        e1.record()
        torch.cuda.synchronize()
        copy_gbs = 10 * 2 * a.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9      # bytes read + written
        del a, b

    shape_problem = None
    if args.shape:
        from mrf_inputs import DIRS4, DIRS8, DIRS16, random_problem, truncated_linear
        f = args.shape.split(":")
        algo_s, (B_s, H_s, W_s), L_s, R_s, K_s = f[0], [int(v) for v in f[1].split("x")], int(f[2]), int(f[3]), int(f[4])
        trunc_s = float(f[5]) if len(f) > 5 else 0.0
        shape_problem = random_problem(19101089, algo_s, B_s, H_s, W_s, L_s, {4: DIRS4, 8: DIRS8, 16: DIRS16}[R_s], K_s)
        if trunc_s > 0:
            shape_problem.pairwise = truncated_linear(L_s, trunc_s, 1.0)
            shape_problem.pairwise_kind, shape_problem.trunc, shape_problem.scale = 1, trunc_s, 1.0
        shape_problem.name = "shape_" + args.shape.replace(":", "_")
    if args.config:
        from mrf_inputs import make_config
        algo = args.algo or make_config(args.config, crop=(4, 4)).algo
        head_run = (args.config, algo, args.dense)
        others = []
    else:
        head_run = HEADLINE
        others = [r for r in ALL_RUNS if r != HEADLINE]
    if shape_problem is not None:
        head = measure_problem(shape_problem, False, args.steps, args.warmup, traffic)
        others = []
    else:
        head = measure(*head_run, args.steps, args.warmup, traffic)
    configs = [head]
    for run in others:
        configs.append(measure(*run, max(2, min(args.steps, 5)), 1, traffic))

    rf, rb = head["roofline_forward"], head["roofline_backward"]
    dominant, other = (rf, rb) if (rb is None or head["forward_sweeps_ms"] >= head["backward_sweeps_ms"]) else (rb, rf)
    out = {
        "metric": METRIC,
        "value": head["updates_per_s"],
        "unit": "message updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "algorithm", "grid", "labels", "directions", "iterations", "pairwise",
                                        "message_updates_per_pass", "passes", "gradients", "kernels")},
        "roofline": dominant,
        "roofline_other": other,
        "forward_sweeps_ms": head["forward_sweeps_ms"], "backward_sweeps_ms": head["backward_sweeps_ms"],
        "library_version": mrf.mrf_version(),
        "configs": configs,
    }
    if args.copy_probe:
        out["copy_probe"] = {"what": "1 GiB device-to-device copy, bytes read + written per second", "value": copy_gbs, "unit": "GB/s"}
    if args.heads:
        out["heads"] = heads(head_run[0], head_run[1])
    if args.energy_protocol:
        out["energy_protocol"] = energy_protocol()
    if args.speed_table:
        out["speed_table"] = speed_table(max(2, min(args.steps, 3)))
    if not args.no_cpu_baseline and shape_problem is None:
        crops = {1: (32, 48), 2: (128, 256), 3: (56, 144), 4: (24, 32), 5: (256, 256)}
        out["cpu_baseline"] = cpu_baseline(head_run[0], head_run[1], crops[head_run[0]])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
