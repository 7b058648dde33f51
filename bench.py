#!/usr/bin/env python3
"""Throughput of the hot path on one MI355X.

A "step" is one forward + one backward pass of TRWP (Alg. 2 + Alg. 4) on the
stereo-shaped configuration: 1 x 256 x 512 grid, L = 96 labels, 4 directions, K = 5,
rho = 0.25, truncated-linear pairwise (the shape of the paper's timing tables, Sec. 5.3).
Inputs are seeded and synthetic and already resident in HBM when the timed region starts.

Prints ONE JSON line.  value = message updates per second, where one message update is
one (node with a predecessor, direction, label, iteration): sum_r E_r * L * K per pass,
divided by the time of forward + backward.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

# Peak of plain fp32 VALU issue: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions/s.
VALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9
# Dense sweep: one (lambda, mu) candidate = 1 FMA + 1 compare + 2 selects = 4 VALU
# instructions, counted as 5 flops (FMA = 2).  None of them has a packed form that applies,
# so the ceiling of this instruction mix is 5/4 flop per lane-instruction.
FLOPS_PER_PAIR, INSTR_PER_PAIR = 5.0, 4.0
ALU_PEAK_TFLOPS = VALU_LANE_OPS_PER_S * FLOPS_PER_PAIR / INSTR_PER_PAIR / 1e12
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), scaled by what
# the same counters read for a copy of known size; filled in from profiles/*.md, keyed by
# (workload, kernel).  None where not measured.
MEASURED_TRAFFIC = {
    # profiles/cfg2_trwp_stereo_kernels.md (backward: average over the 20 launches of a pass)
    ("cfg2_trwp_stereo_256x512_L96", "mrf_fwd_sweep_window_duo"): 251.8e6,
    ("cfg2_trwp_stereo_256x512_L96", "mrf_bwd_sweep_chain"): 283.1e6,
}


def edges_per_direction(pr):
    B, H, W, L = pr.shape
    return [B * max(H - abs(dh), 0) * max(W - abs(dw), 0) for dh, dw in pr.dirs.tolist()]


def cpu_baseline(index, algo):
    """The oracle as it stands, single thread, on a crop of the same recipe."""
    import numpy as np
    from mrf_inputs import make_config
    from oracle import mrf_oracle
    crop = (128, 256)
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
        "sample": "same recipe cropped to %dx%d (L, R, K, rho unchanged), forward %.2f s + backward %.2f s"
                  % (crop[0], crop[1], t1 - t0, t2 - t1),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (default: 2, the metric's)")
    ap.add_argument("--algo", default=None, help="isgmr | trwp (default: the configuration's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a 1 GiB device-to-device copy (calibration of HBM byte counters)")
    ap.add_argument("--tune-mch", type=int, default=0, help="experiment: source labels per wavefront (0 = heuristic)")
    ap.add_argument("--heads", action="store_true",
                    help="also time the energy and SoftMin + L1 heads on the same workload (extra \"heads\" object)")
    ap.add_argument("--tune", action="append", default=[], metavar="KNOB=VALUE",
                    help="experiment: set a kernel-choice knob of mrf_tune (results never depend on them)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from mrf_inputs import make_config
    from gpu_harness import GpuProblem
    import paper_1910_10892_amd as mrf

    mrf.load_library()      # no fallback: raises if libmrfmp.so is missing
    if args.tune_mch:
        mrf.mrf_tune(0, args.tune_mch)
    for kv in args.tune:
        knob, value = kv.split("=")
        mrf.mrf_tune(int(knob), int(value))
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    pr = make_config(args.config, algo=args.algo)
    g = GpuProblem(pr, want_messages=False)
    updates = pr.message_updates()
    E = edges_per_direction(pr)
    B, H, W, L = pr.shape
    R, K = pr.R, pr.K

    # grad_pairwise is asked for only where V is a free (dense) table, as in the segmentation
    # configuration; truncated linear / quadratic V has no per-entry parameters to learn
    want_V = pr.pairwise_kind == 0

    def step():
        g.forward()
        g.backward(want_V=want_V)

    if args.copy_probe:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        a.fill_(1.0)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    # per-kernel time of the scanline sweeps, measured with HIP events that the library
    # records on its own stream around its sweep launches
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    for e in ev:
        e.record()
    torch.cuda.synchronize()
    mrf.mrf_set_sweep_events(ev[0], ev[1])
    fwd_ms, bwd_ms = [], []
    for _ in range(max(3, min(args.steps, 10))):
        g.forward()
        torch.cuda.synchronize()
        fwd_ms.append(ev[0].elapsed_time(ev[1]))
        g.backward(want_V=want_V)
        torch.cuda.synchronize()
        bwd_ms.append(ev[0].elapsed_time(ev[1]))
    mrf.mrf_set_sweep_events(None, None)
    fwd_sweeps_ms = sum(fwd_ms) / len(fwd_ms)
    bwd_sweeps_ms = sum(bwd_ms) / len(bwd_ms)
    n_fwd_launch = K * (R if pr.algo == "trwp" else 1)
    n_bwd_launch = n_fwd_launch

    # Algorithmic work.  Forward: per message update (node, direction, label, iteration) the
    # sweep reads the unary and the other directions' messages (4 B each), writes the message
    # (4 B) and p (1 B), plus q and the edge weight once per node.  Backward: p (1 B), incoming
    # gradient (4 B) and outgoing share (4 B) per label, grad theta read-modify-write once per node
    # and iteration (8 B / R per direction), q + weight + weight gradient (9 B) per node.
    window = mrf.mrf_forward_window(g.prob, g.algo)
    opp = sum(1 for d in pr.dirs.tolist() if [-d[0], -d[1]] in pr.dirs.tolist())
    n_in = R if pr.algo == "trwp" else (R - 1 if opp == R else R)   # label vectors read per update
    fwd_bytes = sum(E) * K * (L * (4 * n_in + 5) + 5)
    bwd_bytes = sum(E) * K * (9 * L + 8 * L / R + 9)
    fwd_gbs = fwd_bytes / (fwd_sweeps_ms * 1e-3) / 1e9
    bwd_gbs = bwd_bytes / (bwd_sweeps_ms * 1e-3) / 1e9
    traffic = lambda k: MEASURED_TRAFFIC.get((pr.name, k))
    # which sweep layouts the library's launch-size rules picked for this workload
    fwd_kernel = mrf.mrf_last_sweep_kernel(False)
    bwd_kernel = mrf.mrf_last_sweep_kernel(True)
    if window > 0:
        # the window sweeps evaluate 2*window-1 candidates per label instead of L: bytes, not pairs, are
        # the resource a faster machine would have to supply
        roof_fwd = {"kernel": fwd_kernel, "bound": "hbm", "achieved": fwd_gbs, "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": fwd_gbs / HBM_PEAK_GBS, "traffic": traffic(fwd_kernel),
                    "launches_per_step": n_fwd_launch, "avg_launch_ms": fwd_sweeps_ms / n_fwd_launch,
                    "window": window}
    else:
        pairs = sum(E) * L * L * K                      # (lambda, mu) candidates of one forward pass
        fwd_tflops = pairs * FLOPS_PER_PAIR / (fwd_sweeps_ms * 1e-3) / 1e12
        roof_fwd = {"kernel": fwd_kernel, "bound": "alu", "achieved": fwd_tflops, "peak": ALU_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": fwd_tflops / ALU_PEAK_TFLOPS, "traffic": traffic(fwd_kernel),
                    "launches_per_step": n_fwd_launch, "avg_launch_ms": fwd_sweeps_ms / n_fwd_launch}
    roof_bwd = {"kernel": bwd_kernel, "bound": "hbm", "achieved": bwd_gbs, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": bwd_gbs / HBM_PEAK_GBS, "traffic": traffic(bwd_kernel),
                "launches_per_step": n_bwd_launch, "avg_launch_ms": bwd_sweeps_ms / n_bwd_launch}
    dominant, other = (roof_fwd, roof_bwd) if fwd_sweeps_ms >= bwd_sweeps_ms else (roof_bwd, roof_fwd)

    out = {
        "metric": "message updates/sec (node*label*dir*iter), %s fwd+bwd" % pr.algo.upper(),
        "value": updates / (ms_per_step * 1e-3),
        "unit": "message updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": pr.name, "algorithm": pr.algo, "grid": [B, H, W], "labels": L, "directions": R,
                   "iterations": K, "pairwise": ["dense", "truncated_linear", "truncated_quadratic"][pr.pairwise_kind],
                   "message_updates_per_pass": updates,
                   "gradients": ["unary", "edge_weight"] + (["pairwise"] if want_V else [])},
        "roofline": dominant,
        "roofline_other": other,
        "forward_sweeps_ms": fwd_sweeps_ms, "backward_sweeps_ms": bwd_sweeps_ms,
        "forward_updates_per_s": updates / (fwd_sweeps_ms * 1e-3),
        "backward_updates_per_s": updates / (bwd_sweeps_ms * 1e-3),
    }
    if args.heads:
        # the two heads around the path, on this workload's final costs and labels: streaming kernels,
        # priced against HBM with their algorithmic bytes
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
        n_edge_dirs = sum(1 for i, d in enumerate(pr.dirs.tolist())
                          if [-d[0], -d[1]] not in pr.dirs.tolist() or pr.dirs.tolist().index([-d[0], -d[1]]) > i)
        e_bytes = N * (1 + 4) + sum(E[i] for i in range(R) if i < R) // R * n_edge_dirs * (4 + 4)   # label, theta(x), per edge: weight, V entry
        l_bytes = N * (L * 4 * 2 + 4 * 2)
        out["heads"] = {
            "energy": {"ms": t_e, "bound": "hbm", "achieved": e_bytes / (t_e * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": e_bytes / (t_e * 1e-3) / 1e9 / HBM_PEAK_GBS},
            "softmin_l1": {"ms": t_l, "bound": "hbm", "achieved": l_bytes / (t_l * 1e-3) / 1e9, "peak": HBM_PEAK_GBS,
                           "unit": "GB/s", "frac": l_bytes / (t_l * 1e-3) / 1e9 / HBM_PEAK_GBS},
        }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.config, pr.algo)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
