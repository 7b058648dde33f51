"""Seeded synthetic MRF problems: shapes and value distributions only.

This module serves both the CPU oracle's tests and the GPU library's tests / bench.
It holds no arithmetic of the message-passing method: it only draws unaries, a
pairwise function, edge weights and an upstream gradient.

The five named configurations stand in for the paper's workloads (Sec. 5.1 stereo and
denoising energies, Sec. 5.2 21-class segmentation, Sec. 5.3 timing at 256x512); none of
those datasets is used or reproduced.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

SEED_BASE = 19101089200

# (dh, dw); index order is also the order TRWP sweeps the directions in
DIRS4 = [(0, 1), (0, -1), (1, 0), (-1, 0)]
DIRS8 = DIRS4 + [(1, 1), (-1, -1), (1, -1), (-1, 1)]
DIRS16 = DIRS8 + [(1, 2), (-1, -2), (2, 1), (-2, -1), (1, -2), (-1, 2), (2, -1), (-2, 1)]

KIND_DENSE, KIND_TRUNC_LINEAR, KIND_TRUNC_QUADRATIC, KIND_DISTANCE = 0, 1, 2, 3


@dataclass
class Problem:
    name: str
    algo: str                     # "isgmr" | "trwp"
    unary: np.ndarray             # [B,H,W,L] float32
    pairwise: np.ndarray          # [L,L] float32, V[mu_source][lambda_dest]
    dirs: np.ndarray              # [R,2] int32
    K: int
    edge_weight: Optional[np.ndarray] = None   # [R,B,H,W] float32 or None
    edge_weight_scalar: float = 1.0
    rho: Optional[np.ndarray] = None           # [R] float32 (TRWP)
    grad_cost: Optional[np.ndarray] = None     # [B,H,W,L] float32
    pairwise_kind: int = KIND_DENSE
    trunc: float = 0.0
    scale: float = 1.0
    meta: dict = field(default_factory=dict)
    rho_edge: Optional[np.ndarray] = None      # [R,B,H,W] float32 (TRWP): rho per directed edge, or None
    pairwise_edge: Optional[np.ndarray] = None # [R,B,H,W,L,L] float32: pairwise potentials per edge, or None

    @property
    def shape(self):
        return tuple(self.unary.shape)

    @property
    def R(self):
        return int(self.dirs.shape[0])

    def message_updates(self) -> int:
        """sum_r E_r * L * K, the unit of the throughput metric."""
        B, H, W, L = self.shape
        tot = 0
        for dh, dw in self.dirs.tolist():
            tot += B * max(H - abs(dh), 0) * max(W - abs(dw), 0)
        return tot * L * self.K


def sgm_penalties(L: int, p1: float, p2: float) -> np.ndarray:
    """The three-penalty pairwise function of SGM (Eq. vsgm): 0 on the diagonal, p1 for label
    distance 1, p2 from distance 2 on."""
    a = np.arange(L)
    d = np.abs(a[:, None] - a[None, :])
    return np.where(d == 0, 0.0, np.where(d == 1, p1, p2)).astype(np.float32)


def truncated_linear(L: int, trunc: float, scale: float = 1.0) -> np.ndarray:
    a = np.arange(L, dtype=np.float32)
    d = np.abs(a[:, None] - a[None, :])
    return (np.minimum(d, np.float32(trunc)) * np.float32(scale)).astype(np.float32)


def truncated_quadratic(L: int, trunc: float, scale: float = 1.0) -> np.ndarray:
    a = np.arange(L, dtype=np.float32)
    d = (a[:, None] - a[None, :]) ** 2
    return (np.minimum(d, np.float32(trunc)) * np.float32(scale)).astype(np.float32)


def mirrored_edge_weights(rng, B, H, W, dirs, draw) -> np.ndarray:
    """One weight per undirected edge, stored at the destination node of both directed
    copies: w[r][i] = w[r-][i-r].  Entries of first nodes are left at 0 (never read)."""
    dirs = [tuple(d) for d in np.asarray(dirs).tolist()]
    R = len(dirs)
    w = np.zeros((R, B, H, W), np.float32)
    done = set()
    for r, (dh, dw) in enumerate(dirs):
        if r in done:
            continue
        hh, ww = H - abs(dh), W - abs(dw)
        if hh <= 0 or ww <= 0:
            continue
        vals = draw(rng, (B, hh, ww)).astype(np.float32)
        # destination nodes of direction r: y in [max(dh,0), H+min(dh,0)), same for x
        ys, xs = max(dh, 0), max(dw, 0)
        w[r, :, ys:ys + hh, xs:xs + ww] = vals
        opp = (-dh, -dw)
        if opp in dirs:
            ro = dirs.index(opp)
            yo, xo = max(-dh, 0), max(-dw, 0)
            w[ro, :, yo:yo + hh, xo:xo + ww] = vals
            done.add(ro)
        done.add(r)
    return w


def _contrast_weights(rng, B, H, W, dirs):
    return mirrored_edge_weights(
        rng, B, H, W, dirs,
        lambda g, shp: np.exp(-np.abs(g.normal(0.0, 0.1, shp)) / 0.1))


def _rectangles_map(rng, H, W, n_rect, lo, hi, base):
    img = np.full((H, W), base, np.float64)
    for _ in range(n_rect):
        y0 = int(rng.integers(0, H)); x0 = int(rng.integers(0, W))
        hh = int(rng.integers(max(H // 16, 1), max(H // 3, 2)))
        ww = int(rng.integers(max(W // 16, 1), max(W // 3, 2)))
        img[y0:y0 + hh, x0:x0 + ww] = rng.uniform(lo, hi)
    return img


def make_config(index: int, crop: Optional[tuple] = None, K: Optional[int] = None,
                algo: Optional[str] = None) -> Problem:
    """index 1..5 = the five benchmark configurations; crop=(H,W) shrinks the grid (the
    recipe is unchanged), K overrides the iteration count, algo picks the algorithm for
    configuration 5 (which names both)."""
    rng = np.random.default_rng(SEED_BASE + index)
    if index == 1:
        H, W = crop or (32, 48)
        B, L, dirs, k = 1, 16, DIRS4, 5
        unary = rng.random((B, H, W, L), dtype=np.float32)
        V = truncated_linear(L, 4.0)
        w = mirrored_edge_weights(rng, B, H, W, dirs, lambda g, s: g.uniform(0.5, 1.5, s))
        a = algo or "isgmr"
        prob = Problem("cfg1_%s_32x48_L16" % a, a, unary, V, np.array(dirs, np.int32), k,
                       edge_weight=w, pairwise_kind=KIND_TRUNC_LINEAR, trunc=4.0, scale=1.0)
    elif index == 2:
        H, W = crop or (256, 512)
        B, L, dirs, k = 1, 96, DIRS4, 5
        disp = np.rint(_rectangles_map(rng, H, W, 12, 0, L - 1, float(rng.integers(0, L)))).astype(np.int64)
        disp = np.clip(disp, 0, L - 1)
        unary = np.abs(rng.normal(0.0, 1.0, (B, H, W, L))).astype(np.float32)
        planted = (0.05 * np.abs(rng.normal(0.0, 1.0, (B, H, W)))).astype(np.float32)
        bb, yy, xx = np.meshgrid(np.arange(B), np.arange(H), np.arange(W), indexing="ij")
        unary[bb, yy, xx, disp[None].repeat(B, 0)] = planted
        V = truncated_linear(L, 8.0)
        w = _contrast_weights(rng, B, H, W, dirs)
        a = algo or "trwp"
        prob = Problem("cfg2_%s_stereo_256x512_L96" % a, a, unary, V, np.array(dirs, np.int32), k,
                       edge_weight=w, rho=np.full(4, 0.25, np.float32),
                       pairwise_kind=KIND_TRUNC_LINEAR, trunc=8.0, scale=1.0)
    elif index == 3:
        H, W = crop or (384, 1248)
        B, L, dirs, k = 1, 192, DIRS8, 3
        unary = rng.random((B, H, W, L), dtype=np.float32)
        V = truncated_linear(L, 2.0)
        a = algo or "isgmr"
        prob = Problem("cfg3_%s_driving_384x1248_L192" % a, a, unary, V, np.array(dirs, np.int32), k,
                       edge_weight=None, edge_weight_scalar=0.5,
                       pairwise_kind=KIND_TRUNC_LINEAR, trunc=2.0, scale=1.0)
    elif index == 4:
        H, W = crop or (256, 256)
        B, L, dirs, k = 1, 256, DIRS4, 10
        ramp = np.linspace(40.0, 200.0, W)[None, :].repeat(H, 0)
        rect = _rectangles_map(rng, H, W, 8, 0.0, 255.0, -1.0)
        img = np.where(rect >= 0, rect, ramp)
        noisy = np.clip(img + rng.normal(0.0, 20.0, (H, W)), 0.0, 255.0)
        lab = np.arange(L, dtype=np.float64)
        unary = (((lab[None, None, :] - noisy[:, :, None]) ** 2) / 255.0 ** 2).astype(np.float32)[None]
        scale = np.float32(1.0 / 255.0 ** 2)
        V = truncated_quadratic(L, 200.0, scale)
        a = algo or "trwp"
        prob = Problem("cfg4_%s_denoise_256x256_L256" % a, a, np.ascontiguousarray(unary), V,
                       np.array(dirs, np.int32), k, edge_weight=None, edge_weight_scalar=1.0,
                       rho=np.full(4, 0.5, np.float32),
                       pairwise_kind=KIND_TRUNC_QUADRATIC, trunc=200.0, scale=float(scale))
    elif index == 5:
        H, W = crop or (512, 512)
        B, L, dirs, k = 4, 21, DIRS4, 5
        logits = rng.normal(0.0, 2.0, (B, H, W, L))
        mx = logits.max(-1, keepdims=True)
        lse = mx + np.log(np.exp(logits - mx).sum(-1, keepdims=True))
        unary = (-(logits - lse)).astype(np.float32)
        A = rng.random((L, L))
        V = ((A + A.T) / 2.0)
        np.fill_diagonal(V, 0.0)
        V = V.astype(np.float32)
        w = _contrast_weights(rng, B, H, W, dirs)
        a = algo or "isgmr"
        prob = Problem("cfg5_%s_segment_4x512x512_L21" % a, a, unary, V, np.array(dirs, np.int32), k,
                       edge_weight=w, rho=np.full(4, 0.5, np.float32), pairwise_kind=KIND_DENSE)
    else:
        raise ValueError("config index must be 1..5")
    if K is not None:
        prob.K = int(K)
    if prob.algo == "trwp" and prob.rho is None:
        prob.rho = np.full(prob.R, 0.5, np.float32)
    prob.grad_cost = rng.normal(0.0, 1.0, prob.unary.shape).astype(np.float32)
    prob.meta = {"config": index, "crop": crop}
    return prob


def random_problem(seed: int, algo: str, B: int, H: int, W: int, L: int, dirs, K: int,
                   integer_valued: bool = False, per_edge: bool = True,
                   symmetric: bool = True, rho=None) -> Problem:
    """Small random problem for unit tests.  integer_valued draws small integers so that
    ties are frequent (exercises the lowest-index tie-break)."""
    rng = np.random.default_rng(seed)
    dirs = np.array(dirs, np.int32).reshape(-1, 2)
    R = dirs.shape[0]
    if integer_valued:
        unary = rng.integers(0, 4, (B, H, W, L)).astype(np.float32)
        V = rng.integers(0, 3, (L, L)).astype(np.float32)
        draw = lambda g, s: g.integers(1, 3, s).astype(np.float64)
    else:
        unary = rng.random((B, H, W, L), dtype=np.float32)
        V = rng.random((L, L), dtype=np.float32)
        draw = lambda g, s: g.uniform(0.5, 1.5, s)
    if symmetric:
        V = ((V + V.T) / 2).astype(np.float32)
        if integer_valued:
            V = np.floor(V).astype(np.float32)
    w = mirrored_edge_weights(rng, B, H, W, dirs, draw) if per_edge else None
    if rho is None:
        rho = np.full(R, 0.5, np.float32)
    prob = Problem("random_%d" % seed, algo, unary, V, dirs, K, edge_weight=w,
                   edge_weight_scalar=0.75, rho=np.broadcast_to(np.asarray(rho, np.float32), (R,)).copy())
    prob.grad_cost = rng.normal(0.0, 1.0, unary.shape).astype(np.float32)
    return prob
