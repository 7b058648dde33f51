"""Plain fp64 definitions of the two heads around the message-passing path -- TEST
INFRASTRUCTURE ONLY (tests, the smoke check and the bench's CPU leg may import it; the
product never does).  numpy, no blocking, no shortcuts.

energy()      the pairwise MRF energy of a labelling (Sec. 3.1, Eq. energy-function)
softmin_l1()  disparity confidences by SoftMin of the final costs, their expectation as the
              regressed disparity, and the standard L1 loss against real-valued ground truth
              (Appendix, Eqs. supp-isgmr-confidence and supp-isgmr-regression and the sentence
              on the loss), with the derivative of the loss with respect to the costs written
              out by the chain rule

Reading taken where the paper leaves a choice: the edge set of Eq. energy-function holds every
undirected neighbour pair once.  Directions come in opposite pairs that describe the same
edges; the energy takes the edges of the first direction of each pair in the order of
`dirs` (and of every direction that has no opposite), with that direction's weights.
"""
from __future__ import annotations

import numpy as np


def energy_directions(dirs):
    """Indices of the directions whose edges enter the energy (see the module docstring)."""
    d = [tuple(int(v) for v in row) for row in np.asarray(dirs).reshape(-1, 2)]
    keep = []
    for r, (dh, dw) in enumerate(d):
        opp = d.index((-dh, -dw)) if (-dh, -dw) in d else -1
        if opp < 0 or r < opp:
            keep.append(r)
    return keep


def energy(unary, pairwise, dirs, labels, edge_weight=None, edge_weight_scalar=1.0, pairwise_edge=None):
    """E(x | Theta) per batch image, float64 [B].  unary [B,H,W,L], pairwise V[mu at i-r][lambda
    at i], labels [B,H,W] integer, edge_weight [R,B,H,W] stored at the destination node i.
    pairwise_edge [R,B,H,W,L,L], if given, holds theta_{i-r,i}(mu,lambda) per edge (stored at the
    destination node i like the weights) and takes the place of edge_weight * pairwise."""
    unary = np.asarray(unary, np.float64)
    V = None if pairwise is None else np.asarray(pairwise, np.float64)
    x = np.asarray(labels).astype(np.int64)
    B, H, W, _ = unary.shape
    dirs = np.asarray(dirs).reshape(-1, 2)
    out = np.zeros(B, np.float64)
    for b in range(B):
        e = 0.0
        for y in range(H):
            for xx in range(W):
                e += unary[b, y, xx, x[b, y, xx]]
        for r in energy_directions(dirs):
            dh, dw = int(dirs[r, 0]), int(dirs[r, 1])
            for y in range(H):
                for xx in range(W):
                    ys, xs = y - dh, xx - dw
                    if 0 <= ys < H and 0 <= xs < W:
                        if pairwise_edge is not None:
                            e += float(pairwise_edge[r, b, y, xx, x[b, ys, xs], x[b, y, xx]])
                            continue
                        w = float(edge_weight[r, b, y, xx]) if edge_weight is not None else float(edge_weight_scalar)
                        e += w * V[x[b, ys, xs], x[b, y, xx]]
        out[b] = e
    return out


def softmin_l1(cost, target, mask=None, beta=0.0):
    """cost [..., L], target [...] (real-valued disparities), mask [...] (non-zero = pixel
    counts) or None.  Returns (disparity [...], loss scalar, grad_cost [..., L]), all float64.

    f = exp(-c) / sum exp(-c) over labels; d = sum_lambda lambda f(lambda);
    loss = mean over counted pixels of l(d - g), with l(x) = |x| (standard L1, beta = 0) or the
    smooth L1 the paper names beside it (beta > 0): l(x) = x^2 / (2 beta) for |x| < beta, else
    |x| - beta / 2 (the usual definition; the paper gives none, beta = 1 is the common choice);
    d loss / d c(lambda) = l'(d - g) / n * (-f(lambda)) * (lambda - d)."""
    c = np.asarray(cost, np.float64)
    g = np.asarray(target, np.float64)
    L = c.shape[-1]
    z = -(c - c.min(axis=-1, keepdims=True))          # the shift cancels in the ratio
    e = np.exp(z)
    f = e / e.sum(axis=-1, keepdims=True)
    lam = np.arange(L, dtype=np.float64)
    d = (f * lam).sum(axis=-1)
    m = np.ones(g.shape, bool) if mask is None else (np.asarray(mask) != 0)
    n = int(m.sum())
    diff = d - g
    if beta > 0.0:
        small = np.abs(diff) < beta
        per_pixel = np.where(small, diff * diff / (2.0 * beta), np.abs(diff) - beta / 2.0)
        slope = np.where(small, diff / beta, np.sign(diff))
    else:
        per_pixel = np.abs(diff)
        slope = np.sign(diff)
    loss = float(per_pixel[m].sum() / n) if n > 0 else 0.0
    s = np.where(m, slope, 0.0) / max(n, 1)
    grad = s[..., None] * (-f) * (lam - d[..., None])
    return d, loss, grad
