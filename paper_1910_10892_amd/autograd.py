"""torch.autograd wrapper around the C-ABI entry points, for end-to-end learning as in Sec. 5.2
of the paper: the final costs c of ISGMR / TRWP as a differentiable function of the unary
potentials, the edge weights and the pairwise function.

Marshalling only: the forward call is mrf_isgmr_forward / mrf_trwp_forward (which store the
argmin indices p, q, Alg. 1 / 2), the backward call is mrf_isgmr_backward /
mrf_trwp_backward (Alg. 3 / 4).  No arithmetic of the method happens here.
"""
from __future__ import annotations

import torch

from . import mrfmp as _m


class _MessagePassing(torch.autograd.Function):
    @staticmethod
    def forward(ctx, unary, pairwise, edge_weight, cfg):
        algo, dirs, K, rho, kind, trunc, scale, w_scalar = cfg
        unary = unary.contiguous()
        pairwise = pairwise.contiguous()
        edge_weight = None if edge_weight is None else edge_weight.contiguous()
        B, H, W, L = unary.shape
        prob = _m.MrfProblem(unary, pairwise, dirs, K, edge_weight, w_scalar, rho, kind, trunc, scale)
        R = prob.R
        dev = unary.device
        cost = torch.empty_like(unary)
        labels = torch.empty((B, H, W), dtype=torch.uint8, device=dev)
        p = torch.empty((K, R, B, H, W, L), dtype=torch.uint8, device=dev)
        q = torch.empty((K, R, B, H, W), dtype=torch.uint8, device=dev)
        code = _m.MRF_ISGMR if algo == "isgmr" else _m.MRF_TRWP
        ws = torch.empty(max(_m.mrf_workspace_bytes(prob, code, False), _m.mrf_workspace_bytes(prob, code, True)),
                         dtype=torch.uint8, device=dev)
        (_m.mrf_isgmr_forward if code == _m.MRF_ISGMR else _m.mrf_trwp_forward)(prob, cost, labels, p, q, None, ws)
        ctx.prob, ctx.code, ctx.ws = prob, code, ws
        ctx.save_for_backward(p, q)
        ctx.has_w = edge_weight is not None
        ctx.mark_non_differentiable(labels)
        return cost, labels

    @staticmethod
    def backward(ctx, grad_cost, _grad_labels):
        p, q = ctx.saved_tensors
        prob = ctx.prob
        B, H, W, L = prob.shape
        dev = grad_cost.device
        need_u, need_v, need_w = ctx.needs_input_grad[0], ctx.needs_input_grad[1], ctx.needs_input_grad[2]
        g_unary = torch.empty((B, H, W, L), dtype=torch.float32, device=dev)
        g_w = torch.empty((prob.R, B, H, W), dtype=torch.float32, device=dev) if (need_w and ctx.has_w) else None
        g_v = torch.empty((L, L), dtype=torch.float32, device=dev) if need_v else None
        fn = _m.mrf_isgmr_backward if ctx.code == _m.MRF_ISGMR else _m.mrf_trwp_backward
        fn(prob, grad_cost.contiguous().float(), p, q, g_unary, g_w, g_v, ctx.ws)
        return (g_unary if need_u else None), g_v, g_w, None


class _MessagePassingEdgeTables(torch.autograd.Function):
    @staticmethod
    def forward(ctx, unary, pairwise_edge, cfg):
        algo, dirs, K, rho, rho_edge = cfg
        unary = unary.contiguous()
        pairwise_edge = pairwise_edge.contiguous()
        B, H, W, L = unary.shape
        prob = _m.MrfProblem(unary, None, dirs, K, rho=rho, rho_edge=rho_edge, pairwise_edge=pairwise_edge)
        R = prob.R
        dev = unary.device
        cost = torch.empty_like(unary)
        labels = torch.empty((B, H, W), dtype=torch.uint8, device=dev)
        p = torch.empty((K, R, B, H, W, L), dtype=torch.uint8, device=dev)
        q = torch.empty((K, R, B, H, W), dtype=torch.uint8, device=dev)
        code = _m.MRF_ISGMR if algo == "isgmr" else _m.MRF_TRWP
        ws = torch.empty(max(_m.mrf_workspace_bytes(prob, code, False), _m.mrf_workspace_bytes(prob, code, True)),
                         dtype=torch.uint8, device=dev)
        (_m.mrf_isgmr_forward if code == _m.MRF_ISGMR else _m.mrf_trwp_forward)(prob, cost, labels, p, q, None, ws)
        ctx.prob, ctx.code, ctx.ws = prob, code, ws
        ctx.save_for_backward(p, q)
        ctx.mark_non_differentiable(labels)
        return cost, labels

    @staticmethod
    def backward(ctx, grad_cost, _grad_labels):
        p, q = ctx.saved_tensors
        prob = ctx.prob
        B, H, W, L = prob.shape
        dev = grad_cost.device
        need_u, need_t = ctx.needs_input_grad[0], ctx.needs_input_grad[1]
        g_unary = torch.empty((B, H, W, L), dtype=torch.float32, device=dev)
        g_t = torch.empty((prob.R, B, H, W, L, L), dtype=torch.float32, device=dev) if need_t else None
        fn = _m.mrf_isgmr_backward if ctx.code == _m.MRF_ISGMR else _m.mrf_trwp_backward
        fn(prob, grad_cost.contiguous().float(), p, q, g_unary, None, g_t, ctx.ws)
        return (g_unary if need_u else None), g_t, None


def message_passing_edge_tables(unary, pairwise_edge, *, algo="isgmr", dirs=((0, 1), (0, -1), (1, 0), (-1, 0)),
                                K=5, rho=None, rho_edge=None):
    """As message_passing, for pairwise potentials given per edge: pairwise_edge [R,B,H,W,L,L],
    entry (r,i,mu,lambda) = theta_{i-r,i}(mu,lambda) stored at the node the edge arrives at
    (L <= 64).  Gradients flow to unary and pairwise_edge (Eq. supp-gradient-pairwise).  rho_edge
    [R,B,H,W]: TRW coefficients per edge (TRWP), in place of rho."""
    if algo not in ("isgmr", "trwp"):
        raise ValueError("algo must be 'isgmr' or 'trwp'")
    if algo == "trwp" and rho is None and rho_edge is None:
        raise ValueError("TRWP needs rho (one value per direction) or rho_edge")
    return _MessagePassingEdgeTables.apply(unary, pairwise_edge, (algo, dirs, int(K), rho, rho_edge))


def message_passing(unary, pairwise, edge_weight=None, *, algo="isgmr", dirs=((0, 1), (0, -1), (1, 0), (-1, 0)),
                    K=5, rho=None, pairwise_kind=0, trunc=0.0, scale=1.0, edge_weight_scalar=1.0):
    """Final costs c [B,H,W,L] (differentiable) and labels x* [B,H,W] (uint8) of K iterations of
    ISGMR or TRWP.  unary [B,H,W,L], pairwise [L,L] (V[mu at i-r][lambda at i]) and edge_weight
    [R,B,H,W] (stored at the destination node of each edge; None = edge_weight_scalar everywhere)
    are float32 CUDA tensors.  Gradients flow to all three (Alg. 3 / 4)."""
    if algo not in ("isgmr", "trwp"):
        raise ValueError("algo must be 'isgmr' or 'trwp'")
    if algo == "trwp" and rho is None:
        raise ValueError("TRWP needs rho (one value per direction)")
    cfg = (algo, dirs, int(K), rho, int(pairwise_kind), float(trunc), float(scale), float(edge_weight_scalar))
    return _MessagePassing.apply(unary, pairwise, edge_weight, cfg)
