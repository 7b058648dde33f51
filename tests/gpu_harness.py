"""Runs an mrf_inputs.Problem through the C-ABI library (via the thin Python binding) and
returns numpy arrays.  Used by the GPU parity tests, the smoke check and the bench."""
from dataclasses import dataclass

import numpy as np
import torch

import paper_1910_10892_amd as mrf


@dataclass
class DeviceResults:
    cost: np.ndarray
    labels: np.ndarray
    p: np.ndarray
    q: np.ndarray
    messages: np.ndarray
    grad_unary: np.ndarray = None
    grad_edge_weight: np.ndarray = None
    grad_pairwise: np.ndarray = None


class GpuProblem:
    """Device-resident copy of a Problem plus every output / workspace buffer."""

    def __init__(self, pr, want_messages=True, device="cuda:0"):
        self.pr = pr
        dev = torch.device(device)
        B, H, W, L = pr.shape
        R, K = pr.R, pr.K
        t = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.pairwise_edge = t(getattr(pr, "pairwise_edge", None))
        self.edge_tables = self.pairwise_edge is not None     # then V and the edge weights are not used
        self.unary, self.edge_weight = t(pr.unary), t(pr.edge_weight)
        self.pairwise = None if self.edge_tables else t(pr.pairwise)
        self.grad_cost = t(pr.grad_cost)
        self.algo = mrf.MRF_ISGMR if pr.algo == "isgmr" else mrf.MRF_TRWP
        self.rho_edge = t(getattr(pr, "rho_edge", None))
        self.prob = mrf.MrfProblem(self.unary, self.pairwise, pr.dirs, K, self.edge_weight,
                                   pr.edge_weight_scalar, pr.rho, pr.pairwise_kind, pr.trunc, pr.scale,
                                   rho_edge=self.rho_edge, pairwise_edge=self.pairwise_edge,
                                   sgm_standard=bool(getattr(pr, "sgm_standard", False)))
        self.cost = torch.empty((B, H, W, L), dtype=torch.float32, device=dev)
        self.labels = torch.empty((B, H, W), dtype=torch.uint8, device=dev)
        self.p = torch.empty((K, R, B, H, W, L), dtype=torch.uint8, device=dev)
        self.q = torch.empty((K, R, B, H, W), dtype=torch.uint8, device=dev)
        self.messages = torch.empty((R, B, H, W, L), dtype=torch.float32, device=dev) if want_messages else None
        self.grad_unary = torch.empty((B, H, W, L), dtype=torch.float32, device=dev)
        self.grad_edge_weight = torch.empty((R, B, H, W), dtype=torch.float32, device=dev)
        self.grad_pairwise = torch.empty((R, B, H, W, L, L) if self.edge_tables else (L, L),
                                         dtype=torch.float32, device=dev)
        nbytes = max(mrf.mrf_workspace_bytes(self.prob, self.algo, False),
                     mrf.mrf_workspace_bytes(self.prob, self.algo, True))
        assert nbytes > 0
        self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev)

    def forward(self):
        fn = mrf.mrf_isgmr_forward if self.algo == mrf.MRF_ISGMR else mrf.mrf_trwp_forward
        fn(self.prob, self.cost, self.labels, self.p, self.q, self.messages, self.workspace)

    def backward(self, want_w=True, want_V=True):
        fn = mrf.mrf_isgmr_backward if self.algo == mrf.MRF_ISGMR else mrf.mrf_trwp_backward
        fn(self.prob, self.grad_cost, self.p, self.q, self.grad_unary,
           self.grad_edge_weight if (want_w and not self.edge_tables) else None,
           self.grad_pairwise if want_V else None, self.workspace)

    def poison_outputs(self):
        """Outputs must be fully overwritten: fill them with garbage first."""
        for x in (self.cost, self.grad_unary, self.grad_edge_weight, self.grad_pairwise, self.messages):
            if x is not None:
                x.fill_(float("nan"))
        for x in (self.labels, self.p, self.q):
            x.fill_(173)
        self.workspace.fill_(0xFF)

    def results(self, backward=True) -> DeviceResults:
        torch.cuda.synchronize()
        n = lambda x: None if x is None else x.cpu().numpy()
        out = DeviceResults(n(self.cost), n(self.labels), n(self.p), n(self.q), n(self.messages))
        if backward:
            out.grad_unary, out.grad_edge_weight, out.grad_pairwise = (
                n(self.grad_unary), n(self.grad_edge_weight), n(self.grad_pairwise))
        return out


def run_gpu(pr, backward=True, want_V=True) -> DeviceResults:
    g = GpuProblem(pr)
    g.poison_outputs()
    g.forward()
    if backward:
        g.backward(want_V=want_V)
    out = g.results(backward)
    if backward and not want_V:
        out.grad_pairwise = None
    return out
