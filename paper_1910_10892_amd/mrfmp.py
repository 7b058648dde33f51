"""ctypes binding of libmrfmp: argument marshalling only.

Function names mirror include/mrfmp.h.  Tensors are torch CUDA(HIP) tensors; the binding
passes their device pointers and the current stream's handle.  There is no fallback: if
the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

from .build import LIB_PATH

MRF_ISGMR, MRF_TRWP = 0, 1
_lib = None


class MrfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = mrf_last_error_detail() if status == -9 else ""
        super().__init__("%s failed: %s (status %d)%s" % (where, mrf_strerror(status), status,
                                                          " [" + detail + "]" if detail else ""))


class _CProblem(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32), ("L", ctypes.c_int32),
        ("R", ctypes.c_int32),
        ("dirs", ctypes.c_void_p),
        ("K", ctypes.c_int32),
        ("unary", ctypes.c_void_p),
        ("pairwise", ctypes.c_void_p),
        ("edge_weight", ctypes.c_void_p),
        ("edge_weight_scalar", ctypes.c_float),
        ("rho", ctypes.c_void_p),
        ("pairwise_kind", ctypes.c_int32),
        ("trunc", ctypes.c_float), ("scale", ctypes.c_float),
        ("rho_edge", ctypes.c_void_p),
        ("pairwise_edge", ctypes.c_void_p),
        ("sgm_standard", ctypes.c_int32),
    ]


def library_path() -> str:
    return LIB_PATH


def load_library():
    """Load libmrfmp.so (built in-tree by paper_1910_10892_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "libmrfmp.so not built: run `python -m paper_1910_10892_amd.build` (needs hipcc)")
    # The tensors this binding is handed live in PyTorch's HIP runtime.  Import torch first, so
    # that the library's dependency on libamdhip64 binds to the copy torch has loaded; loaded
    # the other way round the process ends up with two runtimes and the library's own sees
    # no initialised device.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, ci = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    P = ctypes.POINTER(_CProblem)
    lib.mrf_workspace_bytes.restype = sz
    lib.mrf_workspace_bytes.argtypes = [P, ci, ci]
    lib.mrf_validate.restype = ci
    lib.mrf_validate.argtypes = [P, ci]
    lib.mrf_forward_window.restype = ci
    lib.mrf_forward_window.argtypes = [P, ci]
    for name in ("mrf_isgmr_forward", "mrf_trwp_forward"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
    for name in ("mrf_isgmr_backward", "mrf_trwp_backward"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mrf_scanline_count.restype = ctypes.c_int64
    lib.mrf_scanline_count.argtypes = [ctypes.c_int32] * 4
    lib.mrf_scanline_head.restype = ci
    lib.mrf_scanline_head.argtypes = [ctypes.c_int32] * 4 + [ctypes.c_int64] + [ctypes.POINTER(ctypes.c_int32)] * 3
    lib.mrf_strerror.restype = ctypes.c_char_p
    lib.mrf_last_error_detail.restype = ctypes.c_char_p
    lib.mrf_last_error_detail.argtypes = []
    lib.mrf_last_sweep_kernel.restype = ctypes.c_char_p
    lib.mrf_last_sweep_kernel.argtypes = [ci]
    lib.mrf_last_sweep_launch.restype = ctypes.c_char_p
    lib.mrf_last_sweep_launch.argtypes = [ci]
    lib.mrf_energy_workspace_bytes.restype = sz
    lib.mrf_energy_workspace_bytes.argtypes = [P]
    lib.mrf_energy.restype = ci
    lib.mrf_energy.argtypes = [P, vp, vp, vp, sz, vp]
    lib.mrf_energy_noalloc.restype = ci
    lib.mrf_energy_noalloc.argtypes = [P, vp, vp, vp]
    lib.mrf_softmin_l1_workspace_bytes.restype = sz
    lib.mrf_softmin_l1_workspace_bytes.argtypes = []
    lib.mrf_softmin_l1.restype = ci
    lib.mrf_softmin_l1.argtypes = [ctypes.c_int64, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.mrf_softmin_smooth_l1.restype = ci
    lib.mrf_softmin_smooth_l1.argtypes = [ctypes.c_int64, ctypes.c_int32, vp, vp, vp, ctypes.c_float, vp, vp, vp, vp, sz, vp]
    lib.mrf_workspace_fault.restype = ci
    lib.mrf_workspace_fault.argtypes = [vp, vp]
    lib.mrf_strerror.argtypes = [ci]
    lib.mrf_version.restype = ctypes.c_char_p
    lib.mrf_set_sweep_events.restype = ci
    lib.mrf_set_sweep_events.argtypes = [vp, vp]
    lib.mrf_tune.restype = ci
    lib.mrf_tune.argtypes = [ci, ci]
    _lib = lib
    return lib


def _dev_ptr(t, dtype_name: Optional[str] = None):
    """Device pointer of a contiguous torch tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors must be contiguous and on the GPU")
    if dtype_name is not None and str(t.dtype) != "torch." + dtype_name:
        raise ValueError("expected %s tensor, got %s" % (dtype_name, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


@dataclass
class MrfProblem:
    """Mirror of the C struct mrf_problem.  unary/pairwise/edge_weight are GPU tensors,
    dirs and rho are host sequences."""
    unary: object                 # [B,H,W,L] float32 GPU tensor (may be None for backward)
    pairwise: object              # [L,L] float32 GPU tensor
    dirs: Sequence                # R x (dh, dw)
    K: int
    edge_weight: object = None    # [R,B,H,W] float32 GPU tensor or None
    edge_weight_scalar: float = 1.0
    rho: Optional[Sequence] = None
    pairwise_kind: int = 0
    trunc: float = 0.0
    scale: float = 1.0
    shape: Optional[tuple] = None  # (B,H,W,L); taken from unary when given
    rho_edge: object = None       # [R,B,H,W] float32 GPU tensor or None (TRWP: rho per directed edge)
    pairwise_edge: object = None  # [R,B,H,W,L,L] float32 GPU tensor or None (pairwise potentials per edge)
    sgm_standard: bool = False    # standard single-pass SGM (Eq. sgm_old) instead of the revised update; forward, K = 1

    def __post_init__(self):
        if self.shape is None:
            self.shape = tuple(int(v) for v in self.unary.shape)
        self._dirs = np.ascontiguousarray(np.asarray(self.dirs, np.int32).reshape(-1, 2))
        self._rho = None if self.rho is None else np.ascontiguousarray(
            np.broadcast_to(np.asarray(self.rho, np.float32), (self._dirs.shape[0],)))

    @property
    def R(self):
        return int(self._dirs.shape[0])

    def c_struct(self) -> _CProblem:
        B, H, W, L = self.shape
        c = _CProblem()
        c.B, c.H, c.W, c.L, c.R, c.K = B, H, W, L, self.R, int(self.K)
        c.dirs = self._dirs.ctypes.data
        c.unary = _dev_ptr(self.unary, "float32")
        c.pairwise = _dev_ptr(self.pairwise, "float32")
        c.edge_weight = _dev_ptr(self.edge_weight, "float32")
        c.edge_weight_scalar = float(self.edge_weight_scalar)
        c.rho = None if self._rho is None else self._rho.ctypes.data
        c.pairwise_kind = int(self.pairwise_kind)
        c.trunc, c.scale = float(self.trunc), float(self.scale)
        c.rho_edge = _dev_ptr(self.rho_edge, "float32")
        c.pairwise_edge = _dev_ptr(self.pairwise_edge, "float32")
        c.sgm_standard = 1 if self.sgm_standard else 0
        return c


def _stream_handle(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def mrf_strerror(status: int) -> str:
    return load_library().mrf_strerror(int(status)).decode()


def mrf_last_error_detail() -> str:
    return load_library().mrf_last_error_detail().decode()


def mrf_last_sweep_kernel(backward: bool) -> str:
    return load_library().mrf_last_sweep_kernel(1 if backward else 0).decode()


def mrf_last_sweep_launch(backward: bool) -> str:
    return load_library().mrf_last_sweep_launch(1 if backward else 0).decode()


def mrf_version() -> str:
    return load_library().mrf_version().decode()


def mrf_tune(knob: int, value: int) -> int:
    return int(load_library().mrf_tune(int(knob), int(value)))


def mrf_set_sweep_events(start_event, stop_event) -> int:
    """start_event / stop_event: torch.cuda.Event(enable_timing=True) that have been recorded
    once (so that their HIP handles exist), or None, None to clear."""
    h = lambda e: None if e is None else ctypes.c_void_p(e.cuda_event)
    return int(load_library().mrf_set_sweep_events(h(start_event), h(stop_event)))


def mrf_validate(prob: MrfProblem, algo: int) -> int:
    c = prob.c_struct()
    return int(load_library().mrf_validate(ctypes.byref(c), int(algo)))


def mrf_forward_window(prob: MrfProblem, algo: int) -> int:
    c = prob.c_struct()
    return int(load_library().mrf_forward_window(ctypes.byref(c), int(algo)))


def mrf_workspace_bytes(prob: MrfProblem, algo: int, backward: bool) -> int:
    c = prob.c_struct()
    return int(load_library().mrf_workspace_bytes(ctypes.byref(c), int(algo), int(bool(backward))))


def mrf_scanline_count(H: int, W: int, dh: int, dw: int) -> int:
    return int(load_library().mrf_scanline_count(H, W, dh, dw))


def mrf_scanline_head(H: int, W: int, dh: int, dw: int, t: int):
    y, x, n = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    rc = load_library().mrf_scanline_head(H, W, dh, dw, t, ctypes.byref(y), ctypes.byref(x), ctypes.byref(n))
    if rc != 0:
        raise MrfError(rc, "mrf_scanline_head")
    return y.value, x.value, n.value


def _forward(name, prob, cost, labels, p, q, messages, workspace, stream):
    c = prob.c_struct()
    rc = getattr(load_library(), name)(
        ctypes.byref(c), _dev_ptr(cost, "float32"), _dev_ptr(labels, "uint8"), _dev_ptr(p, "uint8"),
        _dev_ptr(q, "uint8"), _dev_ptr(messages, "float32"), _dev_ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != 0:
        raise MrfError(rc, name)


def _backward(name, prob, grad_cost, p, q, grad_unary, grad_edge_weight, grad_pairwise, workspace, stream):
    c = prob.c_struct()
    rc = getattr(load_library(), name)(
        ctypes.byref(c), _dev_ptr(grad_cost, "float32"), _dev_ptr(p, "uint8"), _dev_ptr(q, "uint8"),
        _dev_ptr(grad_unary, "float32"), _dev_ptr(grad_edge_weight, "float32"),
        _dev_ptr(grad_pairwise, "float32"), _dev_ptr(workspace),
        0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_handle(stream))
    if rc != 0:
        raise MrfError(rc, name)


def mrf_isgmr_forward(prob, cost, labels, p, q, messages, workspace, stream=None):
    _forward("mrf_isgmr_forward", prob, cost, labels, p, q, messages, workspace, stream)


def mrf_trwp_forward(prob, cost, labels, p, q, messages, workspace, stream=None):
    _forward("mrf_trwp_forward", prob, cost, labels, p, q, messages, workspace, stream)


def mrf_isgmr_backward(prob, grad_cost, p, q, grad_unary, grad_edge_weight, grad_pairwise, workspace,
                       stream=None):
    _backward("mrf_isgmr_backward", prob, grad_cost, p, q, grad_unary, grad_edge_weight, grad_pairwise,
              workspace, stream)


def mrf_trwp_backward(prob, grad_cost, p, q, grad_unary, grad_edge_weight, grad_pairwise, workspace,
                      stream=None):
    _backward("mrf_trwp_backward", prob, grad_cost, p, q, grad_unary, grad_edge_weight, grad_pairwise,
              workspace, stream)


def _ws_size(workspace) -> int:
    return 0 if workspace is None else workspace.numel() * workspace.element_size()


def mrf_energy_workspace_bytes(prob) -> int:
    c = prob.c_struct()
    return int(load_library().mrf_energy_workspace_bytes(ctypes.byref(c)))


def mrf_energy(prob, labels, energy, workspace, stream=None):
    """labels [B,H,W] uint8, energy [B] float64 (assigned), workspace uint8 tensor."""
    c = prob.c_struct()
    rc = load_library().mrf_energy(ctypes.byref(c), _dev_ptr(labels, "uint8"), _dev_ptr(energy, "float64"),
                                   _dev_ptr(workspace), _ws_size(workspace), _stream_handle(stream))
    if rc != 0:
        raise MrfError(rc, "mrf_energy")


def mrf_energy_noalloc(prob, labels, energy, stream=None):
    """mrf_energy without a workspace argument (the library's own fixed scratch; batch <= 64)."""
    c = prob.c_struct()
    rc = load_library().mrf_energy_noalloc(ctypes.byref(c), _dev_ptr(labels, "uint8"), _dev_ptr(energy, "float64"),
                                           _stream_handle(stream))
    if rc != 0:
        raise MrfError(rc, "mrf_energy_noalloc")


def mrf_softmin_l1_workspace_bytes() -> int:
    return int(load_library().mrf_softmin_l1_workspace_bytes())


def mrf_softmin_l1(cost, target, mask, disparity, loss, grad_cost, workspace, stream=None):
    """cost [..., L] float32, target [...] float32, mask [...] uint8 or None, disparity [...] float32 or
    None, loss [1] float64, grad_cost like cost or None."""
    L = int(cost.shape[-1])
    n = int(cost.numel() // L)
    rc = load_library().mrf_softmin_l1(n, L, _dev_ptr(cost, "float32"), _dev_ptr(target, "float32"),
                                       _dev_ptr(mask, "uint8"), _dev_ptr(disparity, "float32"),
                                       _dev_ptr(loss, "float64"), _dev_ptr(grad_cost, "float32"),
                                       _dev_ptr(workspace), _ws_size(workspace), _stream_handle(stream))
    if rc != 0:
        raise MrfError(rc, "mrf_softmin_l1")


def mrf_softmin_smooth_l1(cost, target, mask, beta, disparity, loss, grad_cost, workspace, stream=None):
    """mrf_softmin_l1 with the smooth L1 loss (threshold beta > 0)."""
    L = int(cost.shape[-1])
    n = int(cost.numel() // L)
    rc = load_library().mrf_softmin_smooth_l1(n, L, _dev_ptr(cost, "float32"), _dev_ptr(target, "float32"),
                                              _dev_ptr(mask, "uint8"), ctypes.c_float(beta), _dev_ptr(disparity, "float32"),
                                              _dev_ptr(loss, "float64"), _dev_ptr(grad_cost, "float32"),
                                              _dev_ptr(workspace), _ws_size(workspace), _stream_handle(stream))
    if rc != 0:
        raise MrfError(rc, "mrf_softmin_smooth_l1")


def mrf_workspace_fault(workspace, stream=None) -> int:
    """0, or -11 if a wait between wavefronts ran out in the last call that used this workspace
    (synchronises the stream)."""
    return int(load_library().mrf_workspace_fault(_dev_ptr(workspace), _stream_handle(stream)))
