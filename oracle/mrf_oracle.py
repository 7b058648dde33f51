"""ctypes binding of the CPU oracle (oracle/mrf_oracle.c) -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's CPU-baseline leg may import this module.
It holds argument marshalling and the gcc build step, no arithmetic of the method.

Two builds of the same source: ``threads=False`` (single-threaded, the oracle of
record) and ``threads=True`` (-fopenmp over the scanlines of the forward sweeps,
bit-identical by construction, for full-size parity runs).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "mrf_oracle.c"), os.path.join(_HERE, "mrf_oracle_impl.h")]
_LIBS = {False: os.path.join(_HERE, "libmrf_oracle.so"),
         True: os.path.join(_HERE, "libmrf_oracle_omp.so")}
_loaded: dict = {}

# -ffp-contract=off: the only fused multiply-add is the explicit fma()/fmaf() call.
_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra"]


def build(force: bool = False) -> None:
    """Compile both oracle libraries with gcc (a few seconds)."""
    for omp, out in _LIBS.items():
        stale = force or not os.path.exists(out) or any(
            os.path.getmtime(s) > os.path.getmtime(out) for s in _SRC)
        if not stale:
            continue
        cmd = ["gcc", *_CFLAGS, *( ["-fopenmp"] if omp else []), "-o", out, _SRC[0], "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
        _loaded.pop(omp, None)


def _lib(threads: bool):
    if threads not in _loaded:
        build()
        _loaded[threads] = ctypes.CDLL(_LIBS[threads])
    return _loaded[threads]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


@dataclass
class ForwardResult:
    cost: np.ndarray      # [B,H,W,L]
    labels: np.ndarray    # [B,H,W] uint8
    p: np.ndarray         # [K,R,B,H,W,L] uint8
    q: np.ndarray         # [K,R,B,H,W] uint8
    messages: np.ndarray  # [R,B,H,W,L]


@dataclass
class BackwardResult:
    grad_unary: np.ndarray        # [B,H,W,L]
    grad_edge_weight: np.ndarray  # [R,B,H,W]
    grad_pairwise: np.ndarray     # [L,L]
    grad_pairwise_edge: np.ndarray = None   # [R,B,H,W,L,L] (problems with per-edge pairwise potentials)


def _real(dtype):
    dtype = np.dtype(dtype)
    if dtype == np.float32:
        return "f32", ctypes.c_float
    if dtype == np.float64:
        return "f64", ctypes.c_double
    raise TypeError("oracle computes in float32 or float64")


def _common(unary_shape, dirs, dtype):
    B, H, W, L = (int(v) for v in unary_shape)
    dirs = np.ascontiguousarray(np.asarray(dirs, dtype=np.int32).reshape(-1, 2))
    return B, H, W, L, dirs, dirs.shape[0]


def _rho_args(rho, rho_edge, R, shape, dtype):
    """rho[R] and the optional per-edge array [R,B,H,W] (TRWP, Eq. trwp)."""
    if rho is None:
        rho = 1.0
    rho_a = np.ascontiguousarray(np.broadcast_to(np.asarray(rho, dtype=dtype), (R,)))
    rho_e = None if rho_edge is None else np.ascontiguousarray(rho_edge, dtype=dtype)
    if rho_e is not None:
        assert rho_e.shape == (R,) + tuple(shape)
    return rho_a, rho_e


def forward(algo: str, unary, pairwise, dirs, K: int, edge_weight=None, edge_weight_scalar=1.0,
            rho=None, dtype=np.float32, threads: bool = False, rho_edge=None,
            pairwise_edge=None) -> ForwardResult:
    """Alg. 1 (algo='isgmr') or Alg. 2 (algo='trwp').  pairwise_edge [R,B,H,W,L,L]: pairwise
    potentials theta_{i-r,i}(mu,lambda) given per edge; pairwise and the edge weights are then
    not used."""
    sfx, creal = _real(dtype)
    unary = np.ascontiguousarray(unary, dtype=dtype)
    B, H, W, L, dirs, R = _common(unary.shape, dirs, dtype)
    Te = None if pairwise_edge is None else np.ascontiguousarray(pairwise_edge, dtype=dtype)
    if Te is not None:
        assert Te.shape == (R, B, H, W, L, L)
    V = None if (pairwise is None and Te is not None) else np.ascontiguousarray(pairwise, dtype=dtype)
    assert V is None or V.shape == (L, L)
    w = None if edge_weight is None else np.ascontiguousarray(edge_weight, dtype=dtype)
    if w is not None:
        assert w.shape == (R, B, H, W)
    cost = np.empty((B, H, W, L), dtype)
    labels = np.empty((B, H, W), np.uint8)
    p = np.empty((K, R, B, H, W, L), np.uint8)
    q = np.empty((K, R, B, H, W), np.uint8)
    msg = np.empty((R, B, H, W, L), dtype)
    lib = _lib(threads)
    head = [ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(W), ctypes.c_int(L), ctypes.c_int(R),
            _ptr(dirs), ctypes.c_int(K), _ptr(unary), _ptr(V), _ptr(w), creal(edge_weight_scalar)]
    tail = [_ptr(cost), _ptr(labels), _ptr(p), _ptr(q), _ptr(msg)]
    if algo == "isgmr":
        fn = getattr(lib, "mrfo_isgmr_forward_" + sfx)
        rc = fn(*head, _ptr(Te), *tail)
    elif algo == "trwp":
        rho_a, rho_e = _rho_args(rho, rho_edge, R, (B, H, W), dtype)
        fn = getattr(lib, "mrfo_trwp_forward_" + sfx)
        rc = fn(*head, _ptr(rho_a), _ptr(rho_e), _ptr(Te), *tail)
    else:
        raise ValueError(algo)
    if rc != 0:
        raise ValueError("oracle rejected the problem (rc=%d)" % rc)
    return ForwardResult(cost, labels, p, q, msg)


def sgm_standard_forward(unary, pairwise, dirs, edge_weight=None, edge_weight_scalar=1.0,
                         dtype=np.float32) -> ForwardResult:
    """Standard single-pass SGM (Sec. 3.2, Eq. sgm_old and Eq. isgmr-aggregation-old): messages that
    carry the node's own unary, one pass, cost = sum of the messages.  p, q as for K = 1."""
    sfx, creal = _real(dtype)
    unary = np.ascontiguousarray(unary, dtype=dtype)
    B, H, W, L, dirs, R = _common(unary.shape, dirs, dtype)
    V = np.ascontiguousarray(pairwise, dtype=dtype)
    assert V.shape == (L, L)
    w = None if edge_weight is None else np.ascontiguousarray(edge_weight, dtype=dtype)
    cost = np.empty((B, H, W, L), dtype)
    labels = np.empty((B, H, W), np.uint8)
    p = np.empty((1, R, B, H, W, L), np.uint8)
    q = np.empty((1, R, B, H, W), np.uint8)
    msg = np.empty((R, B, H, W, L), dtype)
    fn = getattr(_lib(False), "mrfo_sgm_standard_forward_" + sfx)
    rc = fn(ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(W), ctypes.c_int(L), ctypes.c_int(R), _ptr(dirs),
            _ptr(unary), _ptr(V), _ptr(w), creal(edge_weight_scalar), _ptr(cost), _ptr(labels), _ptr(p), _ptr(q),
            _ptr(msg))
    if rc != 0:
        raise ValueError("oracle rejected the problem (rc=%d)" % rc)
    return ForwardResult(cost, labels, p, q, msg)


def backward(algo: str, shape, pairwise, dirs, K: int, grad_cost, p, q, edge_weight=None,
             edge_weight_scalar=1.0, rho=None, dtype=np.float32, rho_edge=None,
             per_edge_pairwise: bool = False) -> BackwardResult:
    """Alg. 3 (algo='isgmr') or Alg. 4 (algo='trwp'); shape = (B,H,W,L).  per_edge_pairwise: the
    problem gave its pairwise potentials per edge; then the gradient of those [R,B,H,W,L,L]
    (Eq. supp-gradient-pairwise) is returned instead of the gradients of edge weights and V."""
    sfx, creal = _real(dtype)
    B, H, W, L, dirs, R = _common(shape, dirs, dtype)
    V = None if per_edge_pairwise else np.ascontiguousarray(pairwise, dtype=dtype)
    w = None if edge_weight is None else np.ascontiguousarray(edge_weight, dtype=dtype)
    gc = np.ascontiguousarray(grad_cost, dtype=dtype)
    assert gc.shape == (B, H, W, L)
    p = np.ascontiguousarray(p, dtype=np.uint8)
    q = np.ascontiguousarray(q, dtype=np.uint8)
    assert p.shape == (K, R, B, H, W, L) and q.shape == (K, R, B, H, W)
    gu = np.empty((B, H, W, L), dtype)
    gw = None if per_edge_pairwise else np.empty((R, B, H, W), dtype)
    gV = None if per_edge_pairwise else np.empty((L, L), dtype)
    gTe = np.empty((R, B, H, W, L, L), dtype) if per_edge_pairwise else None
    lib = _lib(False)
    head = [ctypes.c_int(B), ctypes.c_int(H), ctypes.c_int(W), ctypes.c_int(L), ctypes.c_int(R),
            _ptr(dirs), ctypes.c_int(K), _ptr(V), _ptr(w), creal(edge_weight_scalar)]
    tail = [_ptr(gc), _ptr(p), _ptr(q), _ptr(gu), _ptr(gw), _ptr(gV), _ptr(gTe)]
    if algo == "isgmr":
        rc = getattr(lib, "mrfo_isgmr_backward_" + sfx)(*head, *tail)
    elif algo == "trwp":
        rho_a, rho_e = _rho_args(rho, rho_edge, R, (B, H, W), dtype)
        rc = getattr(lib, "mrfo_trwp_backward_" + sfx)(*head, _ptr(rho_a), _ptr(rho_e), *tail)
    else:
        raise ValueError(algo)
    if rc != 0:
        raise ValueError("oracle rejected the problem (rc=%d)" % rc)
    return BackwardResult(gu, gw, gV, gTe)


def count_scanlines(H: int, W: int, dh: int, dw: int) -> int:
    lib = _lib(False)
    lib.mrfo_count_scanlines.restype = ctypes.c_long
    return int(lib.mrfo_count_scanlines(H, W, dh, dw))


def openmp_enabled(threads: bool) -> bool:
    return bool(_lib(threads).mrfo_openmp_enabled())
