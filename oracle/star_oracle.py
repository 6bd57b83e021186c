"""ctypes front end of ``star_oracle.c`` (test infrastructure, not product code).

Takes numpy arrays, returns numpy arrays.  Gradient rows are float32 arrays, or
uint16 arrays holding bf16 bit patterns.  See ``star_oracle.c`` for what is
computed and the passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "star_oracle.c")
_LIB = os.path.join(_HERE, "libstar_oracle.so")

W_MEAN, W_STALE, W_EXPLICIT = 0, 1, 2
_WMODES = {"mean": W_MEAN, "stale": W_STALE, "explicit": W_EXPLICIT}


BUILD_FLAGS = ["-std=c11", "-O3", "-ffp-contract=off"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No -march flags: the library may be built
    on one host and run on another.  -ffp-contract=off keeps the fp32 stepwise
    mode free of fused multiply-adds; no fast-math, so the optimisation level
    does not change a result."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC),
                                                                        os.path.getmtime(__file__)):
        subprocess.check_call(["gcc"] + BUILD_FLAGS + ["-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Updates(ctypes.Structure):
    _fields_ = [("U", ctypes.c_int32),
                ("offsets", ctypes.c_void_p), ("members", ctypes.c_void_p),
                ("staleness", ctypes.c_void_p), ("coeff", ctypes.c_void_p), ("lr", ctypes.c_void_p)]


class _HParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("wmode", ctypes.c_int32), ("scale_lr_by_group", ctypes.c_int32)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        # STAR_ORACLE_LIB lets the mutation test point the pins at a deliberately
        # broken build of the oracle (on the CPU) to show that the pins catch it.
        _lib = ctypes.CDLL(os.environ.get("STAR_ORACLE_LIB") or build())
        for name in ("oracle_group_update", "oracle_group_update_f64", "oracle_group_update_f32step",
                     "oracle_group_norms", "oracle_group_reduce", "oracle_gram"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class _Marshal:
    """Holds contiguous copies of the host arrays for the duration of a call."""

    def __init__(self, rows: Sequence[np.ndarray], offsets, members, staleness, coeff, lr_per_update):
        self.rows = []
        dt = None
        for r in rows:
            r = np.ascontiguousarray(r)
            if r.dtype == np.float32:
                d = 0
            elif r.dtype == np.uint16:
                d = 1
            else:
                raise TypeError("gradient rows must be float32 or uint16 (bf16 bits)")
            if dt is not None and d != dt:
                raise TypeError("all rows must share one dtype")
            dt = d
            self.rows.append(r)
        self.dtype = 0 if dt is None else dt
        self.W = len(self.rows)
        self.P = int(self.rows[0].shape[0]) if self.rows else 0
        self.rowptr = (ctypes.c_void_p * max(1, self.W))(*[r.ctypes.data for r in self.rows])
        self.offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        self.members = np.ascontiguousarray(members, dtype=np.int32)
        self.staleness = None if staleness is None else np.ascontiguousarray(staleness, dtype=np.int32)
        self.coeff = None if coeff is None else np.ascontiguousarray(coeff, dtype=np.float32)
        self.lr = None if lr_per_update is None else np.ascontiguousarray(lr_per_update, dtype=np.float32)
        self.U = int(self.offsets.shape[0]) - 1
        self.upd = _Updates(self.U, _ptr(self.offsets), _ptr(self.members), _ptr(self.staleness),
                            _ptr(self.coeff), _ptr(self.lr))


def group_update(params: np.ndarray, momentum: np.ndarray, rows: Sequence[np.ndarray], offsets, members, *,
                 lr: float, momentum_coef: float, weight_decay: float = 0.0, wmode: str = "mean",
                 staleness=None, coeff=None, lr_per_update=None, scale_lr_by_group: bool = False,
                 want_norms: bool = False, mode: str = "exact"):
    """Run U group updates.  Returns (params, momentum, norms or None).

    mode "exact":   fp32 state in, fp64 arithmetic inside the call, fp32 out.
    mode "f64":     params/momentum are float64 arrays, stay float64 (no rounding).
    mode "f32step": fp32 arithmetic, state rounded after every update.
    """
    lib = _load()
    m = _Marshal(rows, offsets, members, staleness, coeff, lr_per_update)
    hp = _HParams(lr, momentum_coef, weight_decay, _WMODES[wmode], int(bool(scale_lr_by_group)))
    P = int(params.shape[0])
    if m.W and m.P != P:
        raise ValueError("row length differs from the shard length")
    norms = np.zeros(max(m.U, 0), dtype=np.float64) if want_norms else None
    if mode == "f64":
        p = np.array(params, dtype=np.float64, copy=True)
        v = np.array(momentum, dtype=np.float64, copy=True)
        rc = lib.oracle_group_update_f64(_ptr(p), _ptr(v), m.rowptr, m.dtype, ctypes.c_int64(P), m.W,
                                         ctypes.byref(m.upd), ctypes.byref(hp), _ptr(norms))
    else:
        p = np.array(params, dtype=np.float32, copy=True)
        v = np.array(momentum, dtype=np.float32, copy=True)
        if mode == "exact":
            scratch = np.empty(2 * max(P, 1), dtype=np.float64)
            rc = lib.oracle_group_update(_ptr(p), _ptr(v), m.rowptr, m.dtype, ctypes.c_int64(P), m.W,
                                         ctypes.byref(m.upd), ctypes.byref(hp), _ptr(norms), _ptr(scratch))
        elif mode == "f32step":
            rc = lib.oracle_group_update_f32step(_ptr(p), _ptr(v), m.rowptr, m.dtype, ctypes.c_int64(P), m.W,
                                                 ctypes.byref(m.upd), ctypes.byref(hp), _ptr(norms))
        else:
            raise ValueError(mode)
    if rc:
        raise ValueError(f"oracle rejected the update stream (code {rc})")
    return p, v, norms


def group_norms(rows: Sequence[np.ndarray], offsets, members, *, wmode: str = "mean", staleness=None,
                coeff=None) -> np.ndarray:
    lib = _load()
    m = _Marshal(rows, offsets, members, staleness, coeff, None)
    norms = np.zeros(max(m.U, 0), dtype=np.float64)
    rc = lib.oracle_group_norms(m.rowptr, m.dtype, ctypes.c_int64(m.P), m.W, ctypes.byref(m.upd),
                                _WMODES[wmode], _ptr(norms))
    if rc:
        raise ValueError(f"oracle rejected the update stream (code {rc})")
    return norms


def group_reduce(rows: Sequence[np.ndarray], offsets, members, *, wmode: str = "mean", staleness=None, coeff=None,
                 want_norms: bool = False):
    """Weighted sum of every group's rows: float64 array [U, P] (and norms [U] if asked)."""
    lib = _load()
    m = _Marshal(rows, offsets, members, staleness, coeff, None)
    out = np.zeros((max(m.U, 0), m.P), dtype=np.float64)
    norms = np.zeros(max(m.U, 0), dtype=np.float64) if want_norms else None
    rc = lib.oracle_group_reduce(_ptr(out), m.rowptr, m.dtype, ctypes.c_int64(m.P), m.W, ctypes.byref(m.upd),
                                 _WMODES[wmode], _ptr(norms))
    if rc:
        raise ValueError(f"oracle rejected the update stream (code {rc})")
    return (out, norms) if want_norms else out


def gram(rows: Sequence[np.ndarray]) -> np.ndarray:
    """Gram matrix of the rows, float64 [W, W]."""
    lib = _load()
    m = _Marshal(rows, [0], [], None, None, None)
    out = np.zeros((m.W, m.W), dtype=np.float64)
    lib.oracle_gram(_ptr(out), m.rowptr, m.dtype, ctypes.c_int64(m.P), m.W)
    return out


def noise_scale(rows: Sequence[np.ndarray], batch_per_worker: float):
    """(grad_sq, trace_cov, noise_scale) straight from the rows, from the model
    g_w = G + e_w, Cov e_w = Sigma / b:  E mean|g_w|^2 = |G|^2 + tr/b and
    E |mean g_w|^2 = |G|^2 + tr/(W b), solved for |G|^2 and tr(Sigma)."""
    R = np.stack([np.asarray(r, dtype=np.float64) for r in rows])
    W = R.shape[0]
    S = float(np.mean(np.sum(R * R, axis=1)))
    gbar = R.mean(axis=0)
    n2 = float(gbar @ gbar)
    tr = batch_per_worker * (S - n2) * W / (W - 1)
    g2 = (W * n2 - S) / (W - 1)
    return g2, tr, tr / g2


def max_rel_err(x: np.ndarray, ref: np.ndarray) -> float:
    """Error measure used by every parity test: max_j |x-ref| / (|ref| + RMS(ref)).
    The RMS term gives elements near zero a scale to be judged against."""
    x = np.asarray(x, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.abs(ref) + rms
    den[den == 0] = 1.0
    return float(np.max(np.abs(x - ref) / den))
