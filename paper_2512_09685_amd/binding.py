"""ctypes binding of libstar.so: argument marshalling only.

Functions carry the names of the C entry points (``include/star.h``).  Tensors
are only asked for their ``data_ptr()``; the stream is passed as its raw
handle.  There is no fallback: if the library is missing or was not built, the
import of this module's functions raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libstar.so")

KERNEL_AUTO, KERNEL_SEQ, KERNEL_AFFINE, KERNEL_AFFINE_MFMA = 0, 1, 2, 3
F32, BF16 = 0, 1
_WMODES = {"mean": 0, "stale": 1, "explicit": 2}
STATUS_NAMES = {0: "STAR_OK", 1: "STAR_ERR_NULL", 2: "STAR_ERR_SHAPE", 3: "STAR_ERR_GROUP", 4: "STAR_ERR_HPARAM",
                5: "STAR_ERR_DTYPE", 6: "STAR_ERR_KERNEL", 7: "STAR_ERR_DEVICE"}


class StarError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class _Updates(ctypes.Structure):
    _fields_ = [("U", ctypes.c_int32), ("offsets", ctypes.c_void_p), ("members", ctypes.c_void_p),
                ("staleness", ctypes.c_void_p), ("coeff", ctypes.c_void_p), ("lr", ctypes.c_void_p)]


class _HParams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("momentum", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("wmode", ctypes.c_int32), ("scale_lr_by_group", ctypes.c_int32)]


class _Options(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("flags", ctypes.c_int32), ("queue_threshold", ctypes.c_int64)]


class _PlanInfo(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int32), ("grad_dtype", ctypes.c_int32), ("rows_used", ctypes.c_int32),
                ("rows_padded", ctypes.c_int32), ("queue_order", ctypes.c_int32), ("launches", ctypes.c_int32),
                ("finishing_launches", ctypes.c_int32), ("tables_inline", ctypes.c_int32),
                ("collapsed_update", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("fma_seq", ctypes.c_double), ("fma_affine", ctypes.c_double)]


OPT_DIRECT_NORMS = 1


def _options(kernel, queue_threshold, direct_norms=False):
    """star_options for a call, or None when the caller left everything at its default (the plain
    entry point is called then)."""
    if kernel is None and queue_threshold is None and not direct_norms:
        return None
    return _Options(int(kernel or 0), OPT_DIRECT_NORMS if direct_norms else 0, int(queue_threshold or 0))


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libstar.so.  Builds it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from . import build as _build
        _build.build_library(force=True)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.star_group_update.restype = ctypes.c_int
    lib.star_group_update.argtypes = [vp, vp, vp, ctypes.c_int, i64, i32, vp, vp, vp, vp]
    lib.star_group_update_noalloc.restype = ctypes.c_int
    lib.star_group_update_noalloc.argtypes = [vp, vp, vp, ctypes.c_int, i64, i32, vp, vp, vp, vp]
    lib.star_group_update_publish.restype = ctypes.c_int
    lib.star_group_update_publish.argtypes = [vp, vp, vp, ctypes.c_int, i64, i32, vp, vp, vp, vp, ctypes.c_int, vp]
    lib.star_group_norms.restype = ctypes.c_int
    lib.star_group_norms.argtypes = [vp, ctypes.c_int, i64, i32, vp, i32, vp, vp]
    lib.star_group_reduce.restype = ctypes.c_int
    lib.star_group_reduce.argtypes = [vp, ctypes.c_int, vp, ctypes.c_int, i64, i32, vp, i32, vp, vp]
    lib.star_plan_affine.restype = ctypes.c_int
    lib.star_plan_affine.argtypes = [i32, vp, vp, vp, vp]
    lib.star_plan_choice.restype = ctypes.c_int
    lib.star_plan_choice.argtypes = [i64, i32, ctypes.c_int, vp, vp, i32, i32, vp, vp]
    lib.star_group_update_opt.restype = ctypes.c_int
    lib.star_group_update_opt.argtypes = [vp, vp, vp, ctypes.c_int, i64, i32, vp, vp, vp, vp, ctypes.c_int, vp, vp]
    lib.star_group_norms_opt.restype = ctypes.c_int
    lib.star_group_norms_opt.argtypes = [vp, ctypes.c_int, i64, i32, vp, i32, vp, vp, vp]
    lib.star_group_reduce_opt.restype = ctypes.c_int
    lib.star_group_reduce_opt.argtypes = [vp, ctypes.c_int, vp, ctypes.c_int, i64, i32, vp, i32, vp, vp, vp]
    lib.star_group_gram.restype = ctypes.c_int
    lib.star_group_gram.argtypes = [vp, ctypes.c_int, i64, i32, vp, vp]
    lib.star_group_gram_opt.restype = ctypes.c_int
    lib.star_group_gram_opt.argtypes = [vp, ctypes.c_int, i64, i32, vp, vp, vp]
    lib.star_plan_even_split.restype = ctypes.c_int
    lib.star_plan_even_split.argtypes = [i32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    lib.star_plan_claims.restype = ctypes.c_int
    lib.star_plan_claims.argtypes = [i32, i32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.star_workspace_bytes.restype = ctypes.c_size_t
    lib.star_workspace_bytes.argtypes = [i64, i32, i32]
    lib.star_last_error.restype = ctypes.c_char_p
    lib.star_version.restype = ctypes.c_char_p
    lib.star_shutdown.restype = None
    _lib = lib
    return lib


def last_error() -> str:
    return load_library().star_last_error().decode()


def _check(status: int):
    if status != 0:
        raise StarError(status, last_error())


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


class UpdateStream:
    """Host-side stream of U worker groups (``star_updates`` of the C header)."""

    def __init__(self, offsets, members, staleness=None, coeff=None, lr=None):
        self.offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        self.members = np.ascontiguousarray(members, dtype=np.int32)
        self.staleness = None if staleness is None else np.ascontiguousarray(staleness, dtype=np.int32)
        self.coeff = None if coeff is None else np.ascontiguousarray(coeff, dtype=np.float32)
        self.lr = None if lr is None else np.ascontiguousarray(lr, dtype=np.float32)
        self.U = int(self.offsets.shape[0]) - 1
        self.c = _Updates(self.U, _np_ptr(self.offsets), _np_ptr(self.members), _np_ptr(self.staleness),
                          _np_ptr(self.coeff), _np_ptr(self.lr))


def _hparams(lr, momentum, weight_decay, wmode, scale_lr_by_group):
    return _HParams(float(lr), float(momentum), float(weight_decay), _WMODES[wmode] if isinstance(wmode, str) else wmode,
                    int(bool(scale_lr_by_group)))


class GradRows:
    """The gradient rows of a shard, marshalled once: the host array of device pointers, the dtype code and
    the shard length.  A parameter server writes its workers' reports into the same buffers every time; passing
    a ``GradRows`` instead of the list of tensors spares every call the per-row checks and pointer look-ups
    (about half a microsecond a row, which on a short shard is more than the kernel takes).  Holds the tensors,
    so the buffers stay alive; it describes their addresses as they are now (do not reallocate them)."""

    def __init__(self, grad_rows: Sequence):
        self.rows = list(grad_rows)
        self.P = int(next(r for r in self.rows if r is not None).shape[0])
        self.ptrs, self.dtype = _rows(self.rows, self.P)

    def __len__(self):
        return len(self.rows)

    def __iter__(self):
        return iter(self.rows)

    def __getitem__(self, i):
        return self.rows[i]


def _rows(grad_rows: Sequence, P: int):
    """(host array of device pointers, dtype code) for a list of 1-D tensors."""
    if isinstance(grad_rows, GradRows):
        if grad_rows.P != P:
            raise ValueError("every gradient row must be a contiguous 1-D tensor of the shard's length")
        return grad_rows.ptrs, grad_rows.dtype
    import torch
    W = len(grad_rows)
    ptrs = (ctypes.c_void_p * max(W, 1))()
    dt = None
    for w, r in enumerate(grad_rows):
        if r is None:
            ptrs[w] = None
            continue
        if r.dtype == torch.float32:
            d = F32
        elif r.dtype == torch.bfloat16:
            d = BF16
        else:
            raise TypeError("gradient rows must be float32 or bfloat16 tensors")
        if dt is not None and d != dt:
            raise TypeError("all gradient rows must share one dtype")
        dt = d
        if not r.is_contiguous() or r.dim() != 1 or r.shape[0] != P:
            raise ValueError("every gradient row must be a contiguous 1-D tensor of the shard's length")
        ptrs[w] = r.data_ptr()
    return ptrs, (F32 if dt is None else dt)


def _stream_handle(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def star_group_update(params, momentum, grad_rows: Sequence, updates: UpdateStream, *, lr: float, momentum_coef: float,
                      weight_decay: float = 0.0, wmode="mean", scale_lr_by_group: bool = False, norms_out=None,
                      stream=None, kernel=None, queue_threshold=None, direct_norms: bool = False) -> None:
    """U group updates of one shard, in place, enqueued on ``stream``
    (default: torch's current stream).  ``params``/``momentum``: float32 CUDA
    tensors [P]; ``grad_rows``: W tensors [P] (float32 or bfloat16);
    ``norms_out``: float32 CUDA tensor [U] or None.  ``kernel`` /
    ``queue_threshold`` / ``direct_norms``: the fields of ``star_options`` (the
    call then goes through ``star_group_update_opt``)."""
    lib = load_library()
    P = int(params.shape[0])
    if not (params.is_contiguous() and momentum.is_contiguous()) or momentum.shape[0] != P:
        raise ValueError("params and momentum must be contiguous and of equal length")
    ptrs, dt = _rows(grad_rows, P)
    hp = _hparams(lr, momentum_coef, weight_decay, wmode, scale_lr_by_group)
    if norms_out is not None and (norms_out.shape[0] < updates.U or not norms_out.is_contiguous()):
        raise ValueError("norms_out must hold U floats")
    opt = _options(kernel, queue_threshold, direct_norms)
    n_ptr = None if norms_out is None else norms_out.data_ptr()
    if opt is None:
        _check(lib.star_group_update(params.data_ptr(), momentum.data_ptr(), ptrs, dt, P, len(grad_rows),
                                     ctypes.byref(updates.c), ctypes.byref(hp), n_ptr, _stream_handle(stream)))
    else:
        _check(lib.star_group_update_opt(params.data_ptr(), momentum.data_ptr(), ptrs, dt, P, len(grad_rows),
                                         ctypes.byref(updates.c), ctypes.byref(hp), n_ptr, None, F32,
                                         ctypes.byref(opt), _stream_handle(stream)))


def star_group_update_noalloc(params, momentum, grad_rows: Sequence, updates: UpdateStream, *, lr: float,
                              momentum_coef: float, weight_decay: float = 0.0, wmode="mean",
                              scale_lr_by_group: bool = False, norms_out=None, stream=None) -> None:
    """star_group_update through the entry point that allocates no device memory
    (its workspace is a fixed array inside the library); at most 256 updates."""
    lib = load_library()
    P = int(params.shape[0])
    if not (params.is_contiguous() and momentum.is_contiguous()) or momentum.shape[0] != P:
        raise ValueError("params and momentum must be contiguous and of equal length")
    ptrs, dt = _rows(grad_rows, P)
    hp = _hparams(lr, momentum_coef, weight_decay, wmode, scale_lr_by_group)
    if norms_out is not None and (norms_out.shape[0] < updates.U or not norms_out.is_contiguous()):
        raise ValueError("norms_out must hold U floats")
    _check(lib.star_group_update_noalloc(params.data_ptr(), momentum.data_ptr(), ptrs, dt, P, len(grad_rows),
                                         ctypes.byref(updates.c), ctypes.byref(hp),
                                         None if norms_out is None else norms_out.data_ptr(), _stream_handle(stream)))


def star_group_update_publish(params, momentum, grad_rows: Sequence, updates: UpdateStream, publish, *, lr: float,
                              momentum_coef: float, weight_decay: float = 0.0, wmode="mean",
                              scale_lr_by_group: bool = False, norms_out=None, stream=None, kernel=None,
                              queue_threshold=None, direct_norms: bool = False) -> None:
    """star_group_update that also writes the updated parameters into ``publish``
    (float32 or bfloat16 CUDA tensor [P]) in the same pass."""
    import torch
    lib = load_library()
    P = int(params.shape[0])
    if not (params.is_contiguous() and momentum.is_contiguous()) or momentum.shape[0] != P:
        raise ValueError("params and momentum must be contiguous and of equal length")
    if publish.shape[0] != P or not publish.is_contiguous() or publish.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("publish must be a contiguous float32 or bfloat16 tensor of the shard's length")
    ptrs, dt = _rows(grad_rows, P)
    hp = _hparams(lr, momentum_coef, weight_decay, wmode, scale_lr_by_group)
    if norms_out is not None and (norms_out.shape[0] < updates.U or not norms_out.is_contiguous()):
        raise ValueError("norms_out must hold U floats")
    opt = _options(kernel, queue_threshold, direct_norms)
    n_ptr = None if norms_out is None else norms_out.data_ptr()
    pdt = F32 if publish.dtype == torch.float32 else BF16
    if opt is None:
        _check(lib.star_group_update_publish(params.data_ptr(), momentum.data_ptr(), ptrs, dt, P, len(grad_rows),
                                             ctypes.byref(updates.c), ctypes.byref(hp), n_ptr, publish.data_ptr(),
                                             pdt, _stream_handle(stream)))
    else:
        _check(lib.star_group_update_opt(params.data_ptr(), momentum.data_ptr(), ptrs, dt, P, len(grad_rows),
                                         ctypes.byref(updates.c), ctypes.byref(hp), n_ptr, publish.data_ptr(), pdt,
                                         ctypes.byref(opt), _stream_handle(stream)))


def star_group_norms(grad_rows: Sequence, updates: UpdateStream, norms_out, *, wmode="mean", stream=None,
                     kernel=None, queue_threshold=None, direct_norms: bool = False) -> None:
    lib = load_library()
    P = int(next(r for r in grad_rows if r is not None).shape[0])
    ptrs, dt = _rows(grad_rows, P)
    if norms_out.shape[0] < updates.U or not norms_out.is_contiguous():
        raise ValueError("norms_out must hold U floats")
    opt = _options(kernel, queue_threshold, direct_norms)
    wm = _WMODES[wmode] if isinstance(wmode, str) else wmode
    if opt is None:
        _check(lib.star_group_norms(ptrs, dt, P, len(grad_rows), ctypes.byref(updates.c), wm, norms_out.data_ptr(),
                                    _stream_handle(stream)))
    else:
        _check(lib.star_group_norms_opt(ptrs, dt, P, len(grad_rows), ctypes.byref(updates.c), wm,
                                        norms_out.data_ptr(), ctypes.byref(opt), _stream_handle(stream)))


def star_group_reduce(out_rows: Sequence, grad_rows: Sequence, updates: UpdateStream, *, wmode="mean", norms_out=None,
                      stream=None, kernel=None, queue_threshold=None) -> None:
    """out_rows[u] = weighted sum of group u's gradient rows (float32 or bfloat16
    CUDA tensors [P], one per group), enqueued on ``stream``."""
    import torch
    lib = load_library()
    P = int(next(r for r in grad_rows if r is not None).shape[0])
    ptrs, dt = _rows(grad_rows, P)
    if len(out_rows) != updates.U:
        raise ValueError("one output row per group is required")
    optrs, odt = _rows(out_rows, P)
    if norms_out is not None and (norms_out.shape[0] < updates.U or not norms_out.is_contiguous()):
        raise ValueError("norms_out must hold U floats")
    opt = _options(kernel, queue_threshold)
    wm = _WMODES[wmode] if isinstance(wmode, str) else wmode
    n_ptr = None if norms_out is None else norms_out.data_ptr()
    if opt is None:
        _check(lib.star_group_reduce(optrs, odt, ptrs, dt, P, len(grad_rows), ctypes.byref(updates.c), wm, n_ptr,
                                     _stream_handle(stream)))
    else:
        _check(lib.star_group_reduce_opt(optrs, odt, ptrs, dt, P, len(grad_rows), ctypes.byref(updates.c), wm, n_ptr,
                                         ctypes.byref(opt), _stream_handle(stream)))


def star_plan_affine(W: int, updates: UpdateStream, *, lr: float, momentum_coef: float, weight_decay: float = 0.0,
                     wmode="mean", scale_lr_by_group: bool = False):
    """Host-only: (M [2,2], B [2,W]) of the collapsed map, float64."""
    lib = load_library()
    hp = _hparams(lr, momentum_coef, weight_decay, wmode, scale_lr_by_group)
    M = np.zeros(4, dtype=np.float64)
    B = np.zeros(2 * max(W, 1), dtype=np.float64)
    _check(lib.star_plan_affine(W, ctypes.byref(updates.c), ctypes.byref(hp), _np_ptr(M), _np_ptr(B)))
    return M.reshape(2, 2), B[:2 * W].reshape(2, W)


def star_plan_choice(P: int, W: int, grad_dtype, updates: UpdateStream, *, lr: float = 0.0, momentum_coef: float = 0.0,
                     weight_decay: float = 0.0, wmode="mean", scale_lr_by_group: bool = False, update: bool = True,
                     want_norms: bool = False, kernel=None, queue_threshold=None, direct_norms: bool = False) -> dict:
    """Host-only: what the library would launch for this call (the fields of
    ``star_plan_info``).  ``grad_dtype``: "f32" | "bf16" or the dtype code."""
    lib = load_library()
    hp = _hparams(lr, momentum_coef, weight_decay, wmode, scale_lr_by_group)
    dt = {"f32": F32, "bf16": BF16}.get(grad_dtype, grad_dtype)
    info = _PlanInfo()
    opt = _options(kernel, queue_threshold, direct_norms)
    _check(lib.star_plan_choice(P, W, dt, ctypes.byref(updates.c), ctypes.byref(hp), int(bool(update)),
                                int(bool(want_norms)), None if opt is None else ctypes.byref(opt), ctypes.byref(info)))
    return {name: getattr(info, name) for name, _ in _PlanInfo._fields_}


def star_group_gram(grad_rows: Sequence, gram_out, *, stream=None, kernel=None, queue_threshold=None) -> None:
    """gram_out (float64 CUDA tensor [W, W]) = Gram matrix of the W gradient rows."""
    lib = load_library()
    P = int(grad_rows[0].shape[0])
    ptrs, dt = _rows(grad_rows, P)
    W = len(grad_rows)
    if gram_out.numel() != W * W or not gram_out.is_contiguous() or gram_out.element_size() != 8:
        raise ValueError("gram_out must be a contiguous float64 tensor of W*W elements")
    opt = _options(kernel, queue_threshold)
    if opt is None:
        _check(lib.star_group_gram(ptrs, dt, P, W, gram_out.data_ptr(), _stream_handle(stream)))
    else:
        _check(lib.star_group_gram_opt(ptrs, dt, P, W, gram_out.data_ptr(), ctypes.byref(opt), _stream_handle(stream)))


def star_noise_scale(gram, batch_per_worker: float):
    """Host-only: (grad_sq, trace_cov, noise_scale) from a W x W Gram matrix (numpy float64)."""
    lib = load_library()
    g = np.ascontiguousarray(gram, dtype=np.float64)
    W = int(g.shape[0])
    a, b, c = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_double(0)
    lib.star_noise_scale.restype = ctypes.c_int
    _check(lib.star_noise_scale(ctypes.c_int32(W), _np_ptr(g), ctypes.c_double(batch_per_worker), ctypes.byref(a),
                                ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


class _ModeChoice(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("x", ctypes.c_int32), ("n_groups", ctypes.c_int32),
                ("n_stragglers", ctypes.c_int32), ("n_clusters", ctypes.c_int32),
                ("time_to_progress", ctypes.c_double)]


MODE_SSGD, MODE_ASGD, MODE_STATIC_X, MODE_DYNAMIC_X = 0, 1, 2, 3


def star_select_mode_ps(iter_time, phi: float, batch_total: float, *, straggler_threshold: float = 0.2,
                        cluster_threshold: float = 0.2):
    """Host-only STAR-H for the parameter-server architecture.  Returns a dict:
    mode, x, time_to_progress, n_stragglers, n_clusters, time_static [N], time_dynamic,
    groups (list of lists of worker ids, fastest first), is_straggler [N]."""
    lib = load_library()
    t = np.ascontiguousarray(iter_time, dtype=np.float64)
    N = int(t.shape[0])
    ch = _ModeChoice()
    ts = np.zeros(max(N, 1), dtype=np.float64)
    td = ctypes.c_double(0)
    offs = np.zeros(N + 1, dtype=np.int32)
    mem = np.zeros(max(N, 1), dtype=np.int32)
    strag = np.zeros(max(N, 1), dtype=np.int32)
    lib.star_select_mode_ps.restype = ctypes.c_int
    st = lib.star_select_mode_ps(ctypes.c_int32(N), _np_ptr(t), ctypes.c_double(phi), ctypes.c_double(batch_total),
                                 ctypes.c_double(straggler_threshold), ctypes.c_double(cluster_threshold),
                                 ctypes.byref(ch), _np_ptr(ts), ctypes.byref(td), _np_ptr(offs), _np_ptr(mem),
                                 _np_ptr(strag))
    if st != 0:
        raise StarError(st, "star_select_mode_ps rejected its arguments")
    groups = [mem[offs[g]:offs[g + 1]].tolist() for g in range(ch.n_groups)]
    return {"mode": ch.mode, "x": ch.x, "time_to_progress": ch.time_to_progress, "n_stragglers": ch.n_stragglers,
            "n_clusters": ch.n_clusters, "time_static": ts[:N].copy(), "time_dynamic": td.value, "groups": groups,
            "offsets": offs[:ch.n_groups + 1].copy(), "members": mem[:N].copy(),
            "is_straggler": strag[:N].astype(bool)}


def star_select_mode_ar(iter_time, child_time, phi: float, batch_total: float, wait_candidates, *,
                        straggler_threshold: float = 0.2):
    """Host-only STAR-H for the all-reduce architecture: (removed x, wait t_w, T_a, table)."""
    lib = load_library()
    t = np.ascontiguousarray(iter_time, dtype=np.float64)
    c = np.ascontiguousarray(child_time, dtype=np.float64)
    w = np.ascontiguousarray(wait_candidates, dtype=np.float64)
    N, nw = int(t.shape[0]), int(w.shape[0])
    x, tw, ta = ctypes.c_int32(0), ctypes.c_double(0), ctypes.c_double(0)
    table = np.full(1 + N * max(nw, 1), np.nan, dtype=np.float64)
    lib.star_select_mode_ar.restype = ctypes.c_int
    st = lib.star_select_mode_ar(ctypes.c_int32(N), _np_ptr(t), _np_ptr(c), ctypes.c_double(phi),
                                 ctypes.c_double(batch_total), ctypes.c_double(straggler_threshold),
                                 ctypes.c_int32(nw), _np_ptr(w) if nw else None, ctypes.byref(x), ctypes.byref(tw),
                                 ctypes.byref(ta), _np_ptr(table))
    if st != 0:
        raise StarError(st, "star_select_mode_ar rejected its arguments")
    return x.value, tw.value, ta.value, table


def star_plan_even_split(workgroups: int, tiles: int):
    """Host-only: (first_tile [G], count [G]) of a short shard's tiles under a launch in queue order."""
    first = np.zeros(max(workgroups, 1), dtype=np.int64)
    count = np.zeros(max(workgroups, 1), dtype=np.int32)
    _check(load_library().star_plan_even_split(workgroups, ctypes.c_int64(tiles), first.ctypes.data, count.ctypes.data))
    return first, count


def star_plan_claims(workgroups: int, tiles_per_claim: int = 3):
    """(first_tile[G], count[G], base) of the work queue's fixed first round."""
    first = np.zeros(max(workgroups, 1), np.int64)
    count = np.zeros(max(workgroups, 1), np.int32)
    base = ctypes.c_int64(0)
    _check(load_library().star_plan_claims(workgroups, tiles_per_claim, first.ctypes.data, count.ctypes.data,
                                           ctypes.byref(base)))
    return first, count, int(base.value)


def star_workspace_bytes(P: int, W: int, U: int) -> int:
    return int(load_library().star_workspace_bytes(P, W, U))


def star_version() -> str:
    return load_library().star_version().decode()


def star_shutdown() -> None:
    load_library().star_shutdown()
