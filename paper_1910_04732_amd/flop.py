"""Thin ctypes binding over ``libflop_hip.so`` (the C ABI of ``include/flop.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.
PyTorch supplies device memory (tensors) and the stream.  Functions carry the
names of the C entry points; each takes torch tensors living on the GPU,
derives pointers and leading dimensions from them and raises ``FlopError`` on
a non-zero status.  There is no CPU fallback: if the library has not been
built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflop_hip.so")

FLOP_F32, FLOP_BF16 = 0, 1
FLOP_GATE_TRAIN, FLOP_GATE_DETERMINISTIC = 0, 1
FLOP_STATIC_SCRATCH_BYTES = 16 << 20
FLOP_OP_FWD, FLOP_OP_BWD, FLOP_OP_EXPECTED_L0, FLOP_OP_COMPACT, FLOP_OP_EMBED_FWD, FLOP_OP_EMBED_BWD, FLOP_OP_GATE_GRAD = range(7)


class FlopError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({status_string(status)})")
        self.status = status


class flop_hc(ctypes.Structure):
    _fields_ = [("beta", ctypes.c_float), ("l", ctypes.c_float), ("r", ctypes.c_float)]


class flop_embed_cluster(ctypes.Structure):
    _fields_ = [("id_begin", ctypes.c_int64), ("id_end", ctypes.c_int64), ("dim", ctypes.c_int64),
                ("E", ctypes.c_void_p), ("lde", ctypes.c_int64), ("O", ctypes.c_void_p), ("ldo", ctypes.c_int64),
                ("z", ctypes.c_void_p), ("dzda", ctypes.c_void_p), ("dE", ctypes.c_void_p), ("ldde", ctypes.c_int64),
                ("dO", ctypes.c_void_p), ("lddo", ctypes.c_int64), ("dlog_alpha", ctypes.c_void_p)]


class flop_gate_grad_pending(ctypes.Structure):
    _fields_ = [("partial", ctypes.c_void_p), ("z", ctypes.c_void_p), ("dzda", ctypes.c_void_p),
                ("dlog_alpha", ctypes.c_void_p), ("r_active", ctypes.c_void_p), ("r", ctypes.c_int64),
                ("chunks", ctypes.c_int32), ("accumulate", ctypes.c_int32)]


class flop_weight_grad_pending(ctypes.Structure):
    _fields_ = [("dtype", ctypes.c_int32), ("n", ctypes.c_int64), ("d", ctypes.c_int64), ("r", ctypes.c_int64),
                ("dout", ctypes.c_int64),
                ("dy", ctypes.c_void_p), ("lddy", ctypes.c_int64), ("g", ctypes.c_void_p), ("ldg", ctypes.c_int64),
                ("dh", ctypes.c_void_p), ("ldh", ctypes.c_int64), ("x", ctypes.c_void_p), ("ldx", ctypes.c_int64),
                ("dP", ctypes.c_void_p), ("lddp", ctypes.c_int64), ("dQ", ctypes.c_void_p), ("lddq", ctypes.c_int64),
                ("split_ws", ctypes.c_void_p), ("split_bytes", ctypes.c_size_t)]


class flop_boundary_job(ctypes.Structure):
    _fields_ = [("items", ctypes.POINTER(flop_gate_grad_pending)), ("count", ctypes.c_int32),
                ("log_alpha", ctypes.c_void_p), ("u", ctypes.c_void_p), ("n_gates", ctypes.c_int64), ("hc", flop_hc),
                ("z", ctypes.c_void_p), ("dzda", ctypes.c_void_p), ("w", ctypes.c_void_p),
                ("l0_sum", ctypes.c_void_p), ("l0_grad", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class flop_trace_record(ctypes.Structure):
    _fields_ = [("kernel_id", ctypes.c_int), ("tiles", ctypes.c_int),
                ("flops", ctypes.c_double), ("ms", ctypes.c_float)]


_lib = None
_vp, _i64, _int, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t


def lib():
    """The loaded C-ABI library.  Raises when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with "
                "`python -c 'import __graft_entry__ as g; g.build()'` (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        L.flop_status_string.argtypes = [_int]
        L.flop_status_string.restype = ctypes.c_char_p
        L.flop_workspace_bytes.argtypes = [_int, _int, _i64, _i64, _i64, _i64]
        L.flop_workspace_bytes.restype = _sz
        L.flop_gate_sample.argtypes = [_vp, _vp, _i64, flop_hc, _int, _vp, _vp, _vp]
        L.flop_fwd.argtypes = [_int] + [_i64] * 4 + [_vp, _i64] * 3 + [_vp, _vp, _i64, _vp, _i64, _vp, _sz, _vp]
        L.flop_bwd.argtypes = ([_int] + [_i64] * 4 + [_vp, _i64] * 4 + [_vp, _vp, _vp, _i64]
                               + [_vp, _i64] * 3 + [_vp, _int, _vp, _sz, _vp])
        L.flop_bwd_static.argtypes = L.flop_bwd.argtypes[:-3] + [_vp]
        L.flop_bwd_static.restype = _int
        L.flop_bwd_deferred.argtypes = L.flop_bwd.argtypes + [ctypes.POINTER(flop_gate_grad_pending)]
        L.flop_bwd_boundary.argtypes = L.flop_bwd.argtypes[:-1] + [ctypes.POINTER(flop_boundary_job), _vp]
        L.flop_fwd_sampling.argtypes = ([_int] + [_i64] * 4 + [_vp, _i64] * 3 + [ctypes.POINTER(flop_boundary_job), _i64]
                                        + [_vp, _i64, _vp, _i64, _vp, _sz, _vp])
        L.flop_gate_grad_finish.argtypes = [ctypes.POINTER(flop_gate_grad_pending), ctypes.c_int32, _vp]
        L.flop_bwd_defer_weights.argtypes = L.flop_bwd.argtypes + [ctypes.POINTER(flop_gate_grad_pending),
                                                                   ctypes.POINTER(flop_weight_grad_pending)]
        L.flop_weight_grad_finish.argtypes = [ctypes.POINTER(flop_weight_grad_pending), ctypes.c_int32, _vp]
        L.flop_mfma_probe.argtypes = [ctypes.c_int, _i64, ctypes.c_int32, _vp, ctypes.POINTER(ctypes.c_double), _vp]
        L.flop_step_boundary.argtypes = [ctypes.POINTER(flop_gate_grad_pending), ctypes.c_int32, _vp, _vp, _i64, flop_hc,
                                         _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.flop_expected_l0.argtypes = [_vp, _vp, _i64, flop_hc, _vp, _vp, _vp, _sz, _vp]
        L.flop_compact.argtypes = ([_int] + [_i64] * 3 + [_vp, _vp, _i64, _vp, _i64, _int, _vp, _vp]
                                   + [_vp, _i64, _vp, _i64, _vp, _vp, _sz, _vp])
        L.flop_embed_fwd.argtypes = [_int, _i64, _vp, ctypes.c_int32, ctypes.POINTER(flop_embed_cluster), _i64,
                                     _vp, _i64, _vp, _sz, _vp]
        L.flop_embed_bwd.argtypes = [_int, _i64, ctypes.c_int32, ctypes.POINTER(flop_embed_cluster), _i64, _vp, _i64,
                                     _vp, _sz, _vp, _vp, _vp, _sz, _vp]
        L.flop_embed_fwd.restype = _int
        L.flop_embed_bwd.restype = _int
        L.flop_gate_grad.argtypes = [_int, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _vp, _int, _vp, _sz, _vp]
        L.flop_gate_grad.restype = _int
        L.flop_fwd_active.argtypes = ([_int] + [_i64] * 4 + [_vp, _i64] * 3 + [_vp, _vp, _vp, _i64, _vp, _i64,
                                      _vp, _sz, _vp])
        L.flop_bwd_active.argtypes = ([_int] + [_i64] * 4 + [_vp, _i64] * 4 + [_vp, _vp, _vp, _vp, _i64]
                                      + [_vp, _i64] * 3 + [_vp, _int, _vp, _sz, _vp])
        L.flop_gather_gates.argtypes = [_vp, _vp, _vp, _i64, _vp, _vp]
        L.flop_expand_grads.argtypes = ([_int] + [_i64] * 3 + [_vp, _vp, _vp, _i64, _vp, _i64, _vp,
                                        _vp, _i64, _vp, _i64, _vp, _vp])
        L.flop_gate_sample_l0.argtypes = [_vp, _vp, _i64, flop_hc, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
        L.flop_gate_sample_l0.restype = _int
        L.flop_topk_mask.argtypes = [_vp, _i64, _i64, _vp, flop_hc, _vp, _vp, _vp]
        L.flop_lagrangian.argtypes = [_vp, _vp, _i64, ctypes.c_float, ctypes.c_float, _vp, _vp, _int, _vp, _vp]
        L.flop_topk_mask.restype = _int
        L.flop_lagrangian.restype = _int
        L.flop_active_prepare.argtypes = ([_int] + [_i64] * 3 + [_vp, _vp, flop_hc, _vp, _i64, _vp, _i64,
                                          _vp, _vp, _vp, _vp, _vp, _i64, _vp, _i64, _vp, _vp, _vp])
        L.flop_active_prepare.restype = _int
        L.flop_fwd_active_indexed.argtypes = ([_int] + [_i64] * 4 + [_vp, _i64] * 3 + [_vp, _vp, _vp, _vp, _i64, _vp, _i64, _vp])
        L.flop_bwd_active_indexed.argtypes = ([_int] + [_i64] * 4 + [_vp, _i64] * 4 + [_vp, _vp, _vp, _vp, _vp, _i64]
                                              + [_vp, _i64] * 3 + [_vp, _int, _vp, _sz, _vp])
        for name in ("flop_fwd_active", "flop_bwd_active", "flop_gather_gates", "flop_expand_grads",
                     "flop_fwd_active_indexed", "flop_bwd_active_indexed"):
            getattr(L, name).restype = _int
        L.flop_bench_force_tile_shape.argtypes = [_int]
        L.flop_bench_phases_begin.argtypes = []
        L.flop_bench_phases_read.argtypes = [_int, _vp, _int]
        L.flop_bench_force_tile_shape.restype = _int
        L.flop_bench_tile_shapes.restype = _int
        L.flop_bench_tile_shape_name.argtypes = [_int]
        L.flop_bench_tile_shape_name.restype = ctypes.c_char_p
        L.flop_trace_begin.argtypes = [_int]
        L.flop_trace_end.argtypes = [ctypes.POINTER(flop_trace_record), _int, ctypes.POINTER(_int)]
        for name in ("flop_trace_begin", "flop_trace_end", "flop_gate_sample", "flop_fwd", "flop_bwd", "flop_expected_l0", "flop_compact"):
            getattr(L, name).restype = _int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().flop_status_string(int(status)).decode()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FLOP_F32
    if t.dtype == torch.bfloat16:
        return FLOP_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _mat(t: torch.Tensor, name: str):
    """(pointer, leading dimension) of a row-major 2-D device tensor."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or not t.is_cuda:
        raise ValueError(f"{name}: need a 2-D device tensor with unit column stride")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])
    return _ptr(t), int(ld)


def _vec(t: Optional[torch.Tensor], name: str, dtype=torch.float32):
    if t is None:
        return None
    if t.dim() != 1 or not t.is_contiguous() or t.dtype != dtype or not t.is_cuda:
        raise ValueError(f"{name}: need a contiguous 1-D {dtype} device tensor")
    return _ptr(t)


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status: int, what: str):
    if status != 0:
        raise FlopError(status, what)


def flop_workspace_bytes(op: int, dt: int, n: int, d: int, r: int, dout: int) -> int:
    return int(lib().flop_workspace_bytes(op, dt, n, d, r, dout))


def workspace(nbytes: int, device) -> Optional[torch.Tensor]:
    """A 256-byte aligned device buffer (torch's allocator aligns to 512 bytes)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def flop_gate_sample(log_alpha, u, hc: flop_hc, mode: int, z, dzda=None, stream=None):
    n = log_alpha.numel()
    _check(lib().flop_gate_sample(_vec(log_alpha, "log_alpha"), _vec(u, "u"), n, hc, mode,
                                  _vec(z, "z"), _vec(dzda, "dzda"), _stream(stream)), "flop_gate_sample")
    return z, dzda


def flop_fwd(x, Q, P, z, g_saved, y, ws=None, stream=None):
    dt = _dt(x)
    n, d = x.shape
    r, dout = Q.shape[0], P.shape[0]
    assert Q.shape == (r, d) and P.shape == (dout, r) and g_saved.shape == (n, r) and y.shape == (n, dout)
    assert Q.dtype == x.dtype and P.dtype == x.dtype and g_saved.dtype == x.dtype and y.dtype == x.dtype
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    gp, ldg = _mat(g_saved, "g_saved")
    yp, ldy = _mat(y, "y")
    _check(lib().flop_fwd(dt, n, d, r, dout, xp, ldx, qp, ldq, pp, ldp, _vec(z, "z"), gp, ldg, yp, ldy,
                          _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "flop_fwd")
    return y


def flop_bwd(dy, x, Q, P, z, dzda, g_saved, dx, dQ, dP, dlog_alpha, ws, accumulate=False, stream=None):
    dt = _dt(x)
    n, d = x.shape
    r, dout = Q.shape[0], P.shape[0]
    assert dy.shape == (n, dout) and Q.shape == (r, d) and P.shape == (dout, r) and g_saved.shape == (n, r)
    dyp, lddy = _mat(dy, "dy")
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    gp, ldg = _mat(g_saved, "g_saved")
    dxp, lddx = (None, 0) if dx is None else _mat(dx, "dx")
    dqp, lddq = (None, 0) if dQ is None else _mat(dQ, "dQ")
    dpp, lddp = (None, 0) if dP is None else _mat(dP, "dP")
    _check(lib().flop_bwd(dt, n, d, r, dout, dyp, lddy, xp, ldx, qp, ldq, pp, ldp,
                          _vec(z, "z"), _vec(dzda, "dzda"), gp, ldg, dxp, lddx, dqp, lddq, dpp, lddp,
                          _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0,
                          _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "flop_bwd")
    return dx, dQ, dP, dlog_alpha


def flop_bwd_static(dy, x, Q, P, z, dzda, g_saved, dx, dQ, dP, dlog_alpha, accumulate=False, stream=None):
    """flop_bwd with its scratch in the library's static device array: no workspace argument, no allocation."""
    dt = _dt(x)
    n, d = x.shape
    r, dout = Q.shape[0], P.shape[0]
    assert dy.shape == (n, dout) and Q.shape == (r, d) and P.shape == (dout, r) and g_saved.shape == (n, r)
    dyp, lddy = _mat(dy, "dy")
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    gp, ldg = _mat(g_saved, "g_saved")
    dxp, lddx = (None, 0) if dx is None else _mat(dx, "dx")
    dqp, lddq = (None, 0) if dQ is None else _mat(dQ, "dQ")
    dpp, lddp = (None, 0) if dP is None else _mat(dP, "dP")
    _check(lib().flop_bwd_static(dt, n, d, r, dout, dyp, lddy, xp, ldx, qp, ldq, pp, ldp,
                                 _vec(z, "z"), _vec(dzda, "dzda"), gp, ldg, dxp, lddx, dqp, lddq, dpp, lddp,
                                 _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0, _stream(stream)),
           "flop_bwd_static")
    return dx, dQ, dP, dlog_alpha


def flop_bwd_deferred(dy, x, Q, P, z, dzda, g_saved, dx, dQ, dP, dlog_alpha, ws, accumulate=False, stream=None):
    """flop_bwd without the last stage of the gate gradient; returns the pending item for flop_gate_grad_finish.
    ``ws`` (and z, dzda, dlog_alpha) must stay alive and untouched until that call."""
    dt = _dt(x)
    n, d = x.shape
    r, dout = Q.shape[0], P.shape[0]
    assert dy.shape == (n, dout) and Q.shape == (r, d) and P.shape == (dout, r) and g_saved.shape == (n, r)
    dyp, lddy = _mat(dy, "dy")
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    gp, ldg = _mat(g_saved, "g_saved")
    dxp, lddx = (None, 0) if dx is None else _mat(dx, "dx")
    dqp, lddq = (None, 0) if dQ is None else _mat(dQ, "dQ")
    dpp, lddp = (None, 0) if dP is None else _mat(dP, "dP")
    pending = flop_gate_grad_pending()
    _check(lib().flop_bwd_deferred(dt, n, d, r, dout, dyp, lddy, xp, ldx, qp, ldq, pp, ldp,
                                   _vec(z, "z"), _vec(dzda, "dzda"), gp, ldg, dxp, lddx, dqp, lddq, dpp, lddp,
                                   _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0,
                                   _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream), ctypes.byref(pending)),
           "flop_bwd_deferred")
    return pending


def flop_bwd_defer_weights(dy, x, Q, P, z, dzda, g_saved, dx, dQ, dP, dlog_alpha, ws, accumulate=False, stream=None):
    """flop_bwd_deferred that also leaves dP and dQ for later; returns (pending gate gradient or None, pending
    weight gradients) for flop_gate_grad_finish / flop_weight_grad_finish.  ``dy``, ``x``, ``g_saved`` and ``ws`` must
    stay alive and untouched until those calls."""
    dt = _dt(x)
    n, d = x.shape
    r, dout = Q.shape[0], P.shape[0]
    assert dy.shape == (n, dout) and Q.shape == (r, d) and P.shape == (dout, r) and g_saved.shape == (n, r)
    dyp, lddy = _mat(dy, "dy")
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    gp, ldg = _mat(g_saved, "g_saved")
    dxp, lddx = (None, 0) if dx is None else _mat(dx, "dx")
    dqp, lddq = (None, 0) if dQ is None else _mat(dQ, "dQ")
    dpp, lddp = (None, 0) if dP is None else _mat(dP, "dP")
    pending = flop_gate_grad_pending()
    weights = flop_weight_grad_pending()
    _check(lib().flop_bwd_defer_weights(dt, n, d, r, dout, dyp, lddy, xp, ldx, qp, ldq, pp, ldp,
                                        _vec(z, "z"), _vec(dzda, "dzda"), gp, ldg, dxp, lddx, dqp, lddq, dpp, lddp,
                                        _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0,
                                        _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream),
                                        ctypes.byref(pending), ctypes.byref(weights)),
           "flop_bwd_defer_weights")
    return (None if dlog_alpha is None else pending), weights


def flop_weight_grad_finish(items, stream=None):
    """dP and dQ of the given pending items (from flop_bwd_defer_weights), up to eight products to a launch."""
    arr = (flop_weight_grad_pending * max(len(items), 1))(*items)
    _check(lib().flop_weight_grad_finish(arr, len(items), _stream(stream)), "flop_weight_grad_finish")


def flop_fwd_sampling(x, Q, P, log_alpha, u, hc: flop_hc, z, dzda, l0_sum, gate_offset, g_saved, y, w=None, l0_grad=None,
                      l0_ws=None, ws=None, stream=None):
    """Gates and Eq.(3) of all ``log_alpha.numel()`` gates of the step plus flop_fwd of the layer whose gates start
    at ``gate_offset``; the gates are computed in the first product's epilogue where the shapes allow it."""
    dt = _dt(x)
    n, d = x.shape
    r, dout = Q.shape[0], P.shape[0]
    assert Q.shape == (r, d) and P.shape == (dout, r) and g_saved.shape == (n, r) and y.shape == (n, dout)
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    gp, ldg = _mat(g_saved, "g_saved")
    yp, ldy = _mat(y, "y")
    val = lambda p: None if p is None else p.value
    job = flop_boundary_job(None, 0, val(_vec(log_alpha, "log_alpha")), val(_vec(u, "u")), log_alpha.numel(), hc,
                            val(_vec(z, "z")), val(_vec(dzda, "dzda")), val(_vec(w, "w")), val(_vec(l0_sum, "l0_sum")),
                            val(_vec(l0_grad, "l0_grad")), val(_ptr(l0_ws)), 0 if l0_ws is None else l0_ws.numel())
    _check(lib().flop_fwd_sampling(dt, n, d, r, dout, xp, ldx, qp, ldq, pp, ldp, ctypes.byref(job), int(gate_offset),
                                   gp, ldg, yp, ldy, _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)),
           "flop_fwd_sampling")


def flop_bwd_boundary(dy, x, Q, P, z, dzda, g_saved, dx, dQ, dP, dlog_alpha, ws, items, log_alpha=None, u=None,
                      hc: Optional[flop_hc] = None, z_next=None, dzda_next=None, l0_sum=None, w=None, l0_grad=None,
                      l0_ws=None, accumulate=False, stream=None):
    """flop_bwd of the step's last layer with the step boundary attached: finishes ``items`` (earlier layers,
    from flop_bwd_deferred) and this layer's gate gradient and, if ``log_alpha`` is given, samples ``z_next`` /
    ``dzda_next`` and Eq.(3) for the next step, on this call's last contraction launch where the shapes allow it."""
    if hc is None:
        hc = flop_hc(1.0, -0.1, 1.1)
    dt = _dt(x)
    n, d = x.shape
    r, dout = Q.shape[0], P.shape[0]
    assert dy.shape == (n, dout) and Q.shape == (r, d) and P.shape == (dout, r) and g_saved.shape == (n, r)
    dyp, lddy = _mat(dy, "dy")
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    gp, ldg = _mat(g_saved, "g_saved")
    dxp, lddx = (None, 0) if dx is None else _mat(dx, "dx")
    dqp, lddq = (None, 0) if dQ is None else _mat(dQ, "dQ")
    dpp, lddp = (None, 0) if dP is None else _mat(dP, "dP")
    arr = (flop_gate_grad_pending * max(len(items), 1))(*items)
    val = lambda p: None if p is None else p.value
    job = flop_boundary_job(arr, len(items), val(_vec(log_alpha, "log_alpha")), val(_vec(u, "u")),
                            0 if log_alpha is None else log_alpha.numel(), hc,
                            val(_vec(z_next, "z_next")), val(_vec(dzda_next, "dzda_next")), val(_vec(w, "w")),
                            val(_vec(l0_sum, "l0_sum")), val(_vec(l0_grad, "l0_grad")), val(_ptr(l0_ws)),
                            0 if l0_ws is None else l0_ws.numel())
    _check(lib().flop_bwd_boundary(dt, n, d, r, dout, dyp, lddy, xp, ldx, qp, ldq, pp, ldp,
                                   _vec(z, "z"), _vec(dzda, "dzda"), gp, ldg, dxp, lddx, dqp, lddq, dpp, lddp,
                                   _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0,
                                   _ptr(ws), 0 if ws is None else ws.numel(), ctypes.byref(job), _stream(stream)),
           "flop_bwd_boundary")


def flop_gate_grad_finish(items, stream=None):
    """Finishes the gate gradients of the given pending items (from flop_bwd_deferred), sixteen to a launch."""
    arr = (flop_gate_grad_pending * max(len(items), 1))(*items)
    _check(lib().flop_gate_grad_finish(arr, len(items), _stream(stream)), "flop_gate_grad_finish")


def flop_mfma_probe(dt: int, iters: int, blocks: int, sink, stream=None) -> float:
    """Launch the matrix-core rate probe; returns the flop count of the launch (the caller times it)."""
    fl = ctypes.c_double(0.0)
    _check(lib().flop_mfma_probe(dt, int(iters), int(blocks), _vec(sink, "sink"), ctypes.byref(fl), _stream(stream)),
           "flop_mfma_probe")
    return fl.value


def flop_step_boundary(items, log_alpha, u, hc: flop_hc, z, dzda, l0_sum, w=None, l0_grad=None, ws=None, stream=None):
    """flop_gate_grad_finish(items) and flop_gate_sample_l0(...) for the next step in one launch; ``z`` / ``dzda``
    must not be the buffers the pending items still read."""
    arr = (flop_gate_grad_pending * max(len(items), 1))(*items)
    n = log_alpha.numel()
    _check(lib().flop_step_boundary(arr, len(items), _vec(log_alpha, "log_alpha"), _vec(u, "u"), n, hc,
                                    _vec(z, "z"), _vec(dzda, "dzda"), _vec(w, "w"), _vec(l0_sum, "l0_sum"),
                                    _vec(l0_grad, "l0_grad"), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)),
           "flop_step_boundary")


def flop_fwd_active(x, Qc, Pc, zc, r_active, g_saved, y, ws=None, stream=None):
    """flop_fwd on compacted factors; ``r_active`` is the device int32 written by flop_compact."""
    dt = _dt(x)
    n, d = x.shape
    r_cap, dout = Qc.shape[0], Pc.shape[0]
    assert Qc.shape == (r_cap, d) and Pc.shape == (dout, r_cap) and g_saved.shape == (n, r_cap) and y.shape == (n, dout)
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Qc, "Qc")
    pp, ldp = _mat(Pc, "Pc")
    gp, ldg = _mat(g_saved, "g_saved")
    yp, ldy = _mat(y, "y")
    _check(lib().flop_fwd_active(dt, n, d, r_cap, dout, xp, ldx, qp, ldq, pp, ldp, _vec(zc, "zc"),
                                 _vec(r_active, "r_active", torch.int32), gp, ldg, yp, ldy,
                                 _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "flop_fwd_active")
    return y


def flop_bwd_active(dy, x, Qc, Pc, zc, dzda_c, r_active, g_saved, dx, dQc, dPc, dlog_alpha_c, ws,
                    accumulate=False, stream=None):
    dt = _dt(x)
    n, d = x.shape
    r_cap, dout = Qc.shape[0], Pc.shape[0]
    assert dy.shape == (n, dout) and Qc.shape == (r_cap, d) and Pc.shape == (dout, r_cap) and g_saved.shape == (n, r_cap)
    dyp, lddy = _mat(dy, "dy")
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Qc, "Qc")
    pp, ldp = _mat(Pc, "Pc")
    gp, ldg = _mat(g_saved, "g_saved")
    dxp, lddx = (None, 0) if dx is None else _mat(dx, "dx")
    dqp, lddq = (None, 0) if dQc is None else _mat(dQc, "dQc")
    dpp, lddp = (None, 0) if dPc is None else _mat(dPc, "dPc")
    _check(lib().flop_bwd_active(dt, n, d, r_cap, dout, dyp, lddy, xp, ldx, qp, ldq, pp, ldp,
                                 _vec(zc, "zc"), _vec(dzda_c, "dzda_c"), _vec(r_active, "r_active", torch.int32),
                                 gp, ldg, dxp, lddx, dqp, lddq, dpp, lddp,
                                 _vec(dlog_alpha_c, "dlog_alpha_c"), 1 if accumulate else 0,
                                 _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "flop_bwd_active")
    return dx, dQc, dPc, dlog_alpha_c


def flop_active_prepare(log_alpha, u, hc: flop_hc, Q, P, z, dzda, r_active, idx, Qc, Pc, zc, dzda_c, stream=None):
    """Gate sampling + compaction of Q, P + gather of dz/dalpha for one training step (two launches; one with
    ``Qc = Pc = None``, which leaves only the index list, the gates and their gathers: what the indexed calls need)."""
    dt = _dt(Q)
    r, d = Q.shape
    dout = P.shape[0] if P is not None else 0
    assert (P is None or P.shape == (dout, r)) and log_alpha.numel() == r
    qp, ldq = _mat(Q, "Q")
    pp, ldp = (None, 0) if P is None else _mat(P, "P")
    qcp, ldqc = (None, 0) if Qc is None else _mat(Qc, "Qc")
    pcp, ldpc = (None, 0) if Pc is None else _mat(Pc, "Pc")
    _check(lib().flop_active_prepare(dt, d, r, dout, _vec(log_alpha, "log_alpha"), _vec(u, "u"), hc, qp, ldq, pp, ldp,
                                     _vec(z, "z"), _vec(dzda, "dzda"), _vec(r_active, "r_active", torch.int32),
                                     _vec(idx, "idx", torch.int32), qcp, ldqc, pcp, ldpc, _vec(zc, "zc"),
                                     _vec(dzda_c, "dzda_c"), _stream(stream)), "flop_active_prepare")
    return r_active, idx


def flop_fwd_active_indexed(x, Q, Pt, zc, idx, r_active, g_active, y, stream=None):
    """Forward on the open components read in place: Q[r, d], Pt[r, dout] (P transposed), index list from
    flop_active_prepare / flop_compact; g_active[n, r] receives the first r_active columns."""
    dt = _dt(x)
    n, d = x.shape
    r, dout = Pt.shape
    assert Q.shape == (r, d) and g_active.shape == (n, r) and y.shape == (n, dout)
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldpt = _mat(Pt, "Pt")
    gp, ldg = _mat(g_active, "g_active")
    yp, ldy = _mat(y, "y")
    _check(lib().flop_fwd_active_indexed(dt, n, d, r, dout, xp, ldx, qp, ldq, pp, ldpt, _vec(zc, "zc"),
                                         _vec(idx, "idx", torch.int32), _vec(r_active, "r_active", torch.int32),
                                         gp, ldg, yp, ldy, _stream(stream)), "flop_fwd_active_indexed")
    return y


def flop_bwd_active_indexed(dy, x, Q, Pt, zc, dzda_c, idx, r_active, g_active, dx, dQ, dPt, dlog_alpha, ws,
                            accumulate=False, stream=None):
    """Backward on the open components read in place; full-size dQ[r, d], dPt[r, dout], dlog_alpha[r] with exact
    zeros for the closed components."""
    dt = _dt(x)
    n, d = x.shape
    r, dout = Pt.shape
    assert dy.shape == (n, dout) and Q.shape == (r, d) and g_active.shape == (n, r)
    dyp, lddy = _mat(dy, "dy")
    xp, ldx = _mat(x, "x")
    qp, ldq = _mat(Q, "Q")
    pp, ldpt = _mat(Pt, "Pt")
    gp, ldg = _mat(g_active, "g_active")
    dxp, lddx = (None, 0) if dx is None else _mat(dx, "dx")
    dqp, lddq = (None, 0) if dQ is None else _mat(dQ, "dQ")
    dpp, lddpt = (None, 0) if dPt is None else _mat(dPt, "dPt")
    _check(lib().flop_bwd_active_indexed(dt, n, d, r, dout, dyp, lddy, xp, ldx, qp, ldq, pp, ldpt,
                                         _vec(zc, "zc"), _vec(dzda_c, "dzda_c"), _vec(idx, "idx", torch.int32),
                                         _vec(r_active, "r_active", torch.int32), gp, ldg, dxp, lddx, dqp, lddq, dpp, lddpt,
                                         _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0,
                                         _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "flop_bwd_active_indexed")
    return dx, dQ, dPt, dlog_alpha


def flop_gather_gates(src, idx, r_active, dst, stream=None):
    _check(lib().flop_gather_gates(_vec(src, "src"), _vec(idx, "idx", torch.int32),
                                   _vec(r_active, "r_active", torch.int32), src.numel(), _vec(dst, "dst"),
                                   _stream(stream)), "flop_gather_gates")
    return dst


def flop_expand_grads(r_active, idx, dQc, dPc, dlog_alpha_c, dQ, dP, dlog_alpha, stream=None):
    """Scatter compacted gradients back to full size (exact zeros for closed components)."""
    ref = dQ if dQ is not None else dP
    dt = _dt(ref) if ref is not None else FLOP_F32
    r = idx.numel()
    d = 0 if dQ is None else dQ.shape[1]
    dout = 0 if dP is None else dP.shape[0]
    dqcp, lddqc = (None, 0) if dQc is None else _mat(dQc, "dQc")
    dpcp, lddpc = (None, 0) if dPc is None else _mat(dPc, "dPc")
    dqp, lddq = (None, 0) if dQ is None else _mat(dQ, "dQ")
    dpp, lddp = (None, 0) if dP is None else _mat(dP, "dP")
    _check(lib().flop_expand_grads(dt, d, r, dout, _vec(r_active, "r_active", torch.int32),
                                   _vec(idx, "idx", torch.int32), dqcp, lddqc, dpcp, lddpc,
                                   _vec(dlog_alpha_c, "dlog_alpha_c"), dqp, lddq, dpp, lddp,
                                   _vec(dlog_alpha, "dlog_alpha"), _stream(stream)), "flop_expand_grads")
    return dQ, dP, dlog_alpha


def flop_gate_sample_l0(log_alpha, u, hc: flop_hc, z, dzda, l0_sum, w=None, l0_grad=None, ws=None, stream=None):
    """Train-mode gates and the (weighted) expected-L0 sum with its gradient in one call."""
    _check(lib().flop_gate_sample_l0(_vec(log_alpha, "log_alpha"), _vec(u, "u"), log_alpha.numel(), hc,
                                     _vec(z, "z"), _vec(dzda, "dzda"), _vec(w, "w"), _vec(l0_sum, "l0_sum"),
                                     _vec(l0_grad, "l0_grad"), _ptr(ws), 0 if ws is None else ws.numel(),
                                     _stream(stream)), "flop_gate_sample_l0")
    return z, dzda, l0_sum, l0_grad


def flop_topk_mask(log_alpha, keep, hc: flop_hc, z, kept=None, keep_device=None, stream=None):
    """Section 4.4 mask: Eq.(3) value for the ``keep`` best gates, 0 for the rest."""
    _check(lib().flop_topk_mask(_vec(log_alpha, "log_alpha"), log_alpha.numel(), int(keep),
                                _vec(keep_device, "keep_device"), hc, _vec(z, "z"),
                                _vec(kept, "kept", torch.int32), _stream(stream)), "flop_topk_mask")
    return z


def flop_lagrangian(size_sum, size_grad, scale, t, lam, dlog_alpha, out, accumulate=False, stream=None):
    """Section 4.3 penalty: gradient for log_alpha and {g, dg/dlambda1, dg/dlambda2}."""
    n = 0 if size_grad is None else size_grad.numel()
    _check(lib().flop_lagrangian(_vec(size_sum, "size_sum"), _vec(size_grad, "size_grad"), n, float(scale), float(t),
                                 _vec(lam, "lambda"), _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0,
                                 _vec(out, "out"), _stream(stream)), "flop_lagrangian")
    return dlog_alpha, out


def flop_expected_l0(log_alpha, hc: flop_hc, out_sum, w=None, grad=None, ws=None, stream=None):
    n = log_alpha.numel()
    _check(lib().flop_expected_l0(_vec(log_alpha, "log_alpha"), _vec(w, "w"), n, hc, _vec(out_sum, "out_sum"),
                                  _vec(grad, "grad"), _ptr(ws), 0 if ws is None else ws.numel(),
                                  _stream(stream)), "flop_expected_l0")
    return out_sum, grad


def flop_compact(z, Q, P, r_out, idx, Qc=None, Pc=None, zc=None, absorb_z_into_Q=False, ws=None, stream=None):
    dt = _dt(Q)
    r, d = Q.shape
    dout = P.shape[0]
    assert P.shape == (dout, r)
    qp, ldq = _mat(Q, "Q")
    pp, ldp = _mat(P, "P")
    qcp, ldqc = (None, 0) if Qc is None else _mat(Qc, "Qc")
    pcp, ldpc = (None, 0) if Pc is None else _mat(Pc, "Pc")
    _check(lib().flop_compact(dt, d, r, dout, _vec(z, "z"), qp, ldq, pp, ldp, 1 if absorb_z_into_Q else 0,
                              _vec(r_out, "r_out", torch.int32), _vec(idx, "idx", torch.int32),
                              qcp, ldqc, pcp, ldpc, _vec(zc, "zc"),
                              _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)), "flop_compact")
    return r_out, idx


def flop_bench_force_tile_shape(shape: int):
    """Test/benchmark aid: every following bf16 transfer-kernel launch uses block shape ``shape`` (-1: automatic)."""
    _check(lib().flop_bench_force_tile_shape(int(shape)), "flop_bench_force_tile_shape")


def flop_bench_tile_shapes():
    """Names of the block shapes, indexed by shape number."""
    return [lib().flop_bench_tile_shape_name(i).decode() for i in range(lib().flop_bench_tile_shapes())]


LIB_PATH_PHASES = os.path.join(_HERE, "libflop_hip_phases.so")   # measurement build (see include/flop_bench.h)


def flop_bench_phases_begin():
    """Measurement build only: clears the per-block phase stamps; the next 16 transfer-kernel launches record."""
    _check(lib().flop_bench_phases_begin(), "flop_bench_phases_begin")


def flop_bench_phases_read(launch: int, max_blocks: int = 4096):
    """Measurement build only: ``(blocks, 5)`` int64 array of 100 MHz wall-clock stamps of launch ``launch``
    (entry, before the main loop, after it, output staged, stores complete); rows of zeros: blocks without a tile."""
    import numpy as np
    buf = np.zeros((max_blocks, 5), dtype=np.uint64)
    n = lib().flop_bench_phases_read(int(launch), buf.ctypes.data, int(max_blocks))
    _check(min(n, 0), "flop_bench_phases_read")
    return buf[:n].astype(np.int64)


def flop_trace_begin(capacity: int):
    _check(lib().flop_trace_begin(int(capacity)), "flop_trace_begin")


def flop_trace_end(max_records: int):
    """Returns a list of ``(kernel_id, tiles, flops, ms)`` in launch order."""
    buf = (flop_trace_record * max_records)()
    cnt = ctypes.c_int(0)
    _check(lib().flop_trace_end(buf, max_records, ctypes.byref(cnt)), "flop_trace_end")
    return [(buf[i].kernel_id, buf[i].tiles, buf[i].flops, buf[i].ms) for i in range(cnt.value)]


def _clusters(clusters, d):
    """Host array of flop_embed_cluster from a list of dicts of device tensors.

    Keys: id_begin, id_end, E, O, z and, for the backward pass, dzda, dE, dO, dlog_alpha (each optional)."""
    arr = (flop_embed_cluster * len(clusters))()
    for c, cl in enumerate(clusters):
        E, O = cl["E"], cl["O"]
        assert O.shape == (E.shape[1], d) and E.shape[0] == cl["id_end"] - cl["id_begin"] and E.dtype == O.dtype
        arr[c].id_begin, arr[c].id_end, arr[c].dim = int(cl["id_begin"]), int(cl["id_end"]), int(E.shape[1])
        ep, lde = _mat(E, "E")
        op, ldo = _mat(O, "O")
        arr[c].E, arr[c].lde, arr[c].O, arr[c].ldo = ep.value, lde, op.value, ldo
        arr[c].z = cl["z"].data_ptr() if _vec(cl["z"], "z") is not None else None
        if cl.get("dzda") is not None:
            arr[c].dzda = _vec(cl["dzda"], "dzda").value
        if cl.get("dE") is not None:
            p, ld = _mat(cl["dE"], "dE")
            arr[c].dE, arr[c].ldde = p.value, ld
        if cl.get("dO") is not None:
            p, ld = _mat(cl["dO"], "dO")
            arr[c].dO, arr[c].lddo = p.value, ld
        if cl.get("dlog_alpha") is not None:
            arr[c].dlog_alpha = _vec(cl["dlog_alpha"], "dlog_alpha").value
    return arr


def flop_embed_fwd(ids, clusters, y, saved, stream=None):
    n, d = y.shape
    assert ids.dtype == torch.int64 and ids.is_contiguous() and ids.numel() == n
    arr = _clusters(clusters, d)
    yp, ldy = _mat(y, "y")
    _check(lib().flop_embed_fwd(_dt(y), n, _ptr(ids), len(clusters), arr, d, yp, ldy,
                                _ptr(saved), saved.numel(), _stream(stream)), "flop_embed_fwd")
    return y


def flop_embed_bwd(dy, clusters, saved, ws, touched_ids=None, n_touched=None, stream=None):
    n, d = dy.shape
    arr = _clusters(clusters, d)
    dyp, lddy = _mat(dy, "dy")
    _check(lib().flop_embed_bwd(_dt(dy), n, len(clusters), arr, d, dyp, lddy, _ptr(saved), saved.numel(),
                                _ptr(touched_ids), _ptr(n_touched), _ptr(ws), ws.numel(), _stream(stream)),
           "flop_embed_bwd")


def flop_gate_grad(dh, g, z, dzda, dlog_alpha, ws, accumulate=False, stream=None):
    n, r = dh.shape
    assert g.shape == (n, r) and g.dtype == dh.dtype
    hp, ldh = _mat(dh, "dh")
    gp, ldg = _mat(g, "g")
    _check(lib().flop_gate_grad(_dt(dh), n, r, hp, ldh, gp, ldg, _vec(z, "z"), _vec(dzda, "dzda"),
                                _vec(dlog_alpha, "dlog_alpha"), 1 if accumulate else 0,
                                _ptr(ws), ws.numel(), _stream(stream)), "flop_gate_grad")
    return dlog_alpha
