"""ctypes binding of libdiloco.so: argument marshalling only.

Every function takes torch tensors (device memory) and scalars, checks nothing the
library does not check itself, passes raw device pointers plus the current HIP stream,
and raises DilocoError on a non-zero status.  There is no fallback: if the shared
library has not been built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdiloco.so")

F32, BF16 = 0, 1
EAGER, DELAYED = 0, 1
COMM_BF16 = 0x100   # OR into `variant`: outer gradients cross the wire in bf16
STATE_NO_MEAN = 0x400   # OR into an EAGER `variant`: the previous mean is formed from prev_local, not kept


def COMM_EXMY(E: int, Mn: int, bias: int) -> int:
    """OR into `variant`: outer gradients cross the wire in the small-float format with E exponent
    bits, Mn mantissa bits and the given exponent bias (DILOCO_COMM_EXMY of the header)."""
    if not (0 <= E <= 15 and 0 <= Mn <= 15 and -128 <= bias <= 127):
        raise ValueError("format fields out of range")
    return 0x200 | (E << 12) | (Mn << 16) | ((bias & 0xFF) << 20)
STATE_TILE = 8192    # DILOCO_STATE_TILE: elements per stream and tile of the packed outer state

OK, ERR_NULL, ERR_SHAPE, ERR_ALIGN, ERR_DTYPE, ERR_HYPER, ERR_ALIAS, ERR_LAUNCH = range(8)

_c_i64 = ctypes.c_int64
_c_dbl = ctypes.c_double
_c_ptr = ctypes.c_void_p
_c_int = ctypes.c_int

# name -> (restype, argtypes): must mirror include/diloco.h and include/diloco_sim.h
SIGNATURES = {
    "diloco_strerror": (ctypes.c_char_p, [_c_int]),
    "diloco_version": (_c_int, []),
    "diloco_inner_adamw": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_int, _c_i64, _c_i64, _c_int,
                                    _c_int, _c_dbl, _c_dbl, _c_dbl, _c_dbl, _c_dbl, _c_i64, _c_ptr]),
    "diloco_outer_sync": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr,
                                   _c_dbl, _c_dbl, _c_int, _c_ptr]),
    "diloco_outer_sync_comm": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr,
                                        _c_dbl, _c_dbl, _c_int, _c_int, _c_ptr]),
    "diloco_outer_eager": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr,
                                    _c_i64, _c_ptr, _c_dbl, _c_dbl, _c_int, _c_int, _c_int, _c_ptr]),
    "diloco_reset": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_i64, _c_ptr]),
    "diloco_packed_state_elems": (_c_i64, [_c_int, _c_i64]),
    "diloco_pack_state": (_c_int, [_c_ptr, _c_int, _c_i64, _c_ptr, _c_ptr, _c_ptr, _c_i64, _c_ptr, _c_ptr]),
    "diloco_unpack_state": (_c_int, [_c_ptr, _c_int, _c_i64, _c_ptr, _c_ptr, _c_ptr, _c_i64, _c_ptr, _c_ptr]),
    "diloco_outer_eager_packed": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_dbl, _c_dbl,
                                           _c_int, _c_int, _c_int, _c_ptr]),
    "diloco_reset_packed": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr]),
    "diloco_stream_offset": (_c_i64, [_c_i64, _c_int, _c_int]),
    "diloco_stream_due": (_c_int, [_c_i64, _c_i64, _c_int, _c_int]),
    "diloco_stream_boundary_count": (_c_i64, [_c_i64, _c_i64, _c_int, _c_int]),
    "diloco_sim_quadratic_inner": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_int, _c_i64, _c_i64, _c_ptr,
                                            _c_ptr, _c_dbl, ctypes.c_uint64, _c_i64, _c_dbl, _c_dbl,
                                            _c_dbl, _c_dbl, _c_dbl, _c_i64, _c_ptr]),
    "diloco_sim_quadratic_phase": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_int, _c_i64, _c_i64, _c_ptr,
                                            _c_ptr, _c_dbl, ctypes.c_uint64, _c_i64, _c_dbl, _c_dbl,
                                            _c_dbl, _c_dbl, _c_dbl, _c_i64, _c_int, _c_ptr]),
    "diloco_sim_stream_rmw": (_c_int, [_c_ptr, _c_int, _c_i64, _c_i64, _c_ptr]),
    "diloco_sim_loss_workspace": (_c_i64, [_c_i64]),
    "diloco_sim_quadratic_loss": (_c_int, [_c_ptr, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr,
                                           _c_i64, _c_ptr, _c_ptr]),
    "diloco_sim_stream_copy": (_c_int, [_c_ptr, _c_ptr, _c_i64, _c_ptr]),
    "diloco_tune": (_c_int, [ctypes.c_char_p, _c_int]),
    "diloco_tune_get": (_c_int, [ctypes.c_char_p]),
}


class DilocoError(RuntimeError):
    def __init__(self, fn: str, status: int, text: str):
        super().__init__(f"{fn} failed with status {status}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2502_12996_amd.build` "
                "(there is no CPU or PyTorch fallback)")
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def strerror(status: int) -> str:
    return lib().diloco_strerror(status).decode()


def version() -> int:
    return lib().diloco_version()


def _check(fn: str, status: int) -> None:
    if status != 0:
        raise DilocoError(fn, status, strerror(status))


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def _row_stride(t: torch.Tensor) -> int:
    """Element stride between replicas of a [M, n] tensor whose rows are contiguous."""
    if t.dim() == 1:
        return t.shape[0]
    assert t.dim() == 2 and (t.shape[1] <= 1 or t.stride(1) == 1), "rows must be contiguous"
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def inner_adamw(theta, m1, m2, grad, *, n=None, lr, beta1, beta2, eps, weight_decay, step,
                stream=None) -> None:
    """diloco_inner_adamw on [M, stride] tensors (first n columns)."""
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    _check("diloco_inner_adamw", lib().diloco_inner_adamw(
        _ptr(theta), _ptr(m1), _ptr(m2), _ptr(grad), M, n, _row_stride(theta),
        _dtype_code(theta), _dtype_code(grad), lr, beta1, beta2, eps, weight_decay, step,
        _stream(stream)))


def outer_sync(theta, anchor, vel, *, n=None, mean_out=None, outer_lr, outer_momentum,
               nesterov=True, comm=None, stream=None) -> None:
    """diloco_outer_sync: theta [M, stride]; anchor, vel (and mean_out) [n] fp32.  comm (COMM_BF16 or
    COMM_EXMY(...)) goes through diloco_outer_sync_comm."""
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    if comm is None:
        _check("diloco_outer_sync", lib().diloco_outer_sync(
            _ptr(theta), _dtype_code(theta), M, n, _row_stride(theta), _ptr(anchor), _ptr(vel),
            _ptr(mean_out), outer_lr, outer_momentum, int(nesterov), _stream(stream)))
    else:
        _check("diloco_outer_sync_comm", lib().diloco_outer_sync_comm(
            _ptr(theta), _dtype_code(theta), M, n, _row_stride(theta), _ptr(anchor), _ptr(vel),
            _ptr(mean_out), outer_lr, outer_momentum, int(nesterov), int(comm), _stream(stream)))


def outer_eager(theta, anchor, vel, prev_local, prev_mean, *, n=None, outer_lr, outer_momentum,
                nesterov=True, variant=EAGER, apply_update=True, stream=None) -> None:
    """diloco_outer_eager: theta [M, stride]; anchor, vel, prev_local [M, state_stride] fp32;
    prev_mean [n] fp32."""
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    ss = _row_stride(anchor)
    assert _row_stride(vel) == ss and _row_stride(prev_local) == ss
    _check("diloco_outer_eager", lib().diloco_outer_eager(
        _ptr(theta), _dtype_code(theta), M, n, _row_stride(theta), _ptr(anchor), _ptr(vel),
        _ptr(prev_local), ss, _ptr(prev_mean), outer_lr, outer_momentum, int(nesterov),
        int(variant), int(apply_update), _stream(stream)))


def packed_state_elems(M: int, n: int) -> int:
    return lib().diloco_packed_state_elems(M, n)


def _state_stride(M, n, *rows):
    ss = None
    for r in rows:
        if r is not None:
            s = _row_stride(r)
            assert ss is None or ss == s, "anchor, vel and prev_local must share one row stride"
            ss = s
    return n if ss is None else ss


def packed_window(state, M: int, offset: int):
    """View of the packed state that starts at parameter index `offset` (a multiple of STATE_TILE)."""
    assert offset % STATE_TILE == 0, "packed-state windows start at tile boundaries"
    return state[(offset // STATE_TILE) * (3 * M + 1) * STATE_TILE:]


def pack_state(state, M, n, *, anchor=None, vel=None, prev_local=None, prev_mean=None,
               stream=None) -> None:
    """diloco_pack_state: rows ([M, state_stride] / [n]) -> packed buffer; None skips."""
    _check("diloco_pack_state", lib().diloco_pack_state(
        _ptr(state), M, n, _ptr(anchor), _ptr(vel), _ptr(prev_local),
        _state_stride(M, n, anchor, vel, prev_local), _ptr(prev_mean), _stream(stream)))


def unpack_state(state, M, n, *, anchor=None, vel=None, prev_local=None, prev_mean=None,
                 stream=None) -> None:
    """diloco_unpack_state: packed buffer -> rows; None skips."""
    _check("diloco_unpack_state", lib().diloco_unpack_state(
        _ptr(state), M, n, _ptr(anchor), _ptr(vel), _ptr(prev_local),
        _state_stride(M, n, anchor, vel, prev_local), _ptr(prev_mean), _stream(stream)))


def outer_eager_packed(theta, state, *, n=None, outer_lr, outer_momentum, nesterov=True,
                       variant=EAGER, apply_update=True, stream=None) -> None:
    """diloco_outer_eager_packed: theta [M, stride]; state from packed_state_elems(M, n)."""
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    _check("diloco_outer_eager_packed", lib().diloco_outer_eager_packed(
        _ptr(theta), _dtype_code(theta), M, n, _row_stride(theta), _ptr(state), outer_lr,
        outer_momentum, int(nesterov), int(variant), int(apply_update), _stream(stream)))


def reset_packed(theta, state, *, n=None, stream=None) -> None:
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    _check("diloco_reset_packed", lib().diloco_reset_packed(
        _ptr(theta), _dtype_code(theta), M, n, _row_stride(theta), _ptr(state), _stream(stream)))


def stream_offset(H: int, F: int, f: int) -> int:
    return lib().diloco_stream_offset(H, F, f)


def stream_due(t: int, H: int, F: int, f: int) -> bool:
    r = lib().diloco_stream_due(t, H, F, f)
    if r < 0:
        raise DilocoError("diloco_stream_due", ERR_SHAPE, "bad schedule arguments")
    return bool(r)


def stream_boundary_count(t: int, H: int, F: int, f: int) -> int:
    r = lib().diloco_stream_boundary_count(t, H, F, f)
    if r < 0:
        raise DilocoError("diloco_stream_boundary_count", ERR_SHAPE, "bad schedule arguments")
    return r


def reset(theta, anchor, *, n=None, stream=None) -> None:
    """diloco_reset: anchor [n] (shared) or [M, anchor_stride] fp32."""
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    astride = 0 if anchor.dim() == 1 else _row_stride(anchor)
    _check("diloco_reset", lib().diloco_reset(
        _ptr(theta), _dtype_code(theta), M, n, _row_stride(theta), _ptr(anchor), astride,
        _stream(stream)))


def sim_quadratic_inner(theta, m1, m2, h, theta_star, *, n=None, noise_std, seed, index_base=0,
                        lr, beta1, beta2, eps, weight_decay, step, stream=None) -> None:
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    _check("diloco_sim_quadratic_inner", lib().diloco_sim_quadratic_inner(
        _ptr(theta), _ptr(m1), _ptr(m2), M, n, _row_stride(theta), _ptr(h), _ptr(theta_star),
        noise_std, seed, index_base, lr, beta1, beta2, eps, weight_decay, step, _stream(stream)))


SIM_MAX_FUSED_STEPS = 64


def sim_quadratic_phase(theta, m1, m2, h, theta_star, *, n=None, noise_std, seed, index_base=0,
                        lr, beta1, beta2, eps, weight_decay, step_first, steps, stream=None) -> None:
    """Steps step_first .. step_first + steps - 1 of sim_quadratic_inner in one pass
    (steps <= SIM_MAX_FUSED_STEPS)."""
    M = theta.shape[0]
    n = theta.shape[1] if n is None else n
    _check("diloco_sim_quadratic_phase", lib().diloco_sim_quadratic_phase(
        _ptr(theta), _ptr(m1), _ptr(m2), M, n, _row_stride(theta), _ptr(h), _ptr(theta_star),
        noise_std, seed, index_base, lr, beta1, beta2, eps, weight_decay, step_first, steps,
        _stream(stream)))


def sim_loss_workspace(n: int) -> int:
    return lib().diloco_sim_loss_workspace(n)


def sim_quadratic_loss(theta, h, theta_star, partials, loss_out, *, n=None, stream=None) -> None:
    """loss_out[0] <- loss at the replica mean of theta ([M, stride], or [n] for one vector)."""
    if theta.dim() == 1:
        M, nn, stride = 1, theta.shape[0], theta.shape[0]
    else:
        M, nn, stride = theta.shape[0], theta.shape[1], _row_stride(theta)
    n = nn if n is None else n
    _check("diloco_sim_quadratic_loss", lib().diloco_sim_quadratic_loss(
        _ptr(theta), M, n, stride, _ptr(h), _ptr(theta_star), _ptr(partials), partials.numel(),
        _ptr(loss_out), _stream(stream)))


def sim_stream_copy(dst, src, *, stream=None) -> None:
    _check("diloco_sim_stream_copy", lib().diloco_sim_stream_copy(
        _ptr(dst), _ptr(src), src.numel(), _stream(stream)))


def sim_stream_rmw(rows, *, n=None, stream=None) -> None:
    """rows [K, stride] fp32: every row's first n elements read and written back in place."""
    K = rows.shape[0]
    n = rows.shape[1] if n is None else n
    _check("diloco_sim_stream_rmw", lib().diloco_sim_stream_rmw(_ptr(rows), K, n, _row_stride(rows),
                                                                _stream(stream)))


def tune(key: str, value: int) -> None:
    _check("diloco_tune", lib().diloco_tune(key.encode(), value))


def tune_get(key: str) -> int:
    return lib().diloco_tune_get(key.encode())
