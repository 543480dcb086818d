"""ctypes binding of libdiloco.so: argument marshalling only.

Every function takes torch tensors (device memory) and scalars, passes raw device pointers
plus the current HIP stream, and raises DilocoError on a non-zero status.  The C ABI sees
addresses only, so what it cannot check is checked here, before any pointer leaves Python:
that every tensor lives on one GPU, has the dtype the entry point reads it as, and spans the
rows, strides and sizes the call names (a host tensor, a float64 buffer or a row shorter than
n would otherwise be a kernel reading and writing out of bounds).  Those checks raise
TypeError / ValueError and nothing is launched.  There is no fallback: if the shared library
has not been built, the first call raises.
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


class Launch(ctypes.Structure):
    """diloco_launch of include/diloco_sim.h: the launch shape of one *_shaped call."""
    _fields_ = [("block", _c_int), ("xcd_remap", _c_int), ("wg_per_cu", _c_int), ("generic_path", _c_int)]


_c_launch = ctypes.POINTER(Launch)

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
    "diloco_inner_adamw_shaped": (_c_int, [_c_ptr, _c_ptr, _c_ptr, _c_ptr, _c_int, _c_i64, _c_i64, _c_int,
                                           _c_int, _c_dbl, _c_dbl, _c_dbl, _c_dbl, _c_dbl, _c_i64, _c_ptr,
                                           _c_launch]),
    "diloco_outer_sync_shaped": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr,
                                          _c_dbl, _c_dbl, _c_int, _c_int, _c_ptr, _c_launch]),
    "diloco_outer_eager_shaped": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr,
                                           _c_i64, _c_ptr, _c_dbl, _c_dbl, _c_int, _c_int, _c_int, _c_ptr,
                                           _c_launch]),
    "diloco_outer_eager_packed_shaped": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_dbl, _c_dbl,
                                                  _c_int, _c_int, _c_int, _c_ptr, _c_launch]),
    "diloco_reset": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_i64, _c_ptr]),
    "diloco_packed_state_elems": (_c_i64, [_c_int, _c_i64]),
    "diloco_pack_state": (_c_int, [_c_ptr, _c_int, _c_i64, _c_ptr, _c_ptr, _c_ptr, _c_i64, _c_ptr, _c_ptr]),
    "diloco_unpack_state": (_c_int, [_c_ptr, _c_int, _c_i64, _c_ptr, _c_ptr, _c_ptr, _c_i64, _c_ptr, _c_ptr]),
    "diloco_outer_eager_packed": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_dbl, _c_dbl,
                                           _c_int, _c_int, _c_int, _c_ptr]),
    "diloco_outer_eager_pingpong": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_dbl, _c_dbl,
                                             _c_int, _c_int, _c_int, _c_ptr]),
    "diloco_outer_eager_pingpong_shaped": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_dbl,
                                                    _c_dbl, _c_int, _c_int, _c_int, _c_ptr, _c_launch]),
    "diloco_outer_eager_overlap2": (_c_int, [_c_ptr, _c_int, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_dbl, _c_dbl,
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
    "diloco_sim_stream_rmw": (_c_int, [_c_ptr, _c_int, _c_i64, _c_i64, _c_ptr, _c_launch]),
    "diloco_sim_stream_sweep": (_c_int, [_c_ptr, _c_int, _c_i64, _c_i64, _c_int, ctypes.c_float, _c_ptr, _c_launch]),
    "diloco_sim_loss_workspace": (_c_i64, [_c_i64]),
    "diloco_sim_quadratic_loss": (_c_int, [_c_ptr, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr,
                                           _c_i64, _c_ptr, _c_ptr]),
    "diloco_sim_quadratic_loss_static": (_c_int, [_c_ptr, _c_int, _c_i64, _c_i64, _c_ptr, _c_ptr, _c_ptr, _c_ptr]),
    "diloco_sim_stream_copy": (_c_int, [_c_ptr, _c_ptr, _c_i64, _c_ptr, _c_launch]),
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


def _launch(launch):
    """None (the library's own choice) or (block, xcd_remap, wg_per_cu[, generic_path]) -> diloco_launch*."""
    if launch is None:
        return None
    if isinstance(launch, Launch):
        return ctypes.byref(launch)
    vals = tuple(int(v) for v in launch)
    if len(vals) == 3:
        vals += (0,)
    if len(vals) != 4:
        raise ValueError("launch is (block, xcd_remap, wg_per_cu[, generic_path])")
    return ctypes.byref(Launch(*vals))


def _row_stride(t: torch.Tensor) -> int:
    """Element stride between replicas of a [M, n] tensor whose rows are contiguous."""
    if t.dim() == 1:
        return t.shape[0]
    if t.dim() != 2 or not (t.shape[1] <= 1 or t.stride(1) == 1):
        raise ValueError("a replica buffer is [M, n] with contiguous rows")
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


class _Args:
    """The tensors of one call: every one on the same GPU, of the stated dtype and large enough."""

    def __init__(self, fn: str, require_gpu: bool = True):
        self.fn = fn
        self.device = None
        self.require_gpu = require_gpu     # False only in CPU unit tests of these checks

    def _common(self, t, name, dtypes):
        if not isinstance(t, torch.Tensor):
            raise TypeError(f"{self.fn}: {name} must be a torch tensor")
        if self.require_gpu and not t.is_cuda:
            raise TypeError(f"{self.fn}: {name} is on {t.device}, the library takes GPU memory only")
        if self.device is None:
            self.device = t.device
        elif t.device != self.device:
            raise ValueError(f"{self.fn}: {name} is on {t.device}, other arguments on {self.device}")
        if t.dtype not in dtypes:
            raise TypeError(f"{self.fn}: {name} is {t.dtype}, expected one of {tuple(dtypes)}")

    def rows(self, t, name, M, n, dtypes=(torch.float32,), stride=None):
        """[M, >= n] replica buffer; returns its row stride (which must equal `stride` if given)."""
        self._common(t, name, dtypes)
        if t.dim() != 2 or t.shape[0] != M:
            raise ValueError(f"{self.fn}: {name} must be [M={M}, >= n] but is {tuple(t.shape)}")
        if n < 0 or t.shape[1] < n:
            raise ValueError(f"{self.fn}: {name} has rows of {t.shape[1]} elements, the call names n={n}")
        s = _row_stride(t)
        if stride is not None and s != stride:
            raise ValueError(f"{self.fn}: {name} has row stride {s}, the other buffers {stride}")
        return s

    def vec(self, t, name, n, dtypes=(torch.float32,), optional=False):
        """Contiguous buffer of at least n elements."""
        if t is None:
            if optional:
                return
            raise TypeError(f"{self.fn}: {name} is required")
        self._common(t, name, dtypes)
        if not t.is_contiguous():
            raise ValueError(f"{self.fn}: {name} must be contiguous")
        if n < 0 or t.numel() < n:
            raise ValueError(f"{self.fn}: {name} holds {t.numel()} elements, the call needs {n}")


_PARAM_DTYPES = (torch.float32, torch.bfloat16)


def _shape_of(theta, n):
    if not isinstance(theta, torch.Tensor) or theta.dim() != 2:
        raise ValueError("theta must be a [M, n] tensor")
    return theta.shape[0], (theta.shape[1] if n is None else int(n))


def inner_adamw(theta, m1, m2, grad, *, n=None, lr, beta1, beta2, eps, weight_decay, step,
                stream=None, launch=None) -> None:
    """diloco_inner_adamw on [M, stride] tensors (first n columns).  launch: explicit launch shape
    (diloco_inner_adamw_shaped)."""
    M, n = _shape_of(theta, n)
    a = _Args("diloco_inner_adamw")
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    a.rows(m1, "m1", M, n, (theta.dtype,), stride)
    a.rows(m2, "m2", M, n, (theta.dtype,), stride)
    a.rows(grad, "grad", M, n, _PARAM_DTYPES, stride)
    args = (_ptr(theta), _ptr(m1), _ptr(m2), _ptr(grad), M, n, stride, _dtype_code(theta), _dtype_code(grad),
            lr, beta1, beta2, eps, weight_decay, step, _stream(stream))
    if launch is None:
        _check("diloco_inner_adamw", lib().diloco_inner_adamw(*args))
    else:
        _check("diloco_inner_adamw_shaped", lib().diloco_inner_adamw_shaped(*args, _launch(launch)))


def outer_sync(theta, anchor, vel, *, n=None, mean_out=None, outer_lr, outer_momentum,
               nesterov=True, comm=None, stream=None, launch=None) -> None:
    """diloco_outer_sync: theta [M, stride]; anchor, vel (and mean_out) [n] fp32.  comm (COMM_BF16 or
    COMM_EXMY(...)) goes through diloco_outer_sync_comm; launch through diloco_outer_sync_shaped."""
    M, n = _shape_of(theta, n)
    a = _Args("diloco_outer_sync")
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    a.vec(anchor, "anchor", n)
    a.vec(vel, "vel", n)
    a.vec(mean_out, "mean_out", n, optional=True)
    head = (_ptr(theta), _dtype_code(theta), M, n, stride, _ptr(anchor), _ptr(vel), _ptr(mean_out), outer_lr,
            outer_momentum, int(nesterov))
    if launch is not None:
        _check("diloco_outer_sync_shaped", lib().diloco_outer_sync_shaped(
            *head, 0 if comm is None else int(comm), _stream(stream), _launch(launch)))
    elif comm is None:
        _check("diloco_outer_sync", lib().diloco_outer_sync(*head, _stream(stream)))
    else:
        _check("diloco_outer_sync_comm", lib().diloco_outer_sync_comm(*head, int(comm), _stream(stream)))


def outer_eager(theta, anchor, vel, prev_local, prev_mean, *, n=None, outer_lr, outer_momentum,
                nesterov=True, variant=EAGER, apply_update=True, stream=None, launch=None) -> None:
    """diloco_outer_eager: theta [M, stride]; anchor, vel, prev_local [M, state_stride] fp32;
    prev_mean [n] fp32.  launch: explicit launch shape (diloco_outer_eager_shaped)."""
    M, n = _shape_of(theta, n)
    a = _Args("diloco_outer_eager")
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    ss = a.rows(anchor, "anchor", M, n)
    a.rows(vel, "vel", M, n, stride=ss)
    a.rows(prev_local, "prev_local", M, n, stride=ss)
    a.vec(prev_mean, "prev_mean", n)
    args = (_ptr(theta), _dtype_code(theta), M, n, stride, _ptr(anchor), _ptr(vel), _ptr(prev_local), ss,
            _ptr(prev_mean), outer_lr, outer_momentum, int(nesterov), int(variant), int(apply_update),
            _stream(stream))
    if launch is None:
        _check("diloco_outer_eager", lib().diloco_outer_eager(*args))
    else:
        _check("diloco_outer_eager_shaped", lib().diloco_outer_eager_shaped(*args, _launch(launch)))


def packed_state_elems(M: int, n: int) -> int:
    return lib().diloco_packed_state_elems(M, n)


def _packed_args(fn, state, M, n):
    need = packed_state_elems(M, n)
    if need < 0:
        raise ValueError(f"{fn}: no packed state for M={M}, n={n}")
    a = _Args(fn)
    a.vec(state, "state", need)
    return a


def _state_rows(a, M, n, anchor, vel, prev_local, prev_mean):
    """Validates the optional row buffers of a pack / unpack call; returns their common stride."""
    ss = None
    for t, name in ((anchor, "anchor"), (vel, "vel"), (prev_local, "prev_local")):
        if t is not None:
            ss = a.rows(t, name, M, n, stride=ss)
    a.vec(prev_mean, "prev_mean", n, optional=True)
    return n if ss is None else ss


def packed_window(state, M: int, offset: int):
    """View of the packed state that starts at parameter index `offset` (a multiple of STATE_TILE)."""
    if offset % STATE_TILE != 0:
        raise ValueError("packed-state windows start at tile boundaries")
    return state[(offset // STATE_TILE) * (3 * M + 1) * STATE_TILE:]


def pack_state(state, M, n, *, anchor=None, vel=None, prev_local=None, prev_mean=None,
               stream=None) -> None:
    """diloco_pack_state: rows ([M, state_stride] / [n]) -> packed buffer; None skips."""
    a = _packed_args("diloco_pack_state", state, M, n)
    ss = _state_rows(a, M, n, anchor, vel, prev_local, prev_mean)
    _check("diloco_pack_state", lib().diloco_pack_state(
        _ptr(state), M, n, _ptr(anchor), _ptr(vel), _ptr(prev_local), ss, _ptr(prev_mean), _stream(stream)))


def unpack_state(state, M, n, *, anchor=None, vel=None, prev_local=None, prev_mean=None,
                 stream=None) -> None:
    """diloco_unpack_state: packed buffer -> rows; None skips."""
    a = _packed_args("diloco_unpack_state", state, M, n)
    ss = _state_rows(a, M, n, anchor, vel, prev_local, prev_mean)
    _check("diloco_unpack_state", lib().diloco_unpack_state(
        _ptr(state), M, n, _ptr(anchor), _ptr(vel), _ptr(prev_local), ss, _ptr(prev_mean), _stream(stream)))


def outer_eager_packed(theta, state, *, n=None, outer_lr, outer_momentum, nesterov=True,
                       variant=EAGER, apply_update=True, stream=None, launch=None) -> None:
    """diloco_outer_eager_packed: theta [M, stride]; state from packed_state_elems(M, n).  launch:
    explicit launch shape (diloco_outer_eager_packed_shaped)."""
    M, n = _shape_of(theta, n)
    a = _packed_args("diloco_outer_eager_packed", state, M, n)
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    args = (_ptr(theta), _dtype_code(theta), M, n, stride, _ptr(state), outer_lr, outer_momentum,
            int(nesterov), int(variant), int(apply_update), _stream(stream))
    if launch is None:
        _check("diloco_outer_eager_packed", lib().diloco_outer_eager_packed(*args))
    else:
        _check("diloco_outer_eager_packed_shaped", lib().diloco_outer_eager_packed_shaped(*args, _launch(launch)))


def outer_eager_pingpong(theta, state_in, state_out, *, n=None, outer_lr, outer_momentum, nesterov=True,
                         variant=EAGER, apply_update=True, stream=None, launch=None) -> None:
    """diloco_outer_eager_pingpong: the packed step reading state_in and writing state_out (two buffers
    of packed_state_elems(M, n) floats that the caller swaps between boundaries)."""
    M, n = _shape_of(theta, n)
    a = _packed_args("diloco_outer_eager_pingpong", state_in, M, n)
    a.vec(state_out, "state_out", packed_state_elems(M, n))
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    args = (_ptr(theta), _dtype_code(theta), M, n, stride, _ptr(state_in), _ptr(state_out), outer_lr, outer_momentum,
            int(nesterov), int(variant), int(apply_update), _stream(stream))
    if launch is None:
        _check("diloco_outer_eager_pingpong", lib().diloco_outer_eager_pingpong(*args))
    else:
        _check("diloco_outer_eager_pingpong_shaped", lib().diloco_outer_eager_pingpong_shaped(*args, _launch(launch)))


def outer_eager_overlap2(theta, state_prev, state_cur, *, n=None, outer_lr, outer_momentum, nesterov=True,
                         variant=EAGER, apply_update=True, stream=None) -> None:
    """diloco_outer_eager_overlap2: 2-outer-steps overlap on two packed buffers; at boundary b pass the
    buffer written at b-1 as state_prev and the one written at b-2 as state_cur (it is overwritten)."""
    M, n = _shape_of(theta, n)
    a = _packed_args("diloco_outer_eager_overlap2", state_prev, M, n)
    a.vec(state_cur, "state_cur", packed_state_elems(M, n))
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    _check("diloco_outer_eager_overlap2", lib().diloco_outer_eager_overlap2(
        _ptr(theta), _dtype_code(theta), M, n, stride, _ptr(state_prev), _ptr(state_cur), outer_lr, outer_momentum,
        int(nesterov), int(variant), int(apply_update), _stream(stream)))


def reset_packed(theta, state, *, n=None, stream=None) -> None:
    M, n = _shape_of(theta, n)
    a = _packed_args("diloco_reset_packed", state, M, n)
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    _check("diloco_reset_packed", lib().diloco_reset_packed(
        _ptr(theta), _dtype_code(theta), M, n, stride, _ptr(state), _stream(stream)))


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
    M, n = _shape_of(theta, n)
    a = _Args("diloco_reset")
    stride = a.rows(theta, "theta", M, n, _PARAM_DTYPES)
    if isinstance(anchor, torch.Tensor) and anchor.dim() == 1:
        a.vec(anchor, "anchor", n)
        astride = 0
    else:
        astride = a.rows(anchor, "anchor", M, n)
    _check("diloco_reset", lib().diloco_reset(
        _ptr(theta), _dtype_code(theta), M, n, stride, _ptr(anchor), astride, _stream(stream)))


def _quadratic_args(fn, theta, m1, m2, h, theta_star, n):
    M, n = _shape_of(theta, n)
    a = _Args(fn)
    stride = a.rows(theta, "theta", M, n)
    a.rows(m1, "m1", M, n, stride=stride)
    a.rows(m2, "m2", M, n, stride=stride)
    a.vec(h, "h", n)
    a.vec(theta_star, "theta_star", n)
    return M, n, stride


def sim_quadratic_inner(theta, m1, m2, h, theta_star, *, n=None, noise_std, seed, index_base=0,
                        lr, beta1, beta2, eps, weight_decay, step, stream=None) -> None:
    M, n, stride = _quadratic_args("diloco_sim_quadratic_inner", theta, m1, m2, h, theta_star, n)
    _check("diloco_sim_quadratic_inner", lib().diloco_sim_quadratic_inner(
        _ptr(theta), _ptr(m1), _ptr(m2), M, n, stride, _ptr(h), _ptr(theta_star),
        noise_std, seed, index_base, lr, beta1, beta2, eps, weight_decay, step, _stream(stream)))


SIM_MAX_FUSED_STEPS = 64


def sim_quadratic_phase(theta, m1, m2, h, theta_star, *, n=None, noise_std, seed, index_base=0,
                        lr, beta1, beta2, eps, weight_decay, step_first, steps, stream=None) -> None:
    """Steps step_first .. step_first + steps - 1 of sim_quadratic_inner in one pass
    (steps <= SIM_MAX_FUSED_STEPS)."""
    M, n, stride = _quadratic_args("diloco_sim_quadratic_phase", theta, m1, m2, h, theta_star, n)
    _check("diloco_sim_quadratic_phase", lib().diloco_sim_quadratic_phase(
        _ptr(theta), _ptr(m1), _ptr(m2), M, n, stride, _ptr(h), _ptr(theta_star),
        noise_std, seed, index_base, lr, beta1, beta2, eps, weight_decay, step_first, steps,
        _stream(stream)))


def sim_loss_workspace(n: int) -> int:
    return lib().diloco_sim_loss_workspace(n)


def _loss_args(fn, theta, h, theta_star, loss_out, n):
    a = _Args(fn)
    if isinstance(theta, torch.Tensor) and theta.dim() == 1:
        M, nn = 1, theta.shape[0]
        n = nn if n is None else int(n)
        a.vec(theta, "theta", n)
        stride = nn
    else:
        M, n = _shape_of(theta, n)
        stride = a.rows(theta, "theta", M, n)
    a.vec(h, "h", n)
    a.vec(theta_star, "theta_star", n)
    a.vec(loss_out, "loss_out", 1, (torch.float64,))
    return a, M, n, stride


def sim_quadratic_loss(theta, h, theta_star, partials, loss_out, *, n=None, stream=None) -> None:
    """loss_out[0] <- loss at the replica mean of theta ([M, stride], or [n] for one vector)."""
    a, M, n, stride = _loss_args("diloco_sim_quadratic_loss", theta, h, theta_star, loss_out, n)
    a.vec(partials, "partials", sim_loss_workspace(n), (torch.float64,))
    _check("diloco_sim_quadratic_loss", lib().diloco_sim_quadratic_loss(
        _ptr(theta), M, n, stride, _ptr(h), _ptr(theta_star), _ptr(partials), partials.numel(),
        _ptr(loss_out), _stream(stream)))


def sim_quadratic_loss_static(theta, h, theta_star, loss_out, *, n=None, stream=None) -> None:
    """sim_quadratic_loss without a workspace argument: the library's own static device array holds
    the partial sums, nothing is allocated."""
    a, M, n, stride = _loss_args("diloco_sim_quadratic_loss_static", theta, h, theta_star, loss_out, n)
    _check("diloco_sim_quadratic_loss_static", lib().diloco_sim_quadratic_loss_static(
        _ptr(theta), M, n, stride, _ptr(h), _ptr(theta_star), _ptr(loss_out), _stream(stream)))


def sim_stream_copy(dst, src, *, stream=None, launch=None) -> None:
    a = _Args("diloco_sim_stream_copy")
    a.vec(src, "src", 0)
    a.vec(dst, "dst", src.numel())
    _check("diloco_sim_stream_copy", lib().diloco_sim_stream_copy(
        _ptr(dst), _ptr(src), src.numel(), _stream(stream), _launch(launch)))


def sim_stream_rmw(rows, *, n=None, stream=None, launch=None) -> None:
    """rows [K, stride] fp32: every row's first n elements read and written back in place."""
    K, n = _shape_of(rows, n)
    a = _Args("diloco_sim_stream_rmw")
    stride = a.rows(rows, "rows", K, min(n, rows.shape[1]))
    _check("diloco_sim_stream_rmw", lib().diloco_sim_stream_rmw(_ptr(rows), K, n, stride, _stream(stream),
                                                                _launch(launch)))


SWEEP_RMW, SWEEP_READ, SWEEP_WRITE = 0, 1, 2


def sim_stream_sweep(rows, mode, *, n=None, fill=0.0, stream=None, launch=None) -> None:
    """sim_stream_rmw with its halves apart: SWEEP_RMW, SWEEP_READ (nothing written) or SWEEP_WRITE
    (every element set to `fill`)."""
    K, n = _shape_of(rows, n)
    a = _Args("diloco_sim_stream_sweep")
    stride = a.rows(rows, "rows", K, min(n, rows.shape[1]))
    _check("diloco_sim_stream_sweep", lib().diloco_sim_stream_sweep(
        _ptr(rows), K, n, stride, int(mode), float(fill), _stream(stream), _launch(launch)))


def tune(key: str, value: int) -> None:
    """The calling thread's launch shape for calls without `launch=` (thread-local in the library)."""
    _check("diloco_tune", lib().diloco_tune(key.encode(), value))


def tune_get(key: str) -> int:
    return lib().diloco_tune_get(key.encode())
