"""ctypes binding of ``libconv1d_mi355x.so`` (the C ABI declared in ``include/conv1d.h``).

Argument marshalling only: torch supplies device memory and the current HIP stream,
every arithmetic step runs in the library's kernels.  There is no CPU fallback; a
missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libconv1d_mi355x.so")

CONV1D_FP32, CONV1D_BF16 = 0, 1
VARIANT_AUTO, VARIANT_GENERIC, VARIANT_SMALLC, VARIANT_IGEMM = 0, 1, 2, 3
PASS_FWD, PASS_BWD_DATA, PASS_BWD_WEIGHT = 0, 1, 2

EXPORTS = (
    "conv1d_out_width", "conv1d_fwd", "conv1d_fwd_ex", "conv1d_bwd_data", "conv1d_bwd_data_ex",
    "conv1d_bwd_weight_workspace_bytes", "conv1d_bwd_workspace_bytes", "conv1d_bwd",
    "conv1d_bwd_weight", "conv1d_bwd_weight_noalloc", "conv1d_set_variant", "conv1d_kernel_name", "conv1d_status_string",
)

_lib = None


class Conv1dError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"conv1d status {status}: {text}")
        self.status = status


def load() -> ctypes.CDLL:
    """Load the shared library; build it first when it is missing or was built from other sources than the tree
    holds (a stale library would silently test and time old kernels)."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build

    if _build.needs_build():
        _build.build(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    i, vp, sz = ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
    geom = [i] * 7
    lib.conv1d_out_width.restype = i
    lib.conv1d_out_width.argtypes = [i] * 4
    lib.conv1d_fwd.restype = i
    lib.conv1d_fwd.argtypes = [vp, vp, vp] + geom + [i, vp]
    lib.conv1d_fwd_ex.restype = i
    lib.conv1d_fwd_ex.argtypes = [vp, vp, vp, vp] + geom + [i, i, vp]
    lib.conv1d_bwd_data_ex.restype = i
    lib.conv1d_bwd_data_ex.argtypes = [vp, vp, vp] + geom + [i, i, vp]
    lib.conv1d_bwd_data.restype = i
    lib.conv1d_bwd_data.argtypes = [vp, vp, vp] + geom + [i, vp]
    lib.conv1d_bwd_weight_workspace_bytes.restype = sz
    lib.conv1d_bwd_weight_workspace_bytes.argtypes = geom + [i]
    lib.conv1d_bwd_weight.restype = i
    lib.conv1d_bwd_weight.argtypes = [vp, vp, vp, vp, sz] + geom + [i, vp]
    lib.conv1d_bwd_workspace_bytes.restype = sz
    lib.conv1d_bwd_workspace_bytes.argtypes = geom + [i]
    lib.conv1d_bwd.restype = i
    lib.conv1d_bwd.argtypes = [vp, vp, vp, vp, vp, vp, sz] + geom + [i, vp]
    lib.conv1d_bwd_weight_noalloc.restype = i
    lib.conv1d_bwd_weight_noalloc.argtypes = [vp, vp, vp] + geom + [i, vp]
    lib.conv1d_set_variant.restype = i
    lib.conv1d_set_variant.argtypes = [i]
    lib.conv1d_kernel_name.restype = ctypes.c_char_p
    lib.conv1d_kernel_name.argtypes = [i] + geom + [i]
    lib.conv1d_status_string.restype = ctypes.c_char_p
    lib.conv1d_status_string.argtypes = [i]
    _lib = lib
    return lib


def _check(status: int) -> None:
    if status != 0:
        raise Conv1dError(status, load().conv1d_status_string(status).decode())


def conv1d_status_string(status: int) -> str:
    return load().conv1d_status_string(status).decode()


def conv1d_out_width(W: int, S: int, dilation: int, padding: int) -> int:
    return int(load().conv1d_out_width(W, S, dilation, padding))


def conv1d_set_variant(variant: int) -> None:
    _check(load().conv1d_set_variant(variant))


def conv1d_kernel_name(pass_: int, N, C, K, W, S, dilation, padding, dtype: int) -> str:
    return load().conv1d_kernel_name(pass_, N, C, K, W, S, dilation, padding, dtype).decode()


def conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, dilation, padding, dtype: int) -> int:
    return int(load().conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, dilation, padding, dtype))


# ---- tensor-level marshalling ----------------------------------------------------------------
def _dtype_code(t) -> int:
    import torch

    if t.dtype == torch.float32:
        return CONV1D_FP32
    if t.dtype == torch.bfloat16:
        return CONV1D_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _stream_ptr(stream) -> int:
    import torch

    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _dev(t, name):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    return t


def conv1d_fwd(x, w, dilation: int, padding: int, out=None, stream=None):
    """y = conv1d_fwd(x[N,C,W], w[K,C,S]) -> float32 [N,K,Q] on x's device."""
    import torch

    _dev(x, "x"), _dev(w, "w")
    N, C, W = x.shape
    K, C2, S = w.shape
    if C2 != C or w.dtype != x.dtype:
        raise ValueError("x and w disagree in channels or dtype")
    Q = conv1d_out_width(W, S, dilation, padding)
    if Q <= 0:
        raise Conv1dError(-1, conv1d_status_string(-1))
    y = out if out is not None else torch.empty((N, K, Q), dtype=torch.float32, device=x.device)
    if tuple(y.shape) != (N, K, Q) or y.dtype != torch.float32:
        raise ValueError("out has the wrong shape or dtype")
    _check(load().conv1d_fwd(x.data_ptr(), w.data_ptr(), _dev(y, "out").data_ptr(), N, C, K, W, S, dilation,
                             padding, _dtype_code(x), _stream_ptr(stream)))
    return y


EPI_RELU, EPI_OUT_BF16 = 1, 2


def conv1d_fwd_ex(x, w, dilation: int, padding: int, bias=None, relu: bool = False, out_bf16: bool = False, out=None,
                  stream=None):
    """y = [bf16](relu?(conv1d_fwd(x, w) + bias?)) in one pass -> float32 or bfloat16 [N,K,Q]."""
    import torch

    _dev(x, "x"), _dev(w, "w")
    N, C, W = x.shape
    K, C2, S = w.shape
    if C2 != C or w.dtype != x.dtype:
        raise ValueError("x and w disagree in channels or dtype")
    if bias is not None and (_dev(bias, "bias").dtype != torch.float32 or tuple(bias.shape) != (K,)):
        raise ValueError("bias must be a float32 tensor [K]")
    Q = conv1d_out_width(W, S, dilation, padding)
    if Q <= 0:
        raise Conv1dError(-1, conv1d_status_string(-1))
    odt = torch.bfloat16 if out_bf16 else torch.float32
    y = out if out is not None else torch.empty((N, K, Q), dtype=odt, device=x.device)
    if tuple(y.shape) != (N, K, Q) or y.dtype != odt:
        raise ValueError("out has the wrong shape or dtype")
    flags = (EPI_RELU if relu else 0) | (EPI_OUT_BF16 if out_bf16 else 0)
    _check(load().conv1d_fwd_ex(x.data_ptr(), w.data_ptr(), bias.data_ptr() if bias is not None else None,
                                _dev(y, "out").data_ptr(), N, C, K, W, S, dilation, padding, _dtype_code(x), flags,
                                _stream_ptr(stream)))
    return y


def conv1d_bwd_data_ex(dy, w, W: int, dilation: int, padding: int, out_bf16: bool = False, out=None, stream=None):
    """dx = conv1d_bwd_data(dy, w), stored as bfloat16 when out_bf16 -> [N,C,W]."""
    import torch

    _dev(dy, "dy"), _dev(w, "w")
    N, K, Q = dy.shape
    K2, C, S = w.shape
    if K2 != K or w.dtype != dy.dtype:
        raise ValueError("dy and w disagree in filters or dtype")
    if conv1d_out_width(W, S, dilation, padding) != Q:
        raise ValueError("dy width does not match the geometry")
    odt = torch.bfloat16 if out_bf16 else torch.float32
    dx = out if out is not None else torch.empty((N, C, W), dtype=odt, device=dy.device)
    if tuple(dx.shape) != (N, C, W) or dx.dtype != odt:
        raise ValueError("out has the wrong shape or dtype")
    _check(load().conv1d_bwd_data_ex(dy.data_ptr(), w.data_ptr(), _dev(dx, "out").data_ptr(), N, C, K, W, S, dilation,
                                     padding, _dtype_code(dy), EPI_OUT_BF16 if out_bf16 else 0, _stream_ptr(stream)))
    return dx


def conv1d_bwd_data(dy, w, W: int, dilation: int, padding: int, out=None, stream=None):
    """dx = conv1d_bwd_data(dy[N,K,Q], w[K,C,S]) -> float32 [N,C,W]."""
    import torch

    _dev(dy, "dy"), _dev(w, "w")
    N, K, Q = dy.shape
    K2, C, S = w.shape
    if K2 != K or w.dtype != dy.dtype:
        raise ValueError("dy and w disagree in filters or dtype")
    if conv1d_out_width(W, S, dilation, padding) != Q:
        raise ValueError("dy width does not match the geometry")
    dx = out if out is not None else torch.empty((N, C, W), dtype=torch.float32, device=dy.device)
    if tuple(dx.shape) != (N, C, W) or dx.dtype != torch.float32:
        raise ValueError("out has the wrong shape or dtype")
    _check(load().conv1d_bwd_data(dy.data_ptr(), w.data_ptr(), _dev(dx, "out").data_ptr(), N, C, K, W, S, dilation,
                                  padding, _dtype_code(dy), _stream_ptr(stream)))
    return dx


def conv1d_bwd_weight(x, dy, S: int, dilation: int, padding: int, out=None, workspace=None, stream=None):
    """dw = conv1d_bwd_weight(x[N,C,W], dy[N,K,Q]) -> float32 [K,C,S]."""
    import torch

    _dev(x, "x"), _dev(dy, "dy")
    N, C, W = x.shape
    N2, K, Q = dy.shape
    if N2 != N or dy.dtype != x.dtype:
        raise ValueError("x and dy disagree in batch or dtype")
    if conv1d_out_width(W, S, dilation, padding) != Q:
        raise ValueError("dy width does not match the geometry")
    code = _dtype_code(x)
    need = conv1d_bwd_weight_workspace_bytes(N, C, K, W, S, dilation, padding, code)
    ws = workspace if workspace is not None else torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    dw = out if out is not None else torch.empty((K, C, S), dtype=torch.float32, device=x.device)
    if tuple(dw.shape) != (K, C, S) or dw.dtype != torch.float32:
        raise ValueError("out has the wrong shape or dtype")
    _check(load().conv1d_bwd_weight(x.data_ptr(), dy.data_ptr(), _dev(dw, "out").data_ptr(), ws.data_ptr(),
                                    ws.numel() * ws.element_size(), N, C, K, W, S, dilation, padding, code,
                                    _stream_ptr(stream)))
    return dw


NOALLOC_SCRATCH_BYTES = 64 << 20


def conv1d_bwd_weight_noalloc(x, dy, S: int, dilation: int, padding: int, out, stream=None):
    """dw = conv1d_bwd_weight(x, dy) into the caller's `out`, partial sums in the library's built-in buffer."""
    import torch

    _dev(x, "x"), _dev(dy, "dy")
    N, C, W = x.shape
    N2, K, Q = dy.shape
    if N2 != N or dy.dtype != x.dtype:
        raise ValueError("x and dy disagree in batch or dtype")
    if conv1d_out_width(W, S, dilation, padding) != Q:
        raise ValueError("dy width does not match the geometry")
    if tuple(out.shape) != (K, C, S) or out.dtype != torch.float32:
        raise ValueError("out has the wrong shape or dtype")
    _check(load().conv1d_bwd_weight_noalloc(x.data_ptr(), dy.data_ptr(), _dev(out, "out").data_ptr(), N, C, K, W, S,
                                            dilation, padding, _dtype_code(x), _stream_ptr(stream)))
    return out


def conv1d_bwd(x, dy, w, dilation: int, padding: int, out_dx=None, out_dw=None, workspace=None, stream=None):
    """(dx, dw) = both backward passes of the layer in one call -> float32 [N,C,W] and [K,C,S]."""
    import torch

    _dev(x, "x"), _dev(dy, "dy"), _dev(w, "w")
    N, C, W = x.shape
    N2, K, Q = dy.shape
    K2, C2, S = w.shape
    if N2 != N or K2 != K or C2 != C or dy.dtype != x.dtype or w.dtype != x.dtype:
        raise ValueError("x, dy and w disagree in shape or dtype")
    if conv1d_out_width(W, S, dilation, padding) != Q:
        raise ValueError("dy width does not match the geometry")
    code = _dtype_code(x)
    need = int(load().conv1d_bwd_workspace_bytes(N, C, K, W, S, dilation, padding, code))
    ws = workspace if workspace is not None else torch.empty(max(need, 256), dtype=torch.uint8, device=x.device)
    dx = out_dx if out_dx is not None else torch.empty((N, C, W), dtype=torch.float32, device=x.device)
    dw = out_dw if out_dw is not None else torch.empty((K, C, S), dtype=torch.float32, device=x.device)
    if tuple(dx.shape) != (N, C, W) or tuple(dw.shape) != (K, C, S) or dx.dtype != torch.float32 or dw.dtype != torch.float32:
        raise ValueError("an output has the wrong shape or dtype")
    _check(load().conv1d_bwd(x.data_ptr(), dy.data_ptr(), w.data_ptr(), _dev(dx, "out_dx").data_ptr(),
                             _dev(dw, "out_dw").data_ptr(), ws.data_ptr(), ws.numel() * ws.element_size(), N, C, K, W, S,
                             dilation, padding, code, _stream_ptr(stream)))
    return dx, dw
