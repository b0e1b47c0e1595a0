"""ctypes binding of libfdl.so: same names as the C ABI (include/fdl.h).

Argument marshalling only: every arithmetic step runs inside the library's
HIP kernels.  There is no fallback: if libfdl.so has not been built, importing
this module raises.  Tensors are torch tensors used as plain device buffers
(`data_ptr()`); raw integer addresses are accepted too, which is what the
host-only tests of the argument checks use.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Union

# torch must be loaded before libfdl.so.  The torch wheel carries its own HIP runtime under the same shared-object
# name as the system one the library was linked against; the dynamic loader keeps whichever copy arrives first for
# both.  Loading the library first would leave torch's allocations and streams and the library's kernels in two
# different runtimes, and every launch on a torch buffer then fails with a device error.
import torch  # noqa: F401  (import order matters)

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libfdl.so")

FDL_F32, FDL_BF16 = 0, 1
FDL_OK, FDL_ERR_NULL, FDL_ERR_SHAPE, FDL_ERR_DTYPE, FDL_ERR_EPS, FDL_ERR_WORKSPACE, FDL_ERR_ALIGN, FDL_ERR_LAUNCH = range(8)

EXPORTS = ("fdl_status_string", "fdl_workspace_bytes", "fdl_forward", "fdl_forward_static", "fdl_backward",
           "fdl_set_phase_events", "fdl_forward_inference_workspace_bytes", "fdl_forward_inference",
           "fdl_linear_relu_workspace_bytes", "fdl_linear_relu_forward", "fdl_linear_relu_backward",
           "fdl_layernorm_forward", "fdl_rmsnorm_forward", "fdl_llama_ffn_workspace_bytes", "fdl_llama_ffn_forward")
FDL_STATIC_SCRATCH_BYTES = 16 * 1024 * 1024
FDL_PHASES = ("F1", "FS", "F2", "B1", "B2", "B3", "B4")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_14279_amd.build` "
                      "(there is no fallback path)")

_vp, _i64, _sz, _f32, _int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float, ctypes.c_int


def _bind(lib):
    """Declare the C signatures of include/fdl.h on a loaded library."""
    lib.fdl_status_string.restype = ctypes.c_char_p
    lib.fdl_status_string.argtypes = [_int]
    lib.fdl_workspace_bytes.restype = _sz
    lib.fdl_workspace_bytes.argtypes = [_int, _i64, _i64, _i64]
    lib.fdl_forward.restype = _int
    lib.fdl_forward.argtypes = [_int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.fdl_forward_static.restype = _int
    lib.fdl_forward_static.argtypes = [_int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _vp, _vp]
    lib.fdl_backward.restype = _int
    lib.fdl_backward.argtypes = [_int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp,
                                 _vp, _sz, _vp]
    lib.fdl_set_phase_events.restype = _int
    lib.fdl_set_phase_events.argtypes = [ctypes.POINTER(_vp), _int]
    for name in ("fdl_forward_inference_workspace_bytes", "fdl_linear_relu_workspace_bytes", "fdl_llama_ffn_workspace_bytes"):
        getattr(lib, name).restype = _sz
        getattr(lib, name).argtypes = [_int, _i64, _i64, _i64]
    lib.fdl_forward_inference.restype = _int
    lib.fdl_forward_inference.argtypes = [_int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _f32, _vp, _vp, _sz, _vp]
    lib.fdl_linear_relu_forward.restype = _int
    lib.fdl_linear_relu_forward.argtypes = [_int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.fdl_linear_relu_backward.restype = _int
    lib.fdl_linear_relu_backward.argtypes = [_int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    lib.fdl_layernorm_forward.restype = _int
    lib.fdl_layernorm_forward.argtypes = [_int, _i64, _i64, _vp, _vp, _vp, _f32, _vp, _vp, _vp, _vp]
    lib.fdl_rmsnorm_forward.restype = _int
    lib.fdl_rmsnorm_forward.argtypes = [_int, _i64, _i64, _vp, _vp, _f32, _vp, _vp]
    lib.fdl_llama_ffn_forward.restype = _int
    lib.fdl_llama_ffn_forward.argtypes = [_int, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    return lib


_lib = _bind(ctypes.CDLL(LIB_PATH))


class FdlError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(fdl_status_string(status))


def _dtype_code(dtype: Union[int, str]) -> int:
    if isinstance(dtype, str):
        return {"f32": FDL_F32, "bf16": FDL_BF16}[dtype]
    return int(dtype)


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t or None
    return t.data_ptr() or None


def _nbytes(t) -> int:
    return t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def fdl_status_string(status: int) -> str:
    return _lib.fdl_status_string(int(status)).decode()


def fdl_workspace_bytes(dtype, M: int, K: int, N: int) -> int:
    return int(_lib.fdl_workspace_bytes(_dtype_code(dtype), M, K, N))


def fdl_forward_raw(dtype, M, K, N, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd,
                    workspace, workspace_bytes, stream) -> int:
    """Direct call, returns the status code (no exception)."""
    return int(_lib.fdl_forward(_dtype_code(dtype), M, K, N, _ptr(X), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                                float(eps), _ptr(Y), _ptr(Zsave), _ptr(mean), _ptr(rstd), _ptr(workspace),
                                int(workspace_bytes), stream))


def fdl_forward_static_raw(dtype, M, K, N, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, stream) -> int:
    return int(_lib.fdl_forward_static(_dtype_code(dtype), M, K, N, _ptr(X), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                                       float(eps), _ptr(Y), _ptr(Zsave), _ptr(mean), _ptr(rstd), stream))


def fdl_backward_raw(dtype, M, K, N, dY, X, W, gamma, Zsave, mean, rstd, dX, dW, db, dgamma, dbeta,
                     workspace, workspace_bytes, stream) -> int:
    return int(_lib.fdl_backward(_dtype_code(dtype), M, K, N, _ptr(dY), _ptr(X), _ptr(W), _ptr(gamma), _ptr(Zsave),
                                 _ptr(mean), _ptr(rstd), _ptr(dX), _ptr(dW), _ptr(db), _ptr(dgamma), _ptr(dbeta),
                                 _ptr(workspace), int(workspace_bytes), stream))


def fdl_forward(dtype, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, workspace, stream=None) -> None:
    """Enqueue the forward pass on `stream` (default: torch's current stream).  Shapes come from X [M,K], W [N,K]."""
    M, K = X.shape
    N = W.shape[0]
    st = fdl_forward_raw(dtype, M, K, N, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd,
                         workspace, _nbytes(workspace), _stream(stream))
    if st != FDL_OK:
        raise FdlError(st)


def fdl_forward_static(dtype, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, stream=None) -> None:
    """fdl_forward on the library's own fixed scratch array (no workspace argument, nothing allocated)."""
    M, K = X.shape
    N = W.shape[0]
    st = fdl_forward_static_raw(dtype, M, K, N, X, W, b, gamma, beta, eps, Y, Zsave, mean, rstd, _stream(stream))
    if st != FDL_OK:
        raise FdlError(st)


def fdl_backward(dtype, dY, X, W, gamma, Zsave, mean, rstd, dX, dW, db, dgamma, dbeta, workspace, stream=None) -> None:
    """Enqueue the backward pass on `stream` (default: torch's current stream)."""
    M, K = X.shape
    N = W.shape[0]
    st = fdl_backward_raw(dtype, M, K, N, dY, X, W, gamma, Zsave, mean, rstd, dX, dW, db, dgamma, dbeta,
                          workspace, _nbytes(workspace), _stream(stream))
    if st != FDL_OK:
        raise FdlError(st)


def fdl_set_phase_events(events) -> None:
    """events: sequence of 2*len(FDL_PHASES) hipEvent_t handles (ints), or None to switch instrumentation off."""
    if events is None:
        st = _lib.fdl_set_phase_events(None, 0)
    else:
        arr = (_vp * len(events))(*[int(e) for e in events])
        st = _lib.fdl_set_phase_events(arr, len(events))
    if st != FDL_OK:
        raise FdlError(st)


# ---------------------------------------------------------------- forward-only variant and sibling operators
def _check(st: int) -> None:
    if st != FDL_OK:
        raise FdlError(st)


def fdl_forward_inference_workspace_bytes(dtype, M: int, K: int, N: int) -> int:
    return int(_lib.fdl_forward_inference_workspace_bytes(_dtype_code(dtype), M, K, N))


def fdl_forward_inference_raw(dtype, M, K, N, X, W, b, gamma, beta, eps, Y, workspace, workspace_bytes, stream) -> int:
    return int(_lib.fdl_forward_inference(_dtype_code(dtype), M, K, N, _ptr(X), _ptr(W), _ptr(b), _ptr(gamma), _ptr(beta),
                                          float(eps), _ptr(Y), _ptr(workspace), int(workspace_bytes), stream))


def fdl_forward_inference(dtype, X, W, b, gamma, beta, eps, Y, workspace, stream=None) -> None:
    """Y = LayerNorm(GELU(X W^T + b)) gamma + beta, nothing saved for backward."""
    M, K = X.shape
    _check(fdl_forward_inference_raw(dtype, M, K, W.shape[0], X, W, b, gamma, beta, eps, Y, workspace, _nbytes(workspace),
                                     _stream(stream)))


def fdl_linear_relu_workspace_bytes(dtype, M: int, K: int, N: int) -> int:
    return int(_lib.fdl_linear_relu_workspace_bytes(_dtype_code(dtype), M, K, N))


def fdl_linear_relu_forward_raw(dtype, M, K, N, X, W, b, Y, workspace, workspace_bytes, stream) -> int:
    return int(_lib.fdl_linear_relu_forward(_dtype_code(dtype), M, K, N, _ptr(X), _ptr(W), _ptr(b), _ptr(Y), _ptr(workspace),
                                            int(workspace_bytes), stream))


def fdl_linear_relu_forward(dtype, X, W, b, Y, workspace, stream=None) -> None:
    M, K = X.shape
    _check(fdl_linear_relu_forward_raw(dtype, M, K, W.shape[0], X, W, b, Y, workspace, _nbytes(workspace), _stream(stream)))


def fdl_linear_relu_backward_raw(dtype, M, K, N, dY, X, W, b, dX, dW, db, workspace, workspace_bytes, stream) -> int:
    return int(_lib.fdl_linear_relu_backward(_dtype_code(dtype), M, K, N, _ptr(dY), _ptr(X), _ptr(W), _ptr(b), _ptr(dX),
                                             _ptr(dW), _ptr(db), _ptr(workspace), int(workspace_bytes), stream))


def fdl_linear_relu_backward(dtype, dY, X, W, b, dX, dW, db, workspace, stream=None) -> None:
    M, K = X.shape
    _check(fdl_linear_relu_backward_raw(dtype, M, K, W.shape[0], dY, X, W, b, dX, dW, db, workspace, _nbytes(workspace),
                                        _stream(stream)))


def fdl_layernorm_forward_raw(dtype, M, N, A, gamma, beta, eps, Y, mean, rstd, stream) -> int:
    return int(_lib.fdl_layernorm_forward(_dtype_code(dtype), M, N, _ptr(A), _ptr(gamma), _ptr(beta), float(eps), _ptr(Y),
                                          _ptr(mean), _ptr(rstd), stream))


def fdl_layernorm_forward(dtype, A, gamma, beta, eps, Y, mean, rstd, stream=None) -> None:
    M, N = A.shape
    _check(fdl_layernorm_forward_raw(dtype, M, N, A, gamma, beta, eps, Y, mean, rstd, _stream(stream)))


def fdl_rmsnorm_forward_raw(dtype, M, N, A, weight, eps, Y, stream) -> int:
    return int(_lib.fdl_rmsnorm_forward(_dtype_code(dtype), M, N, _ptr(A), _ptr(weight), float(eps), _ptr(Y), stream))


def fdl_rmsnorm_forward(dtype, A, weight, eps, Y, stream=None) -> None:
    M, N = A.shape
    _check(fdl_rmsnorm_forward_raw(dtype, M, N, A, weight, eps, Y, _stream(stream)))


def fdl_llama_ffn_workspace_bytes(dtype, M: int, D: int, H: int) -> int:
    return int(_lib.fdl_llama_ffn_workspace_bytes(_dtype_code(dtype), M, D, H))


def fdl_llama_ffn_forward_raw(dtype, M, D, H, X, Wg, Wu, Wd, Y, workspace, workspace_bytes, stream) -> int:
    return int(_lib.fdl_llama_ffn_forward(_dtype_code(dtype), M, D, H, _ptr(X), _ptr(Wg), _ptr(Wu), _ptr(Wd), _ptr(Y),
                                          _ptr(workspace), int(workspace_bytes), stream))


def fdl_llama_ffn_forward(dtype, X, Wg, Wu, Wd, Y, workspace, stream=None) -> None:
    M, D = X.shape
    _check(fdl_llama_ffn_forward_raw(dtype, M, D, Wg.shape[0], X, Wg, Wu, Wd, Y, workspace, _nbytes(workspace),
                                     _stream(stream)))
