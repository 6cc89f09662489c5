"""Thin Python binding of libams.so, the MI355X AMS-Quant weight-only quantized Linear.

Argument marshalling only: every step of the path (quantize, pack, restore, multiply)
runs inside the C-ABI library declared in include/ams.h.  PyTorch is used for device
memory and streams.  There is no fallback: if the library has not been built
(``python __graft_entry__.py``) every call raises.
"""

from __future__ import annotations

import ctypes
import os

import numpy as np

FP533 = 0  # AMS_FMT_FP533_E2M3
FP425 = 1  # AMS_FMT_FP425_E2M2
FP45 = 2  # AMS_FMT_FP45_E2M2
FP433 = 3  # AMS_FMT_FP433_E2M2
FP6 = 4  # AMS_FMT_FP6_E2M3
FP5 = 5  # AMS_FMT_FP5_E2M2
FP4 = 6  # AMS_FMT_FP4_E2M1
SEARCH_SET_BIT = 0  # AMS_SEARCH_SET_BIT
SEARCH_REROUND = 1  # AMS_SEARCH_REROUND
MAX_M = 32

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libams.so")
_lib = None

_i64, _int, _vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p


class AmsError(RuntimeError):
    pass


def load_library():
    """Load libams.so (once) and declare the signatures of include/ams.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise AmsError(f"{_LIB_PATH} is missing: build it with `python __graft_entry__.py`")
    lib = ctypes.CDLL(_LIB_PATH)
    lib.ams_version.restype = _int
    lib.ams_init.restype = _int
    lib.ams_strerror.restype = ctypes.c_char_p
    lib.ams_strerror.argtypes = [_int]
    lib.ams_group_size.argtypes = [_int]
    lib.ams_code_bits.argtypes = [_int]
    lib.ams_packed_bytes.argtypes = [_int, _i64, _i64, ctypes.POINTER(ctypes.c_size_t)]
    lib.ams_canonical_bytes.argtypes = [_int, _i64, _i64, ctypes.POINTER(ctypes.c_size_t)]
    lib.ams_pack.argtypes = [_int, _vp, _i64, _i64, _i64, _vp, _vp, _vp]
    lib.ams_pack_ex.argtypes = [_int, _int, _vp, _i64, _i64, _i64, _vp, _vp, _vp]
    lib.ams_group_scales_count.argtypes = [_int, _i64, _i64, _i64, ctypes.POINTER(ctypes.c_size_t)]
    lib.ams_pack_grouped.argtypes = [_int, _int, _i64, _vp, _i64, _i64, _i64, _vp, _vp, _vp]
    lib.ams_dequant_grouped.argtypes = [_int, _vp, _vp, _i64, _vp, _i64, _i64, _int, _vp]
    lib.ams_linear_grouped.argtypes = [_vp, _vp, _i64, _vp, _vp, _int, _i64, _i64, _int, _vp]
    lib.ams_pack_per_tensor.argtypes = [_int, _int, _vp, _i64, _i64, _i64, _vp, _vp, _vp]
    lib.ams_pack_codes.argtypes = [_int, _vp, _i64, _i64, _vp]
    lib.ams_unpack_host.argtypes = [_int, _vp, _i64, _i64, _vp]
    lib.ams_dequant.argtypes = [_int, _vp, _vp, _vp, _i64, _i64, _int, _vp]
    lib.ams_linear.argtypes = [_vp, _vp, _vp, _vp, _int, _i64, _i64, _int, _vp]
    lib.ams_fp16_linear.argtypes = [_vp, _vp, _vp, _int, _i64, _i64, _vp]
    lib.ams_linear_workspace_bytes.argtypes = [_int, _int, _i64, _i64, ctypes.POINTER(ctypes.c_size_t)]
    lib.ams_linear_static_ws.argtypes = [_vp, _vp, _vp, _vp, _int, _i64, _i64, _int, _vp]
    lib.ams_linear_ws.argtypes = [_vp, _vp, _vp, _vp, _int, _i64, _i64, _int, _vp, ctypes.c_size_t, _vp]
    lib.ams_fp16_linear_ws.argtypes = [_vp, _vp, _vp, _int, _i64, _i64, _vp, ctypes.c_size_t, _vp]
    lib.ams_linear_plan.argtypes = [_int, _int, _i64, _i64, _int, ctypes.c_char_p, ctypes.c_size_t]
    lib.ams_read_probe.argtypes = [_vp, ctypes.c_size_t, _vp, _vp]
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise AmsError(f"{what}: {load_library().ams_strerror(rc).decode()} ({rc})")


def _np_ptr(a: np.ndarray):
    return a.ctypes.data_as(_vp)


def ams_version() -> int:
    return load_library().ams_version()


def ams_init() -> None:
    """Check the current device and raise the kernels' LDS limits (needed only before a first call under stream capture)."""
    _check(load_library().ams_init(), "ams_init")


def ams_packed_bytes(fmt: int, N: int, K: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().ams_packed_bytes(fmt, N, K, ctypes.byref(out)), "ams_packed_bytes")
    return out.value


def ams_canonical_bytes(fmt: int, N: int, K: int) -> int:
    out = ctypes.c_size_t()
    _check(load_library().ams_canonical_bytes(fmt, N, K, ctypes.byref(out)), "ams_canonical_bytes")
    return out.value


def ams_pack_ex(fmt: int, search: int, W: np.ndarray, return_codes: bool = False):
    """Quantize + pack host fp16 weights [N,K] with the given search.  Returns (packed uint8, scales float16[, codes uint8])."""
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 array")
    W = np.ascontiguousarray(W)
    N, K = W.shape
    packed = np.empty(ams_packed_bytes(fmt, N, K), dtype=np.uint8)
    scales = np.empty(N, dtype=np.float16)
    codes = np.empty((N, K), dtype=np.uint8) if return_codes else None
    rc = load_library().ams_pack_ex(fmt, search, _np_ptr(W), N, K, K, _np_ptr(packed), _np_ptr(scales), _np_ptr(codes) if return_codes else None)
    _check(rc, "ams_pack_ex")
    return (packed, scales, codes) if return_codes else (packed, scales)


def ams_pack(fmt: int, W: np.ndarray, return_codes: bool = False):
    """Quantize + pack host fp16 weights [N,K].  Returns (packed uint8, scales float16[, codes uint8])."""
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 array")
    W = np.ascontiguousarray(W)
    N, K = W.shape
    packed = np.empty(ams_packed_bytes(fmt, N, K), dtype=np.uint8)
    scales = np.empty(N, dtype=np.float16)
    codes = np.empty((N, K), dtype=np.uint8) if return_codes else None
    rc = load_library().ams_pack(fmt, _np_ptr(W), N, K, K, _np_ptr(packed), _np_ptr(scales), _np_ptr(codes) if return_codes else None)
    _check(rc, "ams_pack")
    return (packed, scales, codes) if return_codes else (packed, scales)


def ams_pack_codes(fmt: int, codes: np.ndarray) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    N, K = codes.shape
    packed = np.empty(ams_packed_bytes(fmt, N, K), dtype=np.uint8)
    _check(load_library().ams_pack_codes(fmt, _np_ptr(codes), N, K, _np_ptr(packed)), "ams_pack_codes")
    return packed


def ams_unpack_host(fmt: int, packed: np.ndarray, N: int, K: int) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    if packed.size != ams_packed_bytes(fmt, N, K):
        raise ValueError("packed buffer has the wrong size")
    codes = np.empty((N, K), dtype=np.uint8)
    _check(load_library().ams_unpack_host(fmt, _np_ptr(packed), N, K, _np_ptr(codes)), "ams_unpack_host")
    return codes


def _stream():
    import torch

    return torch.cuda.current_stream().cuda_stream


def _dev_ptr(t, dtype=None):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def ams_dequant(fmt: int, W_packed, scales, N: int, K: int, scaled: bool = True, out=None):
    """Restore a packed matrix (uint8 CUDA tensor) to fp16 [N,K] on the GPU."""
    import torch

    if W_packed.numel() != ams_packed_bytes(fmt, N, K):
        raise ValueError("packed buffer has the wrong size")
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=W_packed.device)
    sp = _dev_ptr(scales, torch.float16) if scales is not None else None
    if scales is not None and scales.numel() != N:
        raise ValueError("scales must have N entries")
    rc = load_library().ams_dequant(fmt, _dev_ptr(W_packed, torch.uint8), sp, _dev_ptr(out, torch.float16), N, K, int(scaled), _stream())
    _check(rc, "ams_dequant")
    return out


def ams_linear(W_packed, scales, X, N: int, fmt: int, out=None):
    """Y = X @ DeQ(W)^T on the GPU.  X fp16 [M,K] CUDA tensor; returns fp16 [M,N]."""
    import torch

    M, K = X.shape
    if W_packed.numel() != ams_packed_bytes(fmt, N, K):
        raise ValueError("packed buffer has the wrong size")
    if scales.numel() != N:
        raise ValueError("scales must have N entries")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = load_library().ams_linear(
        _dev_ptr(W_packed, torch.uint8), _dev_ptr(scales, torch.float16), _dev_ptr(X, torch.float16), _dev_ptr(out, torch.float16), M, N, K, fmt, _stream()
    )
    _check(rc, "ams_linear")
    return out


def ams_fp16_linear(W, X, out=None):
    """The fp16 baseline Y = X @ W^T on the GPU.  W fp16 [N,K], X fp16 [M,K]."""
    import torch

    N, K = W.shape
    M = X.shape[0]
    if X.shape[1] != K:
        raise ValueError("X and W disagree in K")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = load_library().ams_fp16_linear(_dev_ptr(W, torch.float16), _dev_ptr(X, torch.float16), _dev_ptr(out, torch.float16), M, N, K, _stream())
    _check(rc, "ams_fp16_linear")
    return out


def ams_read_probe(buf, nbytes: int = None):
    """Measurement aid: a bare streaming read of the first nbytes of a CUDA tensor (default: all of it)."""
    if nbytes is None:
        nbytes = buf.numel() * buf.element_size()
    if nbytes > buf.numel() * buf.element_size():
        raise ValueError("nbytes exceeds the buffer")
    _check(load_library().ams_read_probe(_dev_ptr(buf), nbytes, None, _stream()), "ams_read_probe")


def ams_group_scales_count(fmt: int, N: int, K: int, scale_group: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load_library().ams_group_scales_count(fmt, N, K, scale_group, ctypes.byref(out)), "ams_group_scales_count")
    return out.value


def ams_pack_grouped(fmt: int, W: np.ndarray, scale_group: int, search: int = SEARCH_SET_BIT, return_codes: bool = False):
    """Quantize + pack with one scale per run of scale_group input channels.  The scales come back in the
    order the kernels read them: [strip of 16 rows, run, row inside the strip]."""
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 array")
    W = np.ascontiguousarray(W)
    N, K = W.shape
    packed = np.empty(ams_packed_bytes(fmt, N, K), dtype=np.uint8)
    n_sg = -(-K // scale_group)
    scales = np.empty(ams_group_scales_count(fmt, N, K, scale_group), dtype=np.float16).reshape(-1, n_sg, 16)
    codes = np.empty((N, K), dtype=np.uint8) if return_codes else None
    rc = load_library().ams_pack_grouped(fmt, search, scale_group, _np_ptr(W), N, K, K, _np_ptr(packed), _np_ptr(scales), _np_ptr(codes) if return_codes else None)
    _check(rc, "ams_pack_grouped")
    return (packed, scales, codes) if return_codes else (packed, scales)


def ams_dequant_grouped(fmt: int, W_packed, scales, scale_group: int, N: int, K: int, scaled: bool = True, out=None):
    import torch

    if W_packed.numel() != ams_packed_bytes(fmt, N, K):
        raise ValueError("packed buffer has the wrong size")
    if scales.numel() != ams_group_scales_count(fmt, N, K, scale_group):
        raise ValueError("scale buffer has the wrong size")
    if out is None:
        out = torch.empty((N, K), dtype=torch.float16, device=W_packed.device)
    rc = load_library().ams_dequant_grouped(fmt, _dev_ptr(W_packed, torch.uint8), _dev_ptr(scales, torch.float16), scale_group, _dev_ptr(out, torch.float16), N, K, int(scaled), _stream())
    _check(rc, "ams_dequant_grouped")
    return out


def ams_linear_grouped(W_packed, scales, scale_group: int, X, N: int, fmt: int, out=None):
    import torch

    M, K = X.shape
    if W_packed.numel() != ams_packed_bytes(fmt, N, K):
        raise ValueError("packed buffer has the wrong size")
    if scales.numel() != ams_group_scales_count(fmt, N, K, scale_group):
        raise ValueError("scale buffer has the wrong size")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = load_library().ams_linear_grouped(
        _dev_ptr(W_packed, torch.uint8), _dev_ptr(scales, torch.float16), scale_group, _dev_ptr(X, torch.float16), _dev_ptr(out, torch.float16), M, N, K, fmt, _stream()
    )
    _check(rc, "ams_linear_grouped")
    return out


def ams_linear_workspace_bytes(fmt: int, M: int, N: int, K: int) -> int:
    """Bytes of workspace ams_linear_ws wants for this shape (fmt = -1: the fp16 baseline); may be 0."""
    out = ctypes.c_size_t(0)
    _check(load_library().ams_linear_workspace_bytes(fmt, M, N, K, ctypes.byref(out)), "ams_linear_workspace_bytes")
    return out.value


def ams_linear_ws(W_packed, scales, X, N: int, fmt: int, workspace, out=None):
    """ams_linear with a workspace (a zero-filled uint8 CUDA tensor, reusable from call to call)."""
    import torch

    M, K = X.shape
    if W_packed.numel() != ams_packed_bytes(fmt, N, K):
        raise ValueError("packed buffer has the wrong size")
    if scales.numel() != N:
        raise ValueError("scales must have N entries")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = load_library().ams_linear_ws(
        _dev_ptr(W_packed, torch.uint8), _dev_ptr(scales, torch.float16), _dev_ptr(X, torch.float16), _dev_ptr(out, torch.float16), M, N, K, fmt,
        _dev_ptr(workspace, torch.uint8) if workspace is not None else None, workspace.numel() if workspace is not None else 0, _stream()
    )
    _check(rc, "ams_linear_ws")
    return out


def ams_linear_static_ws(W_packed, scales, X, N: int, fmt: int, out=None):
    """ams_linear_ws with the library's own static scratch as the workspace (allocates nothing)."""
    import torch

    M, K = X.shape
    if W_packed.numel() != ams_packed_bytes(fmt, N, K):
        raise ValueError("packed buffer has the wrong size")
    if scales.numel() != N:
        raise ValueError("scales must have N entries")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = load_library().ams_linear_static_ws(
        _dev_ptr(W_packed, torch.uint8), _dev_ptr(scales, torch.float16), _dev_ptr(X, torch.float16), _dev_ptr(out, torch.float16), M, N, K, fmt, _stream()
    )
    _check(rc, "ams_linear_static_ws")
    return out


def ams_fp16_linear_ws(W, X, workspace, out=None):
    import torch

    N, K = W.shape
    M = X.shape[0]
    if X.shape[1] != K:
        raise ValueError("X and W disagree in K")
    if out is None:
        out = torch.empty((M, N), dtype=torch.float16, device=X.device)
    rc = load_library().ams_fp16_linear_ws(
        _dev_ptr(W, torch.float16), _dev_ptr(X, torch.float16), _dev_ptr(out, torch.float16), M, N, K,
        _dev_ptr(workspace, torch.uint8) if workspace is not None else None, workspace.numel() if workspace is not None else 0, _stream()
    )
    _check(rc, "ams_fp16_linear_ws")
    return out


def ams_linear_plan(fmt: int, M: int, N: int, K: int, with_workspace: bool = False) -> str:
    """Which kernel and launch shape the library would use for this problem (fmt = -1: the fp16 baseline)."""
    buf = ctypes.create_string_buffer(256)
    _check(load_library().ams_linear_plan(fmt, M, N, K, int(with_workspace), buf, len(buf)), "ams_linear_plan")
    return buf.value.decode()


def ams_pack_per_tensor(fmt: int, W: np.ndarray, search: int = SEARCH_SET_BIT, return_codes: bool = False):
    """Quantize + pack with one scale for the whole matrix; returns it once per row, like ams_pack."""
    if W.dtype != np.float16 or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 array")
    W = np.ascontiguousarray(W)
    N, K = W.shape
    packed = np.empty(ams_packed_bytes(fmt, N, K), dtype=np.uint8)
    scales = np.empty(N, dtype=np.float16)
    codes = np.empty((N, K), dtype=np.uint8) if return_codes else None
    rc = load_library().ams_pack_per_tensor(fmt, search, _np_ptr(W), N, K, K, _np_ptr(packed), _np_ptr(scales), _np_ptr(codes) if return_codes else None)
    _check(rc, "ams_pack_per_tensor")
    return (packed, scales, codes) if return_codes else (packed, scales)
