"""ctypes binding with the same names as the C ABI (include/tsvd.h).

Argument marshalling only.  If libtsvd.so has not been built the import of this module still
succeeds (so that the build step can import the package) but every call raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

TSVD_F32 = 0
TSVD_BF16 = 1
TSVD_FEATURE_MAJOR = 0
TSVD_TOKEN_MAJOR = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libtsvd.so")
_lib = None

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_sz = ctypes.c_size_t
_pi64 = ctypes.POINTER(ctypes.c_int64)

_PROTOTYPES = {
    "tsvd_packed_bytes": (_sz, [_i64, _i64, _i64]),
    "tsvd_pack_host": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _sz]),
    "tsvd_unpack_host": (ctypes.c_int, [_vp, _sz, _vp, _vp, _vp, _pi64, _pi64, _pi64]),
    "tsvd_dense_bytes": (_sz, [_i64, _i64]),
    "tsvd_dense_pack_host": (ctypes.c_int, [_vp, _i64, _i64, _vp, _sz]),
    "tsvd_dense_unpack_host": (ctypes.c_int, [_vp, _sz, _vp, _i64, _i64]),
    "tsvd_pack": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _sz, ctypes.POINTER(_vp)]),
    "tsvd_unpack": (ctypes.c_int, [_vp, _vp, _vp, _vp]),
    "tsvd_info": (ctypes.c_int, [_vp, _pi64, _pi64, _pi64, _pi64, _pi64]),
    "tsvd_workspace_bytes": (_sz, [_vp, _i64, ctypes.c_int]),
    "tsvd_forward": (ctypes.c_int, [_vp, _vp, ctypes.c_int, _i64, _i64, _vp, ctypes.c_int, _i64, _vp, _sz, _vp]),
    "tsvd_workspace_bytes_ex": (_sz, [_vp, _i64, ctypes.c_int, ctypes.c_int]),
    "tsvd_forward_ex": (ctypes.c_int, [_vp, _vp, ctypes.c_int, ctypes.c_int, _i64, _i64, _vp, _vp, ctypes.c_int, _i64,
                                       _vp, _sz, _vp]),
    "tsvd_forward_io": (ctypes.c_int, [_vp, _vp, ctypes.c_int, ctypes.c_int, _i64, _i64, _vp, _vp, ctypes.c_int, ctypes.c_int, _i64,
                                       _vp, _sz, _vp]),
    "tsvd_forward_noalloc": (ctypes.c_int, [_vp, _vp, ctypes.c_int, ctypes.c_int, _i64, _i64, _vp, _vp, ctypes.c_int, _i64, _vp]),
    "tsvd_tuning_set": (ctypes.c_int, [ctypes.c_char_p, ctypes.c_int]),
    "tsvd_tuning_reset": (None, []),
    "tsvd_tuning_forward_stages": (ctypes.c_int, [_vp, _vp, ctypes.c_int, ctypes.c_int, _i64, _i64, _vp, _vp, ctypes.c_int, _i64,
                                                  _vp, _sz, _vp, ctypes.c_int]),
    "tsvd_tuning_tile_shapes": (ctypes.c_int, [_vp, ctypes.c_longlong, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]),
    "tsvd_tuning_read_clocks": (ctypes.c_int, [_vp, _vp, ctypes.c_int]),
    "tsvd_ternarize": (ctypes.c_int, [_vp, _i64, _i64, _i64, ctypes.c_double, _vp, _i64, _vp, _vp]),
    "tsvd_fit_scales_workspace": (_sz, [_i64]),
    "tsvd_fit_scales": (ctypes.c_int, [_vp, _i64, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _sz, _vp, _vp]),
    "tsvd_residual": (ctypes.c_int, [_vp, _vp, _i64, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp]),
    "tsvd_leading_singular_pair_workspace": (_sz, [_i64, _i64]),
    "tsvd_leading_singular_pair": (ctypes.c_int, [_vp, _i64, _i64, ctypes.c_int32, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "tsvd_transition": (ctypes.c_int, [_vp, _i64, _i64, ctypes.c_double, ctypes.c_double, _i64, _vp, _vp, _vp, _pi64, _vp, _vp]),
    "tsvd_transition_q": (ctypes.c_int, [_vp, _i64, _i64, ctypes.c_double, ctypes.c_double, _i64, _i64, _vp, _vp, _vp, _pi64, _vp, _vp]),
    "tsvd_conv2d_workspace_bytes": (_sz, [_vp, _vp, _i64, _i64, _i64]),
    "tsvd_conv2d_forward": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, ctypes.c_int, _vp, _sz, _vp]),
    "tsvd_free": (None, [_vp]),
    "tsvd_strerror": (ctypes.c_char_p, [ctypes.c_int]),
}


class TsvdError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {tsvd_strerror(status)} (status {status})")


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libtsvd.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                               "`python -m paper_2308_07641_amd.build` (or __graft_entry__.build())")
        lib = ctypes.CDLL(_LIB_PATH)
        for name, (res, args) in _PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def tsvd_strerror(status: int) -> str:
    return load_library().tsvd_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != 0:
        raise TsvdError(status, where)


def _weights(U, S, V):
    U = np.ascontiguousarray(U, dtype=np.int8)
    V = np.ascontiguousarray(V, dtype=np.int8)
    S = np.ascontiguousarray(S, dtype=np.float32)
    if U.ndim != 2 or V.ndim != 2 or S.ndim != 1 or U.shape[1] != V.shape[0] or S.shape[0] != U.shape[1]:
        raise ValueError("expected U [M,K] int8, S [K] float32, V [K,N] int8")
    return U, S, V


def tsvd_packed_bytes(M: int, K: int, N: int) -> int:
    return int(load_library().tsvd_packed_bytes(M, K, N))


def tsvd_pack_host(U, S, V) -> np.ndarray:
    """Packs into a host uint8 array (no GPU needed)."""
    U, S, V = _weights(U, S, V)
    M, K = U.shape
    N = V.shape[1]
    blob = np.empty(tsvd_packed_bytes(M, K, N), dtype=np.uint8)
    _check(load_library().tsvd_pack_host(U.ctypes.data, S.ctypes.data, V.ctypes.data, M, K, N,
                                         blob.ctypes.data, blob.nbytes), "tsvd_pack_host")
    return blob


def tsvd_unpack_host(blob: np.ndarray):
    """Returns (U, S, V) from a host blob."""
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    lib = load_library()
    M, K, N = _i64(), _i64(), _i64()
    _check(lib.tsvd_unpack_host(blob.ctypes.data, blob.nbytes, None, None, None,
                                ctypes.byref(M), ctypes.byref(K), ctypes.byref(N)), "tsvd_unpack_host")
    U = np.empty((M.value, K.value), dtype=np.int8)
    S = np.empty(K.value, dtype=np.float32)
    V = np.empty((K.value, N.value), dtype=np.int8)
    _check(lib.tsvd_unpack_host(blob.ctypes.data, blob.nbytes, U.ctypes.data, S.ctypes.data, V.ctypes.data,
                                None, None, None), "tsvd_unpack_host")
    return U, S, V


def tsvd_dense_bytes(M: int, K: int) -> int:
    return int(load_library().tsvd_dense_bytes(M, K))


def tsvd_dense_pack_host(U) -> np.ndarray:
    """U int8 [M,K] -> the five-elements-per-byte code (host uint8 array)."""
    U = np.ascontiguousarray(U, dtype=np.int8)
    blob = np.empty(tsvd_dense_bytes(*U.shape), dtype=np.uint8)
    _check(load_library().tsvd_dense_pack_host(U.ctypes.data, U.shape[0], U.shape[1], blob.ctypes.data, blob.nbytes), "tsvd_dense_pack_host")
    return blob


def tsvd_dense_unpack_host(blob: np.ndarray, M: int, K: int) -> np.ndarray:
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    U = np.empty((M, K), dtype=np.int8)
    _check(load_library().tsvd_dense_unpack_host(blob.ctypes.data, blob.nbytes, U.ctypes.data, M, K), "tsvd_dense_unpack_host")
    return U


class Handle:
    """Owner of a tsvd_handle*; free with tsvd_free (also freed on garbage collection)."""

    def __init__(self, ptr: int, M: int, K: int, N: int, keepalive=None):
        self.ptr = ptr
        self.M, self.K, self.N = M, K, N
        self._keepalive = keepalive     # caller-provided device buffer, if any

    def __del__(self):
        try:
            tsvd_free(self)
        except Exception:
            pass


def tsvd_pack(U, S, V, dev_buf=None) -> Handle:
    """Packs and uploads to the current HIP device.  dev_buf: optional torch uint8 CUDA tensor."""
    U, S, V = _weights(U, S, V)
    M, K = U.shape
    N = V.shape[1]
    out = _vp()
    buf_ptr, buf_bytes = None, 0
    if dev_buf is not None:
        buf_ptr, buf_bytes = dev_buf.data_ptr(), dev_buf.numel() * dev_buf.element_size()
    _check(load_library().tsvd_pack(U.ctypes.data, S.ctypes.data, V.ctypes.data, M, K, N,
                                    buf_ptr, buf_bytes, ctypes.byref(out)), "tsvd_pack")
    return Handle(out.value, M, K, N, keepalive=dev_buf)


def tsvd_unpack(h: Handle):
    U = np.empty((h.M, h.K), dtype=np.int8)
    S = np.empty(h.K, dtype=np.float32)
    V = np.empty((h.K, h.N), dtype=np.int8)
    _check(load_library().tsvd_unpack(h.ptr, U.ctypes.data, S.ctypes.data, V.ctypes.data), "tsvd_unpack")
    return U, S, V


def tsvd_info(h: Handle) -> dict:
    vals = [_i64() for _ in range(5)]
    _check(load_library().tsvd_info(h.ptr, *[ctypes.byref(v) for v in vals]), "tsvd_info")
    return dict(zip(("M", "K", "N", "nnzU", "nnzV"), (v.value for v in vals)))


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return TSVD_F32
    if t.dtype == torch.bfloat16:
        return TSVD_BF16
    raise TypeError(f"unsupported activation dtype {t.dtype}")


def tsvd_workspace_bytes(h: Handle, B: int, x_dtype: int) -> int:
    return int(load_library().tsvd_workspace_bytes(h.ptr, B, x_dtype))


def tsvd_forward(h: Handle, x, y=None, workspace=None, stream=None):
    """y[M,B] (fp32) = U (diag(S) (V x)) for x [N,B] (or [N]) fp32/bf16 on the GPU.

    x, y, workspace are torch CUDA tensors used as plain device buffers; the work is
    enqueued on `stream` (default: torch's current stream) and not synchronised.
    """
    import torch
    if not x.is_cuda:
        raise ValueError("x must live on the GPU")
    x2 = x if x.dim() == 2 else x.unsqueeze(1)
    if x2.shape[0] != h.N or x2.stride(1) != 1:
        raise ValueError("x must be [N,B] with unit column stride")
    B = x2.shape[1]
    ldx = x2.stride(0) if x2.shape[0] > 1 else max(B, x2.stride(0))
    if y is None:
        y = torch.empty((h.M, B), dtype=torch.float32, device=x.device)
    if y.dtype != torch.float32 or y.shape != (h.M, B) or y.stride(1) != 1 or not y.is_cuda:
        raise ValueError("y must be a float32 GPU tensor [M,B] with unit column stride")
    ldy = y.stride(0) if y.shape[0] > 1 else max(B, y.stride(0))
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(load_library().tsvd_forward(h.ptr, x2.data_ptr(), _dtype_code(x2), B, ldx, y.data_ptr(), TSVD_F32, ldy,
                                       ws_ptr, ws_bytes, stream), "tsvd_forward")
    return y


def tsvd_workspace_bytes_ex(h: Handle, B: int, x_dtype: int, x_layout: int) -> int:
    return int(load_library().tsvd_workspace_bytes_ex(h.ptr, B, x_dtype, x_layout))


def tsvd_forward_ex(h: Handle, x, x_layout=TSVD_FEATURE_MAJOR, bias=None, y=None, y_dtype=TSVD_F32, workspace=None,
                    stream=None):
    """y[M,B] = U (diag(S) (V x)) + bias, fp32 or bf16; x is [N,B] (feature-major) or [B,N] (token-major).

    Same conventions as tsvd_forward; bias is a float32 GPU tensor [M] or None.
    """
    import torch
    if not x.is_cuda or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-d GPU tensor with unit inner stride")
    token_major = x_layout == TSVD_TOKEN_MAJOR
    B, feat = (x.shape[0], x.shape[1]) if token_major else (x.shape[1], x.shape[0])
    if feat != h.N:
        raise ValueError("x does not have N features")
    ldx = x.stride(0) if x.shape[0] > 1 else max(x.shape[1], x.stride(0))
    ydt = torch.bfloat16 if y_dtype == TSVD_BF16 else torch.float32
    if y is None:
        y = torch.empty((h.M, B), dtype=ydt, device=x.device)
    if y.dtype != ydt or y.shape != (h.M, B) or y.stride(1) != 1 or not y.is_cuda:
        raise ValueError("y must be a GPU tensor [M,B] of the requested type with unit column stride")
    ldy = y.stride(0) if y.shape[0] > 1 else max(B, y.stride(0))
    bias_ptr = None
    if bias is not None:
        if bias.dtype != torch.float32 or bias.shape != (h.M,) or not bias.is_cuda or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous float32 GPU tensor [M]")
        bias_ptr = bias.data_ptr()
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(load_library().tsvd_forward_ex(h.ptr, x.data_ptr(), _dtype_code(x), x_layout, B, ldx, bias_ptr, y.data_ptr(),
                                          y_dtype, ldy, ws_ptr, ws_bytes, stream), "tsvd_forward_ex")
    return y


def tsvd_forward_io(h: Handle, x, x_layout=TSVD_FEATURE_MAJOR, bias=None, y=None, y_dtype=TSVD_F32, y_layout=TSVD_FEATURE_MAJOR,
                    workspace=None, stream=None):
    """tsvd_forward_ex with the layout of y chosen too: [M,B] (feature-major) or [B,M] (token-major)."""
    import torch
    if not x.is_cuda or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-d GPU tensor with unit inner stride")
    B, feat = (x.shape[0], x.shape[1]) if x_layout == TSVD_TOKEN_MAJOR else (x.shape[1], x.shape[0])
    if feat != h.N:
        raise ValueError("x does not have N features")
    ldx = x.stride(0) if x.shape[0] > 1 else max(x.shape[1], x.stride(0))
    ydt = torch.bfloat16 if y_dtype == TSVD_BF16 else torch.float32
    yshape = (B, h.M) if y_layout == TSVD_TOKEN_MAJOR else (h.M, B)
    if y is None:
        y = torch.empty(yshape, dtype=ydt, device=x.device)
    if y.dtype != ydt or tuple(y.shape) != yshape or y.stride(1) != 1 or not y.is_cuda:
        raise ValueError("y must be a GPU tensor of the requested type and layout with unit inner stride")
    ldy = y.stride(0) if y.shape[0] > 1 else max(y.shape[1], y.stride(0))
    bias_ptr = None
    if bias is not None:
        if bias.dtype != torch.float32 or bias.shape != (h.M,) or not bias.is_cuda or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous float32 GPU tensor [M]")
        bias_ptr = bias.data_ptr()
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(load_library().tsvd_forward_io(h.ptr, x.data_ptr(), _dtype_code(x), x_layout, B, ldx, bias_ptr, y.data_ptr(),
                                          y_dtype, y_layout, ldy, ws_ptr, ws_bytes, stream), "tsvd_forward_io")
    return y


TSVD_NOALLOC_MAX_WORKSPACE = 16 << 20


def tsvd_forward_noalloc(h: Handle, x, y, x_layout=TSVD_FEATURE_MAJOR, bias=None, y_dtype=TSVD_F32, stream=None):
    """tsvd_forward_ex on the library's fixed per-GPU workspace; y must be given (nothing is allocated)."""
    import torch
    if not x.is_cuda or x.dim() != 2 or x.stride(1) != 1:
        raise ValueError("x must be a 2-d GPU tensor with unit inner stride")
    token_major = x_layout == TSVD_TOKEN_MAJOR
    B, feat = (x.shape[0], x.shape[1]) if token_major else (x.shape[1], x.shape[0])
    if feat != h.N:
        raise ValueError("x does not have N features")
    ldx = x.stride(0) if x.shape[0] > 1 else max(x.shape[1], x.stride(0))
    ydt = torch.bfloat16 if y_dtype == TSVD_BF16 else torch.float32
    if y.dtype != ydt or y.shape != (h.M, B) or y.stride(1) != 1 or not y.is_cuda:
        raise ValueError("y must be a GPU tensor [M,B] of the requested type with unit column stride")
    ldy = y.stride(0) if y.shape[0] > 1 else max(B, y.stride(0))
    bias_ptr = None
    if bias is not None:
        if bias.dtype != torch.float32 or bias.shape != (h.M,) or not bias.is_cuda or not bias.is_contiguous():
            raise ValueError("bias must be a contiguous float32 GPU tensor [M]")
        bias_ptr = bias.data_ptr()
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(load_library().tsvd_forward_noalloc(h.ptr, x.data_ptr(), _dtype_code(x), x_layout, B, ldx, bias_ptr, y.data_ptr(),
                                               y_dtype, ldy, stream), "tsvd_forward_noalloc")
    return y


# ---- diagnostic interface (include/tsvd_tuning.h): for the tests and the benchmark only
def tsvd_tuning_set(name: str, value: int) -> None:
    if load_library().tsvd_tuning_set(name.encode(), int(value)) != 0:
        raise ValueError(f"unknown tuning switch {name!r}")


def tsvd_tuning_reset() -> None:
    load_library().tsvd_tuning_reset()


def tsvd_tuning_forward_stages(h: Handle, x, y, stage_mask: int, workspace=None, stream=None):
    """tsvd_forward restricted to the kernels in stage_mask (1 column maxima, 2 stage V, 4 stage U)."""
    import torch
    x2 = x if x.dim() == 2 else x.unsqueeze(1)
    B = x2.shape[1]
    ldx = x2.stride(0) if x2.shape[0] > 1 else max(B, x2.stride(0))
    ldy = y.stride(0) if y.shape[0] > 1 else max(B, y.stride(0))
    ws_ptr, ws_bytes = None, 0
    if workspace is not None:
        ws_ptr, ws_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    if stream is None:
        stream = torch.cuda.current_stream(x.device).cuda_stream
    _check(load_library().tsvd_tuning_forward_stages(h.ptr, x2.data_ptr(), _dtype_code(x2), TSVD_FEATURE_MAJOR, B, ldx, None,
                                                     y.data_ptr(), TSVD_F32, ldy, ws_ptr, ws_bytes, stream, int(stage_mask)),
           "tsvd_tuning_forward_stages")
    return y


def tsvd_tuning_tile_shapes(h: Handle, B: int):
    sv, su = ctypes.c_int(-1), ctypes.c_int(-1)
    if load_library().tsvd_tuning_tile_shapes(h.ptr, B, ctypes.byref(sv), ctypes.byref(su)) != 0:
        raise ValueError("tsvd_tuning_tile_shapes")
    return sv.value, su.value


def tsvd_tuning_read_clocks(h: Handle, workgroups: int) -> np.ndarray:
    out = np.zeros((workgroups, 16), dtype=np.int64)
    if load_library().tsvd_tuning_read_clocks(h.ptr, out.ctypes.data, workgroups) != 0:
        raise ValueError("tsvd_tuning_read_clocks: the handle was not packed with TSVD_CLOCKS = 1")
    return out


# ---- direct transition W -> (U, S, V) (include/tsvd_transition.h); torch CUDA tensors as device buffers
def _stream(t, stream):
    import torch
    return torch.cuda.current_stream(t.device).cuda_stream if stream is None else stream


def _need(t, dtype, shape, what):
    if not t.is_cuda or t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous GPU tensor {dtype} {tuple(shape)}")


def tsvd_ternarize(x, theta: float, stream=None):
    """Algorithm 1 for the rows of x [count, n] (float64): returns (t int8 [count, n], status int32 [count])."""
    import torch
    if x.dim() != 2:
        raise ValueError("x must be [count, n]")
    _need(x, torch.float64, x.shape, "x")
    count, n = x.shape
    t = torch.empty((count, n), dtype=torch.int8, device=x.device)
    status = torch.empty((count,), dtype=torch.int32, device=x.device)
    _check(load_library().tsvd_ternarize(x.data_ptr(), n, count, n, float(theta), t.data_ptr(), n, status.data_ptr(),
                                         _stream(x, stream)), "tsvd_ternarize")
    return t, status


def tsvd_fit_scales(U, V, W, stream=None):
    """Eq. (3): S [K] float64 for U int8 [M, K], V int8 [K, N], W float64 [M, N]; also returns the solver's iteration count tensor."""
    import torch
    M, K = U.shape
    N = V.shape[1]
    _need(U, torch.int8, (M, K), "U"); _need(V, torch.int8, (K, N), "V"); _need(W, torch.float64, (M, N), "W")
    S = torch.empty((K,), dtype=torch.float64, device=W.device)
    iters = torch.zeros((1,), dtype=torch.int32, device=W.device)
    nbytes = int(load_library().tsvd_fit_scales_workspace(K))
    ws = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=W.device)
    _check(load_library().tsvd_fit_scales(U.data_ptr(), K, V.data_ptr(), W.data_ptr(), M, K, N, S.data_ptr(), ws.data_ptr(), nbytes,
                                          iters.data_ptr(), _stream(W, stream)), "tsvd_fit_scales")
    return S, iters


def tsvd_residual(W, U, S, V, stream=None):
    """R = W - U diag(S) V (float64 [M, N]) and |R|_F^2 (float64 [1])."""
    import torch
    M, K = U.shape
    N = V.shape[1]
    _need(U, torch.int8, (M, K), "U"); _need(V, torch.int8, (K, N), "V"); _need(W, torch.float64, (M, N), "W")
    _need(S, torch.float64, (K,), "S")
    R = torch.empty_like(W)
    norm2 = torch.empty((1,), dtype=torch.float64, device=W.device)
    _check(load_library().tsvd_residual(W.data_ptr(), U.data_ptr(), K, S.data_ptr(), V.data_ptr(), M, K, N, R.data_ptr(),
                                        norm2.data_ptr(), _stream(W, stream)), "tsvd_residual")
    return R, norm2


def tsvd_leading_singular_pair(R, max_iters: int = 512, stream=None):
    """(u [M], sigma [1], v [N], steps [1]) of R float64 [M, N] by Lanczos bidiagonalisation."""
    import torch
    M, N = R.shape
    _need(R, torch.float64, (M, N), "R")
    u = torch.empty((M,), dtype=torch.float64, device=R.device)
    v = torch.empty((N,), dtype=torch.float64, device=R.device)
    sigma = torch.empty((1,), dtype=torch.float64, device=R.device)
    iters = torch.zeros((1,), dtype=torch.int32, device=R.device)
    nbytes = int(load_library().tsvd_leading_singular_pair_workspace(M, N))
    ws = torch.empty((max(nbytes, 256),), dtype=torch.uint8, device=R.device)
    _check(load_library().tsvd_leading_singular_pair(R.data_ptr(), M, N, int(max_iters), u.data_ptr(), v.data_ptr(), sigma.data_ptr(),
                                                     iters.data_ptr(), ws.data_ptr(), nbytes, _stream(R, stream)),
           "tsvd_leading_singular_pair")
    return u, sigma, v, iters


def tsvd_transition(W, theta: float, tol: float, max_rank: int, stream=None, q: int = 1):
    """Algorithm 2 (q components per iteration) for W float64 [M, N]: returns (U int8 [M, K], S float64 [K],
    V int8 [K, N], errors list with one entry per component, status)."""
    import torch
    M, N = W.shape
    _need(W, torch.float64, (M, N), "W")
    U = torch.empty((M, max_rank), dtype=torch.int8, device=W.device)
    V = torch.empty((max_rank, N), dtype=torch.int8, device=W.device)
    S = torch.empty((max_rank,), dtype=torch.float64, device=W.device)
    rank = _i64(0)
    errors = np.zeros(max_rank, dtype=np.float64)
    status = load_library().tsvd_transition_q(W.data_ptr(), M, N, float(theta), float(tol), int(max_rank), int(q), U.data_ptr(),
                                              S.data_ptr(), V.data_ptr(), ctypes.byref(rank), errors.ctypes.data, _stream(W, stream))
    K = int(rank.value)
    if status != 0 and not (status == 2 and K > 0):
        _check(status, "tsvd_transition")
    return U[:, :K].contiguous(), S[:K].clone(), V[:K, :].contiguous(), errors[:K].tolist(), status


# ---- convolution forms (include/tsvd_conv.h)
class ConvGeometry(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("form", "c_in", "c_out", "k1", "k2", "stride1", "stride2", "pad1", "pad2", "dil1", "dil2", "groups")]


def tsvd_conv2d_forward(h: Handle, form: int, c_in: int, c_out: int, k1: int, k2: int, x, stride=(1, 1), pad=(0, 0), dil=(1, 1),
                        bias=None, y_dtype=TSVD_F32, stream=None, groups=1):
    """y [C_out, images, Ho, Wo] = conv2d(x [C_in, images, H, W] bf16) with the kernel in ternary-SVD form `form`
    (groups > 1: form 0 with per-group factors, see include/tsvd_conv.h)."""
    import torch
    if not x.is_cuda or x.dtype != torch.bfloat16 or x.dim() != 4 or x.shape[0] != c_in or not x.is_contiguous():
        raise ValueError("x must be a contiguous bf16 GPU tensor [C_in, images, H, W]")
    _, images, H, W = x.shape
    g = ConvGeometry(form, c_in, c_out, k1, k2, stride[0], stride[1], pad[0], pad[1], dil[0], dil[1], groups)
    lib = load_library()
    nbytes = int(lib.tsvd_conv2d_workspace_bytes(h.ptr, ctypes.addressof(g), images, H, W))
    if nbytes == 0:
        raise ValueError("geometry does not fit the packed matrix (or is invalid)")
    Ho = (H + 2 * pad[0] - dil[0] * (k1 - 1) - 1) // stride[0] + 1
    Wo = (W + 2 * pad[1] - dil[1] * (k2 - 1) - 1) // stride[1] + 1
    ws = torch.empty((nbytes,), dtype=torch.uint8, device=x.device)
    y = torch.empty((c_out, images, Ho, Wo), dtype=torch.bfloat16 if y_dtype == TSVD_BF16 else torch.float32, device=x.device)
    bias_ptr = None
    if bias is not None:
        _need(bias, torch.float32, (c_out,), "bias")
        bias_ptr = bias.data_ptr()
    _check(lib.tsvd_conv2d_forward(h.ptr, ctypes.addressof(g), x.data_ptr(), images, H, W, bias_ptr, y.data_ptr(), y_dtype,
                                   ws.data_ptr(), nbytes, _stream(x, stream)), "tsvd_conv2d_forward")
    return y


def tsvd_free(h: Handle) -> None:
    if h is not None and getattr(h, "ptr", None):
        load_library().tsvd_free(h.ptr)
        h.ptr = None
