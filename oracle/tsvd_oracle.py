"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

forward() calls the plain C loops of tsvd_oracle.c (fp64, natural order); the
remaining functions restate the paper's operation counts:

  * op_counts      -- supplement Table S1: per token the map costs K
                      multiplications and nnz(U)+nnz(V) = r K (M+N) additions.
  * acceleration   -- supplement Table S2, TSVD row, with the instruction cost
                      model 1 Mul = (d-2) Add of the section "Hardware Cost of
                      Basic Instruction": M N (d-1) / (K (d-2) + r K (M+N)).
  * critical_rank  -- Eq. (2): the rank at which that acceleration equals 1.

Nothing here is imported by the GPU library or its binding.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tsvd_oracle.c")
_LIB = os.path.join(_HERE, "libtsvd_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile tsvd_oracle.c with gcc (-O2, OpenMP) into libtsvd_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p = ctypes.c_void_p
        i64 = ctypes.c_int64
        lib.tsvd_oracle_forward.argtypes = [p, p, p, p, p, i64, i64, i64, i64]
        lib.tsvd_oracle_forward.restype = ctypes.c_int
        lib.tsvd_oracle_forward_vec.argtypes = [p, p, p, p, p, p, i64, i64, i64]
        lib.tsvd_oracle_forward_vec.restype = ctypes.c_int
        lib.tsvd_oracle_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def threads() -> int:
    return int(_load().tsvd_oracle_threads())


def _check(U, S, V, X):
    U = np.ascontiguousarray(U, dtype=np.int8)
    V = np.ascontiguousarray(V, dtype=np.int8)
    S = np.ascontiguousarray(S, dtype=np.float32)
    X = np.asarray(X)
    if X.ndim == 1:
        X = X[:, None]
    X = np.ascontiguousarray(X, dtype=np.float64)      # bf16 / fp32 -> fp64 is exact
    M, K = U.shape
    K2, N = V.shape
    if K2 != K or S.shape != (K,) or X.shape[0] != N:
        raise ValueError("shape mismatch: U [M,K], S [K], V [K,N], X [N,B] expected")
    return U, S, V, X, M, K, N


def forward(U, S, V, X) -> np.ndarray:
    """Y = U (diag(S) (V X)) in fp64; X is [N,B] (or [N]); returns [M,B] float64."""
    U, S, V, X, M, K, N = _check(U, S, V, X)
    B = X.shape[1]
    Y = np.empty((M, B), dtype=np.float64)
    lib = _load()
    if B == 1:
        z = np.empty(K, dtype=np.float64)
        rc = lib.tsvd_oracle_forward_vec(U.ctypes.data, S.ctypes.data, V.ctypes.data,
                                         X.ctypes.data, Y.ctypes.data, z.ctypes.data, M, K, N)
    else:
        rc = lib.tsvd_oracle_forward(U.ctypes.data, S.ctypes.data, V.ctypes.data,
                                     X.ctypes.data, Y.ctypes.data, M, K, N, B)
    if rc == 2:
        raise ValueError("U or V holds an entry outside {-1, 0, +1}")
    if rc != 0:
        raise RuntimeError(f"oracle failed with status {rc}")
    return Y


def forward_columns(U, S, V, X, cols) -> np.ndarray:
    """Outputs for a subset of tokens: columns are independent, so this is exact."""
    X = np.asarray(X)
    return forward(U, S, V, X[:, np.asarray(cols, dtype=np.int64)])


def round_to_bf16(y) -> np.ndarray:
    """Nearest bf16 value (8 significant bits, ties to even) of each fp64 entry, as fp64.

    Written from the definition of the format: split off the binary exponent, round the
    significand to 8 bits with the ties-to-even rule of np.rint, put the exponent back.
    Values below the bf16 normal range (2^-126) are rounded on the fixed subnormal grid 2^-133.
    """
    y = np.asarray(y, dtype=np.float64)
    m, e = np.frexp(y)                                  # y = m * 2^e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)                             # subnormals share the exponent of 2^-126
    m = y / np.ldexp(1.0, e)
    return np.ldexp(np.rint(np.ldexp(m, 8)), e - 8)


def forward_layer(U, S, V, X, bias=None, x_layout="feature_major", y_dtype="f32", y_layout="feature_major") -> np.ndarray:
    """The map as a linear layer uses it: Y = U (diag(S) (V X)) + bias, per token.

    The paper's listing of a converted network (supplement) shows its ternary-SVD linear
    layers with bias=True: the bias [M] is added to every token's output.  x_layout
    "token_major" takes X as [B,N] (one row per token).  y_dtype "bf16" rounds the result
    (after the bias) to the nearest bf16 value; the return is float64, [M,B] or, with y_layout
    "token_major", [B,M]: one row per token, written out token by token below (row b of the
    result is the layer's output for token b, i.e. for column b / row b of X).
    """
    X = np.asarray(X)
    if x_layout == "token_major":
        X = X.T
    elif x_layout != "feature_major":
        raise ValueError("x_layout")
    Y = forward(U, S, V, X)
    if bias is not None:
        b = np.asarray(bias, dtype=np.float64)
        if b.shape != (Y.shape[0],):
            raise ValueError("bias must be [M]")
        Y = Y + b[:, None]
    if y_dtype == "bf16":
        Y = round_to_bf16(Y)
    elif y_dtype != "f32":
        raise ValueError("y_dtype")
    if y_layout == "token_major":
        out = np.empty((Y.shape[1], Y.shape[0]), dtype=np.float64)
        for b in range(Y.shape[1]):
            out[b, :] = Y[:, b]
        return out
    if y_layout != "feature_major":
        raise ValueError("y_layout")
    return Y


def op_counts(U, V) -> dict:
    """Per-token operation counts of supplement Table S1 for given U, V."""
    U = np.asarray(U)
    V = np.asarray(V)
    M, K = U.shape
    N = V.shape[1]
    nnz_u = int(np.count_nonzero(U))
    nnz_v = int(np.count_nonzero(V))
    return {"mults": K, "adds": nnz_u + nnz_v, "adds_U": nnz_u, "adds_V": nnz_v,
            "r": (nnz_u + nnz_v) / float(K * (M + N))}


def acceleration(M: int, N: int, K: int, r: float, d: int) -> float:
    """Cost of W(.) over cost of U diag(S) V(.) in equivalent additions (Table S2)."""
    return M * N * (d - 1) / (K * (d - 2) + r * K * (M + N))


def critical_rank(M: int, N: int, r: float, d: int) -> float:
    """Eq. (2): the rank where TSVD and the dense map cost the same."""
    return (d - 1) * M * N / (d + r * (M + N) - 2)
