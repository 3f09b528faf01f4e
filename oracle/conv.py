"""CPU oracle for the convolution forms of the ternary SVD (TEST INFRASTRUCTURE ONLY).

Section "TSVD in Convolution Layer": the kernel [C_out, C_in, K1, K2] of a convolution is reshaped
into one of four matrices (Eq. (four_shape)),

    form 0: [C_out,           C_in * K1 * K2]      V is a K1 x K2 convolution, U a 1 x 1 convolution
    form 1: [C_out * K1 * K2, C_in          ]      V 1 x 1, U K1 x K2
    form 2: [C_out * K1,      C_in * K2     ]      V 1 x K2, U K1 x 1
    form 3: [C_out * K2,      C_in * K1     ]      V K1 x 1, U 1 x K2

and that matrix is written U diag(S) V.  The oracle does not run the two small convolutions: it
rebuilds the dense kernel from (U, S, V) by undoing the reshape and evaluates the plain definition
of a 2-d convolution (cross-correlation, as in the deep-learning libraries the paper uses) in fp64.
Index order inside a reshaped dimension is row-major in the order written above.

Nothing here is imported by the GPU library or its binding.
"""
from __future__ import annotations

import numpy as np


def dense_kernel(U, S, V, form: int, c_out: int, c_in: int, k1: int, k2: int) -> np.ndarray:
    """The kernel [C_out, C_in, K1, K2] whose reshape (Eq. (four_shape)) equals U diag(S) V."""
    Wm = (np.asarray(U, dtype=np.float64) * np.asarray(S, dtype=np.float64)[None, :]) @ np.asarray(V, dtype=np.float64)
    if form == 0:
        return Wm.reshape(c_out, c_in, k1, k2)
    if form == 1:
        return Wm.reshape(c_out, k1, k2, c_in).transpose(0, 3, 1, 2)
    if form == 2:
        return Wm.reshape(c_out, k1, c_in, k2).transpose(0, 2, 1, 3)
    if form == 3:
        return Wm.reshape(c_out, k2, c_in, k1).transpose(0, 2, 3, 1)
    raise ValueError("form must be 0..3")


def out_size(size: int, k: int, stride: int, pad: int, dil: int) -> int:
    return (size + 2 * pad - dil * (k - 1) - 1) // stride + 1


def conv2d(x, W4, stride=(1, 1), pad=(0, 0), dil=(1, 1), bias=None) -> np.ndarray:
    """y[b, co, oy, ox] = bias[co] + sum_{ci, dy, dx} W4[co, ci, dy, dx] x[b, ci, oy s1 + dy d1 - p1, ox s2 + dx d2 - p2]
    with x zero outside its borders; x is [B, C_in, H, W], the result [B, C_out, Ho, Wo], all fp64."""
    x = np.asarray(x, dtype=np.float64)
    W4 = np.asarray(W4, dtype=np.float64)
    B, c_in, H, Wd = x.shape
    c_out, c_in2, k1, k2 = W4.shape
    if c_in2 != c_in:
        raise ValueError("channel mismatch")
    Ho, Wo = out_size(H, k1, stride[0], pad[0], dil[0]), out_size(Wd, k2, stride[1], pad[1], dil[1])
    xp = np.zeros((B, c_in, H + 2 * pad[0], Wd + 2 * pad[1]))
    xp[:, :, pad[0]:pad[0] + H, pad[1]:pad[1] + Wd] = x
    y = np.zeros((B, c_out, Ho, Wo))
    for dy in range(k1):
        for dx in range(k2):
            ys = dy * dil[0]
            xs = dx * dil[1]
            patch = xp[:, :, ys:ys + (Ho - 1) * stride[0] + 1:stride[0], xs:xs + (Wo - 1) * stride[1] + 1:stride[1]]
            y += np.einsum("oc,bchw->bohw", W4[:, :, dy, dx], patch)
    if bias is not None:
        y += np.asarray(bias, dtype=np.float64)[None, :, None, None]
    return y


def tsvd_conv2d(x, U, S, V, form: int, c_out: int, c_in: int, k1: int, k2: int, stride=(1, 1), pad=(0, 0), dil=(1, 1),
                bias=None) -> np.ndarray:
    """The convolution whose kernel is given in ternary-SVD form."""
    return conv2d(x, dense_kernel(U, S, V, form, c_out, c_in, k1, k2), stride, pad, dil, bias)
