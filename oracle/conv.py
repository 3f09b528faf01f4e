"""CPU oracle for the convolution forms of the ternary SVD (TEST INFRASTRUCTURE ONLY).

Section "TSVD in Convolution Layer": the kernel [C_out, C_in, K1, K2] of a convolution is reshaped
into one of four matrices (Eq. (four_shape)),

    form 0: [C_out,           C_in * K1 * K2]      V is a K1 x K2 convolution, U a 1 x 1 convolution
    form 1: [C_out * K1 * K2, C_in          ]      V 1 x 1, U K1 x K2
    form 2: [C_out * K1,      C_in * K2     ]      V 1 x K2, U K1 x 1
    form 3: [C_out * K2,      C_in * K1     ]      V K1 x 1, U 1 x K2

and that matrix is written U diag(S) V.  For a grouped convolution (the paper's converted ConvNeXt
lists its depth-wise 7 x 7 layers as form 0 with groups = channels and rank 5) every group g has its
own factors: the rows of U belonging to the output channels of g, a block of K / groups ranks, and
the rows of V for those ranks, V_g being [K / groups, (C_in / groups) * K1 * K2].  The oracle does not run the two small convolutions: it
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


def dense_kernel_grouped(U, S, V, groups: int, c_out: int, c_in: int, k1: int, k2: int) -> np.ndarray:
    """Form 0 with groups: the kernel [C_out, C_in / groups, K1, K2] whose block for group g is
    U[rows of g, ranks of g] diag(S[ranks of g]) V[ranks of g, :].  U is [C_out, K], V is
    [K, (C_in / groups) * K1 * K2], ranks of g = [g K / groups, (g + 1) K / groups); entries of U
    outside the rank block of its row's group take no part."""
    U = np.asarray(U, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    S = np.asarray(S, dtype=np.float64)
    K = S.shape[0]
    if c_out % groups or c_in % groups or K % groups:
        raise ValueError("groups must divide C_out, C_in and the rank")
    mg, cg, kg = c_out // groups, c_in // groups, K // groups
    W4 = np.zeros((c_out, cg, k1, k2))
    for g in range(groups):
        rows, ranks = slice(g * mg, (g + 1) * mg), slice(g * kg, (g + 1) * kg)
        W4[rows] = ((U[rows, ranks] * S[None, ranks]) @ V[ranks, :]).reshape(mg, cg, k1, k2)
    return W4


def out_size(size: int, k: int, stride: int, pad: int, dil: int) -> int:
    return (size + 2 * pad - dil * (k - 1) - 1) // stride + 1


def conv2d(x, W4, stride=(1, 1), pad=(0, 0), dil=(1, 1), bias=None, groups: int = 1) -> np.ndarray:
    """y[b, co, oy, ox] = bias[co] + sum_{ci, dy, dx} W4[co, ci, dy, dx] x[b, ci, oy s1 + dy d1 - p1, ox s2 + dx d2 - p2]
    with x zero outside its borders; x is [B, C_in, H, W], the result [B, C_out, Ho, Wo], all fp64.
    With groups > 1, W4 is [C_out, C_in / groups, K1, K2] and output channel co of group
    g = co // (C_out / groups) sees only the input channels g C_in / groups + ci."""
    x = np.asarray(x, dtype=np.float64)
    W4 = np.asarray(W4, dtype=np.float64)
    if groups > 1:
        c_out, cg = W4.shape[0], W4.shape[1]
        if c_out % groups or x.shape[1] != cg * groups:
            raise ValueError("channel mismatch")
        mg = c_out // groups
        parts = [conv2d(x[:, g * cg:(g + 1) * cg], W4[g * mg:(g + 1) * mg], stride, pad, dil, None) for g in range(groups)]
        y = np.concatenate(parts, axis=1)
        if bias is not None:
            y += np.asarray(bias, dtype=np.float64)[None, :, None, None]
        return y
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
                bias=None, groups: int = 1) -> np.ndarray:
    """The convolution whose kernel is given in ternary-SVD form (groups > 1: form 0 only)."""
    if groups > 1:
        if form != 0:
            raise ValueError("grouped convolutions are defined for form 0 only")
        return conv2d(x, dense_kernel_grouped(U, S, V, groups, c_out, c_in, k1, k2), stride, pad, dil, bias, groups)
    return conv2d(x, dense_kernel(U, S, V, form, c_out, c_in, k1, k2), stride, pad, dil, bias)
