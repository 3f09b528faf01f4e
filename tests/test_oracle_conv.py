"""Pins for the convolution oracle: the direct definition by explicit loops on tiny cases, a library
convolution routine, the paper's own worked example F(2, 3), and the two-small-convolutions reading
of each form (V as a convolution, channel-wise S, U as a convolution) evaluated independently."""
import numpy as np
import pytest
import torch

from oracle import conv as oc


def _loops(x, W4, stride, pad, dil, bias=None):
    B, ci, H, W = x.shape
    co, _, k1, k2 = W4.shape
    Ho, Wo = oc.out_size(H, k1, stride[0], pad[0], dil[0]), oc.out_size(W, k2, stride[1], pad[1], dil[1])
    y = np.zeros((B, co, Ho, Wo))
    for b in range(B):
        for o in range(co):
            for oy in range(Ho):
                for ox in range(Wo):
                    acc = 0.0 if bias is None else float(bias[o])
                    for c in range(ci):
                        for dy in range(k1):
                            for dx in range(k2):
                                iy, ix = oy * stride[0] + dy * dil[0] - pad[0], ox * stride[1] + dx * dil[1] - pad[1]
                                if 0 <= iy < H and 0 <= ix < W:
                                    acc += W4[o, c, dy, dx] * x[b, c, iy, ix]
                    y[b, o, oy, ox] = acc
    return y


GEOMS = [((1, 1), (0, 0), (1, 1)), ((2, 1), (1, 2), (1, 1)), ((1, 2), (2, 0), (2, 1)), ((3, 2), (1, 1), (1, 2))]


@pytest.mark.parametrize("stride,pad,dil", GEOMS)
def test_direct_definition_against_loops_and_library(stride, pad, dil):
    rng = np.random.default_rng(sum(stride) + 10 * sum(pad) + 100 * sum(dil))
    x = rng.standard_normal((2, 3, 7, 9))
    W4 = rng.standard_normal((4, 3, 3, 2))
    bias = rng.standard_normal(4)
    got = oc.conv2d(x, W4, stride, pad, dil, bias)
    assert np.allclose(got, _loops(x, W4, stride, pad, dil, bias), atol=1e-12)
    lib = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(W4), torch.from_numpy(bias), stride, pad, dil)
    assert np.allclose(got, lib.numpy(), atol=1e-12)


def test_winograd_f23_row_of_the_paper():
    """The paper's unfolded 1-d example: y1 = w1 x1 + w2 x2 + w3 x3, y2 = w1 x2 + w2 x3 + w3 x4."""
    w = np.array([0.5, -1.25, 2.0])
    x = np.array([1.0, 2.0, -3.0, 4.0])
    y = oc.conv2d(x.reshape(1, 1, 1, 4), w.reshape(1, 1, 1, 3))
    assert np.allclose(y.ravel(), [w @ x[0:3], w @ x[1:4]])


def _two_convolutions(x, U, S, V, form, co, ci, k1, k2, stride, pad, dil):
    """Section "TSVD in Convolution Layer": V(.) as a convolution with kernel_V, the channel-wise
    product with S, U(.) as a convolution with kernel_U; each with a library routine."""
    K = S.shape[0]
    kv = {0: (k1, k2), 1: (1, 1), 2: (1, k2), 3: (k1, 1)}[form]
    ku = {0: (1, 1), 1: (k1, k2), 2: (k1, 1), 3: (1, k2)}[form]
    Vf, Uf = V.astype(np.float64), U.astype(np.float64)
    if form == 0:
        Wv, Wu = Vf.reshape(K, ci, k1, k2), Uf.reshape(co, K, 1, 1)
    elif form == 1:
        Wv, Wu = Vf.reshape(K, ci, 1, 1), Uf.reshape(co, k1, k2, K).transpose(0, 3, 1, 2)
    elif form == 2:
        Wv, Wu = Vf.reshape(K, ci, 1, k2), Uf.reshape(co, k1, K)[:, :, :, None].transpose(0, 2, 1, 3)
    else:
        Wv, Wu = Vf.reshape(K, ci, k1, 1), Uf.reshape(co, k2, K)[:, :, :, None].transpose(0, 2, 3, 1)
    # each spatial dimension is handled (kernel, stride, padding, dilation) by exactly one of the two
    vdim = tuple((form in (0, 3)) if d == 0 else (form in (0, 2)) for d in range(2))
    sv = tuple(stride[d] if vdim[d] else 1 for d in range(2))
    pv = tuple(pad[d] if vdim[d] else 0 for d in range(2))
    dv = tuple(dil[d] if vdim[d] else 1 for d in range(2))
    su = tuple(1 if vdim[d] else stride[d] for d in range(2))
    pu = tuple(0 if vdim[d] else pad[d] for d in range(2))
    du = tuple(1 if vdim[d] else dil[d] for d in range(2))
    t = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(np.ascontiguousarray(Wv)), None, sv, pv, dv)
    z = t * torch.from_numpy(S.astype(np.float64))[None, :, None, None]
    return torch.nn.functional.conv2d(z, torch.from_numpy(np.ascontiguousarray(Wu)), None, su, pu, du).numpy()


@pytest.mark.parametrize("form", [0, 1, 2, 3])
@pytest.mark.parametrize("stride,pad,dil", GEOMS)
def test_forms_equal_two_small_convolutions(form, stride, pad, dil):
    rng = np.random.default_rng(form + 7 * sum(stride) + 31 * sum(pad))
    co, ci, k1, k2, K = 5, 4, 3, 2, 6
    rows = {0: co, 1: co * k1 * k2, 2: co * k1, 3: co * k2}[form]
    cols = {0: ci * k1 * k2, 1: ci, 2: ci * k2, 3: ci * k1}[form]
    U = rng.integers(-1, 2, size=(rows, K)).astype(np.int8)
    V = rng.integers(-1, 2, size=(K, cols)).astype(np.int8)
    S = rng.standard_normal(K).astype(np.float32)
    x = rng.standard_normal((2, ci, 8, 9))
    got = oc.tsvd_conv2d(x, U, S, V, form, co, ci, k1, k2, stride, pad, dil)
    want = _two_convolutions(x, U, S, V, form, co, ci, k1, k2, stride, pad, dil)
    assert got.shape == want.shape
    assert np.allclose(got, want, atol=1e-10)
    # the reshape of the dense kernel gives back U diag(S) V
    W4 = oc.dense_kernel(U, S, V, form, co, ci, k1, k2)
    Wm = (U * S.astype(np.float64)[None, :]) @ V.astype(np.float64)
    back = {0: W4.reshape(co, -1), 1: W4.transpose(0, 2, 3, 1).reshape(co * k1 * k2, ci),
            2: W4.transpose(0, 2, 1, 3).reshape(co * k1, ci * k2), 3: W4.transpose(0, 3, 1, 2).reshape(co * k2, ci * k1)}[form]
    assert np.array_equal(back, Wm)


# ---- grouped / depth-wise convolutions (form 0 with groups, as the paper's converted ConvNeXt lists them)
@pytest.mark.parametrize("groups,cg,mg", [(4, 1, 1), (4, 1, 2), (3, 2, 2), (2, 3, 1)])
@pytest.mark.parametrize("stride,pad,dil", GEOMS)
def test_grouped_definition_against_library_and_block_diagonal(groups, cg, mg, stride, pad, dil):
    rng = np.random.default_rng(groups + 5 * cg + 11 * mg + sum(stride) + 3 * sum(pad))
    ci, co = groups * cg, groups * mg
    x = rng.standard_normal((2, ci, 8, 9))
    W4 = rng.standard_normal((co, cg, 3, 2))
    bias = rng.standard_normal(co)
    got = oc.conv2d(x, W4, stride, pad, dil, bias, groups)
    lib = torch.nn.functional.conv2d(torch.from_numpy(x), torch.from_numpy(W4), torch.from_numpy(bias), stride, pad, dil, groups)
    assert np.allclose(got, lib.numpy(), atol=1e-12)
    # a grouped convolution is an ordinary one whose kernel is zero across groups (explicit loops)
    full = np.zeros((co, ci, 3, 2))
    for o in range(co):
        g = o // mg
        full[o, g * cg:(g + 1) * cg] = W4[o]
    assert np.allclose(got, _loops(x, full, stride, pad, dil, bias), atol=1e-12)


def test_grouped_factors_equal_block_diagonal_factors():
    """Per-group factors (U rows of the group x its rank block, V_g stacked) give the same kernel as
    the ungrouped form 0 with block-diagonal U and V; and each group alone is form 0 of its block."""
    rng = np.random.default_rng(5)
    groups, cg, mg, kg, k1, k2 = 3, 2, 2, 4, 3, 3
    co, ci, K, ng = groups * mg, groups * cg, groups * kg, cg * k1 * k2
    U = np.zeros((co, K), dtype=np.int8)
    Vs = rng.integers(-1, 2, size=(K, ng)).astype(np.int8)
    Vbd = np.zeros((K, ci * k1 * k2), dtype=np.int8)
    for g in range(groups):
        U[g * mg:(g + 1) * mg, g * kg:(g + 1) * kg] = rng.integers(-1, 2, size=(mg, kg))
        Vbd[g * kg:(g + 1) * kg, g * ng:(g + 1) * ng] = Vs[g * kg:(g + 1) * kg]
    S = rng.standard_normal(K).astype(np.float32)
    W4g = oc.dense_kernel_grouped(U, S, Vs, groups, co, ci, k1, k2)
    W4f = oc.dense_kernel(U, S, Vbd, 0, co, ci, k1, k2)
    for o in range(co):
        g = o // mg
        assert np.array_equal(W4f[o, g * cg:(g + 1) * cg], W4g[o])
        W4f[o, g * cg:(g + 1) * cg] = 0
    assert not W4f.any()
    g = 1
    alone = oc.dense_kernel(U[g * mg:(g + 1) * mg, g * kg:(g + 1) * kg], S[g * kg:(g + 1) * kg], Vs[g * kg:(g + 1) * kg], 0, mg, cg, k1, k2)
    assert np.array_equal(alone, W4g[g * mg:(g + 1) * mg])
    # entries of U outside the rank block of the row's group take no part
    U2 = U.copy()
    U2[0, kg:] = 1
    assert np.array_equal(oc.dense_kernel_grouped(U2, S, Vs, groups, co, ci, k1, k2), W4g)
    x = rng.standard_normal((2, ci, 6, 7))
    a = oc.tsvd_conv2d(x, U, S, Vs, 0, co, ci, k1, k2, (1, 1), (1, 1), (1, 1), None, groups)
    b = oc.tsvd_conv2d(x, U, S, Vbd, 0, co, ci, k1, k2, (1, 1), (1, 1), (1, 1))
    assert np.allclose(a, b, atol=1e-12)


def test_depthwise_identity_tap():
    """Depth-wise 7 x 7 whose only tap is the centre with weight s_c: y = s_c x (same padding)."""
    rng = np.random.default_rng(6)
    C, k = 5, 7
    U = np.eye(C, dtype=np.int8)                       # rank 1 per channel
    V = np.zeros((C, k * k), dtype=np.int8)
    V[:, (k // 2) * k + k // 2] = -1
    S = rng.standard_normal(C).astype(np.float32)
    x = rng.standard_normal((2, C, 9, 8))
    y = oc.tsvd_conv2d(x, U, S, V, 0, C, C, k, k, (1, 1), (3, 3), (1, 1), None, C)
    assert np.allclose(y, -S.astype(np.float64)[None, :, None, None] * x, atol=1e-13)
