"""GPU parity of the convolution forms (section "TSVD in Convolution Layer"), through the C ABI,
against the dense-kernel oracle on the same seeded inputs: exact on integer instances, within the
tolerance of the linear map (2e-3 of max|y| for bf16 activations) on random ones."""
import numpy as np
import pytest

import workloads
from oracle import conv as oc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tsvd():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no fallback")
    import paper_2308_07641_amd as t
    t.load_library()
    return t


def _shapes(form, co, ci, k1, k2):
    rows = {0: co, 1: co * k1 * k2, 2: co * k1, 3: co * k2}[form]
    cols = {0: ci * k1 * k2, 1: ci, 2: ci * k2, 3: ci * k1}[form]
    return rows, cols


def _run(tsvd, U, S, V, form, co, ci, k1, k2, x_nchw_bits, geom, bias, y_dtype):
    import torch
    h = tsvd.tsvd_pack(U, S, V)
    # the library's layout is [C][images][H][W]
    x = torch.from_numpy(np.ascontiguousarray(x_nchw_bits.transpose(1, 0, 2, 3)).view(np.int16)).to("cuda:0").view(torch.bfloat16)
    b = None if bias is None else torch.from_numpy(bias).to("cuda:0")
    y = tsvd.tsvd_conv2d_forward(h, form, ci, co, k1, k2, x, *geom, bias=b, y_dtype=y_dtype)
    torch.cuda.synchronize()
    tsvd.tsvd_free(h)
    return y.float().cpu().numpy().astype(np.float64).transpose(1, 0, 2, 3)      # back to [images][C_out][Ho][Wo]


GEOMS = [((1, 1), (0, 0), (1, 1)), ((2, 1), (1, 2), (1, 1)), ((1, 2), (2, 0), (2, 1)), ((2, 2), (1, 1), (1, 1))]


@pytest.mark.parametrize("form", [0, 1, 2, 3])
@pytest.mark.parametrize("geom", GEOMS)
def test_conv_forms_exact_and_random(tsvd, form, geom):
    import paper_2308_07641_amd as t
    co, ci, k1, k2, K, images, H, W = 20, 12, 3, 3, 40, 3, 11, 13
    rows, cols = _shapes(form, co, ci, k1, k2)
    rng = np.random.default_rng(17 * form + sum(geom[0]) + 3 * sum(geom[1]))
    print(f"case conv form={form} geom={geom}", flush=True)
    # exact: small integers everywhere (sums stay far below 2^24, z fits fp16 exactly)
    U = rng.choice([-1, 0, 1], size=(rows, K), p=[0.15, 0.7, 0.15]).astype(np.int8)
    V = rng.choice([-1, 0, 1], size=(K, cols), p=[0.15, 0.7, 0.15]).astype(np.int8)
    S = rng.integers(-2, 3, size=K).astype(np.float32)
    xi = rng.integers(-2, 3, size=(images, ci, H, W)).astype(np.float32)
    bias = rng.integers(-4, 5, size=co).astype(np.float32)
    ref = oc.tsvd_conv2d(xi, U, S, V, form, co, ci, k1, k2, *geom, bias=bias)
    got = _run(tsvd, U, S, V, form, co, ci, k1, k2, workloads.f32_to_bf16_bits(xi), geom, bias, t.TSVD_F32)
    assert got.shape == ref.shape
    assert np.array_equal(got, ref)
    # random values, bf16 activations, fp32 and bf16 output
    S = (np.abs(rng.standard_normal(K)) * 0.05).astype(np.float32)
    xb = workloads.f32_to_bf16_bits(rng.standard_normal((images, ci, H, W)).astype(np.float32))
    xr = workloads.bf16_bits_to_f32(xb)
    bias = rng.standard_normal(co).astype(np.float32) * 0.1
    ref = oc.tsvd_conv2d(xr, U, S, V, form, co, ci, k1, k2, *geom, bias=bias)
    scale = np.max(np.abs(oc.tsvd_conv2d(xr, U, S, V, form, co, ci, k1, k2, *geom)))
    got = _run(tsvd, U, S, V, form, co, ci, k1, k2, xb, geom, bias, t.TSVD_F32)
    assert np.max(np.abs(got - ref)) <= 2e-3 * scale
    gotb = _run(tsvd, U, S, V, form, co, ci, k1, k2, xb, geom, bias, t.TSVD_BF16)
    assert np.all(np.abs(gotb - ref) <= 2e-3 * scale + 2.0 ** -7 * np.abs(ref))


def test_depthwise_7x7_as_a_block_diagonal_map(tsvd):
    """The paper's converted ConvNeXt keeps its depth-wise 7 x 7 convolutions in form 0 with rank 5 per
    channel; grouped convolution is the same map with block-diagonal factors."""
    import paper_2308_07641_amd as t
    C, k, rank, images, H, W = 8, 7, 5, 2, 14, 14
    rng = np.random.default_rng(77)
    U = np.zeros((C, C * rank), dtype=np.int8)
    V = np.zeros((C * rank, C * k * k), dtype=np.int8)
    for c in range(C):
        U[c, c * rank:(c + 1) * rank] = rng.choice([-1, 1], size=rank)
        V[c * rank:(c + 1) * rank, c * k * k:(c + 1) * k * k] = rng.choice([-1, 0, 1], size=(rank, k * k), p=[0.15, 0.7, 0.15])
    S = (np.abs(rng.standard_normal(C * rank)) * 0.1).astype(np.float32)
    xb = workloads.f32_to_bf16_bits(rng.standard_normal((images, C, H, W)).astype(np.float32))
    xr = workloads.bf16_bits_to_f32(xb)
    geom = ((1, 1), (3, 3), (1, 1))
    ref = oc.tsvd_conv2d(xr, U, S, V, 0, C, C, k, k, *geom)
    # the dense kernel of the block-diagonal factors is depth-wise: no cross-channel taps
    W4 = oc.dense_kernel(U, S, V, 0, C, C, k, k)
    assert all(not W4[o, c].any() for o in range(C) for c in range(C) if o != c)
    got = _run(tsvd, U, S, V, 0, C, C, k, k, xb, geom, None, t.TSVD_F32)
    assert got.shape == (images, C, H, W)
    assert np.max(np.abs(got - ref)) <= 2e-3 * np.max(np.abs(ref))


def test_conv_single_image_odd_sizes_and_1x1(tsvd):
    """Column counts that are not multiples of 8 (the gathered matrix pads its rows), a 1 x 1 kernel
    with stride 2 (every form then degenerates to the same map), one image."""
    import paper_2308_07641_amd as t
    rng = np.random.default_rng(88)
    co, ci, K = 10, 6, 12
    U = rng.choice([-1, 0, 1], size=(co, K)).astype(np.int8)
    V = rng.choice([-1, 0, 1], size=(K, ci)).astype(np.int8)
    S = rng.integers(-2, 3, size=K).astype(np.float32)
    xi = rng.integers(-2, 3, size=(1, ci, 7, 5)).astype(np.float32)
    geom = ((2, 2), (0, 0), (1, 1))
    ref = oc.tsvd_conv2d(xi, U, S, V, 0, co, ci, 1, 1, *geom)
    for form in range(4):
        got = _run(tsvd, U, S, V, form, co, ci, 1, 1, workloads.f32_to_bf16_bits(xi), geom, None, t.TSVD_F32)
        assert np.array_equal(got, ref), form


def test_conv_rejects_mismatched_geometry(tsvd):
    import torch
    rng = np.random.default_rng(1)
    U = rng.integers(-1, 2, size=(6, 4)).astype(np.int8)
    V = rng.integers(-1, 2, size=(4, 18)).astype(np.int8)
    h = tsvd.tsvd_pack(U, np.ones(4, dtype=np.float32), V)
    x = torch.zeros((2, 1, 5, 5), dtype=torch.bfloat16, device="cuda:0")
    with pytest.raises(ValueError):
        tsvd.tsvd_conv2d_forward(h, 1, 2, 6, 3, 3, x)             # form 1 needs a [54, 2] matrix
    with pytest.raises(ValueError):
        tsvd.tsvd_conv2d_forward(h, 0, 2, 6, 3, 3, torch.zeros((2, 1, 2, 2), dtype=torch.bfloat16, device="cuda:0"))   # empty output
    y = tsvd.tsvd_conv2d_forward(h, 0, 2, 6, 3, 3, x)
    assert y.shape == (6, 1, 3, 3)
    tsvd.tsvd_free(h)
