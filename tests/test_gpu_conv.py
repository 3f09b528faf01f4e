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


def _run(tsvd, U, S, V, form, co, ci, k1, k2, x_nchw_bits, geom, bias, y_dtype, groups=1):
    import torch
    h = tsvd.tsvd_pack(U, S, V)
    # the library's layout is [C][images][H][W]
    x = torch.from_numpy(np.ascontiguousarray(x_nchw_bits.transpose(1, 0, 2, 3)).view(np.int16)).to("cuda:0").view(torch.bfloat16)
    b = None if bias is None else torch.from_numpy(bias).to("cuda:0")
    y = tsvd.tsvd_conv2d_forward(h, form, ci, co, k1, k2, x, *geom, bias=b, y_dtype=y_dtype, groups=groups)
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


# groups, input / output channels and ranks per group, kernel, (stride, pad, dil), images, H, W
GROUPED = [
    (12, 1, 1, 5, 7, 7, ((1, 1), (3, 3), (1, 1)), 3, 14, 14),      # the paper's depth-wise 7 x 7, rank 5 per channel
    (6, 1, 1, 5, 7, 7, ((2, 2), (3, 3), (1, 1)), 2, 30, 33),       # several row blocks per plane, ragged last block, stride 2
    (5, 1, 2, 4, 3, 3, ((1, 1), (2, 2), (2, 2)), 2, 9, 11),        # channel multiplier 2, dilation
    (3, 2, 3, 6, 3, 2, ((1, 2), (1, 0), (1, 1)), 2, 10, 12),       # two input channels per group, three outputs (4-wide variant)
    (2, 1, 8, 64, 7, 7, ((1, 1), (3, 3), (1, 1)), 1, 8, 8),        # the limits: 8 outputs and 64 ranks per group
    (4, 1, 1, 5, 7, 7, ((1, 1), (3, 3), (1, 1)), 23, 7, 7),        # tiny planes: several images per workgroup, ragged
    (2, 1, 1, 3, 1, 5, ((1, 1), (0, 2), (1, 1)), 1, 3, 300),       # rows wider than a workgroup
]


@pytest.mark.parametrize("case", GROUPED, ids=[f"g{c[0]}_cg{c[1]}_mg{c[2]}_kg{c[3]}_{c[4]}x{c[5]}_{c[8]}x{c[9]}" for c in GROUPED])
def test_grouped_conv_exact_and_random(tsvd, case):
    """Form 0 with groups through the direct kernel: exact on integer instances; on random bf16
    activations within 1e-5 of max|y| (everything after the bf16 input is fp32 arithmetic on at most a
    few thousand terms), far inside the 2e-3 bar of the linear map."""
    import paper_2308_07641_amd as t
    G, cg, mg, kg, k1, k2, geom, images, H, W = case
    ci, co, K, ng = G * cg, G * mg, G * kg, cg * k1 * k2
    rng = np.random.default_rng(1000 + G + 7 * kg + H)
    print(f"case grouped {case}", flush=True)
    U = rng.choice([-1, 0, 1], size=(co, K), p=[0.3, 0.4, 0.3]).astype(np.int8)       # off-block entries are not read
    V = rng.choice([-1, 0, 1], size=(K, ng), p=[0.15, 0.7, 0.15]).astype(np.int8)
    V[0] = 0                                                                           # a rank with no tap at all
    S = rng.integers(-2, 3, size=K).astype(np.float32)
    xi = rng.integers(-2, 3, size=(images, ci, H, W)).astype(np.float32)
    bias = rng.integers(-4, 5, size=co).astype(np.float32)
    ref = oc.tsvd_conv2d(xi, U, S, V, 0, co, ci, k1, k2, *geom, bias=bias, groups=G)
    got = _run(tsvd, U, S, V, 0, co, ci, k1, k2, workloads.f32_to_bf16_bits(xi), geom, bias, t.TSVD_F32, G)
    assert got.shape == ref.shape
    assert np.array_equal(got, ref)
    S = (np.abs(rng.standard_normal(K)) * 0.1).astype(np.float32)
    xb = workloads.f32_to_bf16_bits(rng.standard_normal((images, ci, H, W)).astype(np.float32))
    xr = workloads.bf16_bits_to_f32(xb)
    bias = (rng.standard_normal(co) * 0.1).astype(np.float32)
    ref = oc.tsvd_conv2d(xr, U, S, V, 0, co, ci, k1, k2, *geom, bias=bias, groups=G)
    scale = np.max(np.abs(ref))
    got = _run(tsvd, U, S, V, 0, co, ci, k1, k2, xb, geom, bias, t.TSVD_F32, G)
    assert np.max(np.abs(got - ref)) <= 1e-5 * scale
    gotb = _run(tsvd, U, S, V, 0, co, ci, k1, k2, xb, geom, bias, t.TSVD_BF16, G)
    assert np.all(np.abs(gotb - ref) <= 1e-5 * scale + 2.0 ** -8 * np.abs(ref))
    # the same layer as an ungrouped form 0 with block-diagonal factors (the generic path)
    if G * kg <= 64:
        Ubd = np.zeros_like(U)
        Vbd = np.zeros((K, ci * k1 * k2), dtype=np.int8)
        for g in range(G):
            Ubd[g * mg:(g + 1) * mg, g * kg:(g + 1) * kg] = U[g * mg:(g + 1) * mg, g * kg:(g + 1) * kg]
            Vbd[g * kg:(g + 1) * kg, g * ng:(g + 1) * ng] = V[g * kg:(g + 1) * kg]
        gen = _run(tsvd, Ubd, S, Vbd, 0, co, ci, k1, k2, xb, geom, bias, t.TSVD_F32)
        assert np.max(np.abs(gen - got)) <= 2e-3 * scale


def test_grouped_conv_limits_and_errors(tsvd):
    import torch
    rng = np.random.default_rng(3)
    x = torch.zeros((4, 1, 9, 9), dtype=torch.bfloat16, device="cuda:0")
    U = rng.integers(-1, 2, size=(4, 8)).astype(np.int8)
    V = rng.integers(-1, 2, size=(8, 9)).astype(np.int8)
    h = tsvd.tsvd_pack(U, np.ones(8, dtype=np.float32), V)
    assert tsvd.tsvd_conv2d_forward(h, 0, 4, 4, 3, 3, x, pad=(1, 1), groups=4).shape == (4, 1, 9, 9)
    with pytest.raises(ValueError):
        tsvd.tsvd_conv2d_forward(h, 1, 4, 4, 3, 3, x, groups=4)          # grouped: form 0 only
    with pytest.raises(ValueError):
        tsvd.tsvd_conv2d_forward(h, 0, 4, 4, 3, 3, x, groups=3)          # groups must divide the channels
    with pytest.raises(ValueError):
        tsvd.tsvd_conv2d_forward(h, 0, 4, 4, 3, 3, x, groups=2)          # V would need 2 * 9 columns
    tsvd.tsvd_free(h)
    U = rng.integers(-1, 2, size=(18, 4)).astype(np.int8)               # 9 output channels per group: beyond the limit
    h = tsvd.tsvd_pack(U, np.ones(4, dtype=np.float32), rng.integers(-1, 2, size=(4, 9)).astype(np.int8))
    with pytest.raises(ValueError):
        tsvd.tsvd_conv2d_forward(h, 0, 2, 18, 3, 3, torch.zeros((2, 1, 9, 9), dtype=torch.bfloat16, device="cuda:0"), groups=2)
    tsvd.tsvd_free(h)


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
