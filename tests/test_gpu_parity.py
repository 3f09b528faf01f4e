"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Tolerances (max|y_gpu - y_ref| / max|y_ref| over the whole output):
2e-3 for bf16 activations, 1e-5 for fp32 activations; integer instances must match exactly."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import rel_err, run_forward, to_device

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-3, "f32": 1e-5}


@pytest.fixture(scope="module")
def tsvd():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU: the HIP path has no fallback")
    import paper_2308_07641_amd as t
    t.load_library()
    return t


# ---- exact-integer instances: every partial sum is exact in fp32, so any correct kernel
# ---- agrees with the oracle bit for bit (catches tile, padding and index mistakes).
INT_SHAPES = [
    # M, N, K, B
    (16, 256, 16, 1), (1, 1, 1, 1), (3, 5, 7, 1), (37, 29, 61, 1), (256, 256, 512, 1),
    (300, 513, 270, 1), (64, 48, 200, 3), (64, 48, 200, 5), (33, 300, 257, 8), (50, 70, 90, 16),
    (20, 40, 30, 17), (100, 260, 300, 40),
    (128, 128, 128, 64), (256, 256, 256, 128), (300, 200, 270, 100), (130, 64, 520, 257),
    (512, 256, 384, 256), (260, 100, 300, 1000),
]


@pytest.mark.parametrize("x_dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,N,K,B", INT_SHAPES)
def test_integer_instances_match_bit_for_bit(tsvd, M, N, K, B, x_dtype):
    i = workloads.make_integer_inputs(M, N, K, B, 0.5, x_dtype, seed=M + 3 * N + 7 * K + 11 * B)
    print(f"case int M={M} N={N} K={K} B={B} {x_dtype}", flush=True)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any(), "an output element was not written"
    assert np.array_equal(y, ref)


# ---- random instances within tolerance, ragged shapes spanning several tiles
RAND_SHAPES = [
    (256, 256, 512, 1, 0.5), (1000, 300, 777, 1, 0.6), (2048, 1024, 1536, 1, 0.7),
    (530, 270, 1030, 2, 0.5), (530, 270, 1030, 5, 0.5), (530, 270, 1030, 16, 0.5), (515, 100, 300, 33, 0.6),
    (384, 256, 512, 64, 0.5), (515, 300, 777, 130, 0.6), (1024, 512, 768, 512, 0.5), (300, 2000, 260, 1025, 0.6),
]


@pytest.mark.parametrize("x_dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,N,K,B,p0", RAND_SHAPES)
def test_random_instances_within_tolerance(tsvd, M, N, K, B, p0, x_dtype):
    i = workloads.make_inputs(M, N, K, B, p0, 0.02, x_dtype, seed=99 + M + N + K + B)
    print(f"case rand M={M} N={N} K={K} B={B} {x_dtype}", flush=True)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert rel_err(y, ref) <= TOL[x_dtype]


# ---- every tile shape of the batched kernels on the same ragged instance.  The tuning switches
# ---- (include/tsvd_tuning.h) are looked up per call; normally the shape follows from the problem size, so the
# ---- small test instances above would never reach the large-tile kernels.
TILE_SHAPES = [0, 1, 2, 3, 14, 15, 16]


@pytest.mark.parametrize("fuse", ["1", "0"])
@pytest.mark.parametrize("cfg", TILE_SHAPES)
def test_every_tile_shape_batched(tsvd, cfg, fuse):
    tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_V", cfg)
    tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_U", cfg)
    tsvd.tsvd_tuning_set("TSVD_FUSEMAX", int(fuse))
    print(f"case tile shape {cfg} fuse {fuse}", flush=True)
    i = workloads.make_integer_inputs(300, 200, 520, 300, 0.5, "bf16", seed=4242 + cfg)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert np.array_equal(y, ref)
    j = workloads.make_inputs(515, 300, 777, 600, 0.6, 0.02, "bf16", seed=777 + cfg)
    ref = oracle.forward(j.U, j.S, j.V, j.X)
    y, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert rel_err(y, ref) <= TOL["bf16"]


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_unaligned_rows_gather_kernels(tsvd, cfg):
    """Rows of x that are not 16-byte aligned are copied to aligned rows before the batched kernels;
    with that copy switched off the large-tile kernels gather them element by element."""
    tsvd.tsvd_tuning_set("TSVD_REALIGN", 0)
    tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_V", cfg)
    tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_U", cfg)
    print(f"case gather tile shape {cfg}", flush=True)
    i = workloads.make_integer_inputs(300, 200, 520, 301, 0.5, "bf16", seed=4343 + cfg)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    j = workloads.make_inputs(515, 300, 777, 603, 0.6, 0.02, "bf16", seed=787 + cfg)
    y, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert rel_err(y, oracle.forward(j.U, j.S, j.V, j.X)) <= TOL["bf16"]


@pytest.mark.parametrize("fuse", ["1", "0"])
def test_tile_shape_of_96_rows(tsvd, fuse):
    """The 96 x 64 ring tiles need padded row counts that 96 divides (the shape rule asks for them
    only then): forced here on both stages of instances with 768 and 1536 padded rows."""
    tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_V", 17)
    tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_U", 17)
    tsvd.tsvd_tuning_set("TSVD_FUSEMAX", int(fuse))
    tsvd.tsvd_tuning_set("TSVD_PANEL", 0)
    print(f"case tile shape 17 fuse {fuse}", flush=True)
    i = workloads.make_integer_inputs(700, 200, 760, 300, 0.5, "bf16", seed=1717)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    j = workloads.make_inputs(1500, 300, 1300, 600, 0.6, 0.02, "bf16", seed=1718)
    ref = oracle.forward(j.U, j.S, j.V, j.X)
    y, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert rel_err(y, ref) <= TOL["bf16"]


@pytest.mark.parametrize("waves", ["fp6", "16", "8"])
@pytest.mark.parametrize("M,N,K,B", [(300, 200, 520, 300), (64, 48, 200, 17), (1030, 100, 1000, 70), (2048, 512, 1024, 1000),
                                     (260, 1024, 1024, 129), (129, 1000, 130, 64)])
def test_token_panel_kernel(tsvd, M, N, K, B, waves):
    """Both stages in one launch with z kept in LDS (K <= 1024), forced on small instances: exact
    integers bit for bit, random values within tolerance, and next to identical to the two-launch path.
    "fp6": the kernel on fp4 codes x fp6 planes; "16" / "8": the 16-bit kernel with that many wavefronts."""
    print(f"case panel M={M} N={N} K={K} B={B} {waves}", flush=True)
    i = workloads.make_integer_inputs(M, N, K, B, 0.5, "bf16", seed=5150 + B)
    tsvd.tsvd_tuning_set("TSVD_PANEL", 1)
    tsvd.tsvd_tuning_set("TSVD_PANEL_FP6", int(waves == "fp6"))
    if waves != "fp6":
        tsvd.tsvd_tuning_set("TSVD_PANEL_WAVES", int(waves))
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    j = workloads.make_inputs(M, N, K, B, 0.6, 0.02, "bf16", seed=5151 + B)
    ref = oracle.forward(j.U, j.S, j.V, j.X)
    y1, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert not np.isnan(y1).any()
    assert rel_err(y1, ref) <= TOL["bf16"]
    tsvd.tsvd_tuning_set("TSVD_PANEL", 0)
    y0, h = run_forward(j)
    tsvd.tsvd_free(h)
    # same products; only the fp32 summation order differs between the 16-bit kernels (a different order in
    # stage V can move an fp16 rounding of z by one unit in the last place); the planes round z differently
    assert rel_err(y0, y1) <= (5e-4 if waves == "fp6" else 1e-5)


def test_larger_small_problem_uses_wider_ring_tiles(tsvd):
    """2048 x 1024 outputs per stage: enough 128 x 64 tiles for every compute unit."""
    i = workloads.make_inputs(2048, 512, 2048, 1024, 0.6, 0.02, "bf16", seed=31337)
    print("case rand M=2048 N=512 K=2048 B=1024 bf16", flush=True)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert rel_err(y, ref) <= TOL["bf16"]


# ---- few-token kernel (2 <= B <= 16, bf16): contraction lengths of several LDS slabs with a ragged
# ---- last one, every contraction split, aligned rows (vector loads) and unaligned rows (gather)
# ---- (contractions of at most two slabs normally stay resident in LDS; "0" sends them through the hand-over loop too)
@pytest.mark.parametrize("resident", ["1", "0"])
@pytest.mark.parametrize("kwlog2", ["0", "1", "2", "3"])
@pytest.mark.parametrize("M,N,K,B", [(100, 2300, 4500, 16), (530, 270, 5000, 8), (70, 6000, 300, 7), (200, 4100, 2049, 2)])
def test_few_token_kernel(tsvd, M, N, K, B, kwlog2, resident):
    import torch
    tsvd.tsvd_tuning_set("TSVD_MID_RESIDENT", int(resident))
    tsvd.tsvd_tuning_set("TSVD_MID_KWLOG2", int(kwlog2))
    tsvd.tsvd_tuning_set("TSVD_MID_SW", 2)
    i = workloads.make_integer_inputs(M, N, K, B, 0.5, "bf16", seed=31 + M + B)
    print(f"case few-token int M={M} N={N} K={K} B={B} kw=2^{kwlog2}", flush=True)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    i = workloads.make_inputs(M, N, K, B, 0.6, 0.02, "bf16", seed=32 + M + B)
    print(f"case few-token rand M={M} N={N} K={K} B={B} kw=2^{kwlog2}", flush=True)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    assert not np.isnan(y).any()
    assert rel_err(y, ref) <= TOL["bf16"]
    # the same tokens as columns of a wider, 16-byte-aligned matrix (vector loads, neighbours in the padding lanes)
    xfull = torch.randn((N, 24), dtype=torch.float32, device="cuda:0").to(torch.bfloat16)
    xfull[:, :B] = to_device(i)
    y2 = tsvd.tsvd_forward(h, xfull[:, :B]).cpu().numpy().astype(np.float64)
    assert np.array_equal(y2, y)
    # and against the one-token-at-a-time path
    tsvd.tsvd_tuning_set("TSVD_MID", 0)
    y3 = tsvd.tsvd_forward(h, to_device(i)).cpu().numpy().astype(np.float64)
    tsvd.tsvd_free(h)
    assert rel_err(y3, ref) <= 1e-5 and rel_err(y, y3) <= TOL["bf16"]


@pytest.mark.parametrize("B,ld,col0", [(3, 10, 0), (5, 10, 2), (4, 9, 0), (6, 12, 1), (2, 2, 0), (7, 20, 4)])
def test_few_token_gather_layouts(tsvd, B, ld, col0):
    """Rows that are not 16-byte aligned are gathered: two tokens per 4-byte load when rows start on
    4-byte boundaries (even stride, even first column), one by one otherwise.  The tokens are columns
    col0 .. col0 + B - 1 of a wider matrix whose other columns hold large values that must not leak in."""
    import torch
    M, N, K = 90, 2500, 700
    i = workloads.make_integer_inputs(M, N, K, B, 0.5, "bf16", seed=77 + B + ld)
    print(f"case few-token gather B={B} ld={ld} col0={col0}", flush=True)
    xfull = torch.full((N, ld), 300.0, dtype=torch.bfloat16, device="cuda:0")
    xfull[:, col0:col0 + B] = to_device(i)
    h = tsvd.tsvd_pack(i.U, i.S, i.V)
    y = tsvd.tsvd_forward(h, xfull[:, col0:col0 + B]).cpu().numpy().astype(np.float64)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))


@pytest.mark.parametrize("K", [4096, 4097])
def test_few_token_kernel_at_the_resident_limit(tsvd, K):
    """A contraction of exactly two LDS slabs stays resident; one index more takes the hand-over loop."""
    i = workloads.make_integer_inputs(48, 4096 if K == 4096 else 4100, K, 11, 0.5, "bf16", seed=K)
    print(f"case few-token resident limit K={K}", flush=True)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))


@pytest.mark.parametrize("B", [17, 40, 64])
def test_few_token_kernel_in_groups(tsvd, B):
    """Up to 64 tokens go through the few-token kernel in groups of 16 when the weights are large;
    forced here on a small instance (exact, then random against the oracle and the batched path)."""
    tsvd.tsvd_tuning_set("TSVD_MID_MAX_B", 64)
    i = workloads.make_integer_inputs(150, 300, 2100, B, 0.5, "bf16", seed=41 + B)
    print(f"case few-token groups int B={B}", flush=True)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    i = workloads.make_inputs(150, 300, 2100, B, 0.6, 0.02, "bf16", seed=42 + B)
    print(f"case few-token groups rand B={B}", flush=True)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    assert not np.isnan(y).any()
    assert rel_err(y, ref) <= TOL["bf16"]
    tsvd.tsvd_tuning_set("TSVD_MID_MAX_B", 16)
    y2 = tsvd.tsvd_forward(h, to_device(i)).cpu().numpy().astype(np.float64)
    tsvd.tsvd_free(h)
    assert rel_err(y2, ref) <= TOL["bf16"] and rel_err(y, y2) <= 1e-5    # same arithmetic, other summation order


def test_activation_scale_extremes_few_tokens(tsvd):
    """Per-token scaling of the fp16 intermediate in the few-token kernel."""
    i = workloads.make_inputs(256, 256, 256, 16, 0.5, 0.02, "bf16", seed=78)
    scale = np.ldexp(1.0, np.random.default_rng(2).integers(-60, 60, size=16)).astype(np.float32)
    i.X = i.X * scale[None, :]
    i.X_bits = workloads.f32_to_bf16_bits(i.X)
    i.X = workloads.bf16_bits_to_f32(i.X_bits)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    per_token = np.max(np.abs(y - ref), axis=0) / np.max(np.abs(ref), axis=0)
    assert np.all(per_token <= 2e-3)


def test_activation_scale_extremes_batched(tsvd):
    """The fp16 intermediate of the batched path is rescaled per token: tokens of very different
    magnitude in one batch must all keep their accuracy (error measured per token here)."""
    i = workloads.make_inputs(256, 256, 256, 128, 0.5, 0.02, "bf16", seed=77)
    scale = np.ldexp(1.0, np.random.default_rng(1).integers(-60, 60, size=128)).astype(np.float32)
    i.X = i.X * scale[None, :]
    i.X_bits = workloads.f32_to_bf16_bits(i.X)
    i.X = workloads.bf16_bits_to_f32(i.X_bits)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    per_token = np.max(np.abs(y - ref), axis=0) / np.max(np.abs(ref), axis=0)
    assert np.all(per_token <= 2e-3)


@pytest.mark.parametrize("fused", ["1", "0"])
@pytest.mark.parametrize("x_dtype", ["bf16", "f32"])
@pytest.mark.parametrize("M,N,K", [(256, 256, 512), (1, 1, 1), (37, 29, 61), (500, 300, 250), (1000, 700, 200), (100, 1000, 260)])
def test_small_single_token_fused_launch(tsvd, M, N, K, x_dtype, fused):
    """Small matrices run both stages in one launch of one workgroup ("1"); the two-launch kernels
    must give the same exact results on them ("0")."""
    tsvd.tsvd_tuning_set("TSVD_GEMV_FUSED", int(fused))
    i = workloads.make_integer_inputs(M, N, K, 1, 0.5, x_dtype, seed=3 * M + N + K)
    print(f"case small single token M={M} N={N} K={K} {x_dtype} fused={fused}", flush=True)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    i = workloads.make_inputs(M, N, K, 1, 0.6, 0.02, x_dtype, seed=4 * M + N + K)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    if np.any(ref):
        assert rel_err(y, ref) <= 1e-5          # the single-token arithmetic is exact to fp32 rounding
    else:
        assert not np.any(y)


# ---- single token, both stages in one launch (z handed over between workgroups as tagged words)
ONEPASS_SHAPES = [(300, 513, 270), (1000, 700, 200), (2100, 1030, 1500), (4100, 2050, 4000), (700, 8000, 520),
                  (8200, 1000, 8100)]


@pytest.mark.parametrize("mode", ["onepass", "onepass_help_all", "onepass_poll_once", "two_launches"])
@pytest.mark.parametrize("M,N,K", ONEPASS_SHAPES)
def test_single_token_one_launch(tsvd, M, N, K, mode):
    """The one-launch kernel against the oracle: exact on integer instances, 1e-5 / 2e-3 on random ones, with the
    slices of z arriving from the other workgroups (default), never polled for (every workgroup computes all of z
    itself: the path taken when a slice does not arrive in time), polled for exactly once, and on the two-launch
    kernels that other streams fall back to.  Several calls in a row reuse the handle's hand-over buffer."""
    import torch
    tsvd.tsvd_tuning_set("TSVD_GEMV_FUSED", 0)
    tsvd.tsvd_tuning_set("TSVD_GEMV_ONEPASS", 0 if mode == "two_launches" else 1)      # (off by default: measured slower)
    if mode == "onepass_help_all":
        tsvd.tsvd_tuning_set("TSVD_SPIN_LIMIT", -1)
    elif mode == "onepass_poll_once":
        tsvd.tsvd_tuning_set("TSVD_SPIN_LIMIT", 0)
    print(f"case one launch M={M} N={N} K={K} {mode}", flush=True)
    for x_dtype in ("bf16", "f32"):
        i = workloads.make_integer_inputs(M, N, K, 1, 0.5, x_dtype, seed=5 * M + N + K)
        ref = oracle.forward(i.U, i.S, i.V, i.X)
        h = tsvd.tsvd_pack(i.U, i.S, i.V)
        x = to_device(i)
        for rep in range(3):                                   # the tag of the hand-over buffer advances per call
            y = torch.full((M, 1), float("nan"), dtype=torch.float32, device=x.device)
            tsvd.tsvd_forward(h, x * float(rep + 1), y)
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy().astype(np.float64), ref * (rep + 1)), f"{x_dtype} call {rep}"
        tsvd.tsvd_free(h)
        j = workloads.make_inputs(M, N, K, 1, 0.6, 0.02, x_dtype, seed=6 * M + N + K)
        y, h = run_forward(j)
        tsvd.tsvd_free(h)
        assert rel_err(y, oracle.forward(j.U, j.S, j.V, j.X)) <= (1e-5 if x_dtype == "f32" else 2e-3)


def test_single_token_one_launch_second_stream_falls_back(tsvd):
    """The hand-over buffer belongs to the first stream that uses the handle for a single token; a call on another
    stream takes the two-launch kernels (its own workspace), so concurrent use stays correct."""
    import torch
    tsvd.tsvd_tuning_set("TSVD_GEMV_ONEPASS", 1)
    i = workloads.make_integer_inputs(2100, 1030, 1500, 1, 0.5, "bf16", seed=77)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    h = tsvd.tsvd_pack(i.U, i.S, i.V)
    x = to_device(i)
    side = torch.cuda.Stream()
    ws = [torch.empty(tsvd.tsvd_workspace_bytes(h, 1, tsvd.TSVD_BF16), dtype=torch.uint8, device=x.device) for _ in range(2)]
    y0 = torch.full((2100, 1), float("nan"), dtype=torch.float32, device=x.device)
    y1 = torch.full((2100, 1), float("nan"), dtype=torch.float32, device=x.device)
    torch.cuda.synchronize()
    for _ in range(4):
        tsvd.tsvd_forward(h, x, y0, workspace=ws[0])
        tsvd.tsvd_forward(h, x, y1, workspace=ws[1], stream=side.cuda_stream)
    torch.cuda.synchronize()
    tsvd.tsvd_free(h)
    assert np.array_equal(y0.cpu().numpy().astype(np.float64), ref)
    assert np.array_equal(y1.cpu().numpy().astype(np.float64), ref)


# ---- stage U of a single token on the denser code of U (five elements per byte; measurement path)
@pytest.mark.parametrize("M,N,K", [(300, 513, 270), (1000, 700, 200), (81, 64, 2415), (4100, 2050, 4000), (700, 300, 8100)])
def test_single_token_dense_code(tsvd, M, N, K):
    import torch
    tsvd.tsvd_tuning_set("TSVD_DENSE_U", 1)
    print(f"case dense code M={M} N={N} K={K}", flush=True)
    for x_dtype in ("bf16", "f32"):
        i = workloads.make_integer_inputs(M, N, K, 1, 0.5, x_dtype, seed=9 * M + N + K)
        y, h = run_forward(i)
        tsvd.tsvd_free(h)
        assert not np.isnan(y).any()
        assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X)), x_dtype
        j = workloads.make_inputs(M, N, K, 1, 0.6, 0.02, x_dtype, seed=8 * M + N + K)
        bias = torch.linspace(-1.0, 1.0, M, device="cuda:0")
        h = tsvd.tsvd_pack(j.U, j.S, j.V)
        y = tsvd.tsvd_forward_ex(h, to_device(j), bias=bias).cpu().numpy().astype(np.float64)
        tsvd.tsvd_free(h)
        ref = oracle.forward_layer(j.U, j.S, j.V, j.X, bias=bias.cpu().numpy().astype(np.float64))
        assert np.max(np.abs(y - ref)) <= (1e-5 if x_dtype == "f32" else 2e-3) * np.max(np.abs(oracle.forward(j.U, j.S, j.V, j.X)))


def test_general_single_token_kernel(tsvd):
    """The slab kernel that serves contraction lengths beyond the fast single-token kernel's
    limits, forced on ordinary sizes (exact instance, then a random one per activation type)."""
    tsvd.tsvd_tuning_set("TSVD_GEMV", 0)
    for B in (1, 2, 5):
        i = workloads.make_integer_inputs(300, 513, 270, B, 0.5, "bf16", seed=900 + B)
        print(f"case general kernel int B={B}", flush=True)
        y, h = run_forward(i)
        tsvd.tsvd_free(h)
        assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    for x_dtype in ("bf16", "f32"):
        i = workloads.make_inputs(1000, 300, 777, 3, 0.6, 0.02, x_dtype, seed=901)
        print(f"case general kernel rand {x_dtype}", flush=True)
        y, h = run_forward(i)
        tsvd.tsvd_free(h)
        assert rel_err(y, oracle.forward(i.U, i.S, i.V, i.X)) <= TOL[x_dtype]


def test_long_contraction_single_token(tsvd):
    """N and K beyond 16384: the single-token path falls back to the slab kernel by itself."""
    i = workloads.make_inputs(64, 20000, 17000, 1, 0.6, 0.02, "bf16", seed=902)
    print("case rand M=64 N=20000 K=17000 B=1 bf16", flush=True)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert rel_err(y, oracle.forward(i.U, i.S, i.V, i.X)) <= TOL["bf16"]


@pytest.mark.parametrize("B", [1, 4, 64, 300])
def test_degenerate_inputs(tsvd, B):
    """All-zero factors or activations give exact zeros; an all-zero token inside a batch does not
    disturb its neighbours (its scale is computed from a zero maximum)."""
    base = workloads.make_inputs(130, 96, 200, B, 0.5, 0.02, "bf16", seed=903 + B)
    print(f"case degenerate B={B}", flush=True)
    for which in ("U", "V", "S", "X"):
        i = workloads.Inputs(base.U.copy(), base.S.copy(), base.V.copy(), base.X.copy(), base.X_bits.copy(), "bf16")
        getattr(i, which)[...] = 0
        if which == "X":
            i.X_bits[...] = 0
        y, h = run_forward(i)
        tsvd.tsvd_free(h)
        assert np.array_equal(y, np.zeros_like(y)), which
    if B > 1:
        i = workloads.Inputs(base.U, base.S, base.V, base.X.copy(), base.X_bits.copy(), "bf16")
        i.X[:, B // 2] = 0
        i.X_bits[:, B // 2] = 0x8000          # negative zeros
        ref = oracle.forward(i.U, i.S, i.V, i.X)
        y, h = run_forward(i)
        tsvd.tsvd_free(h)
        assert np.array_equal(y[:, B // 2], np.zeros(y.shape[0]))
        assert rel_err(y, ref) <= TOL["bf16"]


# ---- ranks that are not multiples of the tile: the ranks of the supplement's layer listing (5, 63, 345, 1545, 2415)
# ---- on its layer shapes (768 -> 3072, 768 -> 1000, 3072 -> 768 reduced).  The batched kernels run ceil(K / 128) steps of
# ---- the contraction and only the filled 32-index sub-steps of the last one.
RAGGED_RANKS = [5, 63, 96, 129, 345, 1545, 2415]


@pytest.mark.parametrize("family", ["rule", "ring14", "ring16", "pipe1", "pipe3", "fallback", "panel", "panel6", "fp6", "fp6direct"])
@pytest.mark.parametrize("K", RAGGED_RANKS)
def test_ragged_rank_batched(tsvd, K, family):
    M, N, B = (1000, 768, 200) if K == 2415 else (600, 384, 200)
    if family in ("panel", "panel6") and K > 1024:
        pytest.skip("the token-panel kernel serves ranks up to 1024")
    sw = {"rule": {}, "ring14": {"TSVD_PANEL": 0, "TSVD_FP6": 0, "TSVD_GEMM_CFG_U": 14, "TSVD_GEMM_CFG_V": 15},
          "ring16": {"TSVD_PANEL": 0, "TSVD_FP6": 0, "TSVD_GEMM_CFG_U": 16, "TSVD_GEMM_CFG_V": 16},
          "pipe1": {"TSVD_PANEL": 0, "TSVD_FP6": 0, "TSVD_GEMM_CFG_U": 1, "TSVD_GEMM_CFG_V": 2},
          "pipe3": {"TSVD_PANEL": 0, "TSVD_FP6": 0, "TSVD_GEMM_CFG_U": 3, "TSVD_GEMM_CFG_V": 0},
          "fallback": {"TSVD_PANEL": 0, "TSVD_FP6": 0, "TSVD_REALIGN": 0, "TSVD_GEMM_CFG_U": 2, "TSVD_GEMM_CFG_V": 3},
          "panel": {"TSVD_PANEL": 1, "TSVD_PANEL_FP6": 0},
          "panel6": {"TSVD_PANEL": 1, "TSVD_PANEL_FP6": 1},
          "fp6": {"TSVD_PANEL": 0, "TSVD_FP6": 1, "TSVD_FP6_V": 1, "TSVD_GEMM_CFG_V": 3, "TSVD_FP6_TALL": 3},
          "fp6direct": {"TSVD_PANEL": 0, "TSVD_FP6": 1, "TSVD_FP6_V": 1, "TSVD_GEMM_CFG_V": 3, "TSVD_FP6_TALL": 0}}[family]
    for k, v in sw.items():
        tsvd.tsvd_tuning_set(k, v)
    Bx = B + 1 if family == "fallback" else B                 # odd row pitch: the register-staged kernel
    print(f"case ragged rank K={K} {family}", flush=True)
    i = workloads.make_integer_inputs(M, N, K, Bx, 0.5, "bf16", seed=31 * K + len(family))
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    j = workloads.make_inputs(M, N, K, Bx, 0.7, 0.02, "bf16", seed=32 * K + len(family))
    y, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert rel_err(y, oracle.forward(j.U, j.S, j.V, j.X)) <= TOL["bf16"]


@pytest.mark.parametrize("B", [1, 2, 9])
@pytest.mark.parametrize("K", RAGGED_RANKS)
def test_ragged_rank_few_tokens(tsvd, K, B):
    """The single-token and few-token kernels read whole tiles; the positions of the rank index must agree with theirs."""
    for x_dtype in ("bf16", "f32"):
        i = workloads.make_integer_inputs(520, 300, K, B, 0.5, x_dtype, seed=77 * K + B)
        y, h = run_forward(i)
        tsvd.tsvd_free(h)
        assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X)), f"{x_dtype}"


# ---- the layer form (tsvd_forward_ex): bias, bf16 output, token-major activations, in every
# ---- kernel family.  Exact instances: an integer bias keeps every value an exactly representable
# ---- integer, so the fp32 output must equal the oracle and the bf16 output its exact rounding.
LAYER_CASES = [
    # M, N, K, B, tuning switches that route the call
    (250, 200, 500, 1, {}),                                   # single token, small matrix: one fused launch
    (300, 513, 270, 1, {}),                                   # single-token kernels, two launches
    (300, 513, 270, 2, {"TSVD_GEMV": "0", "TSVD_MID": "0"}),  # general slab kernel, two tokens per pass
    (100, 2300, 4500, 13, {}),                                # few-token kernel
    (130, 64, 520, 257, {}),                                  # unaligned rows: copied to aligned rows, ring kernels
    (130, 64, 520, 257, {"TSVD_REALIGN": "0"}),               # unaligned rows gathered: large-tile fallback
    (130, 64, 520, 264, {}),                                  # ring kernels (aligned rows)
    (300, 200, 270, 72, {"TSVD_MID": "0", "TSVD_GEMM_CFG_U": "0", "TSVD_GEMM_CFG_V": "1"}),   # pipelined large tiles
    (300, 200, 270, 72, {"TSVD_MID": "0", "TSVD_GEMM_CFG_U": "2", "TSVD_GEMM_CFG_V": "3"}),
    (300, 200, 520, 304, {"TSVD_PANEL": "1", "TSVD_PANEL_FP6": "0"}),                            # token-panel kernel, 16 wavefronts
    (300, 200, 520, 304, {"TSVD_PANEL": "1", "TSVD_PANEL_FP6": "0", "TSVD_PANEL_WAVES": "8"}),   # token-panel kernel, 8 wavefronts
    (300, 200, 520, 304, {"TSVD_PANEL": "1", "TSVD_PANEL_FP6": "1"}),                            # token-panel kernel on fp4 codes x fp6 planes
    (300, 200, 520, 304, {"TSVD_PANEL": "0", "TSVD_GEMM_CFG_U": "14", "TSVD_GEMM_CFG_V": "15"}),   # ring kernels, other shapes
    (700, 200, 760, 304, {"TSVD_PANEL": "0", "TSVD_GEMM_CFG_U": "17", "TSVD_GEMM_CFG_V": "17"}),   # ring kernels, 96-row tiles
    (515, 300, 777, 130, {"TSVD_PANEL": "0", "TSVD_FP6": "1", "TSVD_FP6_V": "0", "TSVD_FP6_TALL": "1"}),   # fp4 x fp6 stage U, 512 x 64 tiles
    (300, 200, 270, 100, {"TSVD_PANEL": "0", "TSVD_FP6": "1", "TSVD_FP6_V": "1", "TSVD_GEMM_CFG_V": "3", "TSVD_FP6_TALL": "3"}),   # both stages on planes
    (515, 300, 777, 130, {"TSVD_PANEL": "0", "TSVD_FP6": "1", "TSVD_FP6_V": "1", "TSVD_GEMM_CFG_V": "3", "TSVD_FP6_TALL": "1"}),   # ... stage V writing the planes of z itself
    (260, 296, 300, 130, {"TSVD_PANEL": "0", "TSVD_FP6": "1", "TSVD_FP6_V": "1", "TSVD_GEMM_CFG_V": "3", "TSVD_FP6_TALL": "0"}),   # ... token-major rows 16-byte aligned
    (300, 204, 520, 304, {"TSVD_PANEL": "1", "TSVD_PANEL_FP6": "1"}),                            # fp4 x fp6 token-panel kernel, token-major rows not 16-byte aligned
    (300, 200, 520, 304, {"TSVD_PANEL": "1", "TSVD_PANEL_FP6": "1", "TSVD_TOKEN_MAJOR_COPY": "1"}),   # ... token-major x copied first
]


@pytest.mark.parametrize("M,N,K,B,env", LAYER_CASES)
def test_layer_form_every_kernel_family(tsvd, M, N, K, B, env):
    import torch
    for k, v in env.items():
        tsvd.tsvd_tuning_set(k, int(v))
    dev = "cuda:0"
    rng = np.random.default_rng(M + B)

    def run(i, bias, layout, y_dtype):
        h = tsvd.tsvd_pack(i.U, i.S, i.V)
        x = to_device(i)
        if layout == tsvd.TSVD_TOKEN_MAJOR:
            # one row per token with a padded pitch; the padding is NaN (kernels that read token-major x in place
            # fetch whole 16-byte runs and must drop what lies beyond N)
            xt = torch.full((B, N + 8), float("nan"), dtype=x.dtype, device=dev)
            xt[:, :N] = x.t()
            x = xt[:, :N]
        b = None if bias is None else torch.from_numpy(bias).to(dev)
        y = torch.full((M, B), float("nan"), dtype=torch.bfloat16 if y_dtype == tsvd.TSVD_BF16 else torch.float32, device=dev)
        tsvd.tsvd_forward_ex(h, x, x_layout=layout, bias=b, y=y, y_dtype=y_dtype)
        # the same call with one row per token in y ([B][M], row pitch M + pad: padded and unpadded rows take the
        # vector and the element-wise stores): must hold the same values, and leave the padding alone
        pad = 4 if (M + B) % 2 else 3
        yt = torch.full((B, M + pad), float("nan"), dtype=y.dtype, device=dev)
        tsvd.tsvd_forward_io(h, x, x_layout=layout, bias=b, y=yt[:, :M], y_dtype=y_dtype, y_layout=tsvd.TSVD_TOKEN_MAJOR)
        torch.cuda.synchronize()
        tsvd.tsvd_free(h)
        assert torch.isnan(yt[:, M:]).all()
        assert torch.equal(yt[:, :M].t().contiguous().view(torch.int16 if y_dtype == tsvd.TSVD_BF16 else torch.int32),
                           y.view(torch.int16 if y_dtype == tsvd.TSVD_BF16 else torch.int32)), "token-major y differs"
        return y.float().cpu().numpy().astype(np.float64)

    i = workloads.make_integer_inputs(M, N, K, B, 0.5, "bf16", seed=5 + M + B)
    bias = rng.integers(-8, 9, size=M).astype(np.float32)
    print(f"case layer int M={M} N={N} K={K} B={B} {env}", flush=True)
    ref = oracle.forward_layer(i.U, i.S, i.V, i.X, bias=bias)
    assert np.array_equal(run(i, bias, tsvd.TSVD_FEATURE_MAJOR, tsvd.TSVD_F32), ref)
    assert np.array_equal(run(i, bias, tsvd.TSVD_TOKEN_MAJOR, tsvd.TSVD_F32), ref)
    assert np.array_equal(run(i, bias, tsvd.TSVD_FEATURE_MAJOR, tsvd.TSVD_BF16), oracle.round_to_bf16(ref))
    assert np.array_equal(run(i, None, tsvd.TSVD_TOKEN_MAJOR, tsvd.TSVD_BF16),
                          oracle.round_to_bf16(oracle.forward(i.U, i.S, i.V, i.X)))

    i = workloads.make_inputs(M, N, K, B, 0.6, 0.02, "bf16", seed=6 + M + B)
    bias = rng.standard_normal(M).astype(np.float32)
    print(f"case layer rand M={M} N={N} K={K} B={B} {env}", flush=True)
    ref = oracle.forward_layer(i.U, i.S, i.V, i.X, bias=bias)
    scale = np.max(np.abs(oracle.forward(i.U, i.S, i.V, i.X)))       # the tolerance of the map itself
    for layout in (tsvd.TSVD_FEATURE_MAJOR, tsvd.TSVD_TOKEN_MAJOR):
        y = run(i, bias, layout, tsvd.TSVD_F32)
        assert not np.isnan(y).any()
        assert np.max(np.abs(y - ref)) <= TOL["bf16"] * scale
        # bf16 output: the same error, then at most one step of the bf16 grid apart (a step is at
        # most 2^-7 of the value)
        yb = run(i, bias, layout, tsvd.TSVD_BF16)
        assert np.all(np.abs(yb - oracle.round_to_bf16(ref)) <= TOL["bf16"] * scale + 2.0 ** -7 * np.abs(ref))
        assert np.array_equal(oracle.round_to_bf16(yb), yb)


@pytest.mark.parametrize("B", [1, 3, 40])
def test_layer_form_fp32_activations(tsvd, B):
    import torch
    i = workloads.make_inputs(256, 300, 512, B, 0.5, 0.02, "f32", seed=50 + B)
    bias = np.random.default_rng(B).standard_normal(256).astype(np.float32)
    ref = oracle.forward_layer(i.U, i.S, i.V, i.X, bias=bias)
    h = tsvd.tsvd_pack(i.U, i.S, i.V)
    xt = to_device(i).t().contiguous()
    ws = torch.empty(tsvd.tsvd_workspace_bytes_ex(h, B, tsvd.TSVD_F32, tsvd.TSVD_TOKEN_MAJOR), dtype=torch.uint8, device="cuda:0")
    y = tsvd.tsvd_forward_ex(h, xt, x_layout=tsvd.TSVD_TOKEN_MAJOR, bias=torch.from_numpy(bias).to("cuda:0"), workspace=ws)
    yt = tsvd.tsvd_forward_io(h, xt, x_layout=tsvd.TSVD_TOKEN_MAJOR, bias=torch.from_numpy(bias).to("cuda:0"), workspace=ws,
                              y_layout=tsvd.TSVD_TOKEN_MAJOR)
    torch.cuda.synchronize()
    tsvd.tsvd_free(h)
    assert np.max(np.abs(y.cpu().numpy().astype(np.float64) - ref)) <= 1e-5 * np.max(np.abs(ref))
    ref_t = oracle.forward_layer(i.U, i.S, i.V, i.X, bias=bias, y_layout="token_major")
    assert yt.shape == (B, 256) and np.max(np.abs(yt.cpu().numpy().astype(np.float64) - ref_t)) <= 1e-5 * np.max(np.abs(ref))


def test_strided_inputs_outputs_and_caller_workspace(tsvd):
    import torch
    i = workloads.make_inputs(300, 200, 270, 70, 0.5, 0.02, "bf16", seed=5)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    h = tsvd.tsvd_pack(i.U, i.S, i.V)
    xfull = torch.zeros((200, 91), dtype=torch.bfloat16, device="cuda:0")     # odd stride: slow load path
    xfull[:, :70] = to_device(i)
    yfull = torch.full((300, 75), 7.0, dtype=torch.float32, device="cuda:0")
    ws = torch.empty(tsvd.tsvd_workspace_bytes(h, 70, tsvd.TSVD_BF16), dtype=torch.uint8, device="cuda:0")
    tsvd.tsvd_forward(h, xfull[:, :70], yfull[:, :70], workspace=ws)
    torch.cuda.synchronize()
    y = yfull.cpu().numpy().astype(np.float64)
    assert rel_err(y[:, :70], ref) <= 2e-3
    assert np.all(y[:, 70:] == 7.0)                                           # padding columns untouched
    # a side stream and the handle-owned workspace
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        y2 = tsvd.tsvd_forward(h, xfull[:, :70])
    st.synchronize()
    assert np.array_equal(y2.cpu().numpy(), yfull[:, :70].cpu().numpy())      # deterministic
    tsvd.tsvd_free(h)


def test_device_round_trip_info_and_errors(tsvd):
    import torch
    i = workloads.make_inputs(70, 50, 90, 4, 0.6, 0.02, "f32", seed=8)
    buf = torch.empty(tsvd.tsvd_packed_bytes(70, 90, 50), dtype=torch.uint8, device="cuda:0")
    h = tsvd.tsvd_pack(i.U, i.S, i.V, dev_buf=buf)           # caller-owned device blob
    U, S, V = tsvd.tsvd_unpack(h)
    assert np.array_equal(U, i.U) and np.array_equal(V, i.V) and np.array_equal(S, i.S)
    info = tsvd.tsvd_info(h)
    c = oracle.op_counts(i.U, i.V)
    assert (info["M"], info["K"], info["N"]) == (70, 90, 50)
    assert info["nnzU"] == c["adds_U"] and info["nnzV"] == c["adds_V"]     # Table S1 addition count
    x = to_device(i)
    lib = tsvd.load_library()
    y = torch.zeros((70, 4), dtype=torch.float32, device="cuda:0")
    args = dict(B=4, ldx=4, ldy=4)
    call = lambda **o: lib.tsvd_forward(o.get("h", h.ptr), o.get("x", x.data_ptr()), o.get("xd", 0), o.get("B", 4),
                                        o.get("ldx", 4), o.get("y", y.data_ptr()), o.get("yd", 0), o.get("ldy", 4),
                                        o.get("ws", None), o.get("wsb", 0), None)
    assert call(h=None) == 1 and call(x=None) == 1 and call(y=None) == 1
    assert call(B=0) == 1 and call(ldx=3) == 1 and call(ldy=3) == 1 and call(xd=7) == 1
    assert call(yd=9) == 1
    assert call(ws=x.data_ptr(), wsb=16) == 1                 # workspace too small
    torch.cuda.synchronize()
    assert torch.all(y == 0)                                   # failures leave outputs untouched
    assert call() == 0
    torch.cuda.synchronize()
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    assert rel_err(y.cpu().numpy().astype(np.float64), ref) <= 1e-5
    with pytest.raises(tsvd.TsvdError):
        bad = i.U.copy()
        bad[0, 0] = 5
        tsvd.tsvd_pack(bad, i.S, i.V)
    tsvd.tsvd_free(h)
    tsvd.tsvd_free(h)                                          # double free of the wrapper is a no-op
    lib.tsvd_free(None)


def test_repeated_calls_are_bit_identical(tsvd):
    import torch
    for (M, N, K, B, dt) in ((2048, 1024, 1536, 1, "bf16"), (512, 256, 768, 300, "bf16")):
        i = workloads.make_inputs(M, N, K, B, 0.5, 0.02, dt, seed=21)
        h = tsvd.tsvd_pack(i.U, i.S, i.V)
        x = to_device(i)
        ys = [tsvd.tsvd_forward(h, x).cpu().numpy() for _ in range(3)]
        assert np.array_equal(ys[0], ys[1]) and np.array_equal(ys[0], ys[2])
        tsvd.tsvd_free(h)


# ---- stage U on fp4 codes x three fp6 planes of Z (experimental switch TSVD_FP6=1)
@pytest.mark.parametrize("tile", ["0", "1", "2", "3"])   # 256 x 128, 512 x 64 (where 512 divides the padded rows), 256 x 64, 128 x 64
@pytest.mark.parametrize("stage_v", [False, True, "fp16 z"])
@pytest.mark.parametrize("M,N,K,B", [(300, 200, 270, 100), (515, 300, 777, 130), (1024, 512, 768, 512), (130, 64, 2100, 257),
                                     (512, 300, 1024, 200)])
def test_fp6_planes_stage_u(tsvd, M, N, K, B, stage_v, tile):
    """Z as three E2M3 planes with per-lane block scales, multiplied with the codes as fp4 on the scaled
    128-deep MFMA: exact on integer instances (small integers need one plane), within the tolerance
    of the 16-bit path on random ones and next to identical to it; bias and bf16 output included.
    stage_v: x goes through planes as well (stage V on the same kernel; forced here, with the
    two-kernel form of stage V that it replaces).  With 256- and 512-row tiles that stage V writes the
    planes of z itself; "fp16 z" keeps its older form (fp16 z, column maxima, a pass that makes the planes)."""
    import torch
    if stage_v == "fp16 z" and tile in ("2", "3"):
        pytest.skip("the smaller tiles always go through fp16 z")
    tsvd.tsvd_tuning_set("TSVD_FP6", 1)
    tsvd.tsvd_tuning_set("TSVD_FP6_V", 1 if stage_v else 0)
    tsvd.tsvd_tuning_set("TSVD_FP6_DIRECT", 0 if stage_v == "fp16 z" else 1)
    tsvd.tsvd_tuning_set("TSVD_FP6_TALL", int(tile))
    if stage_v:
        tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_V", 3)
    i = workloads.make_integer_inputs(M, N, K, B, 0.5, "bf16", seed=606 + B)
    print(f"case fp6 int M={M} N={N} K={K} B={B}", flush=True)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    j = workloads.make_inputs(M, N, K, B, 0.6, 0.02, "bf16", seed=607 + B)
    print(f"case fp6 rand M={M} N={N} K={K} B={B}", flush=True)
    ref = oracle.forward(j.U, j.S, j.V, j.X)
    y1, h = run_forward(j)
    assert not np.isnan(y1).any()
    assert rel_err(y1, ref) <= TOL["bf16"]
    bias = torch.linspace(-1.0, 1.0, M, device="cuda:0")
    yb = tsvd.tsvd_forward_ex(h, to_device(j), bias=bias, y_dtype=tsvd.TSVD_BF16).float().cpu().numpy().astype(np.float64)
    refb = ref + bias.cpu().numpy().astype(np.float64)[:, None]
    assert np.all(np.abs(yb - refb) <= TOL["bf16"] * np.max(np.abs(ref)) + 2.0 ** -8 * np.abs(refb))
    tsvd.tsvd_tuning_set("TSVD_FP6", 0)
    y0 = tsvd.tsvd_forward(h, to_device(j)).cpu().numpy().astype(np.float64)
    tsvd.tsvd_free(h)
    assert rel_err(y0, y1) <= 5e-4        # both round Z to about 12 bits, differently


@pytest.mark.parametrize("family", ["panel6", "direct 256x128", "direct 512x64"])
def test_plane_kernels_resolve_three_planes(tsvd, family):
    """Where z goes from the fp32 accumulators straight into three E2M3 planes (the fp4 x fp6 token-panel launch, the
    fp4 x fp6 stage V that writes the planes itself) nothing is rounded to 16 bits on the way: the error is that of
    the planes, about 3e-5 of max |y|, in EVERY 16-token tile.  (A plane converted with a wrong scale costs a factor
    of 30 to 100 in the tiles it touches and still passes the 2e-3 tolerance of the other tests.)"""
    M, N, K, B = (600, 384, 700, 200)
    sw = {"panel6": {"TSVD_PANEL": 1, "TSVD_PANEL_FP6": 1},
          "direct 256x128": {"TSVD_PANEL": 0, "TSVD_FP6": 1, "TSVD_FP6_V": 1, "TSVD_GEMM_CFG_V": 3, "TSVD_FP6_TALL": 0},
          "direct 512x64": {"TSVD_PANEL": 0, "TSVD_FP6": 1, "TSVD_FP6_V": 1, "TSVD_GEMM_CFG_V": 3, "TSVD_FP6_TALL": 1}}[family]
    for k, v in sw.items():
        tsvd.tsvd_tuning_set(k, v)
    print(f"case three planes {family}", flush=True)
    j = workloads.make_inputs(M, N, K, B, 0.7, 0.02, "bf16", seed=4711)
    ref = oracle.forward(j.U, j.S, j.V, j.X)
    y, h = run_forward(j)
    tsvd.tsvd_free(h)
    err = np.abs(y - ref) / np.max(np.abs(ref))
    per_tile = [float(err[:, c:c + 16].max()) for c in range(0, B, 16)]
    assert max(per_tile) <= 1e-4, per_tile


@pytest.mark.parametrize("mode", ["fp16", "fp6"])
def test_outlier_features(tsvd, mode):
    """Activations with outlier features (1 % of the features 300 times larger, as in transformer
    layers): the per-token scaling of z and, on the fp4 x fp6 kernels, the block scales of the planes of
    both stages keep the error at the level of ordinary inputs."""
    tsvd.tsvd_tuning_set("TSVD_FP6", 1 if mode == "fp6" else 0)
    if mode == "fp6":
        tsvd.tsvd_tuning_set("TSVD_FP6_V", 1)
        tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_V", 3)
    i = workloads.make_outlier_inputs(512, 1280, 1024, 300, 0.6, 0.02, seed=77, factor=300.0, share=0.01)
    assert np.max(np.abs(i.X)) > 100.0
    print(f"case outliers {mode}", flush=True)
    ref = oracle.forward(i.U, i.S, i.V, i.X)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert rel_err(y, ref) <= 0.5 * TOL["bf16"]
    rows = np.max(np.abs(y - ref), axis=1) / np.max(np.abs(ref), axis=1)
    assert np.median(rows) <= 0.5 * TOL["bf16"]


@pytest.mark.parametrize("M,N,K,B", [(1024, 512, 768, 512), (512, 300, 1024, 200), (700, 2100, 2300, 130)])
def test_fp6_two_planes_switch(tsvd, M, N, K, B):
    """The accuracy / speed switch of the fp4 x fp6 kernels (two planes instead of three, never chosen by
    default): still within the tolerance of bf16 activations, at about five times the error."""
    tsvd.tsvd_tuning_set("TSVD_FP6", 1)
    tsvd.tsvd_tuning_set("TSVD_FP6_V", 1)
    tsvd.tsvd_tuning_set("TSVD_GEMM_CFG_V", 3)
    tsvd.tsvd_tuning_set("TSVD_FP6_PLANES", 2)
    j = workloads.make_inputs(M, N, K, B, 0.6, 0.02, "bf16", seed=909 + B)
    print(f"case fp6 two planes M={M} N={N} K={K} B={B}", flush=True)
    ref = oracle.forward(j.U, j.S, j.V, j.X)
    y, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert not np.isnan(y).any()
    assert rel_err(y, ref) <= TOL["bf16"]

@pytest.mark.parametrize("seed", [11, 12, 13])
def test_randomized_layer_calls_on_the_plane_kernels(tsvd, seed):
    """Seeded random shapes, layouts, row pitches (NaN in the padding of x, untouched padding of y), bias and output
    types on the fp4 x fp6 token-panel launch and on the fp4 x fp6 stage V that writes the planes of z (both tiles):
    exact on integer instances, within tolerance on random ones."""
    import torch
    dev = "cuda:0"
    rng = np.random.default_rng(seed)
    for trial in range(12):
        fam = ["panel6", "direct0", "direct1"][trial % 3]
        M = int(rng.integers(1, 700))
        N = int(rng.integers(1, 1024 if fam == "panel6" else 1500))
        K = int(rng.integers(1, 1024 if fam == "panel6" else 1800))
        B = int(rng.integers(17, 1500))
        xl, yl, ybf, use_bias = (int(rng.integers(0, 2)) for _ in range(4))
        padx, pady = int(rng.choice([0, 3, 8])), int(rng.choice([0, 1, 4]))
        tsvd.tsvd_tuning_reset()
        sw = {"panel6": {"TSVD_PANEL": 1, "TSVD_PANEL_FP6": 1},
              "direct0": {"TSVD_PANEL": 0, "TSVD_FP6": 1, "TSVD_FP6_V": 1, "TSVD_GEMM_CFG_V": 3, "TSVD_FP6_TALL": 0},
              "direct1": {"TSVD_PANEL": 0, "TSVD_FP6": 1, "TSVD_FP6_V": 1, "TSVD_GEMM_CFG_V": 3, "TSVD_FP6_TALL": 1}}[fam]
        for k, v in sw.items():
            tsvd.tsvd_tuning_set(k, v)
        integer = trial % 2 == 0
        i = (workloads.make_integer_inputs(M, N, K, B, 0.5, "bf16", seed=100 * seed + trial) if integer
             else workloads.make_inputs(M, N, K, B, 0.6, 0.02, "bf16", seed=100 * seed + trial))
        bias = None
        if use_bias:
            bias = rng.integers(-8, 9, size=M).astype(np.float32) if integer else rng.standard_normal(M).astype(np.float32)
        print(f"case trial {trial} {fam} M={M} N={N} K={K} B={B} x_layout={xl} y_layout={yl} bf16={ybf} bias={use_bias} "
              f"padx={padx} pady={pady} integer={integer}", flush=True)
        ref = oracle.forward_layer(i.U, i.S, i.V, i.X, bias=bias)
        h = tsvd.tsvd_pack(i.U, i.S, i.V)
        x = to_device(i)
        xb = torch.full((B, N + padx) if xl else (N, B + padx), float("nan"), dtype=x.dtype, device=dev)
        xx = xb[:, :N] if xl else xb[:, :B]
        xx.copy_(x.t() if xl else x)
        ydt = torch.bfloat16 if ybf else torch.float32
        yb = torch.full((B, M + pady) if yl else (M, B + pady), float("nan"), dtype=ydt, device=dev)
        yy = yb[:, :M] if yl else yb[:, :B]
        b = None if bias is None else torch.from_numpy(bias).to(dev)
        tsvd.tsvd_forward_io(h, xx, x_layout=xl, bias=b, y=yy, y_dtype=tsvd.TSVD_BF16 if ybf else tsvd.TSVD_F32, y_layout=yl)
        torch.cuda.synchronize()
        tsvd.tsvd_free(h)
        got = (yy.t() if yl else yy).float().cpu().numpy().astype(np.float64)
        assert bool(torch.isnan(yb[:, (M if yl else B):]).all()), "padding of y touched"
        assert not np.isnan(got).any()
        want = oracle.round_to_bf16(ref) if ybf else ref
        if integer:
            assert np.array_equal(got, want)
        else:
            scale = np.max(np.abs(oracle.forward(i.U, i.S, i.V, i.X)))
            assert np.all(np.abs(got - want) <= TOL["bf16"] * scale + (2.0 ** -7 * np.abs(ref) if ybf else 0.0))

@pytest.mark.parametrize("M,K", [(17 * 512 + 300, 17 * 512 + 512), (22 * 512, 21 * 512 + 130)])
def test_fp6_tail_tiles(tsvd, M, K):
    """Launches of more than one round of 512 x 64 tiles whose last round would be at most half full end in tiles cut along
    the tokens (stage U, and the stage V that writes the planes of z): a quarter or an eighth of a round left over here,
    ragged rows and tokens; sampled columns against the oracle, and the same bits as the plain launch."""
    import torch
    N, B = 200, 2048 - 37
    for k, v in {"TSVD_PANEL": 0, "TSVD_FP6": 1, "TSVD_FP6_V": 1, "TSVD_GEMM_CFG_V": 3, "TSVD_FP6_TALL": 1}.items():
        tsvd.tsvd_tuning_set(k, v)
    print(f"case fp6 tail M={M} K={K}", flush=True)
    j = workloads.make_inputs(M, N, K, B, 0.6, 0.02, "bf16", seed=M + K)
    cols = sorted(set([0, 15, 16, 31, 32, 63, 64, B - 1, B - 16, B - 17, B - 33, B // 2] + list(np.random.default_rng(3).integers(0, B, 30))))
    ref = oracle.forward_columns(j.U, j.S, j.V, j.X, cols)
    y1, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert not np.isnan(y1).any()
    assert rel_err(y1[:, cols], ref) <= 1e-4            # (three planes, z never rounded to 16 bits)
    tsvd.tsvd_tuning_set("TSVD_FP6_TAIL", 0)
    y0, h = run_forward(j)
    tsvd.tsvd_free(h)
    assert np.array_equal(y0, y1)

@pytest.mark.parametrize("tile", [0, 1])
@pytest.mark.parametrize("M,N,K,B", [(300, 200, 270, 17), (515, 300, 777, 130), (1030, 512, 1024, 300), (64, 1300, 129, 65)])
def test_fp32_activations_batched(tsvd, M, N, K, B, tile):
    """fp32 activations with 17 tokens or more: six E2M3 planes of x (three, and three for what those leave), stage V
    writing six planes of z from its fp32 accumulators, the second set of planes as further blocks of the contraction.
    Exact on integer instances, 1e-5 of max |y| on random ones (measured about 2e-7), bias / bf16 / token-major options,
    and the same result as one token at a time up to that tolerance."""
    import torch
    tsvd.tsvd_tuning_set("TSVD_FP6_TALL", tile)
    i = workloads.make_integer_inputs(M, N, K, B, 0.5, "f32", seed=808 + B)
    print(f"case fp32 batched int M={M} N={N} K={K} B={B} tile={tile}", flush=True)
    y, h = run_forward(i)
    tsvd.tsvd_free(h)
    assert np.array_equal(y, oracle.forward(i.U, i.S, i.V, i.X))
    j = workloads.make_inputs(M, N, K, B, 0.6, 0.02, "f32", seed=809 + B)
    print(f"case fp32 batched rand M={M} N={N} K={K} B={B} tile={tile}", flush=True)
    ref = oracle.forward(j.U, j.S, j.V, j.X)
    y1, h = run_forward(j)
    assert not np.isnan(y1).any()
    assert rel_err(y1, ref) <= TOL["f32"]
    bias = torch.linspace(-1.0, 1.0, M, device="cuda:0")
    refb = ref + bias.cpu().numpy().astype(np.float64)[:, None]
    xt = torch.full((B, N + 3), float("nan"), dtype=torch.float32, device="cuda:0")
    xt[:, :N] = to_device(j).t()
    yt = torch.full((B, M + 1), float("nan"), dtype=torch.float32, device="cuda:0")
    tsvd.tsvd_forward_io(h, xt[:, :N], x_layout=tsvd.TSVD_TOKEN_MAJOR, bias=bias, y=yt[:, :M], y_dtype=tsvd.TSVD_F32, y_layout=tsvd.TSVD_TOKEN_MAJOR)
    assert bool(torch.isnan(yt[:, M:]).all())
    assert np.max(np.abs(yt[:, :M].t().cpu().numpy().astype(np.float64) - refb)) <= TOL["f32"] * np.max(np.abs(ref))
    yb = tsvd.tsvd_forward_ex(h, to_device(j), bias=bias, y_dtype=tsvd.TSVD_BF16).float().cpu().numpy().astype(np.float64)
    assert np.all(np.abs(yb - refb) <= TOL["f32"] * np.max(np.abs(ref)) + 2.0 ** -8 * np.abs(refb))
    tsvd.tsvd_tuning_set("TSVD_GEMM_MIN_B_F32", 1 << 30)      # one token at a time
    y0 = tsvd.tsvd_forward(h, to_device(j)).cpu().numpy().astype(np.float64)
    tsvd.tsvd_free(h)
    assert rel_err(y0, y1) <= TOL["f32"]
