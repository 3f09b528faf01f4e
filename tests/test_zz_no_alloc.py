"""The entry point that allocates nothing (tsvd_forward_noalloc) against tsvd_forward_ex: same kernels on the
library's fixed per-GPU workspace, so the outputs must be identical; two calls in a row, the second smaller."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import rel_err, to_device

pytestmark = pytest.mark.gpu


def _both(tsvd, torch, h, i, bias=None, y_dtype=None):
    x = to_device(i)
    y_dtype = tsvd.TSVD_F32 if y_dtype is None else y_dtype
    ydt = torch.bfloat16 if y_dtype == tsvd.TSVD_BF16 else torch.float32
    B = x.shape[1]
    ws = torch.empty(tsvd.tsvd_workspace_bytes_ex(h, B, tsvd.TSVD_BF16 if i.x_dtype == "bf16" else tsvd.TSVD_F32,
                                                  tsvd.TSVD_FEATURE_MAJOR), dtype=torch.uint8, device=x.device)
    y_ref = torch.full((h.M, B), float("nan"), dtype=ydt, device=x.device)
    y_new = torch.full((h.M, B), float("nan"), dtype=ydt, device=x.device)
    tsvd.tsvd_forward_ex(h, x, bias=bias, y=y_ref, y_dtype=y_dtype, workspace=ws)
    tsvd.tsvd_forward_noalloc(h, x, y_new, bias=bias, y_dtype=y_dtype)
    torch.cuda.synchronize()
    return y_ref, y_new


def test_noalloc_two_calls_second_smaller():
    import torch
    import paper_2308_07641_amd as tsvd
    # first call: batched path (z fp16 [K][B] in the workspace), 1.9 MB of it; second: fewer tokens on a smaller layer
    big = workloads.make_inputs(768, 512, 1024, 300, 0.5, 0.02, "bf16", seed=901)
    small = workloads.make_inputs(320, 200, 300, 40, 0.5, 0.02, "bf16", seed=902)
    hb, hs = tsvd.tsvd_pack(big.U, big.S, big.V), tsvd.tsvd_pack(small.U, small.S, small.V)
    for h, i in ((hb, big), (hs, small)):
        y_ref, y_new = _both(tsvd, torch, h, i)
        assert not torch.isnan(y_new).any()
        assert torch.equal(y_ref, y_new)                   # same kernels, same arithmetic: bit for bit
        ref = oracle.forward(i.U, i.S, i.V, i.X)
        assert rel_err(y_new.cpu().numpy().astype(np.float64), ref) <= 2e-3
    # and once more the large one after the small one (the array keeps the small call's contents)
    y_ref, y_new = _both(tsvd, torch, hb, big)
    assert torch.equal(y_ref, y_new)
    tsvd.tsvd_free(hb)
    tsvd.tsvd_free(hs)


def test_noalloc_single_token_few_tokens_and_layer_options():
    import torch
    import paper_2308_07641_amd as tsvd
    for (M, N, K, B, dt, tol) in ((512, 768, 1024, 1, "f32", 1e-5), (1024, 512, 768, 1, "bf16", 2e-3), (512, 512, 512, 7, "bf16", 2e-3)):
        i = workloads.make_inputs(M, N, K, B, 0.6, 0.02, dt, seed=910 + B + M)
        h = tsvd.tsvd_pack(i.U, i.S, i.V)
        bias = torch.linspace(-1.0, 1.0, M, device="cuda:0")
        y_ref, y_new = _both(tsvd, torch, h, i, bias=bias)
        assert torch.equal(y_ref, y_new)
        ref = oracle.forward_layer(i.U, i.S, i.V, i.X, bias=bias.cpu().numpy().astype(np.float64))
        assert rel_err(y_new.cpu().numpy().astype(np.float64), ref) <= tol
        y_ref, y_new = _both(tsvd, torch, h, i, bias=bias, y_dtype=tsvd.TSVD_BF16)
        assert torch.equal(y_ref.view(torch.int16), y_new.view(torch.int16))
        tsvd.tsvd_free(h)


def test_noalloc_rejects_calls_beyond_the_fixed_workspace():
    import torch
    import paper_2308_07641_amd as tsvd
    i = workloads.make_inputs(256, 256, 4096, 1, 0.5, 0.02, "bf16", seed=920)
    h = tsvd.tsvd_pack(i.U, i.S, i.V)
    B = 4096                                                # z fp16 [4096][4096] = 32 MiB > 16 MiB
    assert tsvd.tsvd_workspace_bytes_ex(h, B, tsvd.TSVD_BF16, tsvd.TSVD_FEATURE_MAJOR) > tsvd.TSVD_NOALLOC_MAX_WORKSPACE
    x = torch.zeros((256, B), dtype=torch.bfloat16, device="cuda:0")
    y = torch.full((256, B), 7.0, dtype=torch.float32, device="cuda:0")
    with pytest.raises(tsvd.TsvdError) as e:
        tsvd.tsvd_forward_noalloc(h, x, y)
    assert e.value.status == 6 and "workspace" in str(e.value)
    torch.cuda.synchronize()
    assert bool((y == 7.0).all())                           # nothing was enqueued
    tsvd.tsvd_free(h)


def test_noalloc_fp32_batches():
    """fp32 batches take the batched kernels on six planes when those fit the fixed workspace (same bits as
    tsvd_forward_ex), and go one token at a time when they do not (same tolerance, no rejection)."""
    import torch
    import paper_2308_07641_amd as tsvd
    i = workloads.make_inputs(300, 200, 520, 40, 0.6, 0.02, "f32", seed=930)
    h = tsvd.tsvd_pack(i.U, i.S, i.V)
    y_ref, y_new = _both(tsvd, torch, h, i)
    assert torch.equal(y_ref, y_new)
    assert rel_err(y_new.cpu().numpy().astype(np.float64), oracle.forward(i.U, i.S, i.V, i.X)) <= 1e-5
    tsvd.tsvd_free(h)
    i = workloads.make_inputs(128, 8192, 8192, 20, 0.6, 0.02, "f32", seed=931)      # planes of x and z: 20 MiB
    h = tsvd.tsvd_pack(i.U, i.S, i.V)
    assert tsvd.tsvd_workspace_bytes_ex(h, 20, tsvd.TSVD_F32, tsvd.TSVD_FEATURE_MAJOR) > tsvd.TSVD_NOALLOC_MAX_WORKSPACE
    y = torch.full((128, 20), float("nan"), dtype=torch.float32, device="cuda:0")
    tsvd.tsvd_forward_noalloc(h, to_device(i), y)
    torch.cuda.synchronize()
    assert rel_err(y.cpu().numpy().astype(np.float64), oracle.forward(i.U, i.S, i.V, i.X)) <= 1e-5
    tsvd.tsvd_free(h)
