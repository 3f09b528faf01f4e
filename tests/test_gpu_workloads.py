"""GPU parity on the named workloads at full size, in the launch configuration bench.py
times.  Where the full output is too much work for the CPU oracle, a seeded subset of tokens
(columns are independent, so this checks those columns exactly) including tile-boundary
columns is compared."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_util import rel_err, run_forward


def _columns(B, count, seed):
    """Tile-boundary columns (all kept) plus a seeded draw over 0..B-1 on top of them."""
    edge = [c for c in (0, 1, 15, 16, 63, 64, 127, 128, 255, 256, 257, B // 2 - 1, B // 2, B - 257, B - 256, B - 129,
                        B - 128, B - 2, B - 1) if 0 <= c < B]
    rng = np.random.default_rng(seed)
    rest = rng.choice(B, size=min(B, count), replace=False).tolist()
    cols = sorted(set(edge + rest))
    for c in (0, B // 2, B - 1, B - 128, B - 256):
        assert c < 0 or c in cols
    assert len(cols) >= min(B, count) and cols[-1] == B - 1
    return cols


def test_columns_cover_the_whole_token_range():
    for B, count in ((2048, 64), (12544, 384), (256, 64)):
        cols = _columns(B, count, 7)
        assert cols[0] == 0 and cols[-1] == B - 1 and len(set(cols)) == len(cols)
        assert sum(c >= B // 2 for c in cols) >= count // 4      # the upper half is sampled too
        assert {B - 1, B - 128, B // 2} <= set(cols)


@pytest.mark.gpu
@pytest.mark.parametrize("name,ncols,tol", [
    ("tiny", None, 1e-5),
    ("bert_ffn_in", None, 2e-3),
    ("convnext_mlp", 384, 2e-3),
    ("opt6b7_fc1_decode", None, 2e-3),
    ("opt66b_fc1_prefill", 64, 2e-3),
    ("opt6b7_fc1_decode_b16", None, 2e-3),
    ("opt6b7_fc1_prefill_b256", 64, 2e-3),
    ("ffn_768x3072_rank1545", 96, 2e-3),
])
def test_named_workload(name, ncols, tol):
    import paper_2308_07641_amd as tsvd
    w = workloads.WORKLOADS[name]
    print(f"workload {name}: M={w.M} N={w.N} K={w.K} B={w.B}", flush=True)
    i = workloads.make_workload(name)
    print("  inputs drawn", flush=True)
    y, h = run_forward(i)
    info = tsvd.tsvd_info(h)
    tsvd.tsvd_free(h)
    print("  gpu done", flush=True)
    assert not np.isnan(y).any()
    assert info["nnzU"] == np.count_nonzero(i.U) and info["nnzV"] == np.count_nonzero(i.V)
    if ncols is None:
        ref = oracle.forward(i.U, i.S, i.V, i.X)
        err = rel_err(y, ref)
    else:
        cols = _columns(w.B, ncols, w.seed)
        ref = oracle.forward_columns(i.U, i.S, i.V, i.X, cols)
        # the tolerance is relative to max|y_ref| of the whole output; the sampled maximum is a
        # lower bound of it, so this check is the stricter one
        err = rel_err(y[:, cols], ref)
    print(f"  rel err {err:.3e}", flush=True)
    assert err <= tol
