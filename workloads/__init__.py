"""Seeded synthetic inputs for the TSVD forward map y = U (diag(S) (V x)).

This module only draws numbers and rounds them to the storage type of the
activations; it holds none of the method's arithmetic.  Both the CPU oracle's
tests and the GPU tests feed the arrays produced here, unchanged, to their
respective implementations.

The five named workloads take only layer *shapes* from the networks the paper
evaluates (BERT, ConvNeXt/Swin, OPT: Experiments section and the per-layer
rank listing in the supplement); weights and activations are i.i.d. draws.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

SEED_BASE = 23080764


@dataclass(frozen=True)
class Workload:
    name: str
    index: int      # 1-based position in the configuration list
    M: int          # output features  (rows of U)
    N: int          # input features   (columns of V)
    K: int          # TSVD rank        (columns of U, rows of V, length of S)
    B: int          # tokens           (columns of X)
    p0: float       # probability of a zero entry in U and V (1 - non-zero rate r)
    s_scale: float  # S = |N(0,1)| * s_scale
    x_dtype: str    # "f32" or "bf16": storage type of the activations

    @property
    def seed(self) -> int:
        return SEED_BASE + 1000 * self.index


WORKLOADS = {
    w.name: w
    for w in (
        Workload("tiny", 1, 256, 256, 512, 1, 0.5, 0.02, "f32"),
        Workload("bert_ffn_in", 2, 3072, 768, 1536, 512, 0.5, 0.02, "bf16"),
        Workload("convnext_mlp", 3, 2048, 512, 1024, 12544, 0.6, 0.02, "bf16"),
        Workload("opt6b7_fc1_decode", 4, 16384, 4096, 8192, 1, 0.6, 0.01, "bf16"),
        Workload("opt66b_fc1_prefill", 5, 36864, 9216, 18432, 2048, 0.6, 0.01, "bf16"),
        # the decode layer with a small batch of tokens (measurement case of the few-token path)
        Workload("opt6b7_fc1_decode_b16", 6, 16384, 4096, 8192, 16, 0.6, 0.01, "bf16"),
        # the same layer on a prefill chunk of 256 tokens (measurement case of the small tiles of the batched path)
        Workload("opt6b7_fc1_prefill_b256", 7, 16384, 4096, 8192, 256, 0.6, 0.01, "bf16"),
        # a 768 -> 3072 layer at a rank of the supplement's layer listing that is no multiple of the tile (1545), with the
        # non-zero rate the paper reports for converted layers (about 0.28), on 4096 tokens (measurement case of ragged ranks)
        Workload("ffn_768x3072_rank1545", 8, 3072, 768, 1545, 4096, 0.72, 0.02, "bf16"),
    )
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def ternary(rng: np.random.Generator, shape, p0: float) -> np.ndarray:
    """i.i.d. entries: 0 with probability p0, +1 and -1 with (1-p0)/2 each (int8)."""
    rows, cols = shape
    out = np.empty((rows, cols), dtype=np.int8)
    step = max(1, (1 << 24) // max(cols, 1))          # bound the fp64 temporary
    hi = p0 + (1.0 - p0) / 2.0
    for r0 in range(0, rows, step):
        u = rng.random((min(step, rows - r0), cols))
        blk = out[r0:r0 + u.shape[0]]
        blk[...] = -1
        blk[u < hi] = 1
        blk[u < p0] = 0
    return out


@dataclass
class Inputs:
    U: np.ndarray        # int8 [M, K]
    S: np.ndarray        # float32 [K]
    V: np.ndarray        # int8 [K, N]
    X: np.ndarray        # float32 [N, B]: the exact values of the activations
    X_bits: np.ndarray | None   # uint16 [N, B] bf16 patterns when x_dtype == "bf16"
    x_dtype: str


def make_inputs(M: int, N: int, K: int, B: int, p0: float, s_scale: float,
                x_dtype: str, seed: int) -> Inputs:
    """Draw U, V, S, X in that order from PCG64(seed)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    U = ternary(rng, (M, K), p0)
    V = ternary(rng, (K, N), p0)
    S = (np.abs(rng.standard_normal(K)) * s_scale).astype(np.float32)
    X = rng.standard_normal((N, B)).astype(np.float32)
    bits = None
    if x_dtype == "bf16":
        bits = f32_to_bf16_bits(X)
        X = bf16_bits_to_f32(bits)
    elif x_dtype != "f32":
        raise ValueError(f"unknown activation type {x_dtype!r}")
    return Inputs(U, S, V, X, bits, x_dtype)


def make_outlier_inputs(M: int, N: int, K: int, B: int, p0: float, s_scale: float, seed: int,
                        factor: float, share: float) -> Inputs:
    """make_inputs with bf16 activations whose features (rows of X) are multiplied by `factor` with
    probability `share`: the outlier channels of transformer activations (a few features two or
    three orders of magnitude above the rest, in every token)."""
    base = make_inputs(M, N, K, B, p0, s_scale, "f32", seed)
    rng = np.random.Generator(np.random.PCG64(seed + 1))
    X = base.X.copy()
    X[rng.random(N) < share] *= np.float32(factor)
    bits = f32_to_bf16_bits(X)
    return Inputs(base.U, base.S, base.V, bf16_bits_to_f32(bits), bits, "bf16")


def make_workload(name: str, B: int | None = None) -> Inputs:
    """Inputs of a named workload; B overrides the token count (same seed)."""
    w = WORKLOADS[name]
    return make_inputs(w.M, w.N, w.K, w.B if B is None else B, w.p0, w.s_scale,
                       w.x_dtype, w.seed)


def make_integer_inputs(M: int, N: int, K: int, B: int, p0: float, x_dtype: str,
                        seed: int, x_max: int = 4) -> Inputs:
    """Integer-valued activations in [-x_max, x_max] and power-of-two S.

    With small sizes every partial sum of the forward map is an integer
    multiple of a power of two below 2**24, so fp32 arithmetic is exact in any
    order and two correct implementations must agree bit for bit.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    U = ternary(rng, (M, K), p0)
    V = ternary(rng, (K, N), p0)
    S = np.ldexp(1.0, rng.integers(-3, 1, size=K)).astype(np.float32)
    S[rng.random(K) < 0.25] *= -1.0
    X = rng.integers(-x_max, x_max + 1, size=(N, B)).astype(np.float32)
    bits = f32_to_bf16_bits(X) if x_dtype == "bf16" else None
    return Inputs(U, S, V, X, bits, x_dtype)
