"""CPU oracle for the direct transition W -> (U, S, V) (TEST INFRASTRUCTURE ONLY).

Plain numpy in fp64, following the section "Direct Transition Algorithm to TSVD form" of the
paper step by step:

  * gamma          -- Theorem 1: the bound gamma_N on the cosine that some ternary vector
                      reaches for every unit vector of dimension N.
  * ternarize      -- Algorithm 1, T(x, theta): the sparsest ternary vector whose angle to x is
                      at most theta.  By Eq. (tran_struct) only the vectors "sign(x) on the q
                      largest magnitudes, zero elsewhere" need to be examined.
  * fit_scales     -- Eq. (3): S* = [(U^T U) o (V V^T)]^+ diag(U^T W V^T), the least-squares
                      scales for fixed ternary factors.
  * transition     -- Algorithm 2: repeat { top-q singular vectors of the residual, ternarize
                      them, append, refit all scales, recompute the residual }.

Nothing here is imported by the GPU library or its binding.
"""
from __future__ import annotations

import numpy as np


def gamma(N: int) -> float:
    """Theorem 1: gamma_N = 1 / sqrt(sum_{k=1..N} (sqrt(k) - sqrt(k-1))^2)."""
    k = np.arange(1, N + 1, dtype=np.float64)
    return float(1.0 / np.sqrt(np.sum((np.sqrt(k) - np.sqrt(k - 1.0)) ** 2)))


def ternarize(x, theta: float) -> np.ndarray:
    """Algorithm 1.  Returns int8 entries in {-1, 0, +1}; raises ValueError if no ternary
    vector lies within the angle theta of x.

    The paper states the algorithm for a unit vector; the angle does not depend on the length of
    x, so x is divided by its norm here (reading: any non-zero x is accepted).
    """
    x = np.asarray(x, dtype=np.float64).ravel()
    length = np.sqrt(np.sum(x * x))
    if not length > 0.0:
        raise ValueError("the zero vector has no direction")
    # Candidate q keeps sign(x) on the q largest magnitudes: its inner product with x is the sum of
    # those magnitudes and its length sqrt(q), so the cosine of its angle to x is
    #   cos_q = (sum of the q largest |x_i|) / (sqrt(q) |x|).
    largest_first = np.sort(np.abs(x))[::-1]
    q_values = np.arange(1, x.size + 1, dtype=np.float64)
    cos_q = np.cumsum(largest_first) / (np.sqrt(q_values) * length)
    close_enough = np.nonzero(cos_q >= np.cos(theta))[0]
    if close_enough.size == 0:
        raise ValueError("no ternary vector within the angle theta")
    threshold = largest_first[close_enough[0]]            # the q-th largest magnitude of the sparsest such q
    t = np.where(np.abs(x) >= threshold, np.where(x >= 0, 1, -1), 0)      # (entries tied with it are kept)
    return t.astype(np.int8)


def fit_scales(U, V, W) -> np.ndarray:
    """Eq. (3): the S that minimises |W - U diag(S) V|_F for fixed U [M,K], V [K,N]."""
    U = np.asarray(U, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    G = (U.T @ U) * (V @ V.T)
    d = np.einsum("mk,mn,kn->k", U, W, V)                 # diag(U^T W V^T)
    return np.linalg.pinv(G) @ d


def transition(W, theta: float, q: int = 1, tol: float | None = None, max_rank: int | None = None, norm: str = "fro"):
    """Algorithm 2.  Stops when the relative error |W - U diag(S) V| / |W| (Frobenius norm, or
    the operator norm with norm="op" as in the paper's random-matrix figure) is at most tol, or
    when the rank reaches max_rank.  Returns (U int8 [M,K], S float64 [K], V int8 [K,N], errors),
    errors[i] being the relative error after iteration i + 1.
    """
    W = np.asarray(W, dtype=np.float64)
    M, N = W.shape
    if tol is None and max_rank is None:
        raise ValueError("an exit condition is needed")
    ordn = 2 if norm == "op" else "fro"
    wnorm = np.linalg.norm(W, ordn)
    U = np.zeros((M, 0), dtype=np.int8)
    V = np.zeros((0, N), dtype=np.int8)
    S = np.zeros(0)
    R = W.copy()
    errors = []
    while True:
        u, _, v = np.linalg.svd(R, full_matrices=False)
        Tu = np.stack([ternarize(u[:, j], theta) for j in range(q)], axis=1)
        Tv = np.stack([ternarize(v[j, :], theta) for j in range(q)], axis=0)
        U = np.concatenate([U, Tu], axis=1)
        V = np.concatenate([V, Tv], axis=0)
        S = fit_scales(U, V, W)
        R = W - (U.astype(np.float64) * S[None, :]) @ V.astype(np.float64)
        errors.append(float(np.linalg.norm(R, ordn) / wnorm))
        if tol is not None and errors[-1] <= tol:
            break
        if max_rank is not None and U.shape[1] >= max_rank:
            break
    return U, S, V, errors
