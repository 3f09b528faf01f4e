"""CPU oracle for the direct transition W -> (U, S, V) (TEST INFRASTRUCTURE ONLY).

Plain numpy in fp64, written from the definitions in the section "Direct Transition Algorithm to
TSVD form" of the paper:

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


def leading_pairs(R, q: int):
    """The q singular pairs of R with the largest singular values: lists of left and right unit vectors."""
    left, _, right_t = np.linalg.svd(np.asarray(R, dtype=np.float64), full_matrices=False)
    return [left[:, j] for j in range(q)], [right_t[j, :] for j in range(q)]


def reconstruction(U, S, V) -> np.ndarray:
    """U diag(S) V as the explicit sum of its rank-one terms S_k u_k v_k^T."""
    U = np.asarray(U, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    out = np.zeros((U.shape[0], V.shape[1]))
    for k in range(U.shape[1]):
        out += S[k] * np.outer(U[:, k], V[k, :])
    return out


def transition(W, theta: float, q: int = 1, tol: float | None = None, max_rank: int | None = None, norm: str = "fro"):
    """Algorithm 2: greedy growth of the ternary factors.  Every round takes the q leading singular pairs of the
    current residual W - U diag(S) V, replaces each vector by its ternary neighbour T(., theta), appends the q
    new components and refits ALL scales by Eq. (3).  Stops when the relative error |W - U diag(S) V| / |W|
    (Frobenius norm, or the operator norm with norm="op" as in the paper's random-matrix figure) is at most tol,
    or when the rank reaches max_rank.  Returns (U int8 [M,K], S float64 [K], V int8 [K,N], errors), errors[i]
    being the relative error after round i + 1.
    """
    W = np.asarray(W, dtype=np.float64)
    M, N = W.shape
    if tol is None and max_rank is None:
        raise ValueError("an exit condition is needed")
    ordn = 2 if norm == "op" else "fro"
    wnorm = np.linalg.norm(W, ordn)
    columns, rows = [], []                     # ternary columns of U, ternary rows of V
    S = np.zeros(0)
    errors = []
    residual = W
    while True:
        lefts, rights = leading_pairs(residual, q)
        columns += [ternarize(u, theta) for u in lefts]
        rows += [ternarize(v, theta) for v in rights]
        U = np.stack(columns, axis=1)
        V = np.stack(rows, axis=0)
        S = fit_scales(U, V, W)
        residual = W - reconstruction(U, S, V)
        errors.append(float(np.linalg.norm(residual, ordn) / wnorm))
        if (tol is not None and errors[-1] <= tol) or (max_rank is not None and len(columns) >= max_rank):
            return U, S, V, errors
