"""Pins for the transition oracle (Algorithm 1, Eq. 3, Algorithm 2, Theorem 1): checked against
what the paper and plain mathematics fix, never against itself or the GPU library."""
import itertools

import numpy as np
import pytest

from oracle import transition as tr

THETA = 0.576          # the paper's working threshold (section "Optimal theta in Practice")


def _cos(x, t):
    t = t.astype(np.float64)
    return float(x @ t / (np.linalg.norm(x) * np.linalg.norm(t)))


def test_gamma_crossover_at_55_56():
    """Remark after Theorem 1: gamma_N stays at or above cos(pi/4) exactly up to N = 55."""
    assert tr.gamma(1) == 1.0
    assert abs(tr.gamma(2) - 1.0 / np.sqrt(1.0 + (np.sqrt(2.0) - 1.0) ** 2)) < 1e-15
    assert tr.gamma(55) >= np.cos(np.pi / 4) > tr.gamma(56)
    g = [tr.gamma(n) for n in range(1, 300)]
    assert all(a > b for a, b in zip(g, g[1:]))                    # decreasing, slowly
    assert tr.gamma(299) > 0.6


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8])
def test_ternarize_is_the_sparsest_ternary_vector_within_theta(n):
    """Brute force over all 3^n - 1 ternary vectors (Eq. (tran_struct) says only n of them matter):
    the result has the fewest non-zeros among the vectors within the angle, and among the vectors
    with that many non-zeros none is closer to x."""
    rng = np.random.default_rng(100 + n)
    every = [np.array(t, dtype=np.int8) for t in itertools.product((-1, 0, 1), repeat=n) if any(t)]
    for trial in range(40):
        x = rng.laplace(size=n)
        theta = rng.uniform(0.2, 1.2)
        within = [t for t in every if _cos(x, t) >= np.cos(theta) - 1e-12]
        if not within:
            with pytest.raises(ValueError):
                tr.ternarize(x, theta)
            continue
        fewest = min(np.count_nonzero(t) for t in within)
        got = tr.ternarize(x, theta)
        assert set(np.unique(got)) <= {-1, 0, 1}
        assert np.count_nonzero(got) == fewest
        assert _cos(x, got) >= np.cos(theta) - 1e-12
        best = max(_cos(x, t) for t in every if np.count_nonzero(t) == fewest)
        assert abs(_cos(x, got) - best) < 1e-12


def test_ternarize_hand_cases_and_scale_invariance():
    # |x| = sqrt(0.62): cos_1 = 0.6/|x| = 0.762, cos_2 = 1.1/(sqrt(2)|x|) = 0.988
    x = np.array([0.6, -0.5, 0.1, 0.0])
    assert np.array_equal(tr.ternarize(x, 0.75), [1, 0, 0, 0])               # cos 0.75 = 0.732 <= cos_1
    assert np.array_equal(tr.ternarize(x, 0.5), [1, -1, 0, 0])               # cos 0.5 = 0.878: needs q = 2
    with pytest.raises(ValueError):
        tr.ternarize(x, 0.1)                                                 # cos 0.1 = 0.995 is never reached
    assert np.array_equal(tr.ternarize(7.5 * x, 0.5), tr.ternarize(x, 0.5))
    assert np.array_equal(tr.ternarize(-x, 0.5), -tr.ternarize(x, 0.5))
    assert np.array_equal(tr.ternarize(np.array([1.0, 1.0, 1.0, 1.0]), 0.1), [1, 1, 1, 1])
    with pytest.raises(ValueError):
        tr.ternarize(np.zeros(4), 0.5)


def test_existence_bound_of_theorem_1():
    """Every unit vector has a ternary vector with cosine >= gamma_N; the vector whose prefix sums
    grow like sqrt(k) attains the bound, so no better bound exists."""
    rng = np.random.default_rng(7)
    for N in (3, 10, 55, 200):
        g = tr.gamma(N)
        for trial in range(50):
            x = rng.standard_normal(N) * rng.uniform(0.1, 3.0, N)
            t = tr.ternarize(x, np.arccos(g) + 1e-9)                  # never raises
            assert _cos(x, t) >= g - 1e-9
        k = np.arange(1, N + 1, dtype=np.float64)
        a = g * (np.sqrt(k) - np.sqrt(k - 1.0))                       # |a| = 1, every cos_q equals gamma_N
        assert abs(np.linalg.norm(a) - 1.0) < 1e-12
        best = max(_cos(a, tr.ternarize(a, th)) for th in np.linspace(np.arccos(g) + 1e-9, 1.5, 40))
        assert abs(best - g) < 1e-9
        with pytest.raises(ValueError):
            tr.ternarize(a, np.arccos(g) - 1e-6)
    # below the crossover a threshold of pi/4 always works
    for trial in range(200):
        tr.ternarize(rng.standard_normal(55), np.pi / 4)


def test_fit_scales_is_the_least_squares_solution():
    """Eq. (3) against the same problem written as an ordinary least-squares system
    vec(W) ~ A s, A[:, k] = vec(u_k v_k), solved by a library routine; also with a duplicated
    component (singular Gram matrix: the pseudo-inverse picks the minimum-norm solution)."""
    rng = np.random.default_rng(11)
    M, N, K = 9, 7, 5
    U = rng.integers(-1, 2, size=(M, K)).astype(np.int8)
    V = rng.integers(-1, 2, size=(K, N)).astype(np.int8)
    W = rng.standard_normal((M, N))
    for dup in (False, True):
        if dup:
            U[:, 4], V[4, :] = U[:, 1], V[1, :]
        A = np.stack([np.outer(U[:, k], V[k, :]).ravel() for k in range(K)], axis=1).astype(np.float64)
        want = np.linalg.lstsq(A, W.ravel(), rcond=None)[0]
        got = tr.fit_scales(U, V, W)
        assert np.allclose(got, want, atol=1e-10)
        # optimality: the residual is orthogonal to every component
        R = W - (U * got[None, :]) @ V.astype(np.float64)
        assert np.allclose(A.T @ R.ravel(), 0.0, atol=1e-9)
    # an exactly representable W is recovered
    S0 = rng.standard_normal(K)
    U[:, 4] = rng.integers(-1, 2, size=M)
    W0 = (U * S0[None, :]) @ V.astype(np.float64)
    assert np.allclose((U * tr.fit_scales(U, V, W0)[None, :]) @ V.astype(np.float64), W0, atol=1e-10)


def test_one_iteration_contracts_as_theorem_2_states():
    """Theorem 2 (q = 1): after one component fitted to the residual alone,
    |R - T_u s T_v|_F^2 <= sin^2(2 theta) sigma_0^2 + |sigma_1..|^2 <= (1 - cos^2(2 theta)/min(M,N)) |R|_F^2."""
    rng = np.random.default_rng(21)
    # (dimensions large enough that a vector within theta = 0.576 exists: for Gaussian-like singular
    # vectors the best cosine is about 0.90 in high dimension and scatters below 0.84 at 40 to 50)
    for (M, N) in ((96, 80), (128, 96), (200, 120)):
        R = rng.laplace(size=(M, N))
        u, sig, v = np.linalg.svd(R, full_matrices=False)
        Tu = tr.ternarize(u[:, 0], THETA).astype(np.float64)
        Tv = tr.ternarize(v[0, :], THETA).astype(np.float64)
        s = float(Tu @ R @ Tv / ((Tu @ Tu) * (Tv @ Tv)))              # the least-squares scale of one component
        left = np.linalg.norm(R - s * np.outer(Tu, Tv)) ** 2
        mid = np.sin(2 * THETA) ** 2 * sig[0] ** 2 + np.sum(sig[1:] ** 2)
        right = (1.0 - np.cos(2 * THETA) ** 2 / min(M, N)) * np.linalg.norm(R) ** 2
        assert left <= mid * (1 + 1e-12) <= right * (1 + 1e-12)


def test_transition_converges_and_keeps_the_papers_sparsity():
    """Algorithm 2 on a Laplace matrix (the paper's random-matrix test, here [128, 64] to stay
    quick): the error never increases (all scales are refitted), the tolerance is reached, and at
    theta = 0.576 the non-zero rate of U and V is about 0.29."""
    rng = np.random.default_rng(3)
    W = rng.laplace(size=(128, 64))
    U, S, V, errs = tr.transition(W, THETA, tol=0.07)
    assert U.shape[1] == V.shape[0] == S.shape[0] == len(errs)
    assert all(b <= a + 1e-12 for a, b in zip(errs, errs[1:]))
    assert errs[-1] <= 0.07 < errs[-2]
    R = W - (U * S[None, :]) @ V.astype(np.float64)
    assert abs(np.linalg.norm(R) / np.linalg.norm(W) - errs[-1]) < 1e-12
    r = (np.count_nonzero(U) + np.count_nonzero(V)) / (U.size + V.size)
    assert 0.25 < r < 0.33
    # the operator-norm variant of the exit test and a rank limit
    U2, S2, V2, e2 = tr.transition(W, THETA, max_rank=10, norm="op")
    assert U2.shape == (128, 10) and len(e2) == 10 and e2[-1] < 1.0
    assert np.array_equal(U2, U[:, :10]) and np.array_equal(V2, V[:10, :])     # the same greedy path


def test_sparsity_at_the_papers_size():
    """[512, 256] Laplace, theta = 0.576: r is about 0.29 (first 24 components)."""
    W = np.random.default_rng(4).laplace(size=(512, 256))
    U, S, V, errs = tr.transition(W, THETA, max_rank=24)
    r = (np.count_nonzero(U) + np.count_nonzero(V)) / (U.size + V.size)
    assert 0.26 < r < 0.32


def test_transition_with_several_components_per_round():
    """q > 1 (the top-q singular pairs of one residual per round).  On an exactly ternary-factorisable matrix
    W = sum_k s_k a_k b_k^T with orthogonal ternary a_k (disjoint supports) and b_k, the singular vectors ARE the
    normalised a_k, b_k, so q = 3 must recover all three components in ONE round with error 0 and S = s; and a
    round with q = 2 must equal two rounds' worth of components while refitting all scales (Eq. 3)."""
    a = np.zeros((12, 3)); b = np.zeros((3, 10))
    a[0:4, 0] = [1, -1, 1, 1]; a[4:8, 1] = [1, 1, -1, 1]; a[8:12, 2] = [-1, 1, 1, 1]
    b[0, 0:3] = [1, 1, -1]; b[1, 3:6] = [1, -1, 1]; b[2, 6:10] = [1, 1, 1, -1]
    s = np.array([5.0, 3.0, 2.0])
    W = (a * s[None, :]) @ b
    U, S, V, errs = tr.transition(W, 0.3, q=3, max_rank=3)
    assert U.shape == (12, 3) and len(errs) == 1 and errs[0] < 1e-12
    for k in range(3):
        sign = 1 if np.array_equal(U[:, k], a[:, k]) else -1
        assert np.array_equal(sign * U[:, k], a[:, k]) and np.array_equal(sign * V[k, :], b[k, :])
    assert np.allclose(S, s, rtol=1e-12)
    # q = 2 on a generic matrix: 2 components per round, every round's scales are the least-squares optimum
    Wg = np.random.default_rng(7).laplace(size=(40, 24))        # (a seed at which every leading vector has a ternary neighbour within theta)
    U2, S2, V2, e2 = tr.transition(Wg, 0.576, q=2, max_rank=8)
    assert U2.shape == (40, 8) and len(e2) == 4 and all(y <= x + 1e-12 for x, y in zip(e2, e2[1:]))
    best = np.linalg.lstsq(np.stack([np.outer(U2[:, k], V2[k, :]).ravel() for k in range(8)], axis=1), Wg.ravel(), rcond=None)[0]
    assert np.allclose(S2, best, rtol=1e-9, atol=1e-12)
    assert np.allclose(tr.reconstruction(U2, S2, V2), (U2 * S2[None, :]) @ V2.astype(np.float64), atol=1e-12)
    # the first round of q = 2 takes the two leading pairs of W itself
    lefts, rights = tr.leading_pairs(Wg, 2)
    for k in range(2):
        assert np.array_equal(U2[:, k], tr.ternarize(lefts[k], 0.576)) and np.array_equal(V2[k, :], tr.ternarize(rights[k], 0.576))
