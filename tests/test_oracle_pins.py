"""Pins for the CPU oracle: it is checked against what the paper and plain
mathematics fix, never against itself or the GPU library."""
import itertools
import os

import numpy as np
import pytest

import oracle
import workloads


def _read_fixture(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":")
            out[key.strip()] = np.array([float(v) for v in vals.split()])
    return out


def _dense(U, S, V):
    """W' = U diag(S) V formed explicitly in fp64 with library matmuls."""
    return (U.astype(np.float64) * S.astype(np.float64)[None, :]) @ V.astype(np.float64)


def _rand(M, N, K, B, seed, p0=0.5, x_dtype="f32"):
    return workloads.make_inputs(M, N, K, B, p0, 0.02, x_dtype, seed)


# ---- P3: worked example ------------------------------------------------------------
def test_hand_example(golden_dir):
    g = _read_fixture(os.path.join(golden_dir, "hand_2x2.txt"))
    U = g["U"].reshape(2, 2).astype(np.int8)
    V = g["V"].reshape(2, 2).astype(np.int8)
    y = oracle.forward(U, g["S"].astype(np.float32), V, g["x"])
    assert np.array_equal(y.ravel(), g["y"])
    assert np.array_equal(_dense(U, g["S"], V), g["W"].reshape(2, 2))


# ---- P5: Winograd F(2,3) is a lossless TSVD of the unfolded convolution ----------------
def test_winograd_f23(golden_dir):
    g = _read_fixture(os.path.join(golden_dir, "winograd_f23.txt"))
    U = g["U"].reshape(2, 4).astype(np.int8)
    V = g["V"].reshape(4, 4).astype(np.int8)
    w = g["w"]
    S = (g["G"].reshape(4, 3) @ w).astype(np.float32)     # exact: halves of short decimals
    y = oracle.forward(U, S, V, g["x"])
    assert np.allclose(y.ravel(), g["y"], rtol=0, atol=1e-12)
    # and for arbitrary taps/inputs against the unfolded cyclic matrix of the paper
    rng = np.random.default_rng(5)
    for _ in range(20):
        w = np.round(rng.standard_normal(3) * 8) / 8          # exactly representable
        x = rng.standard_normal(4)
        Wc = np.array([[w[0], w[1], w[2], 0.0], [0.0, w[0], w[1], w[2]]])
        S = (g["G"].reshape(4, 3) @ w).astype(np.float32)
        y = oracle.forward(U, S, V, x)
        assert np.allclose(y.ravel(), Wc @ x, rtol=0, atol=1e-12)


# ---- P1: the dense identity --------------------------------------------------------
@pytest.mark.parametrize("M,N,K,B", [(4, 4, 4, 1), (8, 8, 8, 3), (3, 5, 7, 2), (37, 29, 61, 5),
                                     (256, 256, 512, 1), (64, 48, 200, 17)])
def test_dense_identity(M, N, K, B):
    i = _rand(M, N, K, B, seed=100 + M + N + K + B)
    y = oracle.forward(i.U, i.S, i.V, i.X)
    ref = _dense(i.U, i.S, i.V) @ i.X.astype(np.float64)
    assert y.shape == (M, B)
    assert np.max(np.abs(y - ref)) <= 1e-12 * max(1.0, np.max(np.abs(ref)))


def test_dense_identity_named_workloads():
    i = workloads.make_workload("tiny")
    y = oracle.forward(i.U, i.S, i.V, i.X)
    ref = _dense(i.U, i.S, i.V) @ i.X.astype(np.float64)
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))
    i = workloads.make_workload("bert_ffn_in", B=8)
    y = oracle.forward(i.U, i.S, i.V, i.X)
    ref = _dense(i.U, i.S, i.V) @ i.X.astype(np.float64)
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))


# ---- P2: brute force ------------------------------------------------------------------
def _brute(U, S, V, X):
    M, K = U.shape
    N, B = X.shape
    Y = [[0.0] * B for _ in range(M)]
    for b in range(B):
        for m in range(M):
            acc = 0.0
            for k in range(K):
                inner = 0.0
                for n in range(N):
                    inner += int(V[k][n]) * float(X[n][b])
                acc += int(U[m][k]) * (float(S[k]) * inner)
            Y[m][b] = acc
    return np.array(Y)


@pytest.mark.parametrize("M,N,K,B", [(4, 4, 4, 1), (8, 8, 8, 2), (3, 5, 7, 3), (1, 1, 1, 1)])
def test_brute_force(M, N, K, B):
    i = _rand(M, N, K, B, seed=7 * M + N)
    y = oracle.forward(i.U, i.S, i.V, i.X)
    assert np.allclose(y, _brute(i.U, i.S, i.V, i.X), rtol=1e-13, atol=1e-15)


def test_all_ternary_rows_of_length_four():
    x = np.array([0.5, -1.25, 3.0, 7.0])
    U = np.array([[1]], dtype=np.int8)
    S = np.array([1.0], dtype=np.float32)
    for row in itertools.product((-1, 0, 1), repeat=4):
        V = np.array([row], dtype=np.int8)
        y = oracle.forward(U, S, V, x)
        assert y[0, 0] == sum(c * v for c, v in zip(row, x))


# ---- P4: special cases that reduce to library routines ---------------------------------
def test_special_cases():
    rng = np.random.default_rng(3)
    K = 9
    eye = np.eye(K, dtype=np.int8)
    S = rng.standard_normal(K).astype(np.float32)
    x = rng.standard_normal((K, 4))
    U = workloads.ternary(rng, (6, K), 0.4)
    V = workloads.ternary(rng, (K, 5), 0.4)
    x5 = rng.standard_normal((5, 4))
    # V = I: y = U (S*x);  U = I: y = S*(V x)
    assert np.allclose(oracle.forward(U, S, eye, x), U.astype(float) @ (S[:, None].astype(float) * x), atol=1e-13)
    assert np.allclose(oracle.forward(eye, S, V, x5), S[:, None].astype(float) * (V.astype(float) @ x5), atol=1e-13)
    # U = V = I, S = 1: identity map;  S = 0: zero map
    assert np.array_equal(oracle.forward(eye, np.ones(K, np.float32), eye, x), x)
    assert np.array_equal(oracle.forward(U, np.zeros(K, np.float32), V, x5), np.zeros((6, 4)))
    # rank one: y = u * s * (v . x)
    u = workloads.ternary(rng, (6, 1), 0.3)
    v = workloads.ternary(rng, (1, 5), 0.3)
    s = np.array([1.75], dtype=np.float32)
    assert np.allclose(oracle.forward(u, s, v, x5), u.astype(float) * 1.75 * (v.astype(float) @ x5), atol=1e-13)


# ---- P6: invariants ------------------------------------------------------------------------
def test_invariants():
    i = _rand(20, 14, 33, 3, seed=11)
    U, S, V, X = i.U, i.S, i.V, i.X.astype(np.float64)
    y = oracle.forward(U, S, V, X)
    # linear in x and in S (powers of two keep the scaling exact)
    assert np.array_equal(oracle.forward(U, S, V, 4.0 * X), 4.0 * y)
    assert np.array_equal(oracle.forward(U, (S * 0.5).astype(np.float32), V, X), 0.5 * y)
    X2 = np.random.default_rng(1).standard_normal(X.shape)
    assert np.allclose(oracle.forward(U, S, V, X + X2), y + oracle.forward(U, S, V, X2), atol=1e-12)
    # flipping the sign of column k of U and of row k of V changes nothing
    U2, V2 = U.copy(), V.copy()
    U2[:, 5] *= -1
    V2[5, :] *= -1
    assert np.array_equal(oracle.forward(U2, S, V2, X), y)
    # flipping only one of them flips that component: differs unless the component is 0
    assert not np.array_equal(oracle.forward(U2, S, V, X), y)
    # permuting the rank index of (U columns, S, V rows) changes only the summation order
    p = np.random.default_rng(2).permutation(33)
    assert np.allclose(oracle.forward(U[:, p], S[p], V[p, :], X), y, rtol=0, atol=1e-13)
    # transposed operands must NOT give the same map
    sq = _rand(12, 12, 12, 2, seed=13)
    a = oracle.forward(sq.U, sq.S, sq.V, sq.X)
    assert not np.allclose(a, oracle.forward(sq.U.T.copy(), sq.S, sq.V, sq.X))
    assert not np.allclose(a, oracle.forward(sq.U, sq.S, sq.V.T.copy(), sq.X))
    assert not np.allclose(a, oracle.forward(sq.V, sq.S, sq.U, sq.X))      # order of the factors


def test_bit_plane_identity():
    """U = U+ - U-, V = V+ - V- with binary planes (section "Connection with BNN")."""
    i = _rand(10, 12, 15, 2, seed=17)
    Up, Um = (i.U > 0).astype(np.int8), (i.U < 0).astype(np.int8)
    Vp, Vm = (i.V > 0).astype(np.int8), (i.V < 0).astype(np.int8)
    X = i.X.astype(np.float64)
    y = oracle.forward(i.U, i.S, i.V, X)
    parts = (oracle.forward(Up, i.S, Vp, X) - oracle.forward(Up, i.S, Vm, X)
             - oracle.forward(Um, i.S, Vp, X) + oracle.forward(Um, i.S, Vm, X))
    assert np.allclose(y, parts, rtol=0, atol=1e-13)
    # one 1 in U+ or U- per non-zero of U: equal addition counts
    assert Up.sum() + Um.sum() == np.count_nonzero(i.U)


def test_rejects_non_ternary():
    U = np.array([[2]], dtype=np.int8)
    with pytest.raises(ValueError):
        oracle.forward(U, np.ones(1, np.float32), np.ones((1, 1), np.int8), np.ones(1))
    with pytest.raises(ValueError):
        oracle.forward(np.ones((1, 1), np.int8), np.ones(1, np.float32), -2 * np.ones((1, 1), np.int8), np.ones(1))


# ---- P7: exact-integer instances ---------------------------------------------------------
@pytest.mark.parametrize("x_dtype", ["f32", "bf16"])
def test_integer_instances_are_exact(x_dtype):
    i = workloads.make_integer_inputs(48, 40, 72, 5, 0.5, x_dtype, seed=23)
    y = oracle.forward(i.U, i.S, i.V, i.X)
    ref = _dense(i.U, i.S, i.V) @ i.X.astype(np.float64)
    assert np.array_equal(y, ref)                       # all sums are exact dyadic rationals
    assert np.array_equal(y, y.astype(np.float32))      # and fit fp32


# ---- B = 1 row-parallel entry agrees with the token-parallel one ------------------------
def test_vector_entry_matches_batched_entry():
    i = _rand(33, 21, 40, 1, seed=29)
    y1 = oracle.forward(i.U, i.S, i.V, i.X)                                  # B = 1 entry
    y2 = oracle.forward(i.U, i.S, i.V, np.concatenate([i.X, i.X], axis=1))   # batched entry
    assert np.array_equal(y1[:, 0], y2[:, 0]) and np.array_equal(y1[:, 0], y2[:, 1])


def test_forward_columns():
    i = _rand(9, 8, 11, 6, seed=31)
    full = oracle.forward(i.U, i.S, i.V, i.X)
    sub = oracle.forward_columns(i.U, i.S, i.V, i.X, [5, 0, 3])
    assert np.array_equal(sub, full[:, [5, 0, 3]])


# ---- P8: statistics of the generators ------------------------------------------------
def test_output_statistics():
    w = workloads.WORKLOADS["bert_ffn_in"]
    i = workloads.make_workload("bert_ffn_in", B=16)
    y = oracle.forward(i.U, i.S, i.V, i.X)
    r = 1.0 - w.p0
    sigma = np.sqrt(r * r * w.K * w.N * (w.s_scale ** 2))   # E[S^2] = scale^2, Var x = 1
    assert abs(y.mean()) < 0.05 * sigma
    assert 0.9 * sigma < y.std() < 1.1 * sigma


# ---- operation counts (supplement Tables S1, S2; Eq. 2) ---------------------------------
def test_op_counts_and_cost_model():
    i = _rand(30, 20, 50, 1, seed=37, p0=0.7)
    c = oracle.op_counts(i.U, i.V)
    assert c["mults"] == 50
    assert c["adds"] == int((i.U != 0).sum() + (i.V != 0).sum())
    assert abs(c["r"] - 0.3) < 0.05
    # at the critical rank the two costs balance (Eq. 2), for several bit widths
    for d in (4, 8, 16, 32):
        Kc = oracle.critical_rank(3072, 768, 0.29, d)
        assert abs(oracle.acceleration(3072, 768, Kc, 0.29, d) - 1.0) < 1e-12
    # vanilla-SVD limit of the preliminaries: r = 1 and Mul = Add (d = 3) gives K = MN/(M+N)
    # up to the K multiplications of diag(S)
    assert abs(oracle.critical_rank(100, 50, 1.0, 3) - 2 * 100 * 50 / (1 + 150)) < 1e-9
    # numbers implied by the paper's cost model at the BERT-like shape, r = 0.5
    assert abs(oracle.acceleration(3072, 768, 1536, 0.5, 32) - 24.4) < 0.05


# ---- the layer form: bias, token-major activations, bf16 output -----------------------------
def test_bf16_rounding_against_known_values_and_the_bit_trick():
    """round_to_bf16 (from the definition of the format) against hand-worked values (ties to
    even, carry into the exponent, subnormals) and against the independent integer bit trick
    of the input generators on fp32-representable values."""
    cases = {
        1.0: 1.0,
        1.0 + 2.0 ** -8: 1.0,                     # tie, even significand below
        1.0 + 3 * 2.0 ** -8: 1.0 + 2.0 ** -6,     # tie, even significand above (1.015625)
        1.0 + 2.0 ** -8 + 2.0 ** -20: 1.0 + 2.0 ** -7,
        1.99609375 + 2.0 ** -9 * 1.5: 2.0,        # rounds up across the binade
        -3.1415926: -3.140625,
        0.0: 0.0,
        2.0 ** -133: 2.0 ** -133,                 # smallest subnormal
        2.0 ** -134 * 1.5: 2.0 ** -133,
        2.0 ** -134: 0.0,                         # tie to even (zero)
    }
    for v, want in cases.items():
        assert oracle.round_to_bf16(np.array([v]))[0] == want, v
    rng = np.random.default_rng(5)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-30, 30, 20000))).astype(np.float32)
    want = workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(a)).astype(np.float64)
    assert np.array_equal(oracle.round_to_bf16(a.astype(np.float64)), want)


def test_layer_form_bias_layout_and_output_type():
    i = _rand(37, 29, 61, 5, seed=12)
    U, S, V, X = i.U, i.S, i.V, i.X
    base = oracle.forward(U, S, V, X)
    bias = np.random.default_rng(13).standard_normal(37).astype(np.float32)
    # bias: the dense product with a column of ones appended (y = [W b] [x; 1]) is the same map
    W1 = np.concatenate([_dense(U, S, V), bias.astype(np.float64)[:, None]], axis=1)
    X1 = np.concatenate([X.astype(np.float64), np.ones((1, X.shape[1]))], axis=0)
    got = oracle.forward_layer(U, S, V, X, bias=bias)
    assert np.allclose(got, W1 @ X1, rtol=1e-12, atol=1e-12)
    assert not np.allclose(got, base)                                    # the bias is not dropped
    assert np.array_equal(oracle.forward_layer(U * 0, S, V, X, bias=bias), np.repeat(bias.astype(np.float64)[:, None], 5, 1))
    # token-major activations are the transposed matrix; a non-square X makes a mix-up a shape error
    assert np.array_equal(oracle.forward_layer(U, S, V, np.ascontiguousarray(X.T), x_layout="token_major"), base)
    with pytest.raises(ValueError):
        oracle.forward_layer(U, S, V, X, x_layout="token_major")
    # bf16 output: within half a unit in the last place (at most 2^-8 relative: 8 significant bits),
    # exactly representable, idempotent
    yb = oracle.forward_layer(U, S, V, X, bias=bias, y_dtype="bf16")
    assert np.all(np.abs(yb - got) <= np.abs(got) * 2.0 ** -8)
    assert np.max(np.abs(yb - got) / np.abs(got)) > 2.0 ** -11           # and it does round
    assert np.array_equal(oracle.round_to_bf16(yb), yb)
    assert np.array_equal(workloads.bf16_bits_to_f32(workloads.f32_to_bf16_bits(yb.astype(np.float32))).astype(np.float64), yb)


def test_layer_form_token_major_output_is_one_row_per_token():
    """y_layout "token_major": row b of the result is the dense layer applied to token b alone (library matmul on
    the explicit W' = U diag(S) V, one token at a time), for both layouts of x; a transposed bias or a swapped
    index would fail on this non-square instance."""
    rng = np.random.default_rng(31)
    M, N, K, B = 7, 5, 9, 4
    U = rng.integers(-1, 2, size=(M, K)).astype(np.int8)
    V = rng.integers(-1, 2, size=(K, N)).astype(np.int8)
    S = rng.standard_normal(K).astype(np.float32)
    X = rng.standard_normal((N, B)).astype(np.float32)
    bias = rng.standard_normal(M).astype(np.float32)
    W = (U.astype(np.float64) * S.astype(np.float64)[None, :]) @ V.astype(np.float64)
    want = np.stack([W @ X[:, b].astype(np.float64) + bias.astype(np.float64) for b in range(B)])     # [B, M]
    got = oracle.forward_layer(U, S, V, X, bias=bias, y_layout="token_major")
    assert got.shape == (B, M) and np.allclose(got, want, rtol=1e-12, atol=1e-12)
    got2 = oracle.forward_layer(U, S, V, np.ascontiguousarray(X.T), bias=bias, x_layout="token_major", y_layout="token_major")
    assert np.array_equal(got, got2)
    assert np.array_equal(got, oracle.forward_layer(U, S, V, X, bias=bias).T)
    with pytest.raises(ValueError):
        oracle.forward_layer(U, S, V, X, y_layout="rows")
