"""Pins for the CPU checker: it is compared with closed forms, invariants,
textbook special cases, library witnesses and brute force on tiny inputs, never
with itself.  The paper prints no worked numeric example for any operator, so
none of the pins is a value taken from it.  Runs without a GPU."""
import itertools
import math

import numpy as np
import pytest

from oracle import compare, ref

rng = np.random.default_rng(20250610)


def f32(a):
    return np.asarray(a, dtype=np.float32)


# ------------------------------------------------------------------ matmul
def test_gemm_identity_weight_is_copy_plus_bias():
    X = f32(rng.uniform(-1, 1, (7, 9)))
    b = f32(rng.uniform(-1, 1, 9))
    Z = ref.gemm_bias(X, np.eye(9, dtype=np.float32), b)
    assert np.array_equal(Z, X.astype(np.float64) + b.astype(np.float64))


def test_gemm_ones_weight_gives_row_sums():
    X = f32(rng.uniform(-1, 1, (5, 33)))
    Z = ref.gemm_bias(X, np.ones((33, 4), np.float32))
    want = X.astype(np.float64).sum(axis=1, keepdims=True) * np.ones((1, 4))
    assert np.allclose(Z, want, rtol=0, atol=1e-13)


def test_gemm_not_transposed_and_brute_force():
    # asymmetric shapes and a non-symmetric W: a transposed operand or swapped
    # index cannot reproduce this
    M, K, N = 3, 5, 7
    X = f32(rng.normal(size=(M, K)))
    W = f32(rng.normal(size=(K, N)))
    b = f32(rng.normal(size=N))
    Z, Dn = ref.gemm_bias(X, W, b, want_norm=True)
    for m, n in itertools.product(range(M), range(N)):
        acc, mag = float(b[n]), abs(float(b[n]))
        for k in range(K):
            acc += float(X[m, k]) * float(W[k, n])
            mag += abs(float(X[m, k])) * abs(float(W[k, n]))
        assert Z[m, n] == pytest.approx(acc, rel=1e-14, abs=1e-15)
        assert Dn[m, n] == pytest.approx(mag, rel=1e-14)


def test_gemm_matches_fp64_library_matmul():
    X = f32(rng.uniform(-1, 1, (64, 256)))
    W = f32(rng.uniform(-1 / 16, 1 / 16, (256, 256)))
    b = f32(rng.uniform(-0.1, 0.1, 256))
    Z, Dn = ref.gemm_bias(X, W, b, want_norm=True)
    want = X.astype(np.float64) @ W.astype(np.float64) + b.astype(np.float64)
    assert np.max(np.abs(Z - want)) <= 1e-12 * np.max(Dn)
    wantD = np.abs(X).astype(np.float64) @ np.abs(W).astype(np.float64) + np.abs(b)
    assert np.allclose(Dn, wantD, rtol=1e-12)


def test_gemm_linear_in_x():
    X1 = f32(rng.normal(size=(4, 6)))
    W = f32(rng.normal(size=(6, 5)))
    Xs = f32(X1 * 2)  # exact in fp32
    assert np.allclose(ref.gemm_bias(Xs, W), 2 * ref.gemm_bias(X1, W), rtol=1e-14)
    # small integers add exactly in fp32, so additivity in X is exact too
    A = f32(rng.integers(-8, 9, (4, 6)))
    Bm = f32(rng.integers(-8, 9, (4, 6)))
    Wi = f32(rng.integers(-8, 9, (6, 5)))
    assert np.array_equal(ref.gemm_bias(A + Bm, Wi), ref.gemm_bias(A, Wi) + ref.gemm_bias(Bm, Wi))


# ---------------------------------------------------------------- relu etc.
def test_relu_pointwise():
    z = np.array([-2.0, -0.0, 0.0, 1e-300, 3.5, -1e-300])
    assert np.array_equal(ref.relu(z), np.array([0.0, 0.0, 0.0, 1e-300, 3.5, 0.0]))


def test_affine_scale_zero_gives_relu_shift_plus_r():
    X = f32(rng.normal(size=(2, 3, 4, 5)))
    R = f32(rng.normal(size=(2, 3, 4, 5)))
    shift = f32([-0.5, 0.25, 1.0])
    T = ref.affine_relu_residual(X, np.zeros(3, np.float32), shift, R)
    want = np.maximum(shift.astype(np.float64), 0)[None, :, None, None] + R.astype(np.float64)
    assert np.array_equal(T, want)


def test_affine_identity_on_nonnegative_input():
    X = f32(np.abs(rng.normal(size=(2, 3, 4, 5))))
    R = f32(rng.normal(size=(2, 3, 4, 5)))
    T = ref.affine_relu_residual(X, np.ones(3, np.float32), np.zeros(3, np.float32), R)
    assert np.array_equal(T, X.astype(np.float64) + R.astype(np.float64))


def test_affine_residual_is_added_after_relu_and_channel_axis():
    # X = -1 everywhere, scale = 1, shift = 0: relu kills the affine part, so
    # T = R exactly (a residual added before the relu would give relu(R-1)).
    X = -np.ones((2, 3, 2, 2), np.float32)
    R = f32(rng.normal(size=(2, 3, 2, 2)))
    T = ref.affine_relu_residual(X, np.ones(3, np.float32), np.zeros(3, np.float32), R)
    assert np.array_equal(T, R.astype(np.float64))
    # per-channel parameters index axis 1, not axis 0 or the plane index
    X = np.ones((2, 3, 2, 2), np.float32)
    scale = f32([1, 2, 4])
    shift = f32([0.5, 0.25, 0.125])
    T = ref.affine_relu_residual(X, scale, shift, np.zeros_like(X))
    for n, c in itertools.product(range(2), range(3)):
        assert np.all(T[n, c] == float(scale[c]) + float(shift[c]))


def test_affine_brute_force():
    X = f32(rng.normal(size=(2, 2, 3, 3)))
    R = f32(rng.normal(size=(2, 2, 3, 3)))
    sc, sh = f32([0.7, -1.3]), f32([0.2, 0.4])
    T = ref.affine_relu_residual(X, sc, sh, R)
    for n, c, h, w in itertools.product(range(2), range(2), range(3), range(3)):
        v = float(X[n, c, h, w]) * float(sc[c]) + float(sh[c])
        assert T[n, c, h, w] == pytest.approx(max(v, 0.0) + float(R[n, c, h, w]), rel=1e-15)


# ------------------------------------------------------------------ softmax
def test_softmax_invariants():
    Z = rng.normal(size=(11, 37)) * 3
    Y = ref.softmax_rows(Z)
    assert np.all(np.abs(Y.sum(axis=1) - 1) <= 1e-14 * 37)
    assert np.all(Y > 0) and np.all(Y <= 1)
    # shift invariance
    assert np.allclose(ref.softmax_rows(Z + 5.0), Y, rtol=1e-12)
    # monotone: order of outputs = order of logits
    assert np.array_equal(np.argsort(Z, axis=1), np.argsort(Y, axis=1))
    # ratio identity y_a / y_b = exp(z_a - z_b)
    assert np.allclose(Y[:, 0] / Y[:, 1], np.exp(Z[:, 0] - Z[:, 1]), rtol=1e-12)


def test_softmax_constant_and_onehot_and_is_rowwise():
    Y = ref.softmax_rows(np.full((3, 8), 2.5))
    assert np.allclose(Y, 1 / 8, rtol=1e-15)
    Z = np.zeros((2, 6))
    Z[0, 4] = 800.0  # would overflow exp() without the max subtraction
    Z[1, 1] = 800.0
    Y = ref.softmax_rows(Z)
    want = np.zeros((2, 6))
    want[0, 4] = want[1, 1] = 1.0
    assert np.allclose(Y, want, atol=1e-300)
    # two-element closed form: softmax([a, b]) = [sigmoid(a-b), sigmoid(b-a)]
    Y = ref.softmax_rows(np.array([[0.3, -1.1]]))
    assert Y[0, 0] == pytest.approx(1 / (1 + math.exp(-1.4)), rel=1e-15)


# ----------------------------------------------------------------- avg pool
def test_avgpool_closed_forms():
    T = np.full((2, 3, 56, 56), 1.25)
    assert np.array_equal(ref.avgpool_hw(T), np.full((2, 3), 1.25))
    ramp = np.arange(3136, dtype=np.float64).reshape(1, 1, 56, 56)
    assert ref.avgpool_hw(ramp)[0, 0] == 1567.5
    A = rng.normal(size=(2, 2, 5, 7))
    B = rng.normal(size=(2, 2, 5, 7))
    assert np.allclose(ref.avgpool_hw(A + B), ref.avgpool_hw(A) + ref.avgpool_hw(B), rtol=1e-13)
    # each plane separately: plane p filled with p
    T = np.arange(6, dtype=np.float64).reshape(2, 3, 1, 1) * np.ones((2, 3, 4, 4))
    assert np.array_equal(ref.avgpool_hw(T), np.arange(6.0).reshape(2, 3))


def test_chain2_matches_numpy_definition():
    X = f32(rng.normal(size=(2, 4, 6, 6)))
    R = f32(rng.normal(size=(2, 4, 6, 6)))
    sc, sh = f32(rng.normal(1, 0.1, 4)), f32(rng.normal(0, 0.1, 4))
    want = (np.maximum(X.astype(np.float64) * sc[None, :, None, None].astype(np.float64)
                       + sh[None, :, None, None].astype(np.float64), 0) + R).mean(axis=(2, 3))
    assert np.allclose(ref.chain2(X, sc, sh, R), want, rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- layernorm
def test_layernorm_mean_zero_and_variance_closed_form():
    X = f32(rng.normal(size=(16, 4096)))
    eps = 1e-5
    Y = ref.layernorm_rows(X, None, None, eps)
    assert np.all(np.abs(Y.mean(axis=1)) <= 1e-14)
    var = X.astype(np.float64).var(axis=1)  # biased
    assert np.allclose(Y.var(axis=1), var / (var + eps), rtol=1e-12)
    # an unbiased (N-1) variance would miss this by 1/4096 ~ 2.4e-4
    assert np.all(np.abs(Y.var(axis=1) - var / (var + eps)) < 1e-9)


def test_layernorm_constant_row_gives_beta_and_affine_axis():
    X = np.full((3, 10), 4.25, np.float32)
    beta = f32(rng.normal(size=10))
    gamma = f32(rng.normal(size=10))
    assert np.array_equal(ref.layernorm_rows(X, gamma, beta, 1e-5), np.tile(beta.astype(np.float64), (3, 1)))
    # gamma / beta index the normalised (last) dim
    X = f32(rng.normal(size=(4, 10)))
    Y0 = ref.layernorm_rows(X, None, None, 1e-5)
    Y1 = ref.layernorm_rows(X, gamma, beta, 1e-5)
    assert np.allclose(Y1, Y0 * gamma.astype(np.float64) + beta.astype(np.float64), rtol=1e-14, atol=1e-16)


def test_layernorm_affine_invariance_and_permutation_and_eps_placement():
    X = f32(rng.normal(size=(5, 64)))
    Xa = f32(X * 4 + 8)  # exact scaling; the sum may round, tolerance covers it
    Y = ref.layernorm_rows(X, None, None, 0.0)
    Ya = ref.layernorm_rows(Xa, None, None, 0.0)
    assert np.allclose(Y, Ya, atol=1e-5)
    perm = rng.permutation(64)
    assert np.allclose(ref.layernorm_rows(X[:, perm], None, None, 1e-5),
                       ref.layernorm_rows(X, None, None, 1e-5)[:, perm], rtol=1e-12, atol=1e-14)
    # eps is inside the root: row [1,-1] has mu 0, var 1 -> y = x / sqrt(1+eps)
    Y = ref.layernorm_rows(f32([[1, -1]]), None, None, 3.0)
    assert np.allclose(Y, [[0.5, -0.5]], rtol=1e-15)


# --------------------------------------------------------------------- gelu
def test_gelu_identities():
    x = rng.normal(size=1000) * 3
    g = ref.gelu_tanh(x)
    gm = ref.gelu_tanh(-x)
    assert ref.gelu_tanh(np.zeros(1))[0] == 0.0
    assert np.allclose(g - gm, x, rtol=1e-14, atol=1e-15)  # tanh is odd
    big = np.array([10.0, 25.0])
    assert np.allclose(ref.gelu_tanh(big), big, rtol=1e-15)
    assert np.all(np.abs(ref.gelu_tanh(-big)) < 1e-15)
    # against the erf form: the tanh form is an approximation of
    # x * Phi(x) with max abs deviation below 5e-4 (about 2e-4 near |x| ~ 2)
    erf_form = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in x])
    assert np.max(np.abs(g - erf_form)) < 5e-4
    # a wrong cubic coefficient or sqrt(2/pi) breaks this printed-constant check
    assert ref.gelu_tanh(np.array([1.0]))[0] == pytest.approx(
        0.5 * (1 + math.tanh(math.sqrt(2 / math.pi) * 1.044715)), rel=1e-15)


# --------------------------------------------------------------------- conv
def test_conv_1x1_equals_gemm():
    Nb, Cc, H, W, K = 2, 5, 3, 4, 6
    x = f32(rng.normal(size=(Nb, Cc, H, W)))
    wt = f32(rng.normal(size=(K, Cc, 1, 1)))
    b = f32(rng.normal(size=K))
    out = ref.conv2d_nchw_bias(x, wt, b, stride=1, pad=0)
    # pixels as rows: [N*H*W, C] @ [C, K]
    Xm = x.transpose(0, 2, 3, 1).reshape(-1, Cc)
    Z = ref.gemm_bias(Xm, np.ascontiguousarray(wt.reshape(K, Cc).T), b)
    want = Z.reshape(Nb, H, W, K).transpose(0, 3, 1, 2)
    assert np.allclose(out, want, rtol=1e-13, atol=1e-15)


def test_conv_centre_delta_is_identity_plus_bias():
    Cc = 4
    x = f32(rng.normal(size=(2, Cc, 6, 5)))
    wt = np.zeros((Cc, Cc, 3, 3), np.float32)
    for c in range(Cc):
        wt[c, c, 1, 1] = 1
    b = f32(rng.normal(size=Cc))
    out = ref.conv2d_nchw_bias(x, wt, b, 1, 1)
    assert np.array_equal(out, x.astype(np.float64) + b.astype(np.float64)[None, :, None, None])


def test_conv_all_ones_counts_valid_taps():
    Cc = 64
    x = np.ones((1, Cc, 56, 56), np.float32)
    wt = np.ones((2, Cc, 3, 3), np.float32)
    out, Dn = ref.conv2d_nchw_bias(x, wt, None, 1, 1, want_norm=True)
    assert out.shape == (1, 2, 56, 56)
    assert np.all(out[:, :, 1:-1, 1:-1] == 576)
    assert np.all(out[:, :, 0, 1:-1] == 384) and np.all(out[:, :, -1, 1:-1] == 384)
    assert np.all(out[:, :, 1:-1, 0] == 384) and np.all(out[:, :, 1:-1, -1] == 384)
    for h, w in [(0, 0), (0, -1), (-1, 0), (-1, -1)]:
        assert np.all(out[:, :, h, w] == 256)
    assert np.array_equal(out, Dn)


def test_conv_single_offcentre_tap_pins_direction_and_axes():
    x = f32(rng.normal(size=(1, 1, 5, 6)))
    wt = np.zeros((1, 1, 3, 3), np.float32)
    wt[0, 0, 0, 1] = 1  # kh = 0, kw = 1  ->  out[h][w] = in[h-1][w]
    out = ref.conv2d_nchw_bias(x, wt, None, 1, 1)
    want = np.zeros((5, 6))
    want[1:, :] = x[0, 0, :-1, :]
    assert np.array_equal(out[0, 0], want)
    wt[:] = 0
    wt[0, 0, 1, 2] = 1  # kh = 1, kw = 2  ->  out[h][w] = in[h][w+1]
    out = ref.conv2d_nchw_bias(x, wt, None, 1, 1)
    want = np.zeros((5, 6))
    want[:, :-1] = x[0, 0, :, 1:]
    assert np.array_equal(out[0, 0], want)


@pytest.mark.parametrize("stride,pad,R", [(1, 1, 3), (2, 1, 3), (1, 0, 3), (2, 0, 1), (1, 2, 3)])
def test_conv_brute_force_and_size_formula(stride, pad, R):
    Nb, Cc, H, W, K = 1, 2, 4, 5, 3
    x = f32(rng.normal(size=(Nb, Cc, H, W)))
    wt = f32(rng.normal(size=(K, Cc, R, R)))
    b = f32(rng.normal(size=K))
    out, Dn = ref.conv2d_nchw_bias(x, wt, b, stride, pad, want_norm=True)
    Ho, Wo = (H + 2 * pad - R) // stride + 1, (W + 2 * pad - R) // stride + 1
    assert out.shape == (Nb, K, Ho, Wo)
    xp = np.zeros((Nb, Cc, H + 2 * pad, W + 2 * pad))
    xp[:, :, pad:pad + H, pad:pad + W] = x
    for k, h, w in itertools.product(range(K), range(Ho), range(Wo)):
        patch = xp[0, :, h * stride:h * stride + R, w * stride:w * stride + R]
        want = float(b[k]) + float(np.sum(patch * wt[k].astype(np.float64)))
        assert out[0, k, h, w] == pytest.approx(want, rel=1e-13, abs=1e-14)
        wantD = abs(float(b[k])) + float(np.sum(np.abs(patch) * np.abs(wt[k]).astype(np.float64)))
        assert Dn[0, k, h, w] == pytest.approx(wantD, rel=1e-13)


def test_conv_batch_and_channel_layout():
    # distinct constant per (n, c) plane, one weight per (k, c): out = sum_c w[k,c] * v[n,c] * taps
    Nb, Cc, K = 2, 3, 2
    v = np.arange(1, Nb * Cc + 1, dtype=np.float32).reshape(Nb, Cc, 1, 1)
    x = v * np.ones((Nb, Cc, 4, 4), np.float32)
    wk = f32([[1, 10, 100], [2, 20, 200]])
    wt = wk[:, :, None, None] * np.ones((K, Cc, 3, 3), np.float32)
    out = ref.conv2d_nchw_bias(x, wt, None, 1, 1)
    for n, k in itertools.product(range(Nb), range(K)):
        assert out[n, k, 1, 1] == 9 * float(np.sum(wk[k] * v[n, :, 0, 0]))


# ---------------------------------------------------------------- attention
def _attention_unfused(Q, K, V, scale):
    """Separately written: whole score matrix, numpy ops."""
    Qd, Kd, Vd = (a.astype(np.float64) for a in (Q, K, V))
    S = np.einsum("bid,bjd->bij", Qd, Kd) * scale
    S = S - S.max(axis=2, keepdims=True)
    P = np.exp(S)
    P /= P.sum(axis=2, keepdims=True)
    return np.einsum("bij,bjd->bid", P, Vd), np.einsum("bij,bjd->bid", P, np.abs(Vd))


def test_attention_special_cases():
    B, L, D = 2, 9, 8
    Q = f32(rng.normal(size=(B, L, D)))
    K = f32(rng.normal(size=(B, 13, D)))
    V = f32(rng.normal(size=(B, 13, D)))
    # constant V
    Vc = np.full_like(V, 0.75)
    assert np.allclose(ref.attention(Q, K, Vc, 0.125), 0.75, rtol=1e-14)
    # Q = 0 -> uniform weights -> column means of V
    O = ref.attention(np.zeros_like(Q), K, V, 0.125)
    assert np.allclose(O, np.broadcast_to(V.astype(np.float64).mean(axis=1, keepdims=True), O.shape), rtol=1e-13, atol=1e-15)
    # one key -> O = V row
    O = ref.attention(Q, K[:, :1], V[:, :1], 0.125)
    assert np.allclose(O, np.broadcast_to(V[:, :1].astype(np.float64), O.shape), rtol=1e-15)


def test_attention_dominant_key_and_scale():
    D = 4
    Q = np.zeros((1, 1, D), np.float32)
    Q[0, 0, 0] = 10
    K = np.zeros((1, 6, D), np.float32)
    K[0, 3, 0] = 40  # score = 400 * scale
    V = f32(rng.normal(size=(1, 6, D)))
    O = ref.attention(Q, K, V, 0.125)  # dominant score +50 over the rest
    assert np.allclose(O[0, 0], V[0, 3], atol=1e-20 + 6 * math.exp(-50) * 4)
    # scale enters the exponent: two keys, scores q.k = a, 0  ->  p0 = sigmoid(scale * a)
    K2 = np.zeros((1, 2, D), np.float32)
    K2[0, 0, 0] = 0.2
    V2 = np.zeros((1, 2, D), np.float32)
    V2[0, 0, :] = 1
    O = ref.attention(Q, K2, V2, 0.125)
    assert O[0, 0, 0] == pytest.approx(1 / (1 + math.exp(-0.125 * 10 * float(np.float32(0.2)))), rel=1e-14)


def test_attention_matches_unfused_composition():
    B, L, Lk, D = 2, 17, 23, 16
    Q = f32(rng.normal(size=(B, L, D)))
    K = f32(rng.normal(size=(B, Lk, D)))
    V = f32(rng.normal(size=(B, Lk, D)))
    O, Dn = ref.attention(Q, K, V, 0.25, want_norm=True)
    wantO, wantD = _attention_unfused(Q, K, V, 0.25)
    assert np.allclose(O, wantO, rtol=1e-12, atol=1e-14)
    assert np.allclose(Dn, wantD, rtol=1e-12)
    # batches are independent: batch 1 alone gives the same rows
    assert np.array_equal(ref.attention(Q[1:], K[1:], V[1:], 0.25), O[1:])


def test_attention_composition_of_pinned_pieces():
    # GEMM -> scale -> softmax -> GEMM from the separately pinned operators
    L, Lk, D = 6, 10, 8
    Q = f32(rng.normal(size=(1, L, D)))
    K = f32(rng.normal(size=(1, Lk, D)))
    V = f32(rng.normal(size=(1, Lk, D)))
    S = ref.gemm_bias(Q[0], np.ascontiguousarray(K[0].T)) * 0.125
    P = ref.softmax_rows(S)
    want = P @ V[0].astype(np.float64)
    assert np.allclose(ref.attention(Q, K, V, 0.125)[0], want, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- chain 1/3
def test_chain1_is_composition_with_fp64_intermediates():
    X = f32(rng.uniform(-1, 1, (8, 32)))
    W = f32(rng.uniform(-1 / 16, 1 / 16, (32, 16)))
    b = f32(rng.uniform(-0.1, 0.1, 16))
    Z = np.maximum(X.astype(np.float64) @ W.astype(np.float64) + b, 0)
    E = np.exp(Z - Z.max(axis=1, keepdims=True))
    want = E / E.sum(axis=1, keepdims=True)
    assert np.allclose(ref.chain1(X, W, b), want, rtol=1e-12)


def test_chain3_matches_numpy_definition():
    X = f32(rng.normal(size=(6, 100)))
    g, b = f32(rng.normal(1, 0.1, 100)), f32(rng.normal(0, 0.1, 100))
    Xd = X.astype(np.float64)
    y = (Xd - Xd.mean(1, keepdims=True)) / np.sqrt(Xd.var(1, keepdims=True) + 1e-5) * g + b
    want = 0.5 * y * (1 + np.tanh(0.7978845608028654 * (y + 0.044715 * y ** 3)))
    assert np.allclose(ref.chain3(X, g, b, 1e-5), want, rtol=1e-12, atol=1e-15)


# --------------------------------------------------- acceptance-rule machinery
def test_pointwise_rule_threshold():
    o = np.array([1.0, -2.0, 0.0, 1e-9])
    rms = math.sqrt(np.mean(o * o))
    assert compare.pointwise(o.copy(), o)
    g = o.copy()
    g[0] += 0.99e-4
    assert compare.pointwise(g, o)
    g[0] = 1.0 + 1.01e-4
    v = compare.pointwise(g, o)
    assert not v and v.index == (0,)
    g = o.copy()
    g[2] = 0.99e-6 * rms  # floor: 1e-4 * 1e-2 * rms
    assert compare.pointwise(g, o)
    g[2] = 1.01e-6 * rms
    assert not compare.pointwise(g, o)
    g = o.copy()
    g[1] = np.nan
    assert not compare.pointwise(g, o)


def test_contraction_rule_threshold():
    o = np.array([[0.5, -0.25]])
    Dn = np.array([[10.0, 4.0]])
    g = o.copy()
    g[0, 0] += 0.0199
    assert compare.contraction(g, o, Dn)
    g[0, 1] -= 0.0081
    v = compare.contraction(g, o, Dn)
    assert not v and v.index == (0, 1)


def test_planted_mistakes_are_caught():
    # mistakes planted in copies of the checker's formulas must fail the rules
    X = f32(rng.normal(size=(4, 256)))
    good = ref.chain3(X, None, None, 1e-5)
    Xd = X.astype(np.float64)
    y = (Xd - Xd.mean(1, keepdims=True)) / np.sqrt(Xd.var(1, ddof=1, keepdims=True) + 1e-5)  # unbiased
    bad = 0.5 * y * (1 + np.tanh(0.7978845608028654 * (y + 0.044715 * y ** 3)))
    assert not compare.pointwise(bad, good)
    erf_form = 0.5 * good * 0 + np.array([[0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in row]
                                         for row in ref.layernorm_rows(X, None, None, 1e-5)])
    assert not compare.pointwise(erf_form, good)


# ---------------------------------------------------------- layout transform
def test_layout_copy_against_numpy_views():
    base = f32(rng.normal(size=2 * 3 * 4 * 5))
    x = base.reshape(2, 3, 4, 5)
    # NCHW -> NHWC: the view has shape [N,H,W,C] and strides of the permuted axes
    v = np.transpose(x, (0, 2, 3, 1))
    got = ref.layout_copy(base, v.shape, [s // 4 for s in v.strides])
    assert np.array_equal(got.view(np.uint32), np.ascontiguousarray(v).view(np.uint32))
    # 2-D transpose, element by element
    m = f32(np.arange(12)).reshape(3, 4)
    got = ref.layout_copy(m, (4, 3), (1, 4))
    for i in range(4):
        for j in range(3):
            assert got[i, j] == m[j, i]
    # strided slice and a broadcast (stride 0)
    v = x[:, ::2, 1:3, :]
    off = (v.__array_interface__["data"][0] - base.__array_interface__["data"][0]) // 4
    got = ref.layout_copy(base[off:], v.shape, [s // 4 for s in v.strides])
    assert np.array_equal(got, v)
    got = ref.layout_copy(f32([1.5, 2.5]), (3, 2), (0, 1))
    assert np.array_equal(got, np.array([[1.5, 2.5]] * 3, np.float32))
    # bit patterns survive (NaN payload, -0)
    odd = np.array([0x7FC12345, 0x80000000, 0x00000001], np.uint32).view(np.float32)
    got = ref.layout_copy(odd, (3,), (1,))
    assert np.array_equal(got.view(np.uint32), odd.view(np.uint32))


# ------------------------------------------- hash dropout, mean (Section 5.3)
def _hash_bigint(h):
    """The three xor-shift steps in arbitrary-precision integers, reduced mod 2^64
    only where a 64-bit register would drop bits (the left shift)."""
    h ^= h >> 17
    h ^= (h << 31) % (1 << 64)
    h ^= h >> 8
    return h


def test_dropout_rand_matches_worked_values():
    import json, os
    cases = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "dropout_hash_cases.json")))["cases"]
    for h0, want in cases:
        assert ref.dropout_rand(h0) == np.float32(want) / np.float32(1000.0), h0
    # shift directions and amounts: a one-bit input lands on the bits the three steps say
    for bit in (0, 5, 17, 30, 33, 40, 63):
        h0 = 1 << bit
        assert ref.dropout_rand(h0) == np.float32(_hash_bigint(h0) % 1000) / np.float32(1000.0)


def test_dropout_mask_uses_row_major_offset_plus_seed():
    M, N, p = 6, 11, 0.5
    ones = np.ones((M, N))
    a = ref.dropout_hash(ones, p, 12345)
    # element (i, j) depends on i*N + j only: the same data flattened to one row gives the same mask
    b = ref.dropout_hash(np.ones((1, M * N)), p, 12345)
    assert np.array_equal(a.reshape(-1), b.reshape(-1))
    # ... and on offset + seed only: seed s is seed 0 shifted by s elements
    c = ref.dropout_hash(np.ones((1, M * N + 7)), p, 12338)
    assert np.array_equal(a.reshape(-1), c.reshape(-1)[7:])
    # the mask itself, element by element, from the worked hash
    for i in range(M):
        for j in range(N):
            r = np.float32(_hash_bigint(i * N + j + 12345) % 1000) / np.float32(1000.0)
            assert a[i, j] == (0.0 if r < np.float32(p) else 2.0)
    # a transposed offset (j*M + i) would give another mask
    t = ref.dropout_hash(np.ones((N, M)), p, 12345).T
    assert not np.array_equal(a, t)


def test_dropout_limits_scale_and_rate():
    Z = rng.normal(size=(50, 40))
    assert np.array_equal(ref.dropout_hash(Z, 0.0, 99), Z)          # p = 0: nothing dropped, scale 1
    out = ref.dropout_hash(Z, 0.25, 99)
    kept = out != 0.0
    assert np.allclose(out[kept], Z[kept] / 0.75, rtol=1e-15, atol=0)  # survivors scaled by 1/(1-p)
    # rand takes the values u/1000, u = h % 1000; exactly those with u/1000 < p are dropped
    big = ref.dropout_hash(np.ones((400, 500)), 0.25, 7)
    rate = 1.0 - np.count_nonzero(big) / big.size
    assert abs(rate - 0.25) < 5 * math.sqrt(0.25 * 0.75 / big.size)
    # the boundary is strict: rand == p survives (p = 0.5 = 500/1000 exactly in fp32)
    h0 = next(h for h in range(10**6) if _hash_bigint(h) % 1000 == 500)
    assert ref.dropout_hash(np.ones((1, 1)), 0.5, h0)[0, 0] == 2.0
    h1 = next(h for h in range(10**6) if _hash_bigint(h) % 1000 == 499)
    assert ref.dropout_hash(np.ones((1, 1)), 0.5, h1)[0, 0] == 0.0
    # the comparison is made in fp32: 0.3 rounds up in fp32, so rand = 300/1000 (which rounds the same way) is kept
    h2 = next(h for h in range(10**6) if _hash_bigint(h) % 1000 == 300)
    assert ref.dropout_hash(np.ones((1, 1)), 0.3, h2)[0, 0] != 0.0


def test_dropout_wraps_in_64_bits():
    # offset + seed wraps, and the left shift drops the high bits
    seed = (1 << 64) - 3
    out = ref.dropout_hash(np.ones((1, 8)), 0.5, seed)
    for j in range(8):
        r = np.float32(_hash_bigint((j + seed) % (1 << 64)) % 1000) / np.float32(1000.0)
        assert out[0, j] == (0.0 if r < np.float32(0.5) else 2.0)


def test_mean_rows_closed_forms():
    assert np.array_equal(ref.mean_rows(np.full((3, 17), 2.5)), np.full(3, 2.5))
    ramp = np.arange(5 * 64, dtype=np.float64).reshape(5, 64)
    assert np.array_equal(ref.mean_rows(ramp), 64 * np.arange(5) + 31.5)   # (N-1)/2 + row start
    Z = rng.normal(size=(9, 37))
    assert np.allclose(ref.mean_rows(Z), Z.sum(axis=1) / 37, rtol=0, atol=1e-15)
    # last axis, not the first: a tall constant-per-column matrix has equal row means
    cols = np.tile(np.arange(4.0), (6, 1))
    assert np.array_equal(ref.mean_rows(cols), np.full(6, 1.5))


def test_chain6_composition_and_softmax_axis():
    M, K, N, p, seed = 12, 9, 20, 0.25, 2506
    X = f32(rng.normal(size=(M, K))); W = f32(rng.normal(size=(K, N))); b = f32(rng.normal(size=N))
    Z = X.astype(np.float64) @ W.astype(np.float64) + b
    mask = np.array([[np.float32(_hash_bigint(i * N + j + seed) % 1000) / np.float32(1000.0) >= np.float32(p)
                      for j in range(N)] for i in range(M)])
    D = np.where(mask, Z / 0.75, 0.0)
    assert np.allclose(ref.chain6(X, W, b, p, seed, "dropout"), D, rtol=0, atol=1e-13)
    mu = D.mean(axis=1)
    assert np.allclose(ref.chain6(X, W, b, p, seed, "mean"), mu, rtol=0, atol=1e-13)
    out = ref.chain6(X, W, b, p, seed)
    e = np.exp(mu - mu.max())
    assert out.shape == (M,)
    assert np.allclose(out, e / e.sum(), rtol=0, atol=1e-15)
    assert abs(out.sum() - 1.0) < 1e-14          # one softmax over the M row means


# ------------------------------------ per-channel affine on planes, 2x2 max pool
def test_scale_shift_planes_channel_axis_and_closed_form():
    T = rng.normal(size=(3, 4, 5, 6))
    sc = f32([1.0, 2.0, -0.5, 0.0]); sh = f32([0.0, 1.0, 3.0, -2.0])
    got = ref.scale_shift_ch(T, sc, sh)
    want = T * sc.astype(np.float64)[None, :, None, None] + sh.astype(np.float64)[None, :, None, None]
    assert np.array_equal(got, want)
    assert np.array_equal(got[:, 3], np.full((3, 5, 6), -2.0))      # scale 0 leaves the shift of channel 3 only
    assert np.array_equal(ref.scale_shift_ch(T, None, None), T)
    assert np.array_equal(ref.scale_shift_ch(T, None, sh), T + sh.astype(np.float64)[None, :, None, None])


def test_maxpool2x2_windows_stride_and_odd_edges():
    # one plane whose value encodes its position: the window maximum is its bottom-right element
    H, W = 6, 8
    T = (np.arange(H)[:, None] * 100 + np.arange(W)[None, :]).astype(np.float64).reshape(1, 1, H, W)
    got = ref.maxpool2x2(T)
    assert got.shape == (1, 1, 3, 4)
    want = (np.arange(1, H, 2)[:, None] * 100 + np.arange(1, W, 2)[None, :]).astype(np.float64)
    assert np.array_equal(got[0, 0], want)
    # a single spike is seen by exactly one window: (y, x) -> (y // 2, x // 2)
    for (y, x) in [(0, 0), (1, 7), (4, 3), (5, 6)]:
        S = np.full((1, 1, H, W), -1.0); S[0, 0, y, x] = 5.0
        P = ref.maxpool2x2(S)
        assert P[0, 0, y // 2, x // 2] == 5.0 and np.count_nonzero(P == 5.0) == 1
    # negative values: the maximum, not the maximum magnitude, and no implicit zero
    N = -np.abs(rng.normal(size=(2, 3, 4, 4))) - 1.0
    assert np.all(ref.maxpool2x2(N) < 0)
    # odd sizes drop the last row / column; planes are independent; numpy witness by reshaping
    Z = rng.normal(size=(2, 3, 7, 9))
    want = Z[:, :, :6, :8].reshape(2, 3, 3, 2, 4, 2).max(axis=(3, 5))
    assert np.array_equal(ref.maxpool2x2(Z), want)
    assert ref.maxpool2x2(np.zeros((1, 1, 1, 5))).shape == (1, 1, 0, 2)


def test_chain7_composition():
    inp = f32(rng.normal(size=(2, 3, 6, 6))); wt = f32(rng.normal(size=(4, 3, 3, 3)) * 0.3)
    b = f32(rng.normal(size=4)); sc = f32(rng.normal(size=4)); sh = f32(rng.normal(size=4))
    out, Dn = ref.chain7(inp, wt, b, sc, sh)
    conv = ref.conv2d_nchw_bias(inp, wt, b)
    aff = conv * sc.astype(np.float64)[None, :, None, None] + sh.astype(np.float64)[None, :, None, None]
    want = np.maximum(aff, 0).reshape(2, 4, 3, 2, 3, 2).max(axis=(3, 5))
    assert np.array_equal(out, want)
    assert Dn.shape == conv.shape and np.all(Dn >= np.abs(aff) - 1e-12)   # the normaliser bounds the value it scales


# -------------------------------------------------- reductions over one axis
def _view(base, shape, stride):
    return np.lib.stride_tricks.as_strided(base, shape=shape, strides=[4 * s for s in stride])


def test_reduce_axis_against_numpy_on_strided_views():
    base = f32(rng.normal(size=4000))
    cases = [((6, 7, 8), (56, 8, 1)),          # contiguous
             ((8, 7, 6), (1, 8, 56)),          # fully permuted
             ((5, 4, 9), (100, 20, 2)),        # gaps and a strided inner dim
             ((3, 6, 5), (0, 5, 1)),           # broadcast outer dim
             ((4, 1, 7), (7, 0, 1)),
             ((12,), (3,))]
    for shape, stride in cases:
        v = _view(base, shape, stride).astype(np.float64)
        for axis in range(len(shape)):
            s, a = ref.reduce_axis(base, shape, stride, axis, "sum", want_abs=True)
            assert np.allclose(s, v.sum(axis=axis), rtol=0, atol=1e-12)
            assert np.allclose(a, np.abs(v).sum(axis=axis), rtol=0, atol=1e-12)
            assert np.allclose(ref.reduce_axis(base, shape, stride, axis, "mean"), v.mean(axis=axis), rtol=0, atol=1e-13)
            assert np.array_equal(ref.reduce_axis(base, shape, stride, axis, "argmax"), v.argmax(axis=axis))
            assert np.array_equal(ref.reduce_axis(base, shape, stride, axis, "argmin"), v.argmin(axis=axis))


def test_eltwise_map_further_unary_steps():
    rng = np.random.default_rng(41)
    x = (rng.standard_normal(500) * 3.0).astype(np.float32)
    x64 = x.astype(np.float64)
    m = lambda steps, a=x: ref.eltwise_map(a, (a.size,), (1,), unary=steps)   # noqa: E731
    # library routines and identities
    assert np.array_equal(m(["abs"]), np.abs(x64)) and np.array_equal(m(["neg"]), -x64) and np.array_equal(m(["square"]), x64 * x64)
    assert np.array_equal(m(["neg", "neg"]), x64) and np.array_equal(m(["abs", "sqrt", "square"]), np.sqrt(np.abs(x64)) ** 2)
    pos = (np.abs(x) + np.float32(0.01)).astype(np.float32)
    assert np.allclose(m(["log"], pos), np.log(pos.astype(np.float64)), rtol=1e-15, atol=0)
    assert np.allclose(m(["log", "exp"], pos), pos.astype(np.float64), rtol=1e-14)
    one = np.array([1.0, np.e], np.float32)
    assert m(["log"], one)[0] == 0.0 and abs(m(["log"], one)[1] - np.log(np.float64(one[1]))) < 1e-16
    # SiLU = x * logistic(x) (the pinned step 8); silu(x) - silu(-x) = x; silu(0) = 0
    assert np.allclose(m(["silu"]), x64 * m(["sigmoid"]), rtol=1e-15, atol=0)
    assert np.allclose(m(["silu"]) - m(["neg", "silu"]), x64, rtol=0, atol=1e-14)
    assert m(["silu"], np.zeros(1, np.float32))[0] == 0.0
    # hard swish: 0 below -3, x above 3, x (x + 3) / 6 between; printed values at -1, 0, 1
    hs = m(["hardswish"])
    assert np.array_equal(hs[x64 <= -3], np.zeros((x64 <= -3).sum())) and np.array_equal(hs[x64 >= 3], x64[x64 >= 3])
    mid = (x64 > -3) & (x64 < 3)
    assert np.allclose(hs[mid], x64[mid] * (x64[mid] + 3.0) / 6.0, rtol=1e-15, atol=0)
    pts = m(["hardswish"], np.array([-1.0, 0.0, 1.0, 3.0, -3.0], np.float32))
    assert np.allclose(pts, [-1.0 / 3.0, 0.0, 2.0 / 3.0, 3.0, 0.0], rtol=1e-15, atol=0)


def test_rmsnorm_invariants_and_closed_forms():
    rng = np.random.default_rng(51)
    X = (rng.standard_normal((6, 37)) * 3.0 + 1.0).astype(np.float32)
    g = rng.standard_normal(37).astype(np.float32)
    x64, g64 = X.astype(np.float64), g.astype(np.float64)
    Y = ref.rmsnorm_rows(X, g, 1e-3)
    # undoing the normalisation gives x * gamma back; without gamma every row has mean square ms / (ms + eps)
    ms = (x64 ** 2).mean(axis=1, keepdims=True)
    assert np.allclose(Y * np.sqrt(ms + 1e-3), x64 * g64, rtol=1e-13, atol=0)
    P = ref.rmsnorm_rows(X, None, 1e-3)
    assert np.allclose((P ** 2).mean(axis=1, keepdims=True), ms / (ms + 1e-3), rtol=1e-13)
    # a row of mean zero: the pinned layer normalisation without beta
    Z = (x64 - x64.mean(axis=1, keepdims=True)).astype(np.float32)
    Z = (Z.astype(np.float64) - Z.astype(np.float64).mean(axis=1, keepdims=True)).astype(np.float32)
    ln = ref.layernorm_rows(Z, g, None, 1e-3)
    mu = Z.astype(np.float64).mean(axis=1, keepdims=True)
    assert np.max(np.abs(mu)) < 1e-7 and np.allclose(ref.rmsnorm_rows(Z, g, 1e-3), ln, rtol=0, atol=1e-6)
    # scaling the row by a (eps = 0) multiplies the result by sign(a); a constant row c gives c / sqrt(c^2 + eps) * gamma
    assert np.allclose(ref.rmsnorm_rows(X * np.float32(-4.0), g, 0.0), -ref.rmsnorm_rows(X, g, 0.0), rtol=1e-13, atol=0)
    C = np.full((1, 37), 2.5, np.float32)
    assert np.allclose(ref.rmsnorm_rows(C, g, 0.75), 2.5 / np.sqrt(6.25 + 0.75) * g64[None, :], rtol=1e-15, atol=0)
    # element by element on a tiny case
    T = rng.standard_normal((2, 5)).astype(np.float32)
    Yt = ref.rmsnorm_rows(T, g[:5], 1e-2)
    for r in range(2):
        m2 = sum(float(v) ** 2 for v in T[r]) / 5
        for n in range(5):
            assert abs(Yt[r, n] - float(T[r, n]) / (m2 + 1e-2) ** 0.5 * float(g[n])) < 1e-14


def test_groupnorm_reduces_to_layernorm_and_closed_forms():
    rng = np.random.default_rng(31)
    X = (rng.standard_normal((3, 12, 5, 7)) * 2.0 + 0.7).astype(np.float32)
    ga = rng.standard_normal(12).astype(np.float32)
    be = rng.standard_normal(12).astype(np.float32)
    # one group: layer normalisation of each image over C*H*W, whose gamma / beta repeat each channel's value over its plane
    ln = ref.layernorm_rows(X.reshape(3, -1), np.repeat(ga, 35), np.repeat(be, 35), 1e-5).reshape(X.shape)
    assert np.allclose(ref.groupnorm_nchw(X, 1, ga, be, 1e-5), ln, rtol=0, atol=1e-12)
    # G groups: layer normalisation of the [N*G, (C/G)*H*W] matrix without affine, then the per-channel affine
    for G in (2, 3, 4, 12):
        plain = ref.layernorm_rows(X.reshape(3 * G, -1), None, None, 1e-5).reshape(X.shape)
        want = plain * ga.astype(np.float64)[None, :, None, None] + be.astype(np.float64)[None, :, None, None]
        assert np.allclose(ref.groupnorm_nchw(X, G, ga, be, 1e-5), want, rtol=0, atol=1e-12), G
    # without affine every group has mean 0 and variance var / (var + eps)
    Y = ref.groupnorm_nchw(X, 4, None, None, 1e-3).reshape(3, 4, -1)
    var = X.astype(np.float64).reshape(3, 4, -1).var(axis=2)
    assert np.allclose(Y.mean(axis=2), 0.0, atol=1e-12) and np.allclose(Y.var(axis=2), var / (var + 1e-3), rtol=1e-12)
    # instance normalisation of a plane of +-1 in equal numbers: mean 0, variance 1 -> +-1 / sqrt(1 + eps)
    P = np.ones((1, 2, 4, 6), np.float32); P[:, :, :, ::2] = -1.0
    assert np.allclose(ref.groupnorm_nchw(P, 2, None, None, 0.21), P / np.sqrt(1.21), rtol=0, atol=1e-15)
    # shifting and scaling the input (a > 0) changes nothing as eps -> 0; a constant group gives beta
    a = ref.groupnorm_nchw(X, 3, ga, be, 0.0)
    b = ref.groupnorm_nchw((X.astype(np.float64) * 4.0 + 8.0).astype(np.float32), 3, ga, be, 0.0)
    assert np.allclose(a, b, rtol=0, atol=1e-5)
    Cst = np.full((2, 4, 3, 3), 2.5, np.float32)
    assert np.array_equal(ref.groupnorm_nchw(Cst, 2, ga[:4], be[:4], 1e-5), np.broadcast_to(be[:4].astype(np.float64)[None, :, None, None], Cst.shape))
    # brute force on a tiny case, element by element
    T = rng.standard_normal((2, 4, 2, 3)).astype(np.float32)
    Yt = ref.groupnorm_nchw(T, 2, ga[:4], be[:4], 1e-2)
    for n in range(2):
        for c in range(4):
            grp = T[n, (c // 2) * 2:(c // 2) * 2 + 2].astype(np.float64).ravel()
            mu = sum(grp) / len(grp)
            var = sum((v - mu) ** 2 for v in grp) / len(grp)
            for h in range(2):
                for w in range(3):
                    assert abs(Yt[n, c, h, w] - ((float(T[n, c, h, w]) - mu) / (var + 1e-2) ** 0.5 * float(ga[c]) + float(be[c]))) < 1e-12


def test_maxpool2d_against_sliding_windows_and_special_cases():
    # numpy: pad with -inf, take every window with sliding_window_view, subsample by the stride
    rng = np.random.default_rng(21)
    for (H, W, k, s, p) in [(9, 11, 3, 2, 1), (8, 8, 2, 2, 0), (7, 10, 3, 1, 1), (12, 5, 5, 3, 2), (6, 6, 3, 2, 0), (5, 9, 1, 2, 0),
                            (10, 10, 7, 2, 3), (4, 4, 4, 4, 0)]:
        T = rng.standard_normal((2, 3, H, W)) - 2.0          # mostly negative: a zero padding would win
        P = np.full((2, 3, H + 2 * p, W + 2 * p), -np.inf)
        P[:, :, p:p + H, p:p + W] = T
        win = np.lib.stride_tricks.sliding_window_view(P, (k, k), axis=(2, 3))[:, :, ::s, ::s]
        want = win.max(axis=(4, 5))
        got = ref.maxpool2d(T, k, s, p)
        assert got.shape == want.shape and np.array_equal(got, want), (H, W, k, s, p)
    # k = 2, s = 2, p = 0 is the 2x2 pooling of the VGG block
    T = rng.standard_normal((2, 2, 9, 7))
    assert np.array_equal(ref.maxpool2d(T, 2, 2, 0), ref.maxpool2x2(T))
    # a ramp increasing along both axes: the window's last element inside the image
    R = (np.arange(8)[:, None] * 100.0 + np.arange(10)[None, :]).reshape(1, 1, 8, 10)
    got = ref.maxpool2d(R, 3, 2, 1)
    for oy in range(4):
        for ox in range(5):
            assert got[0, 0, oy, ox] == min(2 * oy + 1, 7) * 100.0 + min(2 * ox + 1, 9)
    # a 1x1 window at stride 1 is the identity; a window as large as the image gives the global maximum
    assert np.array_equal(ref.maxpool2d(T, 1, 1, 0), T)
    assert np.array_equal(ref.maxpool2d(T[:, :, :7, :], 7, 1, 0)[:, :, 0, 0], T[:, :, :7, :].max(axis=(2, 3)))


def test_avgpool2d_against_sliding_windows_and_special_cases():
    rng = np.random.default_rng(23)
    for (H, W, k, s, p) in [(9, 11, 3, 2, 1), (8, 8, 2, 2, 0), (7, 10, 3, 1, 1), (12, 5, 5, 3, 2), (6, 6, 3, 2, 0), (10, 10, 7, 2, 3)]:
        T = rng.standard_normal((2, 3, H, W)) + 1.0
        P = np.zeros((2, 3, H + 2 * p, W + 2 * p))
        P[:, :, p:p + H, p:p + W] = T
        win = np.lib.stride_tricks.sliding_window_view(P, (k, k), axis=(2, 3))[:, :, ::s, ::s]
        assert np.allclose(ref.avgpool2d(T, k, s, p), win.mean(axis=(4, 5)), rtol=0, atol=1e-14), (H, W, k, s, p)
    # a window as large as the image: the global average pool of chain 2; a 1x1 window: the identity
    T = rng.standard_normal((2, 2, 6, 6))
    assert np.allclose(ref.avgpool2d(T, 6, 1, 0)[:, :, 0, 0], T.mean(axis=(2, 3)), rtol=0, atol=1e-15)
    assert np.array_equal(ref.avgpool2d(T, 1, 1, 0), T)
    # an image of ones, 3x3 / 1 / pad 1: 1 inside, 6/9 on the edges, 4/9 in the corners
    O = ref.avgpool2d(np.ones((1, 1, 5, 5)), 3, 1, 1)[0, 0]
    assert np.allclose(O[1:-1, 1:-1], 1.0) and np.allclose(O[0, 1:-1], 6.0 / 9.0) and np.allclose(O[0, 0], 4.0 / 9.0) and np.allclose(O[-1, -1], 4.0 / 9.0)
    # linear: pool(2 a - 3 b) = 2 pool(a) - 3 pool(b)
    A, B = rng.standard_normal((1, 2, 7, 9)), rng.standard_normal((1, 2, 7, 9))
    assert np.allclose(ref.avgpool2d(2 * A - 3 * B, 3, 2, 1), 2 * ref.avgpool2d(A, 3, 2, 1) - 3 * ref.avgpool2d(B, 3, 2, 1), rtol=0, atol=1e-13)


def test_reduce_axis_max_min_values():
    # against numpy on strided views; the value at the arg-reduction's index; min(x) = -max(-x); a ramp; infinities
    rng = np.random.default_rng(9)
    base = rng.integers(-5, 6, 4000).astype(np.float32)     # full of ties
    for shape, stride in [((7, 9, 11), (99, 11, 1)), ((7, 9, 11), (1, 7, 63)), ((5, 6), (12, 2)), ((13,), (3,)), ((4, 1, 6), (30, 0, 5))]:
        v = np.lib.stride_tricks.as_strided(base, shape, tuple(4 * s for s in stride))
        for axis in range(len(shape)):
            mx = ref.reduce_axis(base, shape, stride, axis, "max")
            mn = ref.reduce_axis(base, shape, stride, axis, "min")
            assert np.array_equal(mx, v.max(axis=axis)) and np.array_equal(mn, v.min(axis=axis))
            am = ref.reduce_axis(base, shape, stride, axis, "argmax")
            assert np.array_equal(mx, np.take_along_axis(v, np.expand_dims(am, axis), axis).squeeze(axis))
            assert np.array_equal(mn, -ref.reduce_axis(-base, shape, stride, axis, "max"))
    x = np.arange(60, dtype=np.float32)
    assert np.array_equal(ref.reduce_axis(x, (3, 4, 5), (20, 5, 1), 1, "max"), x.reshape(3, 4, 5)[:, 3, :])
    assert np.array_equal(ref.reduce_axis(x, (3, 4, 5), (20, 5, 1), 1, "min"), x.reshape(3, 4, 5)[:, 0, :])
    y = np.array([1.0, -np.inf, np.inf, 3.0], np.float32)
    assert ref.reduce_axis(y, (4,), (1,), 0, "max") == np.inf and ref.reduce_axis(y, (4,), (1,), 0, "min") == -np.inf


def test_reduce_axis_closed_forms_and_output_order():
    # x[i][j][k] = 100 i + 10 j + k on a 3 x 4 x 5 grid: sums have closed forms and show which axis went away
    i, j, k = np.meshgrid(np.arange(3), np.arange(4), np.arange(5), indexing="ij")
    x = f32(100 * i + 10 * j + k)
    s0 = ref.reduce_axis(x, (3, 4, 5), (20, 5, 1), 0, "sum")
    assert s0.shape == (4, 5) and np.array_equal(s0, 300 + 3 * (10 * np.arange(4)[:, None] + np.arange(5)[None, :]))
    s1 = ref.reduce_axis(x, (3, 4, 5), (20, 5, 1), 1, "sum")
    assert s1.shape == (3, 5) and np.array_equal(s1, 4 * (100 * np.arange(3)[:, None] + np.arange(5)[None, :]) + 60)
    m2 = ref.reduce_axis(x, (3, 4, 5), (20, 5, 1), 2, "mean")
    assert m2.shape == (3, 4) and np.array_equal(m2, 100 * np.arange(3)[:, None] + 10 * np.arange(4)[None, :] + 2.0)
    # increasing along every axis: argmax is the last index, argmin the first
    for ax, n in enumerate((3, 4, 5)):
        assert np.all(ref.reduce_axis(x, (3, 4, 5), (20, 5, 1), ax, "argmax") == n - 1)
        assert np.all(ref.reduce_axis(x, (3, 4, 5), (20, 5, 1), ax, "argmin") == 0)


def test_arg_reductions_break_ties_towards_the_lowest_index():
    x = f32([2, 7, 7, 1, 7, 1, 1, 3])
    assert ref.reduce_axis(x, (8,), (1,), 0, "argmax") == 1
    assert ref.reduce_axis(x, (8,), (1,), 0, "argmin") == 3
    assert ref.reduce_axis(np.zeros(9, np.float32), (9,), (1,), 0, "argmax") == 0
    # -0 and +0 compare equal: the first of them wins either way
    z = f32([0.0, -0.0, 0.0])
    assert ref.reduce_axis(z, (3,), (1,), 0, "argmin") == 0 and ref.reduce_axis(z, (3,), (1,), 0, "argmax") == 0
    # a broadcast (stride 0) axis is all ties
    assert np.all(ref.reduce_axis(f32(rng.normal(size=5)), (5, 4), (1, 0), 1, "argmax") == 0)
    # magnitudes do not matter, order does
    assert ref.reduce_axis(f32([-5, -1, -9]), (3,), (1,), 0, "argmax") == 1
    assert ref.reduce_axis(f32([-5, -1, -9]), (3,), (1,), 0, "argmin") == 2


# ------------------------------------------------------------ causal attention
def test_causal_attention_closed_forms_and_dense_witness():
    B, L, D = 2, 9, 4
    Q = f32(rng.normal(size=(B, L, D))); K = f32(rng.normal(size=(B, L, D))); V = f32(rng.normal(size=(B, L, D)))
    O = ref.attention(Q, K, V, 0.5, causal=True)
    # the first query sees key 0 only; the last one sees every key, like the unmasked operator
    assert np.allclose(O[:, 0], V[:, 0].astype(np.float64), rtol=0, atol=1e-15)
    assert np.allclose(O[:, -1], ref.attention(Q, K, V, 0.5)[:, -1], rtol=0, atol=1e-14)
    # Q = 0: uniform weights over the visible prefix -> running means of V
    O0 = ref.attention(np.zeros_like(Q), K, V, 0.5, causal=True)
    want = np.cumsum(V.astype(np.float64), axis=1) / np.arange(1, L + 1)[None, :, None]
    assert np.allclose(O0, want, rtol=0, atol=1e-14)
    # dense witness: scores with -inf above the diagonal through the pinned row softmax
    S = 0.5 * np.einsum("bid,bjd->bij", Q.astype(np.float64), K.astype(np.float64))
    S[:, np.triu_indices(L, 1)[0], np.triu_indices(L, 1)[1]] = -np.inf
    P = np.exp(S - S.max(axis=2, keepdims=True)); P /= P.sum(axis=2, keepdims=True)
    assert np.allclose(O, P @ V.astype(np.float64), rtol=0, atol=1e-14)
    # more queries than keys: queries past the last key see all keys; fewer queries: the prefix rule still holds
    Kk, Vv = K[:, :5], V[:, :5]
    Oc = ref.attention(Q, Kk, Vv, 0.5, causal=True)
    assert np.allclose(Oc[:, 5:], ref.attention(Q, Kk, Vv, 0.5)[:, 5:], rtol=0, atol=1e-14)
    assert np.allclose(Oc[:, 2], ref.attention(Q[:, 2:3], Kk[:, :3], Vv[:, :3], 0.5)[:, 0], rtol=0, atol=1e-14)
    # a future key cannot matter: changing K, V beyond the diagonal leaves earlier rows untouched
    K2, V2 = K.copy(), V.copy(); K2[:, 6:] += 3.0; V2[:, 6:] -= 5.0
    assert np.array_equal(ref.attention(Q, K2, V2, 0.5, causal=True)[:, :6], O[:, :6])


# ------------------------------------------------------------- dilated conv
def test_dilated_conv_brute_force_and_tap_positions():
    for (H, W, R, stride, pad, dil) in [(9, 11, 3, 1, 2, 2), (12, 10, 3, 2, 3, 3), (7, 7, 1, 1, 0, 4), (15, 13, 5, 1, 4, 2)]:
        Nb, C, K = 2, 3, 4
        x = f32(rng.normal(size=(Nb, C, H, W))); w = f32(rng.normal(size=(K, C, R, R))); b = f32(rng.normal(size=K))
        got = ref.conv2d_nchw_bias(x, w, b, stride, pad, dil=dil)
        Re = (R - 1) * dil + 1
        Ho, Wo = (H + 2 * pad - Re) // stride + 1, (W + 2 * pad - Re) // stride + 1
        assert got.shape == (Nb, K, Ho, Wo)
        xp = np.zeros((Nb, C, H + 2 * pad, W + 2 * pad)); xp[:, :, pad:pad + H, pad:pad + W] = x
        want = np.zeros((Nb, K, Ho, Wo))
        for kh in range(R):
            for kw in range(R):
                patch = xp[:, :, kh * dil:kh * dil + (Ho - 1) * stride + 1:stride, kw * dil:kw * dil + (Wo - 1) * stride + 1:stride]
                want += np.einsum("nchw,kc->nkhw", patch, w[:, :, kh, kw].astype(np.float64))
        want += b.astype(np.float64)[None, :, None, None]
        assert np.allclose(got, want, rtol=0, atol=1e-12)
    # a filter that is 1 at tap (0, 2) only shifts the image by (-P, 2*dil - P)
    x = f32(rng.normal(size=(1, 1, 8, 8))); w = np.zeros((1, 1, 3, 3), np.float32); w[0, 0, 0, 2] = 1.0
    out = ref.conv2d_nchw_bias(x, w, None, 1, 2, dil=2)      # Re = 5, pad 2: same size
    assert out.shape == (1, 1, 8, 8)
    assert np.array_equal(out[0, 0, 2:, :6], x[0, 0, :6, 2:].astype(np.float64))
    # dil = 1 is the undilated operator
    w3 = f32(rng.normal(size=(2, 1, 3, 3)))
    assert np.array_equal(ref.conv2d_nchw_bias(x, w3, None, 1, 1, dil=1), ref.conv2d_nchw_bias(x, w3, None, 1, 1))


# ------------------------------------------------ elementwise on strided views
def test_eltwise_binary_against_numpy_broadcasting():
    a = f32(rng.normal(size=(4, 5, 6))); row = f32(rng.normal(size=6)); col = f32(rng.normal(size=(4, 1, 1)))
    A = a.astype(np.float64)
    # same shape, a bias row broadcast over the leading dims, a per-slab scalar, a transposed operand
    got = ref.eltwise_binary(a, a[::-1].copy(), (4, 5, 6), (30, 6, 1), (30, 6, 1), "add")
    assert np.array_equal(got, A + A[::-1])
    got = ref.eltwise_binary(a, row, (4, 5, 6), (30, 6, 1), (0, 0, 1), "add", relu_=True)
    assert np.array_equal(got, np.maximum(A + row.astype(np.float64), 0.0))
    got = ref.eltwise_binary(a, col, (4, 5, 6), (30, 6, 1), (1, 0, 0), "mul")
    assert np.array_equal(got, A * col.astype(np.float64))
    sq = f32(rng.normal(size=(7, 7)))
    got = ref.eltwise_binary(sq, sq, (7, 7), (7, 1), (1, 7), "mul")
    assert np.array_equal(got, sq.astype(np.float64) * sq.T.astype(np.float64))
    # closed forms: x + 0 = x, x * 1 = x, relu(x * -1) = relu(-x); an fp32 product is exact in fp64
    z = np.zeros(1, np.float32); one = np.ones(1, np.float32); neg = -one
    assert np.array_equal(ref.eltwise_binary(a, z, (4, 5, 6), (30, 6, 1), (0, 0, 0), "add"), A)
    assert np.array_equal(ref.eltwise_binary(a, one, (4, 5, 6), (30, 6, 1), (0, 0, 0), "mul"), A)
    assert np.array_equal(ref.eltwise_binary(a, neg, (4, 5, 6), (30, 6, 1), (0, 0, 0), "mul", relu_=True), np.maximum(-A, 0.0))
    x = f32([1.0000001, 3.3333333]); y = f32([1.0000002, 0.3333333])
    assert np.array_equal(ref.eltwise_binary(x, y, (2,), (1,), (1,), "mul"), x.astype(np.float64) * y.astype(np.float64))


# ------------------------------------------------ elementwise chains (add, sub, mul, div, sqrt, sin, cos, ...)
def emap(a, unary=(), binary=None, b=None, scale=1.0):
    """contiguous 1-D helper around ref.eltwise_map; a scalar b is broadcast"""
    a = f32(a).reshape(-1)
    if binary is None:
        return ref.eltwise_map(a, (a.size,), (1,), unary, scale=scale)
    b = f32(b).reshape(-1)
    return ref.eltwise_map(a, (a.size,), (1,), unary, binary, b, (0,) if b.size == 1 else (1,), scale)


def test_eltwise_map_known_values():
    assert np.array_equal(emap([4.0, 2.25, 0.0, 1e-10 ** 2], ["sqrt"]), np.array([2.0, 1.5, 0.0, float(np.float32(1e-20)) ** 0.5]))
    assert np.array_equal(emap([0.0], ["sin"]), [0.0]) and np.array_equal(emap([0.0], ["cos"]), [1.0])
    assert np.array_equal(emap([0.0], ["exp"]), [1.0]) and np.array_equal(emap([0.0], ["tanh"]), [0.0])
    assert np.array_equal(emap([0.0], ["sigmoid"]), [0.5])
    assert abs(emap([1.0], ["exp"])[0] - math.e) < 1e-15
    # first-order expansions around pi/6 and pi/2 at the fp32 arguments: tell sin from cos and fix the signs
    x6 = float(np.float32(math.pi / 6)); d6 = x6 - math.pi / 6
    assert abs(emap([x6], ["sin"])[0] - (0.5 + math.sqrt(3) / 2 * d6)) < 1e-14
    assert abs(emap([x6], ["cos"])[0] - (math.sqrt(3) / 2 - 0.5 * d6)) < 1e-14
    x2 = float(np.float32(math.pi / 2)); d2 = x2 - math.pi / 2
    assert abs(emap([x2], ["sin"])[0] - 1.0) < 1e-14 and abs(emap([x2], ["cos"])[0] + d2) < 1e-14
    assert abs(emap([-x2], ["sin"])[0] + 1.0) < 1e-14
    # relu and scale
    assert np.array_equal(emap([-2.0, 0.0, 3.0], ["relu"]), [0.0, 0.0, 3.0])
    assert np.array_equal(emap([-2.0, 0.5], ["scale"], scale=-4.0), [8.0, -2.0])
    assert np.array_equal(emap([-2.0, 0.5, 6.0, 7.5], ["relu6"]), [0.0, 0.5, 6.0, 6.0])
    assert np.array_equal(emap([-2.0, 0.5, 6.0, 7.5], ["relu6"]), ref.relu6(np.array([-2.0, 0.5, 6.0, 7.5])))
    # the constant is the fp32 one
    assert emap([1.0], ["scale"], scale=0.1)[0] == float(np.float32(0.1))


def test_eltwise_map_identities():
    x = f32(rng.normal(size=4000) * 3.0)
    X = x.astype(np.float64)
    s, c = emap(x, ["sin"]), emap(x, ["cos"])
    assert np.max(np.abs(s * s + c * c - 1.0)) < 1e-15 * 4
    # angle addition with an independent second angle: sin(x + y) from the pieces
    y = f32(rng.normal(size=4000))
    xy = (X + y.astype(np.float64)).astype(np.float32)      # the sum as fp32 input, its exact value used below
    dx = xy.astype(np.float64) - X                            # = the second angle actually added
    sd, cd = np.sin(dx), np.cos(dx)                           # small independent angles (library witness)
    assert np.max(np.abs(emap(xy, ["sin"]) - (s * cd + c * sd))) < 1e-14
    assert np.max(np.abs(emap(xy, ["cos"]) - (c * cd - s * sd))) < 1e-14
    p = f32(rng.uniform(0.01, 50.0, size=4000))
    r = emap(p, ["sqrt"])
    assert np.max(np.abs(r * r - p.astype(np.float64)) / p) < 1e-15 * 2 and np.all(r > 0)
    e, en = emap(x, ["exp"]), emap(-x, ["exp"])
    assert np.max(np.abs(e * en - 1.0)) < 1e-15 * 4
    assert np.max(np.abs(emap(x, ["scale", "exp"], scale=2.0) - e * e) / (e * e)) < 1e-15 * 4     # exp(2x) = exp(x)^2
    # tanh and the logistic function from exp, through chains of their own
    e2 = emap(x, ["scale", "exp"], scale=2.0)
    assert np.max(np.abs(emap(x, ["tanh"]) - (e2 - 1.0) / (e2 + 1.0))) < 1e-15 * 4
    sg = emap(x, ["sigmoid"])
    assert np.max(np.abs(sg - 1.0 / (1.0 + en))) < 1e-15
    assert np.max(np.abs(sg + emap(-x, ["sigmoid"]) - 1.0)) < 1e-15
    assert np.max(np.abs(sg - 0.5 * (1.0 + emap(x, ["scale", "tanh"], scale=0.5)))) < 1e-15 * 2
    # the GELU step is the tanh-form GELU pinned above
    assert np.array_equal(emap(x, ["gelu"]), ref.gelu_tanh(X))


def test_eltwise_map_binary_ops_and_step_order():
    a = f32(rng.normal(size=3000)); b = f32(rng.uniform(0.5, 3.0, size=3000) * rng.choice([-1.0, 1.0], size=3000))
    A, B = a.astype(np.float64), b.astype(np.float64)
    # an fp32 sum, difference and product are exact in fp64
    assert np.array_equal(emap(a, (), "add", b), A + B) and np.array_equal(emap(a, (), "mul", b), A * B)
    sub = emap(a, (), "sub", b)
    assert np.array_equal(sub, -emap(b, (), "sub", a)) and np.array_equal(sub, emap(a, (), "add", -b))
    assert np.array_equal(emap(a, (), "sub", a), np.zeros(3000))
    q = emap(a, (), "div", b)
    assert np.max(np.abs(q * B - A) / np.abs(A)) < 1e-15 * 2
    assert np.array_equal(emap(b, (), "div", b), np.ones(3000))
    assert np.array_equal(emap([1.0, 3.0], (), "div", [2.0]), [0.5, 1.5])          # a / b, not b / a; scalar broadcast
    assert np.array_equal(emap([1.0, 3.0], (), "sub", [2.0]), [-1.0, 1.0])
    # the unary steps run after the binary one, in list order
    assert np.array_equal(emap([3.0, -3.0], ["scale", "relu"], scale=-1.0), [0.0, 3.0])
    assert np.array_equal(emap([3.0, -3.0], ["relu", "scale"], scale=-1.0), [-3.0, 0.0])
    assert np.array_equal(emap([3.0, 0.25], ["relu", "sqrt"], "sub", [-1.0]), [2.0, math.sqrt(1.25)])
    assert np.array_equal(emap([5.0, 1.0], ["relu"], "sub", [3.0]), [2.0, 0.0])
    # agrees with the two-operand routine pinned above on its cases
    assert np.array_equal(emap(a, ["relu"], "add", b), ref.eltwise_binary(a, b, (3000,), (1,), (1,), "add", True))
    assert np.array_equal(emap(a, ["relu"], "mul", b), ref.eltwise_binary(a, b, (3000,), (1,), (1,), "mul", True))


def test_eltwise_map_views_by_brute_force():
    a = f32(rng.normal(size=(5, 6, 7))); b = f32(rng.uniform(1.0, 2.0, size=(7, 5)))
    # a permuted to (7, 5, 6) = strides (1, 42, 7); b [7,5] broadcast over the last dim = strides (5, 1, 0)
    got = ref.eltwise_map(a, (7, 5, 6), (1, 42, 7), ["scale"], "div", b, (5, 1, 0), scale=2.0)
    for i in range(7):
        for j in range(5):
            for k in range(6):
                assert got[i, j, k] == float(a[j, k, i]) / float(b[i, j]) * 2.0
    # one operand only: a strided slice, every second column of rows 1..3
    m = f32(rng.uniform(0.0, 9.0, size=(4, 10)))
    got = ref.eltwise_map(m.reshape(-1)[10:], (3, 5), (10, 2), ["sqrt"])
    assert np.array_equal(got, np.sqrt(m[1:, ::2].astype(np.float64)))


def test_scale_const_is_multiplication_by_the_fp32_constant():
    z = rng.normal(size=(5, 7))
    assert np.array_equal(ref.scale_const(z, 1.0), z)
    assert np.array_equal(ref.scale_const(z, -4.0), -4.0 * z)            # a power of two: exact
    assert np.array_equal(ref.scale_const(ref.scale_const(z, 0.5), 8.0), 4.0 * z)
    assert np.array_equal(ref.scale_const(np.ones(3), 0.1), np.full(3, float(np.float32(0.1))))
    assert np.array_equal(ref.scale_const(np.array([2.0, -3.0]), 1.5), [3.0, -4.5])


# ------------------------------------------------ grouped / depthwise conv, relu6
def test_grouped_conv_is_the_dense_conv_with_block_diagonal_weights():
    x = f32(rng.normal(size=(2, 6, 7, 9)))
    for groups, K in ((1, 4), (2, 4), (3, 6), (6, 6), (6, 12)):
        Cg, Kg = 6 // groups, K // groups
        w = f32(rng.normal(size=(K, Cg, 3, 3))); b = f32(rng.normal(size=K))
        dense = np.zeros((K, 6, 3, 3), np.float32)          # block diagonal: zero outside each group's channels
        for k in range(K):
            g = k // Kg
            dense[k, g * Cg:(g + 1) * Cg] = w[k]
        for stride, pad, dil in ((1, 1, 1), (2, 1, 1), (1, 2, 2), (1, 0, 1)):
            got, Dg = ref.conv2d_nchw_grouped(x, w, b, stride, pad, groups, want_norm=True, dil=dil)
            want, Dw = ref.conv2d_nchw_bias(x, dense, b, stride, pad, want_norm=True, dil=dil)
            assert got.shape == want.shape
            assert np.max(np.abs(got - want)) < 1e-13 and np.max(np.abs(Dg - Dw)) < 1e-13


def test_depthwise_conv_closed_forms_and_brute_force():
    x = f32(rng.normal(size=(2, 5, 6, 8)))
    # centre-tap delta filters scaled per channel: out[n,c] = s_c * in[n,c]
    s = f32(rng.normal(size=5))
    w = np.zeros((5, 1, 3, 3), np.float32); w[:, 0, 1, 1] = s
    got = ref.conv2d_nchw_grouped(x, w, None, 1, 1, groups=5)
    assert np.array_equal(got, x.astype(np.float64) * s.astype(np.float64)[None, :, None, None])
    # off-centre tap (kh=0, kw=1): out[h][w] = in[h-1][w], zero in the first row; channels never mix
    w = np.zeros((5, 1, 3, 3), np.float32); w[:, 0, 0, 1] = 1.0
    got = ref.conv2d_nchw_grouped(x, w, None, 1, 1, groups=5)
    assert np.array_equal(got[:, :, 1:, :], x[:, :, :-1, :].astype(np.float64)) and np.all(got[:, :, 0, :] == 0)
    # all-ones: counts the taps inside the image (9 interior, 6 edges, 4 corners), independent of C
    ones = np.ones((1, 3, 5, 5), np.float32)
    got = ref.conv2d_nchw_grouped(ones, np.ones((3, 1, 3, 3), np.float32), None, 1, 1, groups=3)
    assert got[0, 1, 2, 2] == 9 and got[0, 2, 0, 2] == 6 and got[0, 0, 0, 0] == 4
    # brute force, stride 2, with bias
    w = f32(rng.normal(size=(5, 1, 3, 3))); b = f32(rng.normal(size=5))
    got = ref.conv2d_nchw_grouped(x, w, b, 2, 1, groups=5)
    assert got.shape == (2, 5, 3, 4)
    for n, c, h, ww in itertools.product(range(2), range(5), range(3), range(4)):
        acc = float(b[c])
        for kh in range(3):
            for kw in range(3):
                ih, iw = 2 * h - 1 + kh, 2 * ww - 1 + kw
                if 0 <= ih < 6 and 0 <= iw < 8:
                    acc += float(x[n, c, ih, iw]) * float(w[c, 0, kh, kw])
        assert abs(got[n, c, h, ww] - acc) < 1e-13


def test_relu6_clamps_both_ends():
    assert np.array_equal(ref.relu6(np.array([-3.0, -0.0, 0.5, 6.0, 6.5, 1e9])), [0.0, 0.0, 0.5, 6.0, 6.0, 6.0])


# ------------------------------------------------ transposed conv
def test_conv_transpose_is_the_adjoint_of_the_conv():
    # <conv(x, w), y> = <x, conv_transpose(y, w')> with w' = w seen as [C_of_y = K][K_of_result = C][R][S]:
    # the defining property, for strides, paddings and dilations
    for (C, K, H, W, R, stride, pad, dil) in [(3, 4, 7, 8, 3, 1, 1, 1), (2, 5, 9, 9, 3, 2, 1, 1), (4, 2, 10, 7, 5, 2, 2, 1),
                                              (2, 3, 11, 12, 3, 1, 2, 2), (3, 3, 8, 8, 1, 1, 0, 1), (1, 2, 13, 9, 3, 3, 0, 1)]:
        w = f32(rng.normal(size=(K, C, R, R)))
        Hy, Wy = ref.conv_out_hw(H, W, R, R, stride, pad, dil)
        # the transposed conv (no extra output padding) produces the smallest input size that gives Hy x Wy; with
        # stride > 1 that can be up to stride - 1 rows / columns short of H x W, so x is zero there
        Ht, Wt = ref.conv_transpose_out_hw(Hy, Wy, R, R, stride, pad, dil)
        assert Ht <= H and Wt <= W and H - Ht < stride and W - Wt < stride
        x = f32(rng.normal(size=(2, C, H, W)))
        x[:, :, Ht:, :] = 0.0
        x[:, :, :, Wt:] = 0.0
        y = f32(rng.normal(size=(2, K, Hy, Wy)))
        lhs = float(np.sum(ref.conv2d_nchw_bias(x, w, None, stride, pad, dil=dil) * y.astype(np.float64)))
        # the transposed conv of y maps K channels back to C: its weight tensor [K][C][R][S] is w itself
        xt = ref.conv_transpose2d_nchw(y, w, None, stride, pad, dil=dil)
        assert xt.shape == (2, C, Ht, Wt)
        rhs = float(np.sum(xt * x[:, :, :Ht, :Wt].astype(np.float64)))
        assert abs(lhs - rhs) < 1e-10 * max(1.0, abs(lhs))


def test_conv_transpose_closed_forms_and_brute_force():
    x = f32(rng.normal(size=(2, 3, 5, 6)))
    # stride 1: a conv with the filter flipped, input and output channels swapped, padding R - 1 - P
    w = f32(rng.normal(size=(3, 4, 3, 3))); b = f32(rng.normal(size=4))
    got = ref.conv_transpose2d_nchw(x, w, b, 1, 1)
    wf = np.ascontiguousarray(w[:, :, ::-1, ::-1].transpose(1, 0, 2, 3))
    assert np.max(np.abs(got - ref.conv2d_nchw_bias(x, wf, b, 1, 3 - 1 - 1))) < 1e-13
    # 1x1 filter, stride 2: the input lands on the even positions, the rest is the bias
    w1 = f32(rng.normal(size=(3, 2, 1, 1)))
    got = ref.conv_transpose2d_nchw(x, w1, f32([0.5, -1.0]), 2, 0)
    assert got.shape == (2, 2, 9, 11)
    mix = np.einsum("nchw,ck->nkhw", x.astype(np.float64), w1[:, :, 0, 0].astype(np.float64))
    assert np.max(np.abs(got[:, :, ::2, ::2] - (mix + np.array([0.5, -1.0])[None, :, None, None]))) < 1e-13
    assert np.all(got[:, 0, 1::2, :] == 0.5) and np.all(got[:, 1, :, 1::2] == -1.0)
    # all-ones 2x2 filter at stride 2 tiles the output: every output is one input (no overlaps)
    ones = np.ones((1, 1, 2, 2), np.float32)
    got = ref.conv_transpose2d_nchw(x[:1, :1], ones, None, 2, 0)
    assert np.array_equal(got[0, 0], np.kron(x[0, 0].astype(np.float64), np.ones((2, 2))))
    # brute force over the scatter definition, stride 2, padding 1, with the magnitude sum
    w = f32(rng.normal(size=(3, 2, 3, 3)))
    got, Dn = ref.conv_transpose2d_nchw(x, w, None, 2, 1, want_norm=True)
    want = np.zeros(got.shape); mag = np.zeros(got.shape)
    for n, c, ih, iw, k, kh, kw in itertools.product(range(2), range(3), range(5), range(6), range(2), range(3), range(3)):
        oh, ow = 2 * ih - 1 + kh, 2 * iw - 1 + kw
        if 0 <= oh < got.shape[2] and 0 <= ow < got.shape[3]:
            want[n, k, oh, ow] += float(x[n, c, ih, iw]) * float(w[c, k, kh, kw])
            mag[n, k, oh, ow] += abs(float(x[n, c, ih, iw])) * abs(float(w[c, k, kh, kw]))
    assert np.max(np.abs(got - want)) < 1e-13 and np.max(np.abs(Dn - mag)) < 1e-13
