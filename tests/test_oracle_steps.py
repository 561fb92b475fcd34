"""Pins for the single steps of the CPU oracle: brute force on tiny inputs,
closed forms, tabulated values, index arithmetic.  None of these re-type the
oracle's vectorised formula; each is chosen so that a dropped term, a wrong
sign/index or a transposed operand fails."""
import math

import numpy as np
import pytest

from oracle import epd_oracle as O


def _read_golden(name):
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", name)
    rows = []
    with open(path) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append([float(v) for v in line.split()])
    return rows


# ------------------------------------------------------------- linear ----

@pytest.mark.parametrize("m,k,n", [(7, 588, 5), (33, 72, 19), (3, 269, 4), (1, 1, 1)])
def test_linear_vs_triple_loop(m, k, n):
    rng = np.random.default_rng(m * 1000 + k)
    x = rng.standard_normal((m, k))
    W = rng.standard_normal((n, k))
    b = rng.standard_normal(n)
    want = [[0.0] * n for _ in range(m)]
    for i in range(m):
        for j in range(n):
            acc = 0.0
            for t in range(k):
                acc += float(x[i, t]) * float(W[j, t])   # W is [out, in]
            want[i][j] = acc + float(b[j])
    np.testing.assert_allclose(O.linear(x, W, b), np.array(want), rtol=1e-12, atol=1e-12)


def test_linear_one_hot_weight_selects_input_column():
    x = np.arange(12.0).reshape(3, 4)
    W = np.zeros((2, 4)); W[0, 3] = 1.0; W[1, 1] = -2.0
    y = O.linear(x, W, np.array([10.0, 0.0]))
    np.testing.assert_array_equal(y[:, 0], x[:, 3] + 10.0)
    np.testing.assert_array_equal(y[:, 1], -2.0 * x[:, 1])


# -------------------------------------------------------------- norms ----

def test_layer_norm_closed_forms():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 37)) * 3 + 1.5
    eps = 1e-6
    y = O.layer_norm(x, np.ones(37), np.zeros(37), eps)
    np.testing.assert_allclose(y.mean(-1), 0.0, atol=1e-12)
    var = x.var(-1)                       # biased
    np.testing.assert_allclose(y.var(-1), var / (var + eps), rtol=1e-12)
    # constant row -> beta exactly; gain multiplies, shift adds
    beta = rng.standard_normal(37)
    gamma = rng.standard_normal(37)
    yc = O.layer_norm(np.full((1, 37), 4.25), gamma, beta, eps)
    np.testing.assert_allclose(yc[0], beta, atol=1e-12)
    y2 = O.layer_norm(x, gamma, beta, eps)
    np.testing.assert_allclose(y2, y * gamma + beta, rtol=1e-12, atol=1e-12)


def test_layer_norm_two_element_row_by_hand():
    # row (1, 3): mean 2, biased var 1 -> (-1, 1)/sqrt(1+eps)
    eps = 0.21
    y = O.layer_norm(np.array([[1.0, 3.0]]), np.array([2.0, 2.0]), np.array([0.5, 0.5]), eps)
    s = 1.0 / math.sqrt(1.0 + eps)
    np.testing.assert_allclose(y[0], [-2.0 * s + 0.5, 2.0 * s + 0.5], rtol=1e-14)


def test_rms_norm_closed_forms():
    eps = 1e-6
    gamma = np.array([1.0, 2.0, -3.0, 0.5])
    x = np.array([[1.0, -1.0, 1.0, -1.0]])
    y = O.rms_norm(x, gamma, eps)
    np.testing.assert_allclose(y[0], gamma * x[0] / math.sqrt(1.0 + eps), rtol=1e-14)
    # (3, 4): mean square 12.5; no mean subtraction, no shift
    y = O.rms_norm(np.array([[3.0, 4.0]]), np.ones(2), 0.0)
    np.testing.assert_allclose(y[0], [3.0 / math.sqrt(12.5), 4.0 / math.sqrt(12.5)], rtol=1e-14)
    # scale invariance up to eps
    rng = np.random.default_rng(1)
    v = rng.standard_normal((3, 16))
    np.testing.assert_allclose(O.rms_norm(7.0 * v, np.ones(16), 0.0), O.rms_norm(v, np.ones(16), 0.0), rtol=1e-12)


# --------------------------------------------------------------- GELU ----

def test_gelu_erf_against_tabulated_normal_cdf():
    # x * Phi(x), Phi from standard normal tables (Abramowitz & Stegun 26.2)
    for x, phi in _read_golden("normal_cdf.txt"):
        assert abs(float(O.gelu_erf(np.array(x))) - x * phi) < 5e-10, x
        # Phi(-x) = 1 - Phi(x)
        assert abs(float(O.gelu_erf(np.array(-x))) - (-x) * (1.0 - phi)) < 5e-10, x


def test_gelu_erf_against_math_erf_scalar_grid():
    for i in range(-60, 61):
        x = i / 7.0
        want = 0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))
        assert abs(float(O.gelu_erf(np.array(x))) - want) < 1e-14


def test_gelu_limits_and_identities():
    for f in (O.gelu_erf, O.gelu_tanh):
        assert float(f(np.array(0.0))) == 0.0
        assert abs(float(f(np.array(12.0))) - 12.0) < 1e-9
        assert abs(float(f(np.array(-12.0)))) < 1e-9
        # gelu(x) - gelu(-x) = x  (Phi(x) + Phi(-x) = 1; tanh is odd)
        xs = np.linspace(-5, 5, 41)
        np.testing.assert_allclose(f(xs) - f(-xs), xs, atol=1e-12)


def test_gelu_tanh_scalar_formula_and_distance_to_erf():
    c = math.sqrt(2.0 / math.pi)
    for i in range(-40, 41):
        x = i / 5.0
        want = 0.5 * x * (1.0 + math.tanh(c * (x + 0.044715 * x * x * x)))
        assert abs(float(O.gelu_tanh(np.array(x))) - want) < 1e-14
    # the tanh form is an approximation of the erf form: close, not equal
    xs = np.linspace(-4, 4, 161)
    d = np.abs(O.gelu_tanh(xs) - O.gelu_erf(xs))
    assert 1e-5 < d.max() < 1e-3


# ------------------------------------------------------------ softmax ----

def test_softmax_rows():
    s = np.array([[0.0, math.log(2.0), math.log(5.0)], [1000.0, 1000.0, 1000.0]])
    p = O.softmax_rows(s)
    np.testing.assert_allclose(p[0], [1 / 8, 2 / 8, 5 / 8], rtol=1e-14)
    np.testing.assert_allclose(p[1], [1 / 3] * 3, rtol=1e-14)      # no overflow


# ---------------------------------------------------------- attention ----

def _attention_brute(q, k, v, heads):
    N, D = q.shape
    hd = D // heads
    out = np.zeros((N, D))
    for h in range(heads):
        for i in range(N):
            logits = []
            for j in range(N):
                acc = 0.0
                for d in range(hd):
                    acc += q[i, h * hd + d] * k[j, h * hd + d]
                logits.append(acc / math.sqrt(hd))
            mx = max(logits)
            e = [math.exp(z - mx) for z in logits]
            tot = sum(e)
            for d in range(hd):
                out[i, h * hd + d] = sum(e[j] / tot * v[j, h * hd + d] for j in range(N))
    return out


@pytest.mark.parametrize("N,heads,hd", [(4, 1, 8), (16, 3, 8), (16, 2, 72), (9, 2, 16), (32, 1, 128)])
def test_attention_vs_brute_force(N, heads, hd):
    rng = np.random.default_rng(N + hd)
    q, k, v = (rng.standard_normal((N, heads * hd)) for _ in range(3))
    np.testing.assert_allclose(O.attention(q, k, v, heads), _attention_brute(q, k, v, heads),
                               rtol=1e-11, atol=1e-12)


def test_attention_equal_keys_gives_mean_of_values():
    rng = np.random.default_rng(0)
    N, H, hd = 12, 2, 8
    q = rng.standard_normal((N, H * hd))
    k = np.tile(rng.standard_normal((1, H * hd)), (N, 1))
    v = rng.standard_normal((N, H * hd))
    want = np.tile(v.mean(0, keepdims=True), (N, 1))
    np.testing.assert_allclose(O.attention(q, k, v, H), want, rtol=1e-12, atol=1e-12)


def test_attention_dominant_key_selects_its_value_row():
    N, H, hd = 8, 1, 4
    q = np.ones((N, hd))
    k = np.zeros((N, hd)); k[5] = 400.0           # logit 800 vs 0
    v = np.arange(N * hd, dtype=float).reshape(N, hd)
    np.testing.assert_allclose(O.attention(q, k, v, H), np.tile(v[5], (N, 1)), rtol=1e-12)


def test_attention_identity_values_return_probabilities_and_scale():
    # N = hd, V = I  ->  output row i is softmax(q_i . k_j / sqrt(hd)) over j
    N = hd = 4
    q = np.zeros((N, hd)); q[:, 0] = 2.0           # logits: 2 * k_j0 / sqrt(4) = k_j0
    k = np.zeros((N, hd)); k[:, 0] = [0.0, math.log(2.0), math.log(3.0), math.log(4.0)]
    out = O.attention(q, k, np.eye(N), 1)
    np.testing.assert_allclose(out, np.tile(np.array([1, 2, 3, 4]) / 10.0, (N, 1)), rtol=1e-13)


def test_attention_heads_do_not_mix():
    rng = np.random.default_rng(5)
    N, H, hd = 6, 3, 4
    q, k, v = (rng.standard_normal((N, H * hd)) for _ in range(3))
    base = O.attention(q, k, v, H)
    k2 = k.copy(); k2[2, hd:2 * hd] += 1.0         # touch one key of head 1 only
    out = O.attention(q, k2, v, H)
    np.testing.assert_array_equal(out[:, :hd], base[:, :hd])
    np.testing.assert_array_equal(out[:, 2 * hd:], base[:, 2 * hd:])
    assert np.abs(out[:, hd:2 * hd] - base[:, hd:2 * hd]).max() > 1e-3


# ----------------------------------------------------------- patchify ----

@pytest.mark.parametrize("S,p", [(28, 14), (224, 14), (448, 14), (8, 2)])
def test_patchify_index_arithmetic(S, p):
    c, r, col = np.meshgrid(np.arange(3), np.arange(S), np.arange(S), indexing="ij")
    tile = (c * S * S + r * S + col).astype(np.float64)   # pixel value encodes its own index
    a = O.patchify(tile, p)
    g = S // p
    assert a.shape == (g * g, 3 * p * p)
    rng = np.random.default_rng(S)
    for _ in range(200):
        y, x = rng.integers(0, g, 2)
        ch = rng.integers(0, 3); dy, dx = rng.integers(0, p, 2)
        want = ch * S * S + (p * y + dy) * S + (p * x + dx)
        assert a[y * g + x, (ch * p + dy) * p + dx] == want
    # a permutation of the pixels: nothing lost, nothing duplicated
    assert np.array_equal(np.sort(a.ravel()), np.arange(3 * S * S, dtype=np.float64))


def test_patch_and_token_counts():
    assert O.patchify(np.zeros((3, 448, 448)), 14).shape == (1024, 588)
    assert O.patchify(np.zeros((3, 224, 224)), 14).shape == (256, 588)

    class D:  # minimal description
        tile_size, patch, pixel_shuffle, proj_kind, proj_mid = 448, 14, 1, O.PROJ_MLP, 4096
    assert O.tokens_per_tile(D) == 256
    D.pixel_shuffle = 0
    assert O.tokens_per_tile(D) == 1024
    D.proj_kind, D.proj_mid = O.PROJ_RESAMPLER, 64     # one token per learned query
    assert O.tokens_per_tile(D) == 64


# ------------------------------------------------------ pixel shuffle ----

def _shuffle_brute(x, g):
    N, D = x.shape
    out = np.empty((N // 4, 4 * D), dtype=x.dtype)
    for Y in range(g // 2):
        for X in range(g // 2):
            for dy in range(2):
                for dx in range(2):
                    for c in range(D):
                        out[Y * (g // 2) + X, (dy * 2 + dx) * D + c] = x[(2 * Y + dy) * g + (2 * X + dx), c]
    return out


@pytest.mark.parametrize("g,D", [(4, 3), (2, 1), (6, 5), (32, 2)])
def test_pixel_shuffle_brute_force_and_bijection(g, D):
    x = np.arange(g * g * D, dtype=np.int64).reshape(g * g, D)   # element value = its flat index
    y = O.pixel_shuffle_half(x, g)
    assert y.shape == (g * g // 4, 4 * D)
    np.testing.assert_array_equal(y, _shuffle_brute(x, g))
    assert np.array_equal(np.sort(y.ravel()), np.arange(g * g * D))  # exact permutation


def test_pixel_shuffle_inverse_recovers_input():
    g, D = 8, 4
    rng = np.random.default_rng(2)
    x = rng.standard_normal((g * g, D))
    y = O.pixel_shuffle_half(x, g)
    back = np.empty_like(x)
    h = g // 2
    for m in range(h * h):
        Y, X = divmod(m, h)
        for blk in range(4):
            dy, dx = divmod(blk, 2)
            back[(2 * Y + dy) * g + 2 * X + dx] = y[m, blk * D:(blk + 1) * D]
    np.testing.assert_array_equal(back, x)
