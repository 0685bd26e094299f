"""Pins of oracle/layer.py against what the definitions and the mathematics fix (no GPU).

Each operator is checked against something other than itself: closed forms, invariants, special
cases with a known answer, and a brute-force scalar implementation with Python loops on tiny inputs.
"""
import math

import numpy as np
import pytest

from oracle import layer as L


def rng(seed):
    return np.random.default_rng(seed)


# ---- layer normalisation ---------------------------------------------------------------

def test_layernorm_closed_forms():
    r = rng(1)
    x = r.standard_normal((5, 64)) * 3 + 7
    g, b = np.ones(64), np.zeros(64)
    y = L.layernorm(x, g, b, 1e-5)
    assert np.abs(y.mean(axis=1)).max() < 1e-12                       # centred
    var = x.var(axis=1)
    assert np.allclose(y.var(axis=1), var / (var + 1e-5), rtol=1e-12)  # scaled by 1/sqrt(var+eps)
    # affine part: gamma scales, beta shifts, per column
    g2, b2 = r.standard_normal(64), r.standard_normal(64)
    assert np.allclose(L.layernorm(x, g2, b2, 1e-5), y * g2 + b2, rtol=1e-12, atol=1e-12)
    # a constant row has no deviation: the output is beta
    assert np.allclose(L.layernorm(np.full((2, 64), 3.25), g2, b2, 1e-5), np.tile(b2, (2, 1)))
    # eps = 0: invariant to shifting and scaling a row
    assert np.allclose(L.layernorm(4 * x - 9, g, b, 0.0), L.layernorm(x, g, b, 0.0), rtol=1e-10, atol=1e-10)


def test_layernorm_scalar_loop():
    r = rng(2)
    x, g, b = r.standard_normal((3, 7)), r.standard_normal(7), r.standard_normal(7)
    y = L.layernorm(x, g, b, 1e-3)
    for m in range(3):
        mu = sum(x[m]) / 7
        var = sum((v - mu) ** 2 for v in x[m]) / 7
        for k in range(7):
            assert abs(y[m, k] - ((x[m, k] - mu) / math.sqrt(var + 1e-3) * g[k] + b[k])) < 1e-12


# ---- activation --------------------------------------------------------------------------

def test_activations():
    x = np.array([-3.0, -0.5, 0.0, 0.5, 3.0])
    assert np.array_equal(L.activation(x, "relu"), [0, 0, 0, 0.5, 3.0])
    g = L.activation(x, "gelu_tanh")
    for xi, gi in zip(x, g):     # the formula, scalar by scalar
        assert abs(gi - 0.5 * xi * (1 + math.tanh(math.sqrt(2 / math.pi) * (xi + 0.044715 * xi ** 3)))) < 1e-15
    assert g[2] == 0.0 and abs(L.activation(np.array([30.0]), "gelu_tanh")[0] - 30.0) < 1e-12
    assert abs(L.activation(np.array([-30.0]), "gelu_tanh")[0]) < 1e-12
    # within 1e-3 of the exact Gaussian form x * Phi(x) it approximates
    xs = np.linspace(-4, 4, 81)
    exact = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in xs])
    assert np.abs(L.activation(xs, "gelu_tanh") - exact).max() < 1e-3
    with pytest.raises(ValueError):
        L.activation(x, "swish")


# ---- KV cache and attention ----------------------------------------------------------------

def make_case(seed, B=2, T=3, pos0=4, H=2, d=8, S=12):
    r = rng(seed)
    h = H * d
    k_cache = r.standard_normal((B, H, S, d))
    vt_cache = r.standard_normal((B, H, d, S))
    qkv = r.standard_normal((B * T, 3 * h))
    return qkv, k_cache, vt_cache, B, T, pos0, H, d, S


def test_kv_append_places_rows():
    qkv, K, VT, B, T, pos0, H, d, S = make_case(3)
    K0, VT0 = K.copy(), VT.copy()
    L.kv_append(K, VT, qkv, B, T, pos0, H)
    h = H * d
    for b in range(B):
        for t in range(T):
            row = qkv[b * T + t]
            for hd in range(H):
                assert np.array_equal(K[b, hd, pos0 + t], row[h + hd * d: h + (hd + 1) * d])
                assert np.array_equal(VT[b, hd, :, pos0 + t], row[2 * h + hd * d: 2 * h + (hd + 1) * d])
    mask = np.ones(S, bool)
    mask[pos0:pos0 + T] = False
    assert np.array_equal(K[:, :, mask], K0[:, :, mask]) and np.array_equal(VT[:, :, :, mask], VT0[:, :, :, mask])


def attention_scalar(qkv, K, VT, B, T, pos0, H, d, slopes):
    """Brute force with Python scalars only."""
    h = H * d
    out = np.zeros((B * T, h))
    for b in range(B):
        for t in range(T):
            p = pos0 + t
            for hd in range(H):
                q = qkv[b * T + t][hd * d:(hd + 1) * d]
                s = []
                for j in range(p + 1):
                    v = sum(q[e] * K[b, hd, j, e] for e in range(d)) / math.sqrt(d)
                    if slopes is not None:
                        v += slopes[hd] * (j - p)
                    s.append(v)
                mx = max(s)
                w = [math.exp(v - mx) for v in s]
                z = sum(w)
                for e in range(d):
                    out[b * T + t, hd * d + e] = sum(w[j] * VT[b, hd, e, j] for j in range(p + 1)) / z
    return out


@pytest.mark.parametrize("slopes", [None, [0.5, 0.0625]])
def test_attention_matches_scalar_loops(slopes):
    qkv, K, VT, B, T, pos0, H, d, S = make_case(4)
    L.kv_append(K, VT, qkv, B, T, pos0, H)
    got = L.attention(qkv, K, VT, B, T, pos0, H, slopes)
    assert np.allclose(got, attention_scalar(qkv, K, VT, B, T, pos0, H, d, slopes), rtol=1e-12, atol=1e-12)


def test_attention_special_cases():
    qkv, K, VT, B, T, pos0, H, d, S = make_case(5)
    h = H * d
    L.kv_append(K, VT, qkv, B, T, pos0, H)
    # zero queries: uniform weights, the output is the mean of the visible values
    q0 = qkv.copy()
    q0[:, :h] = 0.0
    out = L.attention(q0, K, VT, B, T, pos0, H)
    for b in range(B):
        for t in range(T):
            for hd in range(H):
                assert np.allclose(out[b * T + t, hd * d:(hd + 1) * d], VT[b, hd, :, :pos0 + t + 1].mean(axis=1))
    # zero queries with a position bias: geometric weights exp(slope * (j - p))
    slopes = [0.7, 0.1]
    out = L.attention(q0, K, VT, B, T, pos0, H, slopes)
    p = pos0 + T - 1
    w = np.exp(slopes[0] * (np.arange(p + 1) - p))
    assert np.allclose(out[T - 1, :d], VT[0, 0, :, :p + 1] @ (w / w.sum()))
    # the future is invisible: changing cache entries past a query's position changes nothing for it
    K2, VT2 = K.copy(), VT.copy()
    K2[:, :, pos0 + 1:] += 5.0
    VT2[:, :, :, pos0 + 1:] -= 3.0
    a, b_ = L.attention(qkv, K, VT, B, T, pos0, H), L.attention(qkv, K2, VT2, B, T, pos0, H)
    first = [bb * T for bb in range(B)]                      # t = 0 sees positions 0..pos0 only
    assert np.array_equal(a[first], b_[first]) and not np.allclose(a[T - 1], b_[T - 1])
    # one key far ahead of the rest takes all the weight
    K3 = K.copy()
    K3[0, 0, 2] = 40.0 * qkv[0, :d] / np.linalg.norm(qkv[0, :d])
    big = L.attention(qkv, K3, VT, B, T, pos0, H)
    assert np.allclose(big[0, :d], VT[0, 0, :, 2], atol=1e-6)
    # softmax is invariant to a common shift of the scores: add c * q to every visible key of one head
    # changes q.k by c*|q|^2 for all keys alike
    K4 = K.copy()
    K4[0, 0, :pos0 + 1] += 0.3 * qkv[0, :d]
    assert np.allclose(L.attention(qkv, K4, VT, B, T, pos0, H)[0, :d], a[0, :d], rtol=1e-10, atol=1e-12)


# ---- the layer's wiring ----------------------------------------------------------------------

def test_decoder_layer_wiring():
    r = rng(6)
    B, T, pos0, H, d, S = 2, 2, 1, 2, 8, 6
    h, f = H * d, 32
    x = r.standard_normal((B * T, h)).astype(np.float16).astype(np.float64)
    W = {"qkv": r.standard_normal((3 * h, h)) * 0.2, "out": r.standard_normal((h, h)) * 0.2,
         "fc1": r.standard_normal((f, h)) * 0.2, "fc2": r.standard_normal((h, f)) * 0.2}
    ln = (np.ones(h), np.zeros(h))
    K, VT = np.zeros((B, H, S, d)), np.zeros((B, H, d, S))
    K[:, :, :pos0] = r.standard_normal((B, H, pos0, d))
    VT[:, :, :, :pos0] = r.standard_normal((B, H, d, pos0))

    def run(weights, act="relu"):
        k, v = K.copy(), VT.copy()
        return L.decoder_layer(x, lambda n, a: a @ weights[n].T, ln, ln, k, v, B, T, pos0, H, 1e-5, act), k, v

    # no contribution from either branch: the residual stream passes through unchanged
    zero = {n: np.zeros_like(w) for n, w in W.items()}
    y, _, _ = run(zero)
    assert np.array_equal(y, x)
    # only the attention branch: y = fp16(x + out(attn)), rebuilt here from the pinned operators
    only_attn = dict(W, fc2=np.zeros_like(W["fc2"]))
    y, k, v = run(only_attn)
    h1 = L.round_fp16(L.layernorm(x, *ln, 1e-5))
    qkv = L.round_fp16(h1 @ W["qkv"].T)
    k2, v2 = K.copy(), VT.copy()
    L.kv_append(k2, v2, qkv, B, T, pos0, H)
    a = L.round_fp16(L.attention(qkv, k2, v2, B, T, pos0, H))
    assert np.array_equal(y, L.round_fp16(x + a @ W["out"].T))
    assert np.array_equal(k, k2) and np.array_equal(v, v2)
    # only the feed-forward branch, both activations
    for act in ("relu", "gelu_tanh"):
        only_ffn = dict(W, out=np.zeros_like(W["out"]))
        y, _, _ = run(only_ffn, act)
        h2 = L.round_fp16(L.layernorm(x, *ln, 1e-5))
        fmid = L.round_fp16(L.activation(h2 @ W["fc1"].T, act))
        assert np.array_equal(y, L.round_fp16(x + fmid @ W["fc2"].T))
    # every intermediate is an fp16 value
    y, _, _ = run(W)
    assert np.array_equal(y, y.astype(np.float16).astype(np.float64))
