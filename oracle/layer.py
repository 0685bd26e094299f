"""CPU oracle for the rest of the decoder layer around the four linears (numpy, fp64).

TEST INFRASTRUCTURE ONLY, like the rest of this package: imported by tests/, smoke() and the
cpu_baseline leg of bench.py; the product never imports it and it imports nothing from the product.

What a decoder layer computes is the published pre-LayerNorm transformer decoder block that the
paper's models (OPT, BLOOM) share; LLM-PQ (arXiv 2403.01136) itself adds the per-layer weight
bitwidth (Sec. 4.3) and the pre-allocated KV cache of s + n positions (Sec. 4.1, "KV Storage
Modeling"; Sec. 5).  Each operator below is its textbook definition written out, in fp64:
  layer normalisation   y = (x - mean) / sqrt(var + eps) * gamma + beta, biased variance over the
                        hidden dimension (Ba, Kiros, Hinton 2016, Eq. 3-4)
  attention             softmax(q . k / sqrt(d) + bias) . v per head, a query at position p seeing the
                        cached positions 0..p (Vaswani et al. 2017, Sec. 3.2.1 and the decoder mask of
                        Sec. 3.2.3); optional linear position bias slope_h * (j - p) (Press et al. 2022)
  activation            ReLU, or the tanh form of GELU (Hendrycks, Gimpel 2016, Sec. 2)
Activations travel between operators as fp16 (as in the served models): `decoder_layer` rounds every
operator's output to fp16 before the next one reads it, and each operator is exact fp64 in between.
"""
import math

import numpy as np


def f64(a):
    return np.asarray(a, dtype=np.float64)


def round_fp16(a):
    """fp64 -> nearest fp16 (ties to even) -> fp64: the precision activations have between operators."""
    return np.asarray(a, dtype=np.float64).astype(np.float16).astype(np.float64)


def layernorm(x, gamma, beta, eps):
    """x [M][h]; statistics per row over h; returns fp64 [M][h]."""
    x = f64(x)
    mean = x.mean(axis=1, keepdims=True)
    var = ((x - mean) ** 2).mean(axis=1, keepdims=True)
    return (x - mean) / np.sqrt(var + eps) * f64(gamma)[None, :] + f64(beta)[None, :]


def activation(x, kind):
    x = f64(x)
    if kind == "relu":
        return np.maximum(x, 0.0)
    if kind == "gelu_tanh":
        return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))
    raise ValueError(kind)


def kv_append(k_cache, vt_cache, qkv, n_seqs, T, pos0, n_heads):
    """Write the K and V parts of qkv [n_seqs*T][3h] (token-major; per token q | k | v, heads of d each)
    into the caches at positions pos0 .. pos0+T-1.  k_cache [B][H][S][d]; vt_cache [B][H][d][S] (V is kept
    transposed).  In place; values are copied unchanged."""
    h = qkv.shape[1] // 3
    d = h // n_heads
    q3 = qkv.reshape(n_seqs, T, 3, n_heads, d)
    for b in range(n_seqs):
        for t in range(T):
            k_cache[b, :, pos0 + t, :] = q3[b, t, 1]
            vt_cache[b, :, :, pos0 + t] = q3[b, t, 2]


def attention(qkv, k_cache, vt_cache, n_seqs, T, pos0, n_heads, alibi_slopes=None):
    """Causal attention of the T new tokens of each sequence over cache positions 0 .. pos0+t.
    qkv [n_seqs*T][3h] supplies the queries; the caches must already hold positions < pos0+T.
    Returns fp64 [n_seqs*T][h] (heads concatenated)."""
    h = qkv.shape[1] // 3
    d = h // n_heads
    q = f64(qkv).reshape(n_seqs, T, 3, n_heads, d)[:, :, 0]
    K, VT = f64(k_cache), f64(vt_cache)
    out = np.zeros((n_seqs, T, n_heads, d))
    for b in range(n_seqs):
        for hd in range(n_heads):
            for t in range(T):
                p = pos0 + t
                s = K[b, hd, :p + 1, :] @ q[b, t, hd] / math.sqrt(d)
                if alibi_slopes is not None:
                    s = s + float(alibi_slopes[hd]) * (np.arange(p + 1) - p)
                w = np.exp(s - s.max())
                w /= w.sum()
                out[b, t, hd] = VT[b, hd, :, :p + 1] @ w
    return out.reshape(n_seqs * T, h)


def decoder_layer(x, lin, ln1, ln2, k_cache, vt_cache, n_seqs, T, pos0, n_heads, eps, act, alibi_slopes=None):
    """One pre-LayerNorm decoder layer on x [n_seqs*T][h] (fp16 values).
    lin(name, a) -> fp64 result of linear `name` in {"qkv","out","fc1","fc2"} on fp16-valued input a (the
    caller binds the quantised-linear oracle and the weights); ln1, ln2 = (gamma, beta).
    Updates the caches in place (with the fp16-rounded K and V) and returns the fp16-rounded output as fp64."""
    x = f64(x)
    h1 = round_fp16(layernorm(x, ln1[0], ln1[1], eps))
    qkv = round_fp16(lin("qkv", h1))
    kv_append(k_cache, vt_cache, qkv, n_seqs, T, pos0, n_heads)
    a = round_fp16(attention(qkv, k_cache, vt_cache, n_seqs, T, pos0, n_heads, alibi_slopes))
    x1 = round_fp16(x + lin("out", a))                       # residual added before the one rounding
    h2 = round_fp16(layernorm(x1, ln2[0], ln2[1], eps))
    f = round_fp16(activation(lin("fc1", h2), act))          # activation applied before the one rounding
    return round_fp16(x1 + lin("fc2", f))
