"""GPU parity of the rest of the decoder layer (layer norm, KV append, attention, fused epilogues and the
whole layer) against oracle/layer.py, operator by operator on the same fp16 inputs and end to end.

Operators: fp16 outputs within rel-L2 <= 1e-3 and max-abs <= 1e-2 * max|ref| of the fp64 oracle; the
KV append is a copy and must be bit-exact.  The whole layer chains eight roundings to fp16, each of
which can flip on a 1-ulp difference upstream, so it is compared at rel-L2 <= 2e-3."""
import numpy as np
import pytest

import paper_2403_01136_amd as lpq
from paper_2403_01136_amd import workloads as wl
from gpu_util import check_output, to_dev, u16
from oracle import indicator as OI
from oracle import layer as OL

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU (no fallback path)"
    lpq.load_library()


def f16(a):
    return np.asarray(a, dtype=np.float32).astype(np.float16)


def rng(*key):
    return np.random.default_rng(wl.stream_seed("layer", *key))


@pytest.mark.parametrize("M,h", [(1, 64), (5, 768), (33, 5120), (3, 14336)])
def test_layernorm(M, h):
    r = rng("ln", M, h)
    x = f16(r.standard_normal((M, h)) * 2 + 0.5)
    x[:, :3] *= 30                                        # outlier channels
    g, b = f16(1 + 0.1 * r.standard_normal(h)), f16(0.1 * r.standard_normal(h))
    y = lpq.lpq_layernorm(to_dev(x), to_dev(g), to_dev(b), 1e-5)
    check_output(y, OL.layernorm(x, g, b, 1e-5), "layernorm %dx%d" % (M, h))


@pytest.mark.parametrize("act", [lpq.LPQ_ACT_RELU, lpq.LPQ_ACT_GELU_TANH, lpq.LPQ_ACT_NONE], ids=["relu", "gelu", "none"])
@pytest.mark.parametrize("phase,M", [(lpq.LPQ_DECODE, 7), (lpq.LPQ_DECODE, 40), (lpq.LPQ_PREFILL, 70)], ids=["dec7", "dec40", "pre70"])
def test_fused_epilogue(orc, act, phase, M):
    """act(x . w^T + bias) + residual with one rounding, also when a unit is cut (long K) and in place."""
    import torch
    N, K = 192, 4096
    w = wl.weight_np(N, K, "fused")
    x = wl.act_np(M, K, False, "fused", M)
    r = rng("fused", M)
    bias, res = f16(0.1 * r.standard_normal(N)), f16(r.standard_normal((M, N)))
    qw = lpq.lpq_quantize_pack(to_dev(w), 4, 1, bias=to_dev(bias))
    ref = orc.qlinear(x, w, 4, 1, bias)
    kind = {lpq.LPQ_ACT_RELU: "relu", lpq.LPQ_ACT_GELU_TANH: "gelu_tanh"}.get(act)
    ref = (OL.activation(ref, kind) if kind else ref) + res.astype(np.float64)
    y = to_dev(res).clone()                               # in place: the residual is the output buffer
    lpq.lpq_qlinear_fused(qw, to_dev(x), phase, activation=act, residual=y, y=y)
    check_output(y, ref, "fused epilogue")


def make_state(B, H, d, S, seed, alibi=False, act=lpq.LPQ_ACT_RELU):
    import torch
    r = rng("state", seed)
    h = H * d
    ln = [(f16(1 + 0.1 * r.standard_normal(h)), f16(0.05 * r.standard_normal(h))) for _ in range(2)]
    slopes = (2.0 ** (-8.0 * (np.arange(H) + 1) / H)).astype(np.float32) if alibi else None
    st = lpq.LayerState(H, d, S, B, torch.device("cuda"), tuple(to_dev(a) for a in ln[0]), tuple(to_dev(a) for a in ln[1]),
                        activation=act, alibi_slopes=None if slopes is None else to_dev(slopes))
    return st, ln, slopes


@pytest.mark.parametrize("d", [64, 128])
def test_kv_append_bit_exact(d):
    import torch
    B, H, S, T, pos0 = 3, 5, 128, 7, 40
    st, _, _ = make_state(B, H, d, S, d)
    r = rng("kv", d)
    qkv = f16(r.standard_normal((B * T, 3 * H * d)))
    k0, v0 = f16(r.standard_normal((B, H, S, d))), f16(r.standard_normal((B, H, d, S)))
    st.k_cache.copy_(to_dev(k0)), st.vt_cache.copy_(to_dev(v0))
    lpq.lpq_kv_append(to_dev(qkv), st, B, T, pos0)
    OL.kv_append(k0, v0, qkv, B, T, pos0, H)
    assert np.array_equal(u16(st.k_cache), k0.view(np.uint16)) and np.array_equal(u16(st.vt_cache), v0.view(np.uint16))


@pytest.mark.parametrize("alibi", [False, True], ids=["plain", "alibi"])
@pytest.mark.parametrize("B,H,d,S,T,pos0", [
    (2, 3, 64, 128, 1, 0), (16, 5, 128, 640, 1, 599), (1, 2, 128, 4160, 1, 4100), (3, 4, 64, 256, 1, 77),      # decode
    (2, 3, 128, 256, 100, 0), (1, 2, 64, 320, 130, 150), (2, 2, 128, 128, 16, 5), (1, 1, 128, 64, 3, 0),        # prefill
], ids=["dec_first", "dec_B16_L600", "dec_split_L4101", "dec_d64", "pre_T100", "pre_chunk_d64", "pre_T16", "pre_T3"])
def test_attention(B, H, d, S, T, pos0, alibi):
    import torch
    st, _, slopes = make_state(B, H, d, S, T, alibi)
    r = rng("att", B, H, d, T, pos0)
    qkv = f16(r.standard_normal((B * T, 3 * H * d)))
    qkv[:, :H * d] *= 2.0                                  # sharper softmax
    k = f16(r.standard_normal((B, H, S, d)))
    vt = f16(r.standard_normal((B, H, d, S)))
    k[:, :, pos0 + T:], vt[:, :, :, pos0 + T:] = np.nan, np.nan          # unwritten positions must never matter
    st.k_cache.copy_(to_dev(k)), st.vt_cache.copy_(to_dev(vt))
    lpq.lpq_kv_append(to_dev(qkv), st, B, T, pos0)
    out = lpq.lpq_attention(to_dev(qkv), st, B, T, pos0)
    OL.kv_append(k, vt, qkv, B, T, pos0, H)
    ref = OL.attention(qkv, k[:, :, :pos0 + T], vt[:, :, :, :pos0 + T], B, T, pos0, H, slopes)
    check_output(out, ref, "attention B%d H%d d%d T%d pos0 %d" % (B, H, d, T, pos0))


@pytest.mark.parametrize("bits,scheme,act,alibi", [(4, 1, lpq.LPQ_ACT_RELU, False), (3, 1, lpq.LPQ_ACT_GELU_TANH, True),
                                                   (8, 2, lpq.LPQ_ACT_RELU, False), (16, 0, lpq.LPQ_ACT_RELU, False)],
                         ids=["w4_relu", "w3_gelu_alibi", "i8_relu", "fp16_relu"])
def test_decoder_layer_prefill_then_decode(orc, bits, scheme, act, alibi):
    """A prompt of s tokens in the prefill phase, then three decode steps, against the oracle layer."""
    import torch
    B, H, d, S, s_len, f = 2, 4, 64, 128, 37, 512
    h = H * d
    st, ln, slopes = make_state(B, H, d, S, bits, alibi, act)
    r = rng("layer", bits, scheme)
    shapes = {"qkv": (h, 3 * h), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
    W = {n: f16(r.standard_normal((N, K)) * (1.0 / np.sqrt(K))) for n, (K, N) in shapes.items()}
    bias = {n: f16(0.05 * r.standard_normal(N)) for n, (K, N) in shapes.items()}
    layer = {n: lpq.lpq_quantize_pack(to_dev(W[n]), bits, scheme, bias=to_dev(bias[n])) for n in shapes}
    kind = "relu" if act == lpq.LPQ_ACT_RELU else "gelu_tanh"
    k_ref, vt_ref = np.zeros((B, H, S, d), np.float16), np.zeros((B, H, d, S), np.float16)

    def lin(name, a):
        return orc.qlinear(a.astype(np.float16), W[name], bits, scheme, bias[name])

    ws = None
    pos = 0
    for step, (phase, T) in enumerate([(lpq.LPQ_PREFILL, s_len)] + [(lpq.LPQ_DECODE, 1)] * 3):
        x = f16(r.standard_normal((B * T, h)))
        y, ws = lpq.lpq_decoder_layer(layer, st, phase, B, T, pos, to_dev(x), workspace=ws if step > 1 else None)
        ref = OL.decoder_layer(x, lin, ln[0], ln[1], k_ref, vt_ref, B, T, pos, H, 1e-5, kind, slopes)
        yd = y.cpu().numpy().astype(np.float64)
        rel = np.linalg.norm(yd - ref) / np.linalg.norm(ref)
        assert np.all(np.isfinite(yd)) and rel <= 2e-3, "step %d rel-L2 %.3e" % (step, rel)
        assert np.abs(yd - ref).max() <= 1e-2 * np.abs(ref).max()
        # the caches hold what the oracle's hold, up to the fp16 rounding of qkv (compared as values)
        kd = st.k_cache.cpu().numpy().astype(np.float64)[:, :, :pos + T]
        assert np.linalg.norm(kd - k_ref[:, :, :pos + T].astype(np.float64)) <= 2e-3 * np.linalg.norm(kd)
        pos += T


def test_decoder_layer_at_the_benchmark_shape(orc):
    """One 4-bit OPT-13B-shaped layer (h = 5120, 40 heads of 128, f = 20480) at the two points bench.py and the cost
    model time: a prefill of 4 prompts x 512 tokens, and a decode step of 16 sequences at position 562.  The oracle
    layer runs on what it can finish in seconds: the first 48 tokens of the second prompt (a causal layer's output
    for a token depends on no later token, so that prefix is a prefill of its own), and two of the sixteen sequences
    of the decode step over the 562 cached positions (the cache is filled with seeded values)."""
    import torch
    B, H, d, f, s_len, n_gen = 4, 40, 128, 20480, 512, 100
    h, S, bits, scheme = H * d, 640, 4, 1
    st, ln, _ = make_state(16, H, d, S, "bench_shape")
    r = rng("bench_shape")
    shapes = {"qkv": (h, 3 * h), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
    W = {n: f16(r.standard_normal((N, K), dtype=np.float32) * np.float32(1.0 / np.sqrt(K))) for n, (K, N) in shapes.items()}
    bias = {n: f16(0.05 * r.standard_normal(N)) for n, (K, N) in shapes.items()}
    layer = {n: lpq.lpq_quantize_pack(to_dev(W[n]), bits, scheme, bias=to_dev(bias[n])) for n in shapes}

    def lin(name, a):
        return orc.qlinear(a.astype(np.float16), W[name], bits, scheme, bias[name])

    def compare(y_rows, ref, what):
        yd = y_rows.astype(np.float64)
        rel = np.linalg.norm(yd - ref) / np.linalg.norm(ref)
        assert np.all(np.isfinite(yd)) and rel <= 2e-3, "%s rel-L2 %.3e" % (what, rel)
        assert np.abs(yd - ref).max() <= 1e-2 * np.abs(ref).max(), what

    # prefill: 4 x 512 tokens
    x = f16(r.standard_normal((B * s_len, h), dtype=np.float32))
    y, ws = lpq.lpq_decoder_layer(layer, st, lpq.LPQ_PREFILL, B, s_len, 0, to_dev(x))
    seq, T_chk = 1, 48
    rows = slice(seq * s_len, seq * s_len + T_chk)
    k_ref, vt_ref = np.zeros((1, H, S, d), np.float16), np.zeros((1, H, d, S), np.float16)
    ref = OL.decoder_layer(x[rows], lin, ln[0], ln[1], k_ref, vt_ref, 1, T_chk, 0, H, 1e-5, "relu")
    compare(y[rows].cpu().numpy(), ref, "prefill 4 x 512, prompt %d, first %d tokens" % (seq, T_chk))
    kd = st.k_cache[seq, :, :T_chk].cpu().numpy().astype(np.float64)
    assert np.linalg.norm(kd - k_ref[0, :, :T_chk].astype(np.float64)) <= 2e-3 * np.linalg.norm(kd)

    # decode: 16 sequences at position s + n / 2
    n_seq, pos = 16, s_len + n_gen // 2
    k0 = f16(r.standard_normal((n_seq, H, S, d), dtype=np.float32))
    v0 = f16(r.standard_normal((n_seq, H, d, S), dtype=np.float32))
    st.k_cache.copy_(to_dev(k0)), st.vt_cache.copy_(to_dev(v0))
    xd = f16(r.standard_normal((n_seq, h), dtype=np.float32))
    yd, _ = lpq.lpq_decoder_layer(layer, st, lpq.LPQ_DECODE, n_seq, 1, pos, to_dev(xd))
    yd = yd.cpu().numpy()
    for b in (0, 9):
        kb, vb = k0[b:b + 1].copy(), v0[b:b + 1].copy()
        ref = OL.decoder_layer(xd[b:b + 1], lin, ln[0], ln[1], kb, vb, 1, 1, pos, H, 1e-5, "relu")
        compare(yd[b:b + 1], ref, "decode step, sequence %d of 16 at position %d" % (b, pos))
        assert np.array_equal(u16(st.k_cache[b, :, pos]), kb[0, :, pos].view(np.uint16)) or \
            np.linalg.norm(st.k_cache[b, :, pos].cpu().numpy().astype(np.float64) - kb[0, :, pos].astype(np.float64)) <= 2e-3 * np.linalg.norm(kb[0, :, pos].astype(np.float64))


@pytest.mark.parametrize("stochastic", [False, True], ids=["deterministic", "stochastic"])
@pytest.mark.parametrize("N,K,M", [(1, 128, 1), (70, 640, 33), (5120, 5120, 16), (333, 14336, 5)])
def test_variance_indicator(N, K, M, stochastic):
    """All eight forms of D_W * S_W(b)^2 * G(X) against the fp64 oracle (reductions in fp32 / fp64: 1e-5)."""
    w = wl.weight_np(N, K, "ind", N, K)
    x = wl.act_np(M, K, True, "ind", M)
    if stochastic:
        x = (x.astype(np.float32) + 0.75).astype(np.float16)          # a mean that matters
    got = lpq.lpq_variance_indicator(to_dev(w), to_dev(x), stochastic).cpu().numpy()
    ref = OI.indicator(w, x, stochastic)
    for i, key in enumerate(OI.ORDER):
        assert abs(got[i] - ref[key]) <= 1e-5 * abs(ref[key]) + 1e-300, (key, got[i], ref[key])


def test_decoder_layer_decode_step_in_a_hip_graph(orc):
    """A decode step of the layer captured once (after an eager warm-up, so that nothing is allocated during
    capture) and replayed several times, with eager work and synchronisations between the replays: every
    replay must reproduce the eager result bit for bit, caches included."""
    import torch
    B, H, d, S, f, pos = 4, 4, 64, 128, 512, 40
    h = H * d
    st, ln, _ = make_state(B, H, d, S, "graph")
    r = rng("graph")
    shapes = {"qkv": (h, 3 * h), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
    layer = {n: lpq.lpq_quantize_pack(to_dev(f16(r.standard_normal((N, K)) / np.sqrt(K))), 4, 1) for n, (K, N) in shapes.items()}
    st.k_cache.copy_(to_dev(f16(r.standard_normal((B, H, S, d)))))
    st.vt_cache.copy_(to_dev(f16(r.standard_normal((B, H, d, S)))))
    x = to_dev(f16(r.standard_normal((B, h))))
    y_eager, ws = lpq.lpq_decoder_layer(layer, st, lpq.LPQ_DECODE, B, 1, pos, x)          # warm-up: workspaces exist now
    torch.cuda.synchronize()
    k_eager, v_eager = st.k_cache.clone(), st.vt_cache.clone()
    y_graph = torch.empty_like(y_eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            lpq.lpq_decoder_layer(layer, st, lpq.LPQ_DECODE, B, 1, pos, x, y_graph, ws, stream=side)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(4):
        y_graph.fill_(float("nan"))
        st.k_cache[:, :, pos].fill_(0), st.vt_cache[:, :, :, pos].fill_(0)                 # the step must rewrite its position
        other = lpq.lpq_qlinear_decode(layer["fc1"], x)                                     # eager work between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(u16(y_graph), u16(y_eager)), "replay %d" % replay
        assert torch.equal(st.k_cache, k_eager) and torch.equal(st.vt_cache, v_eager), "replay %d caches" % replay
        assert torch.isfinite(other).all()
