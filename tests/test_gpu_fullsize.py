"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times.

The stage is drawn on the GPU (seeded), quantised by the HIP kernel and run through
lpq_stage_linears exactly as bench.py does.  The oracle then recomputes, from the same fp16 bytes,
  - the packed bytes, scales and zeros of sampled 64-row bands of every linear (bit-exact), and
  - the outputs of sampled (token, output row) pairs: all rows of those bands x sampled tokens,
so every linear of every layer is checked at its real shape; one Freivalds projection per storage
variant (and decode micro-batch) covers every output column of a linear.  Every configuration runs as a
whole stage at every micro-batch of its sweep."""
import numpy as np
import pytest

import paper_2403_01136_amd as lpq
from paper_2403_01136_amd import workloads as wl
from gpu_util import MAX_ABS_FRAC, REL_L2_TOL, u16

pytestmark = pytest.mark.gpu
TILE_BYTES = {3: 768, 4: 1024, 8: 2048, 16: 4096}


def _bands(N, seed):
    nb = N // 64
    rng = np.random.default_rng(seed)
    picks = {0, nb - 1, int(rng.integers(0, nb)), int(rng.integers(0, nb))}
    return sorted(picks)


def _tokens(M, seed):
    if M <= 48:
        return list(range(M))
    rng = np.random.default_rng(seed)
    return sorted({0, 1, 15, 16, 31, 32, 63, 64, 127, 128, M - 1, *[int(t) for t in rng.integers(0, M, 20)]} & set(range(M)))


def _check_linear(orc, qw, w_dev, x_dev, y_dev, bits, scheme, seed, what, check_packed=True):
    import torch
    N, K = w_dev.shape
    M = x_dev.shape[0]
    KT = K // 128
    bands = _bands(N, seed)
    rows = np.concatenate([np.arange(64 * b, 64 * b + 64) for b in bands])
    w_rows = w_dev[torch.from_numpy(rows).cuda()].cpu().numpy()              # [64 * len(bands)][K] fp16
    if check_packed:
        p, s, z = orc.quantize_pack(w_rows, bits, scheme)
        band_bytes = KT * 4 * TILE_BYTES[bits]
        codes = qw.codes.cpu().numpy()
        for i, b in enumerate(bands):
            got = codes[b * band_bytes:(b + 1) * band_bytes]
            assert np.array_equal(got, p[i * band_bytes:(i + 1) * band_bytes]), "%s: packed bytes of band %d differ" % (what, b)
        if scheme == 1:
            gs, gz = u16(qw.scales).reshape(KT, N)[:, rows], u16(qw.zeros).reshape(KT, N)[:, rows]
            assert np.array_equal(gs, s) and np.array_equal(gz, z), "%s: scales / zeros differ" % what
        elif scheme == 2:
            assert np.array_equal(u16(qw.scales)[rows], s), "%s: row scales differ" % what
    toks = _tokens(M, seed + 1)
    x_rows = x_dev[torch.tensor(toks).cuda()].cpu().numpy()
    ref = orc.qlinear(x_rows, w_rows, bits, scheme)                           # fp64 [tokens][rows]
    y = y_dev[torch.tensor(toks).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(y)), what
    rel = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert rel <= REL_L2_TOL, "%s rel-L2 %.3e" % (what, rel)
    assert np.abs(y - ref).max() <= MAX_ABS_FRAC * np.abs(ref).max(), what


def _freivalds(orc, w_dev, x_dev, y_dev, bits, scheme, seed, what):
    """sum_n y[m,n] r[n] == x[m,:] . (W~^T r) for random signs r, over every output column."""
    import torch
    N, K = w_dev.shape
    wd = orc.dequant_weights(w_dev.cpu().numpy(), bits, scheme).astype(np.float64)     # oracle, all rows
    rng = np.random.default_rng(seed)
    r = rng.choice([-1.0, 1.0], N)
    toks = _tokens(x_dev.shape[0], seed + 2)
    x_rows = x_dev[torch.tensor(toks).cuda()].cpu().numpy().astype(np.float64)
    want = x_rows @ (wd.T @ r)
    y = y_dev[torch.tensor(toks).cuda()].cpu().numpy().astype(np.float64)
    got = y @ r
    # each y carries an fp16 rounding (2^-11 relative) and the kernel's error budget; the signed sum of N
    # such errors grows like sqrt(N) times the typical |y|
    tol = 4e-3 * np.sqrt(N) * np.sqrt(np.mean(y * y, axis=1)) + 1e-6
    assert np.all(np.abs(got - want) <= tol), "%s: projection off by %.3e (tol %.3e)" % (what, np.abs(got - want).max(), tol.min())


def _run_config(orc, cfg, layer_ids, decode_Ms, Mp, freivalds_linear="out"):
    """Build the stage once (as bench.py does), then run it at every decode micro-batch of `decode_Ms` and at the
    prefill micro-batch Mp; every linear of every layer is checked at each of them."""
    import torch
    dev = torch.device("cuda:0")
    shapes = wl.linear_shapes(cfg)
    sub = dict(cfg, layers=[cfg["layers"][i] for i in layer_ids])
    layers, ws = [], []
    for li, (bits, scheme) in zip(layer_ids, sub["layers"]):
        lw, lws = {}, {}
        for name in wl.LINEARS:
            K, N = shapes[name]
            w = wl.weight_torch(N, K, dev, cfg["name"], li, name)
            lw[name] = lpq.lpq_quantize_pack(w, bits, scheme)
            lws[name] = w
        layers.append(lw), ws.append(lws)
    seen_variants = set()
    phases = [(lpq.LPQ_DECODE, M) for M in decode_Ms] + [(lpq.LPQ_PREFILL, Mp)]
    for pi, (phase, M) in enumerate(phases):
        xs, ys = [], []
        for li in layer_ids:
            x_h = wl.act_torch(M, cfg["h"], cfg["act_outliers"], dev, cfg["name"], li, "h", M)
            x_f = wl.act_torch(M, cfg["f"], cfg["act_outliers"], dev, cfg["name"], li, "f", M)
            xs.append({n: (x_f if n == "fc2" else x_h) for n in wl.LINEARS})
            ys.append({n: torch.full((M, shapes[n][1]), float("nan"), dtype=torch.float16, device=dev) for n in wl.LINEARS})
        lpq.lpq_stage_linears(lpq.Stage(layers, xs, ys), phase)
        torch.cuda.synchronize()
        for i, (li, (bits, scheme)) in enumerate(zip(layer_ids, sub["layers"])):
            for name in wl.LINEARS:
                what = "%s layer %d %s %d-bit phase %d M=%d" % (cfg["name"], li, name, bits, phase, M)
                assert not torch.isnan(ys[i][name]).any(), what + ": output not fully written"
                _check_linear(orc, layers[i][name], ws[i][name], xs[i][name], ys[i][name], bits, scheme,
                              1000 * li + len(name) + 17 * pi, what, check_packed=(pi == 0))
            if (bits, scheme, phase, min(M, 64)) not in seen_variants:
                seen_variants.add((bits, scheme, phase, min(M, 64)))
                n = freivalds_linear
                _freivalds(orc, ws[i][n], xs[i][n], ys[i][n], bits, scheme, 77 + li, "%s layer %d %s phase %d M=%d" % (cfg["name"], li, n, phase, M))
        del xs, ys


def test_bench_config_full_stage(orc):
    """configs[1]: all 8 layers x 4 linears, decode M=16 and prefill M=2048, as bench.py runs them."""
    cfg = wl.CONFIGS[1]
    _run_config(orc, cfg, list(range(len(cfg["layers"]))), cfg["decode_Ms"], cfg["prefill_M"])


@pytest.mark.parametrize("ci", [2, 3, 4], ids=["opt30b_12_layers", "opt66b_10_layers", "bloom176b_10_layers"])
def test_other_configs_whole_stage(orc, ci):
    """configs[2..4] as whole stages, at every decode micro-batch of their sweeps and at their prefill micro-batch:
    the launch plan (even-share ranges, workgroups per XCD, one decode launch of up to 48 linears -- configs[2] has
    48 -- and one prefill launch per storage variant) depends on the whole list of linears, so a sub-stage would test
    another plan."""
    cfg = wl.CONFIGS[ci]
    _run_config(orc, cfg, list(range(len(cfg["layers"]))), cfg["decode_Ms"], cfg["prefill_M"])


@pytest.mark.parametrize("bits,scheme", [(3, 1), (4, 1), (8, 1), (8, 2), (16, 0)], ids=["w3", "w4", "w8", "i8", "f16"])
def test_single_linear_launches_at_layer_shapes(orc, bits, scheme):
    """One linear per launch, as a decoder layer issues them (OPT-13B shapes): the decode phase then runs in the
    small-launch kernel (a workgroup per group of 2-5 tiles, one or two token tiles; FC2 K-split with its reduce kernel), the prefill phase K-splits
    the launches with few tiles.  Sampled bands and tokens against the oracle, one projection over every column."""
    import torch
    cfg = wl.CONFIGS[1]
    dev = torch.device("cuda:0")
    shapes = wl.linear_shapes(cfg)
    for name in wl.LINEARS:
        K, N = shapes[name]
        w = wl.weight_torch(N, K, dev, "single", bits, name)
        bias = (torch.arange(N, device=dev) % 9 - 4).to(torch.float16) * 0.25
        qw = lpq.lpq_quantize_pack(w, bits, scheme, bias=bias)
        w_host_bias = bias.cpu().numpy()
        for fn, M in ((lpq.lpq_qlinear_decode, 16), (lpq.lpq_qlinear_decode, 5), (lpq.lpq_qlinear_decode, 27), (lpq.lpq_qlinear_prefill, 512),
                      (lpq.lpq_qlinear_prefill, 2048)):
            x = wl.act_torch(M, K, True, dev, "single", name, M)
            y = torch.full((M, N), float("nan"), dtype=torch.float16, device=dev)
            fn(qw, x, y)
            torch.cuda.synchronize()
            what = "single %s %d-bit %s M=%d" % (name, bits, fn.__name__, M)
            assert not torch.isnan(y).any(), what + ": output not fully written"
            y_nobias = (y.float() - bias.float()[None, :]).to(torch.float64)      # the checks below compare x . w~^T
            bands = _bands(N, 5 + M)
            rows = np.concatenate([np.arange(64 * b, 64 * b + 64) for b in bands])
            toks = _tokens(M, 6 + M)
            ref = orc.qlinear(x[torch.tensor(toks).cuda()].cpu().numpy(), w[torch.from_numpy(rows).cuda()].cpu().numpy(), bits, scheme,
                              w_host_bias[rows])
            got = y[torch.tensor(toks).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
            rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
            assert rel <= REL_L2_TOL, "%s rel-L2 %.3e" % (what, rel)
            assert np.abs(got - ref).max() <= MAX_ABS_FRAC * np.abs(ref).max(), what
            if name == "out" and M in (16, 512):
                _freivalds(orc, w, x, y_nobias.to(torch.float16), bits, scheme, 99 + M, what)
        del w, qw
