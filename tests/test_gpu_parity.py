"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bit-exact for codes, scales, zeros, packed words and the fp32 dequantised weights; fp16 outputs
within rel-L2 <= 1e-3 and max-abs <= 1e-2 * max|ref| of the oracle's fp64 result.
Shapes span several 64x128 blocks, ragged row blocks (N not a multiple of the workgroups' 256 rows), ragged token counts, split-K, and the first configuration at full size."""
import numpy as np
import pytest

import paper_2403_01136_amd as lpq
from paper_2403_01136_amd import workloads as wl
from gpu_util import VARIANTS, VARIANT_IDS, check_output, check_packed, to_dev, u16

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU (no fallback path)"
    lpq.load_library()


# ---- a1 + a2: quantise and pack ---------------------------------------------------------

@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("N,K", [(64, 128), (192, 384), (320, 1280)])
def test_quantize_pack_bit_exact(orc, bits, scheme, N, K):
    w = wl.weight_np(N, K, "qp", bits, scheme, N, K)
    qw = lpq.lpq_quantize_pack(to_dev(w), bits, scheme)
    check_packed(qw, orc, w)
    deq = lpq.lpq_unpack_dequant(qw).cpu().numpy()
    assert np.array_equal(deq.view(np.uint32), orc.dequant_weights(w, bits, scheme).view(np.uint32))


@pytest.mark.parametrize("bits,scheme", VARIANTS[:4], ids=VARIANT_IDS[:4])
def test_quantize_pack_edge_groups(orc, bits, scheme):
    """Flat groups, -0/+0, exact grids, ranges whose fp16 scale is subnormal or underflows,
    large magnitudes: bit-equality with the oracle is all that is asked here."""
    rng = np.random.default_rng(5)
    N, K = 64, 1024
    w = wl.weight_np(N, K, "edge", bits, scheme).astype(np.float32)
    w[:, 0:128] = 0.0
    w[:, 128:256] = 0.37
    w[:, 256:384] = -0.0
    w[3, 256] = 0.0
    w[:, 384:512] = (np.arange(128) % 16) * 0.125 - 0.9375
    tiny = rng.integers(0, 40, (N, 128)).astype(np.uint16).view(np.float16).astype(np.float32)
    w[:, 512:640] = tiny                                  # fp16 subnormals: scale subnormal or zero
    w[:, 640:768] = tiny * 64 - 3e-5
    w[:, 768:896] = rng.standard_normal((N, 128)) * 2000   # large magnitudes
    w[:, 896:1024] = np.abs(w[:, 896:1024])               # all positive
    w[5, :] = 0.0                                          # a whole flat row (per-row scheme)
    w = w.astype(np.float16)
    qw = lpq.lpq_quantize_pack(to_dev(w), bits, scheme)
    check_packed(qw, orc, w)
    deq = lpq.lpq_unpack_dequant(qw).cpu().numpy()
    assert np.array_equal(deq.view(np.uint32), orc.dequant_weights(w, bits, scheme).view(np.uint32))


# ---- quantise a weight piecewise, and stream it from host memory (Sec. 5, on-the-fly quantizer) ----

@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
def test_quantize_pack_rows_any_order(orc, bits, scheme):
    """Row windows quantised out of order, from buffers that hold only those rows, give the same packed
    weight as one call over the whole matrix (and the oracle)."""
    import torch
    N, K = 448, 384
    w = wl.weight_np(N, K, "rows", bits, scheme)
    qw = lpq.QWeight(bits, scheme, K, N, torch.device("cuda"))
    for t in (qw.codes, qw.scales, qw.zeros):
        if t is not None:
            t.view(torch.uint8).fill_(0xA5)
    for row0, n_rows in ((256, 192), (0, 64), (64, 0), (128, 128), (64, 64)):
        lpq.lpq_quantize_pack_rows(to_dev(w[row0:row0 + n_rows]), qw, row0)
    check_packed(qw, orc, w)


@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("pinned", [True, False], ids=["pinned", "pageable"])
def test_load_quantize_pack_from_host(orc, bits, scheme, pinned):
    """Streaming from host memory through a staging buffer (several bands of rows, a ragged last one) is
    bit-identical to quantising the resident weight; then the linear runs on the result."""
    import torch
    N, K, M = 704, 256, 8
    w = wl.weight_np(N, K, "load", bits, scheme)
    w_host = torch.from_numpy(w.copy())
    if pinned:
        w_host = w_host.pin_memory()
    staging = torch.empty(192 * K * 2 + 300, dtype=torch.uint8, device="cuda")          # 192-row bands: 3 full + 128 rows
    qw = lpq.lpq_load_quantize_pack(w_host, bits, scheme, staging)
    torch.cuda.synchronize()
    check_packed(qw, orc, w)
    x = wl.act_np(M, K, True, "load", M)
    check_output(lpq.lpq_qlinear_decode(qw, to_dev(x)), orc.qlinear(x, w, bits, scheme), "decode after load %d-bit" % bits)


# ---- a3: decode linear ---------------------------------------------------------------------

@pytest.fixture(params=["rows", "rows_3", "rows_5", "even_share"])
def decode_kernel_choice(request):
    """Up to 64 token rows (32 per pass), a launch that streams little goes to the kernel that gives a group of 16-row tiles a
    workgroup, a larger one to the even-share kernel; lpq_set_decode_routing moves the limit, so small shapes can reach both.
    rows_3 / rows_5 ask for groups of 3 / 5 tiles, which cut across the packed layout's 64-row blocks (the library
    falls back to 4 where the group size does not divide a linear's tiles: N = 320 has 20, N = 192 has 12)."""
    if request.param == "even_share":
        lpq.lpq_set_decode_routing(0, 0)
    elif request.param != "rows":
        lpq.lpq_set_decode_routing(-1, int(request.param[-1]))
    yield request.param
    lpq.lpq_set_decode_routing(-1, -1)


@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("M", [1, 2, 5, 16, 17, 32, 33, 64])
def test_decode_small(orc, bits, scheme, M, decode_kernel_choice):
    if M > 64 and decode_kernel_choice != "even_share":
        pytest.skip("more than 64 token rows always take the even-share kernel")
    N, K = 320, 640         # 5 (fp16: 10) row blocks: the last workgroup has idle waves; 5 steps: idle waves in a row block's workgroup
    w = wl.weight_np(N, K, "dec", bits, scheme)
    x = wl.act_np(M, K, True, "dec", M)
    qw = lpq.lpq_quantize_pack(to_dev(w), bits, scheme)
    y = lpq.lpq_qlinear_decode(qw, to_dev(x))
    check_output(y, orc.qlinear(x, w, bits, scheme), "decode %d-bit M=%d" % (bits, M))


@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("M", [3, 21, 70, 130])
def test_decode_split_k_and_many_rows(orc, bits, scheme, M, decode_kernel_choice):
    """K long enough that the work is cut into several K ranges (fp32 partial sums + reduction, or waves that split
    K); M > 64 runs in several passes; a bias is added exactly once."""
    if M > 64 and decode_kernel_choice != "even_share":
        pytest.skip("more than 64 token rows always take the even-share kernel")
    N, K = 192, 16384
    w = wl.weight_np(N, K, "decsk", bits, scheme)
    x = wl.act_np(M, K, True, "decsk", M)
    bias = (np.arange(N) % 7 - 3).astype(np.float16)
    import torch
    qw = lpq.lpq_quantize_pack(to_dev(w), bits, scheme, bias=to_dev(bias))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    lpq.lpq_qlinear_decode(qw, to_dev(x), y)
    check_output(y, orc.qlinear(x, w, bits, scheme, bias), "decode split-K %d-bit M=%d" % (bits, M))


@pytest.mark.parametrize("bits,scheme", [(3, 1), (4, 1), (8, 1), (8, 2)], ids=["w3", "w4", "w8", "i8sym"])
def test_decode_zero_term_rows_of_unlike_magnitude(orc, bits, scheme):
    """Up to 32 token rows the stage-wide kernel adds the zero term once per unit, as a matrix product with the activations'
    group sums held as fp16 pairs scaled per token row.  Rows 2^-11 and 2^5 times the others in one micro-batch: every row
    keeps the tolerance on its own, whatever its neighbours' scale."""
    lpq.lpq_set_decode_routing(0, 0)
    try:
        N, K = 192, 2048
        w = wl.weight_np(N, K, "zrow", bits, scheme)
        for M in (7, 24):
            x = wl.act_np(M, K, False, "zrow", M).astype(np.float32)
            x *= np.array([2.0 ** -11, 1.0, 2.0 ** 5])[np.arange(M) % 3][:, None]
            x = x.astype(np.float16)
            y = lpq.lpq_qlinear_decode(lpq.lpq_quantize_pack(to_dev(w), bits, scheme), to_dev(x))
            ref = orc.qlinear(x, w, bits, scheme)
            for m in range(M):
                check_output(y[m:m + 1], ref[m:m + 1], "decode %d-bit M=%d row %d" % (bits, M, m))
    finally:
        lpq.lpq_set_decode_routing(-1, -1)


@pytest.mark.parametrize("bits,scheme", [(3, 1), (8, 2)], ids=["w3", "i8sym"])
def test_decode_zero_term_very_long_rows(orc, bits, scheme):
    """K = 66048 is 516 groups: more than a thread of the group-sum kernel keeps in registers, so it reads the row twice;
    the 516 groups are also not a multiple of the 16 a matrix instruction of the zero term covers."""
    lpq.lpq_set_decode_routing(0, 0)
    try:
        N, K = 128, 66048
        w = wl.weight_np(N, K, "zlong", bits, scheme)
        for M in (3, 18):
            x = wl.act_np(M, K, True, "zlong", M)
            y = lpq.lpq_qlinear_decode(lpq.lpq_quantize_pack(to_dev(w), bits, scheme), to_dev(x))
            check_output(y, orc.qlinear(x, w, bits, scheme), "decode %d-bit M=%d K=%d" % (bits, M, K))
    finally:
        lpq.lpq_set_decode_routing(-1, -1)


@pytest.mark.parametrize("bits,scheme", [(3, 1), (8, 2)], ids=["w3", "i8"])
def test_decode_longest_rows_and_the_limit_on_k(orc, bits, scheme):
    """The decode kernels' descriptors keep K / 128 in 16 bits.  At the largest K they hold (65535 steps of 128 columns)
    one-hot activation rows read single columns of the dequantised weight out of the product -- first, last and middle
    groups -- and each is compared with the oracle on that group's 128 columns alone (quantisation is per group);
    one step more is refused with LPQ_ERR_UNSUPPORTED and nothing is written."""
    import torch
    N, KT = 64, 65535
    K = KT * 128
    gen = torch.Generator(device="cuda").manual_seed(23)
    w = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float16)
    qw = lpq.lpq_quantize_pack(w, bits, scheme)
    cols = [0, 127, 128, 5 * 128 + 77, (KT // 2) * 128 + 3, (KT - 1) * 128, K - 1]
    x = torch.zeros((len(cols), K), dtype=torch.float16, device="cuda")
    for i, c in enumerate(cols):
        x[i, c] = 1.0 + i / 8.0
    y = lpq.lpq_qlinear_decode(qw, x)
    torch.cuda.synchronize()
    y_host = y.cpu().numpy().astype(np.float64)
    for i, c in enumerate(cols):
        g = c // 128
        if scheme == 2:      # one scale per row over the whole of K: the oracle needs the row's largest magnitude, kept in a 129th group
            wmax = w.abs().amax(dim=1, keepdim=True)
            wg = torch.cat([w[:, g * 128:(g + 1) * 128], wmax.expand(N, 128)], dim=1).cpu().numpy()
            xg = np.zeros((1, 256), dtype=np.float16)
        else:
            wg = w[:, g * 128:(g + 1) * 128].cpu().numpy()
            xg = np.zeros((1, 128), dtype=np.float16)
        xg[0, c % 128] = np.float16(1.0 + i / 8.0)
        ref = orc.qlinear(xg, wg, bits, scheme)
        check_output(torch.from_numpy(y_host[i:i + 1]), ref, "decode %d-bit K=%d, column %d" % (bits, K, c))
    del qw, w, x, y
    K2 = K + 128
    w2 = torch.zeros((N, K2), dtype=torch.float16, device="cuda")
    qw2 = lpq.lpq_quantize_pack(w2, bits, scheme)
    x2 = torch.zeros((2, K2), dtype=torch.float16, device="cuda")
    y2 = torch.full((2, N), float("nan"), dtype=torch.float16, device="cuda")
    with pytest.raises(lpq.LpqError) as err:
        lpq.lpq_qlinear_decode(qw2, x2, y2)
    assert err.value.status == 8
    torch.cuda.synchronize()
    assert torch.isnan(y2).all(), "a refused call wrote outputs"


# ---- a4: prefill linear --------------------------------------------------------------------

@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("M", [1, 7, 128, 130, 300])
def test_prefill_small(orc, bits, scheme, M):
    N, K = 320, 640         # 5 row blocks: the second workgroup has one active wave
    w = wl.weight_np(N, K, "pre", bits, scheme)
    x = wl.act_np(M, K, True, "pre", M)
    bias = (np.arange(N) % 5 - 2).astype(np.float16) if M == 7 else None
    import torch
    qw = lpq.lpq_quantize_pack(to_dev(w), bits, scheme, bias=None if bias is None else to_dev(bias))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    lpq.lpq_qlinear_prefill(qw, to_dev(x), y)
    check_output(y, orc.qlinear(x, w, bits, scheme, bias), "prefill %d-bit M=%d" % (bits, M))


@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("M,K", [(7, 8192), (260, 8192), (300, 4224)])
def test_prefill_split_k(orc, bits, scheme, M, K):
    """Few tiles and a long K: the library cuts K into ranges (fp32 partial sums, second kernel).  K = 4224 is
    33 steps, which no split count divides; the bias is added exactly once."""
    N = 320
    w = wl.weight_np(N, K, "presk", bits, scheme)
    x = wl.act_np(M, K, True, "presk", M)
    bias = (np.arange(N) % 5 - 2).astype(np.float16)
    import torch
    qw = lpq.lpq_quantize_pack(to_dev(w), bits, scheme, bias=to_dev(bias))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    lpq.lpq_qlinear_prefill(qw, to_dev(x), y)
    check_output(y, orc.qlinear(x, w, bits, scheme, bias), "prefill split-K %d-bit M=%d" % (bits, M))


@pytest.mark.parametrize("bits,scheme", VARIANTS, ids=VARIANT_IDS)
@pytest.mark.parametrize("mag", [2.0 ** -12, 2.0 ** -6, 2.0 ** 5], ids=["x_2e-12", "x_2e-6", "x_2e5"])
def test_activation_magnitude(orc, bits, scheme, mag, decode_kernel_choice):
    """The tolerance holds whatever the scale of the activations (tiny ones near the fp16 subnormal
    range, large ones short of overflow in the outputs): no step of the kernels may cost them bits."""
    if decode_kernel_choice in ("rows_3", "rows_5"):
        pytest.skip("N = 128 has 8 tiles: groups of 3 or 5 do not apply")
    N, K = 128, 512
    w = wl.weight_np(N, K, "mag", bits, scheme)
    for M, fn, tag in [(8, lpq.lpq_qlinear_decode, "decode"), (40, lpq.lpq_qlinear_decode, "decode"),
                       (64, lpq.lpq_qlinear_prefill, "prefill")]:
        x = (wl.act_np(M, K, False, "mag", M).astype(np.float32) * mag).astype(np.float16)
        y = fn(lpq.lpq_quantize_pack(to_dev(w), bits, scheme), to_dev(x))
        check_output(y, orc.qlinear(x, w, bits, scheme), "%s %d-bit M=%d x*%g" % (tag, bits, M, mag))


RANDOM_SHAPES = [(N, K, M, v) for i, (N, K, M) in enumerate([
    (192, 4096, 1), (320, 1024, 7), (960, 384, 16), (1280, 1024, 19), (1600, 128, 32), (2048, 2048, 45), (960, 4096, 64),
    (1280, 384, 5), (320, 4096, 27), (1600, 1024, 16), (2048, 128, 3), (192, 2048, 33)]) for v in [VARIANTS[i % len(VARIANTS)]]]


@pytest.mark.parametrize("N,K,M,variant", RANDOM_SHAPES, ids=["N%d_K%d_M%d_%s" % (N, K, M, VARIANT_IDS[VARIANTS.index(v)]) for N, K, M, v in RANDOM_SHAPES])
def test_decode_shapes_that_vary_the_workgroup_plan(orc, N, K, M, variant):
    """A single decode linear picks its workgroup shape from N, K and M (groups of 2-5 tiles, K splits, one or two
    token tiles, one or two passes): shapes whose tile counts divide by 3 or 5 or neither, long and one-step K,
    every range of M, with a bias and a residual, every element against the oracle."""
    import torch
    bits, scheme = variant
    w = wl.weight_np(N, K, "plan", N, K, bits, scheme)
    x = wl.act_np(M, K, True, "plan", N, K, M)
    bias = ((np.arange(N) % 5) - 2).astype(np.float16) * np.float16(0.5)
    res = wl.act_np(M, N, False, "plan-res", N, K, M)
    qw = lpq.lpq_quantize_pack(to_dev(w), bits, scheme, bias=to_dev(bias))
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    lpq.lpq_qlinear_fused(qw, to_dev(x), lpq.LPQ_DECODE, residual=to_dev(res), y=y)
    ref = orc.qlinear(x, w, bits, scheme, bias) + res.astype(np.float64)
    check_output(y, ref, "decode N=%d K=%d M=%d %d-bit" % (N, K, M, bits))


def test_decode_and_prefill_agree_and_are_deterministic(orc):
    N, K, M = 128, 2048, 24
    w = wl.weight_np(N, K, "agree")
    x = to_dev(wl.act_np(M, K, True, "agree"))
    qw = lpq.lpq_quantize_pack(to_dev(w), 4, 1)
    yd1, yd2 = lpq.lpq_qlinear_decode(qw, x), lpq.lpq_qlinear_decode(qw, x)
    yp1, yp2 = lpq.lpq_qlinear_prefill(qw, x), lpq.lpq_qlinear_prefill(qw, x)
    assert np.array_equal(u16(yd1), u16(yd2)) and np.array_equal(u16(yp1), u16(yp2))
    ref = orc.qlinear(x.cpu().numpy(), w, 4, 1)
    check_output(yd1, ref, "decode")
    check_output(yp1, ref, "prefill")


# ---- a5: stage of layers with per-layer bits -----------------------------------------------

def _build_stage(cfg_key, h, f, qkv_n, layer_specs, M, outliers):
    import torch
    shapes = {"qkv": (h, qkv_n), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
    layers, xs, ys, host = [], [], [], []
    for li, (bits, scheme) in enumerate(layer_specs):
        lw, lx, ly, lh = {}, {}, {}, {}
        x_h = wl.act_np(M, h, outliers, cfg_key, li, "h")
        x_f = wl.act_np(M, f, outliers, cfg_key, li, "f")
        xd_h, xd_f = to_dev(x_h), to_dev(x_f)
        for name, (K, N) in shapes.items():
            w = wl.weight_np(N, K, cfg_key, li, name)
            lw[name] = lpq.lpq_quantize_pack(to_dev(w), bits, scheme)
            lx[name] = xd_f if name == "fc2" else xd_h
            ly[name] = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
            lh[name] = (w, x_f if name == "fc2" else x_h)
        layers.append(lw), xs.append(lx), ys.append(ly), host.append(lh)
    return lpq.Stage(layers, xs, ys), ys, host


@pytest.mark.parametrize("phase,M", [(lpq.LPQ_DECODE, 1), (lpq.LPQ_DECODE, 16), (lpq.LPQ_DECODE, 24), (lpq.LPQ_DECODE, 40),
                                     (lpq.LPQ_PREFILL, 128)],
                         ids=["decode_M1", "decode_M16", "decode_M24", "decode_M40", "prefill_M128"])
def test_stage_mixed_bits_small(orc, phase, M, decode_kernel_choice):
    if decode_kernel_choice in ("rows_3", "rows_5"):
        pytest.skip("the stage's linears have 16, 48 and 64 tiles: no group of 3 or 5 fits them all")
    specs = [(16, 0), (8, 1), (4, 1), (3, 1), (8, 2), (3, 1)]
    stage, ys, host = _build_stage("stage_small", 256, 1024, 768, specs, M, True)
    lpq.lpq_stage_linears(stage, phase)
    for li, (bits, scheme) in enumerate(specs):
        for name in wl.LINEARS:
            w, x = host[li][name]
            check_output(ys[li][name], orc.qlinear(x, w, bits, scheme), "layer %d %s" % (li, name))


@pytest.mark.parametrize("phase,M", [(lpq.LPQ_DECODE, 3), (lpq.LPQ_DECODE, 20), (lpq.LPQ_DECODE, 70), (lpq.LPQ_PREFILL, 130), (lpq.LPQ_PREFILL, 300)],
                         ids=["decode_M3", "decode_M20", "decode_M70", "prefill_M130", "prefill_M300"])
def test_stage_with_more_linears_than_one_launch_holds(orc, phase, M, decode_kernel_choice):
    """A stage of 13 layers = 52 linears: a grouped decode launch holds at most 48, so the decode phase takes two
    launches that share the workspace, and a storage variant with more than 40 linears takes two prefill launches
    (here the 4-bit variant has 44).  Every element of every output is checked."""
    if decode_kernel_choice in ("rows_3", "rows_5"):
        pytest.skip("the stage's linears have 16, 32 and 48 tiles: no group of 3 or 5 fits them all")
    specs = [(4, 1)] * 11 + [(3, 1)] * 2
    stage, ys, host = _build_stage("stage_52", 256, 512, 768, specs, M, True)
    lpq.lpq_stage_linears(stage, phase)
    for li, (bits, scheme) in enumerate(specs):
        for name in wl.LINEARS:
            w, x = host[li][name]
            check_output(ys[li][name], orc.qlinear(x, w, bits, scheme), "layer %d %s" % (li, name))


@pytest.mark.parametrize("phase", [lpq.LPQ_DECODE, lpq.LPQ_PREFILL], ids=["decode", "prefill"])
def test_config0_full(orc, phase):
    """First configuration at full size: one OPT-125m-shaped layer, 4-bit grouped, decode M = 1 and
    prefill M = 128; packed data bit-exact, every output element compared."""
    cfg = wl.CONFIGS[0]
    M = cfg["decode_Ms"][0] if phase == lpq.LPQ_DECODE else cfg["prefill_M"]
    stage, ys, host = _build_stage(cfg["name"], cfg["h"], cfg["f"], cfg["qkv_n"], cfg["layers"], M, cfg["act_outliers"])
    for name in wl.LINEARS:
        check_packed(stage.keep[0][0][name], orc, host[0][name][0])
    lpq.lpq_stage_linears(stage, phase)
    bits, scheme = cfg["layers"][0]
    for name in wl.LINEARS:
        w, x = host[0][name]
        check_output(ys[0][name], orc.qlinear(x, w, bits, scheme), name)
