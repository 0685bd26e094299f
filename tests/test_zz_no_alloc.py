"""The entry point that allocates nothing (lpq_stage_linears_noalloc) against lpq_stage_linears and the oracle.

Two calls in a row through the C ABI, the second with a smaller input: the static scratch array keeps the first
call's partial tiles, which the second must not pick up.  Collected last (file name), so that a failure here hides
no other test; passes alone in a fresh process and after the other tests (the library's own workspace may or may
not exist by then: this entry point never touches it)."""
import numpy as np
import pytest

import paper_2403_01136_amd as lpq
from paper_2403_01136_amd import workloads as wl
from gpu_util import check_output, to_dev

pytestmark = pytest.mark.gpu


def _stage(key, h, f, qkv_n, specs, M):
    import torch
    shapes = {"qkv": (h, qkv_n), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
    layers, xs, host = [], [], []
    for li, (bits, scheme) in enumerate(specs):
        lw, lx, lh = {}, {}, {}
        x_h, x_f = wl.act_np(M, h, True, key, li, "h", M), wl.act_np(M, f, True, key, li, "f", M)
        xd_h, xd_f = to_dev(x_h), to_dev(x_f)
        for name, (K, N) in shapes.items():
            w = wl.weight_np(N, K, key, li, name)
            lw[name] = lpq.lpq_quantize_pack(to_dev(w), bits, scheme)
            lx[name] = xd_f if name == "fc2" else xd_h
            lh[name] = (w, x_f if name == "fc2" else x_h)
        layers.append(lw), xs.append(lx), host.append(lh)

    def outputs():
        return [{n: torch.full((M, layers[li][n].N), float("nan"), dtype=torch.float16, device="cuda") for n in shapes}
                for li in range(len(specs))]
    return layers, xs, host, outputs


# (hidden, ffn, specs, M): first a stage whose even-share launch cuts units into partial tiles (the streaming kernel,
# forced by the routing call), then a smaller one; decode at 16 and 27 rows and at few rows
CASES = [
    ((512, 2048, [(3, 1), (4, 1), (8, 1), (8, 2), (16, 0), (4, 1)], 27), (256, 1024, [(4, 1), (3, 1)], 5)),
    ((512, 2048, [(4, 1), (3, 1), (8, 2)], 16), (256, 512, [(3, 1)], 1)),
]


@pytest.mark.parametrize("even_share", [True, False], ids=["even_share", "rows"])
@pytest.mark.parametrize("case", range(len(CASES)))
def test_noalloc_matches_stage_linears_twice_in_a_row(orc, case, even_share):
    import torch
    lpq.load_library()
    if even_share:
        lpq.lpq_set_decode_routing(0, 0)
    try:
        for h, f, specs, M in CASES[case]:                      # the second call is the smaller one
            layers, xs, host, outputs = _stage("noalloc%d" % case, h, f, 3 * h, specs, M)
            y_ref, y_new = outputs(), outputs()
            lpq.lpq_stage_linears(lpq.Stage(layers, xs, y_ref), lpq.LPQ_DECODE)
            lpq.lpq_stage_linears_noalloc(lpq.Stage(layers, xs, y_new), lpq.LPQ_DECODE)
            torch.cuda.synchronize()
            for li, (bits, scheme) in enumerate(specs):
                for name in wl.LINEARS:
                    what = "case %d h=%d M=%d layer %d %s" % (case, h, M, li, name)
                    a, b = y_ref[li][name], y_new[li][name]
                    assert not torch.isnan(b).any(), what + ": output not fully written"
                    # same kernels, same order of additions: the two entry points agree bit for bit
                    assert torch.equal(a.view(torch.int16), b.view(torch.int16)), what
                    w, x = host[li][name]
                    check_output(b, orc.qlinear(x, w, bits, scheme), what)
    finally:
        lpq.lpq_set_decode_routing(-1, -1)


def test_noalloc_prefill_and_many_rows(orc):
    """A stage-wide prefill launch needs no partial sums and runs (one that the library splits over K may be refused);
    a decode call of 300 rows runs in passes of 64 rows, whose partial tiles the static array holds."""
    import torch
    h, f, specs, M = 256, 1024, [(4, 1), (16, 0)], 300
    layers, xs, host, outputs = _stage("noalloc_pre", h, f, 3 * h, specs, M)
    ys = outputs()
    try:
        lpq.lpq_stage_linears_noalloc(lpq.Stage(layers, xs, ys), lpq.LPQ_PREFILL)
        torch.cuda.synchronize()
        for li, (bits, scheme) in enumerate(specs):
            for name in wl.LINEARS:
                w, x = host[li][name]
                check_output(ys[li][name], orc.qlinear(x, w, bits, scheme), "prefill layer %d %s" % (li, name))
    except lpq.LpqError as e:            # a K-split launch: legitimately refused, never allocated
        assert e.status == 6
    lpq.lpq_set_decode_routing(0, 0)
    try:
        ys = outputs()
        lpq.lpq_stage_linears_noalloc(lpq.Stage(layers, xs, ys), lpq.LPQ_DECODE)
        torch.cuda.synchronize()
        for li, (bits, scheme) in enumerate(specs):
            for name in wl.LINEARS:
                w, x = host[li][name]
                check_output(ys[li][name], orc.qlinear(x, w, bits, scheme), "decode 300 rows, layer %d %s" % (li, name))
    finally:
        lpq.lpq_set_decode_routing(-1, -1)


def test_noalloc_size_limit():
    """A decode launch whose prepared activations (up to 16 rows, 2 bytes per token row and column of every 3-bit linear;
    here four feed-forward matrices of K = 2^20 at 16 rows: 128 MiB) do not fit the static array beside its partial tiles
    is refused with LPQ_ERR_BUFSIZE; nothing is allocated instead and nothing is launched."""
    import torch
    lpq.load_library()
    h, f, M = 128, 1 << 20, 16
    shapes = {"qkv": (h, 3 * h), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
    gen = torch.Generator(device="cuda").manual_seed(7)
    layers, xs, ys = [], [], []
    x_h = torch.randn((M, h), generator=gen, device="cuda", dtype=torch.float16)
    x_f = torch.randn((M, f), generator=gen, device="cuda", dtype=torch.float16)
    for li in range(4):
        lw = {}
        for name, (K, N) in shapes.items():
            w = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float16)
            lw[name] = lpq.lpq_quantize_pack(w, 3, 1)
            del w
        layers.append(lw)
        xs.append({n: (x_f if n == "fc2" else x_h) for n in shapes})
        ys.append({n: torch.full((M, shapes[n][1]), float("nan"), dtype=torch.float16, device="cuda") for n in shapes})
    lpq.lpq_set_decode_routing(0, 0)
    try:
        with pytest.raises(lpq.LpqError) as err:
            lpq.lpq_stage_linears_noalloc(lpq.Stage(layers, xs, ys), lpq.LPQ_DECODE)
        assert err.value.status == 6
        torch.cuda.synchronize()
        assert all(torch.isnan(y).all() for l in ys for y in l.values()), "a refused call wrote outputs"
        lpq.lpq_stage_linears(lpq.Stage(layers, xs, ys), lpq.LPQ_DECODE)          # the allocating entry point takes it
        torch.cuda.synchronize()
        assert all(torch.isfinite(y).all() for l in ys for y in l.values())
    finally:
        lpq.lpq_set_decode_routing(-1, -1)


def test_noalloc_under_graph_capture():
    """What the entry point is for: a decode step captured into a HIP graph (no allocation may happen while a stream
    captures) and replayed with new activations in the same buffers.  Every replay equals the eager call on the same
    inputs bit for bit; eager work and synchronisations sit between the replays."""
    import torch
    lpq.load_library()
    h, f, specs, M = 256, 1024, [(3, 1), (4, 1), (8, 2), (16, 0)], 16
    layers, xs, host, outputs = _stage("noalloc_graph", h, f, 3 * h, specs, M)
    lpq.lpq_set_decode_routing(0, 0)
    try:
        y_graph, y_eager = outputs(), outputs()
        stage_g, stage_e = lpq.Stage(layers, xs, y_graph), lpq.Stage(layers, xs, y_eager)
        lpq.lpq_stage_linears_noalloc(stage_g, lpq.LPQ_DECODE)           # once outside the capture: per-device set-up happens here
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            lpq.lpq_stage_linears_noalloc(stage_g, lpq.LPQ_DECODE)
        gen = torch.Generator(device="cuda").manual_seed(11)
        for rep in range(3):
            for lx in xs:                                                 # new activations, same buffers
                for t in {id(v): v for v in lx.values()}.values():
                    t.copy_(torch.randn(t.shape, generator=gen, device="cuda", dtype=torch.float32).to(torch.float16))
            for ly in y_graph:
                for t in ly.values():
                    t.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            lpq.lpq_stage_linears_noalloc(stage_e, lpq.LPQ_DECODE)
            torch.cuda.synchronize()
            for li in range(len(specs)):
                for name in wl.LINEARS:
                    a, b = y_graph[li][name], y_eager[li][name]
                    assert not torch.isnan(a).any(), "replay %d layer %d %s: output not fully written" % (rep, li, name)
                    assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "replay %d layer %d %s" % (rep, li, name)
    finally:
        lpq.lpq_set_decode_routing(-1, -1)
