#!/usr/bin/env python3
"""Benchmark of the quantized-linear hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--only decode|prefill|all] [--no-per-config]

Headline workload: the largest configuration that one GPU holds, configs[4] -- the BLOOM-176B-shaped pipeline share
(10 consecutive layers, all 3-bit, g = 128, 10 GB packed) with seeded synthetic weights and activations.  One "step"
is one decode-phase pass of lpq_stage_linears over the whole stage at the decode micro-batch (M = 16); the
prefill-phase pass (M = 4 x 512) and the quantise+pack pass are timed in the same run and reported in the same JSON
line.  `per_config` then holds every configuration (1-4) at every decode micro-batch of its sweep and at its prefill
micro-batch, each with its time and its fraction of the HBM or matrix-core peak, plus -- as context only -- what the
vendor's fp16 GEMM reaches on the same shapes and data.  Inputs are resident in HBM before any timed region starts.

Prints ONE JSON line: the contract fields, plus `roofline` (dominant kernel: decode, HBM-bound), `prefill`
(TFLOP/s and its MFMA roofline), `per_config`, `quantize`, `layer`, `loader` and `cpu_baseline` (the CPU oracle
timed on a bounded sample of the same workload on this machine's host cores).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_F16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16 matrix peak, published


def build_stage(cfg, M, device, quant_times=None):
    """Draw, quantise and pack every linear of the stage on the GPU; returns (Stage, ys)."""
    import torch
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import workloads as wl
    shapes = wl.linear_shapes(cfg)
    layers, xs, ys = [], [], []
    for li, (bits, scheme) in enumerate(cfg["layers"]):
        lw, lx, ly = {}, {}, {}
        x_h = wl.act_torch(M, cfg["h"], cfg["act_outliers"], device, cfg["name"], li, "h", M)
        x_f = wl.act_torch(M, cfg["f"], cfg["act_outliers"], device, cfg["name"], li, "f", M)
        for name in wl.LINEARS:
            K, N = shapes[name]
            w = wl.weight_torch(N, K, device, cfg["name"], li, name)
            if quant_times is not None:       # timed on the second pass into the same buffers (no allocation in the timed region)
                lw[name] = lpq.lpq_quantize_pack(w, bits, scheme)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                lpq.lpq_quantize_pack_rows(w, lw[name], 0)
                e1.record()
                torch.cuda.synchronize()
                quant_times.append((K * N, e0.elapsed_time(e1)))
            else:
                lw[name] = lpq.lpq_quantize_pack(w, bits, scheme)
            del w
            lx[name] = x_f if name == "fc2" else x_h
            ly[name] = torch.empty((M, N), dtype=torch.float16, device=device)
        layers.append(lw), xs.append(lx), ys.append(ly)
    return lpq.Stage(layers, xs, ys), ys


def reuse_stage(stage, M, cfg, device):
    """A second Stage over the same packed weights with fresh activations of M rows."""
    import torch
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import workloads as wl
    layers = stage.keep[0]
    xs, ys = [], []
    for li in range(len(layers)):
        x_h = wl.act_torch(M, cfg["h"], cfg["act_outliers"], device, cfg["name"], li, "h", M)
        x_f = wl.act_torch(M, cfg["f"], cfg["act_outliers"], device, cfg["name"], li, "f", M)
        xs.append({n: (x_f if n == "fc2" else x_h) for n in wl.LINEARS})
        ys.append({n: torch.empty((M, layers[li][n].N), dtype=torch.float16, device=device) for n in wl.LINEARS})
    return lpq.Stage(layers, xs, ys), ys


def time_phase(stage, phase, steps, warmup):
    """W untimed + exactly K timed passes, bracketed by synchronize; HIP events on the launch stream."""
    import torch
    import paper_2403_01136_amd as lpq
    for _ in range(warmup):
        lpq.lpq_stage_linears(stage, phase)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        lpq.lpq_stage_linears(stage, phase)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def act_bytes(cfg, M):
    from paper_2403_01136_amd import workloads as wl
    return sum(2 * M * K + 2 * M * N for _ in cfg["layers"] for (K, N) in wl.linear_shapes(cfg).values())


def cpu_baseline(cfg, M, budget_weights=1.5e9):
    """The CPU oracle (as it stands) on a bounded sample of the same workload: for every layer of the
    stage, `budget_rows` output rows of its FC1 linear (about budget_weights weights in all: 10-30 s of
    host work), quantise -> dequantise -> fp64 matmul at the decode micro-batch.  Reported in the metric's
    unit: packed-weight bytes of the sample per second."""
    import numpy as np
    import oracle
    from paper_2403_01136_amd import workloads as wl
    K, N = wl.linear_shapes(cfg)["fc1"]
    budget_rows = int(min(N, max(64, budget_weights / (K * len(cfg["layers"])) // 64 * 64)))
    cores = len(os.sched_getaffinity(0))
    x = wl.act_np(M, K, cfg["act_outliers"], cfg["name"], "cpu_baseline")
    ws = [wl.weight_np(budget_rows, K, cfg["name"], li, "fc1", "cpu_baseline") for li in range(len(cfg["layers"]))]
    oracle.default()
    t0 = time.perf_counter()
    nbytes = 0
    for w, (bits, scheme) in zip(ws, cfg["layers"]):
        oracle.qlinear(x, w, bits, scheme)
        nbytes += wl.packed_bytes(bits, scheme, K, budget_rows)
    dt = time.perf_counter() - t0
    return {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle", "seconds": round(dt, 2),
            "sample": "%d rows of FC1 (K=%d) of each of the %d layers, quantize+dequant+fp64 matmul at M=%d"
                      % (budget_rows, K, len(cfg["layers"]), M)}


def loader_bench(cfg, device, layer=2, staging_mib=64, reps=3):
    """On-the-fly quantised loading (Sec. 5 of the paper) of one layer's four fp16 weights from pinned host
    memory: lpq_load_quantize_pack against a plain host-to-device copy of the same bytes (the PCIe bound)."""
    import torch
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import workloads as wl
    bits, scheme = cfg["layers"][layer]
    shapes = wl.linear_shapes(cfg)
    hosts = []
    for name in wl.LINEARS:
        K, N = shapes[name]
        w = wl.weight_torch(N, K, device, cfg["name"], layer, name)
        h = torch.empty((N, K), dtype=torch.float16, pin_memory=True)
        h.copy_(w)
        hosts.append(h)
        del w
    torch.cuda.synchronize()
    nbytes = sum(h.numel() * 2 for h in hosts)
    staging = torch.empty(staging_mib << 20, dtype=torch.uint8, device=device)
    dst = torch.empty(max(h.numel() for h in hosts), dtype=torch.float16, device=device)

    def timed(fn):
        best = None
        for _ in range(reps + 1):                      # the first pass warms up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            best = dt if best is None or _ == 1 else min(best, dt)
        return best

    keep = []
    t_load = timed(lambda: keep.__setitem__(slice(None), [lpq.lpq_load_quantize_pack(h, bits, scheme, staging) for h in hosts]))
    t_copy = timed(lambda: [dst[:h.numel()].view(h.shape).copy_(h, non_blocking=True) for h in hosts])
    return {"metric": "on-the-fly quantised load, fp16 source GB/s from pinned host memory", "value": nbytes / t_load / 1e9,
            "unit": "GB/s", "ms": t_load * 1e3, "bytes": nbytes, "bits": bits,
            "workload": "the four linears of layer %d of %s, staging %d MiB" % (layer, cfg["name"], staging_mib),
            "h2d_copy_GBs": nbytes / t_copy / 1e9, "frac_of_h2d_copy": t_copy / t_load}


def layer_bench(cfg, device, layer=2, n_heads=None, head_dim=128, n_gen=100, steps=20):
    """One whole decoder layer (layer norms, quantised linears with fused epilogues, KV cache, attention):
    the per-layer latency l_{i,j,b} that the paper's cost model consumes (Sec. 4.3), at the prefill
    micro-batch (eta prompts of s tokens) and at the decode micro-batch (xi sequences) with s + n/2 cached
    positions, as the paper averages the decode cost."""
    import torch
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import workloads as wl
    bits, scheme = cfg["layers"][layer]
    h, f = cfg["h"], cfg["f"]
    H = n_heads or h // head_dim
    shapes = wl.linear_shapes(cfg)
    Mp, xi = cfg["prefill_M"], cfg["decode_Ms"][-1 if cfg["name"] != "bloom176b_share10_w3" else 2]
    s_len = 512 if Mp % 512 == 0 else Mp
    eta = Mp // s_len
    S = ((s_len + n_gen + 63) // 64) * 64
    batch = max(eta, xi)
    lw = {}
    for name in wl.LINEARS:
        K, N = shapes[name]
        w = wl.weight_torch(N, K, device, cfg["name"], layer, name)
        lw[name] = lpq.lpq_quantize_pack(w, bits, scheme)
        del w
    ones, zeros = torch.ones(h, dtype=torch.float16, device=device), torch.zeros(h, dtype=torch.float16, device=device)
    st = lpq.LayerState(H, head_dim, S, batch, device, (ones, zeros), (ones, zeros))
    wbytes = sum(q.nbytes for q in lw.values())

    def timed(phase, n_seqs, T, pos0):
        x = wl.act_torch(n_seqs * T, h, cfg["act_outliers"], device, cfg["name"], layer, "layer", T)
        y, ws = lpq.lpq_decoder_layer(lw, st, phase, n_seqs, T, pos0, x)
        for _ in range(2):
            lpq.lpq_decoder_layer(lw, st, phase, n_seqs, T, pos0, x, y, ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            lpq.lpq_decoder_layer(lw, st, phase, n_seqs, T, pos0, x, y, ws)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / steps

    ms_pre = timed(lpq.LPQ_PREFILL, eta, s_len, 0)
    pos_dec = s_len + n_gen // 2
    ms_dec = timed(lpq.LPQ_DECODE, xi, 1, pos_dec)
    lin_flops = 2.0 * Mp * sum(K * N for K, N in shapes.values())
    att_flops = 4.0 * eta * H * head_dim * s_len * (s_len + 1) / 2          # q.k and p.v over the causal half
    kv_bytes = 2.0 * xi * (pos_dec + 1) * h * 2
    act_bytes = 2.0 * xi * (h * 9 + 3 * h + 2 * f)                          # rows read and written by the operators, fp16
    return {"workload": "one %d-bit layer of %s: h=%d, %d heads of %d, f=%d; prefill %d x %d tokens; decode %d sequences at "
                        "position %d (s + n/2)" % (bits, cfg["name"], h, H, head_dim, f, eta, s_len, xi, pos_dec),
            "prefill_ms": ms_pre, "prefill_TFLOPs": (lin_flops + att_flops) / ms_pre / 1e9,
            "decode_ms": ms_dec, "decode_GBs": (wbytes + kv_bytes + act_bytes) / ms_dec / 1e6,
            "decode_bytes": {"weights": wbytes, "kv_cache": kv_bytes, "activations": act_bytes},
            "decode_frac_of_hbm_peak": (wbytes + kv_bytes + act_bytes) / ms_dec / 1e6 / HBM_PEAK_GBS}


def traffic_from_profiles(cfg, phase, M):
    """HBM bytes per launch as measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, scaled by the
    copy calibration) and recorded in profiles/hbm_traffic.json for this workload; None if absent."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        rec = json.load(open(path))
    except (OSError, ValueError):
        return None
    return rec.get("%s/%s M=%d" % (cfg["name"], phase, M))


def headline_decode_m(ci, cfg):
    """The decode micro-batch the headline is quoted at: 16 for the BLOOM-176B share (the middle of its sweep), else
    the configuration's last (largest) one."""
    return 16 if ci == 4 else cfg["decode_Ms"][-1]


def decode_point(stage_w, cfg, M, device, steps, warmup):
    """One decode sweep point: a Stage over the resident packed weights with activations of M rows."""
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import workloads as wl
    stage, _ = reuse_stage(stage_w, M, cfg, device)
    ms, wall = time_phase(stage, lpq.LPQ_DECODE, steps, warmup)
    wbytes = wl.stage_packed_bytes(cfg)
    algo = wbytes + act_bytes(cfg, M)
    return {"M": M, "ms": ms, "host_ms": wall, "packed_weight_GBs": wbytes / ms / 1e6, "algorithmic_GBs": algo / ms / 1e6,
            "frac_of_hbm_peak": algo / ms / 1e6 / HBM_PEAK_GBS, "algorithmic_bytes": algo}


def prefill_point(stage_w, cfg, device, steps, warmup):
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import workloads as wl
    Mp = cfg["prefill_M"]
    stage, _ = reuse_stage(stage_w, Mp, cfg, device)
    ms, wall = time_phase(stage, lpq.LPQ_PREFILL, steps, warmup)
    flops = wl.stage_flops(cfg, Mp)
    return {"M": Mp, "ms": ms, "host_ms": wall, "TFLOPs": flops / ms / 1e9, "frac_of_mfma_peak": flops / ms / 1e9 / MFMA_F16_PEAK_TFLOPS,
            "flops": flops, "steps": steps, "warmup": warmup}


def vendor_gemm_point(cfg, device, steps=5):
    """Context only, not this library: the vendor's fp16 GEMM (torch.matmul) on the four linear shapes of the
    configuration at its prefill micro-batch, same seeded operands, all layers' FLOPs -- what a plain library
    GEMM on unquantised weights reaches on this machine on the same data."""
    import torch
    from paper_2403_01136_amd import workloads as wl
    Mp = cfg["prefill_M"]
    total_ms, flops = 0.0, 0.0
    for name, (K, N) in wl.linear_shapes(cfg).items():
        w = wl.weight_torch(N, K, device, cfg["name"], 0, name)
        x = wl.act_torch(Mp, K, cfg["act_outliers"], device, cfg["name"], 0, "f" if name == "fc2" else "h", Mp)
        y = torch.empty((Mp, N), dtype=torch.float16, device=device)
        for _ in range(2):
            torch.matmul(x, w.t(), out=y)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            torch.matmul(x, w.t(), out=y)
        e1.record()
        torch.cuda.synchronize()
        total_ms += e0.elapsed_time(e1) / steps
        flops += 2.0 * Mp * K * N
        del w, x, y
    return {"kind": "torch.matmul fp16 (vendor GEMM library), one layer's four shapes", "TFLOPs": flops / total_ms / 1e9,
            "frac_of_mfma_peak": flops / total_ms / 1e9 / MFMA_F16_PEAK_TFLOPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4, help="headline configuration (default: the largest, configs[4])")
    ap.add_argument("--decode-m", type=int, default=None)
    ap.add_argument("--only", choices=["all", "decode", "prefill", "layer"], default="all")
    ap.add_argument("--no-per-config", action="store_true", help="time the headline configuration only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-loader", action="store_true", help="skip the host-to-device quantised-load measurement")
    ap.add_argument("--no-layer", action="store_true", help="skip the whole-decoder-layer measurement")
    ap.add_argument("--no-vendor-gemm", action="store_true", help="skip the vendor GEMM context figure")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy 3 times, so a --pmc run can scale FETCH_SIZE / WRITE_SIZE by it")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: the library runs on ONE GPU only (a pipeline stage is an independent unit: with more GPUs each "
              "runs its own stage and only activations cross); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no fallback", file=sys.stderr)
        sys.exit(3)
    lpq.load_library()
    device = torch.device("cuda:0")
    ci = args.config
    cfg = wl.CONFIGS[ci]
    Md = args.decode_m or headline_decode_m(ci, cfg)
    Mp = cfg["prefill_M"]
    side_cfg = wl.CONFIGS[1]           # the decoder-layer and loader legs stay on the OPT-13B shapes

    if args.only == "layer":          # the whole-decoder-layer measurement alone (for profiling it)
        print(json.dumps({"metric": "decoder layer latency", "unit": "ms", "n_gpus": 1, "data": "synthetic",
                          "layer": layer_bench(side_cfg, device, layer=2, steps=args.steps)}))
        return
    qt = []
    stage_d, _ = build_stage(cfg, Md, device, quant_times=qt)
    wbytes = wl.stage_packed_bytes(cfg)
    out = {"metric": "decode packed-weight GB/s", "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16", "data": "synthetic",
           "config": {"workload": "configs[%d] %s: %d layers, bits %s, g=128, decode M=%d, prefill M=%d"
                                  % (ci, cfg["name"], len(cfg["layers"]), [b for b, _ in cfg["layers"]], Md, Mp),
                      "packed_weight_bytes": wbytes}}
    n_w = sum(n for n, _ in qt)
    q_ms = sum(t for _, t in qt)
    out["quantize"] = {"value": n_w / q_ms / 1e6, "unit": "Gweights/s", "ms_total": round(q_ms, 3),
                       "fp16_read_GBs": round(2 * n_w / q_ms / 1e6, 1)}

    if args.only in ("all", "decode"):
        ms, wall = time_phase(stage_d, lpq.LPQ_DECODE, args.steps, args.warmup)
        algo = wbytes + act_bytes(cfg, Md)
        out.update({"value": wbytes / ms / 1e6, "ms_per_step": ms, "host_ms_per_step": wall})
        out["roofline"] = {"bound": "hbm", "achieved": algo / ms / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": algo / ms / 1e6 / HBM_PEAK_GBS, "traffic": None,
                           "kernel": "decode_prepare_kernel + decode_kernel + decode_fixup_kernel (one grouped decode launch of the stage)",
                           "algorithmic_bytes_per_launch": algo}
    psteps, pwarm = max(3, args.steps // 10), max(1, args.warmup // 5)
    if args.only in ("all", "prefill"):
        pp = prefill_point(stage_d, cfg, device, psteps, pwarm)
        out["prefill"] = {"metric": "prefill TFLOP/s", "value": pp["TFLOPs"], "unit": "TFLOP/s", "ms_per_step": pp["ms"],
                          "steps": psteps, "warmup": pwarm,
                          "roofline": {"bound": "mfma", "achieved": pp["TFLOPs"], "peak": MFMA_F16_PEAK_TFLOPS,
                                       "unit": "TFLOP/s", "frac": pp["frac_of_mfma_peak"], "traffic": None,
                                       "kernel": "prefill_kernel / prefill_ring_kernel (one grouped launch per storage variant)",
                                       "algorithmic_flops_per_step": pp["flops"]}}
        if args.only == "prefill":
            out.update({"metric": "prefill TFLOP/s", "unit": "TFLOP/s", "value": pp["TFLOPs"],
                        "ms_per_step": pp["ms"], "steps": psteps, "warmup": pwarm, "roofline": out["prefill"]["roofline"]})
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=device).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 3}
        del src, dst
    for phase, M, roof in (("decode", Md, out.get("roofline") if args.only != "prefill" else None),
                           ("prefill", Mp, out.get("prefill", {}).get("roofline"))):
        measured = traffic_from_profiles(cfg, phase, M)
        if measured and roof is not None:
            roof["traffic"] = measured["bytes_per_launch"]
            roof["traffic_source"] = measured["source"]

    # every configuration of the benchmark x every decode sweep point x its prefill micro-batch
    if args.only == "all" and not args.no_per_config:
        per = {}
        for cj in (ci,) + tuple(c for c in range(1, len(wl.CONFIGS)) if c != ci):
            cfg_j = wl.CONFIGS[cj]
            if cj != ci:
                del stage_d
                torch.cuda.empty_cache()
                stage_d, _ = build_stage(cfg_j, 1, device)
            rec = {"workload": "%s: %d layers, bits %s" % (cfg_j["name"], len(cfg_j["layers"]), sorted({b for b, _ in cfg_j["layers"]})),
                   "packed_weight_bytes": wl.stage_packed_bytes(cfg_j),
                   "decode": [decode_point(stage_d, cfg_j, M, device, 20, 5) for M in cfg_j["decode_Ms"]],
                   "prefill": prefill_point(stage_d, cfg_j, device, 3, 1)}
            if not args.no_vendor_gemm:
                rec["vendor_gemm_context"] = vendor_gemm_point(cfg_j, device)
            per["configs[%d]" % cj] = rec
        out["per_config"] = per
    del stage_d
    torch.cuda.empty_cache()
    if not args.no_layer and args.only == "all":
        out["layer"] = layer_bench(side_cfg, device, layer=2)
    if not args.no_loader and args.only == "all":
        out["loader"] = loader_bench(side_cfg, device, layer=2)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, Md)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
