"""Latency cost model of one decoder layer on this GPU, and a plan built from it (LLM-PQ, Sec. 4.1 and 4.3).

Times lpq_decoder_layer over a grid of batch sizes and lengths per precision, fits the paper's two regressions
through lpq_latency_fit (prefill on v, s, vs, vs^2; decode on v, v(t+s), t+s), scores them on workloads that were
not in the grid (batch 3, 5 or 7; prompt lengths drawn from 128..512; past lengths 384 or 768, as in the paper's
Sec. 6.2 fidelity test), and feeds the predicted per-layer latencies with variance indicators from
lpq_variance_indicator and the memory model to lpq_plan_adabits and lpq_plan_bitwidth_transfer.

    python -m paper_2403_01136_amd.costmodel [--h 5120 --f 20480 --layers 40 --devices 4 --device-gb 8]

prints one JSON object.  Inputs are synthetic (seeded random weights and activations of the model's shapes).
Everything measured runs in the HIP kernels; everything fitted or planned runs in the library's host code.
"""
import argparse
import json
import sys

import numpy as np

import paper_2403_01136_amd as lpq
from paper_2403_01136_amd import workloads as wl

PRECISIONS = ((3, lpq.LPQ_ASYM_GROUP), (4, lpq.LPQ_ASYM_GROUP), (8, lpq.LPQ_ASYM_GROUP), (16, lpq.LPQ_FP16))
PREFILL_GRID = [(v, s) for v in (1, 2, 4, 8) for s in (128, 256, 384, 512)]
DECODE_GRID = [(v, c) for v in (1, 2, 4, 8, 16) for c in (128, 256, 512, 1024)]


def unseen_workloads(seed, n=50):
    """(prefill (v, s), decode (v, ctx)) pairs outside the grids."""
    r = np.random.default_rng(seed)
    pre = [(int(r.choice([3, 5, 7])), int(r.integers(128, 513))) for _ in range(n)]
    dec = [(int(r.choice([3, 5, 7])), int(r.choice([384, 768]))) for _ in range(n)]
    return pre, dec


class LayerTimer:
    """One decoder layer of the given shape at one precision, with its KV cache, ready to be timed."""

    def __init__(self, h, f, head_dim, bits, scheme, max_batch, max_seq, device, tag="costmodel"):
        import torch
        self.h, self.device, self.tag = h, device, tag
        shapes = {"qkv": (h, 3 * h), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
        self.lw = {}
        for name, (K, N) in shapes.items():
            w = wl.weight_torch(N, K, device, tag, bits, name)
            self.lw[name] = lpq.lpq_quantize_pack(w, bits, scheme)
            del w
        ones, zeros = torch.ones(h, dtype=torch.float16, device=device), torch.zeros(h, dtype=torch.float16, device=device)
        self.state = lpq.LayerState(h // head_dim, head_dim, max_seq, max_batch, device, (ones, zeros), (ones, zeros))
        # the decode timings read the cache up to their position: give it finite contents
        self.state.k_cache.normal_(0, 1)
        self.state.vt_cache.normal_(0, 1)

    def seconds(self, phase, n_seqs, T, pos0, reps=10):
        import torch
        x = wl.act_torch(n_seqs * T, self.h, True, self.device, self.tag, "x", n_seqs, T)
        y, ws = lpq.lpq_decoder_layer(self.lw, self.state, phase, n_seqs, T, pos0, x)
        lpq.lpq_decoder_layer(self.lw, self.state, phase, n_seqs, T, pos0, x, y, ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            lpq.lpq_decoder_layer(self.lw, self.state, phase, n_seqs, T, pos0, x, y, ws)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3


def measure(timer, prefill_points, decode_points, reps=10):
    pre = [timer.seconds(lpq.LPQ_PREFILL, v, s, 0, reps) for v, s in prefill_points]
    dec = [timer.seconds(lpq.LPQ_DECODE, v, 1, c, reps) for v, c in decode_points]
    return np.array(pre), np.array(dec)


def fit_and_score(train_points, train_t, test_points, test_t, phase):
    tv, tl = np.array(train_points, float).T
    coef = lpq.lpq_latency_fit(phase, tv, tl, train_t)
    qv, ql = np.array(test_points, float).T
    err_train = np.abs(lpq.lpq_latency_predict(phase, coef, tv, tl) - train_t) / train_t
    err_test = np.abs(lpq.lpq_latency_predict(phase, coef, qv, ql) - test_t) / test_t
    return coef, err_train, err_test


def layer_indicators(h, f, n_layers, device, tag="costmodel"):
    """omega[i][b] for b in 3, 4, 8, 16: the layer's four operators summed, group-wise scaling factors, deterministic
    rounding; layer i's weights are scaled by a seeded factor so that layers differ as trained ones do."""
    import torch
    shapes = {"qkv": (h, 3 * h), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}
    r = np.random.default_rng(wl.stream_seed(tag, "layer-scale"))
    scale = np.exp(r.normal(0.0, 0.5, n_layers))
    omega = np.zeros((n_layers, 4))
    base = {}
    for name, (K, N) in shapes.items():
        w = wl.weight_torch(N, K, device, tag, "omega", name)
        x = wl.act_torch(256, K, True, device, tag, "omega-x", name)
        base[name] = lpq.lpq_variance_indicator(w, x).cpu().numpy()[:3]      # bits 3, 4, 8 at the quantiser's granularity
        del w, x
    torch.cuda.synchronize()
    per_layer = sum(base.values())
    for i in range(n_layers):
        omega[i, :3] = per_layer * scale[i] ** 2                              # S_W scales with the weights' magnitude
    return omega


def run(args):
    import torch
    device = torch.device("cuda:0")
    max_seq = 1088                                                             # 1024 cached positions + the new one, 64-aligned
    pre_test, dec_test = unseen_workloads(args.seed)
    report = {"shape": {"h": args.h, "f": args.f, "head_dim": args.head_dim}, "data": "synthetic", "precisions": {}}
    models = {}
    for bits, scheme in PRECISIONS:
        timer = LayerTimer(args.h, args.f, args.head_dim, bits, scheme, 16, max_seq, device)
        t_pre, t_dec = measure(timer, PREFILL_GRID, DECODE_GRID, args.reps)
        q_pre, q_dec = measure(timer, pre_test, dec_test, args.reps)
        c_pre, e_pre_tr, e_pre = fit_and_score(PREFILL_GRID, t_pre, pre_test, q_pre, lpq.LPQ_PREFILL)
        c_dec, e_dec_tr, e_dec = fit_and_score(DECODE_GRID, t_dec, dec_test, q_dec, lpq.LPQ_DECODE)
        models[bits] = (c_pre, c_dec)
        report["precisions"][str(bits)] = {
            "prefill_coef": c_pre.tolist(), "decode_coef": c_dec.tolist(),
            "prefill_grid_ms": [[v, sl, round(float(t) * 1e3, 4)] for (v, sl), t in zip(PREFILL_GRID, t_pre)],
            "decode_grid_ms": [[v, c, round(float(t) * 1e3, 4)] for (v, c), t in zip(DECODE_GRID, t_dec)],
            "prefill_ms_range": [float(t_pre.min() * 1e3), float(t_pre.max() * 1e3)],
            "decode_ms_range": [float(t_dec.min() * 1e3), float(t_dec.max() * 1e3)],
            "prefill_err_grid_mean": float(e_pre_tr.mean()), "prefill_err_unseen_mean": float(e_pre.mean()),
            "prefill_err_unseen_max": float(e_pre.max()),
            "decode_err_grid_mean": float(e_dec_tr.mean()), "decode_err_unseen_mean": float(e_dec.mean()),
            "decode_err_unseen_max": float(e_dec.max())}
        del timer
        torch.cuda.empty_cache()
        print("precision %d done" % bits, file=sys.stderr, flush=True)
    errs = [report["precisions"][str(b)][k] for b, _ in PRECISIONS for k in ("prefill_err_unseen_mean", "decode_err_unseen_mean")]
    report["mean_unseen_error"] = float(np.mean(errs))

    # the plan: L layers on N equal devices of a stated budget, latencies from the fitted models
    bits = [b for b, _ in PRECISIONS]
    eta, xi, B, s, n = args.eta, args.xi, args.batch, args.prompt, args.generate
    slow = np.array([float(e) for e in args.slowdown.split(",")] if args.slowdown else [1.0] * args.devices)
    if slow.shape != (args.devices,):
        raise SystemExit("--slowdown needs one factor per device")
    lat_pre = np.outer(slow, [lpq.lpq_latency_predict(lpq.LPQ_PREFILL, models[b][0], [eta], [s])[0] for b in bits])
    lat_dec = np.outer(slow, [lpq.lpq_latency_predict(lpq.LPQ_DECODE, models[b][1], [xi], [s + n / 2])[0] for b in bits])
    mem = np.array([lpq.lpq_mem_layer_bytes(args.h, args.f, b) + lpq.lpq_mem_kv_bytes(B, s, n, args.h) for b in bits])
    omega = layer_indicators(args.h, args.f, args.layers, device)
    problem = lpq.PlanProblem(bits=bits, omega=omega, lat_pre=lat_pre, lat_dec=lat_dec, mem=mem, cap=[args.device_gb * 1e9] * args.devices,
                              emb=lpq.lpq_mem_embedding_bytes(args.vocab, args.h, args.pos, args.h), B=B, eta=eta, xi=xi, n=n,
                              theta=args.theta)
    q0, counts, choice = lpq.lpq_plan_adabits(problem)
    plan = {"devices": args.devices, "device_gb": args.device_gb, "slowdown": slow.tolist(), "layers": args.layers, "B": B, "eta": eta, "xi": xi, "s": s, "n": n,
            "theta": args.theta, "lat_pre_ms": (lat_pre[0] * 1e3).tolist(), "lat_dec_ms": (lat_dec[0] * 1e3).tolist()}
    if counts is None:
        plan["adabits"] = None
    else:
        start = lpq.lpq_plan_objective(problem, counts, choice)
        obj, c2, ch2, rounds = lpq.lpq_plan_bitwidth_transfer(problem, counts, choice)
        plan.update({"adabits": {"counts": counts, "bits": [bits[k] for k in choice], "objective": start},
                     "bitwidth_transfer": {"counts": c2, "bits": [bits[k] for k in ch2], "objective": obj, "rounds": rounds}})
    report["plan"] = plan
    return report


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--h", type=int, default=5120)
    ap.add_argument("--f", type=int, default=20480)
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--layers", type=int, default=40)
    ap.add_argument("--vocab", type=int, default=50272)
    ap.add_argument("--pos", type=int, default=2050)
    ap.add_argument("--devices", type=int, default=4)
    ap.add_argument("--device-gb", type=float, default=8.0)
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--eta", type=int, default=4)
    ap.add_argument("--xi", type=int, default=16)
    ap.add_argument("--prompt", type=int, default=512)
    ap.add_argument("--generate", type=int, default=100)
    ap.add_argument("--theta", type=float, default=1e-4)
    ap.add_argument("--slowdown", type=str, default="",
                    help="comma-separated factor per device on the measured latencies (stands in for slower devices); default all 1")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--seed", type=int, default=0)
    print(json.dumps(run(ap.parse_args())))


if __name__ == "__main__":
    main()
