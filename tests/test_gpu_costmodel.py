"""The latency cost model measured on the GPU (Sec. 4.1) and the plan built from it (Sec. 4.3, Algorithm 2).

The timings come from lpq_decoder_layer; the fit runs in the library's host code and is compared with the
oracle's least squares on the same measured samples; the plan is checked for validity with the oracle's objective."""
import argparse

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def small_args(**kw):
    a = dict(h=1024, f=4096, head_dim=64, layers=12, vocab=8192, pos=2050, devices=3, device_gb=0.1, batch=8, eta=2, xi=4,
             prompt=256, generate=64, theta=1e-4, reps=3, seed=1, slowdown="1,1,3")
    a.update(kw)
    return argparse.Namespace(**a)


def test_fit_on_measured_samples_matches_oracle_and_plan_is_valid():
    import torch
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import costmodel as cm
    from oracle import planner as P
    device = torch.device("cuda:0")
    timer = cm.LayerTimer(1024, 4096, 64, 4, lpq.LPQ_ASYM_GROUP, 16, 1088, device)
    pre_pts, dec_pts = cm.PREFILL_GRID, cm.DECODE_GRID
    t_pre, t_dec = cm.measure(timer, pre_pts, dec_pts, reps=3)
    assert np.all(t_pre > 0) and np.all(t_dec > 0) and np.all(np.isfinite(t_pre)) and np.all(np.isfinite(t_dec))
    for phase, name, pts, t in ((lpq.LPQ_PREFILL, "prefill", pre_pts, t_pre), (lpq.LPQ_DECODE, "decode", dec_pts, t_dec)):
        v, length = np.array(pts, float).T
        got, want = lpq.lpq_latency_fit(phase, v, length, t), P.fit_latency(name, v, length, t)
        X = P.prefill_features(v, length) if name == "prefill" else P.decode_features(v, length)
        assert np.all(np.abs(got - want) * np.abs(X).max(axis=0) <= 1e-8 * t.max())
        assert np.allclose(lpq.lpq_latency_predict(phase, got, v, length), P.predict_latency(name, want, v, length), rtol=1e-8)
    # prefill time grows with the work: the largest grid point costs more than the smallest
    assert t_pre[-1] > t_pre[0]


def test_costmodel_report_and_plan():
    import paper_2403_01136_amd as lpq
    from paper_2403_01136_amd import costmodel as cm
    from oracle import planner as P
    args = small_args()
    rep = cm.run(args)
    assert set(rep["precisions"]) == {"3", "4", "8", "16"}
    for p in rep["precisions"].values():
        assert len(p["prefill_coef"]) == 5 and len(p["decode_coef"]) == 4
        assert 0 <= p["prefill_err_unseen_mean"] < 1.0 and 0 <= p["decode_err_unseen_mean"] < 1.0
    plan = rep["plan"]
    assert plan["adabits"] is not None
    bits = [3, 4, 8, 16]
    for key in ("adabits", "bitwidth_transfer"):
        counts, b = plan[key]["counts"], plan[key]["bits"]
        assert sum(counts) == args.layers and min(counts) >= 1 and len(b) == args.layers and set(b) <= set(bits)
        # memory: every device's layers fit the stated budget by the oracle's memory model
        start = 0
        for j, c in enumerate(counts):
            need = sum(P.layer_weight_bytes(args.h, args.f, bb) + P.kv_bytes(args.batch, args.prompt, args.generate, args.h)
                       for bb in b[start:start + c])
            need += P.embedding_bytes(args.vocab, args.h, args.pos, args.h) if j == 0 else 0
            assert need <= args.device_gb * 1e9
            start += c
    assert plan["bitwidth_transfer"]["objective"] <= plan["adabits"]["objective"]
