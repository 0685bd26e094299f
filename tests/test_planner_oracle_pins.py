"""Pins of oracle/planner.py against what the paper prints and the mathematics fix (no GPU)."""
import itertools
import math

import numpy as np
import pytest

from oracle import planner as P


# ---- memory cost model ---------------------------------------------------------------------------

OPT30B = dict(L=48, h1=7168, h2=28672, vocab=50272, pos=2050)


def test_memory_model_matches_the_papers_example():
    # Sec. 4.1 gives the embeddings + LM head of OPT-30b as 1.4 GB of a 60 GB fp16 model
    m = OPT30B
    emb = P.embedding_bytes(m["vocab"], m["h1"], m["pos"], m["h1"])
    total = emb + m["L"] * P.layer_weight_bytes(m["h1"], m["h2"], 16)
    # 1,470,787,584 B = 1.47e9 B = 1.37 GiB, printed as 1.4 GB; the whole model 60.7e9 B, printed as 60 GB
    assert emb == (2 * 50272 * 7168 + 2050 * 7168) * 2 == 1470787584
    assert 1.35 <= emb / 2 ** 30 <= 1.45 and 59.5e9 <= total <= 61e9
    assert 0.02 < emb / total < 0.03


def test_memory_model_structure():
    h1, h2 = 1024, 4096
    w16 = P.layer_weight_bytes(h1, h2, 16)
    # the quantised part scales with the bitwidth, the layer-norm term does not
    for b in (3, 4, 8):
        assert P.layer_weight_bytes(h1, h2, b) - 6 * h1 == (w16 - 6 * h1) * b / 16
    assert P.layer_weight_bytes(h1, h2, 4, rmsnorm=True) == P.layer_weight_bytes(h1, h2, 4) - 2 * h1
    # counted weight by weight: q, k, v, out of h1 x h1 and two MLP matrices of h1 x h2
    n_weights = 4 * h1 * h1 + 2 * h1 * h2
    assert P.layer_weight_bytes(h1, h2, 8) == n_weights + 6 * h1
    # projections only when the embedding width differs from the hidden width
    assert P.embedding_bytes(100, 64, 10, 64) == (100 * 64 + 10 * 64 + 100 * 64) * 2
    assert P.embedding_bytes(100, 32, 10, 64) == (100 * 32 + 10 * 32 + 2 * 64 * 32 + 100 * 32) * 2
    # KV: K and V, fp16, every reserved position of every request
    assert P.kv_bytes(4, 512, 100, h1) == 2 * 4 * 612 * h1 * 2
    assert P.kv_bytes(4, 512, 100, h1, bit_kv=8) == P.kv_bytes(4, 512, 100, h1) / 2


# ---- latency regression ---------------------------------------------------------------------------------

def test_regression_recovers_a_flop_law_and_a_byte_law():
    h1 = 512
    v, s = np.meshgrid([1, 2, 4, 8], [128, 256, 384, 512])
    v, s = v.ravel(), s.ravel()
    # prefill time proportional to the layer's FLOPs: 24 v s h1^2 from the linears + 4 v s^2 h1 from attention
    t = 3e-15 * (24 * v * s * h1 * h1 + 4 * v * s * s * h1) + 7e-6
    c = P.fit_latency("prefill", v, s, t)
    assert np.allclose(c, [7e-6, 0, 0, 3e-15 * 24 * h1 * h1, 3e-15 * 4 * h1], rtol=1e-6, atol=1e-12)
    # decode time proportional to bytes: weights (constant), activations (v), KV (v * ctx)
    ctx = s
    t = 2e-12 * (12 * h1 * h1 * 0.5 + 40 * v * h1 + 4 * v * ctx * h1)
    c = P.fit_latency("decode", v, ctx, t)
    assert np.allclose(c, [2e-12 * 6 * h1 * h1, 2e-12 * 40 * h1, 2e-12 * 4 * h1, 0], rtol=1e-6, atol=1e-13)
    assert np.allclose(P.predict_latency("decode", c, [3, 5], [384, 768]),
                       2e-12 * (6 * h1 * h1 + 40 * np.array([3, 5]) * h1 + 4 * np.array([3 * 384, 5 * 768]) * h1))


def test_regression_is_least_squares():
    r = np.random.default_rng(0)
    v, s = r.integers(1, 9, 40), r.integers(64, 513, 40)
    t = r.random(40)
    for phase, feats in (("prefill", lambda: [np.ones(40), v, s, v * s, v * s * s]),
                         ("decode", lambda: [np.ones(40), v, v * s, s])):
        c = P.fit_latency(phase, v, s, t)
        res = t - P.predict_latency(phase, c, v, s)
        for f in feats():                                   # residual orthogonal to every regressor
            assert abs(np.dot(res, f)) < 1e-6 * np.linalg.norm(f)
        for k in range(len(c)):                             # and no nearby coefficient vector does better
            d = np.zeros(len(c))
            d[k] = 1e-3 * max(abs(c[k]), 1e-9)
            assert np.sum((t - P.predict_latency(phase, c + d, v, s)) ** 2) >= np.sum(res ** 2)


# ---- the objective ------------------------------------------------------------------------------------------

def tiny_problem(seed=0, L=5, N=2, bits=(4, 8, 16), **kw):
    r = np.random.default_rng(seed)
    nb = len(bits)
    scale = r.random(L) + 0.5
    omega = np.array([[scale[i] * 4.0 ** (-k) * (1 + 0.1 * r.random()) for k in range(nb)] for i in range(L)])
    lat_pre = np.array([[(1.0 + 0.3 * j) * (1.3 - 0.1 * k) * 1e-2 for k in range(nb)] for j in range(N)])
    lat_dec = np.array([[(1.0 + 0.5 * j) * (0.3 + 0.25 * k) * 1e-3 for k in range(nb)] for j in range(N)])
    lat_pre *= 1 + 0.05 * r.random(lat_pre.shape)
    lat_dec *= 1 + 0.05 * r.random(lat_dec.shape)
    mem = np.array([b / 8.0 + 0.25 for b in bits])          # binary fractions: sums are exact
    args = dict(bits=bits, omega=omega, lat_pre=lat_pre, lat_dec=lat_dec, mem=mem, cap=np.full(N, 4.25), emb=0.5,
                B=8, eta=2, xi=4, n=20, theta=1.0)
    args.update(kw)
    return P.Problem(**args)


def test_objective_worked_by_hand():
    # two stages, three layers, bits (4, 16); every number chosen to be summed by hand
    p = P.Problem(bits=(4, 16), omega=[[4, 1], [8, 2], [16, 3]], lat_pre=[[10, 6], [20, 12]], lat_dec=[[1, 2], [3, 5]],
                  mem=[1, 4], cap=[6, 5], emb=1, B=6, eta=2, xi=3, n=11, theta=0.5)
    # stage 0 = layers 0,1 at (16, 4): memory 4 + 1 + emb 1 = 6 <= 6; stage 1 = layer 2 at 16: 4 <= 5
    # T_pre = (6 + 10, 12) -> max 16, sum 28;  T_dec = (2 + 1, 5) -> max 5, sum 8
    # mu_pre = 3, mu_dec = 2: (3-1)*16 + (2-1)*(11-1)*5 + 28 + 8 = 32 + 50 + 36 = 118;  omega = 1 + 8 + 3 = 12 -> + 6
    assert P.objective(p, [2, 1], [1, 0, 1]) == 124.0
    assert P.objective(p, [2, 1], [1, 0, 1], with_latency=False) == 6.0
    # one more 16-bit layer on stage 0 does not fit (4 + 4 + 1 > 6)
    assert P.objective(p, [2, 1], [1, 1, 1]) == P.INF
    # the embeddings count on the first device only: stage 1 may hold 4 + 1 = 5
    assert P.objective(p, [1, 2], [1, 0, 1]) < P.INF and P.objective(p, [1, 2], [1, 1, 1]) == P.INF
    # a slow link sets the pace of its phase: T_max^pre = 40 instead of 16 adds (3-1) * 24
    p.comm_pre = np.array([40.0, 0.0])
    assert P.objective(p, [2, 1], [1, 0, 1]) == 124.0 + 48.0
    # malformed plans
    assert P.objective(p, [3, 0], [0, 0, 0]) == P.INF and P.objective(p, [1, 1], [0, 0, 0]) == P.INF


def test_objective_single_stage_single_microbatch():
    p = tiny_problem(1, L=4, N=1, B=4, eta=4, xi=4, cap=np.full(1, 100.0))
    ch = [0, 1, 2, 1]
    want = sum(p.lat_pre[0][c] + p.lat_dec[0][c] for c in ch) + sum(p.omega[i][c] for i, c in enumerate(ch))
    assert abs(P.objective(p, [4], ch) - want) < 1e-12


def test_partitions_enumerated():
    parts = list(P.all_partitions(6, 3))
    assert len(parts) == math.comb(5, 2) and len({tuple(c) for c in parts}) == len(parts)
    assert all(sum(c) == 6 and min(c) >= 1 for c in parts)


# ---- exact optimum and adabits -----------------------------------------------------------------------------------

def test_adabits_known_answers():
    # room for everything at the highest precision: that is the answer, with zero loss beyond omega at 16 bits
    p = tiny_problem(2, cap=np.full(2, 100.0))
    o, counts, choice = P.adabits(p)
    assert choice == [2] * 5 and abs(o - p.omega[:, 2].sum()) < 1e-12
    # room for the lowest precision only: a 4-bit layer takes 0.75
    p = tiny_problem(2, cap=np.array([2.0, 2.25]))       # device 0: emb 0.5 + 2 x 0.75 = 2.0; device 1: 3 x 0.75 = 2.25
    o, counts, choice = P.adabits(p)
    assert counts == [2, 3] and choice == [0] * 5
    # nothing fits
    p = tiny_problem(2, cap=np.array([1.0, 1.0]))
    assert P.adabits(p)[0] == P.INF
    # exactly one upgrade affordable on device 1: it goes to the layer (of that stage) that gains most
    p = tiny_problem(3, cap=np.array([2.0, 2.75]))       # 3 x 0.75 + 0.5 extra = one 4 -> 8 bit upgrade
    o, counts, choice = P.adabits(p)
    assert counts == [2, 3] and sorted(choice[2:]) == [0, 0, 1] and choice[:2] == [0, 0]
    gain = p.omega[2:, 0] - p.omega[2:, 1]
    assert choice[2 + int(np.argmax(gain))] == 1


def test_exact_optimum_dominates_random_plans():
    p = tiny_problem(4)
    best, counts, choice = P.exact_optimum(p)
    assert best == P.objective(p, counts, choice) < P.INF
    r = np.random.default_rng(0)
    for _ in range(300):
        c = list(P.all_partitions(p.L, p.N))[r.integers(0, 4)]
        ch = r.integers(0, 3, p.L).tolist()
        assert P.objective(p, c, ch) >= best
    # a huge theta makes quality everything: the optimum is the adabits plan's objective value
    p = tiny_problem(4, theta=1e9)
    assert abs(P.exact_optimum(p)[0] - P.objective(p, *P.adabits(p)[1:])) <= 1e-6 * P.exact_optimum(p)[0]


# ---- assignment inside a stage --------------------------------------------------------------------------------------

def test_best_assignment_against_all_permutations():
    r = np.random.default_rng(5)
    for n, ms in ((4, [0, 0, 1, 2]), (5, [2, 2, 2, 0, 1]), (3, [1, 1, 1]), (1, [2])):
        w = r.random((n, 3))
        got, choice = P.best_assignment(w, ms)
        want = min(sum(w[i][c] for i, c in enumerate(perm)) for perm in set(itertools.permutations(ms)))
        assert abs(got - want) < 1e-12 and sorted(choice) == sorted(ms)
        assert abs(sum(w[i][c] for i, c in enumerate(choice)) - want) < 1e-12


# ---- Algorithm 2 -------------------------------------------------------------------------------------------------------

def test_transfer_rules():
    rules = P.transfer_rules((3, 4, 8, 16))
    as_bits = {((3, 4, 8, 16)[a], (3, 4, 8, 16)[b], n) for a, b, n in rules}
    # the paper's example: one 8-bit layer of the other stage against two 4-bit layers of the straggler
    assert (4, 8, 2) in as_bits and (8, 16, 2) in as_bits and (4, 16, 4) in as_bits and (3, 16, 5) in as_bits
    assert (16, 4, 1) in as_bits and (4, 3, 1) in as_bits and len(rules) == 12
    # a rule never lets the straggler's weight memory grow when b_st < b_pi
    assert all(n * a <= b for a, b, n in as_bits if a < b)


def test_exchange_moves_what_the_rule_says():
    counts, ms = [3, 2], [[0, 0, 1], [1, 2]]
    # rule (4, 8, 2) with straggler 0: two 4-bit layers go to stage 1, one 8-bit layer comes back
    c2, m2 = P.exchange(counts, ms, 0, 1, (0, 1, 2))
    assert c2 == [2, 3] and m2 == [[1, 1], [0, 0, 2]]
    assert P.exchange(counts, ms, 1, 0, (0, 1, 2)) is None          # stage 1 owns no 4-bit layers
    assert P.exchange(counts, ms, 0, 1, (1, 0, 1)) is None          # stage 1 owns no 4-bit layer to hand back
    assert ms == [[0, 0, 1], [1, 2]]                                # inputs untouched
    # a stage in between keeps its multiset
    c3, m3 = P.exchange([2, 1, 1], [[0, 0], [2], [1]], 0, 2, (0, 1, 2))
    assert c3 == [1, 1, 2] and m3 == [[1], [2], [0, 0]]


@pytest.mark.parametrize("seed", range(6))
def test_bitwidth_transfer_improves_and_is_bounded_by_the_optimum(seed):
    p = tiny_problem(10 + seed, theta=[0.01, 0.1, 1.0][seed % 3])
    o_ada, counts, choice = P.adabits(p)
    start = P.objective(p, counts, choice)
    obj, c2, ch2, rounds = P.bitwidth_transfer(p, counts, choice)
    best = P.exact_optimum(p)[0]
    assert best - 1e-12 <= obj <= start + 1e-12
    assert abs(obj - P.objective(p, c2, ch2)) < 1e-12 and sum(c2) == p.L and min(c2) >= 1
    # a local optimum: no single exchange from the result improves it
    ms = P.multisets_of(c2, ch2)
    for st in range(p.N):
        for pi in range(p.N):
            for rule in P.transfer_rules(p.bits):
                if st != pi and st == int(np.argmax(P.stage_rank_key(p, c2, ch2))):
                    moved = P.exchange(c2, ms, st, pi, rule)
                    if moved:
                        assert P.objective(p, moved[0], P.choice_from_multisets(p, *moved)) >= obj


def test_bitwidth_transfer_relieves_a_slow_stage():
    # stage 1 is four times slower and the quality weight is negligible: the best plan moves layers off it.
    # Start from the even split at 8 bits everywhere; memory allows 4 layers per device at 8 bits, or more at 4 bits.
    L, bits = 6, (4, 8)
    omega = np.full((L, 2), 1e-9)
    lat_pre = np.array([[1.0, 1.0], [4.0, 4.0]])
    lat_dec = np.array([[0.1, 0.1], [0.4, 0.4]])
    p = P.Problem(bits=bits, omega=omega, lat_pre=lat_pre, lat_dec=lat_dec, mem=[0.5, 1.0], cap=[4.0, 4.0], emb=0.0,
                  B=4, eta=1, xi=2, n=10, theta=1.0)
    obj, counts, choice, rounds = P.bitwidth_transfer(p, [3, 3], [1] * 6)
    # nothing 4-bit exists at the start, so only (8 -> 4, nums 1) rules apply and they change no latency: no move
    assert rounds == 0 and counts == [3, 3]
    # with 4-bit layers on the straggler, rule (4, 8, 2) hands two of them over for one 8-bit layer.  By hand:
    # mu_pre = 4, mu_dec = 2, n = 10.  Start [3, 3]: T_pre = (3, 12), T_dec = (.3, 1.2):
    #   3 * 12 + 1 * 9 * 1.2 + 15 + 1.5 = 63.3.   After the exchange [4, 2]: T_pre = (4, 8), T_dec = (.4, .8):
    #   3 * 8 + 9 * .8 + 12 + 1.2 = 44.4.   Then the straggler owns one 4-bit layer only: no rule moves a layer, end.
    start = [1, 1, 1, 0, 0, 0]
    assert abs(P.objective(p, [3, 3], start) - 63.3) < 1e-6
    obj, counts, choice, rounds = P.bitwidth_transfer(p, [3, 3], start)
    assert rounds == 1 and counts == [4, 2] and abs(obj - 44.4) < 1e-6
    assert P.multisets_of(counts, choice) == [[0, 0, 1, 1], [0, 1]]
    # the program's optimum puts five layers on the fast device: 3 * 5 + 9 * .5 + 9 + .9 = 29.4 (the heuristic
    # stops above it: its rules move layers only in exchange for a wider one)
    assert abs(P.exact_optimum(p)[0] - 29.4) < 1e-6
