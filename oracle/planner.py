"""CPU oracle of the assigner's cost models and of the bitwidth-transfer heuristic (numpy, fp64).

TEST INFRASTRUCTURE ONLY, like the rest of this package: imported by tests/, smoke() and the
cpu_baseline leg of bench.py; the product never imports it and it imports nothing from the product.

What is written out here, from LLM-PQ (arXiv 2403.01136):
  memory cost model      Sec. 4.1 "Memory Cost Model": bytes of the embeddings, of one decoder layer at a
                         bitwidth, of the KV cache reserved for s + n positions
  latency cost model     Sec. 4.1 "Latency Cost Model": a linear regression per phase and precision, prefill on
                         v, s, vs, vs^2 and decode on v, v(t+s), t+s (least squares, with an intercept)
  objective              Sec. 4.3, Eq. (1) with its constraints on stage times, communication times and device
                         memory: pipeline latency of a batch plus theta times the summed variance indicator,
                         infinite if a device runs out of memory
  exact optimum          the same program solved by enumerating every contiguous partition and every bitwidth
                         choice (tiny instances only); `adabits` is that program without the latency terms
  bitwidth transfer      Sec. 4.3, Algorithm 2: start from a plan, repeatedly exchange layers between the
                         slowest stage and another one by the rules (b_st, b_pi, nums) while the objective improves

Readings taken where the text leaves a choice (all listed again in the build's design notes):
  * position embeddings count pos_s * d_t entries (the prose), not d_p * h_1 (the printed sum);
  * the layer-norm term of a layer is 6 h_1 bytes (4 h_1 with RMSNorm), as printed;
  * the KV cache of a stage holds the whole global batch B; peak temporary memory is a per-device constant;
  * one model's decoder layers share a shape, so latencies carry no layer index: l[j][b];
  * Eq. (1) is taken as printed: T_dec enters once, the (n - 1) factor multiplies only the T_max^dec term;
  * every stage holds at least one layer;
  * a plan is the layer count of each stage plus each stage's multiset of bitwidths; which of the stage's layers
    gets which of its bitwidths is always the choice with the least summed indicator ("find optimal layers");
  * the rules are C = {(a, b, max(1, b // a)) : a != b in BITs}: the straggler hands `nums` layers of a bits to the
    other stage and takes one layer of b bits back; stages in between keep their counts and multisets (their
    windows of layers shift); a rule is valid if both stages own those layers and every device still has room;
  * stages are ranked by (ceil(B/eta)) * T_pre,j + (ceil(B/xi) - 1) * (n - 1) * T_dec,j + T_dec,j, the coefficient the
    stage's times would have in Eq. (1) if it were the slowest in both phases; the scan visits every other stage,
    fastest first, and the strictly best exchange of a scan is applied; equal objectives keep the first found.
"""
import itertools
import math

import numpy as np
from scipy.optimize import linear_sum_assignment

INF = float("inf")


# ---- memory cost model (Sec. 4.1) ----------------------------------------------------------------

def embedding_bytes(vocab, d_t, pos, h1):
    """Token and position embeddings, the two projections if h1 != d_t, and the LM head, all fp16."""
    proj = 2 * h1 * d_t if h1 != d_t else 0
    return (vocab * d_t + pos * d_t + proj + vocab * d_t) * 2


def layer_weight_bytes(h1, h2, bit, rmsnorm=False):
    """Linear weights of one decoder layer at `bit` bits each, plus the layer-norm term."""
    return (4 * h1 * h1 + 2 * h1 * h2) * bit / 8.0 + (4 * h1 if rmsnorm else 6 * h1)


def kv_bytes(v, s, n, h1, bit_kv=16):
    """K and V of one layer for v requests of s prompt + n generated positions."""
    return 2.0 * v * (s + n) * h1 * bit_kv / 8.0


# ---- latency cost model (Sec. 4.1) ------------------------------------------------------------------

def prefill_features(v, s):
    v, s = np.asarray(v, float), np.asarray(s, float)
    return np.stack([np.ones_like(v), v, s, v * s, v * s * s], axis=-1)


def decode_features(v, ctx):
    """ctx = t + s, the number of positions already in the cache."""
    v, ctx = np.asarray(v, float), np.asarray(ctx, float)
    return np.stack([np.ones_like(v), v, v * ctx, ctx], axis=-1)


def fit_latency(phase, v, length, t):
    X = prefill_features(v, length) if phase == "prefill" else decode_features(v, length)
    coef, *_ = np.linalg.lstsq(X, np.asarray(t, float), rcond=None)
    return coef


def predict_latency(phase, coef, v, length):
    X = prefill_features(v, length) if phase == "prefill" else decode_features(v, length)
    return X @ np.asarray(coef, float)


# ---- plans and the objective (Sec. 4.3, Eq. 1) --------------------------------------------------------

class Problem:
    """Everything Eq. (1) and its constraints read.  bits: the allowed bitwidths, ascending.
    omega[i][k]: indicator of layer i at bits[k].  lat_pre[j][k], lat_dec[j][k]: seconds of one layer at bits[k] on
    device j at the prefill / decode micro-batch.  mem[k]: bytes a layer at bits[k] reserves (weights + KV).
    cap[j]: bytes device j offers (temporary memory already taken off); emb: bytes the first device also holds.
    comm_pre[j], comm_dec[j]: seconds P/f_j of the send from stage j (0 to ignore)."""

    def __init__(self, bits, omega, lat_pre, lat_dec, mem, cap, emb, B, eta, xi, n, theta, comm_pre=None, comm_dec=None):
        self.bits = list(bits)
        self.omega = np.asarray(omega, float)
        self.lat_pre = np.asarray(lat_pre, float)
        self.lat_dec = np.asarray(lat_dec, float)
        self.mem = np.asarray(mem, float)
        self.cap = np.asarray(cap, float)
        self.emb = float(emb)
        self.B, self.eta, self.xi, self.n, self.theta = B, eta, xi, n, float(theta)
        self.L, self.N = self.omega.shape[0], self.cap.shape[0]
        self.comm_pre = np.zeros(self.N) if comm_pre is None else np.asarray(comm_pre, float)
        self.comm_dec = np.zeros(self.N) if comm_dec is None else np.asarray(comm_dec, float)

    def mu_pre(self):
        return math.ceil(self.B / self.eta)

    def mu_dec(self):
        return math.ceil(self.B / self.xi)


def stage_windows(counts):
    start = 0
    for c in counts:
        yield start, start + c
        start += c


def stage_times(p, counts, choice):
    """choice[i] = index into p.bits of layer i.  Returns (T_pre,j) and (T_dec,j)."""
    tp, td = np.zeros(p.N), np.zeros(p.N)
    for j, (a, b) in enumerate(stage_windows(counts)):
        for i in range(a, b):
            tp[j] += p.lat_pre[j][choice[i]]
            td[j] += p.lat_dec[j][choice[i]]
    return tp, td


def memory_ok(p, counts, choice):
    for j, (a, b) in enumerate(stage_windows(counts)):
        need = sum(p.mem[choice[i]] for i in range(a, b)) + (p.emb if j == 0 else 0.0)
        if need > p.cap[j]:
            return False
    return True


def objective(p, counts, choice, with_latency=True):
    """Eq. (1); INF if a stage is empty or a device lacks memory."""
    if len(counts) != p.N or sum(counts) != p.L or min(counts) < 1 or not memory_ok(p, counts, choice):
        return INF
    quality = p.theta * sum(p.omega[i][choice[i]] for i in range(p.L))
    if not with_latency:
        return quality
    tp, td = stage_times(p, counts, choice)
    tmax_pre = max(tp.max(), p.comm_pre.max())
    tmax_dec = max(td.max(), p.comm_dec.max())
    t_pre, t_dec = sum(tp.tolist()), sum(td.tolist())              # plain left-to-right sums
    lat = (p.mu_pre() - 1) * tmax_pre + (p.mu_dec() - 1) * (p.n - 1) * tmax_dec + t_pre + t_dec
    return lat + quality


def all_partitions(L, N):
    """Every way to cut L layers into N consecutive non-empty stages."""
    for cuts in itertools.combinations(range(1, L), N - 1):
        edges = (0,) + cuts + (L,)
        yield [edges[k + 1] - edges[k] for k in range(N)]


def exact_optimum(p, with_latency=True):
    """Enumeration of the whole program (tiny instances).  Returns (objective, counts, choice)."""
    best = (INF, None, None)
    nb = len(p.bits)
    for counts in all_partitions(p.L, p.N):
        for choice in itertools.product(range(nb), repeat=p.L):
            o = objective(p, counts, choice, with_latency)
            if o < best[0]:
                best = (o, list(counts), list(choice))
    return best


def adabits(p):
    return exact_optimum(p, with_latency=False)


# ---- which layer of a stage gets which of the stage's bitwidths ------------------------------------------

def best_assignment(omega_window, multiset):
    """omega_window [n][nb]; multiset: n indices into bits.  Least summed indicator over all ways to hand the
    multiset's entries to the n layers.  Returns (sum, choice per layer)."""
    n = len(multiset)
    if n == 0:
        return 0.0, []
    cost = np.asarray(omega_window, float)[:, list(multiset)]        # layer x slot
    r, c = linear_sum_assignment(cost)
    choice = [0] * n
    for layer, slot in zip(r, c):
        choice[layer] = multiset[slot]
    return float(cost[r, c].sum()), choice


def choice_from_multisets(p, counts, multisets):
    choice = []
    for (a, b), ms in zip(stage_windows(counts), multisets):
        choice += best_assignment(p.omega[a:b], sorted(ms))[1]
    return choice


def multisets_of(counts, choice):
    return [sorted(choice[a:b]) for a, b in stage_windows(counts)]


# ---- Algorithm 2: bitwidth transfer -------------------------------------------------------------------------

def transfer_rules(bits):
    """(index of b_st, index of b_pi, nums) for every ordered pair of different bitwidths."""
    return [(ia, ib, max(1, b // a)) for ia, a in enumerate(bits) for ib, b in enumerate(bits) if a != b]


def stage_rank_key(p, counts, choice):
    tp, td = stage_times(p, counts, choice)
    return p.mu_pre() * tp + ((p.mu_dec() - 1) * (p.n - 1) + 1) * td


def exchange(counts, multisets, st, pi, rule):
    """The plan after the straggler st hands `nums` layers of b_st to pi and takes one of b_pi back; None if either
    stage does not own those layers."""
    ia, ib, nums = rule
    if multisets[st].count(ia) < nums or multisets[pi].count(ib) < 1:
        return None
    ms = [list(m) for m in multisets]
    for _ in range(nums):
        ms[st].remove(ia)
        ms[pi].append(ia)
    ms[pi].remove(ib)
    ms[st].append(ib)
    new_counts = [len(m) for m in ms]
    return new_counts, [sorted(m) for m in ms]


def bitwidth_transfer(p, counts, choice, max_rounds=10000):
    """Algorithm 2 from a given starting plan.  Returns (objective, counts, choice, rounds applied)."""
    counts = list(counts)
    multisets = multisets_of(counts, choice)
    choice = choice_from_multisets(p, counts, multisets)
    obj0 = objective(p, counts, choice)
    rules = transfer_rules(p.bits)
    rounds = 0
    while rounds < max_rounds:
        key = stage_rank_key(p, counts, choice)
        order = sorted(range(p.N), key=lambda j: (key[j], j))         # ascending; ties by stage index
        st = order[-1]
        sol = None
        for pi in order[:-1]:
            for rule in rules:
                moved = exchange(counts, multisets, st, pi, rule)
                if moved is None:
                    continue
                c2, m2 = moved
                ch2 = choice_from_multisets(p, c2, m2)
                o = objective(p, c2, ch2)                               # INF if memory is exceeded: not valid
                if o < obj0:
                    obj0, sol = o, (c2, m2, ch2)
        if sol is None:
            break
        counts, multisets, choice = sol
        rounds += 1
    return obj0, counts, choice, rounds
