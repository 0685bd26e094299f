"""CPU oracle of the variance indicator (numpy, fp64).  TEST INFRASTRUCTURE ONLY, like the rest of oracle/.

LLM-PQ (arXiv 2403.01136) Sec. 4.2, Theorem 1 and the Proposition "Variance Indicator" (Eq. 3): the extra
output variance of a linear operator whose weight W is quantised to b bits is estimated as
    D_W * S_W(b)^2 * G(X),
with D_W the number of weights, S_W(b) the scaling factor ((W_max - W_min) / (2^b - 1) asymmetric,
max(|W_max|, |W_min|) / (2^(b-1) - 1) symmetric) and G(X) = Var[X] / 4 for deterministic rounding or
(E[X]^2 + Var[X]) / 6 for stochastic rounding; a layer's indicator is the sum over its linear operators.

Two forms are returned.  "tensor": the paper's expression as printed, one scaling factor for the whole
matrix.  "group": the same expression with the granularity of the quantiser that is actually used here -- a
scale per (row, 128 columns) for the asymmetric scheme and per row for the symmetric one -- i.e. the sum over
scale groups of (weights in the group) * (the group's scaling factor)^2, which reduces to the printed form when
there is one group.  Scaling factors are exact quotients of the fp16 weights (not rounded to fp16); E and Var
are taken over all elements of X (population variance).
"""
import numpy as np

BITS = (3, 4, 8)
GROUP = 128


def g_of_x(x, stochastic):
    x = np.asarray(x, dtype=np.float64)
    mean, var = x.mean(), x.var()
    return (mean * mean + var) / 6.0 if stochastic else var / 4.0


def indicator(w, x, stochastic=False):
    """w [N][K], x [M][K] (fp16 values).  Returns a dict: ("group", b) and ("tensor", b) for b in 3, 4, 8
    (asymmetric), ("group", "8s") and ("tensor", "8s") for the symmetric 8-bit scheme."""
    w = np.asarray(w, dtype=np.float64)
    n, k = w.shape
    g = g_of_x(x, stochastic)
    grp = w.reshape(n, k // GROUP, GROUP)
    range_sq = ((grp.max(axis=2) - grp.min(axis=2)) ** 2).sum()          # sum over (row, group) of (max - min)^2
    absmax_sq = (np.abs(w).max(axis=1) ** 2).sum()                       # sum over rows of max|w|^2
    out = {}
    for b in BITS:
        out[("group", b)] = GROUP * range_sq / (2 ** b - 1) ** 2 * g
        out[("tensor", b)] = n * k * ((w.max() - w.min()) / (2 ** b - 1)) ** 2 * g
    out[("group", "8s")] = k * absmax_sq / 127.0 ** 2 * g
    out[("tensor", "8s")] = n * k * (np.abs(w).max() / 127.0) ** 2 * g
    return out


ORDER = [("group", 3), ("group", 4), ("group", 8), ("group", "8s"), ("tensor", 3), ("tensor", 4), ("tensor", 8), ("tensor", "8s")]
