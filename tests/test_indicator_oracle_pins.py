"""Pins of oracle/indicator.py (Sec. 4.2, Eq. 3) against closed forms and invariants; no GPU."""
import math

import numpy as np

from oracle import indicator as I


def test_closed_form_single_group():
    # one row, one group: the group form and the printed (tensor) form coincide; values by hand
    w = np.zeros((1, 128)); w[0, 3] = 1.5; w[0, 77] = -0.5          # range 2, max|w| 1.5, D = 128
    x = np.array([[1.0, 3.0] * 64])                                  # E = 2, Var = 1
    det, sto = I.indicator(w, x, False), I.indicator(w, x, True)
    for b in (3, 4, 8):
        want = 128 * (2.0 / (2 ** b - 1)) ** 2
        assert math.isclose(det[("group", b)], want / 4) and math.isclose(det[("tensor", b)], want / 4)
        assert math.isclose(sto[("group", b)], want * (4 + 1) / 6)
    want = 128 * (1.5 / 127) ** 2
    assert math.isclose(det[("group", "8s")], want / 4) and math.isclose(det[("tensor", "8s")], want / 4)


def test_invariants():
    r = np.random.default_rng(3)
    w = r.standard_normal((64, 384)); x = r.standard_normal((9, 384)) + 0.3
    a = I.indicator(w, x)
    # a scaling factor is homogeneous: c * W scales the indicator by c^2, and so does c * X
    for key, v in I.indicator(3 * w, x).items():
        assert math.isclose(v, 9 * a[key], rel_tol=1e-12)
    for key, v in I.indicator(w, -2 * x).items():
        assert math.isclose(v, 4 * a[key], rel_tol=1e-12)
    # bitwidths: only the denominator changes
    assert math.isclose(a[("group", 3)] / a[("group", 4)], (15 / 7) ** 2, rel_tol=1e-12)
    assert math.isclose(a[("tensor", 4)] / a[("tensor", 8)], (255 / 15) ** 2, rel_tol=1e-12)
    # a group's range never exceeds the matrix's: finer scales can only lower the estimate
    for b in (3, 4, 8, "8s"):
        assert a[("group", b)] <= a[("tensor", b)] * (1 + 1e-12)
    # shifting X leaves the deterministic form alone and raises the stochastic one by D S^2 (2 m c + c^2) / 6
    assert math.isclose(I.indicator(w, x + 5)[("group", 4)], a[("group", 4)], rel_tol=1e-10)
    s0, s1 = I.indicator(w, x, True)[("tensor", 4)], I.indicator(w, x + 5, True)[("tensor", 4)]
    d_s2 = 64 * 384 * ((w.max() - w.min()) / 15) ** 2
    assert math.isclose(s1 - s0, d_s2 * (2 * x.mean() * 5 + 25) / 6, rel_tol=1e-9)
    # constant input: no variance, so deterministic rounding adds none
    assert I.indicator(w, np.full((4, 384), 2.5))[("group", 8)] == 0.0
    # permuting rows, or columns within a group, changes nothing
    p = r.permutation(64)
    cols = np.arange(384).reshape(3, 128); cols = np.concatenate([c[r.permutation(128)] for c in cols])
    b_ = I.indicator(w[p][:, cols], x[:, cols])
    for key in a:
        assert math.isclose(a[key], b_[key], rel_tol=1e-12)


def test_scalar_loops():
    r = np.random.default_rng(4)
    w = r.standard_normal((3, 256)); x = r.standard_normal((2, 256))
    a = I.indicator(w, x, True)
    xs = [float(v) for v in x.ravel()]
    m = sum(xs) / len(xs); var = sum((v - m) ** 2 for v in xs) / len(xs)
    g = (m * m + var) / 6
    tot = 0.0
    for n in range(3):
        for j in range(2):
            grp = [float(v) for v in w[n, 128 * j:128 * j + 128]]
            tot += 128 * ((max(grp) - min(grp)) / 15) ** 2
    assert math.isclose(a[("group", 4)], tot * g, rel_tol=1e-12)
    rows = sum(256 * (max(abs(float(v)) for v in w[n]) / 127) ** 2 for n in range(3))
    assert math.isclose(a[("group", "8s")], rows * g, rel_tol=1e-12)
