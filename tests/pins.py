"""Pins of the CPU oracle: checks against what the paper and the mathematics fix.

Each pin takes an ``oracle.Oracle`` instance and raises AssertionError on failure, so the
same pins run against the real oracle (test_oracle_pins.py) and against copies with a
planted mistake (test_oracle_mutants.py), which every pin set must catch.

None of these re-types the oracle's code path: they use closed forms, exact rational
arithmetic, numpy's own float16 / float64 routines, invariants, or a bit-by-bit reading of the
storage-format description.

Citations are to LLM-PQ (arXiv 2403.01136): Sec. 2.4 (quantise / dequantise), Sec. 4.2
(scaling factors), Sec. 4.1 (bit/8 bytes per weight), App. A.1 (|err| <= s/2).
"""
from fractions import Fraction

import numpy as np

FP16, ASYM, SYM = 0, 1, 2
ASYM_BITS = (3, 4, 8)


def f16(a):
    return np.asarray(a, dtype=np.float16)


def as_f16(u16):
    return np.asarray(u16, dtype=np.uint16).view(np.float16)


def synth_w(N, K, seed, outliers=True):
    rng = np.random.default_rng(seed)
    w = rng.standard_normal((N, K)).astype(np.float32) * np.float32(0.02)
    if outliers:
        m = rng.random((N, K)) < 0.001
        w[m] *= 20
    return w.astype(np.float16)


# ---------------------------------------------------------------------------------------
# fp16 conversions against numpy's float16 (an independent, IEEE-correct implementation)
# ---------------------------------------------------------------------------------------

def pin_fp16_conversions(orc):
    allh = np.arange(65536, dtype=np.uint16)
    want = allh.view(np.float16).astype(np.float32)
    got = np.array([orc.h2f(int(b)) for b in allh], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32)[~np.isnan(want)], want.view(np.uint32)[~np.isnan(want)])
    assert np.all(np.isnan(got[np.isnan(want)]))
    rng = np.random.default_rng(7)
    # random magnitudes over the whole fp16 range incl. subnormals and overflow
    v = (rng.standard_normal(20000) * np.exp2(rng.uniform(-30, 17, 20000))).astype(np.float32)
    # exact ties between neighbouring fp16 values, and their fp32 neighbours
    h = rng.integers(0, 0x7bff, 5000).astype(np.uint16)
    lo, hi = h.view(np.float16).astype(np.float64), (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    mid = ((lo + hi) / 2).astype(np.float32)
    ties = np.concatenate([mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9)), -mid])
    edge = np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, -1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0001,
                     2.0 ** -14, 2.0 ** -14 * 0.9999, np.inf, -np.inf], dtype=np.float32)
    with np.errstate(over="ignore"):
        for vals in (v, ties, edge):
            want16 = vals.astype(np.float16).view(np.uint16)
            got16 = np.array([orc.f2h(float(t)) for t in vals], dtype=np.uint16)
            assert np.array_equal(got16, want16), np.flatnonzero(got16 != want16)[:5]


# ---------------------------------------------------------------------------------------
# P1: storage format.  Density (Sec. 4.1), round trip, and a bit-by-bit reading of the
# format's prose description that uses none of the oracle's word arithmetic.
# ---------------------------------------------------------------------------------------

def spec_bit_positions(bits, n, k, K):
    """Absolute bit positions (LSB first) inside the packed byte string of the code of weight
    (row n, column k) -- read off the format description, one bit at a time."""
    KT = K // 128
    tile_bytes = 16 * 128 * bits // 8
    block, t, r = n // 64, n % 4, (n % 64) // 4          # tile t of a 64-row block holds rows 4r + t
    kt, kk = k // 128, k % 128
    j, kq, e = kk // 32, (kk % 32) // 8, kk % 8
    lane = 16 * kq + r
    tile_bit0 = 8 * tile_bytes * ((block * KT + kt) * 4 + t)
    if bits == 4:
        start = 8 * 16 * lane + 32 * j + 4 * (e // 2) + 16 * (e % 2)
        return [tile_bit0 + start + i for i in range(4)]
    if bits == 3:
        c = 8 * j + e
        P, h = c // 2, c % 2
        base = tile_bit0 + 8 * 12 * lane
        if P < 15:
            return [base + 32 * (P // 5) + 16 * h + 3 * (P % 5) + i for i in range(3)]
        return [base + 32 * i + 16 * h + 15 for i in range(3)]
    if bits == 8:
        byte = 1024 * (j // 2) + 16 * lane + 8 * (j % 2) + e
        return [tile_bit0 + 8 * byte + i for i in range(8)]
    if bits == 16:
        byte = 1024 * j + 16 * lane + 2 * e
        return [tile_bit0 + 8 * byte + i for i in range(16)]
    raise ValueError(bits)


def spec_pack(codes, bits):
    """Pack int codes [N][K] by setting single bits at spec_bit_positions (slow, tiny inputs)."""
    N, K = codes.shape
    out = np.zeros(N * K * bits // 8, dtype=np.uint8)
    for n in range(N):
        for k in range(K):
            c = int(codes[n, k]) & ((1 << bits) - 1)
            for i, p in enumerate(spec_bit_positions(bits, n, k, K)):
                if (c >> i) & 1:
                    out[p // 8] |= 1 << (p % 8)
    return out


def spec_unpack_one(packed, bits, K, n, k, signed=False):
    c = 0
    for i, p in enumerate(spec_bit_positions(bits, n, k, K)):
        c |= ((int(packed[p // 8]) >> (p % 8)) & 1) << i
    if signed and c >= 128:
        c -= 256
    return c


def pin_pack_density_and_roundtrip(orc):
    rng = np.random.default_rng(11)
    for bits, scheme in ((3, ASYM), (4, ASYM), (8, ASYM), (8, SYM)):
        for (N, K) in ((64, 128), (192, 384)):
            cb, sb, zb = orc.packed_sizes(bits, scheme, K, N)
            assert cb * 8 == K * N * bits                       # Sec. 4.1: bit/8 bytes per weight
            assert sb == (N * (K // 128) * 2 if scheme == ASYM else N * 2)
            assert zb == (sb if scheme == ASYM else 0)
            lo, hi = (0, (1 << bits) - 1) if scheme == ASYM else (-127, 127)
            pats = [rng.integers(lo, hi + 1, (N, K)), np.full((N, K), lo), np.full((N, K), hi),
                    np.where((np.arange(K)[None, :] + np.arange(N)[:, None]) % 2, lo, hi)]
            for codes in pats:
                codes = codes.astype(np.int32)
                p = orc.pack(codes, bits, scheme)
                assert p.dtype == np.uint8 and p.size == cb
                assert np.array_equal(orc.unpack(p, bits, scheme, K, N), codes)
    cb, sb, zb = orc.packed_sizes(16, FP16, 256, 64)
    assert (cb, sb, zb) == (256 * 64 * 2, 0, 0)
    for bad_n in (16, 32, 96):
        try:
            orc.packed_sizes(4, ASYM, 128, bad_n)
        except ValueError:
            continue
        raise AssertionError("N must be a multiple of 64")


def pin_pack_matches_format_description(orc):
    rng = np.random.default_rng(12)
    N, K = 128, 256
    for bits, scheme in ((3, ASYM), (4, ASYM), (8, ASYM), (8, SYM)):
        lo, hi = (0, (1 << bits) - 1) if scheme == ASYM else (-127, 127)
        codes = rng.integers(lo, hi + 1, (N, K)).astype(np.int32)
        assert np.array_equal(orc.pack(codes, bits, scheme), spec_pack(codes, bits))
        # every bit of the packed buffer is used exactly once (dense, no overlap)
        seen = np.zeros(N * K * bits, dtype=np.int32)
        for n in range(N):
            for k in range(K):
                for pos in spec_bit_positions(bits, n, k, K):
                    seen[pos] += 1
        assert np.all(seen == 1)
    # one-hot probes: a single code set to all-ones lights exactly its own bits
    for bits in (3, 4, 8):
        for (n, k) in ((0, 0), (5, 31), (63, 127), (65, 130), (127, 255), (9, 94), (9, 95), (70, 7)):
            codes = np.zeros((N, K), np.int32)
            codes[n, k] = (1 << bits) - 1
            p = orc.pack(codes, bits, ASYM)
            on = np.flatnonzero(np.unpackbits(p, bitorder="little"))
            assert list(on) == sorted(spec_bit_positions(bits, n, k, K))
    # stored order of scales and zeros: group-major, index g * N + n
    nat = rng.integers(0, 65535, (N, K // 128)).astype(np.uint16)
    st = orc.store_scales(nat, K)
    assert st.shape == (K // 128, N)
    for n in (0, 1, 63, 64, 127):
        for g in range(K // 128):
            assert st.reshape(-1)[g * N + n] == nat[n, g]
    w = synth_w(N, K, 13)
    packed, s_st, z_st = orc.quantize_pack(w, 4, ASYM)
    codes, s_nat, z_nat = orc.quantize(w, 4, ASYM)
    assert np.array_equal(s_st, s_nat.T) and np.array_equal(z_st, z_nat.T) and np.array_equal(packed, orc.pack(codes, 4, ASYM))
    _, s_row, z_row = orc.quantize_pack(w, 8, SYM)
    assert s_row.shape == (N,) and z_row is None
    # 16-bit layers: the fp16 bit patterns, unchanged, at the positions the description gives
    p16 = orc.pack_fp16(w)
    assert np.array_equal(p16, spec_pack(w.view(np.uint16).astype(np.int64), 16))
    assert np.array_equal(orc.unpack_fp16(p16, K, N), w.view(np.uint16))
    assert np.array_equal(np.sort(p16.view(np.uint16)), np.sort(w.view(np.uint16).reshape(-1)))


# ---------------------------------------------------------------------------------------
# P7: values on an exact grid -- Sec. 2.4's formulas give the codes in closed form
# ---------------------------------------------------------------------------------------

def pin_exact_grid_examples(orc, golden_lines=None):
    for bits in ASYM_BITS:
        q = (1 << bits) - 1
        for lo, step in ((-0.9375, 0.125), (0.5, 2.0 ** -6), (-3.0, 0.25)):
            if abs(lo) + q * step >= 2048 * step:
                continue                     # keep every grid value exactly representable in fp16
            idx = (np.arange(128) * 5 + 3) % (q + 1)
            idx[7], idx[100] = 0, q          # both ends present
            w = np.tile(f16(lo + idx * step), (64, 1))
            assert np.array_equal(w[0].astype(np.float64), lo + idx * step)
            codes, s, z = orc.quantize(w, bits, ASYM)
            assert np.array_equal(codes, np.tile(idx, (64, 1)))
            assert np.all(as_f16(s) == np.float16(step)) and np.all(as_f16(z) == np.float16(lo))
            d = orc.dequant(codes, s, z, bits, ASYM)
            assert np.array_equal(d.astype(np.float64), w.astype(np.float64))
    if golden_lines is not None:
        # the hand-written fixture: "bits | values... | scale zero | codes..."
        for line in golden_lines:
            bits, vals, sz, codes = [t.strip() for t in line.split("|")]
            bits = int(bits)
            vals = np.array([float(t) for t in vals.split()])
            want = np.array([int(t) for t in codes.split()])
            scale, zero = [float(t) for t in sz.split()]
            reps = 128 // len(vals)
            w = np.tile(f16(np.tile(vals, reps)), (64, 1))
            c, s, z = orc.quantize(w, bits, ASYM)
            assert np.array_equal(c[3], np.tile(want, reps))
            assert float(as_f16(s)[3, 0]) == scale and float(as_f16(z)[3, 0]) == zero


# ---------------------------------------------------------------------------------------
# P2 / P3 and exact-arithmetic check of O1-O4 on the synthetic weight distribution
# ---------------------------------------------------------------------------------------

def pin_rtn_against_exact_arithmetic(orc):
    """Scale, zero and codes against Fractions: scale is the fp16 nearest to
    (max-min)/(2^b-1), zero is the minimum, each code is a nearest integer of
    (w-zero)/scale (Sec. 2.4), dequant is scale*code+zero to fp32 accuracy."""
    N, K = 64, 256
    w = synth_w(N, K, 21)
    check_rows = (0, 1, 2, 3, 17, 42, 63)
    wf = w.astype(np.float64)
    for bits in ASYM_BITS:
        q = (1 << bits) - 1
        codes, s, z = orc.quantize(w, bits, ASYM)
        sf, zf = as_f16(s).astype(np.float64), as_f16(z).astype(np.float64)
        deq = orc.dequant(codes, s, z, bits, ASYM).astype(np.float64)
        assert codes.min() >= 0 and codes.max() <= q
        for n in check_rows:
            for g in range(K // 128):
                grp = wf[n, 128 * g:128 * g + 128]
                lo, hi = grp.min(), grp.max()
                assert zf[n, g] == lo
                exact_s = (Fraction(hi) - Fraction(lo)) / q
                # fp16 nearest (double rounding through fp32 may add 2^-13 of an fp16 ulp)
                ulp = Fraction(np.spacing(np.float16(sf[n, g])).astype(np.float64))
                assert abs(Fraction(sf[n, g]) - exact_s) <= ulp / 2 * (1 + Fraction(1, 4096))
                for k in range(128):
                    t = (Fraction(grp[k]) - Fraction(zf[n, g])) / Fraction(sf[n, g])
                    c = int(codes[n, 128 * g + k])
                    want = min(max(t, 0), q)
                    assert abs(c - want) <= Fraction(1, 2) + Fraction(1, 1 << 20), (n, g, k, c, float(t))
                    dq = Fraction(sf[n, g]) * c + Fraction(zf[n, g])
                    assert abs(Fraction(deq[n, 128 * g + k]) - dq) <= abs(dq) / (1 << 23)
                # P3: both ends of the code range are used
                assert codes[n, 128 * g + int(np.argmin(grp))] == 0
                assert codes[n, 128 * g + int(np.argmax(grp))] == q


def pin_error_bound_half_scale(orc):
    """App. A.1: |w - dequant(w)| <= s/2 for every element (tiny slack for fp32 rounding)."""
    N, K = 64, 512
    for seed, outl in ((31, True), (32, False)):
        w = synth_w(N, K, seed, outl)
        wf = w.astype(np.float64)
        for bits in ASYM_BITS:
            codes, s, z = orc.quantize(w, bits, ASYM)
            d = orc.dequant(codes, s, z, bits, ASYM).astype(np.float64)
            sf = np.repeat(as_f16(s).astype(np.float64), 128, axis=1)
            assert np.all(np.abs(wf - d) <= sf / 2 * (1 + 2.0 ** -9))
            # a coarser grid can only be worse on average: 3-bit error > 8-bit error
        e3 = np.abs(wf - orc.dequant(*orc.quantize(w, 3, ASYM), 3, ASYM)).mean()
        e8 = np.abs(wf - orc.dequant(*orc.quantize(w, 8, ASYM), 8, ASYM)).mean()
        assert e3 > 10 * e8
        # per-row symmetric scheme: S = max|w| / 127 (Sec. 4.2), codes in [-127, 127]
        codes, s, z = orc.quantize(w, 8, SYM)
        assert z is None and codes.min() >= -127 and codes.max() <= 127
        sf = as_f16(s).astype(np.float64)
        amax = np.abs(wf).max(axis=1)
        assert np.all(np.abs(sf - amax / 127) <= np.spacing(as_f16(s)).astype(np.float64) / 2 * (1 + 2.0 ** -12))
        d = orc.dequant(codes, s, None, 8, SYM).astype(np.float64)
        assert np.all(np.abs(wf - d) <= sf[:, None] / 2 * (1 + 2.0 ** -9))
        assert np.all(np.abs(codes[np.arange(N), np.abs(wf).argmax(axis=1)]) == 127)
        c2, s2, _ = orc.quantize((-w).astype(np.float16), 8, SYM)
        assert np.array_equal(c2, -codes) and np.array_equal(s2, s)


def pin_degenerate_groups(orc):
    """Flat groups (max == min): scale 1, codes 0, dequant exact; -0 and +0 give zero +0."""
    w = np.zeros((64, 384), np.float16)
    w[:, 128:256] = np.float16(0.37)
    w[:, 256:] = np.float16(-0.0)
    w[3, 256] = np.float16(0.0)
    for bits in ASYM_BITS:
        codes, s, z = orc.quantize(w, bits, ASYM)
        assert np.all(codes == 0) and np.all(s == 0x3C00)
        assert np.all(z[:, 0] == 0) and np.all(as_f16(z)[:, 1] == np.float16(0.37)) and np.all(z[:, 2] == 0)
        d = orc.dequant(codes, s, z, bits, ASYM)
        assert np.array_equal(d, w.astype(np.float32))
    codes, s, _ = orc.quantize(np.zeros((64, 128), np.float16), 8, SYM)
    assert np.all(codes == 0) and np.all(s == 0x3C00)
    # tiny range whose scale underflows fp16 entirely -> treated as flat
    w = np.zeros((64, 128), np.float16)
    w[:, 5] = np.float16(2.0 ** -24)
    codes, s, z = orc.quantize(w, 8, ASYM)          # 2^-24/255 rounds to 0 in fp16
    assert np.all(s == 0x3C00) and np.all(codes == 0)
    # range so small that the fp16 scale is a subnormal rounded down: (w - zero) / scale
    # overshoots 2^b - 1 and the code must be clamped to the top of the range
    w = np.zeros((64, 128), np.float16)
    w[:, 9] = as_f16(np.uint16(9))                  # 9 * 2^-24
    codes, s, z = orc.quantize(w, 3, ASYM)          # 9/7 * 2^-24 -> fp16 subnormal 1 * 2^-24
    assert np.all(s == 1) and np.all(codes[:, 9] == 7) and codes.max() == 7 and codes.min() == 0


def pin_scale_invariance(orc):
    """P8: multiplying the weights by 2^k leaves the codes unchanged and multiplies scale
    and zero by 2^k exactly (all formulas are homogeneous; rounding is scale-free)."""
    w = synth_w(64, 256, 41, outliers=False)
    for bits, scheme in ((3, ASYM), (4, ASYM), (8, ASYM), (8, SYM)):
        c0, s0, z0 = orc.quantize(w, bits, scheme)
        for k in (1, 3, 5, 9):
            wk = (w.astype(np.float32) * np.float32(2.0 ** k)).astype(np.float16)
            assert np.array_equal(wk.astype(np.float64), w.astype(np.float64) * 2.0 ** k)
            c, s, z = orc.quantize(wk, bits, scheme)
            assert np.array_equal(c, c0)
            assert np.array_equal(as_f16(s).astype(np.float64), as_f16(s0).astype(np.float64) * 2.0 ** k)
            if z is not None:
                assert np.array_equal(as_f16(z).astype(np.float64), as_f16(z0).astype(np.float64) * 2.0 ** k)


def pin_groups_and_rows_are_independent(orc):
    """Granularity: one (row, 128-column) group for the grouped scheme, one row for the per-row
    scheme.  Changing one group / row must not change any other group's / row's result."""
    w = synth_w(128, 384, 51)
    for bits in ASYM_BITS:
        c0, s0, z0 = orc.quantize(w, bits, ASYM)
        w2 = w.copy()
        w2[7, 128:256] = (w2[7, 128:256].astype(np.float32) * 3 + 0.1).astype(np.float16)
        c, s, z = orc.quantize(w2, bits, ASYM)
        keep = np.ones((128, 384), bool)
        keep[7, 128:256] = False
        assert np.array_equal(c[keep], c0[keep])
        gk = np.ones((128, 3), bool)
        gk[7, 1] = False
        assert np.array_equal(s[gk], s0[gk]) and np.array_equal(z[gk], z0[gk])
        assert not np.array_equal(s[7, 1], s0[7, 1])
        # shifting the group boundary matters: the statistics really are per 128 columns
        sub = orc.quantize(np.ascontiguousarray(w[:64, 128:256]), bits, ASYM)
        assert np.array_equal(sub[0], c0[:64, 128:256]) and np.array_equal(sub[1][:, 0], s0[:64, 1])
    c0, s0, _ = orc.quantize(w, 8, SYM)
    w2 = w.copy()
    w2[9] = (w2[9].astype(np.float32) * 2.5).astype(np.float16)
    c, s, _ = orc.quantize(w2, 8, SYM)
    keep = np.arange(128) != 9
    assert np.array_equal(c[keep], c0[keep]) and np.array_equal(s[keep], s0[keep]) and s[9] != s0[9]


# ---------------------------------------------------------------------------------------
# P4: the 16-bit path is a plain matmul (numpy's float64 matmul is the library routine)
# ---------------------------------------------------------------------------------------

def pin_fp16_path_is_plain_matmul(orc):
    rng = np.random.default_rng(61)
    for (M, K, N) in ((1, 128, 64), (5, 256, 192), (17, 384, 128)):
        w = synth_w(N, K, 62 + M)
        x = rng.standard_normal((M, K)).astype(np.float16)
        want = x.astype(np.float64) @ w.astype(np.float64).T
        got = orc.qlinear(x, w, 16, FP16)
        assert got.shape == (M, N)
        assert np.allclose(got, want, rtol=1e-12, atol=1e-12)
        p, s, z = orc.quantize_pack(w, 16, FP16)
        assert s is None and z is None and np.array_equal(orc.unpack_fp16(p, K, N), w.view(np.uint16))
        bias = rng.standard_normal(N).astype(np.float16)
        gotb = orc.matmul(x, orc.fp16_to_f32(w), bias)
        assert np.allclose(gotb, want + bias.astype(np.float64)[None, :], rtol=1e-12, atol=1e-12)
    # a non-symmetric probe that a transposed operand or swapped index cannot survive
    M, K, N = 3, 128, 64
    x = np.zeros((M, K), np.float16)
    w = np.zeros((N, K), np.float16)
    x[2, 5] = 2.0
    w[11, 5] = 3.0
    y = orc.qlinear(x, w, 16, FP16)
    assert y[2, 11] == 6.0 and np.count_nonzero(y) == 1


# ---------------------------------------------------------------------------------------
# P6: brute force on tiny shapes, reading the code bits straight from the packed words
# ---------------------------------------------------------------------------------------

def pin_brute_force_tiny(orc):
    rng = np.random.default_rng(71)
    for (M, K, N) in ((1, 128, 64), (3, 256, 64), (5, 128, 128)):
        w = synth_w(N, K, 72 + M + K)
        x = rng.standard_normal((M, K)).astype(np.float16)
        for bits, scheme in ((3, ASYM), (4, ASYM), (8, ASYM), (8, SYM)):
            packed, s, z = orc.quantize_pack(w, bits, scheme)
            y = orc.qlinear(x, w, bits, scheme)
            sf = as_f16(s).astype(np.longdouble)
            zf = None if z is None else as_f16(z).astype(np.longdouble)
            want = np.zeros((M, N), np.longdouble)
            for n in range(N):
                wt = np.zeros(K, np.longdouble)
                for k in range(K):
                    c = spec_unpack_one(packed, bits, K, n, k, signed=(scheme == SYM))
                    if scheme == ASYM:
                        g = k // 128          # stored order of scales and zeros: g * N + n
                        wt[k] = sf.reshape(-1)[g * N + n] * c + zf.reshape(-1)[g * N + n]
                    else:
                        wt[k] = sf[n] * c
                for m in range(M):
                    want[m, n] = np.sum(x[m].astype(np.longdouble) * wt)
            # the oracle rounds s*c+z to fp32 once (2^-24 relative) before the fp64 sum
            tol = 2.0 ** -22 * np.abs(x.astype(np.float64)) @ np.abs(orc.dequant_weights(w, bits, scheme).astype(np.float64)).T
            assert np.all(np.abs(y - want.astype(np.float64)) <= tol + 1e-300)


# ---------------------------------------------------------------------------------------
# P5: deterministic output-error bound that follows from App. A.1
# ---------------------------------------------------------------------------------------

def pin_output_error_bound(orc):
    rng = np.random.default_rng(81)
    M, K, N = 4, 512, 64
    w = synth_w(N, K, 82)
    x = rng.standard_normal((M, K)).astype(np.float16)
    x[:, [3, 200]] *= np.float16(30)
    y_fp = x.astype(np.float64) @ w.astype(np.float64).T
    prev = None
    for bits in (8, 4, 3):
        codes, s, z = orc.quantize(w, bits, ASYM)
        y = orc.qlinear(x, w, bits, ASYM)
        half = np.repeat(as_f16(s).astype(np.float64), 128, axis=1) / 2 * (1 + 2.0 ** -9)
        bound = np.abs(x.astype(np.float64)) @ half.T
        err = np.abs(y - y_fp)
        assert np.all(err <= bound)
        assert err.max() > 0                      # quantisation really changed the result
        if prev is not None:
            assert np.linalg.norm(err) > prev     # fewer bits, larger error
        prev = np.linalg.norm(err)
    codes, s, _ = orc.quantize(w, 8, SYM)
    y = orc.qlinear(x, w, 8, SYM)
    bound = np.abs(x.astype(np.float64)).sum(axis=1)[:, None] * (as_f16(s).astype(np.float64)[None, :] / 2 * (1 + 2.0 ** -9))
    assert np.all(np.abs(y - y_fp) <= bound)


def pin_matmul_linearity_and_freivalds(orc):
    """O5 by properties: linear in x, and the random-projection identity
    sum_n y[m,n] r[n] == x[m,:] . (W~^T r) computed with numpy in float64 (P9)."""
    rng = np.random.default_rng(91)
    M, K, N = 6, 384, 64
    w = synth_w(N, K, 92)
    x = rng.standard_normal((M, K)).astype(np.float16)
    for bits, scheme in ((4, ASYM), (3, ASYM), (8, SYM)):
        wd = orc.dequant_weights(w, bits, scheme).astype(np.float64)
        y = orc.qlinear(x, w, bits, scheme)
        r = rng.choice([-1.0, 1.0], N)
        assert np.allclose(y @ r, x.astype(np.float64) @ (wd.T @ r), rtol=1e-11, atol=1e-11)
        x2 = (x.astype(np.float32) * 2).astype(np.float16)
        assert np.allclose(orc.qlinear(x2, w, bits, scheme), 2 * y, rtol=1e-13, atol=0)


ALL_PINS = [
    pin_fp16_conversions,
    pin_pack_density_and_roundtrip,
    pin_pack_matches_format_description,
    pin_exact_grid_examples,
    pin_rtn_against_exact_arithmetic,
    pin_error_bound_half_scale,
    pin_degenerate_groups,
    pin_scale_invariance,
    pin_groups_and_rows_are_independent,
    pin_fp16_path_is_plain_matmul,
    pin_brute_force_tiny,
    pin_output_error_bound,
    pin_matmul_linearity_and_freivalds,
]
