"""Helpers of the GPU parity tests: move seeded inputs to the device, compare with the oracle."""
import numpy as np

REL_L2_TOL = 1e-3          # tolerance of the fp16 outputs against the fp64 oracle
MAX_ABS_FRAC = 1e-2        # max |y - ref| <= 1e-2 * max |ref|

VARIANTS = [(3, 1), (4, 1), (8, 1), (8, 2), (16, 0)]
VARIANT_IDS = ["w3", "w4", "w8", "i8sym", "fp16"]


def to_dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def u16(t):
    """fp16 torch tensor -> numpy uint16 bit patterns on the host."""
    return t.detach().cpu().numpy().view(np.uint16)


def check_packed(qw, orc, w_np):
    """Bit-exact comparison of codes / scales / zeros with the oracle's quantise + pack."""
    p, s, z = orc.quantize_pack(w_np, qw.bits, qw.scheme)
    got = qw.codes.cpu().numpy()
    assert got.size == p.size
    bad = np.flatnonzero(got != p)
    assert bad.size == 0, "packed bytes differ at %s (of %d)" % (bad[:8], p.size)
    if s is not None:
        assert np.array_equal(u16(qw.scales).reshape(s.shape), s), "scales differ"
    if z is not None:
        assert np.array_equal(u16(qw.zeros).reshape(z.shape), z), "zeros differ"


def check_output(y_dev, ref, what=""):
    y = y_dev.detach().cpu().numpy().astype(np.float64)
    assert y.shape == ref.shape, (y.shape, ref.shape)
    assert np.all(np.isfinite(y)), what
    rel = np.linalg.norm(y - ref) / max(np.linalg.norm(ref), 1e-30)
    mx = np.abs(y - ref).max()
    assert rel <= REL_L2_TOL, "%s rel-L2 %.3e" % (what, rel)
    assert mx <= MAX_ABS_FRAC * np.abs(ref).max(), "%s max-abs %.3e vs max|ref| %.3e" % (what, mx, np.abs(ref).max())
    return rel
