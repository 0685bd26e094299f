"""CPU oracle for the mixed-precision quantized-linear path (ctypes view of lpq_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by the
cpu_baseline leg of bench.py.  The product (the HIP library and its binding) never imports
this package, and this package imports nothing from the product.

Every function works on numpy arrays on the host.  fp16 data travels as uint16 bit patterns
(``arr.view(np.uint16)``) so that no conversion happens outside lpq_oracle.c.

Steps follow LLM-PQ (arXiv 2403.01136): Sec. 2.4 (quantise / dequantise formulas),
Sec. 4.2 (asymmetric and symmetric scaling factors), Sec. 4.1 (bit/8 bytes per weight),
App. A.1 (rounding error bound).
"""
import ctypes
import os
import subprocess

import numpy as np

FP16, ASYM_GROUP, SYM_CHANNEL = 0, 1, 2
GROUP = 128
BLOCK_ROWS = 64

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lpq_oracle.c")
_LIB = os.path.join(_HERE, "liblpq_oracle.so")


def build(force=False):
    """Compile lpq_oracle.c with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-fPIC",
             "-shared", "-Wno-unknown-pragmas", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a, shape=None):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


class Oracle:
    """All oracle entry points bound to one compiled copy of lpq_oracle.c.

    The module-level functions below use the default build; tests that plant a mistake in a
    copy of the C source (to show that the pins catch it) load that copy through
    ``Oracle(path_to_so)``.
    """

    FP16, ASYM_GROUP, SYM_CHANNEL = FP16, ASYM_GROUP, SYM_CHANNEL
    GROUP, BLOCK_ROWS = GROUP, BLOCK_ROWS

    def __init__(self, libpath=None):
        if libpath is None:
            libpath = build()
        L = ctypes.CDLL(libpath)
        vp, i, l = ctypes.c_void_p, ctypes.c_int, ctypes.c_long
        L.lpq_oracle_h2f.restype = ctypes.c_float
        L.lpq_oracle_h2f.argtypes = [ctypes.c_uint16]
        L.lpq_oracle_f2h.restype = ctypes.c_uint16
        L.lpq_oracle_f2h.argtypes = [ctypes.c_float]
        L.lpq_oracle_packed_sizes.argtypes = [i, i, l, l, vp, vp, vp]
        L.lpq_oracle_quantize.argtypes = [vp, i, i, l, l, vp, vp, vp]
        L.lpq_oracle_pack.argtypes = [vp, i, i, l, l, vp]
        L.lpq_oracle_unpack.argtypes = [vp, i, i, l, l, vp]
        L.lpq_oracle_store_scales.argtypes = [vp, l, l, vp]
        L.lpq_oracle_pack_fp16.argtypes = [vp, l, l, vp]
        L.lpq_oracle_unpack_fp16.argtypes = [vp, l, l, vp]
        L.lpq_oracle_dequant.argtypes = [vp, vp, vp, i, i, l, l, vp]
        L.lpq_oracle_fp16_to_f32.argtypes = [vp, l, vp]
        L.lpq_oracle_matmul.argtypes = [vp, vp, l, l, l, vp, vp]
        self._L = L

    def h2f(self, bits):
        return float(self._L.lpq_oracle_h2f(int(bits)))

    def f2h(self, value):
        return int(self._L.lpq_oracle_f2h(float(value)))

    def packed_sizes(self, bits, scheme, K, N):
        c, s, z = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
        rc = self._L.lpq_oracle_packed_sizes(bits, scheme, K, N, ctypes.byref(c), ctypes.byref(s), ctypes.byref(z))
        if rc:
            raise ValueError("bad descriptor bits=%r scheme=%r K=%r N=%r" % (bits, scheme, K, N))
        return c.value, s.value, z.value

    def quantize(self, w, bits, scheme):
        """O1-O3 (first half).  w: [N][K] fp16 (or its uint16 view).
        Returns codes int32 [N][K], scales uint16, zeros uint16 (None for the per-row scheme)."""
        w = _u16(w)
        N, K = w.shape
        G = K // GROUP
        codes = np.empty((N, K), np.int32)
        if scheme == ASYM_GROUP:
            scales, zeros = np.empty((N, G), np.uint16), np.empty((N, G), np.uint16)
        else:
            scales, zeros = np.empty((N,), np.uint16), None
        rc = self._L.lpq_oracle_quantize(_ptr(w), bits, scheme, K, N, _ptr(codes), _ptr(scales), _ptr(zeros))
        if rc:
            raise ValueError("lpq_oracle_quantize rc=%d" % rc)
        return codes, scales, zeros

    def pack(self, codes, bits, scheme):
        """O3 (second half).  codes int32 [N][K] -> packed bytes uint8 [K*N*bits/8]."""
        codes = np.ascontiguousarray(codes, np.int32)
        N, K = codes.shape
        nbytes, _, _ = self.packed_sizes(bits, scheme, K, N)
        out = np.empty((nbytes,), np.uint8)
        rc = self._L.lpq_oracle_pack(_ptr(codes), bits, scheme, K, N, _ptr(out))
        if rc:
            raise ValueError("lpq_oracle_pack rc=%d" % rc)
        return out

    def unpack(self, packed, bits, scheme, K, N):
        packed = np.ascontiguousarray(packed, np.uint8)
        assert packed.size == self.packed_sizes(bits, scheme, K, N)[0]
        codes = np.empty((N, K), np.int32)
        rc = self._L.lpq_oracle_unpack(_ptr(packed), bits, scheme, K, N, _ptr(codes))
        if rc:
            raise ValueError("lpq_oracle_unpack rc=%d" % rc)
        return codes

    def dequant(self, codes, scales, zeros, bits, scheme):
        """O4.  Returns float32 [N][K] = scale * code + zero (fp32 multiply, then fp32 add)."""
        codes = np.ascontiguousarray(codes, np.int32)
        N, K = codes.shape
        scales = _u16(scales)
        zeros = None if zeros is None else _u16(zeros)
        out = np.empty((N, K), np.float32)
        rc = self._L.lpq_oracle_dequant(_ptr(codes), _ptr(scales), _ptr(zeros), bits, scheme, K, N, _ptr(out))
        if rc:
            raise ValueError("lpq_oracle_dequant rc=%d" % rc)
        return out

    def fp16_to_f32(self, w):
        w = _u16(w)
        out = np.empty(w.shape, np.float32)
        self._L.lpq_oracle_fp16_to_f32(_ptr(w), w.size, _ptr(out))
        return out

    def matmul(self, x, w_deq, bias=None):
        """O5.  x: [M][K] fp16, w_deq: [N][K] float32 -> y float64 [M][N], accumulated in fp64."""
        x = _u16(x)
        w_deq = np.ascontiguousarray(w_deq, np.float32)
        M, K = x.shape
        N, K2 = w_deq.shape
        assert K == K2
        bias = None if bias is None else _u16(bias, (N,))
        y = np.empty((M, N), np.float64)
        rc = self._L.lpq_oracle_matmul(_ptr(x), _ptr(w_deq), M, K, N, _ptr(bias), _ptr(y))
        if rc:
            raise ValueError("lpq_oracle_matmul rc=%d" % rc)
        return y

    def store_scales(self, natural, K):
        """Scales or zeros in natural [N][K/128] order -> the stored [K/128][N] order."""
        natural = _u16(natural)
        N, G = natural.shape
        assert G == K // GROUP
        out = np.empty((G, N), np.uint16)
        rc = self._L.lpq_oracle_store_scales(_ptr(natural), K, N, _ptr(out))
        if rc:
            raise ValueError("lpq_oracle_store_scales rc=%d" % rc)
        return out

    def pack_fp16(self, w):
        """16-bit layers: fp16 [N][K] -> the same values in stored (tile) order, as bytes."""
        w = _u16(w)
        N, K = w.shape
        out = np.empty((N * K * 2,), np.uint8)
        rc = self._L.lpq_oracle_pack_fp16(_ptr(w), K, N, _ptr(out))
        if rc:
            raise ValueError("lpq_oracle_pack_fp16 rc=%d" % rc)
        return out

    def unpack_fp16(self, packed, K, N):
        packed = np.ascontiguousarray(packed, np.uint8)
        assert packed.size == N * K * 2
        out = np.empty((N, K), np.uint16)
        rc = self._L.lpq_oracle_unpack_fp16(_ptr(packed), K, N, _ptr(out))
        if rc:
            raise ValueError("lpq_oracle_unpack_fp16 rc=%d" % rc)
        return out

    def quantize_pack(self, w, bits, scheme):
        """O1-O3 in one call, everything in stored order: (packed uint8, scales uint16 | None,
        zeros uint16 | None); grouped scales and zeros are [K/128][N], per-row scales [N]."""
        w = _u16(w)
        if scheme == FP16:
            return self.pack_fp16(w), None, None
        codes, scales, zeros = self.quantize(w, bits, scheme)
        if scheme == ASYM_GROUP:
            K = w.shape[1]
            scales, zeros = self.store_scales(scales, K), self.store_scales(zeros, K)
        return self.pack(codes, bits, scheme), scales, zeros

    def dequant_weights(self, w, bits, scheme):
        """O1-O4: the fp32 weights the quantised layer really multiplies by."""
        w = _u16(w)
        if scheme == FP16:
            return self.fp16_to_f32(w)
        codes, scales, zeros = self.quantize(w, bits, scheme)
        return self.dequant(codes, scales, zeros, bits, scheme)

    def qlinear(self, x, w, bits, scheme, bias=None):
        """O1-O5: reference output (float64 [M][N]) of one quantised linear."""
        return self.matmul(x, self.dequant_weights(w, bits, scheme), bias)


_default = None


def default():
    global _default
    if _default is None:
        _default = Oracle()
    return _default


def _forward(name):
    def f(*a, **k):
        return getattr(default(), name)(*a, **k)
    f.__name__ = name
    f.__doc__ = getattr(Oracle, name).__doc__
    return f


h2f = _forward('h2f')
f2h = _forward('f2h')
packed_sizes = _forward('packed_sizes')
quantize = _forward('quantize')
pack = _forward('pack')
unpack = _forward('unpack')
store_scales = _forward('store_scales')
pack_fp16 = _forward('pack_fp16')
unpack_fp16 = _forward('unpack_fp16')
dequant = _forward('dequant')
fp16_to_f32 = _forward('fp16_to_f32')
matmul = _forward('matmul')
quantize_pack = _forward('quantize_pack')
dequant_weights = _forward('dequant_weights')
qlinear = _forward('qlinear')
