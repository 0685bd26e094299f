"""MI355X-native mixed-precision quantized linears (the hot path of LLM-PQ, arXiv 2403.01136).

Thin Python binding of the C-ABI library declared in include/lpq.h: argument marshalling only.
Every step of the path (quantise, pack, decode and prefill linears, stage dispatch) runs in the
HIP kernels of liblpq.so; torch is used to allocate device memory and to name the stream.
There is no CPU fallback: if the library is missing, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblpq.so")

LPQ_FP16, LPQ_ASYM_GROUP, LPQ_SYM_CHANNEL = 0, 1, 2
LPQ_PREFILL, LPQ_DECODE = 0, 1
LPQ_OK = 0
LINEARS = ("qkv", "out", "fc1", "fc2")
EXPORTS = ("lpq_packed_sizes", "lpq_quantize_pack", "lpq_quantize_pack_rows", "lpq_load_quantize_pack",
           "lpq_qlinear_prefill", "lpq_qlinear_decode", "lpq_qlinear_fused", "lpq_stage_linears", "lpq_stage_linears_noalloc", "lpq_layernorm",
           "lpq_kv_append", "lpq_attention", "lpq_decoder_layer_workspace", "lpq_decoder_layer", "lpq_variance_indicator",
           "lpq_mem_embedding_bytes", "lpq_mem_layer_bytes", "lpq_mem_kv_bytes", "lpq_latency_fit", "lpq_latency_predict",
           "lpq_plan_objective", "lpq_plan_adabits", "lpq_plan_bitwidth_transfer",
           "lpq_workspace_policy", "lpq_workspace_reserve", "lpq_workspace_bytes", "lpq_set_decode_routing",
           "lpq_unpack_dequant",
           "lpq_status_str")
LPQ_ACT_NONE, LPQ_ACT_RELU, LPQ_ACT_GELU_TANH = 0, 1, 2


class lpq_qdesc(ctypes.Structure):
    _fields_ = [("bits", ctypes.c_int32), ("scheme", ctypes.c_int32), ("group_size", ctypes.c_int32),
                ("K", ctypes.c_int32), ("N", ctypes.c_int32)]


class lpq_qweight(ctypes.Structure):
    _fields_ = [("d", lpq_qdesc), ("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p),
                ("zeros", ctypes.c_void_p), ("bias", ctypes.c_void_p)]


class lpq_layer(ctypes.Structure):
    _fields_ = [(n, lpq_qweight) for n in LINEARS]


class lpq_layer_io(ctypes.Structure):
    _fields_ = [("x_" + n, ctypes.c_void_p) for n in LINEARS] + [("y_" + n, ctypes.c_void_p) for n in LINEARS]


class lpq_epilogue(ctypes.Structure):
    _fields_ = [("activation", ctypes.c_int32), ("residual", ctypes.c_void_p)]


class lpq_layer_cfg(ctypes.Structure):
    _fields_ = [("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("max_seq", ctypes.c_int32),
                ("activation", ctypes.c_int32), ("ln_eps", ctypes.c_float)]


class lpq_layer_state(ctypes.Structure):
    _fields_ = [("ln1_gamma", ctypes.c_void_p), ("ln1_beta", ctypes.c_void_p), ("ln2_gamma", ctypes.c_void_p),
                ("ln2_beta", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("vt_cache", ctypes.c_void_p),
                ("alibi_slopes", ctypes.c_void_p)]


class lpq_model_shape(ctypes.Structure):
    _fields_ = [("h1", ctypes.c_int64), ("h2", ctypes.c_int64), ("vocab", ctypes.c_int64), ("d_t", ctypes.c_int64),
                ("pos", ctypes.c_int64), ("rmsnorm", ctypes.c_int32), ("pad", ctypes.c_int32)]


_dp, _ip = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)


class lpq_plan_problem(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int32), ("N", ctypes.c_int32), ("n_bits", ctypes.c_int32), ("pad", ctypes.c_int32),
                ("bits", _ip), ("omega", _dp), ("lat_pre", _dp), ("lat_dec", _dp), ("mem", _dp), ("cap", _dp),
                ("comm_pre", _dp), ("comm_dec", _dp), ("emb", ctypes.c_double), ("theta", ctypes.c_double),
                ("B", ctypes.c_int32), ("eta", ctypes.c_int32), ("xi", ctypes.c_int32), ("n", ctypes.c_int32)]


class LpqError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        RuntimeError.__init__(self, "%s failed: status %d (%s)" % (where, status, status_str(status)))


_lib = None


def load_library():
    """Load liblpq.so (after torch, so both share one HIP runtime).  Raises if it is not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("%s is not built; run `python -m paper_2403_01136_amd.build` "
                               "(there is no fallback path)" % LIB_PATH)
        import torch  # noqa: F401  (loads the HIP runtime this library must share)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, szp = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_size_t)
        L.lpq_packed_sizes.argtypes = [ctypes.POINTER(lpq_qdesc), szp, szp, szp]
        L.lpq_quantize_pack.argtypes = [vp, ctypes.POINTER(lpq_qdesc), ctypes.POINTER(lpq_qweight), vp]
        L.lpq_quantize_pack_rows.argtypes = [vp, ctypes.POINTER(lpq_qdesc), i32, i32, ctypes.POINTER(lpq_qweight), vp]
        L.lpq_load_quantize_pack.argtypes = [vp, ctypes.POINTER(lpq_qdesc), ctypes.POINTER(lpq_qweight), vp, ctypes.c_size_t, vp]
        L.lpq_qlinear_prefill.argtypes = [ctypes.POINTER(lpq_qweight), vp, i32, vp, vp]
        L.lpq_qlinear_decode.argtypes = [ctypes.POINTER(lpq_qweight), vp, i32, vp, vp]
        L.lpq_stage_linears.argtypes = [ctypes.POINTER(lpq_layer), i32, ctypes.c_int, i32, ctypes.POINTER(lpq_layer_io), vp]
        L.lpq_stage_linears_noalloc.argtypes = [ctypes.POINTER(lpq_layer), i32, ctypes.c_int, i32, ctypes.POINTER(lpq_layer_io), vp]
        L.lpq_qlinear_fused.argtypes = [ctypes.POINTER(lpq_qweight), vp, i32, vp, ctypes.POINTER(lpq_epilogue), ctypes.c_int, vp]
        L.lpq_variance_indicator.argtypes = [vp, i32, i32, vp, i32, i32, vp, vp]
        L.lpq_layernorm.argtypes = [vp, vp, vp, ctypes.c_float, i32, i32, vp, vp]
        cfgp, stp = ctypes.POINTER(lpq_layer_cfg), ctypes.POINTER(lpq_layer_state)
        L.lpq_kv_append.argtypes = [vp, cfgp, stp, i32, i32, i32, vp]
        L.lpq_attention.argtypes = [vp, cfgp, stp, i32, i32, i32, vp, vp]
        L.lpq_decoder_layer_workspace.argtypes = [ctypes.POINTER(lpq_layer), cfgp, i32]
        L.lpq_decoder_layer.argtypes = [ctypes.POINTER(lpq_layer), cfgp, stp, ctypes.c_int, i32, i32, i32, vp, vp, vp, ctypes.c_size_t, vp]
        L.lpq_unpack_dequant.argtypes = [ctypes.POINTER(lpq_qweight), vp, vp]
        shp, pp, i64 = ctypes.POINTER(lpq_model_shape), ctypes.POINTER(lpq_plan_problem), ctypes.c_int64
        L.lpq_mem_embedding_bytes.argtypes = [shp]
        L.lpq_mem_layer_bytes.argtypes = [shp, i32]
        L.lpq_mem_kv_bytes.argtypes = [shp, i64, i64, i64, i32]
        L.lpq_latency_fit.argtypes = [ctypes.c_int, i32, _dp, _dp, _dp, _dp]
        L.lpq_latency_predict.argtypes = [ctypes.c_int, _dp, i32, _dp, _dp, _dp]
        L.lpq_plan_objective.argtypes = [pp, _ip, _ip, i32, _dp]
        L.lpq_plan_adabits.argtypes = [pp, _ip, _ip, _dp]
        L.lpq_plan_bitwidth_transfer.argtypes = [pp, _ip, _ip, _dp, _ip]
        L.lpq_workspace_policy.argtypes = [ctypes.c_size_t, i32, ctypes.c_size_t, szp]
        L.lpq_workspace_reserve.argtypes = [ctypes.c_size_t]
        L.lpq_workspace_bytes.argtypes = []
        L.lpq_set_decode_routing.argtypes = [i32, i32]
        L.lpq_status_str.argtypes = [ctypes.c_int]
        L.lpq_status_str.restype = ctypes.c_char_p
        other = {"lpq_decoder_layer_workspace": ctypes.c_size_t, "lpq_workspace_bytes": ctypes.c_size_t, "lpq_mem_embedding_bytes": ctypes.c_double,
                 "lpq_mem_layer_bytes": ctypes.c_double, "lpq_mem_kv_bytes": ctypes.c_double}
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = other.get(name, ctypes.c_int)
        _lib = L
    return _lib


def status_str(status):
    return load_library().lpq_status_str(int(status)).decode()


def _check(status, where):
    if status != LPQ_OK:
        raise LpqError(status, where)


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_desc(bits, scheme, K, N):
    return lpq_qdesc(bits, scheme, 128 if scheme == LPQ_ASYM_GROUP else 0, K, N)


def lpq_packed_sizes(bits, scheme, K, N):
    """(code_bytes, scale_bytes, zero_bytes) of a weight; host-only."""
    d = make_desc(bits, scheme, K, N)
    c, s, z = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(load_library().lpq_packed_sizes(ctypes.byref(d), ctypes.byref(c), ctypes.byref(s), ctypes.byref(z)), "lpq_packed_sizes")
    return c.value, s.value, z.value


class QWeight:
    """Caller-owned packed buffers of one linear (torch tensors on the GPU) plus the ABI struct."""

    def __init__(self, bits, scheme, K, N, device, bias=None):
        import torch
        self.bits, self.scheme, self.K, self.N = bits, scheme, K, N
        cb, sb, zb = lpq_packed_sizes(bits, scheme, K, N)
        self.codes = torch.empty(cb, dtype=torch.uint8, device=device)
        self.scales = torch.empty(sb // 2, dtype=torch.float16, device=device) if sb else None
        self.zeros = torch.empty(zb // 2, dtype=torch.float16, device=device) if zb else None
        self.bias = bias
        self.nbytes = cb + sb + zb

    def struct(self):
        return lpq_qweight(make_desc(self.bits, self.scheme, self.K, self.N), self.codes.data_ptr(),
                           self.scales.data_ptr() if self.scales is not None else None,
                           self.zeros.data_ptr() if self.zeros is not None else None,
                           self.bias.data_ptr() if self.bias is not None else None)


def _fp16_2d(t, name):
    import torch
    if t.dtype != torch.float16 or t.dim() != 2 or not t.is_contiguous() or not t.is_cuda:
        raise ValueError("%s must be a contiguous 2-D fp16 CUDA tensor" % name)
    return t


def lpq_quantize_pack(w, bits, scheme, bias=None, stream=None):
    """w: fp16 [N][K] on the GPU -> QWeight (quantised and packed by the HIP kernel)."""
    w = _fp16_2d(w, "w")
    N, K = w.shape
    qw = QWeight(bits, scheme, K, N, w.device, bias)
    st, d = qw.struct(), make_desc(bits, scheme, K, N)
    _check(load_library().lpq_quantize_pack(w.data_ptr(), ctypes.byref(d), ctypes.byref(st), _stream(stream)), "lpq_quantize_pack")
    return qw


def lpq_quantize_pack_rows(w_rows, qw, row0, stream=None):
    """Quantise rows [row0, row0 + len(w_rows)) of the weight behind `qw` from w_rows (fp16 [n_rows][K] on the GPU)."""
    w_rows = _fp16_2d(w_rows, "w_rows") if w_rows.shape[0] else w_rows
    st, d = qw.struct(), make_desc(qw.bits, qw.scheme, qw.K, qw.N)
    _check(load_library().lpq_quantize_pack_rows(w_rows.data_ptr() if w_rows.shape[0] else qw.codes.data_ptr(), ctypes.byref(d),
                                                 int(row0), int(w_rows.shape[0]), ctypes.byref(st), _stream(stream)),
           "lpq_quantize_pack_rows")
    return qw


def lpq_load_quantize_pack(w_host, bits, scheme, staging, device=None, bias=None, stream=None):
    """w_host: fp16 [N][K] in HOST memory (pinned for asynchronous copies); staging: uint8 CUDA tensor that
    receives one band of rows at a time -> QWeight, bit-identical to lpq_quantize_pack of the whole weight."""
    import torch
    if w_host.dtype != torch.float16 or w_host.dim() != 2 or not w_host.is_contiguous() or w_host.is_cuda:
        raise ValueError("w_host must be a contiguous 2-D fp16 host tensor")
    if staging.dtype != torch.uint8 or not staging.is_cuda or not staging.is_contiguous():
        raise ValueError("staging must be a contiguous uint8 CUDA tensor")
    N, K = w_host.shape
    qw = QWeight(bits, scheme, K, N, staging.device if device is None else device, bias)
    st, d = qw.struct(), make_desc(bits, scheme, K, N)
    _check(load_library().lpq_load_quantize_pack(w_host.data_ptr(), ctypes.byref(d), ctypes.byref(st), staging.data_ptr(),
                                                 staging.numel(), _stream(stream)), "lpq_load_quantize_pack")
    qw._host_source = w_host          # the copies read it until the stream has caught up
    return qw


def _qlinear(fn_name, qw, x, y, stream):
    import torch
    x = _fp16_2d(x, "x")
    M, K = x.shape
    if K != qw.K:
        raise ValueError("x has %d columns, weight has K=%d" % (K, qw.K))
    if y is None:
        y = torch.empty((M, qw.N), dtype=torch.float16, device=x.device)
    else:
        _fp16_2d(y, "y")
        if tuple(y.shape) != (M, qw.N):
            raise ValueError("y must be [%d][%d]" % (M, qw.N))
    st = qw.struct()
    _check(getattr(load_library(), fn_name)(ctypes.byref(st), x.data_ptr(), M, y.data_ptr(), _stream(stream)), fn_name)
    return y


def lpq_qlinear_prefill(qw, x, y=None, stream=None):
    return _qlinear("lpq_qlinear_prefill", qw, x, y, stream)


def lpq_qlinear_decode(qw, x, y=None, stream=None):
    return _qlinear("lpq_qlinear_decode", qw, x, y, stream)


def lpq_qlinear_fused(qw, x, phase, activation=LPQ_ACT_NONE, residual=None, y=None, stream=None):
    """y = fp16(act(x . w~^T + bias) + residual) with one rounding; residual may be y itself."""
    import torch
    x = _fp16_2d(x, "x")
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, qw.N), dtype=torch.float16, device=x.device)
    if residual is not None and tuple(_fp16_2d(residual, "residual").shape) != (M, qw.N):
        raise ValueError("residual must be [%d][%d]" % (M, qw.N))
    st = qw.struct()
    ep = lpq_epilogue(int(activation), residual.data_ptr() if residual is not None else None)
    _check(load_library().lpq_qlinear_fused(ctypes.byref(st), x.data_ptr(), M, _fp16_2d(y, "y").data_ptr(), ctypes.byref(ep),
                                            int(phase), _stream(stream)), "lpq_qlinear_fused")
    return y


def lpq_layernorm(x, gamma, beta, eps, y=None, stream=None):
    import torch
    x = _fp16_2d(x, "x")
    if y is None:
        y = torch.empty_like(x)
    _check(load_library().lpq_layernorm(x.data_ptr(), gamma.data_ptr(), beta.data_ptr(), float(eps), x.shape[0], x.shape[1],
                                        y.data_ptr(), _stream(stream)), "lpq_layernorm")
    return y


class LayerState:
    """Caller-owned state of one decoder layer: layer-norm parameters, the pre-allocated KV cache
    (k_cache [batch][heads][max_seq][head_dim], vt_cache [batch][heads][head_dim][max_seq]), optional ALiBi slopes."""

    def __init__(self, n_heads, head_dim, max_seq, batch, device, ln1, ln2, activation=LPQ_ACT_RELU, ln_eps=1e-5, alibi_slopes=None):
        import torch
        self.cfg = lpq_layer_cfg(n_heads, head_dim, max_seq, int(activation), float(ln_eps))
        self.ln1, self.ln2, self.alibi = ln1, ln2, alibi_slopes
        self.k_cache = torch.zeros((batch, n_heads, max_seq, head_dim), dtype=torch.float16, device=device)
        self.vt_cache = torch.zeros((batch, n_heads, head_dim, max_seq), dtype=torch.float16, device=device)

    def struct(self):
        return lpq_layer_state(self.ln1[0].data_ptr(), self.ln1[1].data_ptr(), self.ln2[0].data_ptr(), self.ln2[1].data_ptr(),
                               self.k_cache.data_ptr(), self.vt_cache.data_ptr(),
                               self.alibi.data_ptr() if self.alibi is not None else None)


def lpq_kv_append(qkv, state, n_seqs, T, pos0, stream=None):
    st = state.struct()
    _check(load_library().lpq_kv_append(_fp16_2d(qkv, "qkv").data_ptr(), ctypes.byref(state.cfg), ctypes.byref(st), n_seqs, T, pos0,
                                        _stream(stream)), "lpq_kv_append")


def lpq_attention(qkv, state, n_seqs, T, pos0, out=None, stream=None):
    import torch
    qkv = _fp16_2d(qkv, "qkv")
    if out is None:
        out = torch.empty((qkv.shape[0], qkv.shape[1] // 3), dtype=torch.float16, device=qkv.device)
    st = state.struct()
    _check(load_library().lpq_attention(qkv.data_ptr(), ctypes.byref(state.cfg), ctypes.byref(st), n_seqs, T, pos0, out.data_ptr(),
                                        _stream(stream)), "lpq_attention")
    return out


def lpq_decoder_layer(layer, state, phase, n_seqs, T, pos0, x, y=None, workspace=None, stream=None):
    """layer: dict name -> QWeight (qkv, out, fc1, fc2); state: LayerState.  Returns (y, workspace)."""
    import torch
    x = _fp16_2d(x, "x")
    if y is None:
        y = torch.empty_like(x)
    ls = lpq_layer(*[layer[n].struct() for n in LINEARS])
    need = load_library().lpq_decoder_layer_workspace(ctypes.byref(ls), ctypes.byref(state.cfg), x.shape[0])
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    st = state.struct()
    _check(load_library().lpq_decoder_layer(ctypes.byref(ls), ctypes.byref(state.cfg), ctypes.byref(st), int(phase), n_seqs, T, pos0,
                                            x.data_ptr(), y.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "lpq_decoder_layer")
    return y, workspace


def lpq_variance_indicator(w, x, stochastic=False, stream=None):
    """Eight forms of D_W * S_W(b)^2 * G(X) (see include/lpq.h) as a float64 CUDA tensor of 8 values."""
    import torch
    w, x = _fp16_2d(w, "w"), _fp16_2d(x, "x")
    if x.shape[1] != w.shape[1]:
        raise ValueError("x and w must have the same number of columns")
    out = torch.empty(8, dtype=torch.float64, device=w.device)
    _check(load_library().lpq_variance_indicator(w.data_ptr(), w.shape[1], w.shape[0], x.data_ptr(), x.shape[0], int(bool(stochastic)),
                                                 out.data_ptr(), _stream(stream)), "lpq_variance_indicator")
    return out


class Stage:
    """Marshalled arguments of lpq_stage_linears, built once and reused across calls.

    layers: list of dicts name -> QWeight; xs / ys: lists of dicts name -> fp16 tensors
    ([M][K] inputs, [M][N] outputs).  Holds references so the buffers stay alive."""

    def __init__(self, layers, xs, ys):
        self.n = len(layers)
        self.keep = (layers, xs, ys)
        self.M = next(iter(xs[0].values())).shape[0]
        self.layers = (lpq_layer * self.n)()
        self.io = (lpq_layer_io * self.n)()
        for i in range(self.n):
            for name in LINEARS:
                qw, x, y = layers[i][name], _fp16_2d(xs[i][name], "x"), _fp16_2d(ys[i][name], "y")
                if tuple(x.shape) != (self.M, qw.K) or tuple(y.shape) != (self.M, qw.N):
                    raise ValueError("layer %d %s: x/y shapes do not match the weight" % (i, name))
                setattr(self.layers[i], name, qw.struct())
                setattr(self.io[i], "x_" + name, x.data_ptr())
                setattr(self.io[i], "y_" + name, y.data_ptr())


def lpq_stage_linears(stage, phase, stream=None):
    """Run all 4 * n_layers linears of a Stage in the given phase (LPQ_PREFILL / LPQ_DECODE)."""
    _check(load_library().lpq_stage_linears(stage.layers, stage.n, phase, stage.M, stage.io, _stream(stream)), "lpq_stage_linears")


def lpq_stage_linears_noalloc(stage, phase, stream=None):
    """lpq_stage_linears with the partial sums in the library's static scratch array: allocates nothing."""
    _check(load_library().lpq_stage_linears_noalloc(stage.layers, stage.n, phase, stage.M, stage.io, _stream(stream)),
           "lpq_stage_linears_noalloc")


# ---- cost models and planner: host arrays in, host arrays out (numpy only carries the buffers) -------------------

def _shape(h1, h2=1, vocab=1, d_t=None, pos=0, rmsnorm=False):
    return lpq_model_shape(h1, h2, vocab, h1 if d_t is None else d_t, pos, int(bool(rmsnorm)), 0)


def _nonneg(value, where):
    if value < 0:
        raise ValueError("%s: bad argument" % where)
    return value


def lpq_mem_embedding_bytes(vocab, d_t, pos, h1):
    m = _shape(h1, 1, vocab, d_t, pos)
    return _nonneg(load_library().lpq_mem_embedding_bytes(ctypes.byref(m)), "lpq_mem_embedding_bytes")


def lpq_mem_layer_bytes(h1, h2, bit, rmsnorm=False):
    m = _shape(h1, h2, rmsnorm=rmsnorm)
    return _nonneg(load_library().lpq_mem_layer_bytes(ctypes.byref(m), bit), "lpq_mem_layer_bytes")


def lpq_mem_kv_bytes(v, s, n, h1, bit_kv=16):
    m = _shape(h1)
    return _nonneg(load_library().lpq_mem_kv_bytes(ctypes.byref(m), v, s, n, bit_kv), "lpq_mem_kv_bytes")


def _f64(a):
    import numpy as np
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    import numpy as np
    return np.ascontiguousarray(a, dtype=np.int32)


def lpq_latency_fit(phase, v, length, t):
    """Coefficients (5 for LPQ_PREFILL, 4 for LPQ_DECODE) of the layer-latency regression."""
    import numpy as np
    v, length, t = _f64(v).ravel(), _f64(length).ravel(), _f64(t).ravel()
    if not (len(v) == len(length) == len(t)):
        raise ValueError("v, length and t must have one value per sample")
    coef = np.zeros(5 if phase == LPQ_PREFILL else 4)
    _check(load_library().lpq_latency_fit(int(phase), len(t), v.ctypes.data_as(_dp), length.ctypes.data_as(_dp),
                                          t.ctypes.data_as(_dp), coef.ctypes.data_as(_dp)), "lpq_latency_fit")
    return coef


def lpq_latency_predict(phase, coef, v, length):
    import numpy as np
    coef, v, length = _f64(coef).ravel(), _f64(v).ravel(), _f64(length).ravel()
    if len(coef) != (5 if phase == LPQ_PREFILL else 4) or len(v) != len(length):
        raise ValueError("coefficient or sample count does not match the phase")
    out = np.zeros(len(v))
    _check(load_library().lpq_latency_predict(int(phase), coef.ctypes.data_as(_dp), len(v), v.ctypes.data_as(_dp),
                                              length.ctypes.data_as(_dp), out.ctypes.data_as(_dp)), "lpq_latency_predict")
    return out


class PlanProblem:
    """Marshalled lpq_plan_problem; keeps the arrays it points to alive."""

    def __init__(self, bits, omega, lat_pre, lat_dec, mem, cap, emb, B, eta, xi, n, theta, comm_pre=None, comm_dec=None):
        self.bits, self.omega = _i32(bits), _f64(omega)
        self.lat_pre, self.lat_dec, self.mem, self.cap = _f64(lat_pre), _f64(lat_dec), _f64(mem), _f64(cap)
        self.comm_pre = None if comm_pre is None else _f64(comm_pre)
        self.comm_dec = None if comm_dec is None else _f64(comm_dec)
        self.L, self.N, nb = self.omega.shape[0], self.cap.shape[0], self.bits.shape[0]
        if self.omega.shape != (self.L, nb) or self.lat_pre.shape != (self.N, nb) or self.lat_dec.shape != (self.N, nb) \
                or self.mem.shape != (nb,) or any(c is not None and c.shape != (self.N,) for c in (self.comm_pre, self.comm_dec)):
            raise ValueError("array shapes do not match L, N and the number of bitwidths")
        ptr = lambda a: None if a is None else a.ctypes.data_as(_dp)
        self.struct = lpq_plan_problem(self.L, self.N, nb, 0, self.bits.ctypes.data_as(_ip), ptr(self.omega), ptr(self.lat_pre),
                                       ptr(self.lat_dec), ptr(self.mem), ptr(self.cap), ptr(self.comm_pre), ptr(self.comm_dec),
                                       float(emb), float(theta), int(B), int(eta), int(xi), int(n))


def lpq_plan_objective(problem, counts, choice, with_latency=True):
    counts, choice = _i32(counts), _i32(choice)
    if counts.shape != (problem.N,) or choice.shape != (problem.L,):
        raise ValueError("counts needs N entries and choice L entries")
    obj = ctypes.c_double()
    _check(load_library().lpq_plan_objective(ctypes.byref(problem.struct), counts.ctypes.data_as(_ip), choice.ctypes.data_as(_ip),
                                             int(bool(with_latency)), ctypes.byref(obj)), "lpq_plan_objective")
    return obj.value


def lpq_plan_adabits(problem):
    """(objective, counts, choice) of a least-indicator plan that fits the devices; counts is None if none fits."""
    import numpy as np
    counts, choice, obj = np.zeros(problem.N, np.int32), np.zeros(problem.L, np.int32), ctypes.c_double()
    _check(load_library().lpq_plan_adabits(ctypes.byref(problem.struct), counts.ctypes.data_as(_ip), choice.ctypes.data_as(_ip),
                                           ctypes.byref(obj)), "lpq_plan_adabits")
    if obj.value == float("inf"):
        return obj.value, None, None
    return obj.value, counts.tolist(), choice.tolist()


def lpq_plan_bitwidth_transfer(problem, counts, choice):
    """(objective, counts, choice, rounds) after Algorithm 2 from the given plan."""
    counts, choice = _i32(counts).copy(), _i32(choice).copy()
    if counts.shape != (problem.N,) or choice.shape != (problem.L,):
        raise ValueError("counts needs N entries and choice L entries")
    obj, rounds = ctypes.c_double(), ctypes.c_int32()
    _check(load_library().lpq_plan_bitwidth_transfer(ctypes.byref(problem.struct), counts.ctypes.data_as(_ip),
                                                     choice.ctypes.data_as(_ip), ctypes.byref(obj), ctypes.byref(rounds)),
           "lpq_plan_bitwidth_transfer")
    return obj.value, counts.tolist(), choice.tolist(), rounds.value


def lpq_workspace_policy(have_bytes, reserved, need_bytes):
    """Bytes the library would allocate for a request of need_bytes (0 = reuse the block); raises LpqError if a reservation forbids it."""
    alloc = ctypes.c_size_t(0)
    _check(load_library().lpq_workspace_policy(int(have_bytes), int(bool(reserved)), int(need_bytes), ctypes.byref(alloc)), "lpq_workspace_policy")
    return alloc.value


def lpq_workspace_reserve(nbytes):
    _check(load_library().lpq_workspace_reserve(int(nbytes)), "lpq_workspace_reserve")


def lpq_workspace_bytes():
    return int(load_library().lpq_workspace_bytes())


def lpq_set_decode_routing(rows_max_mib=-1, rows_tiles=-1):
    _check(load_library().lpq_set_decode_routing(int(rows_max_mib), int(rows_tiles)), "lpq_set_decode_routing")


def lpq_unpack_dequant(qw, stream=None):
    """Test helper: fp32 [N][K] weights read back from the packed buffers on the GPU."""
    import torch
    out = torch.empty((qw.N, qw.K), dtype=torch.float32, device=qw.codes.device)
    st = qw.struct()
    _check(load_library().lpq_unpack_dequant(ctypes.byref(st), out.data_ptr(), _stream(stream)), "lpq_unpack_dequant")
    return out
