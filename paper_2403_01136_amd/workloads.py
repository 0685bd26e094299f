"""Seeded synthetic inputs and the five benchmark configurations.

This module holds no arithmetic of the method (no quantiser, no packing, no matmul): it only
draws random fp16 weights and activations and names shapes.  It is the one piece of code that
the CPU oracle's tests and the HIP path's tests both use, so that both sides see the same
bytes.

Recipe (stand-in for the OPT / BLOOM linears the paper serves; the trained weights are not
used): weights fp16, i.i.d. N(0, 0.02^2), then an independent 0.1 % of entries multiplied by
20; activations fp16, i.i.d. N(0, 1), and for every configuration but the first, 6 seeded
input channels multiplied by 30.  Layout: W [N][K] (K contiguous), x [M][K].
"""
import zlib

import numpy as np

BASE_SEED = 20240301
FP16, ASYM_GROUP, SYM_CHANNEL = 0, 1, 2
LINEARS = ("qkv", "out", "fc1", "fc2")


def _cfg(name, h, f, layers, prefill_M, decode_Ms, act_outliers, qkv_n=None):
    return dict(name=name, h=h, f=f, qkv_n=qkv_n or 3 * h, layers=layers, prefill_M=prefill_M,
                decode_Ms=decode_Ms, act_outliers=act_outliers)


def _g(bits):
    return (16, FP16) if bits == 16 else (bits, ASYM_GROUP)


CONFIGS = [
    _cfg("opt125m_layer_w4", 768, 3072, [_g(4)], 128, [1], False),
    _cfg("opt13b_stage8_mixed", 5120, 20480, [_g(b) for b in (16, 8, 4, 4, 3, 3, 4, 8)], 2048, [16], True),
    _cfg("opt30b_stage12_w3w4", 7168, 28672, [_g(b) for b in (3, 4) * 6], 1024, [1, 8, 32], True),
    _cfg("opt66b_stage10_i8w4", 9216, 36864, [(8, SYM_CHANNEL)] * 5 + [_g(4)] * 5, 4096, [24], True),
    _cfg("bloom176b_share10_w3", 14336, 57344, [_g(3)] * 10, 2048, [1, 4, 16, 64], True, qkv_n=43008),
]


def linear_shapes(cfg):
    """name -> (K, N) of the four linears of one decoder layer."""
    h, f = cfg["h"], cfg["f"]
    return {"qkv": (h, cfg["qkv_n"]), "out": (h, h), "fc1": (h, f), "fc2": (f, h)}


def packed_bytes(bits, scheme, K, N):
    """Bytes of codes + scales + zeros of one linear (the numerator of the decode metric)."""
    code = K * N * bits // 8
    if scheme == ASYM_GROUP:
        return code + 2 * (N * (K // 128) * 2)
    if scheme == SYM_CHANNEL:
        return code + N * 2
    return code


def stage_packed_bytes(cfg):
    return sum(packed_bytes(b, s, K, N) for (b, s) in cfg["layers"] for (K, N) in linear_shapes(cfg).values())


def stage_flops(cfg, M):
    return sum(2 * M * K * N for _ in cfg["layers"] for (K, N) in linear_shapes(cfg).values())


def stream_seed(*key):
    """A 63-bit seed from the base seed and a key such as (config, layer, linear, kind)."""
    text = repr((BASE_SEED,) + tuple(key)).encode()
    return ((zlib.crc32(text) << 31) ^ zlib.adler32(text[::-1]) ^ (BASE_SEED << 7)) & ((1 << 63) - 1)


# ---- host (numpy) generators: small cases, same bytes for oracle and GPU ---------------


def weight_np(N, K, *key):
    rng = np.random.default_rng(stream_seed("w", *key))
    w = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.02)
    mask = rng.random((N, K), dtype=np.float32) < np.float32(0.001)
    w[mask] *= np.float32(20.0)
    return w.astype(np.float16)


def act_np(M, K, outliers, *key):
    rng = np.random.default_rng(stream_seed("x", *key))
    x = rng.standard_normal((M, K), dtype=np.float32)
    if outliers:
        ch = rng.choice(K, size=min(6, K), replace=False)
        x[:, ch] *= np.float32(30.0)
    return x.astype(np.float16)


# ---- device (torch) generators: full-size cases, drawn where they are used -------------


def weight_torch(N, K, device, *key):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(stream_seed("w", *key))
    w = torch.randn((N, K), generator=g, device=device, dtype=torch.float32) * 0.02
    mask = torch.rand((N, K), generator=g, device=device, dtype=torch.float32) < 0.001
    w = torch.where(mask, w * 20.0, w)
    return w.to(torch.float16)


def act_torch(M, K, outliers, device, *key):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(stream_seed("x", *key))
    x = torch.randn((M, K), generator=g, device=device, dtype=torch.float32)
    if outliers:
        ch = torch.randperm(K, generator=g, device=device)[:6]
        x[:, ch] *= 30.0
    return x.to(torch.float16)
