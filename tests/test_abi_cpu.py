"""C-ABI checks that need no GPU: the library loads, exports every symbol the header declares,
reports sizes, and rejects bad arguments on the host before any HIP call."""
import ctypes
import os
import re

import pytest

import paper_2403_01136_amd as lpq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "lpq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lpq_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = lpq.load_library()
    names = header_functions()
    assert set(names) == set(lpq.EXPORTS), names
    for name in names:
        assert getattr(lib, name) is not None


def test_packed_sizes_are_dense():
    # Sec. 4.1: bytes = weights * bit / 8; scale and zero are fp16 per (row, 128 columns)
    for bits, scheme in ((3, 1), (4, 1), (8, 1), (8, 2), (16, 0)):
        for K, N in ((128, 64), (5120, 15360), (57344, 14336)):
            c, s, z = lpq.lpq_packed_sizes(bits, scheme, K, N)
            assert c * 8 == K * N * bits
            assert s == (N * (K // 128) * 2 if scheme == 1 else (N * 2 if scheme == 2 else 0))
            assert z == (s if scheme == 1 else 0)


@pytest.mark.parametrize("bits,scheme,K,N,status", [
    (5, 1, 128, 64, 2), (2, 1, 128, 64, 2), (4, 7, 128, 64, 3), (16, 1, 128, 64, 3), (3, 2, 128, 64, 3), (4, 0, 128, 64, 3),
    (4, 1, 100, 64, 4), (4, 1, 128, 16, 4), (4, 1, 128, 96, 4), (4, 1, 0, 64, 4), (4, 1, 128, -64, 4),
])
def test_bad_descriptors(bits, scheme, K, N, status):
    with pytest.raises(lpq.LpqError) as e:
        lpq.lpq_packed_sizes(bits, scheme, K, N)
    assert e.value.status == status


def test_group_size_must_be_128_for_grouped_scheme():
    lib = lpq.load_library()
    c = ctypes.c_size_t()
    d = lpq.lpq_qdesc(4, 1, 64, 128, 64)
    assert lib.lpq_packed_sizes(ctypes.byref(d), ctypes.byref(c), ctypes.byref(c), ctypes.byref(c)) == 3
    assert lib.lpq_packed_sizes(None, ctypes.byref(c), ctypes.byref(c), ctypes.byref(c)) == 1
    d = lpq.lpq_qdesc(4, 1, 128, 128, 64)
    assert lib.lpq_packed_sizes(ctypes.byref(d), None, ctypes.byref(c), ctypes.byref(c)) == 1


def test_entry_points_validate_before_touching_the_device():
    lib = lpq.load_library()
    d = lpq.make_desc(4, 1, 128, 64)
    fake = 0x10000          # never dereferenced: every call below must fail validation first
    good = lpq.lpq_qweight(d, fake, fake, fake, None)
    # NULL pointers
    assert lib.lpq_quantize_pack(None, ctypes.byref(d), ctypes.byref(good), None) == 1
    assert lib.lpq_qlinear_decode(ctypes.byref(good), None, 1, fake, None) == 1
    assert lib.lpq_qlinear_prefill(ctypes.byref(good), fake, 1, None, None) == 1
    nz = lpq.lpq_qweight(d, fake, fake, None, None)
    assert lib.lpq_qlinear_decode(ctypes.byref(nz), fake, 1, fake, None) == 1
    assert lib.lpq_unpack_dequant(ctypes.byref(good), None, None) == 1
    assert lib.lpq_stage_linears(None, 1, 1, 1, None, None) == 1
    # M < 1
    assert lib.lpq_qlinear_decode(ctypes.byref(good), fake, 0, fake, None) == 4
    assert lib.lpq_qlinear_prefill(ctypes.byref(good), fake, -3, fake, None) == 4
    # alignment
    assert lib.lpq_qlinear_decode(ctypes.byref(good), fake + 2, 1, fake, None) == 5
    odd = lpq.lpq_qweight(d, fake + 8, fake, fake, None)
    assert lib.lpq_qlinear_prefill(ctypes.byref(odd), fake, 1, fake, None) == 5
    assert lib.lpq_quantize_pack(fake + 4, ctypes.byref(d), ctypes.byref(good), None) == 5
    # descriptor mismatch between desc and out
    d2 = lpq.make_desc(3, 1, 128, 64)
    assert lib.lpq_quantize_pack(fake, ctypes.byref(d2), ctypes.byref(good), None) == 4
    # row windows: on 64-row boundaries and inside W
    d3 = lpq.make_desc(4, 1, 128, 192)
    w3 = lpq.lpq_qweight(d3, fake, fake, fake, None)
    for row0, n_rows in ((32, 64), (0, 100), (128, 128), (-64, 64), (0, -64)):
        assert lib.lpq_quantize_pack_rows(fake, ctypes.byref(d3), row0, n_rows, ctypes.byref(w3), None) == 4
    assert lib.lpq_quantize_pack_rows(None, ctypes.byref(d3), 0, 64, ctypes.byref(w3), None) == 1
    assert lib.lpq_quantize_pack_rows(fake + 2, ctypes.byref(d3), 0, 64, ctypes.byref(w3), None) == 5
    # loader: NULL host or staging pointer, misaligned pointers, staging too small for 64 rows
    assert lib.lpq_load_quantize_pack(None, ctypes.byref(d3), ctypes.byref(w3), fake, 1 << 20, None) == 1
    assert lib.lpq_load_quantize_pack(fake, ctypes.byref(d3), ctypes.byref(w3), None, 1 << 20, None) == 1
    assert lib.lpq_load_quantize_pack(fake + 8, ctypes.byref(d3), ctypes.byref(w3), fake, 1 << 20, None) == 5
    assert lib.lpq_load_quantize_pack(fake, ctypes.byref(d3), ctypes.byref(w3), fake + 4, 1 << 20, None) == 5
    assert lib.lpq_load_quantize_pack(fake, ctypes.byref(d3), ctypes.byref(w3), fake, 64 * 128 * 2 - 1, None) == 6
    assert lib.lpq_load_quantize_pack(fake, ctypes.byref(d2), ctypes.byref(w3), fake, 1 << 20, None) == 4
    # fused epilogue: unknown activation, misaligned residual, unknown phase
    ep = lpq.lpq_epilogue(7, None)
    assert lib.lpq_qlinear_fused(ctypes.byref(good), fake, 1, fake, ctypes.byref(ep), 1, None) == 8
    ep = lpq.lpq_epilogue(1, fake + 2)
    assert lib.lpq_qlinear_fused(ctypes.byref(good), fake, 1, fake, ctypes.byref(ep), 1, None) == 5
    assert lib.lpq_qlinear_fused(ctypes.byref(good), fake, 1, fake, None, 3, None) == 8
    assert lib.lpq_qlinear_fused(ctypes.byref(good), None, 1, fake, None, 1, None) == 1
    # layer norm
    assert lib.lpq_layernorm(None, fake, fake, 1e-5, 1, 64, fake, None) == 1
    for M, h in ((0, 64), (1, 60), (1, 0), (1, 16392)):
        assert lib.lpq_layernorm(fake, fake, fake, 1e-5, M, h, fake, None) == 4
    assert lib.lpq_layernorm(fake, fake + 2, fake, 1e-5, 1, 64, fake, None) == 5
    # attention and KV cache: head size, cache length, positions
    st = lpq.lpq_layer_state(fake, fake, fake, fake, fake, fake, None)
    for cfg, n_seqs, T, pos0 in ((lpq.lpq_layer_cfg(4, 96, 128, 1, 1e-5), 1, 1, 0), (lpq.lpq_layer_cfg(4, 64, 100, 1, 1e-5), 1, 1, 0),
                                 (lpq.lpq_layer_cfg(4, 64, 128, 1, 1e-5), 1, 2, 127), (lpq.lpq_layer_cfg(4, 64, 128, 1, 1e-5), 0, 1, 0),
                                 (lpq.lpq_layer_cfg(0, 64, 128, 1, 1e-5), 1, 1, 0), (lpq.lpq_layer_cfg(4, 64, 128, 1, 1e-5), 1, 1, -1)):
        assert lib.lpq_kv_append(fake, ctypes.byref(cfg), ctypes.byref(st), n_seqs, T, pos0, None) == 4
        assert lib.lpq_attention(fake, ctypes.byref(cfg), ctypes.byref(st), n_seqs, T, pos0, fake, None) == 4
    cfg = lpq.lpq_layer_cfg(4, 64, 128, 1, 1e-5)
    no_cache = lpq.lpq_layer_state(fake, fake, fake, fake, None, fake, None)
    assert lib.lpq_attention(fake, ctypes.byref(cfg), ctypes.byref(no_cache), 1, 1, 0, fake, None) == 1
    assert lib.lpq_attention(fake + 2, ctypes.byref(cfg), ctypes.byref(st), 1, 1, 0, fake, None) == 5
    # decoder layer: weights must fit hidden = heads * head_dim; workspace size is checked
    h, f = 256, 512
    mk = lambda K, N: lpq.lpq_qweight(lpq.make_desc(4, 1, K, N), fake, fake, fake, None)
    layer = lpq.lpq_layer(mk(h, 3 * h), mk(h, h), mk(h, f), mk(f, h))
    need = lib.lpq_decoder_layer_workspace(ctypes.byref(layer), ctypes.byref(cfg), 8)
    assert need == 8 * (5 * h + f) * 2 and lib.lpq_decoder_layer_workspace(None, ctypes.byref(cfg), 8) == 0
    args = (ctypes.byref(layer), ctypes.byref(cfg), ctypes.byref(st), 1, 8, 1, 0, fake, fake, fake)
    assert lib.lpq_decoder_layer(*args, need - 1, None) == 6
    wrong = lpq.lpq_layer(mk(h, 3 * h), mk(h, h), mk(h, f), mk(f, 2 * h))
    assert lib.lpq_decoder_layer(ctypes.byref(wrong), *args[1:], need, None) == 4
    bad_act = lpq.lpq_layer_cfg(4, 64, 128, 9, 1e-5)
    assert lib.lpq_decoder_layer(args[0], ctypes.byref(bad_act), *args[2:], need, None) == 8
    assert lib.lpq_decoder_layer(args[0], args[1], args[2], 1, 8, 1, 0, None, fake, fake, need, None) == 1
    # variance indicator
    assert lib.lpq_variance_indicator(None, 128, 64, fake, 1, 0, fake, None) == 1
    assert lib.lpq_variance_indicator(fake, 128, 64, fake, 1, 0, None, None) == 1
    for K, N, M in ((100, 64, 1), (0, 64, 1), (128, 0, 1), (128, 64, 0)):
        assert lib.lpq_variance_indicator(fake, K, N, fake, M, 0, fake, None) == 4
    assert lib.lpq_variance_indicator(fake + 2, 128, 64, fake, 1, 0, fake, None) == 5
    assert lib.lpq_variance_indicator(fake, 128, 64, fake, 1, 0, fake + 4, None) == 5
    # bad bits inside a weight
    bad = lpq.lpq_qweight(lpq.lpq_qdesc(5, 1, 128, 128, 64), fake, fake, fake, None)
    assert lib.lpq_qlinear_decode(ctypes.byref(bad), fake, 1, fake, None) == 2
    # stage: bad layer count, bad phase, one bad layer rejects the whole call
    layers = (lpq.lpq_layer * 1)()
    io = (lpq.lpq_layer_io * 1)()
    assert lib.lpq_stage_linears(layers, 0, 1, 1, io, None) == 4
    assert lib.lpq_stage_linears(layers, 1, 5, 1, io, None) == 8
    assert lib.lpq_stage_linears(layers, 1, 1, 1, io, None) != 0      # zeroed layer: bits = 0
    for i in range(9):
        assert isinstance(lpq.status_str(i), str) and lpq.status_str(i)
    assert lpq.status_str(99) == "unknown status"


def test_workspace_growth_policy():
    """The per-device workspace never frees a block it has handed out: a larger need allocates a new block
    (need + 25 %, at least 8 MiB), a need that fits reuses the block, and once a reservation is in force a
    larger need is an error instead of an allocation.  (Pure host function: what the library does on a device
    is this policy followed by one hipMalloc.)"""
    MiB = 1 << 20
    assert lpq.lpq_workspace_policy(0, False, 1) == 8 * MiB                    # first use: the floor
    assert lpq.lpq_workspace_policy(8 * MiB, False, 8 * MiB) == 0              # fits: reuse
    assert lpq.lpq_workspace_policy(8 * MiB, False, 8 * MiB + 1) == 8 * MiB + 1 + (8 * MiB + 1) // 4
    assert lpq.lpq_workspace_policy(8 * MiB, False, 64 * MiB) == 80 * MiB      # growth leaves headroom
    assert lpq.lpq_workspace_policy(80 * MiB, True, 80 * MiB) == 0             # reserved and large enough
    with pytest.raises(lpq.LpqError) as err:
        lpq.lpq_workspace_policy(80 * MiB, True, 80 * MiB + 1)                 # reserved: no growth
    assert err.value.status == 6
    assert lpq.load_library().lpq_workspace_policy(0, 0, 1, None) == 1
    # a sequence of needs never shrinks the block and allocates only when a need exceeds it
    have, allocs = 0, 0
    for need in (1, 4 * MiB, 9 * MiB, 3 * MiB, 11 * MiB, 12 * MiB, 200 * MiB, 10 * MiB):
        a = lpq.lpq_workspace_policy(have, False, need)
        if a:
            assert a >= need and a > have
            have, allocs = a, allocs + 1
        assert have >= need
    assert allocs == 4


def test_decode_routing_arguments():
    lib = lpq.load_library()
    assert lib.lpq_set_decode_routing(0, 0) == 0 and lib.lpq_set_decode_routing(-1, 5) == 0
    for mib, tiles in ((5000, 0), (192, 1), (192, 6)):
        assert lib.lpq_set_decode_routing(mib, tiles) == 4
    assert lib.lpq_set_decode_routing(-1, -1) == 0
