"""Host-side checks of the C ABI: the library loads, exports every symbol that
include/cmoe.h declares, and rejects bad arguments before any HIP call (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

import paper_2510_02345_amd as cm
from paper_2510_02345_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "cmoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cmoe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = cm.lib()
    names = _declared_symbols()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def _create(**kw):
    base = dict(d=128, d_ff=512, G=2, K=4, r=4, top_k=1, q_group=32, activation=0)
    base.update(kw)
    cfg = B.Config(*[base[n] for n in ("d", "d_ff", "G", "K", "r", "top_k", "q_group", "activation")])
    h = C.c_void_p()
    rc = cm.lib().cmoe_create(C.byref(cfg), C.byref(h))
    return rc, h


def test_create_validates_configuration():
    rc, h = _create()
    assert rc == B.OK and h.value
    assert cm.lib().cmoe_destroy(h) == B.OK
    assert cm.lib().cmoe_destroy(None) == B.ERR_INVALID_ARG
    for bad in (dict(d=100), dict(d_ff=500), dict(r=5), dict(top_k=5), dict(top_k=9, K=16), dict(q_group=12),
                dict(q_group=48), dict(G=65), dict(K=33), dict(K=32, r=32), dict(activation=1), dict(d=16384)):
        rc, h = _create(**bad)
        assert rc == B.ERR_UNSUPPORTED, bad
        assert not h.value
    for bad in (dict(d=0), dict(G=-1), dict(top_k=0)):
        rc, h = _create(**bad)
        assert rc == B.ERR_INVALID_ARG, bad
    assert cm.lib().cmoe_create(None, None) == B.ERR_INVALID_ARG


def test_workspace_bytes_monotone_and_covers_intermediates():
    rc, h = _create(d=768, d_ff=3072, G=2, K=4, r=8, top_k=2, q_group=32)
    L = cm.lib()
    assert L.cmoe_workspace_bytes(None, 10) == 0
    assert L.cmoe_workspace_bytes(h, -1) == 0
    w0, w1, w2 = (L.cmoe_workspace_bytes(h, t) for t in (0, 1000, 4096))
    assert 0 < w0 < w1 < w2
    # at least the f16 hidden activations A [T][d_ff] and y_base_sorted [T][d]
    assert w2 - w0 >= 4096 * (3072 + 768) * 2
    L.cmoe_destroy(h)


def test_workspace_for_t_max_serves_every_smaller_t():
    # the weight-streaming path (up to 256 tokens) and the matrix-core path lay the workspace
    # out differently; a buffer sized for T_max must still be large enough for any T <= T_max
    L = cm.lib()
    shapes = [dict(d=4096, d_ff=14336, G=8, K=8, r=32, top_k=2, q_group=128),
              dict(d=768, d_ff=3072, G=2, K=4, r=8, top_k=2, q_group=32),
              dict(d=8192, d_ff=128, G=64, K=2, r=4, top_k=2, q_group=128),
              dict(d=128, d_ff=512, G=2, K=4, r=4, top_k=1, q_group=32)]
    for kw in shapes:
        rc, h = _create(**kw)
        assert rc == B.OK
        ts = [0, 1, 16, 64, 255, 256, 257, 258, 300, 511, 512, 513, 1000, 1024, 4096]
        sizes = [L.cmoe_workspace_bytes(h, t) for t in ts]
        for i in range(1, len(ts)):
            assert sizes[i] >= sizes[i - 1], (kw, ts[i - 1], ts[i], sizes[i - 1], sizes[i])
        for top_g in (1, 2):
            m = [L.cmoe_workspace_bytes_multi(h, t, top_g) for t in ts]
            for i in range(1, len(ts)):
                assert m[i] >= m[i - 1], (kw, top_g, ts[i])
            assert all(a >= b for a, b in zip(m, sizes))
        L.cmoe_destroy(h)


def test_calls_reject_bad_arguments_without_touching_the_gpu():
    rc, h = _create()
    L = cm.lib()
    w = B.Weights()                                   # all NULL
    assert L.cmoe_route(h, C.byref(w), None, 4, None, None, None, None) == B.ERR_INVALID_ARG
    assert L.cmoe_route(h, None, None, 0, None, None, None, None) == B.ERR_INVALID_ARG
    assert L.cmoe_route(None, C.byref(w), None, 0, None, None, None, None) == B.ERR_INVALID_ARG
    fake = 0x1000                                     # aligned, never dereferenced on the host
    w2 = B.Weights(*([fake] * 13))
    assert L.cmoe_route(h, C.byref(w2), fake, -1, fake, fake, fake, None) == B.ERR_INVALID_ARG
    assert L.cmoe_route(h, C.byref(w2), fake + 2, 4, fake, fake, fake, None) == B.ERR_INVALID_ARG   # misaligned x
    assert L.cmoe_route(h, C.byref(w2), fake, 0, fake, fake, fake, None) == B.OK                    # T = 0 no-op
    # workspace checks come before any launch
    assert L.cmoe_permute(h, fake, 8, fake, fake, fake, None, 0, None) == B.ERR_WORKSPACE
    assert L.cmoe_permute(h, fake, 8, fake, fake, fake, fake + 16, 1 << 30, None) == B.ERR_WORKSPACE  # misaligned
    assert L.cmoe_permute(h, fake, 8, fake, fake, fake, fake, 16, None) == B.ERR_WORKSPACE            # too small
    assert L.cmoe_ffn_forward(h, C.byref(w2), fake, 8, fake, fake, fake, fake, fake, fake, fake, 16, None) == B.ERR_WORKSPACE
    assert L.cmoe_ffn_forward(h, C.byref(w), fake, 8, fake, fake, fake, fake, fake, fake, fake, 1 << 30, None) == B.ERR_INVALID_ARG
    assert L.cmoe_combine(h, C.byref(w2), fake, fake, fake, fake, fake, fake, fake, 8, None, fake, 1 << 30, None) == B.ERR_INVALID_ARG
    assert L.cmoe_forward(h, C.byref(w2), fake, 8, fake, fake, fake, fake, fake, fake, fake, fake, 16, None) == B.ERR_WORKSPACE
    assert L.cmoe_last_hip_error(h) == 0
    assert cm.status_string(B.ERR_WORKSPACE).startswith("workspace")
    assert cm.status_string(B.OK) == "ok"
    L.cmoe_destroy(h)


def test_timing_names():
    L = cm.lib()
    names = [L.cmoe_timing_name(i).decode() for i in range(8)]
    assert names[0] == "route" and "gemm1_fused" in names and L.cmoe_timing_name(99) == b""


def test_new_entry_points_reject_bad_arguments_without_touching_the_gpu():
    rc, h = _create()
    L = cm.lib()
    fake = 0x1000
    w2 = B.Weights(*([fake] * 13))
    # routing statistics: EMA rates outside [0, 1], missing state, workspace
    args = [h, fake, 8, fake, fake, fake]
    tail = [fake, fake, fake, fake, fake, fake]
    assert L.cmoe_route_stats(*args, 1.5, 0.1, *tail, fake, 1 << 30, None) == B.ERR_INVALID_ARG
    assert L.cmoe_route_stats(*args, 0.05, -0.1, *tail, fake, 1 << 30, None) == B.ERR_INVALID_ARG
    assert L.cmoe_route_stats(*args, 0.05, 0.1, None, fake, fake, fake, fake, fake, fake, 1 << 30, None) == B.ERR_INVALID_ARG
    assert L.cmoe_route_stats(*args, 0.05, 0.1, *tail, fake, 16, None) == B.ERR_WORKSPACE
    # routing variants: top_g beyond G or 8, non-positive temperature
    for top_g, tau in ((0, 1.0), (3, 1.0), (9, 1.0), (1, 0.0), (2, -1.0)):
        opt = B.RouteOptions(top_g, tau, 0)
        assert L.cmoe_route_multi(h, C.byref(w2), C.byref(opt), fake, 4, fake, fake, fake, None) == B.ERR_INVALID_ARG
    assert L.cmoe_route_multi(h, C.byref(w2), None, fake, 4, fake, fake, fake, None) == B.ERR_INVALID_ARG
    ok = B.RouteOptions(2, 0.7, 1)
    assert L.cmoe_route_multi(h, C.byref(w2), C.byref(ok), fake, 0, fake, fake, fake, None) == B.OK   # T = 0 no-op
    assert L.cmoe_workspace_bytes_multi(h, 1024, 3) == 0 and L.cmoe_workspace_bytes_multi(h, 1024, 0) == 0
    assert L.cmoe_workspace_bytes_multi(h, 1024, 2) > L.cmoe_workspace_bytes(h, 2048)
    assert L.cmoe_forward_multi(h, C.byref(w2), C.byref(ok), fake, 8, fake, fake, fake, fake, fake, fake, fake, fake,
                                16, None) == B.ERR_WORKSPACE
    L.cmoe_destroy(h)
    # compression: shapes outside the supported set give no workspace size and are refused
    good = B.CompressConfig(256, 128, 2, 4, 8, 32, 16, 2, 0, 0.0)
    assert L.cmoe_compress_workspace_bytes(C.byref(good)) > 2 * 8 * 256 * 128 * 2        # Delta and its transpose
    for bad in (B.CompressConfig(250, 128, 2, 4, 8, 32, 16, 2, 0, 0.0),      # out_dim not a multiple of 64
                B.CompressConfig(256, 128, 2, 4, 8, 48, 16, 2, 0, 0.0),      # q_group does not divide
                B.CompressConfig(256, 128, 2, 4, 8, 32, 4, 2, 0, 0.0),       # sketch narrower than r
                B.CompressConfig(256, 128, 2, 4, 8, 32, 64, 2, 0, 0.0),      # sketch wider than 48
                B.CompressConfig(256, 128, 2, 4, 40, 32, 48, 2, 0, 0.0)):    # r > 32
        assert L.cmoe_compress_workspace_bytes(C.byref(bad)) == 0
        assert L.cmoe_compress(C.byref(bad), fake, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 40,
                               None) == B.ERR_UNSUPPORTED
    assert L.cmoe_compress(C.byref(good), None, fake, fake, fake, fake, fake, fake, fake, fake, 1 << 40,
                           None) == B.ERR_INVALID_ARG
    assert L.cmoe_compress(C.byref(good), fake, fake, fake, fake, fake, fake, fake, fake, fake, 16, None) == B.ERR_WORKSPACE
    assert L.cmoe_quantize_int4(fake, 4, 64, 24, fake, fake, None) == B.ERR_INVALID_ARG    # q does not divide L
    assert L.cmoe_quantize_int4(fake, 0, 64, 8, fake, fake, None) == B.OK                  # no rows: no-op


def test_backward_rejects_bad_arguments_without_touching_the_gpu():
    rc, h = _create(d=768, d_ff=3072, G=2, K=4, r=8, top_k=2, q_group=32)
    L = cm.lib()
    fake = 0x1000
    w2 = B.Weights(*([fake] * 13))
    g = B.Grads(*([fake] * 9))
    need = L.cmoe_backward_workspace_bytes(h, 4096)
    # per-token and per-pair FP16 activations and the transposed bases at least
    assert need > (8 * 2 + 12) * 4096 * 3072 + 4 * 2 * 768 * 3072
    assert L.cmoe_backward_workspace_bytes(h, -1) == 0 and L.cmoe_backward_workspace_bytes(None, 8) == 0
    assert L.cmoe_backward(h, C.byref(w2), fake, fake, 8, fake, fake, None, fake, need, None) == B.ERR_INVALID_ARG
    assert L.cmoe_backward(h, C.byref(w2), None, fake, 8, fake, fake, C.byref(g), fake, need, None) == B.ERR_INVALID_ARG
    assert L.cmoe_backward(h, C.byref(w2), fake, fake, -1, fake, fake, C.byref(g), fake, need, None) == B.ERR_INVALID_ARG
    g_bad = B.Grads(*([fake] * 9))
    g_bad.dw1_base = None
    assert L.cmoe_backward(h, C.byref(w2), fake, fake, 8, fake, fake, C.byref(g_bad), fake, need, None) == B.ERR_INVALID_ARG
    assert L.cmoe_backward(h, C.byref(w2), fake, fake, 8, fake, fake, C.byref(g), fake, 16, None) == B.ERR_WORKSPACE
    assert L.cmoe_backward(h, C.byref(w2), fake, fake, 8, fake, fake, C.byref(g), None, need, None) == B.ERR_WORKSPACE
    L.cmoe_destroy(h)
    # more than 64 experts are supported too (pairs sorted by expert in two passes)
    rc, h = _create(d=64, d_ff=64, G=20, K=8, r=4, top_k=2, q_group=8)
    assert rc == B.OK
    assert L.cmoe_backward_workspace_bytes(h, 8) > 0
    assert L.cmoe_backward(h, C.byref(w2), fake, fake, 8, fake, fake, C.byref(g), fake, 16, None) == B.ERR_WORKSPACE
    L.cmoe_destroy(h)


def test_pack_weights_rejects_bad_arguments_without_touching_the_gpu():
    rc, h = _create(d=768, d_ff=3072, G=2, K=4, r=8, top_k=2, q_group=32)
    L = cm.lib()
    fake = 0x1000
    w2 = B.Weights(*([fake] * 13))
    assert w2.packed is None                                    # canonical arrays only by default
    need = L.cmoe_packed_bytes(h)
    # both bases in FP16 blocks plus the FP16 panels of the four factor tensors (K*r = 32 rank rows per cluster)
    assert need == 4 * 2 * 768 * 3072 + 2 * 2 * 32 * 2 * (768 + 3072) and L.cmoe_packed_bytes(None) == 0
    assert L.cmoe_pack_weights(h, C.byref(w2), None, need, None) == B.ERR_INVALID_ARG
    assert L.cmoe_pack_weights(h, C.byref(w2), 0x1010, need, None) == B.ERR_INVALID_ARG      # not 256-byte aligned
    assert L.cmoe_pack_weights(h, C.byref(w2), fake, need - 1, None) == B.ERR_WORKSPACE
    assert L.cmoe_pack_weights(h, None, fake, need, None) == B.ERR_INVALID_ARG
    nobase = B.Weights(*([fake] * 13))
    nobase.w2_base = None
    assert L.cmoe_pack_weights(h, C.byref(nobase), fake, need, None) == B.ERR_INVALID_ARG
    nofactor = B.Weights(*([fake] * 13))
    nofactor.u2_s = None
    assert L.cmoe_pack_weights(h, C.byref(nofactor), fake, need, None) == B.ERR_INVALID_ARG
    # a misaligned packed pointer is refused by the calls that would read it
    bad = B.Weights(*([fake] * 13))
    bad.packed = 0x1008
    assert L.cmoe_ffn_forward(h, C.byref(bad), fake, 8, fake, fake, fake, fake, fake, fake, fake, 1 << 40,
                              None) == B.ERR_INVALID_ARG
    # bases: the canonical arrays or the packed copy; with neither, or with only one of the two
    # canonical arrays and no packed copy, the call is refused before any GPU work
    nob = B.Weights(*([fake] * 13))
    nob.w1_base = None
    assert L.cmoe_ffn_forward(h, C.byref(nob), fake, 8, fake, fake, fake, fake, fake, fake, fake, 16,
                              None) == B.ERR_INVALID_ARG
    nob.w2_base = None
    nob.packed = fake                  # packed copy alone: accepted (here it fails later, on the workspace size)
    assert L.cmoe_ffn_forward(h, C.byref(nob), fake, 8, fake, fake, fake, fake, fake, fake, fake, 16,
                              None) == B.ERR_WORKSPACE
    L.cmoe_destroy(h)
