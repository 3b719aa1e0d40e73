"""Pins of the FP64 oracle against what the paper and the mathematics fix.

None of these tests touches the GPU.  Each pins one part of oracle/cmoe_oracle.py to
something other than itself: hand-typed tables, brute-force scalar loops, library
routines of a different implementation (math.erf, numpy stable argsort), closed
forms the paper states, and invariants of the method.
"""
import math
import os

import numpy as np
import pytest

import cmoe_inputs as ci
from oracle import cmoe_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_closed_forms.txt")


def _golden():
    out = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            out[k] = float(v)
    return out


# ------------------------------------------------------------------ INT4 (Sec. 3.4)
def test_int4_all_codes_both_nibbles():
    # two's-complement table typed by hand
    table = {0: 0, 1: 1, 2: 2, 3: 3, 4: 4, 5: 5, 6: 6, 7: 7, 8: -8, 9: -7, 10: -6, 11: -5, 12: -4, 13: -3, 14: -2, 15: -1}
    for lo in range(16):
        for hi in range(16):
            b = np.array([[lo | (hi << 4)]], dtype=np.uint8)
            codes = orc.unpack_int4(b)
            assert codes.shape == (1, 2)
            assert codes[0, 0] == table[lo] and codes[0, 1] == table[hi]
    for scale in (0.0, 1.0, 0.0123, 6.1e-5, 1024.0):
        s16 = np.array([[scale]], dtype=np.float16)
        packed = np.arange(256, dtype=np.uint8).reshape(1, 256)
        # one group covering all 512 elements
        val = orc.dequant_int4(packed, s16, 512)
        for byte in range(256):
            assert val[0, 2 * byte] == float(s16[0, 0]) * table[byte & 15]
            assert val[0, 2 * byte + 1] == float(s16[0, 0]) * table[byte >> 4]


def test_int4_group_boundaries_and_roundtrip():
    rng = np.random.default_rng(1)
    w = rng.standard_normal((3, 2, 128)) * 0.02
    q = 32
    packed, scales = ci.quantize_int4(w, q)
    assert packed.shape == (3, 2, 64) and scales.shape == (3, 2, 4)
    val = orc.dequant_int4(packed, scales, q)
    # element n uses scale n // q: check by a scalar loop
    for e in range(3):
        for rr in range(2):
            for n in range(128):
                byte = int(packed[e, rr, n // 2])
                code = (byte >> 4) if (n & 1) else (byte & 15)
                code = code - 16 if code >= 8 else code
                assert val[e, rr, n] == float(scales[e, rr, n // q]) * code
    # quantisation error at most half a step (plus the fp16 rounding of the scale)
    step = np.repeat(scales.astype(np.float64), q, axis=-1)
    assert np.all(np.abs(val - w) <= 0.5 * step * (1 + 2e-3) + 1e-12)
    # an all-zero group decodes to exact zeros
    w[0, 0, :32] = 0
    packed, scales = ci.quantize_int4(w, q)
    assert np.all(orc.dequant_int4(packed, scales, q)[0, 0, :32] == 0)


# ------------------------------------------------------------------ routing (Sec. 3.3)
def _brute_route(x, rc, re, K, k, bias):
    T, d = x.shape
    G = rc.shape[0]
    cid, eidx, gates = [], [], []
    for t in range(T):
        z = [sum(float(rc[g, i]) * float(x[t, i]) for i in range(d)) + (float(bias[g]) if bias is not None else 0.0)
             for g in range(G)]
        # Eq. 9 softmax, then the most probable group
        m = max(z)
        p = [math.exp(v - m) for v in z]
        sp = sum(p)
        p = [v / sp for v in p]
        c = max(range(G), key=lambda g: (p[g], -g))
        l = [sum(float(re[c * K + j, i]) * float(x[t, i]) for i in range(d)) for j in range(K)]
        m = max(l)
        pe = [math.exp(v - m) for v in l]
        spe = sum(pe)
        pe = [v / spe for v in pe]                       # Eq. 10
        order = sorted(range(K), key=lambda j: (-pe[j], j))[:k]
        tot = sum(pe[j] for j in order)
        cid.append(c)
        eidx.append([c * K + j for j in order])
        gates.append([pe[j] / tot for j in order])
    return np.array(cid), np.array(eidx), np.array(gates)


@pytest.mark.parametrize("G,K,k", [(2, 4, 1), (2, 4, 2), (4, 4, 2), (3, 5, 3), (1, 8, 2), (4, 2, 2)])
def test_route_matches_bruteforce_softmax_argsort(G, K, k):
    cfg = ci.small_config(T=48, d=24, d_ff=32, G=G, K=K, r=4, k=k, q=8, seed=100 + G * 10 + K)
    w = ci.generate(cfg, with_weights=False)
    bias = np.linspace(-0.3, 0.3, G).astype(np.float32)
    for b in (None, bias):
        cid, eidx, gate, z, l = orc.route(w["x"], w["router_cluster"], w["router_expert"], K, k, b)
        bc, be, bg = _brute_route(w["x"], w["router_cluster"], w["router_expert"], K, k, b)
        assert np.array_equal(cid, bc)
        assert np.array_equal(eidx, be)
        assert np.allclose(gate, bg, rtol=1e-12, atol=1e-15)
        assert np.allclose(gate.sum(axis=1), 1.0, atol=1e-14)
        assert cid.dtype == np.int32 and eidx.dtype == np.int32


def test_route_special_cases():
    cfg = ci.small_config(T=64, d=32, G=2, K=4, k=1, q=8)
    w = ci.generate(cfg, with_weights=False)
    _, eidx, gate, _, l = orc.route(w["x"], w["router_cluster"], w["router_expert"], 4, 1)
    assert np.all(gate == 1.0)                         # k = 1: the gate is exactly one
    # K = k: every expert of the cluster is selected, gates are the Eq. 10 probabilities
    cid, eidx, gate, _, l = orc.route(w["x"], w["router_cluster"], w["router_expert"], 4, 4)
    assert np.array_equal(np.sort(eidx - cid[:, None] * 4, axis=1), np.tile(np.arange(4), (64, 1)))
    p = np.exp(l) / np.exp(l).sum(axis=1, keepdims=True)
    assert np.allclose(np.sort(gate, axis=1), np.sort(p, axis=1), rtol=1e-12)
    # G = 1: a flat top-k router over all experts
    cid, eidx, gate, _, _ = orc.route(w["x"], w["router_cluster"][:1], w["router_expert"][:4], 4, 2)
    assert np.all(cid == 0)
    full = w["x"].astype(np.float64) @ w["router_expert"][:4].astype(np.float64).T
    assert np.array_equal(eidx, np.argsort(-full, axis=1, kind="stable")[:, :2])


def test_route_ties_lowest_index_wins():
    x = np.ones((3, 8), dtype=np.float16)
    rc = np.zeros((3, 8), dtype=np.float16)            # all cluster logits equal -> cluster 0
    re = np.zeros((12, 8), dtype=np.float16)
    re[1] = 1
    re[2] = 1                                          # experts 1 and 2 tie for first
    cid, eidx, gate, _, _ = orc.route(x, rc, re, 4, 3)
    assert np.all(cid == 0)
    assert np.array_equal(eidx[0], [1, 2, 0])
    assert gate[0, 0] == gate[0, 1]


def test_input_margin_is_enforced():
    for cfg in (ci.config(0), ci.small_config(T=512, d=32, G=4, K=4, k=2, q=8)):
        w = ci.generate(cfg, with_weights=False)
        _, _, _, z, l = orc.route(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, w["cluster_bias"])
        zs = np.sort(z, axis=1)
        assert np.all(zs[:, -1] - zs[:, -2] >= ci.MARGIN)
        ls = -np.sort(-l, axis=1)
        for a in range(min(cfg.k + 1, cfg.K) - 1):
            assert np.all(ls[:, a] - ls[:, a + 1] >= ci.MARGIN)


# ------------------------------------------------------------------ permutation
@pytest.mark.parametrize("T,G", [(0, 3), (1, 1), (257, 4), (1000, 8)])
def test_permute_matches_stable_argsort(T, G):
    rng = np.random.default_rng(T + G)
    cid = rng.integers(0, G, size=T).astype(np.int32)
    if T > 10:
        cid[cid == 1] = 0                              # leave a cluster empty
    offsets, perm, inv = orc.permute(cid, G)
    assert np.array_equal(perm, np.argsort(cid, kind="stable"))
    assert np.array_equal(offsets, np.concatenate([[0], np.cumsum(np.bincount(cid, minlength=G))]))
    assert np.array_equal(inv[perm], np.arange(T))
    assert np.array_equal(perm[inv], np.arange(T))
    assert np.all(np.diff(cid[perm]) >= 0)


# ------------------------------------------------------------------ FFN value
def _gelu_scalar(u):
    return 0.5 * u * (1.0 + math.erf(u / math.sqrt(2.0)))


def test_gelu_spot_values_and_identities():
    u = np.linspace(-6, 6, 241)
    g = orc.gelu(u)
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert np.allclose(g - orc.gelu(-u), u, atol=1e-15)             # GELU(u) - GELU(-u) = u
    assert np.allclose(g, [_gelu_scalar(v) for v in u], rtol=1e-14, atol=1e-16)
    assert abs(orc.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)


def _brute_forward(w, x, K, k, q):
    """Every sum written out as scalar loops, straight from the definition."""
    T, d = x.shape
    G, d_ff, _ = w["w1_base"].shape
    E = G * K
    r = w["v1_q"].shape[1]

    def deq(name, e, rho, n):
        byte = int(w[name + "_q"][e, rho, n // 2])
        code = (byte >> 4) if (n & 1) else (byte & 15)
        code = code - 16 if code >= 8 else code
        return float(w[name + "_s"][e, rho, n // q]) * code

    cid, eidx, gate = _brute_route(x, w["router_cluster"], w["router_expert"], K, k, w.get("cluster_bias"))
    y = np.zeros((T, d))
    for t in range(T):
        c = int(cid[t])
        for jj in range(k):
            e = int(eidx[t, jj])
            h = []
            for o in range(d_ff):
                acc = 0.0
                for i in range(d):
                    wv = float(w["w1_base"][c, o, i]) + sum(deq("u1", e, rho, o) * deq("v1", e, rho, i) for rho in range(r))
                    acc += wv * float(x[t, i])
                h.append(_gelu_scalar(acc))
            for o in range(d):
                acc = 0.0
                for i in range(d_ff):
                    wv = float(w["w2_base"][c, o, i]) + sum(deq("u2", e, rho, o) * deq("v2", e, rho, i) for rho in range(r))
                    acc += wv * h[i]
                y[t, o] += gate[t, jj] * acc
    return cid, eidx, gate, y


def test_forward_matches_scalar_bruteforce():
    cfg = ci.small_config(T=6, d=8, d_ff=12, G=2, K=3, r=2, k=2, q=4, factor_std=0.3, seed=7)
    w = ci.generate(cfg)
    out = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    cid, eidx, gate, y = _brute_forward(w, w["x"], cfg.K, cfg.k, cfg.q)
    assert np.array_equal(out["cluster_id"], cid)
    assert np.array_equal(out["expert_idx"], eidx)
    assert np.allclose(out["gate"], gate, rtol=1e-12)
    assert np.allclose(out["y"], y, rtol=1e-11, atol=1e-13)
    # the factors are large enough here that dropping any residual term is visible
    w0 = dict(w)
    for n in ("u1", "u2"):
        w0[n + "_s"] = np.zeros_like(w[n + "_s"])
    y0 = orc.forward_naive(w0, w["x"], cfg.K, cfg.k, cfg.q)["y"]
    assert np.abs(y0 - y).max() > 1e-2 * np.abs(y).max()


def test_single_expert_zero_residual_is_dense_ffn():
    # G = K = k = 1 and zero residuals: the layer is W2 GELU(W1 x)
    cfg = ci.small_config(T=5, d=16, d_ff=24, G=1, K=1, r=2, k=1, q=8, seed=3)
    w = ci.generate(cfg)
    for n in ("v1", "u1", "v2", "u2"):
        w[n + "_s"] = np.zeros_like(w[n + "_s"])
    y = orc.forward_naive(w, w["x"], 1, 1, cfg.q)["y"]
    W1 = w["w1_base"][0].astype(np.float64)
    W2 = w["w2_base"][0].astype(np.float64)
    X = w["x"].astype(np.float64)
    ref = np.zeros_like(y)
    for t in range(5):
        h = [_gelu_scalar(v) for v in W1 @ X[t]]
        ref[t] = W2 @ np.array(h)
    assert np.allclose(y, ref, rtol=1e-13, atol=1e-15)


def test_zero_residual_all_experts_equal_base():
    # invariant (i): Eq. 6/7 with Delta W = 0: every expert of a cluster is the base
    cfg = ci.small_config(T=40, d=16, d_ff=32, G=2, K=4, r=4, k=2, q=8, seed=11)
    w = ci.generate(cfg)
    for n in ("v1", "v2"):
        w[n + "_s"] = np.zeros_like(w[n + "_s"])
    out = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    cid = out["cluster_id"]
    rng = np.random.default_rng(0)
    other = (cid[:, None] * cfg.K + rng.integers(0, cfg.K, size=(cfg.T, cfg.k))).astype(np.int32)
    y_other = orc.ffn_naive(w, w["x"], other, out["gate"], cfg.K, cfg.q)
    assert np.allclose(out["y"], y_other, rtol=1e-12, atol=1e-14)
    X = w["x"].astype(np.float64)
    for t in range(cfg.T):
        c = cid[t]
        ref = w["w2_base"][c].astype(np.float64) @ orc.gelu(w["w1_base"][c].astype(np.float64) @ X[t])
        assert np.allclose(out["y"][t], ref, rtol=1e-12, atol=1e-14)


def test_base_is_mean_of_materialised_experts():
    # Eq. 6: if the residuals of a cluster sum to zero, the mean of its experts is the base
    cfg = ci.small_config(T=4, d=16, d_ff=16, G=1, K=2, r=2, k=1, q=8, seed=5)
    w = ci.generate(cfg)
    for n in ("v1", "v2"):                           # expert 1 = mirror image of expert 0
        w[n + "_q"][1] = w[n + "_q"][0]
        w[n + "_s"][1] = w[n + "_s"][0]
    for n in ("u1", "u2"):
        codes = orc.unpack_int4(w[n + "_q"][0]).astype(np.int8)
        w[n + "_q"][1] = ci.pack_int4(-codes)
        w[n + "_s"][1] = w[n + "_s"][0]
    W1a, W2a = orc.expert_weights(w, 0, 2, cfg.q)
    W1b, W2b = orc.expert_weights(w, 1, 2, cfg.q)
    assert np.allclose((W1a + W1b) / 2, w["w1_base"][0].astype(np.float64), atol=1e-15)
    assert np.allclose((W2a + W2b) / 2, w["w2_base"][0].astype(np.float64), atol=1e-15)
    assert np.abs(W1a - W1b).max() > 0


@pytest.mark.parametrize("seed,k", [(21, 1), (22, 2), (23, 3)])
def test_rewrite_equals_naive(seed, k):
    # invariant (ii): base product shared + linearity of the second base matrix
    cfg = ci.small_config(T=16, d=32, d_ff=48, G=3, K=4, r=4, k=k, q=8, factor_std=0.2, seed=seed)
    w = ci.generate(cfg)
    out = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    rw = orc.ffn_rewrite(w, w["x"], out["perm"], out["offsets"], out["expert_idx"], out["gate"], cfg.K, cfg.q)
    scale = np.abs(out["y"]).max()
    assert np.abs(rw["y"] - out["y"]).max() <= 1e-12 * scale
    assert np.array_equal(rw["y_sorted"], rw["y"][out["perm"]])
    # the residual terms matter at this factor size (a dropped term would show)
    assert np.abs(rw["y_base_sorted"] - rw["y_sorted"]).max() > 1e-3 * scale


def test_expert_weights_orientation():
    # W1_e[o][i] = W1_base[o][i] + sum_rho U1[rho][o] V1[rho][i], checked on single entries
    cfg = ci.small_config(T=2, d=8, d_ff=16, G=1, K=2, r=2, k=1, q=8, factor_std=0.5, seed=9)
    w = ci.generate(cfg)
    f = {n: orc.dequant_int4(w[n + "_q"], w[n + "_s"], cfg.q) for n in ("v1", "u1", "v2", "u2")}
    W1, W2 = orc.expert_weights(w, 1, 2, cfg.q)
    assert W1.shape == (16, 8) and W2.shape == (8, 16)
    for (o, i) in ((0, 0), (15, 7), (3, 5)):
        ref = float(w["w1_base"][0, o, i]) + sum(f["u1"][1, rho, o] * f["v1"][1, rho, i] for rho in range(2))
        assert abs(W1[o, i] - ref) < 1e-15
    for (o, i) in ((0, 0), (7, 15), (5, 3)):
        ref = float(w["w2_base"][0, o, i]) + sum(f["u2"][1, rho, o] * f["v2"][1, rho, i] for rho in range(2))
        assert abs(W2[o, i] - ref) < 1e-15


# ------------------------------------------------------------------ closed forms the paper states
def test_paper_closed_forms():
    g = _golden()
    assert orc.compression_ratio(4096, 4096, 8, 16) == pytest.approx(g["cr_square_d4096_K8_r16"], rel=1e-14)
    assert 8 / (1 + 2 * 8 * 16 / 4096) == pytest.approx(g["cr_square_d4096_K8_r16"], rel=1e-14)
    assert orc.storage_elements_per_group(4096, 4096, 8, 16) == int(g["storage_elements_d4096_K8_r16"])
    E, G, K, d = 128, 16, 8, 768
    assert (2 * d * E) / orc.routing_flops_per_token(d, G, K) == pytest.approx(g["routing_reduction_E128_G16_K8"], rel=1e-14)


def test_generated_buffers_match_storage_closed_form():
    cfg = ci.small_config(T=8, d=64, d_ff=128, G=2, K=4, r=4, k=2, q=32)
    w = ci.generate(cfg)
    per_group_w1 = w["w1_base"][0].size + (w["u1_q"][:cfg.K].size + w["v1_q"][:cfg.K].size) * 2
    assert per_group_w1 == orc.storage_elements_per_group(cfg.d, cfg.d_ff, cfg.K, cfg.r)
    per_group_w2 = w["w2_base"][0].size + (w["u2_q"][:cfg.K].size + w["v2_q"][:cfg.K].size) * 2
    assert per_group_w2 == orc.storage_elements_per_group(cfg.d_ff, cfg.d, cfg.K, cfg.r)
    fl = ci.flops_per_token(cfg)
    assert fl["router"] == orc.routing_flops_per_token(cfg.d, cfg.G, cfg.K)


def test_zipf_config_loads():
    cfg = ci.scaled(ci.config(2), T=4096)
    w = ci.generate(cfg, with_weights=False)
    cid, *_ = orc.route(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, w["cluster_bias"])
    load = np.bincount(cid, minlength=cfg.G) / cfg.T
    target = 1 / np.arange(1, cfg.G + 1)
    target /= target.sum()
    assert np.abs(load - target).max() < 0.01


# ------------------------------------------------------------------ routing statistics
def test_expert_loads_against_bincount_and_total():
    rng = np.random.default_rng(7)
    E, T, k = 24, 500, 3
    eidx = np.stack([rng.permutation(E)[:k] for _ in range(T)])
    loads = orc.expert_loads(eidx, E)
    assert loads.sum() == T * k
    assert np.array_equal(loads, np.bincount(eidx.reshape(-1), minlength=E))
    assert np.array_equal(orc.expert_loads(np.zeros((0, k), dtype=np.int64), E), np.zeros(E, dtype=np.int64))


def test_load_cv_closed_forms():
    import statistics
    # perfectly balanced -> 0; everything on one of E experts -> sqrt(E - 1)
    assert orc.load_cv([7, 7, 7, 7]) == 0.0
    for E in (2, 8, 64):
        one = [0] * E
        one[3 % E] = 1234
        assert orc.load_cv(one) == pytest.approx(math.sqrt(E - 1), rel=1e-14)
    # population standard deviation over the mean, by another routine; scale invariant
    loads = [3, 9, 4, 0, 11, 5]
    want = statistics.pstdev(loads) / statistics.mean(loads)
    assert orc.load_cv(loads) == pytest.approx(want, rel=1e-14)
    assert orc.load_cv([10 * n for n in loads]) == pytest.approx(want, rel=1e-14)
    assert orc.load_cv([0, 0, 0]) == 0.0


def test_centroid_ema_bruteforce_and_closed_form():
    rng = np.random.default_rng(11)
    E, T, k, d, beta = 6, 40, 2, 5, 0.05
    x = rng.standard_normal((T, d))
    eidx = np.stack([rng.permutation(E - 1)[:k] for _ in range(T)])   # expert E-1 never selected
    mu0 = rng.standard_normal((E, d))
    got = orc.centroid_ema(mu0, x, eidx, beta)
    # scalar loops: a token counts for each of its k experts
    for e in range(E):
        cnt, acc = 0, [0.0] * d
        for t in range(T):
            if e in [int(v) for v in eidx[t]]:
                cnt += 1
                for i in range(d):
                    acc[i] += x[t, i]
        for i in range(d):
            want = mu0[e, i] if cnt == 0 else (1 - beta) * mu0[e, i] + beta * acc[i] / cnt
            assert got[e, i] == pytest.approx(want, rel=1e-13, abs=1e-15)
    assert np.array_equal(got[E - 1], mu0[E - 1])          # no token: unchanged
    # the same batch n times: mu_n = xbar + (1 - beta)^n (mu_0 - xbar)   (Eq. 5 unrolled)
    mu, n = mu0.copy(), 25
    for _ in range(n):
        mu = orc.centroid_ema(mu, x, eidx, beta)
    rows = np.nonzero((eidx == 0).any(axis=1))[0]
    xbar = x[rows].mean(axis=0)
    assert np.allclose(mu[0], xbar + (1 - beta) ** n * (mu0[0] - xbar), rtol=1e-12, atol=1e-14)
    # beta = 1 replaces the centroid by the batch mean
    assert np.allclose(orc.centroid_ema(mu0, x, eidx, 1.0)[0], xbar, rtol=1e-13)


def test_cluster_activity_sequence():
    G, lam = 3, 0.25
    act, idle = np.zeros(G), np.zeros(G, dtype=np.int64)
    steps = [[0, 0, 2], [2], [0, 1, 1], []]
    hits = [[1, 0, 1], [0, 0, 1], [1, 1, 0], [0, 0, 0]]
    want_idle = [[0, 1, 0], [1, 2, 0], [0, 0, 1], [1, 1, 2]]
    a = [0.0] * G
    for cid, h, wi in zip(steps, hits, want_idle):
        act, idle, counts = orc.cluster_activity(act, idle, np.array(cid, dtype=np.int64), G, lam)
        a = [(1 - lam) * a[g] + lam * h[g] for g in range(G)]
        assert np.allclose(act, a, rtol=1e-15)
        assert list(idle) == wi
        assert list(counts) == [cid.count(g) for g in range(G)]
    # a cluster hit every step tends to 1: act_n = 1 - (1 - lam)^n
    act = np.zeros(1)
    idle = np.zeros(1, dtype=np.int64)
    for n in range(1, 9):
        act, idle, _ = orc.cluster_activity(act, idle, np.array([0]), 1, lam)
        assert act[0] == pytest.approx(1 - (1 - lam) ** n, rel=1e-14)


# ------------------------------------------------------------------ compression (Sec. 3.2, 3.4)
def test_base_mean_exact_and_within_half_ulp():
    # integers: every sum and the division by K = 4 are exact in FP16, so Eq. 6 is hand-checkable
    W = np.zeros((8, 2, 3), dtype=np.float16)
    for e in range(8):
        W[e] = 4 * (e % 4) + np.arange(6).reshape(2, 3) * 8
    base = orc.base_mean(W, 2, 4)
    want = 6.0 + np.arange(6).reshape(2, 3) * 8.0          # mean of 0, 4, 8, 12 is 6
    assert np.array_equal(base[0].astype(np.float64), want) and np.array_equal(base[1], base[0])
    # random values: the FP16 result is the FP64 mean to within one rounding of the result
    rng = np.random.default_rng(3)
    W = rng.standard_normal((6, 16, 32)).astype(np.float16)
    base = orc.base_mean(W, 2, 3).astype(np.float64)
    exact = W.astype(np.float64).reshape(2, 3, 16, 32).mean(axis=1)
    ulp = np.spacing(np.abs(exact).astype(np.float16)).astype(np.float64)
    assert np.all(np.abs(base - exact) <= 0.5 * ulp + 1e-6 * ulp + 2.0 ** -24 * np.abs(exact) * 4)


def test_truncated_svd_is_eckart_young_optimum():
    rng = np.random.default_rng(5)
    out_d, in_d, r = 24, 40, 5
    delta = rng.standard_normal((out_d, in_d))
    U, V, err, sv = orc.truncated_svd_factors(delta, r)
    # the error is the tail of the spectrum, computed by another routine (eigenvalues of D D^T)
    ev = np.sort(np.linalg.eigvalsh(delta @ delta.T))[::-1]
    assert err == pytest.approx(math.sqrt(ev[r:].sum()), rel=1e-10)
    assert np.linalg.norm(delta - U @ V) == pytest.approx(err, rel=1e-10)
    # no other rank-r product does better: random rank-r factors and a perturbed optimum
    for _ in range(20):
        A, B = rng.standard_normal((out_d, r)), rng.standard_normal((r, in_d))
        coef = np.linalg.lstsq(A, delta, rcond=None)[0]                   # best V for this U
        assert np.linalg.norm(delta - A @ coef) >= err * (1 - 1e-12)
        assert np.linalg.norm(delta - (U + 1e-3 * A) @ V) >= err * (1 - 1e-12)
    # an exactly rank-r matrix is reproduced
    low = rng.standard_normal((out_d, r)) @ rng.standard_normal((r, in_d))
    U2, V2, err2, _ = orc.truncated_svd_factors(low, r)
    assert err2 <= 1e-12 * np.linalg.norm(low) and np.allclose(U2 @ V2, low, atol=1e-12)
    # rows of V are orthonormal, columns of U orthogonal with the singular values as norms
    assert np.allclose(V @ V.T, np.eye(r), atol=1e-12)
    assert np.allclose(np.linalg.norm(U, axis=0), sv[:r], rtol=1e-12)


def test_quantiser_fp32_table_and_agreement_with_fp64_form():
    # one group of 8, absmax 7 -> scale 1: codes are the rounded values, ties to even
    w = np.array([[7.0, -7.0, 0.5, 1.5, 2.5, -0.5, -1.5, 3.49]], dtype=np.float32)
    packed, scale = orc.quantize_int4_f32(w, 8)
    assert scale.tolist() == [[1.0]]
    assert orc.unpack_int4(packed).tolist() == [[7, -7, 0, 2, 2, 0, -2, 3]]
    # absmax 3.5 -> scale 0.5: value = code / 2; all-zero group -> scale 0, codes 0
    w = np.array([[3.5, -3.5, 1.0, 0.25, 0, 0, 0, 0], [0] * 8], dtype=np.float32)
    packed, scale = orc.quantize_int4_f32(w, 8)
    assert scale[:, 0].tolist() == [0.5, 0.0]
    assert orc.unpack_int4(packed).tolist() == [[7, -7, 2, 0, 0, 0, 0, 0], [0] * 8]
    # dequantised error is at most half a step; same codes as the float64 form used for the
    # synthetic inputs wherever no value sits within 1e-6 of a rounding boundary
    rng = np.random.default_rng(9)
    w = (rng.standard_normal((5, 64)) * 0.02).astype(np.float32)
    packed, scale = orc.quantize_int4_f32(w, 16)
    deq = orc.dequant_int4(packed, scale, 16)
    step = np.repeat(scale.astype(np.float64), 16, axis=-1)
    assert np.all(np.abs(deq - w) <= 0.5 * step * (1 + 1e-6) + 1e-12)
    p64, s64 = ci.quantize_int4(w, 16)
    assert np.array_equal(scale, s64)
    frac = np.abs(w / np.where(step > 0, step, 1)) % 1.0
    safe = np.abs(frac - 0.5) > 1e-4
    assert np.array_equal(orc.unpack_int4(packed)[safe], orc.unpack_int4(p64)[safe])


def test_cosine_gate_and_reconstruction_error_closed_forms():
    a = np.array([[1.0, 0.0], [0.0, 2.0]])
    assert orc.cosine_to_base(a, 3 * a) == pytest.approx(1.0)
    assert orc.cosine_to_base(a, -a) == pytest.approx(-1.0)
    assert orc.cosine_to_base(np.array([[1.0, 0.0]]), np.array([[0.0, 5.0]])) == 0.0
    assert orc.cosine_to_base(np.zeros((2, 2)), a) == 0.0
    assert orc.cosine_to_base(np.array([[1.0, 1.0]]), np.array([[1.0, 0.0]])) == pytest.approx(1 / math.sqrt(2))
    rng = np.random.default_rng(2)
    W = rng.standard_normal((6, 9))
    base = rng.standard_normal((6, 9))
    U, V = rng.standard_normal((6, 2)), rng.standard_normal((2, 9))
    # zero factors: the error is the residual's share of W; exact factors: zero
    assert orc.reconstruction_error(W, base, np.zeros((6, 2)), np.zeros((2, 9))) == pytest.approx(
        np.linalg.norm(W - base) / np.linalg.norm(W), rel=1e-14)
    assert orc.reconstruction_error(base + U @ V, base, U, V) <= 1e-15
    assert orc.residual(W.astype(np.float16), base.astype(np.float16)).dtype == np.float64


# ------------------------------------------------------------------ routing variants (Sec. 3.3, 3.5)
def test_route_multi_reduces_to_route():
    cfg = ci.small_config("rm", T=80, d=32, d_ff=32, G=4, K=4, r=4, k=2, q=8, seed=21)
    w = ci.generate(cfg)
    cid, eidx, gate, _, _ = orc.route(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k)
    cids, eidx2, gate2, p = orc.route_multi(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k)
    assert np.array_equal(cids[:, 0], cid) and np.array_equal(eidx2[:, 0], eidx)
    assert np.allclose(gate2[:, 0], gate, rtol=1e-14)
    assert np.allclose(p.sum(axis=1), 1.0, rtol=1e-14)


@pytest.mark.parametrize("top_g,tau,scale", [(2, 1.0, False), (3, 0.7, True), (1, 0.7, True), (4, 2.0, False)])
def test_route_multi_bruteforce(top_g, tau, scale):
    cfg = ci.small_config("rmb", T=30, d=16, d_ff=32, G=4, K=3, r=4, k=2, q=8, seed=22)
    w = ci.generate(cfg)
    x = w["x"].astype(np.float64)
    rc, re = w["router_cluster"].astype(np.float64), w["router_expert"].astype(np.float64)
    cids, eidx, gate, _ = orc.route_multi(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, top_g, tau,
                                          scale)
    for t in range(cfg.T):
        z = [sum(rc[g][i] * x[t][i] for i in range(cfg.d)) for g in range(cfg.G)]
        pz = [math.exp(v / tau) for v in z]
        pz = [v / sum(pz) for v in pz]
        sel = sorted(range(cfg.G), key=lambda g: (-z[g], g))[:top_g]
        assert list(cids[t]) == sel
        wsum = sum(pz[g] for g in sel)
        got_total = 0.0
        for a, c in enumerate(sel):
            l = [sum(re[c * cfg.K + j][i] * x[t][i] for i in range(cfg.d)) for j in range(cfg.K)]
            top = sorted(range(cfg.K), key=lambda j: (-l[j], j))[:cfg.k]
            assert list(eidx[t, a]) == [c * cfg.K + j for j in top]
            ex = [math.exp(l[j] / tau) for j in top]
            wa = pz[c] if scale else pz[c] / wsum
            for jj in range(cfg.k):
                assert gate[t, a, jj] == pytest.approx(wa * ex[jj] / sum(ex), rel=1e-12)
            got_total += float(gate[t, a].sum())
        assert got_total == pytest.approx(wsum if scale else 1.0, rel=1e-12)


def test_route_multi_temperature_and_full_fanout():
    cfg = ci.small_config("rmt", T=50, d=32, d_ff=32, G=3, K=4, r=4, k=2, q=8, seed=23)
    w = ci.generate(cfg)
    a1 = orc.route_multi(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, 2, 1.0)
    a2 = orc.route_multi(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, 2, 1e6)
    # the temperature never changes which clusters / experts are selected; a very large one
    # flattens the weights: 1 / top_g per cluster, 1 / k inside it
    assert np.array_equal(a1[0], a2[0]) and np.array_equal(a1[1], a2[1])
    assert np.allclose(a2[2], 1.0 / (2 * cfg.k), rtol=1e-4)
    # all clusters selected and scaled by their probability: the weights sum to one
    full = orc.route_multi(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, cfg.G, 0.7, True)
    assert np.allclose(full[2].sum(axis=(1, 2)), 1.0, rtol=1e-13)


def test_forward_multi_is_sum_of_selected_dense_ffns():
    cfg = ci.small_config("fm", T=6, d=16, d_ff=32, G=3, K=2, r=4, k=1, q=8, seed=24)
    w = ci.generate(cfg)
    out = orc.forward_naive_multi(w, w["x"], cfg.K, cfg.k, cfg.q, top_g=2, temperature=0.7, scale_by_cluster_prob=True)
    f = None
    for t in range(cfg.T):
        acc = np.zeros(cfg.d)
        for a in range(2):
            e = int(out["expert_idx"][t, a, 0])
            W1, W2 = orc.expert_weights(w, e, cfg.K, cfg.q, f)
            h = W1 @ w["x"][t].astype(np.float64)
            acc += out["gate"][t, a, 0] * (W2 @ np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in h]))
        assert np.allclose(out["y"][t], acc, rtol=1e-12, atol=1e-14)


def test_ffn_dense_equals_compressed_form_with_exact_factors():
    # dense experts built FROM a compressed layer reproduce that layer's output exactly
    cfg = ci.small_config("fd", T=12, d=16, d_ff=32, G=2, K=2, r=4, k=2, q=8, seed=25)
    w = ci.generate(cfg)
    W1 = np.stack([orc.expert_weights(w, e, cfg.K, cfg.q)[0] for e in range(cfg.E)])
    W2 = np.stack([orc.expert_weights(w, e, cfg.K, cfg.q)[1] for e in range(cfg.E)])
    ref = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    y = orc.ffn_dense(W1, W2, w["x"], ref["expert_idx"], ref["gate"])
    assert np.allclose(y, ref["y"], rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ backward pass (Sec. 3.5)
def test_gelu_grad_is_the_derivative():
    u = np.linspace(-4, 4, 41)
    eps = 1e-6
    num = (orc.gelu(u + eps) - orc.gelu(u - eps)) / (2 * eps)
    assert np.allclose(orc.gelu_grad(u), num, rtol=1e-8, atol=1e-9)
    assert orc.gelu_grad(0.0) == pytest.approx(0.5) and orc.gelu_grad(10.0) == pytest.approx(1.0, abs=1e-12)


def test_backward_matches_central_differences():
    """L = sum(dy * y) with the selection frozen and the gates recomputed from the logits, written
    here with scalar loops and math.erf; every gradient the oracle returns against central
    differences of that function."""
    cfg = ci.small_config("bw", T=4, d=6, d_ff=8, G=2, K=2, r=2, k=2, q=2, seed=31)
    w = ci.generate(cfg)
    E, T, d, f_, r, k, K = cfg.E, cfg.T, cfg.d, cfg.d_ff, cfg.r, cfg.k, cfg.K
    ref = orc.forward_naive(w, w["x"], K, k, cfg.q)
    eidx = ref["expert_idx"]
    rng = np.random.default_rng(32)
    dy = rng.standard_normal((T, d))
    fac = {n: orc.dequant_int4(w[n + "_q"], w[n + "_s"], cfg.q) for n in ("v1", "u1", "v2", "u2")}
    P = dict(x=w["x"].astype(np.float64), re=w["router_expert"].astype(np.float64),
             b1=w["w1_base"].astype(np.float64), b2=w["w2_base"].astype(np.float64), **fac)

    def loss(P):
        tot = 0.0
        for t in range(T):
            ls = [sum(P["re"][eidx[t, j]][i] * P["x"][t][i] for i in range(d)) for j in range(k)]
            m = max(ls)
            ex = [math.exp(v - m) for v in ls]
            g = [v / sum(ex) for v in ex]
            for j in range(k):
                e = int(eidx[t, j]); c = e // K
                W1 = P["b1"][c] + P["u1"][e].T @ P["v1"][e]
                W2 = P["b2"][c] + P["u2"][e].T @ P["v2"][e]
                h = W1 @ P["x"][t]
                a = np.array([0.5 * v * (1 + math.erf(v / math.sqrt(2))) for v in h])
                tot += g[j] * float(dy[t] @ (W2 @ a))
        return tot

    got = orc.backward_naive(w, w["x"], dy, eidx, ref["gate"], K, cfg.q)
    names = dict(x="dx", re="d_router_expert", b1="dw1_base", b2="dw2_base", u1="du1", v1="dv1", u2="du2", v2="dv2")
    eps = 1e-6
    for pn, gn in names.items():
        arr = P[pn]
        for _ in range(12):
            idx = tuple(int(rng.integers(0, s)) for s in arr.shape)
            old = arr[idx]
            arr[idx] = old + eps
            lp = loss(P)
            arr[idx] = old - eps
            lm = loss(P)
            arr[idx] = old
            num = (lp - lm) / (2 * eps)
            assert got[gn][idx] == pytest.approx(num, rel=2e-6, abs=2e-8), (pn, idx)
    # experts that no token selected get no gradient; the base gradient is the sum over its experts
    unused = [e for e in range(E) if e not in set(eidx.reshape(-1).tolist())]
    for e in unused:
        assert not got["du1"][e].any() and not got["d_router_expert"][e].any()


def test_backward_sampled_is_a_slice_of_the_full_backward():
    """The token-wise / hidden-unit-wise form used at sizes where the dense per-expert gradients
    do not fit must return exactly the corresponding slices of backward_naive, which the
    central differences above pin."""
    cfg = ci.small_config("bws", T=70, d=16, d_ff=24, G=3, K=3, r=4, k=2, q=4, seed=33)
    w = ci.generate(cfg)
    ref = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    rng = np.random.default_rng(34)
    dy = rng.standard_normal((cfg.T, cfg.d))
    full = orc.backward_naive(w, w["x"], dy, ref["expert_idx"], ref["gate"], cfg.K, cfg.q)
    tokens = np.array([0, 3, 17, 42, 69])
    hidden = np.array([1, 5, 23])
    got = orc.backward_sampled(w, w["x"], dy, ref["expert_idx"], ref["gate"], cfg.K, cfg.q, tokens, hidden)
    assert np.allclose(got["dx"], full["dx"][tokens], rtol=1e-11, atol=1e-13)
    assert np.allclose(got["dgate_logits"], full["dgate_logits"][tokens], rtol=1e-11, atol=1e-13)
    assert np.allclose(got["dw1_base"], full["dw1_base"][:, hidden, :], rtol=1e-11, atol=1e-13)
    assert np.allclose(got["dw2_base"], full["dw2_base"][:, :, hidden], rtol=1e-11, atol=1e-13)
    assert np.allclose(got["du1"], full["du1"][:, :, hidden], rtol=1e-11, atol=1e-13)
    assert np.allclose(got["dv2"], full["dv2"][:, :, hidden], rtol=1e-11, atol=1e-13)
    assert np.abs(full["dgate_logits"]).max() > 1e-3 and np.abs(full["du1"]).max() > 1e-3


# ------------------------------------------------------------------ the bars themselves
def test_error_metrics_hand_values():
    # y_ref = (3, 4), y = (3, 5): one element off by 1; RMS(y_ref) = sqrt((9 + 16) / 2) = sqrt(12.5),
    # sum |y_ref| = 7.  RMS(y) would be sqrt(17) and sum |y| = 8: a metric normalised by y instead
    # of y_ref, or by a plain mean of |y_ref| (3.5), gives other numbers.
    m = orc.error_metrics(np.array([3.0, 5.0]), np.array([3.0, 4.0]))
    assert m["max_over_rms"] == pytest.approx(1.0 / math.sqrt(12.5), rel=1e-15)
    assert m["mean_rel"] == pytest.approx(1.0 / 7.0, rel=1e-15)
    assert m["rms"] == pytest.approx(math.sqrt(12.5), rel=1e-15)
    # two dimensions, signs, and an FP16 input: the maximum runs over every element, the RMS and
    # the sums over the whole array (not per row, not per column)
    y_ref = np.array([[1.0, -2.0, 2.0], [-4.0, 0.0, 0.0]])
    y = np.array([[1.0, -2.5, 2.0], [-4.0, 0.25, 0.0]], dtype=np.float16)
    m = orc.error_metrics(y, y_ref)
    assert m["max_over_rms"] == pytest.approx(0.5 / math.sqrt(25.0 / 6.0), rel=1e-15)
    assert m["mean_rel"] == pytest.approx(0.75 / 9.0, rel=1e-15)
    # identical arrays: zero; empty arrays: zero, no division
    assert orc.error_metrics(y_ref, y_ref)["max_over_rms"] == 0.0 and orc.error_metrics(y_ref, y_ref)["mean_rel"] == 0.0
    e = orc.error_metrics(np.zeros((0, 4)), np.zeros((0, 4)))
    assert e["max_over_rms"] == 0.0 and e["mean_rel"] == 0.0


def test_error_metrics_cases_the_bars_must_reject():
    # the bars of the GPU tests: max / RMS <= 1e-2 and mean-rel <= 2e-3
    rng = np.random.default_rng(17)
    y_ref = rng.standard_normal((64, 32))
    rms = math.sqrt(float((y_ref ** 2).mean()))
    # one element off by 2 % of the RMS: only the maximum bar trips
    y = y_ref.copy()
    y[5, 7] += 0.02 * rms
    m = orc.error_metrics(y, y_ref)
    assert m["max_over_rms"] == pytest.approx(0.02, rel=1e-12) and m["max_over_rms"] > 1e-2 and m["mean_rel"] < 2e-3
    # every element off by 0.5 % of its own size: only the mean-relative bar trips
    y = y_ref * 1.005
    m = orc.error_metrics(y, y_ref)
    assert m["mean_rel"] == pytest.approx(0.005, rel=1e-9) and m["mean_rel"] > 2e-3
    assert m["max_over_rms"] == pytest.approx(0.005 * np.abs(y_ref).max() / rms, rel=1e-9)
    # FP16 rounding of the reference passes both, a dropped 10 % term fails both
    m = orc.error_metrics(y_ref.astype(np.float16), y_ref)
    assert m["max_over_rms"] < 1e-2 and m["mean_rel"] < 2e-3
    m = orc.error_metrics(0.9 * y_ref, y_ref)
    assert m["max_over_rms"] > 1e-2 and m["mean_rel"] > 2e-3


def test_residual_exact_case_and_sign():
    # Eq. 7's residual is W_e - W_base (not the reverse), in float64, exact on FP16 inputs
    W_e = np.array([[1.5, -2.0, 0.0]], dtype=np.float16)
    base = np.array([[0.25, 1.0, -3.0]], dtype=np.float16)
    d = orc.residual(W_e, base)
    assert d.dtype == np.float64 and d.tolist() == [[1.25, -3.0, 3.0]]
    # base + residual gives the expert back exactly, for values whose FP16 sum would round
    rng = np.random.default_rng(23)
    W_e = rng.standard_normal((8, 8)).astype(np.float16)
    base = (rng.standard_normal((8, 8)) * 1e-3).astype(np.float16)
    assert np.array_equal(base.astype(np.float64) + orc.residual(W_e, base), W_e.astype(np.float64))


def test_base_and_quantiser_meet_their_definitions_in_fp64():
    """Eq. 6 and the quantiser of Sec. 3.4 written out in FP64, independent of the order and
    precision in which base_mean / quantize_int4_f32 take their steps: the stored base is a
    nearest FP16 neighbour of the exact mean, the scale the FP16 rounding of absmax / 7, every
    code the integer nearest to w / scale (either neighbour at a tie), clipped to [-7, 7]."""
    rng = np.random.default_rng(31)
    G, K = 3, 5
    W = rng.standard_normal((G * K, 12, 20)).astype(np.float16)
    base = orc.base_mean(W, G, K).astype(np.float64)
    exact = W.astype(np.float64).reshape(G, K, 12, 20).sum(axis=1) / K
    # the two FP16 neighbours that bracket the exact mean
    f = exact.astype(np.float16).astype(np.float64)
    below = np.where(f <= exact, f, np.nextafter(exact.astype(np.float16), np.float16(-np.inf)).astype(np.float64))
    above = np.where(f >= exact, f, np.nextafter(exact.astype(np.float16), np.float16(np.inf)).astype(np.float64))
    assert np.all(below <= exact) and np.all(exact <= above)
    nearest = np.where(exact - below <= above - exact, below, above)
    tie = np.abs((exact - below) - (above - exact)) <= 2.0 ** -24 * np.abs(exact) * 8   # FP32 sum rounding
    assert np.all((base == nearest) | (tie & ((base == below) | (base == above))))
    # and it is the correctly rounded (ties to even) FP16 value of the exact mean almost everywhere:
    # only the double rounding through FP32 can differ, next to a tie
    assert np.mean(base == f) > 0.999

    q = 8
    w = (rng.standard_normal((7, 64)) * 0.03).astype(np.float32)
    w[2, :q] = 0.0
    packed, scale = orc.quantize_int4_f32(w, q)
    codes = orc.unpack_int4(packed).astype(np.float64)
    w64 = w.astype(np.float64).reshape(7, 64 // q, q)
    absmax = np.abs(w64).max(axis=-1)
    assert np.array_equal(scale, (absmax / 7.0).astype(np.float16))          # FP64 quotient, rounded once
    s = scale.astype(np.float64)
    c = codes.reshape(7, 64 // q, q)
    assert np.all(np.abs(c) <= 7)
    live = s > 0
    ratio = w64[live] / s[live][:, None]
    want = np.clip(ratio, -7.0, 7.0)
    # nearest integer to the clipped ratio; at a tie (within FP32 rounding of the division) either neighbour
    assert np.all(np.abs(c[live] - want) <= 0.5 + 1e-6)
    assert np.all(c[~live] == 0)
    # the reconstruction w ~ scale * code is within half a step wherever no clipping took place
    inside = np.abs(ratio) <= 7.0
    assert np.all(np.abs(s[live][:, None] * c[live] - w64[live])[inside] <= 0.5 * np.broadcast_to(s[live][:, None], ratio.shape)[inside] * (1 + 1e-6))


def test_route_nan_logits_rank_last_and_slots_stay_distinct():
    # reading for non-finite inputs: NaN ranks below every number, lowest index among equals
    G, K, k, d = 3, 4, 3, 8
    rng = np.random.default_rng(77)
    rc = rng.standard_normal((G, d)).astype(np.float16)
    re = rng.standard_normal((G * K, d)).astype(np.float16)
    x = rng.standard_normal((4, d)).astype(np.float16)
    x[0, :] = np.float16(np.nan)                       # every logit of token 0 is NaN
    with np.errstate(invalid="ignore"):
        cid, eidx, gate, z, l = orc.route(x, rc, re, K, k)
    assert cid[0] == 0 and eidx[0].tolist() == [0, 1, 2]
    # one NaN router row: that expert is chosen only when nothing else is left
    re2 = re.copy()
    c1 = int(cid[1])
    best = int(eidx[1, 0])
    re2[best, 0] = np.float16(np.nan)                  # the former winner of token 1 now has a NaN logit
    with np.errstate(invalid="ignore"):
        cid2, eidx2, _, _, l2 = orc.route(x[1:2], rc, re2, K, k)
    assert cid2[0] == c1 and best not in eidx2[0].tolist()
    assert eidx2[0].tolist() == [e for e in eidx[1].tolist() if e != best] + [e for e in range(c1 * K, c1 * K + K)
                                                                           if e not in eidx[1].tolist()][:1]
    # k = K with one NaN: all K experts are named once, the NaN one last
    with np.errstate(invalid="ignore"):
        _, eidx3, _, _, _ = orc.route(x[1:2], rc, re2, K, K)
    assert sorted(eidx3[0].tolist()) == list(range(c1 * K, c1 * K + K)) and eidx3[0, -1] == best
    # the variants follow the same rule for clusters
    with np.errstate(invalid="ignore"):
        cids, e4, _, _ = orc.route_multi(x[:1], rc, re, K, k, top_g=2)
    assert cids[0].tolist() == [0, 1] and e4[0].tolist() == [[0, 1, 2], [4, 5, 6]]
