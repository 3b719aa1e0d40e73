"""GPU parity: the HIP library (through the C ABI) against the FP64 oracle.

Bars: routing indices, permutation and offsets bit-exact; gates to 1e-5; layer output
max|y - y_ref| <= 1e-2 * RMS(y_ref) and sum|y - y_ref| / sum|y_ref| <= 2e-3.
Intermediates (y_base_sorted, s_down) use the same max/RMS bar.
"""
import numpy as np
import pytest

import cmoe_inputs as ci
from oracle import cmoe_oracle as orc

pytestmark = pytest.mark.gpu

MAX_OVER_RMS = 1e-2
MEAN_REL = 2e-3


def _layer(cfg, w, T_max=None, pack=True):
    import paper_2510_02345_amd as cm
    return cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, T_max if T_max is not None else cfg.T,
                    pack=pack)


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _sync():
    import torch
    torch.cuda.synchronize()


def _check_y(y, y_ref, what):
    m = orc.error_metrics(y, y_ref)
    print(f"{what}: max/rms={m['max_over_rms']:.3e} mean_rel={m['mean_rel']:.3e}", flush=True)
    assert np.all(np.isfinite(np.asarray(y, dtype=np.float64))), what
    assert m["max_over_rms"] <= MAX_OVER_RMS, (what, m)
    assert m["mean_rel"] <= MEAN_REL, (what, m)
    return m


def _stepwise(cfg, w=None, pack=True, drop_canonical=False):
    """Each entry point on its own against the oracle, then cmoe_forward."""
    print(f"case {cfg} pack={pack} drop_canonical={drop_canonical}", flush=True)
    w = w if w is not None else ci.generate(cfg)
    ref = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    rw = orc.ffn_rewrite(w, w["x"], ref["perm"], ref["offsets"], ref["expert_idx"], ref["gate"], cfg.K, cfg.q)
    layer = _layer(cfg, w, pack=pack)
    if drop_canonical:
        layer.drop_canonical_bases()
    x = _dev(w["x"])

    cid, eidx, gate = layer.route(x)
    _sync()
    assert np.array_equal(cid.cpu().numpy(), ref["cluster_id"])
    assert np.array_equal(eidx.cpu().numpy(), ref["expert_idx"])
    assert np.allclose(gate.cpu().numpy(), ref["gate"], rtol=1e-5, atol=1e-6)

    # each later step is fed the oracle's inputs, so an upstream error cannot hide
    perm, inv, offsets = layer.permute(_dev(ref["cluster_id"]))
    _sync()
    assert np.array_equal(offsets.cpu().numpy(), ref["offsets"])
    assert np.array_equal(perm.cpu().numpy(), ref["perm"])
    assert np.array_equal(inv.cpu().numpy(), ref["inv_perm"])

    g32 = _dev(ref["gate"].astype(np.float32))
    yb, s = layer.ffn_forward(x, _dev(ref["perm"]), _dev(ref["offsets"]), _dev(ref["expert_idx"]), g32)
    _sync()
    if cfg.T:
        _check_y(yb.cpu().numpy(), rw["y_base_sorted"], "y_base_sorted")
        _check_y(s.cpu().numpy(), rw["s"], "s_down")

    yb_ref = _dev(rw["y_base_sorted"].astype(np.float16))
    s_ref = _dev(rw["s"].astype(np.float32))
    y = layer.combine(yb_ref, s_ref, _dev(ref["perm"]), _dev(ref["inv_perm"]), _dev(ref["offsets"]),
                      _dev(ref["expert_idx"]), g32)
    _sync()
    if cfg.T:
        _check_y(y.cpu().numpy(), ref["y"], "combine")

    out = layer.forward(x)
    _sync()
    assert np.array_equal(out["cluster_id"].cpu().numpy(), ref["cluster_id"])
    assert np.array_equal(out["expert_idx"].cpu().numpy(), ref["expert_idx"])
    assert np.array_equal(out["perm"].cpu().numpy(), ref["perm"])
    assert np.array_equal(out["inv_perm"].cpu().numpy(), ref["inv_perm"])
    assert np.array_equal(out["offsets"].cpu().numpy(), ref["offsets"])
    m = None
    if cfg.T:
        m = _check_y(out["y"].cpu().numpy(), ref["y"], "forward")
    layer.close()
    return m, ref


SMALL = [
    # several row tiles and a ragged tail in every cluster; K*r = 32
    ci.small_config("ragged", T=777, d=128, d_ff=384, G=3, K=4, r=8, k=2, q=32, seed=41),
    # K*r = 16 < 32 (padded rank panel), k = 1
    ci.small_config("padded", T=300, d=64, d_ff=192, G=2, K=4, r=4, k=1, q=8, seed=42),
    # one cluster, r = 32, all K selected
    ci.small_config("flat", T=130, d=192, d_ff=256, G=1, K=3, r=32, k=3, q=64, seed=43),
    # many clusters, few tokens: most row tiles nearly empty, some clusters empty
    ci.small_config("sparse", T=19, d=64, d_ff=128, G=16, K=2, r=16, k=2, q=16, seed=44),
    # k = 4 of K = 8, r = 4: two experts share an 8-row group of the rank panel
    ci.small_config("k4", T=257, d=128, d_ff=256, G=2, K=8, r=4, k=4, q=32, seed=45),
    ci.small_config("one", T=1, d=64, d_ff=64, G=2, K=2, r=8, k=2, q=8, seed=46),
    # more than 128 router rows and more than 64 expert slots: wavefront-per-token router,
    # no secondary expert sort
    ci.small_config("manyexperts", T=400, d=64, d_ff=128, G=20, K=8, r=4, k=2, q=8, seed=51),
    # weight-streaming path, several 16-token passes per cluster, d_ff not a multiple of the
    # 2048-column chunk of the per-expert kernel, four experts per token
    ci.small_config("stream_passes", T=250, d=128, d_ff=2176, G=2, K=8, r=4, k=4, q=32, seed=52),
    # weight-streaming path with k * r = 256 (four groups of 64 rank values per token)
    ci.small_config("stream_k8", T=40, d=64, d_ff=128, G=1, K=8, r=32, k=8, q=16, seed=53),
    # large-T path with K * r = 256: factor panels read from global memory, separate combine
    ci.small_config("wide_rank", T=600, d=128, d_ff=256, G=2, K=8, r=32, k=2, q=32, seed=54),
    # the largest supported rank panel, K * r = 512
    ci.small_config("max_rank", T=300, d=64, d_ff=128, G=1, K=16, r=32, k=2, q=8, seed=55),
    # exactly at and just above the switch between the two paths
    ci.small_config("switch_256", T=256, d=64, d_ff=192, G=3, K=4, r=8, k=2, q=8, seed=56),
    # the widest supported model dimension and cluster count, both paths
    ci.small_config("max_d_big", T=300, d=8192, d_ff=128, G=64, K=2, r=4, k=2, q=128, seed=57),
    ci.small_config("max_d_stream", T=50, d=8192, d_ff=128, G=64, K=2, r=4, k=2, q=128, seed=58),
    # k = 8 of K = 32 experts per cluster (the largest top-k), large-T path
    ci.small_config("k8_of_32", T=400, d=64, d_ff=128, G=2, K=32, r=4, k=8, q=8, seed=59),
]


@pytest.mark.parametrize("cfg", SMALL, ids=[c.name for c in SMALL])
def test_small_shapes_every_entry_point(cfg):
    _stepwise(cfg)


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[7]], ids=lambda c: c.name)
def test_pre_activations_far_outside_the_gelu_polynomial_range(cfg):
    # x scaled by 6: the pre-activations have a standard deviation of about 6, so most of them
    # lie beyond the interval on which the kernels evaluate Phi by a polynomial, on both sides
    # (the logits and their gaps scale with x, the routing decisions stay the generator's)
    w = ci.generate(cfg)
    w["x"] = (w["x"].astype(np.float32) * 6.0).astype(np.float16)
    h = w["w1_base"][0].astype(np.float64) @ w["x"][: min(cfg.T, 64)].astype(np.float64).T
    assert np.mean(np.abs(h) > 3.75) > 0.4
    _stepwise(cfg, w=w)


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[7]], ids=lambda c: c.name)
def test_nan_in_a_base_weight_reaches_exactly_the_outputs_it_feeds(cfg):
    # one NaN in row 5 of W1_base of cluster 0: hidden unit 5 of every token of that cluster is
    # NaN before and after the activation, so all of those tokens' outputs are NaN and no
    # other token's (the activation must not turn a NaN into a number)
    w = ci.generate(cfg)
    w1 = w["w1_base"].copy()
    w1[0, 5, 7] = np.nan
    w = dict(w, w1_base=w1)
    with np.errstate(invalid="ignore"):
        ref = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    hit = ref["cluster_id"] == 0
    assert hit.any() and not hit.all()
    assert np.all(np.isnan(ref["y"][hit])) and np.all(np.isfinite(ref["y"][~hit]))
    layer = _layer(cfg, w)
    y = layer.forward(_dev(w["x"]))["y"].cpu().numpy()
    _sync()
    assert np.all(np.isnan(y[hit]))
    _check_y(y[~hit], ref["y"][~hit], "tokens of the other clusters")
    layer.close()


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[9], SMALL[12], SMALL[7], SMALL[13]], ids=lambda c: c.name)
def test_canonical_bases_without_the_packed_copy(cfg):
    # the layer reads the caller's row-major bases when no packed copy is given (both paths)
    _stepwise(cfg, pack=False)


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[7], SMALL[8], SMALL[12], SMALL[13]], ids=lambda c: c.name)
def test_packed_copy_as_the_only_resident_bases(cfg):
    # after packing, w1_base / w2_base are freed and passed as NULL: both paths (and every
    # entry point) read the bases from the packed buffer alone
    _stepwise(cfg, drop_canonical=True)


def test_resident_weight_bytes_with_one_copy_of_the_bases():
    # C1: bases once (packed) + INT4 factors + FP16 panels + routers
    cfg = ci.config(1)
    w = ci.generate(cfg)
    layer = _layer(cfg, w)
    both = layer.resident_weight_bytes()
    layer.drop_canonical_bases()
    one = layer.resident_weight_bytes()
    bases = 2 * 2 * cfg.G * cfg.d * cfg.d_ff
    assert both - one == bases
    E, L = cfg.G * cfg.K, cfg.d + cfg.d_ff
    factors = 2 * E * cfg.r * (L // 2 + 2 * (L // cfg.q))
    panels = 4 * cfg.G * 32 * ((cfg.K * cfg.r + 31) // 32) * L
    routers = 2 * (cfg.G + E) * cfg.d
    assert abs(one - (bases + factors + panels + routers)) <= 4096
    ref = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    out = layer.forward(_dev(w["x"]))
    _sync()
    _check_y(out["y"].cpu().numpy(), ref["y"], "forward, packed bases only")
    layer.close()


def test_packed_and_canonical_bases_give_identical_outputs():
    # the packed copy only changes where the operand tiles are fetched from: same products,
    # same order, bit-identical y
    import torch
    cfg = ci.config(1)
    w = ci.generate(cfg)
    x = _dev(w["x"])
    ys = []
    for pack in (True, False):
        layer = _layer(cfg, w, pack=pack)
        ys.append(layer.forward(x)["y"].clone())
        _sync()
        layer.close()
    assert torch.equal(ys[0], ys[1])
    # the same on the weight-streaming path
    cfg = SMALL[7]
    w = ci.generate(cfg)
    x = _dev(w["x"])
    ys = []
    for pack in (True, False):
        layer = _layer(cfg, w, pack=pack)
        ys.append(layer.forward(x)["y"].clone())
        _sync()
        layer.close()
    assert torch.equal(ys[0], ys[1])


def test_empty_input_is_a_noop():
    cfg = ci.small_config("empty", T=0, d=64, d_ff=128, G=2, K=2, r=8, k=2, q=8, seed=47)
    _stepwise(cfg)


def test_empty_cluster_weights_never_read():
    # all tokens forced into cluster 1 by the bias; the weights of cluster 0 are NaN / garbage
    cfg = ci.small_config("onecluster", T=200, d=64, d_ff=128, G=2, K=4, r=8, k=2, q=8, seed=48)
    w = ci.generate(cfg)
    w["cluster_bias"] = np.array([-100.0, 100.0], dtype=np.float32)
    for n in ("w1_base", "w2_base"):
        w[n][0] = np.float16(np.nan)
    for n in ("v1", "u1", "v2", "u2"):
        w[n + "_s"][:cfg.K] = np.float16(np.nan)
    _stepwise(cfg, w)


def test_residual_path_is_live():
    # factors ten times larger: the residual terms are far above the tolerance, so a
    # path that dropped or mis-indexed them would fail here
    cfg = ci.small_config("bigres", T=500, d=128, d_ff=512, G=2, K=4, r=8, k=2, q=32, factor_std=0.2, seed=49)
    w = ci.generate(cfg)
    m, ref = _stepwise(cfg, w)
    w0 = dict(w)
    for n in ("u1", "u2"):
        w0[n + "_s"] = np.zeros_like(w[n + "_s"])
    y0 = orc.ffn_naive(w0, w["x"], ref["expert_idx"], ref["gate"], cfg.K, cfg.q)
    assert orc.error_metrics(y0, ref["y"])["max_over_rms"] > 20 * MAX_OVER_RMS


def test_forward_is_deterministic():
    import torch
    cfg = ci.small_config("det", T=1500, d=128, d_ff=512, G=3, K=4, r=16, k=2, q=32, seed=50)
    w = ci.generate(cfg)
    layer = _layer(cfg, w)
    x = _dev(w["x"])
    a = layer.forward(x)
    _sync()
    ya = a["y"].clone()
    layer.ws.fill_(0x7f)
    b = layer.forward(x)
    _sync()
    assert torch.equal(ya, b["y"])
    layer.close()


@pytest.mark.parametrize("idx", [0, 1])
def test_config_full_output(idx):
    _stepwise(ci.config(idx))


def _sampled(cfg, n_sample, seed=0):
    """Full-size run through cmoe_forward; indices checked on every token, the output on
    a random sample of tokens that the dense per-expert oracle computes one by one."""
    print(f"case {cfg}", flush=True)
    w = ci.generate(cfg)
    cid, eidx, gate, _, _ = orc.route(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, w["cluster_bias"])
    offsets, perm, inv = orc.permute(cid, cfg.G)
    layer = _layer(cfg, w)
    out = layer.forward(_dev(w["x"]))
    _sync()
    assert np.array_equal(out["cluster_id"].cpu().numpy(), cid)
    assert np.array_equal(out["expert_idx"].cpu().numpy(), eidx)
    assert np.allclose(out["gate"].cpu().numpy(), gate, rtol=1e-5, atol=1e-6)
    assert np.array_equal(out["offsets"].cpu().numpy(), offsets)
    assert np.array_equal(out["perm"].cpu().numpy(), perm)
    assert np.array_equal(out["inv_perm"].cpu().numpy(), inv)
    y = out["y"].cpu().numpy()
    assert np.all(np.isfinite(y.astype(np.float32)))
    rng = np.random.default_rng(seed)
    rows = np.sort(rng.choice(cfg.T, size=min(n_sample, cfg.T), replace=False))
    # always include the first and last sorted row of every cluster (tile edges)
    edges = [perm[o] for o in offsets[:-1] if o < cfg.T] + [perm[o - 1] for o in offsets[1:] if o > 0]
    rows = np.unique(np.concatenate([rows, np.array(edges, dtype=np.int64)]))
    y_ref = orc.ffn_naive(w, w["x"][rows], eidx[rows], gate[rows], cfg.K, cfg.q)
    _check_y(y[rows], y_ref, f"{cfg.name} sampled {len(rows)} tokens")
    layer.close()


def test_config2_zipf_loads_sampled():
    _sampled(ci.config(2), 4096)


def test_config3_large_T_sampled():
    _sampled(ci.config(3), 1024)


def test_config4_weight_bound():
    _sampled(ci.config(4), 64)


def _all_tokens(cfg):
    """Full-size run through cmoe_forward with the output checked on EVERY token against the
    plain definition (dense per-expert FFNs, FP64), every routing output bit-exact."""
    print(f"case {cfg} (all tokens)", flush=True)
    w = ci.generate(cfg)
    ref = orc.forward_naive(w, w["x"], cfg.K, cfg.k, cfg.q)
    layer = _layer(cfg, w)
    out = layer.forward(_dev(w["x"]))
    _sync()
    for n in ("cluster_id", "expert_idx", "offsets", "perm", "inv_perm"):
        assert np.array_equal(out[n].cpu().numpy(), ref[n]), n
    assert np.allclose(out["gate"].cpu().numpy(), ref["gate"], rtol=1e-5, atol=1e-6)
    y = out["y"].cpu().numpy()
    _check_y(y, ref["y"], f"{cfg.name} all {cfg.T} tokens")
    # no 256-row slot of the launch may hide behind the aggregate: the bars hold per slot of
    # sorted rows as well (max against the global RMS)
    rms = orc.error_metrics(y, ref["y"])["rms"]
    diff = np.abs(y.astype(np.float64) - ref["y"])[ref["perm"]]
    per_slot = diff.reshape(-1, 256, cfg.d).max(axis=(1, 2)) / rms if cfg.T % 256 == 0 else diff.max(axis=1) / rms
    assert per_slot.max() <= MAX_OVER_RMS
    layer.close()
    return w, ref


def test_config2_zipf_loads_all_tokens():
    _all_tokens(ci.config(2))


def test_config3_large_T_all_tokens_and_split_entry_points():
    cfg = ci.config(3)
    w, ref = _all_tokens(cfg)
    # the same size through the separate entry points (cmoe_ffn_forward with a plain store,
    # the FP32 s reduction, cmoe_combine), fed the oracle's routing; checked on sampled tokens
    layer = _layer(cfg, w)
    x = _dev(w["x"])
    g32 = _dev(ref["gate"].astype(np.float32))
    yb, s = layer.ffn_forward(x, _dev(ref["perm"]), _dev(ref["offsets"]), _dev(ref["expert_idx"]), g32)
    y = layer.combine(yb, s, _dev(ref["perm"]), _dev(ref["inv_perm"]), _dev(ref["offsets"]), _dev(ref["expert_idx"]), g32)
    _sync()
    rng = np.random.default_rng(5)
    rows = np.sort(rng.choice(cfg.T, size=384, replace=False))
    edges = [ref["perm"][o] for o in ref["offsets"][:-1]] + [ref["perm"][o - 1] for o in ref["offsets"][1:]]
    rows = np.unique(np.concatenate([rows, np.array(edges, dtype=np.int64)]))
    cid_s = ref["cluster_id"][rows]
    off_s, perm_s, inv_s = orc.permute(cid_s, cfg.G)
    rw = orc.ffn_rewrite(w, w["x"][rows], perm_s, off_s, ref["expert_idx"][rows], ref["gate"][rows], cfg.K, cfg.q)
    yb_gpu = yb.cpu().numpy()[ref["inv_perm"][rows]]
    _check_y(yb_gpu, rw["y_base_sorted"][inv_s], "C3 y_base_sorted, separate entry points, sampled")
    _check_y(s.cpu().numpy()[rows], rw["s"], "C3 s_down, separate entry points, sampled")
    _check_y(y.cpu().numpy(), ref["y"], "C3 ffn_forward + combine, all tokens")
    layer.close()


def test_workspace_for_t_max_serves_smaller_batches_on_both_paths():
    # one layer, one workspace sized for 300 tokens: batches of 300 (matrix cores) and of 200 and
    # 256 (weight streaming) run in it; d large enough that the two layouts differ in size
    cfg = ci.small_config("ws_switch", T=300, d=1024, d_ff=256, G=8, K=2, r=4, k=2, q=64, seed=60)
    w = ci.generate(cfg)
    layer = _layer(cfg, w, T_max=300)
    for T in (300, 200, 256, 257, 1):
        x = w["x"][:T]
        ref = orc.forward_naive(w, x, cfg.K, cfg.k, cfg.q)
        out = layer.forward(_dev(x))
        _sync()
        assert np.array_equal(out["expert_idx"].cpu().numpy(), ref["expert_idx"])
        assert np.array_equal(out["perm"].cpu().numpy(), ref["perm"])
        _check_y(out["y"].cpu().numpy(), ref["y"], f"T={T} in a workspace for 300")
    layer.close()


NAN_CASES = [
    # weight-streaming router (one workgroup per token)
    ci.small_config("nan_small", T=40, d=64, d_ff=128, G=3, K=4, r=4, k=3, q=8, seed=61),
    # matrix-core router (more than 256 tokens, at most 128 router rows)
    ci.small_config("nan_mfma", T=300, d=64, d_ff=128, G=3, K=4, r=4, k=3, q=8, seed=62),
    # one wavefront per token (more than 128 router rows)
    ci.small_config("nan_wave", T=300, d=64, d_ff=128, G=20, K=8, r=4, k=3, q=8, seed=63),
]


@pytest.mark.parametrize("cfg", NAN_CASES, ids=[c.name for c in NAN_CASES])
def test_non_finite_logits_still_give_distinct_slots_of_one_cluster(cfg):
    # a NaN ranks below every number, equal ranks go to the lowest index: every router path and
    # the oracle name the same experts for tokens or router rows that hold NaN
    w = ci.generate(cfg)
    x = w["x"].copy()
    x[3, :] = np.float16(np.nan)                      # every logit of token 3 is NaN
    re = w["router_expert"].copy()
    re[1, 0] = np.float16(np.nan)                     # expert 1 (cluster 0) has a NaN logit for every token
    w2 = dict(w)
    w2["router_expert"] = re
    with np.errstate(invalid="ignore"):
        cid, eidx, gate, _, _ = orc.route(x, w["router_cluster"], re, cfg.K, cfg.k, w["cluster_bias"])
    layer = _layer(cfg, w2)
    g_cid, g_eidx, g_gate = layer.route(_dev(x))
    _sync()
    g_eidx = g_eidx.cpu().numpy()
    assert np.array_equal(g_cid.cpu().numpy(), cid)
    assert np.array_equal(g_eidx, eidx)
    assert g_eidx[3].tolist() == list(range(cfg.k))
    for t in range(cfg.T):
        assert len(set(g_eidx[t].tolist())) == cfg.k and np.all(g_eidx[t] // cfg.K == cid[t])
    # the variants: two clusters per token
    with np.errstate(invalid="ignore"):
        cids, e2, _, _ = orc.route_multi(x, w["router_cluster"], re, cfg.K, cfg.k, top_g=2)
    m_cid, m_eidx, _ = layer.route_multi(_dev(x), 2, 1.0, False)
    _sync()
    safe = np.ones(cfg.T, bool)
    z = x.astype(np.float64) @ w["router_cluster"].astype(np.float64).T
    zs = -np.sort(-np.nan_to_num(z, nan=-np.inf), axis=1)[:, :3]
    with np.errstate(invalid="ignore"):
        safe &= ~(np.abs(zs[:, 1] - zs[:, 2]) < 1e-3)          # the generator separates only the top two clusters
    safe[3] = True
    assert np.array_equal(m_cid.cpu().numpy()[safe], cids[safe])
    me = m_eidx.cpu().numpy()
    assert me[3].tolist() == [list(range(cfg.k)), list(range(cfg.K, cfg.K + cfg.k))]
    for t in range(cfg.T):
        for a in range(2):
            assert len(set(me[t, a].tolist())) == cfg.k
    layer.close()
