"""GPU parity of cmoe_backward (through the C ABI) against the FP64 oracle's dense chain rule.

The selection (expert_idx, gate) is the oracle's, frozen.  Bar per gradient tensor:
max|g - g_ref| <= 2e-2 * RMS(g_ref) (twice the forward bar: a weight gradient of a sparsely
hit expert is a sum over few rows, its RMS is taken over many zeros) and
sum|g - g_ref| / sum|g_ref| <= 2e-3 (the forward bar).
"""
import numpy as np
import pytest

import cmoe_inputs as ci
from oracle import cmoe_oracle as orc

pytestmark = pytest.mark.gpu

NAMES = ("dx", "d_router_expert", "dw1_base", "dw2_base", "du1", "dv1", "du2", "dv2")


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _run(cfg, w=None, dy_scale=1.0, pack=True, drop_canonical=False):
    import torch
    import paper_2510_02345_amd as cm
    print(f"case {cfg}", flush=True)
    w = w if w is not None else ci.generate(cfg)
    rng = np.random.default_rng(cfg.seed + 7)
    dy = (dy_scale * rng.standard_normal((cfg.T, cfg.d))).astype(np.float16)
    cid, eidx, gate, _, _ = orc.route(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, w["cluster_bias"])
    ref = orc.backward_naive(w, w["x"], dy, eidx, gate, cfg.K, cfg.q)
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, cfg.T, pack=pack)
    if drop_canonical:
        layer.drop_canonical_bases()
    out = layer.backward(_dev(w["x"]), _dev(dy), _dev(eidx.astype(np.int32)), _dev(gate.astype(np.float32)))
    torch.cuda.synchronize()
    res = {}
    for n in NAMES + ("d_logits",):
        got = out[n].cpu().numpy().astype(np.float64)
        want = ref["dgate_logits" if n == "d_logits" else n]
        assert got.shape == want.shape, n
        assert np.all(np.isfinite(got)), n
        if want.size == 0:
            continue
        if not np.any(want):        # top_k = 1: the gate is constant, its gradient exactly zero
            assert np.abs(got).max() <= 1e-6, n
            continue
        m = orc.error_metrics(got, want)
        print(f"  {n}: max/rms={m['max_over_rms']:.3e} mean_rel={m['mean_rel']:.3e}", flush=True)
        res[n] = m
    for n, m in res.items():
        assert m["max_over_rms"] <= 2e-2, (n, m)
        assert m["mean_rel"] <= 2e-3, (n, m)
    layer.close()
    return out, ref


SMALL = [
    ci.small_config("bw_ragged", T=777, d=128, d_ff=384, G=3, K=4, r=8, k=2, q=32, seed=141),
    ci.small_config("bw_k1", T=300, d=64, d_ff=192, G=2, K=4, r=4, k=1, q=8, seed=142),
    ci.small_config("bw_flat_r32", T=130, d=192, d_ff=256, G=1, K=3, r=32, k=3, q=64, seed=143),
    ci.small_config("bw_sparse", T=19, d=64, d_ff=128, G=16, K=2, r=16, k=2, q=16, seed=144),
    ci.small_config("bw_k4", T=1500, d=128, d_ff=256, G=2, K=8, r=4, k=4, q=32, seed=145),
    ci.small_config("bw_one", T=1, d=64, d_ff=64, G=2, K=2, r=8, k=2, q=8, seed=146),
    # the largest top-k (8 of 32 experts per cluster) and the largest rank panel (K * r = 512)
    ci.small_config("bw_k8_of_32", T=400, d=64, d_ff=128, G=2, K=32, r=4, k=8, q=8, seed=153),
    ci.small_config("bw_max_rank", T=300, d=64, d_ff=128, G=1, K=16, r=32, k=2, q=8, seed=154),
    # the widest model dimension
    ci.small_config("bw_max_d", T=300, d=8192, d_ff=128, G=4, K=2, r=4, k=2, q=128, seed=155),
]


@pytest.mark.parametrize("cfg", SMALL, ids=[c.name for c in SMALL])
def test_backward_small(cfg):
    _run(cfg)


def test_backward_config1():
    _run(ci.config(1))


def test_backward_canonical_bases_without_the_packed_copy():
    _run(SMALL[0], pack=False)


@pytest.mark.parametrize("cfg", [SMALL[0], SMALL[8]], ids=lambda c: c.name)
def test_backward_packed_copy_as_the_only_resident_bases(cfg):
    # w1_base / w2_base freed and passed as NULL after packing: the transposed operands and the
    # forward base product of the backward pass are all built from the packed buffer
    _run(cfg, drop_canonical=True)


def test_backward_live_residual_and_gate_path():
    # factors ten times larger and a sharper router: the low-rank terms and the gate path are
    # far above the tolerance, so dropping either would fail
    cfg = ci.small_config("bw_bigres", T=500, d=128, d_ff=512, G=2, K=4, r=8, k=2, q=32, factor_std=0.2, seed=147)
    w = ci.generate(cfg)
    out, ref = _run(cfg, w)
    cid, eidx, gate, _, _ = orc.route(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, w["cluster_bias"])
    w0 = dict(w)
    for n in ("u1", "u2"):
        w0[n + "_s"] = np.zeros_like(w[n + "_s"])
    rng = np.random.default_rng(cfg.seed + 7)
    dy = rng.standard_normal((cfg.T, cfg.d)).astype(np.float16)
    ref0 = orc.backward_naive(w0, w["x"], dy, eidx, gate, cfg.K, cfg.q)
    assert orc.error_metrics(ref0["dx"], ref["dx"])["max_over_rms"] > 0.2
    assert np.sqrt((ref["dgate_logits"] ** 2).mean()) > 1e-2


def test_backward_empty_cluster_weights_never_read():
    cfg = ci.small_config("bw_onecluster", T=200, d=64, d_ff=128, G=2, K=4, r=8, k=2, q=8, seed=148)
    w = ci.generate(cfg)
    w["cluster_bias"] = np.array([-100.0, 100.0], dtype=np.float32)
    for n in ("w1_base", "w2_base"):
        w[n][0] = np.float16(np.nan)
    for n in ("v1", "u1", "v2", "u2"):
        w[n + "_s"][:cfg.K] = np.float16(np.nan)
    out, ref = _run(cfg, w)
    for n in ("dw1_base", "dw2_base"):
        assert not out[n][0].any()
    for n in ("du1", "dv1", "du2", "dv2", "d_router_expert"):
        assert not out[n][:cfg.K].any()


@pytest.mark.parametrize("G,K", [(2, 2), (20, 8)])
def test_backward_no_tokens_gives_zero_gradients(G, K):
    import torch
    import paper_2510_02345_amd as cm
    cfg = ci.small_config("bw_empty", T=0, d=64, d_ff=128, G=G, K=K, r=8, k=2, q=8, seed=149)
    w = ci.generate(cfg)
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, 16)
    e = torch.empty((0, cfg.k), dtype=torch.int32, device="cuda:0")
    out = layer.backward(torch.empty((0, cfg.d), dtype=torch.float16, device="cuda:0"),
                         torch.empty((0, cfg.d), dtype=torch.float16, device="cuda:0"), e, e.float())
    torch.cuda.synchronize()
    for n in NAMES[1:]:
        assert not out[n].any(), n
    layer.close()


def test_backward_is_deterministic():
    import torch
    import paper_2510_02345_amd as cm
    cfg = ci.small_config("bw_det", T=1500, d=128, d_ff=512, G=3, K=4, r=16, k=2, q=32, seed=150)
    w = ci.generate(cfg)
    rng = np.random.default_rng(5)
    dy = _dev(rng.standard_normal((cfg.T, cfg.d)).astype(np.float16))
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, cfg.T)
    x = _dev(w["x"])
    f = layer.forward(x)
    a = layer.backward(x, dy, f["expert_idx"], f["gate"])
    torch.cuda.synchronize()
    a = {n: v.clone() for n, v in a.items()}
    layer.bw_ws.fill_(0x7f)
    b = layer.backward(x, dy, f["expert_idx"], f["gate"])
    torch.cuda.synchronize()
    for n in a:
        assert torch.equal(a[n], b[n]), n
    layer.close()


def test_backward_more_than_64_experts():
    # 160 and 128 experts: pairs sorted by expert in two passes, rank products in slices of 64 experts
    _run(ci.small_config("bw_many", T=400, d=64, d_ff=128, G=20, K=8, r=4, k=2, q=8, seed=151))
    _run(ci.small_config("bw_many_clusters", T=3000, d=64, d_ff=128, G=64, K=2, r=8, k=2, q=16, seed=152))


def _sampled(cfg, clusters, n_tok, hidden, seed=0):
    """Full-size run; dx and d_logits checked on sampled tokens of a few clusters, the weight
    gradients on sampled hidden units (rows of dW1, columns of dW2) over every expert."""
    import torch
    import paper_2510_02345_amd as cm
    print(f"case {cfg}", flush=True)
    w = ci.generate(cfg)
    rng = np.random.default_rng(cfg.seed + 7)
    dy = rng.standard_normal((cfg.T, cfg.d)).astype(np.float16)
    cid, eidx, gate, _, _ = orc.route(w["x"], w["router_cluster"], w["router_expert"], cfg.K, cfg.k, w["cluster_bias"])
    pool = np.nonzero(np.isin(cid, clusters))[0]
    tokens = np.sort(np.random.default_rng(seed).choice(pool, size=min(n_tok, len(pool)), replace=False))
    hidden = np.asarray(hidden)
    ref = orc.backward_sampled(w, w["x"], dy, eidx, gate, cfg.K, cfg.q, tokens, hidden)
    print("oracle done", flush=True)
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, cfg.T)
    out = layer.backward(_dev(w["x"]), _dev(dy), _dev(eidx.astype(np.int32)), _dev(gate.astype(np.float32)))
    torch.cuda.synchronize()
    ti, hi = _dev(tokens), _dev(hidden)
    got = dict(dx=out["dx"][ti], dgate_logits=out["d_logits"][ti], dw1_base=out["dw1_base"][:, hi, :],
               dw2_base=out["dw2_base"][:, :, hi], du1=out["du1"][:, :, hi], dv2=out["dv2"][:, :, hi])
    for n in NAMES[1:]:
        assert bool(torch.isfinite(out[n]).all()), n
    for n, g in got.items():
        m = orc.error_metrics(g.cpu().numpy().astype(np.float64), ref[n])
        print(f"  {n}: max/rms={m['max_over_rms']:.3e} mean_rel={m['mean_rel']:.3e}", flush=True)
        assert m["max_over_rms"] <= 2e-2, (n, m)
        assert m["mean_rel"] <= 2e-3, (n, m)
    layer.close()


def test_backward_config2_zipf_loads_sampled():
    _sampled(ci.config(2), clusters=[0, 3], n_tok=64, hidden=[0, 1, 2047, 2048, 4095])


def test_backward_config3_sampled():
    _sampled(ci.config(3), clusters=[2, 7], n_tok=64, hidden=[0, 255, 256, 4097, 8191])


def test_backward_config4_weight_bound_sampled():
    # 64 tokens, every cluster hit, r = 32: tokens of one cluster, a few hidden units
    _sampled(ci.config(4), clusters=[5], n_tok=8, hidden=[0, 1023, 1024, 14335])
