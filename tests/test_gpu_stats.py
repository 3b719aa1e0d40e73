"""GPU parity of cmoe_route_stats (through the C ABI) against the FP64 oracle.

Bars: expert loads, cluster loads and idle counters bit-exact; the load CV to 1e-6
relative (FP64 on both sides, rounded to FP32 by the library); centroids and cluster
activity to 1e-5 relative to the largest magnitude of the row (FP32 sums of at most T
FP16 values in a fixed order against FP64).
"""
import numpy as np
import pytest

import cmoe_inputs as ci
from oracle import cmoe_oracle as orc

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _run_steps(cfg, n_steps=2, beta=0.05, lam=0.25, drop_cluster=None):
    import torch
    import paper_2510_02345_amd as cm
    print(f"case {cfg}", flush=True)
    w = ci.generate(cfg)
    if drop_cluster is not None:
        bias = np.zeros(cfg.G, dtype=np.float32)
        bias[drop_cluster] = -100.0
        w["cluster_bias"] = bias
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, cfg.T)
    E = cfg.G * cfg.K
    rng = np.random.default_rng(cfg.seed + 1000)
    mu0 = rng.standard_normal((E, cfg.d)).astype(np.float32)
    mu_ref, act_ref, idle_ref = mu0.astype(np.float64), np.zeros(cfg.G), np.zeros(cfg.G, dtype=np.int64)
    mu, act, idle = _dev(mu0), _dev(np.zeros(cfg.G, dtype=np.float32)), _dev(np.zeros(cfg.G, dtype=np.int32))
    x = w["x"]
    for step in range(n_steps):
        xs = np.ascontiguousarray(np.roll(x, step * 7, axis=0))   # a different batch every step
        cid, eidx, _, _, _ = orc.route(xs, w["router_cluster"], w["router_expert"], cfg.K, cfg.k, w["cluster_bias"])
        offsets, perm, _ = orc.permute(cid, cfg.G)
        load, cload, cv = layer.route_stats(_dev(xs), _dev(perm.astype(np.int32)), _dev(offsets.astype(np.int32)),
                                            _dev(eidx.astype(np.int32)), mu, act, idle, beta, lam)
        torch.cuda.synchronize()
        loads_ref = orc.expert_loads(eidx, E)
        mu_ref = orc.centroid_ema(mu_ref, xs, eidx, beta)
        act_ref, idle_ref, counts_ref = orc.cluster_activity(act_ref, idle_ref, cid, cfg.G, lam)
        assert np.array_equal(load.cpu().numpy(), loads_ref)
        assert np.array_equal(cload.cpu().numpy(), counts_ref)
        assert np.array_equal(idle.cpu().numpy(), idle_ref)
        assert float(cv.cpu()[0]) == pytest.approx(orc.load_cv(loads_ref), rel=1e-6, abs=1e-12)
        assert np.allclose(act.cpu().numpy(), act_ref, rtol=1e-5, atol=1e-7)
        got = mu.cpu().numpy().astype(np.float64)
        scale = np.abs(mu_ref).max(axis=1, keepdims=True) + 1e-30
        err = np.abs(got - mu_ref) / scale
        print(f"step {step}: centroid max rel err {err.max():.2e}, CV {float(cv.cpu()[0]):.4f}", flush=True)
        assert err.max() <= 1e-5
        unused = np.nonzero(loads_ref == 0)[0]
        if step == 0 and unused.size:
            assert np.array_equal(mu.cpu().numpy()[unused], mu0[unused])   # no token: bit-for-bit unchanged
    layer.close()


STATS = [
    ci.small_config("st_ragged", T=777, d=128, d_ff=128, G=3, K=4, r=4, k=2, q=32, seed=61),
    ci.small_config("st_sparse", T=19, d=64, d_ff=64, G=16, K=2, r=4, k=2, q=16, seed=62),
    ci.small_config("st_k4", T=300, d=2112, d_ff=64, G=2, K=8, r=4, k=4, q=32, seed=63),   # two column chunks
    ci.small_config("st_one", T=1, d=64, d_ff=64, G=2, K=2, r=4, k=1, q=8, seed=64),
]


@pytest.mark.parametrize("cfg", STATS, ids=[c.name for c in STATS])
def test_route_stats_small(cfg):
    _run_steps(cfg, n_steps=3)


def test_route_stats_idle_cluster():
    # one cluster never receives a token: its experts keep their centroids, its idle count grows
    cfg = ci.small_config("st_idle", T=200, d=64, d_ff=64, G=4, K=2, r=4, k=2, q=8, seed=65)
    _run_steps(cfg, n_steps=3, drop_cluster=2)


def test_route_stats_empty_step():
    import torch
    import paper_2510_02345_amd as cm
    cfg = ci.small_config("st_empty", T=0, d=64, d_ff=64, G=2, K=2, r=4, k=2, q=8, seed=66)
    w = ci.generate(cfg)
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, 16)
    mu0 = np.arange(4 * 64, dtype=np.float32).reshape(4, 64)
    mu, act, idle = _dev(mu0), _dev(np.full(2, 0.5, dtype=np.float32)), _dev(np.array([3, 0], dtype=np.int32))
    x = torch.empty((0, 64), dtype=torch.float16, device="cuda:0")
    e = torch.empty((0, 2), dtype=torch.int32, device="cuda:0")
    p = torch.empty((0,), dtype=torch.int32, device="cuda:0")
    load, cload, cv = layer.route_stats(x, p, _dev(np.zeros(3, dtype=np.int32)), e, mu, act, idle, 0.05, 0.25)
    torch.cuda.synchronize()
    assert np.array_equal(load.cpu().numpy(), np.zeros(4, dtype=np.int32))
    assert np.array_equal(cload.cpu().numpy(), np.zeros(2, dtype=np.int32))
    assert float(cv.cpu()[0]) == 0.0
    assert np.array_equal(mu.cpu().numpy(), mu0)
    assert np.allclose(act.cpu().numpy(), [0.375, 0.375])
    assert np.array_equal(idle.cpu().numpy(), [4, 1])
    layer.close()


def test_route_stats_config3():
    _run_steps(ci.config(3), n_steps=1)
