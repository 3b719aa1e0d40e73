"""GPU parity of the compression entry points (through the C ABI) against the FP64 oracle.

Bars: base matrices and INT4 codes / scales bit-exact (decisions in the kernel's FP32);
reconstruction errors and cosines to 1e-3 relative / 1e-4 absolute (FP32 tile sums against
FP64); the rank-r factors are judged by what is unique about them, their Frobenius error,
which must lie within 2 % above the truncated SVD's (Eckart-Young optimum) and cannot lie
below it by more than the FP16 rounding of the residual.
"""
import numpy as np
import pytest

import cmoe_inputs as ci
from oracle import cmoe_oracle as orc

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _sync():
    import torch
    torch.cuda.synchronize()


@pytest.mark.parametrize("rows,L,q", [(7, 64, 8), (33, 256, 32), (5, 2048, 128), (1, 128, 2)])
def test_quantiser_bit_exact(rows, L, q):
    import paper_2510_02345_amd as cm
    rng = np.random.default_rng(rows * 1000 + L)
    w = (rng.standard_normal((rows, L)) * 0.05).astype(np.float32)
    w[0, :q] = 0.0                                   # an all-zero group
    w[-1, -q:] = np.float32(1e-9)                    # a group whose scale rounds to zero in FP16
    w[rows // 2, :q] = np.linspace(-3.5, 3.5, q, dtype=np.float32)   # exact ties at scale 0.5
    codes, scales = cm.quantize_int4(_dev(w), q)
    _sync()
    want_codes, want_scales = orc.quantize_int4_f32(w, q)
    assert np.array_equal(scales.cpu().numpy().view(np.uint16), want_scales.view(np.uint16))
    assert np.array_equal(codes.cpu().numpy(), want_codes)
    _check_quantiser_definition(w, q, codes.cpu().numpy(), scales.cpu().numpy())


def _check_quantiser_definition(w, q, codes, scales):
    """The quantiser of Sec. 3.4 written out in FP64, with no reference to the order or precision
    of the kernel's steps: scale = the FP16 value nearest to absmax / 7 (either neighbour where
    the quotient sits within FP32 rounding of the midpoint), code = the integer nearest to
    w / scale clipped to [-7, 7] (either neighbour within FP32 rounding of a tie), zeros where the
    scale is zero."""
    rows, L = w.shape
    w64 = w.astype(np.float64).reshape(rows, L // q, q)
    quot = np.abs(w64).max(axis=-1) / 7.0
    s = scales.astype(np.float64)
    near = quot.astype(np.float16).astype(np.float64)
    other = np.where(near <= quot, np.nextafter(quot.astype(np.float16), np.float16(np.inf)),
                     np.nextafter(quot.astype(np.float16), np.float16(-np.inf))).astype(np.float64)
    tie = np.abs(np.abs(quot - near) - np.abs(quot - other)) <= 2.0 ** -22 * np.abs(quot)
    assert np.all((s == near) | (tie & (s == other)))
    c = orc.unpack_int4(codes).astype(np.float64).reshape(rows, L // q, q)
    live = s > 0
    assert np.all(c[~live] == 0) and np.all(np.abs(c) <= 7)
    ratio = np.clip(w64[live] / s[live][:, None], -7.0, 7.0)
    assert np.all(np.abs(c[live] - ratio) <= 0.5 + 2.0 ** -20 * (1.0 + np.abs(ratio)))


def _check_base_definition(W, G, K, base):
    """Eq. 6 in FP64: the stored base is the FP16 value nearest to the exact mean of the cluster's
    experts; the other FP16 neighbour only where the mean sits within FP32 rounding of the midpoint."""
    exact = W.astype(np.float64).reshape((G, K) + W.shape[1:]).sum(axis=1) / K
    b = base.astype(np.float64)
    near = exact.astype(np.float16).astype(np.float64)
    other = np.where(near <= exact, np.nextafter(exact.astype(np.float16), np.float16(np.inf)),
                     np.nextafter(exact.astype(np.float16), np.float16(-np.inf))).astype(np.float64)
    tie = np.abs(np.abs(exact - near) - np.abs(exact - other)) <= 2.0 ** -21 * np.abs(exact) + 1e-30
    assert np.all((b == near) | (tie & (b == other)))
    assert np.mean(b == near) > 0.999


def test_reconstruction_error_of_a_given_stored_form():
    import paper_2510_02345_amd as cm
    G, K, r, q, out_d, in_d = 2, 3, 8, 32, 192, 128
    W = ci.generate_dense_experts(G, K, out_d, in_d, rank=6, residual_rel=0.2, noise_rel=0.02, seed=71)
    base = orc.base_mean(W, G, K)
    rng = np.random.default_rng(72)
    uq, us = ci.quantize_int4(rng.standard_normal((G * K, r, out_d)) * 0.05, q)
    vq, vs = ci.quantize_int4(rng.standard_normal((G * K, r, in_d)) * 0.05, q)
    err = cm.reconstruction_error(_dev(W), _dev(base), _dev(uq), _dev(us), _dev(vq), _dev(vs), G, K, r, q)
    _sync()
    for e in range(G * K):
        U = orc.dequant_int4(uq[e], us[e], q).T          # [out][r]
        V = orc.dequant_int4(vq[e], vs[e], q)            # [r][in]
        want = orc.reconstruction_error(W[e], base[e // K], U, V)
        assert float(err[e]) == pytest.approx(want, rel=1e-4)


CASES = [
    # (name, G, K, out, in, true rank, residual, noise, r, sketch, q)
    ("decaying", 2, 4, 256, 128, 12, 0.3, 0.01, 8, 16, 32),
    ("wide_in", 1, 3, 128, 320, 20, 0.2, 0.02, 16, 24, 64),
    ("r32", 2, 2, 192, 256, 40, 0.3, 0.01, 32, 40, 32),
    ("noise_only", 1, 4, 128, 128, 4, 0.0, 0.05, 4, 12, 8),
    # an odd number of sketch rows (the round-robin Jacobi then has an idle index every round)
    ("odd_sketch", 1, 3, 128, 192, 10, 0.3, 0.01, 8, 13, 32),
    # the widest sketch
    ("sketch48", 1, 2, 128, 128, 30, 0.3, 0.01, 32, 48, 32),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_compress_against_truncated_svd(case):
    import paper_2510_02345_amd as cm
    name, G, K, out_d, in_d, rank0, res, noise, r, sketch, q = case
    print(f"case {case}", flush=True)
    W = ci.generate_dense_experts(G, K, out_d, in_d, rank0, res, noise, seed=80 + len(name))
    omega = ci.sketch_rows(sketch, in_d, seed=90 + len(name))
    o = cm.compress(_dev(W), _dev(omega), G, K, r, q, n_iter=2)
    _sync()
    base = orc.base_mean(W, G, K)
    assert np.array_equal(o["base"].cpu().numpy().view(np.uint16), base.view(np.uint16))
    _check_base_definition(W, G, K, o["base"].cpu().numpy())
    rep = o["report"].cpu().numpy()
    uq, us = o["u_q"].cpu().numpy(), o["u_s"].cpu().numpy()
    vq, vs = o["v_q"].cpu().numpy(), o["v_s"].cpu().numpy()
    for e in range(G * K):
        delta = orc.residual(W[e], base[e // K])
        U_svd, V_svd, opt, _ = orc.truncated_svd_factors(delta, r)
        wn = np.linalg.norm(W[e].astype(np.float64))
        opt_rel, floor = opt / wn, 2.0 ** -10 * np.linalg.norm(delta) / wn
        # what the layer would compute with: the returned codes and scales, dequantised and
        # measured by the oracle, not by the library
        U = orc.dequant_int4(uq[e], us[e], q).T          # [out][r]
        V = orc.dequant_int4(vq[e], vs[e], q)            # [r][in]
        stored = orc.reconstruction_error(W[e], base[e // K], U, V)
        # the yardstick for the stored form: the truncated SVD's own factors through the same
        # INT4 format (rank-major rows, FP16 scale per q codes), quantised by the oracle
        Uq = orc.dequant_int4(*orc.quantize_int4_f32(U_svd.T.astype(np.float32), q), q).T
        Vq = orc.dequant_int4(*orc.quantize_int4_f32(V_svd.astype(np.float32), q), q)
        svd_stored = orc.reconstruction_error(W[e], base[e // K], Uq, Vq)
        # the split of the singular values between the factors: all on U (above), or all on V
        # as the library does; the better of the two is the yardstick
        sv = np.linalg.norm(U_svd, axis=0)
        sv = np.where(sv > 0, sv, 1.0)
        Uq2 = orc.dequant_int4(*orc.quantize_int4_f32((U_svd / sv).T.astype(np.float32), q), q).T
        Vq2 = orc.dequant_int4(*orc.quantize_int4_f32((V_svd * sv[:, None]).astype(np.float32), q), q)
        svd_stored = min(svd_stored, orc.reconstruction_error(W[e], base[e // K], Uq2, Vq2))
        print(f"  e{e}: rank-{r} error {rep[e, 1]:.5f} (optimum {opt_rel:.5f}); stored form {stored:.5f} "
              f"(library reports {rep[e, 0]:.5f}; INT4 truncated SVD {svd_stored:.5f})", flush=True)
        assert rep[e, 1] <= opt_rel * 1.02 + floor
        assert rep[e, 1] >= opt_rel * 0.995 - floor
        assert rep[e, 2] == pytest.approx(orc.cosine_to_base(delta, base[e // K]), abs=1e-4)
        assert rep[e, 3] == 0.0
        assert rep[e, 0] == pytest.approx(stored, rel=1e-3, abs=1e-6)      # the report is the error of the output
        assert stored <= 1.1 * svd_stored + floor
        assert stored >= opt_rel * 0.995 - floor                          # nothing of rank r beats the optimum
    # the error the library reports for its own output is the error of that output
    again = cm.reconstruction_error(_dev(W), _dev(base), o["u_q"], o["u_s"], o["v_q"], o["v_s"], G, K, r, q)
    _sync()
    assert np.allclose(again.cpu().numpy(), rep[:, 0], rtol=1e-6)
    assert uq.shape == (G * K, r, out_d // 2) and vs.shape == (G * K, r, in_d // q) and us.dtype == np.float16
    assert vq.dtype == np.uint8


def test_exactly_low_rank_residual_is_recovered():
    import paper_2510_02345_amd as cm
    # Delta_e = L_e - mean_j L_j has rank at most K * rank = 8 = r
    G, K, out_d, in_d, r = 1, 4, 128, 192, 8
    W = ci.generate_dense_experts(G, K, out_d, in_d, rank=2, residual_rel=0.3, noise_rel=0.0, seed=101)
    base = orc.base_mean(W, G, K)
    o = cm.compress(_dev(W), _dev(ci.sketch_rows(16, in_d, seed=102)), G, K, r, 32, n_iter=2)
    _sync()
    rep = o["report"].cpu().numpy()
    for e in range(K):
        delta = orc.residual(W[e], base[0])
        _, _, opt, sv = orc.truncated_svd_factors(delta, r)
        rel = np.linalg.norm(delta) / np.linalg.norm(W[e].astype(np.float64))
        # the residual of FP16 matrices against the FP16 mean is low rank only up to FP16 rounding
        assert opt <= 2e-3 * np.linalg.norm(delta)
        # [1] is a difference of two FP32 sums of FP16-rounded values: floor about 1 % of ||Delta||
        assert rep[e, 1] <= 1e-2 * rel
        assert rep[e, 0] <= 0.2 * rel        # stored form: INT4 steps of both factors


def test_gate_zeroes_the_factors():
    import paper_2510_02345_amd as cm
    G, K, out_d, in_d, r, q = 2, 2, 128, 128, 4, 32
    W = ci.generate_dense_experts(G, K, out_d, in_d, rank=4, residual_rel=0.3, noise_rel=0.01, seed=111)
    base = orc.base_mean(W, G, K)
    # threshold above every possible cosine: all experts are gated off
    o = cm.compress(_dev(W), _dev(ci.sketch_rows(8, in_d, seed=112)), G, K, r, q, n_iter=1, use_gate=True,
                    gate_gamma=2.0)
    _sync()
    rep = o["report"].cpu().numpy()
    assert np.all(rep[:, 3] == 1.0)
    assert not o["u_q"].cpu().numpy().any() and not o["v_q"].cpu().numpy().any()
    assert not o["u_s"].cpu().numpy().view(np.uint16).any() and not o["v_s"].cpu().numpy().view(np.uint16).any()
    for e in range(G * K):
        want = orc.reconstruction_error(W[e], base[e // K], np.zeros((out_d, r)), np.zeros((r, in_d)))
        assert rep[e, 0] == pytest.approx(want, rel=1e-4)
    # threshold below every cosine: nothing is gated
    o2 = cm.compress(_dev(W), _dev(ci.sketch_rows(8, in_d, seed=112)), G, K, r, q, n_iter=1, use_gate=True,
                     gate_gamma=-2.0)
    _sync()
    assert np.all(o2["report"].cpu().numpy()[:, 3] == 0.0) and o2["u_q"].cpu().numpy().any()


def test_compressed_layer_runs_forward_close_to_the_dense_layer():
    """Dense experts -> cmoe_compress (both matrices) -> cmoe_forward, against the dense layer
    evaluated by the oracle.  The compressed layer is an approximation: the bar is the size of
    the compression error, far below what a mis-oriented or mis-laid-out factor would give."""
    import torch
    import paper_2510_02345_amd as cm
    G, K, d, d_ff, r, q, k, T = 2, 4, 128, 256, 8, 32, 2, 300
    E = G * K
    W1 = ci.generate_dense_experts(G, K, d_ff, d, rank=1, residual_rel=0.5, noise_rel=0.0, seed=121)
    W2 = ci.generate_dense_experts(G, K, d, d_ff, rank=1, residual_rel=0.5, noise_rel=0.0, seed=122)
    cfg = ci.small_config("e2e", T=T, d=d, d_ff=d_ff, G=G, K=K, r=r, k=k, q=q, seed=123)
    w = ci.generate(cfg)                     # routers and tokens (with the routing margin) from here
    c1 = cm.compress(_dev(W1), _dev(ci.sketch_rows(16, d, seed=124)), G, K, r, q, n_iter=2)
    c2 = cm.compress(_dev(W2), _dev(ci.sketch_rows(16, d_ff, seed=125)), G, K, r, q, n_iter=2)
    _sync()
    # residuals of rank <= K = 4 under a sketch of 16 rows: the orthonormalisation must cope with
    # a rank-deficient sketch for every expert alike
    for c in (c1, c2):
        err = c["report"][:, 0].cpu().numpy()
        assert err.max() < 0.08 and err.max() <= 1.2 * np.median(err)
    weights = dict(router_cluster=w["router_cluster"], router_expert=w["router_expert"], cluster_bias=None,
                   w1_base=c1["base"], w2_base=c2["base"],
                   v1_q=c1["v_q"], v1_s=c1["v_s"], u1_q=c1["u_q"], u1_s=c1["u_s"],
                   v2_q=c2["v_q"], v2_s=c2["v_s"], u2_q=c2["u_q"], u2_s=c2["u_s"])
    layer = cm.Layer(d, d_ff, G, K, r, k, q, weights, T)
    out = layer.forward(_dev(w["x"]))
    _sync()
    cid, eidx, gate, _, _ = orc.route(w["x"], w["router_cluster"], w["router_expert"], K, k)
    assert np.array_equal(out["expert_idx"].cpu().numpy(), eidx)
    y_dense = orc.ffn_dense(W1, W2, w["x"], eidx, gate)
    y = out["y"].float().cpu().numpy().astype(np.float64)
    rel = np.linalg.norm(y - y_dense) / np.linalg.norm(y_dense)
    # without the residuals (base only) the output is far off: the factors carry real weight
    y_base = orc.ffn_dense(np.repeat(orc.base_mean(W1, G, K), K, axis=0), np.repeat(orc.base_mean(W2, G, K), K, axis=0),
                           w["x"], eidx, gate)
    rel_base = np.linalg.norm(y_base - y_dense) / np.linalg.norm(y_dense)
    print(f"compressed vs dense layer: {rel:.4f}; base only: {rel_base:.4f}", flush=True)
    assert rel_base > 0.2
    assert rel < 0.08
    layer.close()


def test_single_expert_clusters_have_no_residual():
    # K = 1: the base is the expert itself (Eq. 6), the residual is exactly zero
    import paper_2510_02345_amd as cm
    G, K, out_d, in_d, r, q = 3, 1, 128, 64, 4, 16
    W = ci.generate_dense_experts(G, K, out_d, in_d, rank=2, residual_rel=0.3, noise_rel=0.01, seed=131)
    o = cm.compress(_dev(W), _dev(ci.sketch_rows(8, in_d, seed=132)), G, K, r, q, n_iter=1)
    _sync()
    assert np.array_equal(o["base"].cpu().numpy().view(np.uint16), W.view(np.uint16))
    rep = o["report"].cpu().numpy()
    assert np.all(np.isfinite(rep)) and np.all(rep[:, :3] == 0.0)
    assert not o["u_q"].cpu().numpy().any() and not o["v_q"].cpu().numpy().any()
