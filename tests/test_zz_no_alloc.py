"""cmoe_permute_static (the entry point that takes no workspace and allocates nothing)
against cmoe_permute, through the C ABI: bit-exact outputs on two calls in a row, the second
with a smaller input, so that whatever the first call left in the library's device array
cannot leak into the second."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_permute_static_matches_permute_on_consecutive_calls():
    import torch
    import paper_2510_02345_amd as cm
    import cmoe_inputs as ci
    from paper_2510_02345_amd import binding as B
    cfg = ci.small_config("static", T=64, d=64, d_ff=64, G=7, K=2, r=4, k=1, q=8, seed=301)
    w = ci.generate(cfg)
    T_big, T_small = 5000, 2300          # both above one workgroup's 1024 tokens: the array is in use
    layer = cm.Layer(cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q, w, T_big)
    rng = np.random.default_rng(302)
    # all output buffers exist before the calls: the calls themselves allocate nothing
    outs = {T: [torch.empty((T,), dtype=torch.int32, device="cuda:0"), torch.empty((T,), dtype=torch.int32, device="cuda:0"),
                torch.empty((cfg.G + 1,), dtype=torch.int32, device="cuda:0")] for T in (T_big, T_small, 700, 0)}
    ids = {T: torch.from_numpy(rng.integers(0, cfg.G, size=T).astype(np.int32)).to("cuda:0") for T in outs}
    torch.cuda.synchronize()
    for T in (T_big, T_small, 700, 0, T_big):
        print(f"cmoe_permute_static T={T}", flush=True)
        perm, inv, offsets = layer.permute_static(ids[T], *outs[T])
        torch.cuda.synchronize()
        want = layer.permute(ids[T])
        torch.cuda.synchronize()
        assert torch.equal(offsets, want[2])
        assert torch.equal(perm, want[0])
        assert torch.equal(inv, want[1])
        c = ids[T].cpu().numpy()
        assert np.array_equal(perm.cpu().numpy(), np.argsort(c, kind="stable").astype(np.int32))
    # beyond the stated maximum: rejected before any work
    rc = cm.lib().cmoe_permute_static(layer._h, 256, B.C.c_int32(1048577), 256, 256, outs[0][2].data_ptr(), None)
    assert rc == B.ERR_UNSUPPORTED
    layer.close()
