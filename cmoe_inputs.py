"""Seeded synthetic inputs for the clustered, compressed MoE FFN layer.

This module only *draws and encodes* inputs.  It serves both the CPU oracle's
tests and the HIP path's tests/bench, and therefore contains none of the
layer's arithmetic: no routing decision, no dequantisation, no FFN.  The one
matrix product below (`_logit_gaps`) is input conditioning: it measures how
close the two-stage router's logits are to a tie so that such tokens can be
redrawn; it never produces an expected value.

Shapes and statistics follow the paper's workloads (Sec. 3.2, 3.3, 3.4 and the
experimental setup in Sec. 4): d = 768 base width, K = E/G in {4, 8}, residual
rank r in {4, 8, 16, 32}, top-1 cluster then top-k (k = 2) experts, FP16 bases
and routers, INT4 group-quantised low-rank factors.  The datasets the paper
measures on are not used; only these shapes are.

Layouts (all C-contiguous numpy arrays):
  x               [T][d]            float16
  router_cluster  [G][d]            float16   group prototypes u_g
  router_expert   [G*K][d]          float16   expert vectors v_i, cluster-major
  cluster_bias    [G] float32 or None         load-skew bias (benchmark only)
  w1_base         [G][d_ff][d]      float16   W1_base(c), out-major
  w2_base         [G][d][d_ff]      float16   W2_base(c), out-major
  v1_q,u1_q,v2_q,u2_q [E][r][L/2]   uint8     two INT4 codes per byte,
                                              L = d, d_ff, d_ff, d
  v1_s,u1_s,v2_s,u2_s [E][r][L/q]   float16   one scale per q consecutive codes
INT4 code: two's-complement nibble in [-8, 7]; element n of a row sits in byte
n // 2, even n in the low nibble.  value = scale * code (symmetric, no zero
point).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

MARGIN = 1e-3  # minimum gap between logits whose order decides an index


@dataclass(frozen=True)
class LayerConfig:
    name: str
    T: int
    d: int
    d_ff: int
    G: int
    K: int
    r: int
    k: int
    q: int
    router: str = "uniform"      # "uniform" | "zipf" | "all_hit"
    factor_std: float = 0.02
    seed: int = 0

    @property
    def E(self) -> int:
        return self.G * self.K


_SEED_BASE = 20251002 * 10

CONFIGS = (
    LayerConfig("C0", 256, 128, 512, 2, 4, 4, 1, 32, "uniform", seed=_SEED_BASE + 0),
    LayerConfig("C1", 4096, 768, 3072, 2, 4, 8, 2, 32, "uniform", seed=_SEED_BASE + 1),
    LayerConfig("C2", 16384, 1024, 4096, 4, 4, 16, 2, 64, "zipf", seed=_SEED_BASE + 2),
    LayerConfig("C3", 32768, 2048, 8192, 8, 8, 16, 2, 64, "uniform", seed=_SEED_BASE + 3),
    LayerConfig("C4", 64, 4096, 14336, 8, 8, 32, 2, 128, "all_hit", seed=_SEED_BASE + 4),
)


def config(index_or_name) -> LayerConfig:
    if isinstance(index_or_name, int):
        return CONFIGS[index_or_name]
    for c in CONFIGS:
        if c.name == index_or_name:
            return c
    raise KeyError(index_or_name)


def small_config(name="S", **kw) -> LayerConfig:
    """A free-form small configuration for tests."""
    base = dict(T=64, d=64, d_ff=128, G=2, K=4, r=4, k=2, q=32, router="uniform",
                factor_std=0.02, seed=1234)
    base.update(kw)
    return LayerConfig(name, **base)


# --------------------------------------------------------------------------
# INT4 group-wise symmetric quantiser + packer (encoding of the stored factors)
# --------------------------------------------------------------------------
def quantize_int4(w: np.ndarray, q: int):
    """w [..., L] float -> (packed uint8 [..., L/2], scales float16 [..., L/q]).

    scale = fp16(absmax / 7) per group of q consecutive elements; code =
    clip(rint(w / scale), -7, 7) (round half to even); an all-zero group gets
    scale 0 and codes 0.
    """
    L = w.shape[-1]
    assert L % q == 0 and q % 2 == 0
    g = w.reshape(*w.shape[:-1], L // q, q).astype(np.float64)
    absmax = np.abs(g).max(axis=-1)
    scale = (absmax / 7.0).astype(np.float16)
    s64 = scale.astype(np.float64)
    safe = np.where(s64 > 0, s64, 1.0)
    codes = np.clip(np.rint(g / safe[..., None]), -7, 7).astype(np.int8)
    codes = np.where(s64[..., None] > 0, codes, 0).astype(np.int8)
    codes = codes.reshape(*w.shape[:-1], L)
    return pack_int4(codes), scale


def pack_int4(codes: np.ndarray) -> np.ndarray:
    """codes int8 in [-8, 7], [..., L] -> uint8 [..., L/2]; even n in the low nibble."""
    u = (codes.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


# --------------------------------------------------------------------------
# tie conditioning
# --------------------------------------------------------------------------
def _logit_gaps(x16, rc16, re16, bias, K, k):
    """Smallest gap that decides a routing index, per token (float64).

    Gap between the two largest cluster logits, and the adjacent gaps among the
    k + 1 largest logits inside the cluster that has the largest one.
    """
    x = x16.astype(np.float64)
    z = x @ rc16.astype(np.float64).T
    if bias is not None:
        z = z + bias.astype(np.float64)[None, :]
    G = z.shape[1]
    zs = np.sort(z, axis=1)
    gap = zs[:, -1] - zs[:, -2] if G > 1 else np.full(len(x), np.inf)
    c = np.argmax(z, axis=1)
    l_all = x @ re16.astype(np.float64).T            # [T][E]
    idx = c[:, None] * K + np.arange(K)[None, :]
    l = np.take_along_axis(l_all, idx, axis=1)        # [T][K]
    ls = -np.sort(-l, axis=1)
    m = min(k + 1, K)
    for a in range(m - 1):
        gap = np.minimum(gap, ls[:, a] - ls[:, a + 1])
    return gap, c


def _zipf_bias(x16, rc16, G, s=1.0, iters=200):
    """Bias on the cluster logits so that the cluster loads follow Zipf(s)."""
    target = 1.0 / np.arange(1, G + 1) ** s
    target /= target.sum()
    z = x16.astype(np.float64) @ rc16.astype(np.float64).T
    bias = np.zeros(G)
    for _ in range(iters):
        load = np.bincount(np.argmax(z + bias[None, :], axis=1), minlength=G) / len(z)
        if np.abs(load - target).max() < 2e-3:
            break
        bias += 0.5 * np.log(target / np.maximum(load, 1e-6))
        bias -= bias.mean()
    return bias.astype(np.float32)


# --------------------------------------------------------------------------
# generator
# --------------------------------------------------------------------------
def _normal16(rng, shape, std):
    out = np.empty(shape, dtype=np.float16)
    flat = out.reshape(shape[0], -1)
    for i in range(shape[0]):                      # slab-wise: bounded temporaries
        flat[i] = (rng.standard_normal(flat.shape[1], dtype=np.float32) * np.float32(std)).astype(np.float16)
    return out


def generate(cfg: LayerConfig, with_weights: bool = True) -> Dict[str, Optional[np.ndarray]]:
    """Draw all tensors of one layer call.  One random sub-stream per tensor, in
    the fixed order x, router_cluster, router_expert, w1_base, w2_base, v1, u1,
    v2, u2 (so a tensor does not change when another one's shape does)."""
    T, d, d_ff, G, K, r, k, q = cfg.T, cfg.d, cfg.d_ff, cfg.G, cfg.K, cfg.r, cfg.k, cfg.q
    E = G * K
    ss = np.random.SeedSequence(cfg.seed).spawn(9)
    rngs = [np.random.Generator(np.random.PCG64(s)) for s in ss]
    out: Dict[str, Optional[np.ndarray]] = {}

    rx = rngs[0]
    x = rx.standard_normal((T, d), dtype=np.float32).astype(np.float16)
    rc = (rngs[1].standard_normal((G, d)) / np.sqrt(d)).astype(np.float16)
    re = (rngs[2].standard_normal((E, d)) / np.sqrt(d)).astype(np.float16)

    bias = None
    if cfg.router == "zipf":
        bias = _zipf_bias(x, rc, G)

    # redraw tokens whose routing would hinge on a near-tie (or, for "all_hit",
    # redraw everything until every cluster receives a token)
    for _ in range(1000):
        gap, c = _logit_gaps(x, rc, re, bias, K, k)
        bad = np.nonzero(gap < MARGIN)[0]
        if len(bad):
            x[bad] = rx.standard_normal((len(bad), d), dtype=np.float32).astype(np.float16)
            continue
        if cfg.router == "all_hit" and T >= G and len(np.unique(c)) < G:
            x = rx.standard_normal((T, d), dtype=np.float32).astype(np.float16)
            continue
        break
    else:
        raise RuntimeError("could not condition the router inputs")

    out.update(x=x, router_cluster=rc, router_expert=re, cluster_bias=bias)
    if not with_weights:
        return out

    out["w1_base"] = _normal16(rngs[3], (G, d_ff, d), 1.0 / np.sqrt(d))
    out["w2_base"] = _normal16(rngs[4], (G, d, d_ff), 1.0 / np.sqrt(d_ff))
    for name, rng, L in (("v1", rngs[5], d), ("u1", rngs[6], d_ff), ("v2", rngs[7], d_ff), ("u2", rngs[8], d)):
        w = rng.standard_normal((E, r, L), dtype=np.float32) * np.float32(cfg.factor_std)
        out[name + "_q"], out[name + "_s"] = quantize_int4(w, q)
    return out


def generate_dense_experts(G: int, K: int, out_dim: int, in_dim: int, rank: int, residual_rel: float,
                           noise_rel: float, seed: int, decay: float = 0.8) -> np.ndarray:
    """Dense expert matrices with the structure the compression assumes (Sec. 3.1, 3.2: experts
    of a cluster are correlated): W_e = B_c + residual_rel * L_e + noise_rel * N_e, float16
    [G*K][out][in].  B_c ~ N(0, 1/in_dim) is common to the cluster, L_e is a rank-`rank`
    matrix with geometrically decaying singular values, N_e is white noise; L_e and N_e are
    scaled to Frobenius norm ||B_c||.  (The low-rank product below only shapes the data.)"""
    rng = np.random.default_rng(np.random.SeedSequence(seed))
    W = np.empty((G * K, out_dim, in_dim), dtype=np.float16)
    for c in range(G):
        B = rng.standard_normal((out_dim, in_dim)) / np.sqrt(in_dim)
        nb = np.linalg.norm(B)
        for j in range(K):
            P = rng.standard_normal((out_dim, rank)) * (decay ** np.arange(rank))
            L = P @ rng.standard_normal((rank, in_dim))
            N = rng.standard_normal((out_dim, in_dim))
            W[c * K + j] = (B + residual_rel * nb * L / np.linalg.norm(L)
                            + noise_rel * nb * N / np.linalg.norm(N)).astype(np.float16)
    return W


def sketch_rows(sketch: int, in_dim: int, seed: int) -> np.ndarray:
    """Gaussian test rows of the randomised range finder, float16 [sketch][in_dim]."""
    rng = np.random.default_rng(np.random.SeedSequence(seed))
    return rng.standard_normal((sketch, in_dim)).astype(np.float16)


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# closed-form work model of the method (used by bench and tests, Sec. 3.2/3.3)
# --------------------------------------------------------------------------
def flops_per_token(cfg: LayerConfig) -> Dict[str, int]:
    base = 4 * cfg.d * cfg.d_ff
    resid = cfg.k * 4 * cfg.r * (cfg.d + cfg.d_ff)
    router = 2 * cfg.d * (cfg.G + cfg.K)
    return dict(base=base, residual=resid, router=router, total=base + resid + router)


def algorithmic_bytes(cfg: LayerConfig, clusters_hit: Optional[int] = None, experts_hit: Optional[int] = None) -> Dict[str, int]:
    G = cfg.G if clusters_hit is None else clusters_hit
    E = cfg.E if experts_hit is None else experts_hit
    bases = G * 2 * cfg.d * cfg.d_ff * 2
    per_expert = 2 * cfg.r * (cfg.d + cfg.d_ff)            # INT4 elements of the four factors
    factors = E * (per_expert // 2 + 2 * per_expert // cfg.q)
    routers = (cfg.G + cfg.E) * cfg.d * 2
    xy = 2 * cfg.T * cfg.d * 2
    return dict(bases=bases, factors=factors, routers=routers, xy=xy, total=bases + factors + routers + xy)
