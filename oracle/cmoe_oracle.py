"""FP64 CPU oracle of the clustered, compressed MoE FFN layer forward.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests, the smoke check and the bench's CPU-baseline leg do.  It shares no
code with the HIP library and never receives a value computed by it.

What it computes (every function names the passage it follows):

  * the expert weights are a per-cluster shared base plus a rank-r product of two
    factors, W_e = W_base(c) + U_e V_e                      (Sec. 3.2, Eq. 7);
  * the factors are stored as INT4 codes with one FP16 scale per group of q
    consecutive codes; bases and routers are FP16           (Sec. 3.4);
  * routing is two-stage: cluster logits z_g = u_g . x, the cluster with the
    largest softmax probability wins (Eq. 9); inside it, logits l_i = v_i . x,
    softmax over the cluster (Eq. 10), the k most probable experts are kept
    (Sec. 3.3);
  * the layer output is the gate-weighted sum of the k selected experts'
    two-matrix GELU FFNs.

`forward_naive` is the plain definition: every expert matrix is materialised
densely and each selected expert's FFN is evaluated on its own.  `ffn_rewrite`
is the same function in the method's cheaper form (base product once per token,
Sec. 3.2 after Eq. 7; second matrix by linearity) and also returns the
intermediates the HIP path exposes.  All arithmetic is float64 on the exact
values of the FP16 / INT4 inputs.  numpy's float64 `@` is used as the matrix
product primitive; nothing is blocked, fused or reordered beyond that.

Readings where the paper is silent (also listed in the design notes):
  - FFN form: y_e = W2_e GELU(W1_e x), no biases, GELU(u) = u/2 (1 + erf(u/sqrt 2)).
  - W is out x in, y = W x; U_e is out x r, V_e is r x in; both factors are
    stored rank-major [r][long dimension].
  - Gates: softmax over the k selected in-cluster logits (equivalently the Eq. 10
    probabilities of the selected experts renormalised to sum to one); the cluster
    probability does not scale the output.
  - Ties: the lowest index wins; the k experts are listed by descending logit.
  - INT4: symmetric two's-complement codes in [-8, 7], value = scale * code, no
    zero point; element n in byte n // 2, even n in the low nibble.
  - An optional per-cluster bias may be added to the cluster logits (used only to
    skew cluster loads in one benchmark configuration; None = the paper's form).

Parity pins: see tests/test_oracle_pins.py.  The end-to-end output on the large
configurations has no external value to pin to (the paper prints none): it is
pinned through the naive-vs-rewrite identity, brute-force scalar loops on tiny
inputs, and special cases that reduce to a dense FFN written with math.erf.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf


# ---------------------------------------------------------------- Sec. 3.4
def unpack_int4(packed: np.ndarray) -> np.ndarray:
    """uint8 [..., L/2] -> integer codes [..., L] in [-8, 7] (float64)."""
    lo = (packed & 0x0F).astype(np.int16)
    hi = (packed >> 4).astype(np.int16)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.float64)
    out[..., 0::2] = lo
    out[..., 1::2] = hi
    return out


def dequant_int4(packed: np.ndarray, scales: np.ndarray, q: int) -> np.ndarray:
    """Stored factor -> float64 [..., L]: value[n] = scale[n // q] * code[n]  (Sec. 3.4)."""
    codes = unpack_int4(packed)
    s = np.repeat(scales.astype(np.float64), q, axis=-1)
    assert s.shape == codes.shape
    return s * codes


# ---------------------------------------------------------------- Sec. 3.3
def route(x, router_cluster, router_expert, K, k, cluster_bias=None):
    """Two-stage routing (Sec. 3.3, Eq. 9 and Eq. 10).

    Returns cluster_id [T] int32, expert_idx [T][k] int32 (global slot c*K + j,
    descending logit), gate [T][k] float64, and the logits (z [T][G], l [T][K]).
    """
    X = x.astype(np.float64)
    U = router_cluster.astype(np.float64)
    V = router_expert.astype(np.float64)
    T = X.shape[0]
    z = X @ U.T
    if cluster_bias is not None:
        z = z + cluster_bias.astype(np.float64)[None, :]
    # Eq. 9: p_g = softmax(z)_g; the largest p_g is the largest z_g.  argmax
    # returns the first maximum = lowest index on ties.
    cluster_id = np.argmax(_rank_key(z), axis=1).astype(np.int32)
    l = np.empty((T, K), dtype=np.float64)
    for c in range(U.shape[0]):
        rows = np.nonzero(cluster_id == c)[0]
        if len(rows):
            l[rows] = X[rows] @ V[c * K:(c + 1) * K].T
    # Eq. 10 then top-k: stable sort of -l lists equal logits by ascending index
    order = np.argsort(-_rank_key(l), axis=1, kind="stable")[:, :k]
    lsel = np.take_along_axis(l, order, axis=1)
    ex = np.exp(lsel - lsel[:, :1])
    gate = ex / ex.sum(axis=1, keepdims=True)
    expert_idx = (cluster_id[:, None].astype(np.int64) * K + order).astype(np.int32)
    return cluster_id, expert_idx, gate, z, l


def _rank_key(logits):
    """Sec. 3.3 ranks finite logits and says nothing about NaN.  Reading taken: a NaN ranks
    below every number (as -inf), equal ranks go to the lowest index, so a selection always
    names distinct experts of one cluster whatever the inputs hold."""
    return np.where(np.isnan(logits), -np.inf, logits)


def route_multi(x, router_cluster, router_expert, K, k, top_g=1, temperature=1.0, scale_by_cluster_prob=False,
                cluster_bias=None):
    """Routing variants of Sec. 3.3 / 3.5: the top_g most probable clusters are kept (Eq. 9,
    "Top-g_1 groups"), each contributes its own top-k experts (Eq. 10), and both softmaxes
    take logits divided by the router temperature (Sec. 3.5).

    Cluster weight w_a: p_g of Eq. 9 itself when scale_by_cluster_prob, else p_g renormalised
    over the selected clusters (1 for top_g = 1).  gate[t][a][j] = w_a * softmax over the k
    selected in-cluster logits / temperature.  Selection does not depend on the temperature.
    Returns cluster_ids [T][top_g] int32 (descending probability, lowest index on ties),
    expert_idx [T][top_g][k] int32, gate [T][top_g][k] float64, p [T][G] float64."""
    X = x.astype(np.float64)
    U = router_cluster.astype(np.float64)
    V = router_expert.astype(np.float64)
    T, G = X.shape[0], U.shape[0]
    z = X @ U.T
    if cluster_bias is not None:
        z = z + cluster_bias.astype(np.float64)[None, :]
    zt = z / temperature
    pe = np.exp(zt - zt.max(axis=1, keepdims=True))
    p = pe / pe.sum(axis=1, keepdims=True)
    cluster_ids = np.argsort(-_rank_key(z), axis=1, kind="stable")[:, :top_g].astype(np.int32)
    psel = np.take_along_axis(p, cluster_ids.astype(np.int64), axis=1)
    wgt = psel if scale_by_cluster_prob else psel / psel.sum(axis=1, keepdims=True)
    expert_idx = np.empty((T, top_g, k), dtype=np.int32)
    gate = np.empty((T, top_g, k), dtype=np.float64)
    for a in range(top_g):
        for c in range(G):
            rows = np.nonzero(cluster_ids[:, a] == c)[0]
            if len(rows) == 0:
                continue
            l = X[rows] @ V[c * K:(c + 1) * K].T
            order = np.argsort(-_rank_key(l), axis=1, kind="stable")[:, :k]
            lsel = np.take_along_axis(l, order, axis=1) / temperature
            ex = np.exp(lsel - lsel[:, :1])
            gate[rows, a] = wgt[rows, a][:, None] * ex / ex.sum(axis=1, keepdims=True)
            expert_idx[rows, a] = c * K + order
    return cluster_ids, expert_idx, gate, p


def forward_naive_multi(w, x, K, k, q, top_g=1, temperature=1.0, scale_by_cluster_prob=False):
    """The layer with the routing variants: the dense FFNs of all top_g * k selected experts,
    mixed with the gates of route_multi."""
    cluster_ids, expert_idx, gate, _ = route_multi(x, w["router_cluster"], w["router_expert"], K, k, top_g,
                                                   temperature, scale_by_cluster_prob, w.get("cluster_bias"))
    T = x.shape[0]
    y = ffn_naive(w, x, expert_idx.reshape(T, top_g * k), gate.reshape(T, top_g * k), K, q)
    return dict(cluster_ids=cluster_ids, expert_idx=expert_idx, gate=gate, y=y)


def permute(cluster_id, G):
    """Stable counting sort of token indices by cluster (the single-device part of
    group-level dispatch, Sec. 3.3).  Returns offsets [G+1], perm [T], inv_perm [T]."""
    T = len(cluster_id)
    counts = [0] * G
    for t in range(T):
        counts[int(cluster_id[t])] += 1
    offsets = [0] * (G + 1)
    for c in range(G):
        offsets[c + 1] = offsets[c] + counts[c]
    cursor = list(offsets[:G])
    perm = np.empty(T, dtype=np.int32)
    inv_perm = np.empty(T, dtype=np.int32)
    for t in range(T):
        c = int(cluster_id[t])
        perm[cursor[c]] = t
        inv_perm[t] = cursor[c]
        cursor[c] += 1
    return np.asarray(offsets, dtype=np.int32), perm, inv_perm


# ---------------------------------------------------------------- Sec. 3.2
def gelu(u):
    return 0.5 * u * (1.0 + _erf(u / np.sqrt(2.0)))


def _factors(w, q):
    return {n: dequant_int4(w[n + "_q"], w[n + "_s"], q) for n in ("v1", "u1", "v2", "u2")}


def expert_weights(w, e, K, q, f=None):
    """Dense W1_e [d_ff][d] and W2_e [d][d_ff] of expert slot e (Eq. 7):
    W_e = W_base(c) + U_e V_e with U_e = u[e].T (out x r) and V_e = v[e] (r x in)."""
    f = f if f is not None else _factors(w, q)
    c = e // K
    W1 = w["w1_base"][c].astype(np.float64) + f["u1"][e].T @ f["v1"][e]
    W2 = w["w2_base"][c].astype(np.float64) + f["u2"][e].T @ f["v2"][e]
    return W1, W2


def ffn_naive(w, x, expert_idx, gate, K, q):
    """y[t] = sum_j gate[t][j] * W2_e GELU(W1_e x[t]),  e = expert_idx[t][j].  Each
    expert matrix is materialised (Eq. 7) and applied to the tokens that chose it."""
    X = x.astype(np.float64)
    T, d = X.shape
    k = expert_idx.shape[1]
    y = np.zeros((T, d), dtype=np.float64)
    f = _factors(w, q)
    for e in np.unique(expert_idx):
        W1, W2 = expert_weights(w, int(e), K, q, f)
        for j in range(k):
            rows = np.nonzero(expert_idx[:, j] == e)[0]
            if len(rows) == 0:
                continue
            h = X[rows] @ W1.T
            y[rows] += gate[rows, j][:, None] * (gelu(h) @ W2.T)
    return y


def ffn_dense(W1, W2, x, expert_idx, gate):
    """The uncompressed layer the method starts from: y[t] = sum_j gate[t][j] W2_e GELU(W1_e x[t])
    with dense expert matrices W1 [E][d_ff][d], W2 [E][d][d_ff]."""
    X = x.astype(np.float64)
    y = np.zeros((X.shape[0], W2.shape[1]), dtype=np.float64)
    for e in np.unique(expert_idx):
        A, B = W1[int(e)].astype(np.float64), W2[int(e)].astype(np.float64)
        for j in range(expert_idx.shape[1]):
            rows = np.nonzero(expert_idx[:, j] == e)[0]
            if len(rows):
                y[rows] += gate[rows, j][:, None] * (gelu(X[rows] @ A.T) @ B.T)
    return y


def forward_naive(w, x, K, k, q):
    """The layer by its definition: route, then the selected experts' dense FFNs."""
    G = w["router_cluster"].shape[0]
    cluster_id, expert_idx, gate, _, _ = route(x, w["router_cluster"], w["router_expert"], K, k, w.get("cluster_bias"))
    y = ffn_naive(w, x, expert_idx, gate, K, q)
    offsets, perm, inv_perm = permute(cluster_id, G)
    return dict(cluster_id=cluster_id, expert_idx=expert_idx, gate=gate, offsets=offsets, perm=perm,
                inv_perm=inv_perm, y=y)


def ffn_rewrite(w, x, perm, offsets, expert_idx, gate, K, q):
    """The same function in the method's form (Sec. 3.2: the base product is shared by
    all experts of the cluster that see the token; by linearity of the second base
    matrix the gate-weighted sum is taken before it):

      Hb  = W1_base(c) x                    t1_j = V1_e x
      a_j = GELU(Hb + U1_e t1_j)            A    = sum_j g_j a_j
      s_j = V2_e a_j                        y    = W2_base(c) A + sum_j g_j U2_e s_j

    Rows of Hb, A, y_base_sorted, y_sorted are in cluster-sorted order (row p is
    token perm[p]); t1 and s are [T][k][r] in token order.
    """
    X = x.astype(np.float64)
    T, d = X.shape
    k = expert_idx.shape[1]
    G = len(offsets) - 1
    f = _factors(w, q)
    r = f["v1"].shape[1]
    d_ff = w["w1_base"].shape[1]
    Hb = np.zeros((T, d_ff))
    A = np.zeros((T, d_ff))
    t1 = np.zeros((T, k, r))
    s = np.zeros((T, k, r))
    y_base_sorted = np.zeros((T, d))
    y_sorted = np.zeros((T, d))
    for c in range(G):
        lo, hi = int(offsets[c]), int(offsets[c + 1])
        if hi == lo:
            continue
        toks = perm[lo:hi]
        Hb[lo:hi] = X[toks] @ w["w1_base"][c].astype(np.float64).T
    for p in range(T):
        t = int(perm[p])
        for j in range(k):
            e = int(expert_idx[t, j])
            t1[t, j] = f["v1"][e] @ X[t]
            a = gelu(Hb[p] + f["u1"][e].T @ t1[t, j])
            A[p] += gate[t, j] * a
            s[t, j] = f["v2"][e] @ a
    for c in range(G):
        lo, hi = int(offsets[c]), int(offsets[c + 1])
        if hi == lo:
            continue
        y_base_sorted[lo:hi] = A[lo:hi] @ w["w2_base"][c].astype(np.float64).T
    y = np.zeros((T, d))
    for p in range(T):
        t = int(perm[p])
        acc = y_base_sorted[p].copy()
        for j in range(k):
            e = int(expert_idx[t, j])
            acc += gate[t, j] * (f["u2"][e].T @ s[t, j])
        y_sorted[p] = acc
        y[t] = acc
    return dict(Hb=Hb, t1=t1, A=A, s=s, y_base_sorted=y_base_sorted, y_sorted=y_sorted, y=y)



# ---------------------------------------------------------------- backward pass (training, Sec. 3.5)
# Gradients of the layer output for a given routing.  The expert choice is piecewise constant
# in x and in the router weights, so it carries no gradient; the gates do (softmax over the
# selected in-cluster logits).  Factors are differentiated as the real-valued matrices they
# dequantise to.  With W_e = W_base(c) + U_e V_e (Eq. 7):
#   dW_base(c) = sum over the cluster's experts of dW_e,  dU_e = dW_e V_e^T,  dV_e = U_e^T dW_e.
def gelu_grad(u):
    """d/du [u Phi(u)] = Phi(u) + u phi(u), Phi / phi the standard normal CDF / density."""
    u = np.asarray(u, dtype=np.float64)
    return 0.5 * (1.0 + _erf(u / np.sqrt(2.0))) + u * np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)


def backward_naive(w, x, dy, expert_idx, gate, K, q):
    """Gradients of L = sum(dy * y), y the layer output for the given selection (expert_idx
    [T][k], gate [T][k] = softmax over the selected logits), by the chain rule on dense
    per-expert matrices.  Returns dx [T][d], d_router_expert [E][d], dw1_base [G][d_ff][d],
    dw2_base [G][d][d_ff], and per expert du1 [E][r][d_ff], dv1 [E][r][d], du2 [E][r][d],
    dv2 [E][r][d_ff] in the stored (rank-major) orientation.  float64."""
    X = np.asarray(x, dtype=np.float64)
    DY = np.asarray(dy, dtype=np.float64)
    T, d = X.shape
    k = expert_idx.shape[1]
    G = w["w1_base"].shape[0]
    d_ff = w["w1_base"].shape[1]
    E = G * K
    f = _factors(w, q)
    r = f["u1"].shape[1]
    RE = w["router_expert"].astype(np.float64)
    dx = np.zeros((T, d))
    d_re = np.zeros((E, d))
    dW1 = np.zeros((E, d_ff, d))
    dW2 = np.zeros((E, d, d_ff))
    dg = np.zeros((T, k))
    for e in np.unique(expert_idx):
        e = int(e)
        W1, W2 = expert_weights(w, e, K, q, f)
        for j in range(k):
            rows = np.nonzero(expert_idx[:, j] == e)[0]
            if len(rows) == 0:
                continue
            h = X[rows] @ W1.T                       # [n][d_ff]
            a = gelu(h)
            o = a @ W2.T                             # [n][d]
            dg[rows, j] = (DY[rows] * o).sum(axis=1)
            do = gate[rows, j][:, None] * DY[rows]
            da = do @ W2
            dh = da * gelu_grad(h)
            dx[rows] += dh @ W1
            dW2[e] += do.T @ a
            dW1[e] += dh.T @ X[rows]
    # gates: g = softmax(l_sel); dl_j = g_j (dg_j - sum_i g_i dg_i); l_j = v_{e_j} . x
    dl = gate * (dg - (gate * dg).sum(axis=1, keepdims=True))
    for j in range(k):
        ej = expert_idx[:, j].astype(np.int64)
        dx += dl[:, j][:, None] * RE[ej]
        np.add.at(d_re, ej, dl[:, j][:, None] * X)
    dw1_base = dW1.reshape(G, K, d_ff, d).sum(axis=1)
    dw2_base = dW2.reshape(G, K, d, d_ff).sum(axis=1)
    du1 = np.zeros((E, r, d_ff)); dv1 = np.zeros((E, r, d)); du2 = np.zeros((E, r, d)); dv2 = np.zeros((E, r, d_ff))
    for e in np.unique(expert_idx):     # an expert without tokens has dW = 0 whatever its factors hold
        e = int(e)
        U1, V1, U2, V2 = f["u1"][e].T, f["v1"][e], f["u2"][e].T, f["v2"][e]     # U [out][r], V [r][in]
        du1[e] = (dW1[e] @ V1.T).T
        dv1[e] = U1.T @ dW1[e]
        du2[e] = (dW2[e] @ V2.T).T
        dv2[e] = U2.T @ dW2[e]
    return dict(dx=dx, d_router_expert=d_re, dw1_base=dw1_base, dw2_base=dw2_base, du1=du1, dv1=dv1, du2=du2,
                dv2=dv2, dgate_logits=dl)


def backward_sampled(w, x, dy, expert_idx, gate, K, q, tokens, hidden):
    """The part of backward_naive that can be computed one by one at any size, by the same
    chain rule on materialised expert matrices (Eq. 7):
      dx [len(tokens)][d], dgate_logits [len(tokens)][k]   of the given tokens (each depends
          on its own token only);
      for the given hidden indices n (rows of W1_e, columns of W2_e), whose h and da columns
      over all tokens cost one matrix-vector product each:
          dw1_base [G][len(hidden)][d], dw2_base [G][d][len(hidden)],
          du1 [E][r][len(hidden)], dv2 [E][r][len(hidden)].
    float64."""
    X = np.asarray(x, dtype=np.float64)
    DY = np.asarray(dy, dtype=np.float64)
    tokens = np.asarray(tokens, dtype=np.int64)
    hidden = np.asarray(hidden, dtype=np.int64)
    T, d = X.shape
    k = expert_idx.shape[1]
    G = w["w1_base"].shape[0]
    E = G * K
    f = _factors(w, q)
    r = f["u1"].shape[1]
    RE = w["router_expert"].astype(np.float64)
    nt, nh = len(tokens), len(hidden)
    dx = np.zeros((nt, d))
    dg = np.zeros((nt, k))
    dw1 = np.zeros((G, nh, d)); dw2 = np.zeros((G, d, nh))
    du1 = np.zeros((E, r, nh)); dv2 = np.zeros((E, r, nh))
    e_tok = expert_idx[tokens]
    for e in np.unique(expert_idx):
        e = int(e)
        c = e // K
        # sampled tokens: the whole chain through the dense matrices of this expert
        if np.any(e_tok == e):
            W1, W2 = expert_weights(w, e, K, q, f)
            for j in range(k):
                sel = np.nonzero(e_tok[:, j] == e)[0]
                if len(sel) == 0:
                    continue
                rows = tokens[sel]
                h = X[rows] @ W1.T
                a = gelu(h)
                dg[sel, j] = (DY[rows] * (a @ W2.T)).sum(axis=1)
                dh = ((gate[rows, j][:, None] * DY[rows]) @ W2) * gelu_grad(h)
                dx[sel] += dh @ W1
        # sampled hidden units: row n of W1_e and column n of W2_e against every pair of e
        tt, jj = np.nonzero(expert_idx == e)
        Xe = X[tt]
        DOe = gate[tt, jj][:, None] * DY[tt]
        w1rows = w["w1_base"][c][hidden].astype(np.float64) + f["u1"][e][:, hidden].T @ f["v1"][e]      # [nh][d]
        w2cols = w["w2_base"][c][:, hidden].astype(np.float64) + f["u2"][e].T @ f["v2"][e][:, hidden]   # [d][nh]
        h = Xe @ w1rows.T                    # [n_e][nh]
        dh = (DOe @ w2cols) * gelu_grad(h)
        dW1 = dh.T @ Xe                      # rows `hidden` of dW1_e
        dW2 = DOe.T @ gelu(h)                # columns `hidden` of dW2_e
        dw1[c] += dW1
        dw2[c] += dW2
        du1[e] = f["v1"][e] @ dW1.T
        dv2[e] = f["u2"][e] @ dW2
    gt = gate[tokens]
    dl = gt * (dg - (gt * dg).sum(axis=1, keepdims=True))
    for j in range(k):
        dx += dl[:, j][:, None] * RE[e_tok[:, j].astype(np.int64)]
    return dict(dx=dx, dgate_logits=dl, dw1_base=dw1, dw2_base=dw2, du1=du1, dv2=dv2)


# ---------------------------------------------------------------- compression (Sec. 3.2, 3.4)
# Construction of the stored form from dense expert matrices W_e [out][in]: the base of a
# cluster is the mean of its experts (Eq. 6), each expert keeps a rank-r factorisation of
# its residual (Eq. 7; the truncated SVD is the best one, Sec. 3.2), the factors are
# quantised to INT4 with one FP16 scale per q codes (Sec. 3.4), and an optional gate zeroes
# the residual of an expert whose cosine similarity to the base is below a threshold
# (Sec. 3.4).
def base_mean(W, G, K):
    """Eq. 6.  W [G*K][out][in] float16 -> base [G][out][in] float16.  The stored value is an
    FP16 rounding, so the sum is taken the way the kernel takes it: FP32, experts in index
    order, divided by K, rounded to nearest even."""
    W = np.asarray(W)
    base = np.empty((G,) + W.shape[1:], dtype=np.float16)
    for c in range(G):
        acc = np.zeros(W.shape[1:], dtype=np.float32)
        for j in range(K):
            acc = acc + W[c * K + j].astype(np.float32)
        base[c] = (acc / np.float32(K)).astype(np.float16)
    return base


def residual(W_e, base_c):
    """Delta W_e = W_e - W_base(c) (Eq. 7), float64, against the STORED (FP16) base."""
    return np.asarray(W_e, dtype=np.float64) - np.asarray(base_c, dtype=np.float64)


def truncated_svd_factors(delta, r):
    """Best rank-r factors of the residual (Sec. 3.2): delta ~ U V with U [out][r] (left
    singular vectors times singular values) and V [r][in]; also the optimal Frobenius error
    sqrt(sum_{i > r} sigma_i^2) and the singular values."""
    u, sv, vt = np.linalg.svd(np.asarray(delta, dtype=np.float64), full_matrices=False)
    U = u[:, :r] * sv[:r]
    V = vt[:r]
    return U, V, float(np.sqrt((sv[r:] ** 2).sum())), sv


def quantize_int4_f32(w, q):
    """Sec. 3.4 quantiser of a factor row block, decisions in FP32 as the kernel takes them:
    scale = fp16(absmax / 7) per group of q consecutive elements (absmax / 7 in FP32, rounded
    to nearest even); code = clip(rint(w / scale), -7, 7) with the division in FP32 and ties
    to even; a group whose scale rounds to 0 gets codes 0.
    w [..., L] float32 -> (packed uint8 [..., L/2], scales float16 [..., L/q])."""
    w = np.asarray(w, dtype=np.float32)
    L = w.shape[-1]
    g = w.reshape(w.shape[:-1] + (L // q, q))
    absmax = np.abs(g).max(axis=-1)
    scale = (absmax / np.float32(7.0)).astype(np.float16)
    s32 = scale.astype(np.float32)
    safe = np.where(s32 > 0, s32, np.float32(1.0))
    codes = np.clip(np.rint(g / safe[..., None]), -7, 7).astype(np.int16)
    codes = np.where(s32[..., None] > 0, codes, 0).reshape(w.shape)
    u = (codes & 0xF).astype(np.uint8)
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8), scale


def cosine_to_base(delta, base_c):
    """Cosine similarity of vec(Delta W_e) and vec(W_base(c)) (the gate of Sec. 3.4); 0 if
    either is zero."""
    a = np.asarray(delta, dtype=np.float64).reshape(-1)
    b = np.asarray(base_c, dtype=np.float64).reshape(-1)
    den = np.sqrt((a * a).sum()) * np.sqrt((b * b).sum())
    return float((a * b).sum() / den) if den > 0 else 0.0


def reconstruction_error(W_e, base_c, U, V):
    """|| W_e - (W_base(c) + U V) ||_F / || W_e ||_F: the relative Frobenius reconstruction
    error of Sec. 3.2.  U [out][r], V [r][in] are the values the layer would use."""
    W_e = np.asarray(W_e, dtype=np.float64)
    diff = W_e - np.asarray(base_c, dtype=np.float64) - np.asarray(U, dtype=np.float64) @ np.asarray(V, dtype=np.float64)
    return float(np.sqrt((diff * diff).sum()) / np.sqrt((W_e * W_e).sum()))


# ---------------------------------------------------------------- routing statistics
# By-products of one routing step that the method's control loops consume: expert loads
# and their coefficient of variation (Sec. 4, evaluation metrics), the activation
# centroids of the experts (Sec. 3.1, Eq. 5) and the per-cluster activity that drives
# offloading and prefetch (Sec. 3.4).
def expert_loads(expert_idx, E):
    """n_e = number of (token, slot) assignments to expert e in this step: a token counts
    once for each of its k selected experts.  int64 [E]."""
    loads = np.zeros(E, dtype=np.int64)
    for e in np.asarray(expert_idx).reshape(-1):
        loads[int(e)] += 1
    return loads


def load_cv(loads):
    """I_load: standard deviation of the expert loads over their mean (Sec. 4).  The
    deviation is taken over the E experts as a population (divide by E); 0 if no token."""
    n = np.asarray(loads, dtype=np.float64)
    mean = n.sum() / n.size
    if mean == 0.0:
        return 0.0
    var = ((n - mean) ** 2).sum() / n.size
    return float(np.sqrt(var) / mean)


def centroid_ema(mu, x, expert_idx, beta):
    """Eq. 5: mu_e <- (1 - beta) mu_e + beta xbar_e with xbar_e the mean embedding of the
    tokens assigned to expert e in this step; experts that received no token keep mu_e."""
    mu = np.array(mu, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    expert_idx = np.asarray(expert_idx)
    for e in range(mu.shape[0]):
        rows = np.nonzero((expert_idx == e).any(axis=1))[0]
        if rows.size == 0:
            continue
        xbar = x[rows].sum(axis=0) / rows.size
        mu[e] = (1.0 - beta) * mu[e] + beta * xbar
    return mu


def cluster_activity(act, idle, cluster_id, G, lam):
    """Sec. 3.4: s_g = 1 if cluster g received a token in this step, else 0;
    act_g <- (1 - lam) act_g + lam s_g (the rolling predictor of a cluster being
    selected); idle_g = number of consecutive steps without a token (0 after a hit).
    Returns (act float64 [G], idle int64 [G], tokens per cluster int64 [G])."""
    counts = np.zeros(G, dtype=np.int64)
    for c in np.asarray(cluster_id).reshape(-1):
        counts[int(c)] += 1
    hit = counts > 0
    act = (1.0 - lam) * np.asarray(act, dtype=np.float64) + lam * hit.astype(np.float64)
    idle = np.where(hit, 0, np.asarray(idle, dtype=np.int64) + 1)
    return act, idle, counts

# ---------------------------------------------------------------- closed forms
def storage_elements_per_group(d_in, d_out, K, r):
    """Stored elements of one cluster's weight matrix after compression (Sec. 3.2)."""
    return d_in * d_out + K * r * (d_in + d_out)


def compression_ratio(d_in, d_out, K, r):
    """Eq. 8."""
    return K * d_in * d_out / storage_elements_per_group(d_in, d_out, K, r)


def routing_flops_per_token(d, G, K):
    """Two dot products of length d per logit, G + K logits (Sec. 3.3)."""
    return 2 * d * (G + K)


# ---------------------------------------------------------------- error metrics
def error_metrics(y, y_ref):
    """max|y - y_ref| / RMS(y_ref) and sum|y - y_ref| / sum|y_ref| (the two bars)."""
    y = np.asarray(y, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    diff = np.abs(y - y_ref)
    rms = np.sqrt(np.mean(y_ref ** 2))
    return dict(max_over_rms=float(diff.max() / rms) if diff.size else 0.0,
                mean_rel=float(diff.sum() / np.abs(y_ref).sum()) if diff.size else 0.0,
                rms=float(rms))
