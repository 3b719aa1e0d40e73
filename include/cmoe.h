/*
 * cmoe.h -- C ABI of the clustered, compressed Mixture-of-Experts FFN layer for AMD MI355X
 * (gfx950): forward pass, routing variants and statistics, construction of the stored form
 * from dense experts, and the backward pass.
 *
 * The layer (notation of the paper, arXiv 2510.02345):
 *   - E = G*K experts are organised in G clusters of uniform size K (Sec. 3.1).
 *   - Every expert weight matrix is a per-cluster shared base plus a rank-r residual,
 *     W_e = W_base(c) + U_e V_e (Sec. 3.2, Eq. 7).  Bases are FP16, the factors are
 *     INT4 codes with one FP16 scale per group of q_group consecutive codes (Sec. 3.4).
 *   - A token x in R^d is routed in two stages (Sec. 3.3): cluster logits z_g = u_g.x,
 *     softmax (Eq. 9), the most probable cluster c wins; in-cluster logits l_i = v_i.x,
 *     softmax over the cluster (Eq. 10), the top_k most probable experts are selected
 *     and their probabilities renormalised to gates that sum to one.
 *   - y = sum_j gate_j * W2_{e_j} GELU(W1_{e_j} x), evaluated with the base products
 *     shared (Sec. 3.2, the sentence after Eq. 7): W1_base(c) x is computed once per
 *     token, and by linearity W2_base(c) (sum_j gate_j a_j) once per token.
 *
 * Conventions
 *   - Every pointer named in cmoe_weights and every tensor argument is a DEVICE
 *     pointer owned by the caller, 16-byte aligned, valid until the stream has
 *     finished the call.  cmoe_config / cmoe_weights structs themselves are HOST memory
 *     and are read before the call returns.
 *   - Calls only enqueue work on the given hipStream_t (passed as void*; NULL = the
 *     default stream); they never synchronise, never read device memory from the host
 *     and never allocate or free device memory.  Outputs are valid once the stream
 *     has been synchronised.
 *   - All matrices are row-major; "cmoe_f16" is the bit pattern of an IEEE binary16.
 *   - Every function returns CMOE_OK (0) or a negative error code; argument checks are
 *     done before any HIP call, so a rejected call has no side effect.  T = 0 is a
 *     valid no-op.  Weights of a cluster that receives no token are never read.
 *   - Indices are int32.  expert_idx holds global expert slots c*K + j.
 *   - Tie-break everywhere: the lowest index wins; the top_k experts are listed by
 *     descending logit.
 */
#ifndef CMOE_H
#define CMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t cmoe_f16;

enum {
  CMOE_OK = 0,
  CMOE_ERR_INVALID_ARG = -1, /* NULL / misaligned pointer, negative size, bad handle          */
  CMOE_ERR_UNSUPPORTED = -2, /* a shape outside the supported set (see cmoe_create)           */
  CMOE_ERR_WORKSPACE = -3,   /* workspace NULL, misaligned or smaller than cmoe_workspace_bytes */
  CMOE_ERR_HIP = -4          /* a HIP call failed; see cmoe_last_hip_error                    */
};

/* Hyper-parameters of one layer (Sec. 3.1-3.4). */
typedef struct {
  int32_t d;          /* model width                                                */
  int32_t d_ff;       /* hidden width of the expert FFN                             */
  int32_t G;          /* number of clusters                                         */
  int32_t K;          /* experts per cluster (uniform, Sec. 3.1)                    */
  int32_t r;          /* rank of the residual factors (Sec. 3.2): 4, 8, 16 or 32    */
  int32_t top_k;      /* experts kept inside the selected cluster (Sec. 3.3)        */
  int32_t q_group;    /* INT4 scale-group length along the long dimension (Sec. 3.4) */
  int32_t activation; /* 0 = GELU, erf form                                         */
} cmoe_config;

/* Stored parameters.  Expert slot e = c*K + j belongs to cluster c (cluster-major).
 * Factor tensors are rank-major: row rho of expert e holds L values along the long
 * dimension (L = d for v1 and u2, d_ff for u1 and v2), element n in byte n/2 with even
 * n in the low nibble, codes two's-complement in [-8, 7], value = scale[n/q_group]*code.
 *   W1_e[o][i] = w1_base[c][o][i] + sum_rho u1[e][rho][o] * v1[e][rho][i]   (d_ff x d)
 *   W2_e[o][i] = w2_base[c][o][i] + sum_rho u2[e][rho][o] * v2[e][rho][i]   (d x d_ff)
 */
typedef struct {
  const cmoe_f16 *router_cluster; /* [G][d]       group prototypes u_g (Sec. 3.3)          */
  const cmoe_f16 *router_expert;  /* [G*K][d]     expert routing vectors v_i               */
  const float *cluster_bias;      /* [G] or NULL  added to z_g; NULL = the paper's router  */
  const cmoe_f16 *w1_base;        /* [G][d_ff][d]   (may be NULL when packed is set)       */
  const cmoe_f16 *w2_base;        /* [G][d][d_ff]   (may be NULL when packed is set)       */
  const uint8_t *v1_q, *u1_q, *v2_q, *u2_q; /* [G*K][r][L/2]                                */
  const cmoe_f16 *v1_s, *u1_s, *v2_s, *u2_s; /* [G*K][r][L/q_group]                         */
  const void *packed; /* NULL, or the buffer cmoe_pack_weights filled from THESE bases (below)  */
} cmoe_weights;

typedef struct cmoe_handle cmoe_handle;

/* Validates the configuration and creates a handle (host state only).
 * Supported: d and d_ff multiples of 64 with d <= 8192; 1 <= G <= 64; 1 <= K <= 32;
 * r in {4, 8, 16, 32}; K*r <= 512; 1 <= top_k <= min(K, 8); q_group a multiple of 8 dividing d and
 * d_ff; activation = 0.  Anything else: CMOE_ERR_UNSUPPORTED. */
int cmoe_create(const cmoe_config *cfg, cmoe_handle **out);
int cmoe_destroy(cmoe_handle *h);

/* One-time preparation of the stored parameters for the matrix-core kernels (weights are
 * static across forward calls, Sec. 3.4; the canonical layouts above stay the interface).
 * packed holds, per cluster, W1_base as [d/32][d_ff][32] and W2_base as [d_ff/32][d][32]: the 32
 * contraction elements of consecutive rows are contiguous, so one direct-to-LDS load
 * instruction fetches 1 KiB of contiguous memory instead of 16 pieces a row apart; and the
 * FP16 operand panels of the four INT4 factor tensors of every cluster (2 * KRp * (d + d_ff)
 * FP16 values per cluster, KRp = K*r rounded up to 32), so that no call dequantises them
 * again.  cmoe_packed_bytes is the size of that buffer (about 4*G*d*d_ff + 4*G*KRp*(d + d_ff)
 * bytes; 0 for a bad handle); packed is a caller-owned device buffer, 256-byte aligned.  Set
 * cmoe_weights.packed to it and every call reads the bases from it, whatever the token count
 * (cmoe_ffn_forward, cmoe_forward, cmoe_forward_multi, cmoe_backward); the calls that take
 * more than 256 tokens also read the factor panels from it (cmoe_combine too), the calls
 * with fewer tokens decode the INT4 factors on the fly.  With packed == NULL the canonical
 * arrays are read (and, above 256 tokens, the factors of the clusters that received tokens
 * dequantised per call).  Once packed is set, w1_base and w2_base may be NULL: the packed
 * buffer is then the only resident copy of the bases (the INT4 factor tensors and the
 * routers must stay valid).  The caller packs again after changing a base or a factor.
 * Packing reads every cluster's canonical bases and factors. */
size_t cmoe_packed_bytes(const cmoe_handle *h);
int cmoe_pack_weights(cmoe_handle *h, const cmoe_weights *w, void *packed, size_t packed_bytes,
                      void *stream);

/* Bytes of device workspace that cmoe_permute / cmoe_ffn_forward / cmoe_combine /
 * cmoe_forward need for up to T_max tokens (one buffer serves all of them; contents
 * need not be preserved between calls).  Returns 0 for a NULL handle or T_max < 0. */
size_t cmoe_workspace_bytes(const cmoe_handle *h, int32_t T_max);

/* Sec. 3.3, both stages.  x [T][d] f16 ->
 *   cluster_id [T]        argmax_g (u_g.x + bias_g)
 *   expert_idx [T][top_k] global slots of the top_k largest v_i.x inside that cluster
 *   gate       [T][top_k] f32, softmax over the selected logits (sums to one) */
int cmoe_route(cmoe_handle *h, const cmoe_weights *w, const cmoe_f16 *x, int32_t T,
               int32_t *cluster_id, int32_t *expert_idx, float *gate, void *stream);

/* Group-level dispatch on one device (Sec. 3.3): stable counting sort of tokens by
 * cluster.  offsets [G+1] exclusive prefix sum of cluster loads; perm [T] token of
 * sorted row p; inv_perm [T] sorted row of token t. */
int cmoe_permute(cmoe_handle *h, const int32_t *cluster_id, int32_t T, int32_t *perm,
                 int32_t *inv_perm, int32_t *offsets, void *workspace, size_t workspace_bytes,
                 void *stream);

/* cmoe_permute for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * outputs as cmoe_permute; the per-block histogram that cmoe_permute keeps in the workspace
 * lives in a device array inside the library (256 KiB per GPU, held until the process ends),
 * which limits the call to CMOE_PERMUTE_STATIC_MAX_TOKENS tokens: more returns
 * CMOE_ERR_UNSUPPORTED before any HIP call.  The call allocates and frees nothing; the
 * first call on a device looks up the array's address on that device.  Every call on a GPU
 * uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race
 * and must be serialised by the caller.  Nothing in the array is carried from call to call. */
#define CMOE_PERMUTE_STATIC_MAX_TOKENS 1048576
int cmoe_permute_static(cmoe_handle *h, const int32_t *cluster_id, int32_t T, int32_t *perm,
                        int32_t *inv_perm, int32_t *offsets, void *stream);

/* Expert computation with base reuse (Sec. 3.2), in cluster-sorted row order p
 * (token t = perm[p], cluster c, experts e_j, gates g_j):
 *   Hb = W1_base(c) x_t;  a_j = GELU(Hb + U1_{e_j}(V1_{e_j} x_t));  A = sum_j g_j a_j
 *   y_base_sorted[p] = W2_base(c) A            [T][d] f16
 *   s_down[t][j]     = V2_{e_j} a_j            [T][top_k][r] f32, token order */
int cmoe_ffn_forward(cmoe_handle *h, const cmoe_weights *w, const cmoe_f16 *x, int32_t T,
                     const int32_t *perm, const int32_t *offsets, const int32_t *expert_idx,
                     const float *gate, cmoe_f16 *y_base_sorted, float *s_down, void *workspace,
                     size_t workspace_bytes, void *stream);

/* Residual of the second matrix, gated combine and return to token order:
 *   y[t] = y_base_sorted[inv_perm[t]] + sum_j g_j U2_{e_j} s_down[t][j]     [T][d] f16 */
int cmoe_combine(cmoe_handle *h, const cmoe_weights *w, const cmoe_f16 *y_base_sorted,
                 const float *s_down, const int32_t *perm, const int32_t *inv_perm,
                 const int32_t *offsets, const int32_t *expert_idx, const float *gate, int32_t T,
                 cmoe_f16 *y, void *workspace, size_t workspace_bytes, void *stream);

/* The whole layer: route -> permute -> ffn_forward -> combine on one stream.
 * cluster_id, expert_idx, gate, perm, inv_perm, offsets are outputs as above (all
 * required, caller-allocated). */
int cmoe_forward(cmoe_handle *h, const cmoe_weights *w, const cmoe_f16 *x, int32_t T, cmoe_f16 *y,
                 int32_t *cluster_id, int32_t *expert_idx, float *gate, int32_t *perm,
                 int32_t *inv_perm, int32_t *offsets, void *workspace, size_t workspace_bytes,
                 void *stream);

/* Routing statistics of one step, from the routing and dispatch outputs above
 * (perm, offsets from cmoe_permute; expert_idx from cmoe_route; all device pointers):
 *   expert_load  [E] i32   assignments per expert, a token counting once for each of its
 *                          top_k experts                       (loads of Sec. 4)
 *   i_load       [1] f32   their coefficient of variation, population standard deviation
 *                          over the mean, 0 when T = 0         (load-balance metric, Sec. 4)
 *   mu           [E][d] f32, in/out: mu_e <- (1 - beta) mu_e + beta * mean of the x rows
 *                          assigned to e; unchanged for an expert without tokens
 *                                                              (Sec. 3.1, Eq. 5)
 *   cluster_load [G] i32   tokens per cluster
 *   cluster_act  [G] f32, in/out: act_g <- (1 - lam) act_g + lam * [cluster_load_g > 0]
 *   cluster_idle [G] i32, in/out: consecutive steps without a token, 0 after a hit
 *                                                              (Sec. 3.4)
 * The caller owns and initialises the in/out state.  Deterministic (fixed summation
 * order).  Errors as for the other entry points. */
int cmoe_route_stats(cmoe_handle *h, const cmoe_f16 *x, int32_t T, const int32_t *perm,
                     const int32_t *offsets, const int32_t *expert_idx, float beta, float lam,
                     float *mu, float *cluster_act, int32_t *cluster_idle, int32_t *expert_load,
                     int32_t *cluster_load, float *i_load, void *workspace, size_t workspace_bytes,
                     void *stream);

/* ---- Routing variants (Sec. 3.3 "Top-g_1 groups", Sec. 3.5 router temperature) ----
 * top_g clusters are kept per token (1 <= top_g <= min(G, 8), listed by descending
 * probability, lowest index on ties) and each contributes its own top_k experts.  Both
 * softmaxes (Eq. 9, Eq. 10) take logits divided by temperature (> 0); the selection does
 * not depend on it.  The mixing weight of expert j of the a-th selected cluster is
 *   gate[t][a][j] = w_a * softmax_j(l_sel / temperature),
 *   w_a = p_g of Eq. 9 when scale_by_cluster_prob != 0, else p_g renormalised over the
 *         selected clusters (1 for top_g = 1: then this is cmoe_route with a temperature).
 * A (token, selected cluster) pair is a "virtual token" vt = t * top_g + a: cluster_id
 * [T*top_g], expert_idx [T*top_g][top_k], gate [T*top_g][top_k], and perm / inv_perm
 * [T*top_g] of cmoe_forward_multi are indexed by vt; the permutation is the stable sort of
 * the virtual tokens by cluster, the shared-base products are computed once per virtual
 * token (which reads row vt / top_g of x: x is not replicated), and y[t] is the sum of its
 * top_g virtual tokens' outputs. */
typedef struct cmoe_route_options {
  int32_t top_g;
  float temperature;
  int32_t scale_by_cluster_prob;
} cmoe_route_options;

int cmoe_route_multi(cmoe_handle *h, const cmoe_weights *w, const cmoe_route_options *opt,
                     const cmoe_f16 *x, int32_t T, int32_t *cluster_id, int32_t *expert_idx,
                     float *gate, void *stream);
/* Workspace of cmoe_forward_multi for up to T_max tokens (0 for a bad handle or top_g). */
size_t cmoe_workspace_bytes_multi(const cmoe_handle *h, int32_t T_max, int32_t top_g);
int cmoe_forward_multi(cmoe_handle *h, const cmoe_weights *w, const cmoe_route_options *opt,
                       const cmoe_f16 *x, int32_t T, cmoe_f16 *y, int32_t *cluster_id,
                       int32_t *expert_idx, float *gate, int32_t *perm, int32_t *inv_perm,
                       int32_t *offsets, void *workspace, size_t workspace_bytes, void *stream);

/* ---- Construction of the compressed form from dense expert matrices (Sec. 3.2, 3.4) ----
 * One weight matrix of the layer at a time: W [G*K][out_dim][in_dim] f16, experts stored
 * cluster-major (call it once for the first and once for the second matrix of the FFN).
 *   base   [G][out_dim][in_dim] f16   mean of the cluster's K experts (Eq. 6): FP32 sum in
 *                                     expert order, divided by K, rounded to nearest even
 *   u_q/u_s, v_q/v_s                  INT4 codes and FP16 scales (format of cmoe_weights) of
 *                                     the rank-r factors of Delta_e = W_e - base(c) (Eq. 7):
 *                                     U_e as [r][out_dim], V_e as [r][in_dim]
 *   report [G*K][4] f32               [0] ||W_e - base - U V||_F / ||W_e||_F with the stored
 *                                     (dequantised) factors, [1] the same for the FP32
 *                                     rank-r factors before quantisation (from norms, good
 *                                     to about 1 % of ||Delta_e|| / ||W_e||), [2] cosine of
 *                                     vec(Delta_e) and vec(base(c)), [3] 1 if gated off
 * The factors are the best rank-r pair inside the subspace reached by a randomised
 * subspace iteration: omega [sketch][in_dim] f16 holds the caller's random test rows
 * (r <= sketch <= 48; sketch = r + 8 and n_iter = 2 reproduce the truncated SVD's error
 * to within about one percent on decaying spectra).  use_gate != 0: experts whose cosine
 * [2] is below gate_gamma get all-zero factors (the optional gate of Sec. 3.4).
 * Supported: out_dim, in_dim multiples of 64 and of q_group; K <= 64; r <= 32; q_group
 * even; 0 <= n_iter <= 16.  The quantiser (Sec. 3.4): scale = f16(absmax / 7) per q_group
 * consecutive elements, code = clip(rint(w / scale), -7, 7), decisions in FP32, codes 0
 * where the scale rounds to 0.  All pointers are device pointers, 16-byte aligned. */
typedef struct cmoe_compress_config {
  int32_t out_dim, in_dim, G, K, r, q_group;
  int32_t sketch;     /* rows of the random sketch, r <= sketch <= 48 */
  int32_t n_iter;     /* subspace (power) iterations                  */
  int32_t use_gate;   /* 0: no gate                                   */
  float gate_gamma;
} cmoe_compress_config;

size_t cmoe_compress_workspace_bytes(const cmoe_compress_config *cfg); /* 0 if unsupported */
int cmoe_compress(const cmoe_compress_config *cfg, const cmoe_f16 *W, const cmoe_f16 *omega,
                  cmoe_f16 *base, uint8_t *u_q, cmoe_f16 *u_s, uint8_t *v_q, cmoe_f16 *v_s,
                  float *report, void *workspace, size_t workspace_bytes, void *stream);

/* The quantiser alone: src [rows][L] f32 -> codes [rows][L/2], scales [rows][L/q_group]. */
int cmoe_quantize_int4(const float *src, int64_t rows, int32_t L, int32_t q_group, uint8_t *codes,
                       cmoe_f16 *scales, void *stream);

/* err [G*K] f32 = ||W_e - base(c) - U_e V_e||_F / ||W_e||_F for a given stored form
 * (workspace of cmoe_compress_workspace_bytes(cfg); sketch / n_iter / gate are ignored). */
int cmoe_reconstruction_error(const cmoe_compress_config *cfg, const cmoe_f16 *W, const cmoe_f16 *base,
                              const uint8_t *u_q, const cmoe_f16 *u_s, const uint8_t *v_q,
                              const cmoe_f16 *v_s, float *err, void *workspace, size_t workspace_bytes,
                              void *stream);

/* ---- Backward pass for a frozen selection (training step of Sec. 3.5) ----
 * Gradients of L = sum(dy * y), y = the layer output of Sec. 3.2 / Eq. 7 for the given
 * expert_idx [T][top_k] and gate [T][top_k] (the softmax of Eq. 10 over the selected
 * logits, as cmoe_route returns them).  The selection itself (cluster and expert argmax)
 * is piecewise constant and carries no gradient; the cluster router receives none.
 * Precondition (not checked): the top_k experts of a token lie in one cluster, as
 * cmoe_route produces them; the shared-base products are taken once per token.
 * All outputs are FP32 device buffers and are overwritten:
 *   dx              [T][d]         through the experts and through the gate logits
 *   d_logits        [T][top_k]     dL / d(selected expert logits); may be NULL
 *   d_router_expert [G*K][d]       rows v_i of the expert router
 *   dw1_base [G][d_ff][d], dw2_base [G][d][d_ff]     = sum over the cluster of dW_e
 *   du1 [G*K][r][d_ff], dv1 [G*K][r][d], du2 [G*K][r][d], dv2 [G*K][r][d_ff]
 *                                  with respect to the DEQUANTISED factors, in the stored
 *                                  rank-major orientation: dU = dW V^T, dV = U^T dW
 * Experts that received no token get zero gradients and their stored weights are not read.
 * The shared-base products are computed once per token, the rank-r products once per
 * (token, expert) pair (Sec. 3.2).  Matrix operands are FP16, accumulation, the hidden
 * pre-activations and the gate path are FP32.  T = 0 writes zero
 * weight gradients.  Deterministic (fixed summation order). */
typedef struct cmoe_grads {
  float *dx, *d_logits, *d_router_expert, *dw1_base, *dw2_base, *du1, *dv1, *du2, *dv2;
} cmoe_grads;

/* Workspace of cmoe_backward for up to T_max tokens (0 for a bad handle, T_max < 0 or an
 * unsupported shape): per-token and per-pair activations, about
 * (8 * top_k + 12) * T_max * d_ff bytes, plus the transposed bases, 4 * G * d * d_ff bytes,
 * the rank panels and partial results. */
size_t cmoe_backward_workspace_bytes(const cmoe_handle *h, int32_t T_max);
int cmoe_backward(cmoe_handle *h, const cmoe_weights *w, const cmoe_f16 *x, const cmoe_f16 *dy,
                  int32_t T, const int32_t *expert_idx, const float *gate, const cmoe_grads *grads,
                  void *workspace, size_t workspace_bytes, void *stream);

/* hipError_t (as int) of the last failed HIP call made through this handle, 0 if none. */
int cmoe_last_hip_error(const cmoe_handle *h);
const char *cmoe_status_string(int status);

/* Name and average duration (ms) bookkeeping for benchmarking: when enabled, every kernel
 * launched through the handle is bracketed by HIP events on its stream.
 * cmoe_timing_read synchronises those events and writes, for each of n_max slots, the
 * accumulated milliseconds and launch counts; returns the number of slots used and resets
 * the accumulators.  Slot names: cmoe_timing_name(i).  Not for production use. */
int cmoe_timing_enable(cmoe_handle *h, int on);
int cmoe_timing_read(cmoe_handle *h, double *ms_sum, int32_t *count, int32_t n_max);
const char *cmoe_timing_name(int32_t slot);

/* Benchmark calibration: n_workgroups workgroups (one per compute unit: 256) run iters
 * iterations of the grouped products' inner schedule - 64 FP16 matrix-core instructions
 * (16 x 16 x 32) per iteration and SIMD on operands of random mantissas read from LDS - with no
 * global memory traffic, so that every matrix-core issue slot is used.  FLOPs = n_workgroups *
 * 8 * iters * 32 * 16384; the rate over the call's duration is what the power management lets
 * the matrix cores sustain on this machine.  ticks [2] u64 (device, zeroed by the caller): sums
 * over the workgroups of shader-clock cycles and of constant-rate (100 MHz) ticks spent in the
 * loop; sink [n_workgroups * 512] f32 (device) receives the accumulators.  zero_operands != 0
 * runs the same loop on operands that are all 0.0 (the rate without the data-dependent part of
 * the power draw).  Not for production use. */
int cmoe_calibrate_mfma(int32_t n_workgroups, int32_t iters, int32_t zero_operands, uint64_t *ticks, float *sink,
                        void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CMOE_H */
