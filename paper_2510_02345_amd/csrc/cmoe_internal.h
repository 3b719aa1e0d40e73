// Internal declarations shared by the HIP translation units of libcmoe.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cmoe.h"

typedef _Float16 half_t;
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));

// Derived sizes of one layer.
struct cmoe_dims {
  int d, d_ff, G, K, r, k, q;
  int KR;   // K * r: concatenated rank rows of one cluster
  int KRp;  // KR rounded up to a multiple of 32 (one 32-row MFMA block)
};

enum cmoe_timing_slot {
  TS_ROUTE = 0,
  TS_PERMUTE,
  TS_DEQUANT,
  TS_T1,
  TS_GEMM1,
  TS_SREDUCE,
  TS_GEMM2,
  TS_COMBINE,
  TS_GEMM1_BASE,
  TS_RESID_UP,
  TS_STATS,
  TS_BACKWARD,
  TS_COUNT
};

struct cmoe_timing {
  bool on = false;
  static const int MAX_EV = 4096;
  hipEvent_t ev[MAX_EV][2];
  int slot_of[MAX_EV];
  int n_ev = 0;
  int n_created = 0;
};

struct cmoe_handle {
  uint32_t magic;
  cmoe_dims dm;
  int last_hip_error;
  cmoe_timing tm;
};

// Workspace layout for T tokens (byte offsets, all 256-byte aligned).
struct cmoe_ws_layout {
  size_t blk_counts;  // int32 [n_blocks][max(G,64)] permute: per-block histogram -> bases
  size_t sort_i32;    // int32 [2][T]          expert-pair order inside clusters: rowmap, perm2
  size_t v1cat;       // f16 [G][KRp][d]       dequantised V1, rows kk = j*r + rho
  size_t u1t;         // f16 [G][d_ff][KRp]    dequantised U1, transposed
  size_t v2p;         // f16 [G][KRp][d_ff]    dequantised V2
  size_t u2t;         // f16 [G][d][KRp]       dequantised U2, transposed
  size_t t1ext;       // f16 [T][k][r]         t1_j = V1 x of the selected experts, sorted rows (expanded
                      //                       one-hot over the cluster's rank rows only in registers)
  size_t a;           // f16 [T][d_ff]         gated hidden activations, cluster-sorted rows; stored as
                      //                       [d_ff/32][T][32] on the matrix-core path
  size_t ures;        // f32 [T][d]            residual-down term, sorted rows (weight-streaming path only)
  size_t stats_part;  // f32 [slots][K][d]     routing statistics: per-slot sums of x per expert
  size_t stats_cnt;   // i32 [slots][K]        and their row counts
  size_t spart;       // f32 [n_parts][T][k][r] partial V2 a per row tile of d_ff
  size_t yb;          // f16 [T][d]            cmoe_forward only: y_base_sorted
  size_t sdown;       // f32 [T][k][r]         cmoe_forward only: s_down
  size_t total;
};

// The caller's buffer filled by cmoe_pack_weights (byte offsets, 256-byte aligned): the two
// bases in 32-column blocks, then the FP16 operand panels of the four INT4 factors of every
// cluster (the layouts of v1cat / u1t / v2p / u2t above), so that a forward call neither
// re-tiles nor dequantises anything that does not change between calls.
struct cmoe_packed_layout {
  size_t w1, w2, v1cat, u1t, v2p, u2t, total;
};
inline cmoe_packed_layout cmoe_packed(const cmoe_dims& dm) {
  cmoe_packed_layout L;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = (off + bytes + 255) / 256 * 256;
    return at;
  };
  const size_t mat = sizeof(half_t) * dm.G * (size_t)dm.d * dm.d_ff;
  L.w1 = take(mat);
  L.w2 = take(mat);
  L.v1cat = take(sizeof(half_t) * dm.G * (size_t)dm.KRp * dm.d);
  L.u1t = take(sizeof(half_t) * dm.G * (size_t)dm.d_ff * dm.KRp);
  L.v2p = take(sizeof(half_t) * dm.G * (size_t)dm.KRp * dm.d_ff);
  L.u2t = take(sizeof(half_t) * dm.G * (size_t)dm.d * dm.KRp);
  L.total = off;
  return L;
}

static const int PERMUTE_BLOCK = 1024;  // tokens per workgroup in the permutation kernels
static const int G1_BN = 256;           // rows of d_ff per workgroup tile (= per s partial) in the fused up-projection
static const int SKINNY_T = 256;        // at most this many tokens: weight-streaming kernels
static const int SKINNY_SN = 2048;      // columns of d_ff per s partial in the weight-streaming path

cmoe_ws_layout cmoe_layout(const cmoe_dims& dm, int T);

// Kernel launchers (each returns the hipError_t of its launch).
hipError_t launch_route(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int* cluster_id,
                        int* expert_idx, float* gate, hipStream_t st);
hipError_t launch_route_mfma(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int* cluster_id,
                             int* expert_idx, float* gate, hipStream_t st);
hipError_t launch_permute(const cmoe_dims& dm, const int* cluster_id, int T, int* perm, int* inv_perm, int* offsets,
                          int* blk_counts, hipStream_t st);
hipError_t launch_permute_static(const cmoe_dims& dm, const int* cluster_id, int T, int* perm, int* inv_perm,
                                 int* offsets, hipStream_t st);
hipError_t launch_permute_bins(int bins, const int* keys, int T, int* perm, int* inv_perm, int* offsets,
                               int* blk_counts, hipStream_t st);
hipError_t launch_pair_sort(const cmoe_dims& dm, const int* perm, const int* offsets, const int* expert_idx, int T,
                            int* rowmap, int* perm2, hipStream_t st);
hipError_t launch_dequant_ffn(const cmoe_dims& dm, const cmoe_weights& w, const int* offsets, half_t* v1cat,
                              half_t* u1t, half_t* v2p, half_t* u2t, hipStream_t st);
hipError_t launch_dequant_u2(const cmoe_dims& dm, const cmoe_weights& w, const int* offsets, half_t* u2t,
                             hipStream_t st);
hipError_t launch_t1(const cmoe_dims& dm, const half_t* x, int x_div, int T, const int* perm, const int* offsets,
                     const int* expert_idx, const half_t* v1cat, half_t* t1ext, hipStream_t st);
hipError_t launch_gemm1(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int x_div, int T, const int* perm,
                        const int* offsets, const int* expert_idx, const float* gate, const half_t* u1t,
                        const half_t* v2p, const half_t* t1ext, half_t* a, float* spart, hipStream_t st);
hipError_t launch_sreduce(const cmoe_dims& dm, int T, const int* perm, const float* spart, int n_parts,
                          float* s_down, hipStream_t st);
hipError_t launch_skinny_hb(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int x_div, int T, const int* perm,
                            const int* offsets, const int* expert_idx, half_t* t1, half_t* hb, hipStream_t st);
hipError_t launch_route_multi(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int top_g,
                              float temperature, int scale, int* cluster_id, int* expert_idx, float* gate,
                              hipStream_t st);
hipError_t launch_route_multi_mfma(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int top_g,
                                   float temperature, int scale, int* cluster_id, int* expert_idx, float* gate,
                                   hipStream_t st);
hipError_t launch_sum_groups(const half_t* yrep, int T, int top_g, int d, half_t* y, hipStream_t st);
hipError_t launch_skinny_rows(const half_t* X, const half_t* W, const int* offsets, int n_groups, int N, int Kc,
                              int max_rows, half_t* out, hipStream_t st);
size_t stats_partial_slots(const cmoe_dims& dm, int T);
hipError_t launch_route_stats(const cmoe_dims& dm, const half_t* x, int T, const int* perm, const int* offsets,
                              const int* expert_idx, float beta, float lam, float* mu, float* cluster_act,
                              int* cluster_idle, int* expert_load, int* cluster_load, float* i_load, float* part,
                              int* cnt, hipStream_t st);
hipError_t launch_skinny_add(const cmoe_dims& dm, const half_t* y_base_sorted, const float* ures, const int* perm,
                             int T, half_t* y, hipStream_t st);
hipError_t launch_skinny_resid_up(const cmoe_dims& dm, const cmoe_weights& w, int T, const int* perm,
                                  const int* expert_idx, const float* gate, const half_t* t1, half_t* a,
                                  float* spart, hipStream_t st);
hipError_t launch_skinny_combine(const cmoe_dims& dm, const cmoe_weights& w, const half_t* y_base_sorted,
                                 const float* s_down, const int* inv_perm, const int* expert_idx, const float* gate,
                                 int T, half_t* y, hipStream_t st);
hipError_t launch_skinny_down(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T, const int* offsets,
                              half_t* y_base_sorted, const int* perm, const int* expert_idx, const float* gate,
                              const float* spart, int n_parts, float* ures, hipStream_t st);
hipError_t launch_gemm2(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T, const int* offsets,
                        const int* rowmap, half_t* y_base_sorted, hipStream_t st);
hipError_t launch_gemm2_combine(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T,
                                const int* offsets, const int* rperm, const half_t* u2t, const float* s_down,
                                const int* expert_idx, const float* gate, half_t* y, hipStream_t st);
hipError_t launch_combine(const cmoe_dims& dm, const half_t* u2t, const half_t* y_base_sorted, const float* s_down,
                          const int* perm, const int* offsets, const int* expert_idx, const float* gate, int T,
                          half_t* y, hipStream_t st);

// Workspace of the backward pass (byte offsets).  M = T * top_k pair rows; Tpad = columns of
// the transposed copies whose groups (clusters) are padded to 32.
struct cmoe_bw_layout {
  int M, Tpad;
  size_t blk_counts, cid, permc, invc, offc, permm, invm, offe, sort_tmp, off_tmp, krange_c;
  size_t srow_c, ssrc_c;
  size_t offx_f, gidx_f, offx_d, gidx_d, dl;
  size_t v1p, u2p, u1p, v2p;                  // f16 rank panels [E][32][L]
  size_t w1bt, w2bt;                          // f16 transposed bases
  size_t hb, dab, rh, rda;                    // f16 [T][d_ff] x2 (token order), [M][d_ff] x2 (sorted pairs)
  size_t a16, dh16, dhsum16, ag16;            // f16 [M][d_ff] x2, [T][d_ff] x2
  size_t t1, uy, qq, ss;                      // f16 [M][32] rank-space rows of the pairs
  size_t dxb, dxr;                            // f16 [T][d], [M][d]
  size_t xct, dyct, dhst, agt;                // f16 transposed copies, Tpad columns
  size_t rgpart;                              // f32 [4][E][r][max(d, d_ff)] partial factor gradients
  size_t total;
};
cmoe_bw_layout cmoe_backward_layout(const cmoe_dims& dm, int T);
hipError_t launch_backward(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, const half_t* dy, int T,
                           const int* expert_idx, const float* gate, const cmoe_grads& out, char* ws,
                           const cmoe_bw_layout& L, hipStream_t st);
hipError_t launch_gemm_plain(const half_t* W, long w_gstride, int ldw, int N, const half_t* X, int ldx,
                             const int* gather, int x_div, int Kc, const int* offsets, int n_groups, int rows,
                             const int* krange, const int* rowmap, void* out, int ldo, bool out_f32, hipStream_t st,
                             long kstep_w = 0, long kstep_x = 0);
hipError_t launch_pack_bases(const cmoe_dims& dm, const cmoe_weights& w, half_t* packed, hipStream_t st);
