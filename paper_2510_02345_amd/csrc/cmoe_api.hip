// C ABI of libcmoe: argument validation, workspace carving, kernel sequencing.
// The operations are those of Sec. 3.2-3.4 of the paper; see include/cmoe.h.
#include <new>

#include "cmoe_internal.h"

static const uint32_t CMOE_MAGIC = 0x636d6f65u;

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

cmoe_ws_layout cmoe_layout(const cmoe_dims& dm, int T) {
  cmoe_ws_layout L;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  size_t Tz = (size_t)(T > 0 ? T : 0);
  size_t n_blocks = (Tz + PERMUTE_BLOCK - 1) / PERMUTE_BLOCK;
  size_t n_tiles = (T <= SKINNY_T) ? ((size_t)dm.d_ff + SKINNY_SN - 1) / SKINNY_SN
                                   : ((size_t)dm.d_ff + G1_BN - 1) / G1_BN;
  L.blk_counts = take(sizeof(int32_t) * (n_blocks + 1) * (dm.G > 64 ? dm.G : 64));
  L.sort_i32 = take(sizeof(int32_t) * 2 * Tz);
  L.v1cat = take(sizeof(half_t) * dm.G * dm.KRp * dm.d);
  L.u1t = take(sizeof(half_t) * dm.G * dm.d_ff * dm.KRp);
  L.v2p = take(sizeof(half_t) * dm.G * dm.KRp * dm.d_ff);
  L.u2t = take(sizeof(half_t) * dm.G * dm.d * dm.KRp);
  L.t1ext = take(sizeof(half_t) * Tz * dm.k * dm.r);
  L.a = take(sizeof(half_t) * Tz * dm.d_ff);
  L.ures = take(T <= SKINNY_T ? sizeof(float) * Tz * dm.d : 0);
  L.stats_part = take(sizeof(float) * stats_partial_slots(dm, T) * dm.K * dm.d);
  L.stats_cnt = take(sizeof(int32_t) * stats_partial_slots(dm, T) * dm.K);
  L.spart = take(sizeof(float) * n_tiles * Tz * dm.k * dm.r);
  L.yb = take(sizeof(half_t) * Tz * dm.d);
  L.sdown = take(sizeof(float) * Tz * dm.k * dm.r);
  L.total = off;
  return L;
}

static bool handle_ok(const cmoe_handle* h) { return h != nullptr && h->magic == CMOE_MAGIC; }
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static bool ptr_ok(const void* p) { return p != nullptr && aligned16(p); }

extern "C" int cmoe_create(const cmoe_config* cfg, cmoe_handle** out) {
  if (cfg == nullptr || out == nullptr) return CMOE_ERR_INVALID_ARG;
  *out = nullptr;
  const cmoe_config& c = *cfg;
  if (c.d <= 0 || c.d_ff <= 0 || c.G <= 0 || c.K <= 0 || c.r <= 0 || c.top_k <= 0 || c.q_group <= 0)
    return CMOE_ERR_INVALID_ARG;
  if (c.d % 64 != 0 || c.d_ff % 64 != 0 || c.d > 8192) return CMOE_ERR_UNSUPPORTED;
  if (c.G > 64 || c.K > 32) return CMOE_ERR_UNSUPPORTED;
  if (!(c.r == 4 || c.r == 8 || c.r == 16 || c.r == 32)) return CMOE_ERR_UNSUPPORTED;
  if (c.K * c.r > 512) return CMOE_ERR_UNSUPPORTED;
  if (c.top_k > c.K || c.top_k > 8) return CMOE_ERR_UNSUPPORTED;
  if (c.q_group % 8 != 0 || c.d % c.q_group != 0 || c.d_ff % c.q_group != 0) return CMOE_ERR_UNSUPPORTED;
  if (c.activation != 0) return CMOE_ERR_UNSUPPORTED;
  cmoe_handle* h = new (std::nothrow) cmoe_handle();
  if (h == nullptr) return CMOE_ERR_INVALID_ARG;
  h->magic = CMOE_MAGIC;
  h->dm.d = c.d;
  h->dm.d_ff = c.d_ff;
  h->dm.G = c.G;
  h->dm.K = c.K;
  h->dm.r = c.r;
  h->dm.k = c.top_k;
  h->dm.q = c.q_group;
  h->dm.KR = c.K * c.r;
  h->dm.KRp = (h->dm.KR + 31) / 32 * 32;
  h->last_hip_error = 0;
  *out = h;
  return CMOE_OK;
}

extern "C" int cmoe_destroy(cmoe_handle* h) {
  if (!handle_ok(h)) return CMOE_ERR_INVALID_ARG;
  for (int i = 0; i < h->tm.n_created; ++i) {
    (void)hipEventDestroy(h->tm.ev[i][0]);
    (void)hipEventDestroy(h->tm.ev[i][1]);
  }
  h->magic = 0;
  delete h;
  return CMOE_OK;
}

// A call with T tokens carves the layout of T, and the two paths (weight streaming up to
// SKINNY_T tokens, matrix cores above) lay the buffer out differently, so a buffer "for up to
// T_max tokens" must hold the larger of the two: each layout grows with T inside its own
// range, hence the largest weight-streaming layout is that of min(T_max, SKINNY_T).
static size_t workspace_for_up_to(const cmoe_dims& dm, int T_max) {
  const size_t big = cmoe_layout(dm, T_max).total;
  const size_t small = cmoe_layout(dm, T_max < SKINNY_T ? T_max : SKINNY_T).total;
  return big > small ? big : small;
}

extern "C" size_t cmoe_workspace_bytes(const cmoe_handle* h, int32_t T_max) {
  if (!handle_ok(h) || T_max < 0) return 0;
  return workspace_for_up_to(h->dm, T_max);
}

extern "C" int cmoe_last_hip_error(const cmoe_handle* h) { return handle_ok(h) ? h->last_hip_error : 0; }

extern "C" const char* cmoe_status_string(int status) {
  switch (status) {
    case CMOE_OK: return "ok";
    case CMOE_ERR_INVALID_ARG: return "invalid argument";
    case CMOE_ERR_UNSUPPORTED: return "unsupported configuration";
    case CMOE_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case CMOE_ERR_HIP: return "HIP call failed";
    default: return "unknown status";
  }
}

// ---------------------------------------------------------------- per-kernel timing
static const char* const kSlotNames[TS_COUNT] = {"route", "permute", "dequant", "t1", "gemm1_fused",
                                                 "s_reduce", "gemm2", "combine", "gemm1_base",
                                                 "residual_up", "route_stats", "backward"};

extern "C" const char* cmoe_timing_name(int32_t slot) {
  return (slot >= 0 && slot < TS_COUNT) ? kSlotNames[slot] : "";
}

extern "C" int cmoe_timing_enable(cmoe_handle* h, int on) {
  if (!handle_ok(h)) return CMOE_ERR_INVALID_ARG;
  h->tm.on = on != 0;
  h->tm.n_ev = 0;
  return CMOE_OK;
}

extern "C" int cmoe_timing_read(cmoe_handle* h, double* ms_sum, int32_t* count, int32_t n_max) {
  if (!handle_ok(h) || ms_sum == nullptr || count == nullptr || n_max < 0) return CMOE_ERR_INVALID_ARG;
  int n = n_max < TS_COUNT ? n_max : TS_COUNT;
  for (int i = 0; i < n; ++i) {
    ms_sum[i] = 0.0;
    count[i] = 0;
  }
  for (int i = 0; i < h->tm.n_ev; ++i) {
    float ms = 0.f;
    hipError_t e = hipEventSynchronize(h->tm.ev[i][1]);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, h->tm.ev[i][0], h->tm.ev[i][1]);
    if (e != hipSuccess) {
      h->last_hip_error = (int)e;
      return CMOE_ERR_HIP;
    }
    int s = h->tm.slot_of[i];
    if (s < n) {
      ms_sum[s] += ms;
      count[s] += 1;
    }
  }
  h->tm.n_ev = 0;
  return n;
}

namespace {
// Brackets one launch with events when timing is on.
struct Timed {
  cmoe_handle* h;
  hipStream_t st;
  int idx = -1;
  Timed(cmoe_handle* h_, int slot, hipStream_t st_) : h(h_), st(st_) {
    cmoe_timing& t = h->tm;
    if (!t.on || t.n_ev >= cmoe_timing::MAX_EV) return;
    if (t.n_ev >= t.n_created) {
      if (hipEventCreate(&t.ev[t.n_created][0]) != hipSuccess) return;
      if (hipEventCreate(&t.ev[t.n_created][1]) != hipSuccess) return;
      t.n_created++;
    }
    idx = t.n_ev++;
    t.slot_of[idx] = slot;
    (void)hipEventRecord(t.ev[idx][0], st);
  }
  ~Timed() {
    if (idx >= 0) (void)hipEventRecord(h->tm.ev[idx][1], st);
  }
};
}  // namespace

#define CMOE_LAUNCH(slot, expr)                \
  do {                                         \
    hipError_t e_;                             \
    {                                          \
      Timed timed_(h, slot, st);               \
      e_ = (expr);                             \
    }                                          \
    if (e_ != hipSuccess) {                    \
      h->last_hip_error = (int)e_;             \
      return CMOE_ERR_HIP;                     \
    }                                          \
  } while (0)

static bool weights_route_ok(const cmoe_weights* w) {
  return w != nullptr && ptr_ok(w->router_cluster) && ptr_ok(w->router_expert) &&
         (w->cluster_bias == nullptr || (reinterpret_cast<uintptr_t>(w->cluster_bias) & 3u) == 0);
}
// The bases: the canonical arrays, or the re-tiled copy alone (every kernel reads the copy
// when there is one, so a caller that has packed may drop the canonical arrays).
static bool bases_ok(const cmoe_weights* w) {
  if (!aligned16(w->packed) || !aligned16(w->w1_base) || !aligned16(w->w2_base)) return false;
  return w->packed != nullptr || (w->w1_base != nullptr && w->w2_base != nullptr);
}
static bool weights_ffn_ok(const cmoe_weights* w) {
  return w != nullptr && bases_ok(w) && ptr_ok(w->v1_q) && ptr_ok(w->u1_q) && ptr_ok(w->v2_q) && ptr_ok(w->v1_s) &&
         ptr_ok(w->u1_s) && ptr_ok(w->v2_s);
}
static bool weights_combine_ok(const cmoe_weights* w) { return w != nullptr && ptr_ok(w->u2_q) && ptr_ok(w->u2_s); }

static int check_ws(const cmoe_handle* h, int T, const void* ws, size_t bytes) {
  if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) & 255u) != 0) return CMOE_ERR_WORKSPACE;
  if (bytes < cmoe_layout(h->dm, T).total) return CMOE_ERR_WORKSPACE;
  return CMOE_OK;
}

// ---------------------------------------------------------------- entry points
extern "C" int cmoe_route(cmoe_handle* h, const cmoe_weights* w, const cmoe_f16* x, int32_t T, int32_t* cluster_id,
                          int32_t* expert_idx, float* gate, void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!weights_route_ok(w)) return CMOE_ERR_INVALID_ARG;
  if (T == 0) return CMOE_OK;
  if (!ptr_ok(x) || !ptr_ok(cluster_id) || !ptr_ok(expert_idx) || !ptr_ok(gate)) return CMOE_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  CMOE_LAUNCH(TS_ROUTE, launch_route(h->dm, *w, (const half_t*)x, T, cluster_id, expert_idx, gate, st));
  return CMOE_OK;
}

extern "C" int cmoe_permute(cmoe_handle* h, const int32_t* cluster_id, int32_t T, int32_t* perm, int32_t* inv_perm,
                            int32_t* offsets, void* workspace, size_t workspace_bytes, void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!ptr_ok(offsets)) return CMOE_ERR_INVALID_ARG;
  if (T > 0 && (!ptr_ok(cluster_id) || !ptr_ok(perm) || !ptr_ok(inv_perm))) return CMOE_ERR_INVALID_ARG;
  int rc = check_ws(h, T, workspace, workspace_bytes);
  if (rc != CMOE_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  cmoe_ws_layout L = cmoe_layout(h->dm, T);
  char* ws = (char*)workspace;
  CMOE_LAUNCH(TS_PERMUTE,
              launch_permute(h->dm, cluster_id, T, perm, inv_perm, offsets, (int*)(ws + L.blk_counts), st));
  return CMOE_OK;
}

extern "C" int cmoe_permute_static(cmoe_handle* h, const int32_t* cluster_id, int32_t T, int32_t* perm,
                                   int32_t* inv_perm, int32_t* offsets, void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!ptr_ok(offsets)) return CMOE_ERR_INVALID_ARG;
  if (T > 0 && (!ptr_ok(cluster_id) || !ptr_ok(perm) || !ptr_ok(inv_perm))) return CMOE_ERR_INVALID_ARG;
  if (T > CMOE_PERMUTE_STATIC_MAX_TOKENS) return CMOE_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  CMOE_LAUNCH(TS_PERMUTE, launch_permute_static(h->dm, cluster_id, T, perm, inv_perm, offsets, st));
  return CMOE_OK;
}

// y_fused != NULL: when the shapes allow it, the down-projection also applies the residual of
// the second matrix and writes y in token order (y_base_sorted is then not produced);
// *fused tells the caller whether that happened.
static int ffn_impl(cmoe_handle* h, const cmoe_weights* w, const cmoe_f16* x, int32_t T, const int32_t* perm,
                    const int32_t* offsets, const int32_t* expert_idx, const float* gate, cmoe_f16* y_base_sorted,
                    float* s_down, cmoe_f16* y_fused, bool* fused, int x_div, void* workspace, size_t workspace_bytes,
                    void* stream);

extern "C" int cmoe_ffn_forward(cmoe_handle* h, const cmoe_weights* w, const cmoe_f16* x, int32_t T,
                                const int32_t* perm, const int32_t* offsets, const int32_t* expert_idx,
                                const float* gate, cmoe_f16* y_base_sorted, float* s_down, void* workspace,
                                size_t workspace_bytes, void* stream) {
  return ffn_impl(h, w, x, T, perm, offsets, expert_idx, gate, y_base_sorted, s_down, nullptr, nullptr, 1, workspace,
                  workspace_bytes, stream);
}

static int ffn_impl(cmoe_handle* h, const cmoe_weights* w, const cmoe_f16* x, int32_t T, const int32_t* perm,
                    const int32_t* offsets, const int32_t* expert_idx, const float* gate, cmoe_f16* y_base_sorted,
                    float* s_down, cmoe_f16* y_fused, bool* fused, int x_div, void* workspace, size_t workspace_bytes,
                    void* stream) {
  if (fused) *fused = false;
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!weights_ffn_ok(w)) return CMOE_ERR_INVALID_ARG;
  if (T == 0) return CMOE_OK;
  if (!ptr_ok(x) || !ptr_ok(perm) || !ptr_ok(offsets) || !ptr_ok(expert_idx) || !ptr_ok(gate) ||
      !ptr_ok(y_base_sorted) || !ptr_ok(s_down))
    return CMOE_ERR_INVALID_ARG;
  int rc = check_ws(h, T, workspace, workspace_bytes);
  if (rc != CMOE_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const cmoe_dims& dm = h->dm;
  cmoe_ws_layout L = cmoe_layout(dm, T);
  char* ws = (char*)workspace;
  // factor panels: from the packed buffer when there is one, else dequantised per call
  const bool pk = w->packed != nullptr;
  const cmoe_packed_layout PL = cmoe_packed(dm);
  const char* pkb = (const char*)w->packed;
  half_t* v1cat = pk ? (half_t*)(pkb + PL.v1cat) : (half_t*)(ws + L.v1cat);
  half_t* u1t = pk ? (half_t*)(pkb + PL.u1t) : (half_t*)(ws + L.u1t);
  half_t* v2p = pk ? (half_t*)(pkb + PL.v2p) : (half_t*)(ws + L.v2p);
  half_t* t1ext = (half_t*)(ws + L.t1ext);
  half_t* a = (half_t*)(ws + L.a);
  float* spart = (float*)(ws + L.spart);
  if (T <= SKINNY_T) {
    // few tokens: the layer is bound by streaming the base matrices once; the small
    // per-expert products ride along in the two stream launches
    const int n_parts = (dm.d_ff + SKINNY_SN - 1) / SKINNY_SN;
    CMOE_LAUNCH(TS_GEMM1_BASE,
                launch_skinny_hb(dm, *w, (const half_t*)x, x_div, T, perm, offsets, expert_idx, t1ext, a, st));
    CMOE_LAUNCH(TS_RESID_UP, launch_skinny_resid_up(dm, *w, T, perm, expert_idx, gate, t1ext, a, spart, st));
    if (y_fused != nullptr && weights_combine_ok(w)) {
      float* ures = (float*)(ws + L.ures);
      CMOE_LAUNCH(TS_GEMM2, launch_skinny_down(dm, *w, a, T, offsets, (half_t*)y_base_sorted, perm, expert_idx, gate,
                                               spart, n_parts, ures, st));
      CMOE_LAUNCH(TS_COMBINE, launch_skinny_add(dm, (const half_t*)y_base_sorted, ures, perm, T, (half_t*)y_fused, st));
      *fused = true;
      return CMOE_OK;
    }
    CMOE_LAUNCH(TS_SREDUCE, launch_sreduce(dm, T, perm, spart, n_parts, s_down, st));
    CMOE_LAUNCH(TS_GEMM2, launch_skinny_down(dm, *w, a, T, offsets, (half_t*)y_base_sorted, nullptr, nullptr, nullptr,
                                             nullptr, 0, nullptr, st));
    return CMOE_OK;
  }
  // inside each cluster, order the rows by their selected experts; all intermediates live
  // in that refined order, the down-projection writes its rows back to the caller's
  // cluster-sorted (or token) order
  int* rm = (int*)(ws + L.sort_i32);
  int* p2 = rm + (size_t)T;
  CMOE_LAUNCH(TS_PERMUTE, launch_pair_sort(dm, perm, offsets, expert_idx, T, rm, p2, st));
  const int* rperm = p2;
  const int* rowmap = rm;
  // when the combine is fused into the down-projection its U2 panel joins the same launch
  const bool fuse = y_fused != nullptr && dm.KRp <= 128 && weights_combine_ok(w);
  half_t* u2t = !fuse ? nullptr : pk ? (half_t*)(pkb + PL.u2t) : (half_t*)(ws + L.u2t);
  if (!pk) CMOE_LAUNCH(TS_DEQUANT, launch_dequant_ffn(dm, *w, offsets, v1cat, u1t, v2p, u2t, st));
  CMOE_LAUNCH(TS_T1, launch_t1(dm, (const half_t*)x, x_div, T, rperm, offsets, expert_idx, v1cat, t1ext, st));
  CMOE_LAUNCH(TS_GEMM1, launch_gemm1(dm, *w, (const half_t*)x, x_div, T, rperm, offsets, expert_idx, gate, u1t, v2p,
                                     t1ext, a, spart, st));
  CMOE_LAUNCH(TS_SREDUCE, launch_sreduce(dm, T, rperm, spart, (dm.d_ff + G1_BN - 1) / G1_BN, s_down, st));
  if (fuse) {
    CMOE_LAUNCH(TS_GEMM2, launch_gemm2_combine(dm, *w, a, T, offsets, rperm, u2t, s_down, expert_idx, gate,
                                               (half_t*)y_fused, st));
    *fused = true;
    return CMOE_OK;
  }
  CMOE_LAUNCH(TS_GEMM2, launch_gemm2(dm, *w, a, T, offsets, rowmap, (half_t*)y_base_sorted, st));
  return CMOE_OK;
}

extern "C" int cmoe_combine(cmoe_handle* h, const cmoe_weights* w, const cmoe_f16* y_base_sorted,
                            const float* s_down, const int32_t* perm, const int32_t* inv_perm,
                            const int32_t* offsets, const int32_t* expert_idx, const float* gate, int32_t T,
                            cmoe_f16* y, void* workspace, size_t workspace_bytes, void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!weights_combine_ok(w)) return CMOE_ERR_INVALID_ARG;
  if (T == 0) return CMOE_OK;
  if (!ptr_ok(y_base_sorted) || !ptr_ok(s_down) || !ptr_ok(perm) || !ptr_ok(inv_perm) || !ptr_ok(offsets) ||
      !ptr_ok(expert_idx) || !ptr_ok(gate) || !ptr_ok(y))
    return CMOE_ERR_INVALID_ARG;
  int rc = check_ws(h, T, workspace, workspace_bytes);
  if (rc != CMOE_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  const cmoe_dims& dm = h->dm;
  cmoe_ws_layout L = cmoe_layout(dm, T);
  if (T <= SKINNY_T) {
    CMOE_LAUNCH(TS_COMBINE, launch_skinny_combine(dm, *w, (const half_t*)y_base_sorted, s_down, inv_perm,
                                                  expert_idx, gate, T, (half_t*)y, st));
    return CMOE_OK;
  }
  half_t* u2t = (half_t*)((char*)workspace + L.u2t);
  if (w->packed != nullptr)
    u2t = (half_t*)((const char*)w->packed + cmoe_packed(dm).u2t);
  else
    CMOE_LAUNCH(TS_DEQUANT, launch_dequant_u2(dm, *w, offsets, u2t, st));
  CMOE_LAUNCH(TS_COMBINE, launch_combine(dm, u2t, (const half_t*)y_base_sorted, s_down, perm, offsets, expert_idx,
                                         gate, T, (half_t*)y, st));
  return CMOE_OK;
}

static bool route_opt_ok(const cmoe_handle* h, const cmoe_route_options* o) {
  return o != nullptr && o->top_g >= 1 && o->top_g <= 8 && o->top_g <= h->dm.G && o->temperature > 0.f &&
         o->temperature < 1e30f;
}
// y of the virtual tokens, summed per token at the end
static size_t rep_bytes(const cmoe_dims& dm, size_t Tv) { return align_up(sizeof(half_t) * Tv * dm.d, 256); }

extern "C" int cmoe_route_multi(cmoe_handle* h, const cmoe_weights* w, const cmoe_route_options* opt,
                                const cmoe_f16* x, int32_t T, int32_t* cluster_id, int32_t* expert_idx, float* gate,
                                void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!route_opt_ok(h, opt) || !weights_route_ok(w)) return CMOE_ERR_INVALID_ARG;
  if (T == 0) return CMOE_OK;
  if (!ptr_ok(x) || !ptr_ok(cluster_id) || !ptr_ok(expert_idx) || !ptr_ok(gate)) return CMOE_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  CMOE_LAUNCH(TS_ROUTE, launch_route_multi(h->dm, *w, (const half_t*)x, T, opt->top_g, opt->temperature,
                                           opt->scale_by_cluster_prob != 0, cluster_id, expert_idx, gate, st));
  return CMOE_OK;
}

extern "C" size_t cmoe_workspace_bytes_multi(const cmoe_handle* h, int32_t T_max, int32_t top_g) {
  if (!handle_ok(h) || T_max < 0 || top_g < 1 || top_g > 8 || top_g > h->dm.G) return 0;
  if ((int64_t)T_max * top_g > INT32_MAX) return 0;
  const int Tv = T_max * top_g;
  return align_up(workspace_for_up_to(h->dm, Tv), 256) + rep_bytes(h->dm, (size_t)Tv);
}

extern "C" int cmoe_forward_multi(cmoe_handle* h, const cmoe_weights* w, const cmoe_route_options* opt,
                                  const cmoe_f16* x, int32_t T, cmoe_f16* y, int32_t* cluster_id,
                                  int32_t* expert_idx, float* gate, int32_t* perm, int32_t* inv_perm,
                                  int32_t* offsets, void* workspace, size_t workspace_bytes, void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!route_opt_ok(h, opt) || !weights_route_ok(w) || !weights_ffn_ok(w) || !weights_combine_ok(w))
    return CMOE_ERR_INVALID_ARG;
  if ((int64_t)T * opt->top_g > INT32_MAX) return CMOE_ERR_UNSUPPORTED;
  if (!ptr_ok(offsets)) return CMOE_ERR_INVALID_ARG;
  if (T > 0 && (!ptr_ok(x) || !ptr_ok(y) || !ptr_ok(cluster_id) || !ptr_ok(expert_idx) || !ptr_ok(gate) ||
                !ptr_ok(perm) || !ptr_ok(inv_perm)))
    return CMOE_ERR_INVALID_ARG;
  const int g1 = opt->top_g, Tv = T * g1;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return CMOE_ERR_WORKSPACE;
  const size_t base_bytes = align_up(cmoe_layout(h->dm, Tv).total, 256), rb = rep_bytes(h->dm, (size_t)Tv);
  if (workspace_bytes < base_bytes + rb) return CMOE_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  const cmoe_dims& dm = h->dm;
  char* ws = (char*)workspace;
  half_t* yrep = (half_t*)(ws + base_bytes);
  int rc = cmoe_route_multi(h, w, opt, x, T, cluster_id, expert_idx, gate, stream);
  if (rc != CMOE_OK) return rc;
  // from here on the virtual tokens are ordinary tokens of the single-cluster path
  rc = cmoe_permute(h, cluster_id, Tv, perm, inv_perm, offsets, workspace, base_bytes, stream);
  if (rc != CMOE_OK || T == 0) return rc;
  cmoe_ws_layout L = cmoe_layout(dm, Tv);
  cmoe_f16* yb = (cmoe_f16*)(ws + L.yb);
  float* s_down = (float*)(ws + L.sdown);
  bool fused = false;
  // virtual token vt reads row vt / top_g of x
  rc = ffn_impl(h, w, x, Tv, perm, offsets, expert_idx, gate, yb, s_down, (cmoe_f16*)yrep, &fused, g1, workspace,
                base_bytes, stream);
  if (rc != CMOE_OK) return rc;
  if (!fused) {
    rc = cmoe_combine(h, w, yb, s_down, perm, inv_perm, offsets, expert_idx, gate, Tv, (cmoe_f16*)yrep, workspace,
                      base_bytes, stream);
    if (rc != CMOE_OK) return rc;
  }
  CMOE_LAUNCH(TS_COMBINE, launch_sum_groups(yrep, T, g1, dm.d, (half_t*)y, st));
  return CMOE_OK;
}

extern "C" int cmoe_route_stats(cmoe_handle* h, const cmoe_f16* x, int32_t T, const int32_t* perm,
                                const int32_t* offsets, const int32_t* expert_idx, float beta, float lam, float* mu,
                                float* cluster_act, int32_t* cluster_idle, int32_t* expert_load,
                                int32_t* cluster_load, float* i_load, void* workspace, size_t workspace_bytes,
                                void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!(beta >= 0.f && beta <= 1.f) || !(lam >= 0.f && lam <= 1.f)) return CMOE_ERR_INVALID_ARG;
  if (!ptr_ok(offsets) || !ptr_ok(mu) || !ptr_ok(cluster_act) || !ptr_ok(cluster_idle) || !ptr_ok(expert_load) ||
      !ptr_ok(cluster_load) || !ptr_ok(i_load))
    return CMOE_ERR_INVALID_ARG;
  if (T > 0 && (!ptr_ok(x) || !ptr_ok(perm) || !ptr_ok(expert_idx))) return CMOE_ERR_INVALID_ARG;
  int rc = check_ws(h, T, workspace, workspace_bytes);
  if (rc != CMOE_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  cmoe_ws_layout L = cmoe_layout(h->dm, T);
  char* ws = (char*)workspace;
  CMOE_LAUNCH(TS_STATS, launch_route_stats(h->dm, (const half_t*)x, T, perm, offsets, expert_idx, beta, lam, mu,
                                           cluster_act, cluster_idle, expert_load, cluster_load, i_load,
                                           (float*)(ws + L.stats_part), (int*)(ws + L.stats_cnt), st));
  return CMOE_OK;
}

extern "C" size_t cmoe_packed_bytes(const cmoe_handle* h) {
  if (!handle_ok(h)) return 0;
  return cmoe_packed(h->dm).total;
}

extern "C" int cmoe_pack_weights(cmoe_handle* h, const cmoe_weights* w, void* packed, size_t packed_bytes,
                                 void* stream) {
  if (!handle_ok(h) || w == nullptr || !ptr_ok(w->w1_base) || !ptr_ok(w->w2_base)) return CMOE_ERR_INVALID_ARG;
  if (!ptr_ok(w->v1_q) || !ptr_ok(w->u1_q) || !ptr_ok(w->v2_q) || !ptr_ok(w->u2_q) || !ptr_ok(w->v1_s) ||
      !ptr_ok(w->u1_s) || !ptr_ok(w->v2_s) || !ptr_ok(w->u2_s))
    return CMOE_ERR_INVALID_ARG;
  if (packed == nullptr || (reinterpret_cast<uintptr_t>(packed) & 255u) != 0) return CMOE_ERR_INVALID_ARG;
  if (packed_bytes < cmoe_packed_bytes(h)) return CMOE_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  hipError_t e = launch_pack_bases(h->dm, *w, (half_t*)packed, st);
  if (e != hipSuccess) {
    h->last_hip_error = (int)e;
    return CMOE_ERR_HIP;
  }
  return CMOE_OK;
}

extern "C" size_t cmoe_backward_workspace_bytes(const cmoe_handle* h, int32_t T_max) {
  if (!handle_ok(h) || T_max < 0) return 0;
  if ((size_t)T_max * h->dm.k > ((size_t)1 << 30)) return 0;
  return cmoe_backward_layout(h->dm, T_max).total;
}

extern "C" int cmoe_backward(cmoe_handle* h, const cmoe_weights* w, const cmoe_f16* x, const cmoe_f16* dy, int32_t T,
                             const int32_t* expert_idx, const float* gate, const cmoe_grads* grads, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (!handle_ok(h) || T < 0 || grads == nullptr) return CMOE_ERR_INVALID_ARG;
  if (!weights_route_ok(w) || !weights_ffn_ok(w) || !weights_combine_ok(w)) return CMOE_ERR_INVALID_ARG;
  if ((size_t)T * h->dm.k > ((size_t)1 << 30)) return CMOE_ERR_UNSUPPORTED;
  const cmoe_grads& g = *grads;
  if (!ptr_ok(g.d_router_expert) || !ptr_ok(g.dw1_base) || !ptr_ok(g.dw2_base) || !ptr_ok(g.du1) || !ptr_ok(g.dv1) ||
      !ptr_ok(g.du2) || !ptr_ok(g.dv2) || (g.d_logits != nullptr && !aligned16(g.d_logits)))
    return CMOE_ERR_INVALID_ARG;
  if (T > 0 && (!ptr_ok(x) || !ptr_ok(dy) || !ptr_ok(expert_idx) || !ptr_ok(gate) || !ptr_ok(g.dx)))
    return CMOE_ERR_INVALID_ARG;
  if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return CMOE_ERR_WORKSPACE;
  const cmoe_bw_layout L = cmoe_backward_layout(h->dm, T);
  if (workspace_bytes < L.total) return CMOE_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  CMOE_LAUNCH(TS_BACKWARD, launch_backward(h->dm, *w, (const half_t*)x, (const half_t*)dy, T, expert_idx, gate, g,
                                           (char*)workspace, L, st));
  return CMOE_OK;
}

extern "C" int cmoe_forward(cmoe_handle* h, const cmoe_weights* w, const cmoe_f16* x, int32_t T, cmoe_f16* y,
                            int32_t* cluster_id, int32_t* expert_idx, float* gate, int32_t* perm, int32_t* inv_perm,
                            int32_t* offsets, void* workspace, size_t workspace_bytes, void* stream) {
  if (!handle_ok(h) || T < 0) return CMOE_ERR_INVALID_ARG;
  if (!weights_route_ok(w) || !weights_ffn_ok(w) || !weights_combine_ok(w)) return CMOE_ERR_INVALID_ARG;
  if (!ptr_ok(offsets)) return CMOE_ERR_INVALID_ARG;
  if (T > 0 && (!ptr_ok(x) || !ptr_ok(y) || !ptr_ok(cluster_id) || !ptr_ok(expert_idx) || !ptr_ok(gate) ||
                !ptr_ok(perm) || !ptr_ok(inv_perm)))
    return CMOE_ERR_INVALID_ARG;
  int rc = check_ws(h, T, workspace, workspace_bytes);
  if (rc != CMOE_OK) return rc;
  cmoe_ws_layout L = cmoe_layout(h->dm, T);
  char* ws = (char*)workspace;
  cmoe_f16* yb = (cmoe_f16*)(ws + L.yb);
  float* s_down = (float*)(ws + L.sdown);
  rc = cmoe_route(h, w, x, T, cluster_id, expert_idx, gate, stream);
  if (rc != CMOE_OK) return rc;
  rc = cmoe_permute(h, cluster_id, T, perm, inv_perm, offsets, workspace, workspace_bytes, stream);
  if (rc != CMOE_OK || T == 0) return rc;
  bool fused = false;
  rc = ffn_impl(h, w, x, T, perm, offsets, expert_idx, gate, yb, s_down, y, &fused, 1, workspace, workspace_bytes,
                stream);
  if (rc != CMOE_OK || fused) return rc;
  return cmoe_combine(h, w, yb, s_down, perm, inv_perm, offsets, expert_idx, gate, T, y, workspace, workspace_bytes,
                      stream);
}
