// Backward pass of the layer for a frozen selection (the training step of Sec. 3.5): the
// gradients of L = sum(dy * y) with respect to x, the expert-router rows, the shared bases
// and the dequantised low-rank factors, for y of Sec. 3.2 / Eq. 7 with the gates of Eq. 10.
//
// The base reuse of Sec. 3.2 carries over to every product of the chain rule.  With
// W_e = B_c + U_e V_e, tokens sorted by cluster and (token, expert) pairs m = t k + j sorted
// by expert:
//   h_m  = B1 x_t + U1 (V1 x_t)                 base product once per token, rank-r per pair
//   da_m = B2^T dy_t + V2^T (U2^T dy_t)         likewise
//   a_m = GELU(h_m), dg_m = da_m . a_m, dh_m = g_m da_m GELU'(h_m)
//   dx_t = B1^T (sum_j dh_m) + sum_j V1^T (U1^T dh_m) + gate path
//   dB1_c = sum_{t in c} (sum_j dh_m) x_t^T     dB2_c = sum_{t in c} dy_t (sum_j g_m a_m)^T
//   dU1_e = sum_m dh_m (V1 x_t)^T   dV1_e = sum_m (U1^T dh_m) x_t^T
//   dU2_e = sum_m g_m dy_t (V2 a_m)^T   dV2_e = sum_m g_m (U2^T dy_t) a_m^T
// The five products with a base and the four products into rank space (V1 x, U2^T dy,
// U1^T dh, V2 a; rank panels padded to 32 rows) run on the grouped matrix-core kernel of the
// forward pass.  The two base gradients contract over the tokens of a cluster: they use
// transposed copies that pad every cluster to a multiple of 32 columns and are stored in
// 32-column blocks.  The ways back from rank space (U1 t, V2^T u, V1^T q) and the factor
// gradients (r output rows per expert) are vector-ALU kernels that stream the pair rows of
// an expert once.
#include "cmoe_internal.h"

namespace {

constexpr int RP = 32;   // padded rank

__device__ __forceinline__ float nib_val(unsigned byte, int odd) {
  return (float)(odd ? ((int)(byte << 24) >> 28) : ((int)(byte << 28) >> 28));
}

// FP16 panel of one INT4 factor F [E][r][L] (value = scale * code): rows_out [E][32][L], rank
// rows >= r zero.  Experts without pairs are skipped: their stored factors are never read.
// Block (L / 256, E).
__global__ __launch_bounds__(256) void bw_panel_kernel(const uint8_t* __restrict__ qv, const half_t* __restrict__ sv,
                                                       int L, int q, int r, const int* __restrict__ offe,
                                                       half_t* __restrict__ rows_out) {
  const int e = blockIdx.y;
  if (offe[e + 1] == offe[e]) return;
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= L) return;
  for (int rho = 0; rho < RP; ++rho) {
    float f = 0.f;
    if (rho < r) {
      const size_t row = (size_t)e * r + rho;
      f = (float)sv[row * (L / q) + i / q] * nib_val(qv[row * (L / 2) + i / 2], i & 1);
    }
    rows_out[((size_t)e * RP + rho) * L + i] = (half_t)f;
  }
}

// cluster of a token = cluster of its first selected expert
__global__ __launch_bounds__(256) void bw_cluster_kernel(const int* __restrict__ expert_idx, int T, int k, int K,
                                                         int* __restrict__ cid) {
  const int t = blockIdx.x * 256 + threadIdx.x;
  if (t < T) cid[t] = expert_idx[(size_t)t * k] / K;
}

// More than 64 experts: the pairs are sorted by expert in two stable counting sorts, by the
// expert's index inside its cluster and then by cluster.
// mode 0: key[i] = expert_idx[i] % K;  mode 1: key[i] = expert_idx[perm_a[i]] / K.
__global__ __launch_bounds__(256) void bw_key_kernel(const int* __restrict__ expert_idx,
                                                     const int* __restrict__ perm_a, int M, int K, int E, int mode,
                                                     int* __restrict__ key) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M) return;
  const int e = min(max(expert_idx[mode ? perm_a[i] : i], 0), E - 1);
  key[i] = mode ? e / K : e % K;
}

// permm[i] = perm_a[perm_b[i]], invm[permm[i]] = i, and the expert offsets from the sorted
// keys: offe[e] = first sorted row whose expert is >= e, offe[E] = M.
__global__ __launch_bounds__(256) void bw_compose_kernel(const int* __restrict__ expert_idx,
                                                         const int* __restrict__ perm_a,
                                                         const int* __restrict__ perm_b, int M, int E,
                                                         int* __restrict__ permm, int* __restrict__ invm,
                                                         int* __restrict__ offe) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= M) return;
  const int m = perm_a[perm_b[i]];
  permm[i] = m;
  invm[m] = i;
  const int e = min(max(expert_idx[m], 0), E - 1);
  const int prev = i > 0 ? min(max(expert_idx[perm_a[perm_b[i - 1]]], 0), E - 1) : -1;
  for (int x = prev + 1; x <= e; ++x) offe[x] = i;
  if (i == M - 1)
    for (int x = e + 1; x <= E; ++x) offe[x] = M;
}

// Column ranges of the group-padded transposed copies and, for every padded column qc, the
// sorted row it holds (-1: padding), the source row perm[row] / div and its gate.
// krange[2g] = first column of group g, krange[2g+1] = its rows rounded up to 32.
__global__ __launch_bounds__(256) void bw_map_kernel(const int* __restrict__ off, const int* __restrict__ perm,
                                                     const float* __restrict__ gate, int n_groups, int div, int Npad,
                                                     int* __restrict__ krange, int* __restrict__ srow,
                                                     int* __restrict__ ssrc, float* __restrict__ sgate) {
  __shared__ int start[65];
  if (threadIdx.x == 0) {
    int at = 0;
    for (int g = 0; g < n_groups; ++g) {
      start[g] = at;
      at += (off[g + 1] - off[g] + 31) / 32 * 32;
    }
    start[n_groups] = at;
  }
  __syncthreads();
  if (blockIdx.x == 0)
    for (int g = threadIdx.x; g < n_groups; g += 256) {
      krange[2 * g] = start[g];
      krange[2 * g + 1] = start[g + 1] - start[g];
    }
  const int qc = blockIdx.x * 256 + threadIdx.x;
  if (qc >= Npad) return;
  int row = -1;
  for (int g = 0; g < n_groups; ++g)
    if (qc >= start[g] && qc < start[g + 1]) {
      const int local = qc - start[g];
      if (local < off[g + 1] - off[g]) row = off[g] + local;
    }
  srow[qc] = row;
  const int m = row >= 0 ? perm[row] : 0;
  ssrc[qc] = row >= 0 ? m / div : -1;
  if (sgate != nullptr) sgate[qc] = row >= 0 ? gate[m] : 0.f;
}

__global__ __launch_bounds__(256) void bw_zero_kernel(int* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// offx[g] = g * I (g <= n_groups) and gidx[p] = p % I for the n_groups * I rows of a
// weight gradient.
__global__ __launch_bounds__(256) void bw_rows_kernel(int n_groups, int I, int* __restrict__ offx,
                                                      int* __restrict__ gidx) {
  const size_t p = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (p <= (size_t)n_groups) offx[p] = (int)p * I;
  if (p < (size_t)n_groups * I) gidx[p] = (int)(p % I);
}

// One token per block.  For its k pairs (sorted rows p_j = invm[t k + j]):
//   h = hb[t] + rh[p_j], da = dab[t] + rda[p_j]          FP32 sums of FP16 base and rank parts
//   a16[p_j] = GELU(h), dh16[p_j] = g_j da GELU'(h), dg_j = da . GELU(h)
//   dhsum16[t] = sum_j dh, ag16[t] = sum_j g_j GELU(h)
// and the softmax backward over the selected logits (Eq. 10):
//   dl_j = g_j (dg_j - sum_i g_i dg_i).
// The gate gradient is a difference of nearly equal dg of experts that share a base: the
// base parts hb, dab enter every dg_j of the token with the same rounding, so the
// differences keep the relative accuracy of the rank parts.
template <int KMAX>
__global__ __launch_bounds__(256) void bw_act_kernel(const half_t* __restrict__ hb, const half_t* __restrict__ dab,
                                                     const half_t* __restrict__ rh, const half_t* __restrict__ rda,
                                                     const int* __restrict__ invm, const float* __restrict__ gate,
                                                     int k, int d_ff, half_t* __restrict__ a16,
                                                     half_t* __restrict__ dh16, half_t* __restrict__ dhsum16,
                                                     half_t* __restrict__ ag16, float* __restrict__ dl) {
  __shared__ float red[KMAX][4];
  const size_t t = blockIdx.x;
  size_t prow[KMAX];
  float g[KMAX], dot[KMAX];
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    prow[j] = j < k ? (size_t)invm[t * k + j] : 0;
    g[j] = j < k ? gate[t * k + j] : 0.f;
    dot[j] = 0.f;
  }
  for (int col = threadIdx.x * 4; col < d_ff; col += 1024) {
    const half4 hv = __builtin_nontemporal_load((const half4*)(hb + t * d_ff + col));
    const half4 dv = __builtin_nontemporal_load((const half4*)(dab + t * d_ff + col));
    float dhs[4] = {0.f, 0.f, 0.f, 0.f}, ags[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      if (j >= k) break;
      const half4 r1 = __builtin_nontemporal_load((const half4*)(rh + prow[j] * d_ff + col));
      const half4 r2 = __builtin_nontemporal_load((const half4*)(rda + prow[j] * d_ff + col));
      half4 ao, ho;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float u = (float)hv[i] + (float)r1[i], z = (float)dv[i] + (float)r2[i];
        const float cdf = 0.5f * (1.f + erff(u * 0.70710678118654752f));
        const float pdf = 0.3989422804014327f * __expf(-0.5f * u * u);
        const float a = u * cdf, dh = g[j] * z * (cdf + u * pdf);
        dot[j] += z * a;
        ao[i] = (half_t)a;
        ho[i] = (half_t)dh;
        dhs[i] += dh;
        ags[i] += g[j] * a;
      }
      __builtin_nontemporal_store(ao, (half4*)(a16 + prow[j] * d_ff + col));
      __builtin_nontemporal_store(ho, (half4*)(dh16 + prow[j] * d_ff + col));
    }
    *(half4*)(dhsum16 + t * d_ff + col) = half4{(half_t)dhs[0], (half_t)dhs[1], (half_t)dhs[2], (half_t)dhs[3]};
    *(half4*)(ag16 + t * d_ff + col) = half4{(half_t)ags[0], (half_t)ags[1], (half_t)ags[2], (half_t)ags[3]};
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int j = 0; j < KMAX; ++j) {
    float v = dot[j];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) red[j][wave] = v;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float dg[KMAX], mean = 0.f;
#pragma unroll
    for (int j = 0; j < KMAX; ++j) {
      dg[j] = (red[j][0] + red[j][1]) + (red[j][2] + red[j][3]);
      mean += g[j] * dg[j];
    }
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
      if (j < k) dl[t * k + j] = g[j] * (dg[j] - mean);
  }
}

// dx[t] = dxb[t] + sum_j dxr[t k + j] + sum_j dl_j v_{e_j}: shared-base part, per-pair
// residual part, and the gate path of Eq. 10.
__global__ __launch_bounds__(256) void bw_dx_kernel(const half_t* __restrict__ dxb, const half_t* __restrict__ dxr,
                                                    const float* __restrict__ dl, const int* __restrict__ expert_idx,
                                                    const half_t* __restrict__ router_expert, int k, int d,
                                                    float* __restrict__ dx) {
  const size_t t = blockIdx.x;
  const int col = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (col >= d) return;
  const half4 b4 = *(const half4*)(dxb + t * d + col);
  float4v acc = {(float)b4[0], (float)b4[1], (float)b4[2], (float)b4[3]};
  for (int j = 0; j < k; ++j) {
    const half4 r4 = *(const half4*)(dxr + (t * k + j) * d + col);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += (float)r4[i];
    const float c = dl[t * k + j];
    const half4 v = *(const half4*)(router_expert + (size_t)expert_idx[t * k + j] * d + col);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] += c * (float)v[i];
  }
  *(float4v*)(dx + t * d + col) = acc;
}

// d v_e = sum over the pair rows of expert e of dl_m x_t: part[run][e][col], the rows of the
// expert cut into DR_SPLIT runs added in row order (bw_rankgrad_finish_kernel adds the runs).
// Block (E, ceil(d / 1024), DR_SPLIT).
constexpr int DR_SPLIT = 4;
__global__ __launch_bounds__(256) void bw_drouter_kernel(const half_t* __restrict__ x, const int* __restrict__ permm,
                                                         const int* __restrict__ offe, const float* __restrict__ dl,
                                                         int k, int d, int E, float* __restrict__ part) {
  const int e = blockIdx.x, sp = blockIdx.z;
  const int col = (blockIdx.y * 256 + threadIdx.x) * 4;
  if (col >= d) return;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  const int lo = offe[e], n = offe[e + 1] - lo;
  const int per = (n + DR_SPLIT - 1) / DR_SPLIT;
  const int p_lo = lo + sp * per, p_hi = min(lo + n, p_lo + per);
  for (int p0 = p_lo; p0 < p_hi; p0 += 8) {
    half4 v[8];
    float c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const bool ok = p0 + u < p_hi;
      const int m = ok ? permm[p0 + u] : 0;
      c[u] = ok ? dl[m] : 0.f;
      v[u] = *(const half4*)(x + (size_t)(m / k) * d + col);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] += c[u] * (float)v[u][i];
  }
  *(float4v*)(part + ((size_t)sp * E + e) * d + col) = float4v{acc[0], acc[1], acc[2], acc[3]};
}

// out[z][i][qc] = scale[qc] * src[z][idx[qc]][i] (zero where idx[qc] < 0; idx == NULL: row
// qc), i < I (a multiple of 16), qc < Npad (a multiple of 64); with blocked != 0 the same
// values in the layout [Npad / 32][I][32].  Matrices z whose group in
// skip_off is empty are skipped.  src_blk != 0: src[z] is stored as [I / 32][rows][32] with
// src_blk = rows * 32 (the re-tiled copy of a base matrix) instead of row-major with row
// stride ld.  Block (Npad / 64, ceil(I / 64), Z): 64 x 64 tile through LDS.
__global__ __launch_bounds__(256) void bw_transpose_kernel(const half_t* __restrict__ src, int ld, long src_blk, int I,
                                                           const int* __restrict__ idx,
                                                           const float* __restrict__ scale, int Npad,
                                                           const int* __restrict__ skip_off, size_t zstride,
                                                           int blocked, half_t* __restrict__ out) {
  __shared__ half_t tile[64][72];
  const int z = blockIdx.z;
  if (skip_off != nullptr && skip_off[z + 1] == skip_off[z]) return;
  src += z * zstride;
  out += z * zstride;
  const int q0 = blockIdx.x * 64, i0 = blockIdx.y * 64, tid = threadIdx.x;
  {
    const int ql = tid >> 2, part = tid & 3;
    const int row = idx != nullptr ? idx[q0 + ql] : q0 + ql;
    half8 a = {0, 0, 0, 0, 0, 0, 0, 0}, b = a;
    if (row >= 0 && i0 + part * 16 < I) {
      const int col = i0 + part * 16;   // 16 columns inside one 32-column block
      const half_t* sp = src_blk ? src + (size_t)(col >> 5) * src_blk + (size_t)row * 32 + (col & 31)
                                 : src + (size_t)row * ld + col;
      a = *(const half8*)sp;
      b = *(const half8*)(sp + 8);
      if (scale != nullptr) {
        const float s = scale[q0 + ql];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          a[i] = (half_t)(s * (float)a[i]);
          b[i] = (half_t)(s * (float)b[i]);
        }
      }
    }
    *(half8*)&tile[ql][part * 16] = a;
    *(half8*)&tile[ql][part * 16 + 8] = b;
  }
  __syncthreads();
  const int il = tid >> 2, part = tid & 3;
  if (i0 + il >= I) return;
  half8 a, b;
#pragma unroll
  for (int u = 0; u < 8; ++u) {
    a[u] = tile[part * 16 + u][il];
    b[u] = tile[part * 16 + 8 + u][il];
  }
  // blocked: [Npad / 32][I][32], the operand layout whose contraction blocks are contiguous
  const int qq = q0 + part * 16;
  half_t* dst = blocked ? out + ((size_t)(qq >> 5) * I + i0 + il) * 32 + (qq & 31)
                        : out + (size_t)(i0 + il) * Npad + qq;
  *(half8*)dst = a;
  *(half8*)(dst + 8) = b;
}

// Rank-space rows back to full width: out[row(p)][n] = sum_{rho < R} t[p][rho] P[e][rho][n] for
// the sorted pair rows p of expert e (P = a [E][32][L] panel), row(p) = rowmap ? rowmap[p] : p.
// A thread keeps its 4 columns of the R panel rows in registers (as FP16 pairs of rank rows,
// multiplied by v_dot2_f32_f16: exact products, FP32 sums) and walks the rows of its run.
// Block (ceil(L / 1024), E, RX_SPLIT).
constexpr int RX_SPLIT = 8;
template <int R, class OutT>
__global__ __launch_bounds__(256) void bw_rankexpand_kernel(const half_t* __restrict__ t,
                                                            const half_t* __restrict__ P, int L,
                                                            const int* __restrict__ offe,
                                                            const int* __restrict__ rowmap, OutT* __restrict__ out) {
  const int e = blockIdx.y, sp = blockIdx.z;
  const int col = (blockIdx.x * 256 + threadIdx.x) * 4;
  if (col >= L) return;
  const int lo = offe[e], n = offe[e + 1] - lo;
  const int per = (n + RX_SPLIT - 1) / RX_SPLIT;
  const int p0 = lo + sp * per, p1 = min(lo + n, p0 + per);
  if (p0 >= p1) return;
  // the panel rows in pairs (rho, rho + 1): one two-element dot product per pair and column
  half2v w[R / 2][4];
#pragma unroll
  for (int q2 = 0; q2 < R / 2; ++q2) {
    const half4 v0 = *(const half4*)(P + ((size_t)e * RP + 2 * q2) * L + col);
    const half4 v1 = *(const half4*)(P + ((size_t)e * RP + 2 * q2 + 1) * L + col);
#pragma unroll
    for (int i = 0; i < 4; ++i) w[q2][i] = half2v{v0[i], v1[i]};
  }
  for (int pb = p0; pb < p1; pb += 4) {
    float acc[4][4];
    size_t row[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int p = min(pb + u, p1 - 1);
      row[u] = rowmap != nullptr ? (size_t)rowmap[p] : (size_t)p;
      const half2v* tp = (const half2v*)(t + (size_t)p * RP);
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[u][i] = 0.f;
#pragma unroll
      for (int q2 = 0; q2 < R / 2; ++q2) {
        const half2v tv = tp[q2];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[u][i] = __builtin_amdgcn_fdot2(tv, w[q2][i], acc[u][i], false);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (pb + u >= p1) break;
      if constexpr (sizeof(OutT) == 2)
        __builtin_nontemporal_store(half4{(half_t)acc[u][0], (half_t)acc[u][1], (half_t)acc[u][2], (half_t)acc[u][3]},
                                    (half4*)(out + row[u] * L + col));
      else
        *(float4v*)(out + row[u] * L + col) = float4v{acc[u][0], acc[u][1], acc[u][2], acc[u][3]};
    }
  }
}

template <class OutT>
void rankexpand(int r, const half_t* t, const half_t* P, int L, const int* offe, const int* rowmap, int E, OutT* out,
                hipStream_t st) {
  const dim3 grid((L + 1023) / 1024, E, RX_SPLIT), block(256);
  switch (r) {
    case 4: hipLaunchKernelGGL((bw_rankexpand_kernel<4, OutT>), grid, block, 0, st, t, P, L, offe, rowmap, out); break;
    case 8: hipLaunchKernelGGL((bw_rankexpand_kernel<8, OutT>), grid, block, 0, st, t, P, L, offe, rowmap, out); break;
    case 16: hipLaunchKernelGGL((bw_rankexpand_kernel<16, OutT>), grid, block, 0, st, t, P, L, offe, rowmap, out); break;
    default: hipLaunchKernelGGL((bw_rankexpand_kernel<32, OutT>), grid, block, 0, st, t, P, L, offe, rowmap, out); break;
  }
}

// Factor gradients: part[sp][e][rho][n] = sum over the sorted pair rows p of expert e in
// split sp of t[p][rho] * D[row(p)][n], rho < R; row(p) = p (D in sorted pair order) or
// permm[p] / k (D = x or dy); a gate factor is folded into t beforehand (bw_scale_kernel).
// Products are exact (FP16 x FP16), sums FP32.  The rows of an expert are cut
// into RG_SPLIT equal runs, added in row order; bw_rankgrad_finish_kernel adds the runs in
// order.  One thread owns C consecutive columns n.  Block (ceil(L / (256 C)), E, RG_SPLIT).
constexpr int RG_SPLIT = 4;
template <int R, int C>
__global__ __launch_bounds__(256) void bw_rankgrad_kernel(const half_t* __restrict__ t, const half_t* __restrict__ D,
                                                          int L, const int* __restrict__ offe,
                                                          const int* __restrict__ permm, int k, int gather,
                                                          int E, float* __restrict__ part) {
  typedef _Float16 halfC __attribute__((ext_vector_type(C)));
  const int e = blockIdx.y, sp = blockIdx.z;
  const int col = (blockIdx.x * 256 + threadIdx.x) * C;
  if (col >= L) return;
  const int lo = offe[e], n = offe[e + 1] - lo;
  const int per = (n + RG_SPLIT - 1) / RG_SPLIT;
  const int p0 = lo + sp * per, p1 = min(lo + n, p0 + per);
  float acc[R][C];
#pragma unroll
  for (int rho = 0; rho < R; ++rho)
#pragma unroll
    for (int i = 0; i < C; ++i) acc[rho][i] = 0.f;
  // Four rows per batch, multiplied in pairs of rows: acc += t[p][rho] D[p][n] +
  // t[p+1][rho] D[p+1][n] is one v_dot2_f32_f16.  The loads of the next batch are issued
  // before the current one is used, so that a wavefront keeps eight rows in flight.
  auto load = [&](int pb, halfC (&v)[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int p = min(pb + u, p1 - 1);
      const size_t row = gather ? (size_t)(permm[p] / k) : (size_t)p;
      v[u] = *(const halfC*)(D + row * L + col);
    }
  };
  halfC cur[4], nxt[4];
  if (p0 < p1) load(p0, cur);
  for (int pb = p0; pb < p1; pb += 4) {
    if (pb + 4 < p1) load(pb + 4, nxt);
    const half_t* tp[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (pb + u >= p1) cur[u] = halfC{};          // rows past the run contribute nothing
      tp[u] = t + (size_t)min(pb + u, p1 - 1) * RP;
    }
#pragma unroll
    for (int u = 0; u < 4; u += 2) {
      half2v dv[C];
#pragma unroll
      for (int i = 0; i < C; ++i) dv[i] = half2v{cur[u][i], cur[u + 1][i]};
#pragma unroll
      for (int rho = 0; rho < R; ++rho) {
        const half2v tv = half2v{tp[u][rho], tp[u + 1][rho]};
#pragma unroll
        for (int i = 0; i < C; ++i) acc[rho][i] = __builtin_amdgcn_fdot2(tv, dv[i], acc[rho][i], false);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) cur[u] = nxt[u];
  }
#pragma unroll
  for (int rho = 0; rho < R; ++rho) {
    float* dst = part + (((size_t)sp * E + e) * R + rho) * L + col;
#pragma unroll
    for (int i = 0; i < C; i += 4) *(float4v*)(dst + i) = float4v{acc[rho][i], acc[rho][i + 1], acc[rho][i + 2], acc[rho][i + 3]};
  }
}

// out[i] = part[0][i] + part[1][i] + ... in split order, i < n (a multiple of 4)
__global__ __launch_bounds__(256) void bw_rankgrad_finish_kernel(const float* __restrict__ part, size_t n,
                                                                 float* __restrict__ out) {
  const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  float4v acc = *(const float4v*)(part + i);
  for (int sp = 1; sp < RG_SPLIT; ++sp) acc += *(const float4v*)(part + sp * n + i);
  *(float4v*)(out + i) = acc;
}

// t[p][rho] *= gate[permm[p]] for the M sorted pair rows (32 rank columns each)
__global__ __launch_bounds__(256) void bw_scale_kernel(half_t* __restrict__ t, const int* __restrict__ permm,
                                                       const float* __restrict__ gate, int M) {
  const int idx = blockIdx.x * 256 + threadIdx.x, p = idx >> 2;
  if (p >= M) return;
  const float g = gate[permm[p]];
  half8* v = (half8*)(t + (size_t)p * RP + (idx & 3) * 8);
  half8 x = *v;
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = (half_t)(g * (float)x[i]);
  *v = x;
}

template <int R>
void rankgrad_r(const half_t* t, const half_t* D, int L, const int* offe, const int* permm, int k, int gather,
                int E, float* part, float* out, hipStream_t st) {
  constexpr int C = R >= 32 ? 4 : 8;
  hipLaunchKernelGGL((bw_rankgrad_kernel<R, C>), dim3((L + 256 * C - 1) / (256 * C), E, RG_SPLIT), dim3(256), 0, st, t,
                     D, L, offe, permm, k, gather, E, part);
  const size_t n = (size_t)E * R * L;
  hipLaunchKernelGGL(bw_rankgrad_finish_kernel, dim3((unsigned)((n / 4 + 255) / 256)), dim3(256), 0, st, part, n, out);
}

void rankgrad(int r, const half_t* t, const half_t* D, int L, const int* offe, const int* permm, int k, int gather,
              int E, float* part, float* out, hipStream_t st) {
  switch (r) {
    case 4: rankgrad_r<4>(t, D, L, offe, permm, k, gather, E, part, out, st); break;
    case 8: rankgrad_r<8>(t, D, L, offe, permm, k, gather, E, part, out, st); break;
    case 16: rankgrad_r<16>(t, D, L, offe, permm, k, gather, E, part, out, st); break;
    default: rankgrad_r<32>(t, D, L, offe, permm, k, gather, E, part, out, st); break;
  }
}

inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

void transpose(const half_t* src, int ld, int I, const int* idx, const float* scale, int Npad, half_t* out,
               hipStream_t st) {
  hipLaunchKernelGGL(bw_transpose_kernel, dim3(Npad / 64, (I + 63) / 64, 1), dim3(256), 0, st, src, ld, 0L, I, idx, scale,
                     Npad, (const int*)nullptr, (size_t)0, 1, out);
}

}  // namespace

cmoe_bw_layout cmoe_backward_layout(const cmoe_dims& dm, int T) {
  cmoe_bw_layout L;
  const size_t E = (size_t)dm.G * dm.K, G = dm.G, Tz = (size_t)(T > 0 ? T : 0), M = Tz * dm.k;
  const size_t d = dm.d, f = dm.d_ff, r = dm.r;
  L.M = (int)M;
  L.Tpad = (int)((Tz + 32 * G + 63) / 64 * 64);
  const size_t Tp = L.Tpad;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off = up256(off + bytes);
    return at;
  };
  const size_t n_blocks = (M + PERMUTE_BLOCK - 1) / PERMUTE_BLOCK;
  L.blk_counts = take(sizeof(int) * (n_blocks + 1) * 64);
  L.cid = take(sizeof(int) * Tz);
  L.permc = take(sizeof(int) * Tz);
  L.invc = take(sizeof(int) * Tz);
  L.offc = take(sizeof(int) * (G + 1));
  L.permm = take(sizeof(int) * M);
  L.invm = take(sizeof(int) * M);
  L.offe = take(sizeof(int) * (E + 1));
  L.sort_tmp = take(E > 64 ? sizeof(int) * 4 * M : 0);   // key, perm_a, perm_b, scratch inverse
  L.off_tmp = take(sizeof(int) * 65);
  L.krange_c = take(sizeof(int) * 2 * G);
  L.srow_c = take(sizeof(int) * Tp);
  L.ssrc_c = take(sizeof(int) * Tp);
  L.offx_f = take(sizeof(int) * (G + 1));
  L.gidx_f = take(sizeof(int) * G * f);
  L.offx_d = take(sizeof(int) * (G + 1));
  L.gidx_d = take(sizeof(int) * G * d);
  L.dl = take(sizeof(float) * M);
  L.v1p = take(sizeof(half_t) * E * 32 * d);
  L.u2p = take(sizeof(half_t) * E * 32 * d);
  L.u1p = take(sizeof(half_t) * E * 32 * f);
  L.v2p = take(sizeof(half_t) * E * 32 * f);
  L.w1bt = take(sizeof(half_t) * G * f * d);
  L.w2bt = take(sizeof(half_t) * G * f * d);
  L.hb = take(sizeof(half_t) * Tz * f);
  L.dab = take(sizeof(half_t) * Tz * f);
  L.rh = take(sizeof(half_t) * M * f);
  L.rda = take(sizeof(half_t) * M * f);
  L.a16 = take(sizeof(half_t) * M * f);
  L.dh16 = take(sizeof(half_t) * M * f);
  L.dhsum16 = take(sizeof(half_t) * Tz * f);
  L.ag16 = take(sizeof(half_t) * Tz * f);
  L.t1 = take(sizeof(half_t) * M * 32);
  L.uy = take(sizeof(half_t) * M * 32);
  L.qq = take(sizeof(half_t) * M * 32);
  L.ss = take(sizeof(half_t) * M * 32);
  L.dxb = take(sizeof(half_t) * Tz * d);
  L.dxr = take(sizeof(half_t) * M * d);
  L.xct = take(sizeof(half_t) * d * Tp);
  L.dyct = take(sizeof(half_t) * d * Tp);
  L.dhst = take(sizeof(half_t) * f * Tp);
  L.agt = take(sizeof(half_t) * f * Tp);
  L.rgpart = take(sizeof(float) * RG_SPLIT * E * r * (f > d ? f : d));
  L.total = off;
  return L;
}

hipError_t launch_backward(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, const half_t* dy, int T,
                           const int* expert_idx, const float* gate, const cmoe_grads& out, char* ws,
                           const cmoe_bw_layout& L, hipStream_t st) {
  const int E = dm.G * dm.K, G = dm.G, d = dm.d, f = dm.d_ff, r = dm.r, k = dm.k, M = L.M, Tpad = L.Tpad;
  auto I = [&](size_t o) { return (int*)(ws + o); };
  auto H = [&](size_t o) { return (half_t*)(ws + o); };
  auto F = [&](size_t o) { return (float*)(ws + o); };
  int *permc = I(L.permc), *offc = I(L.offc), *permm = I(L.permm), *invm = I(L.invm), *offe = I(L.offe);
  int* krc = I(L.krange_c);
  float* dl = out.d_logits ? out.d_logits : F(L.dl);
  const long mat = (long)f * d;
  // the bases: from the re-tiled copy when the caller keeps one (the canonical arrays may
  // then be absent), else the canonical arrays
  const bool pk = w.packed != nullptr;
  const cmoe_packed_layout PL = cmoe_packed(dm);
  const half_t* w1b = pk ? (const half_t*)((const char*)w.packed + PL.w1) : (const half_t*)w.w1_base;
  const half_t* w2b = pk ? (const half_t*)((const char*)w.packed + PL.w2) : (const half_t*)w.w2_base;
  hipError_t err;
#define BW_CHECK(call)                    \
  do {                                    \
    err = (call);                         \
    if (err != hipSuccess) return err;    \
  } while (0)
#define BW_GEMM(...) BW_CHECK(launch_gemm_plain(__VA_ARGS__, st))
  // a product over expert groups, at most 64 groups per launch (the kernel finds the group of
  // a tile by a linear walk over the offsets); rows are addressed absolutely, so a launch
  // over a slice of the offsets needs no other change
  auto rank_gemm = [&](const half_t* P, int L_, const half_t* X, int ldx, const int* gather, int x_div,
                       half_t* outp) -> hipError_t {
    for (int e0 = 0; e0 < E; e0 += 64) {
      hipError_t rc = launch_gemm_plain(P + (size_t)e0 * RP * L_, (long)RP * L_, L_, RP, X, ldx, gather, x_div, L_,
                                        offe + e0, E - e0 < 64 ? E - e0 : 64, M, nullptr, nullptr, outp, RP, false, st);
      if (rc != hipSuccess) return rc;
    }
    return hipSuccess;
  };

  // tokens sorted by cluster, pairs sorted by expert (both stable)
  if (T > 0)
    hipLaunchKernelGGL(bw_cluster_kernel, dim3((T + 255) / 256), dim3(256), 0, st, expert_idx, T, k, dm.K, I(L.cid));
  BW_CHECK(launch_permute_bins(G, I(L.cid), T, permc, I(L.invc), offc, I(L.blk_counts), st));
  if (E <= 64) {
    BW_CHECK(launch_permute_bins(E, expert_idx, M, permm, invm, offe, I(L.blk_counts), st));
  } else if (M > 0) {
    int *key = I(L.sort_tmp), *perm_a = key + M, *perm_b = key + 2 * (size_t)M, *scratch = key + 3 * (size_t)M;
    const dim3 gm((M + 255) / 256), blk(256);
    hipLaunchKernelGGL(bw_key_kernel, gm, blk, 0, st, expert_idx, (const int*)nullptr, M, dm.K, E, 0, key);
    BW_CHECK(launch_permute_bins(dm.K, key, M, perm_a, scratch, I(L.off_tmp), I(L.blk_counts), st));
    hipLaunchKernelGGL(bw_key_kernel, gm, blk, 0, st, expert_idx, (const int*)perm_a, M, dm.K, E, 1, key);
    BW_CHECK(launch_permute_bins(G, key, M, perm_b, scratch, I(L.off_tmp), I(L.blk_counts), st));
    hipLaunchKernelGGL(bw_compose_kernel, gm, blk, 0, st, expert_idx, (const int*)perm_a, (const int*)perm_b, M, E,
                       permm, invm, offe);
  } else {
    hipLaunchKernelGGL(bw_zero_kernel, dim3((E + 256) / 256), dim3(256), 0, st, offe, E + 1);
  }
  hipLaunchKernelGGL(bw_map_kernel, dim3((Tpad + 255) / 256), dim3(256), 0, st, offc, permc, (const float*)nullptr, G,
                     1, Tpad, krc, I(L.srow_c), I(L.ssrc_c), (float*)nullptr);
  hipLaunchKernelGGL(bw_rows_kernel, dim3((unsigned)(((size_t)G * f + 256) / 256)), dim3(256), 0, st, G, f,
                     I(L.offx_f), I(L.gidx_f));
  hipLaunchKernelGGL(bw_rows_kernel, dim3((unsigned)(((size_t)G * d + 256) / 256)), dim3(256), 0, st, G, d,
                     I(L.offx_d), I(L.gidx_d));
  // no token: the products below find empty groups and write zero gradients
  if (T > 0) {
    // operand panels: rank factors and transposed bases
    const int q = dm.q;
    hipLaunchKernelGGL(bw_panel_kernel, dim3((d + 255) / 256, E), dim3(256), 0, st, (const uint8_t*)w.v1_q,
                       (const half_t*)w.v1_s, d, q, r, offe, H(L.v1p));
    hipLaunchKernelGGL(bw_panel_kernel, dim3((f + 255) / 256, E), dim3(256), 0, st, (const uint8_t*)w.u1_q,
                       (const half_t*)w.u1_s, f, q, r, offe, H(L.u1p));
    hipLaunchKernelGGL(bw_panel_kernel, dim3((d + 255) / 256, E), dim3(256), 0, st, (const uint8_t*)w.u2_q,
                       (const half_t*)w.u2_s, d, q, r, offe, H(L.u2p));
    hipLaunchKernelGGL(bw_panel_kernel, dim3((f + 255) / 256, E), dim3(256), 0, st, (const uint8_t*)w.v2_q,
                       (const half_t*)w.v2_s, f, q, r, offe, H(L.v2p));
    // w1bt = B1^T ([d][d_ff] per cluster), w2bt = B2^T ([d_ff][d]), both in 32-column blocks
    hipLaunchKernelGGL(bw_transpose_kernel, dim3(f / 64, d / 64, G), dim3(256), 0, st, w1b, d, pk ? (long)f * 32 : 0L, d,
                       (const int*)nullptr, (const float*)nullptr, f, offc, (size_t)mat, 1, H(L.w1bt));
    hipLaunchKernelGGL(bw_transpose_kernel, dim3(d / 64, f / 64, G), dim3(256), 0, st, w2b, f, pk ? (long)d * 32 : 0L, f,
                       (const int*)nullptr, (const float*)nullptr, d, offc, (size_t)mat, 1, H(L.w2bt));
    BW_CHECK(hipGetLastError());

    // h = B1 x + U1 (V1 x): base product per token (token order), rank part per pair
    if (pk)   // packed W1: [d/32][d_ff][32] per cluster
      BW_CHECK(launch_gemm_plain(w1b, mat, 32, f, x, d, permc, 1, d, offc, G, T, nullptr, permc,
                                 H(L.hb), f, false, st, (long)f * 32, 0));
    else
      BW_GEMM(w1b, mat, d, f, x, d, permc, 1, d, offc, G, T, nullptr, permc, H(L.hb), f, false);
    BW_CHECK(rank_gemm(H(L.v1p), d, x, d, permm, k, H(L.t1)));
    rankexpand(r, H(L.t1), H(L.u1p), f, offe, nullptr, E, H(L.rh), st);
    // da = B2^T dy + V2^T (U2^T dy)
    BW_CHECK(launch_gemm_plain(H(L.w2bt), mat, 32, f, dy, d, permc, 1, d, offc, G, T, nullptr, permc, H(L.dab), f, false,
                               st, (long)f * 32, 0));
    BW_CHECK(rank_gemm(H(L.u2p), d, dy, d, permm, k, H(L.uy)));
    rankexpand(r, H(L.uy), H(L.v2p), f, offe, nullptr, E, H(L.rda), st);
    if (k <= 2)
      hipLaunchKernelGGL(bw_act_kernel<2>, dim3(T), dim3(256), 0, st, H(L.hb), H(L.dab), H(L.rh), H(L.rda), invm, gate, k,
                         f, H(L.a16), H(L.dh16), H(L.dhsum16), H(L.ag16), dl);
    else
      hipLaunchKernelGGL(bw_act_kernel<8>, dim3(T), dim3(256), 0, st, H(L.hb), H(L.dab), H(L.rh), H(L.rda), invm, gate, k,
                         f, H(L.a16), H(L.dh16), H(L.dhsum16), H(L.ag16), dl);
    // dx = B1^T (sum_j dh) + sum_j V1^T (U1^T dh) + gate path
    BW_CHECK(launch_gemm_plain(H(L.w1bt), mat, 32, d, H(L.dhsum16), f, permc, 1, f, offc, G, T, nullptr, permc, H(L.dxb), d,
                               false, st, (long)d * 32, 0));
    BW_CHECK(rank_gemm(H(L.u1p), f, H(L.dh16), f, nullptr, 1, H(L.qq)));
    rankexpand(r, H(L.qq), H(L.v1p), d, offe, permm, E, H(L.dxr), st);
    hipLaunchKernelGGL(bw_dx_kernel, dim3(T, (d / 4 + 255) / 256), dim3(256), 0, st, H(L.dxb), H(L.dxr), dl, expert_idx,
                       (const half_t*)w.router_expert, k, d, out.dx);
    // s = V2 a per pair
    BW_CHECK(rank_gemm(H(L.v2p), f, H(L.a16), f, nullptr, 1, H(L.ss)));
    // transposed, cluster-padded copies for the base gradients (contraction over tokens),
    // stored in 32-column blocks
    const int* ssrc_c = I(L.ssrc_c);
    transpose(x, d, d, ssrc_c, nullptr, Tpad, H(L.xct), st);
    transpose(dy, d, d, ssrc_c, nullptr, Tpad, H(L.dyct), st);
    transpose(H(L.dhsum16), f, f, ssrc_c, nullptr, Tpad, H(L.dhst), st);
    transpose(H(L.ag16), f, f, ssrc_c, nullptr, Tpad, H(L.agt), st);
    BW_CHECK(hipGetLastError());
  }
  static_assert(DR_SPLIT == RG_SPLIT, "the finish kernel adds RG_SPLIT runs");
  hipLaunchKernelGGL(bw_drouter_kernel, dim3(E, (d / 4 + 255) / 256, DR_SPLIT), dim3(256), 0, st, x, permm, offe, dl,
                     k, d, E, F(L.rgpart));
  hipLaunchKernelGGL(bw_rankgrad_finish_kernel, dim3((unsigned)(((size_t)E * d / 4 + 255) / 256)), dim3(256), 0, st,
                     (const float*)F(L.rgpart), (size_t)E * d, out.d_router_expert);
  // base gradients: contraction over the tokens of a cluster
  // (operands in the blocked layout [Tpad / 32][rows][32]: row stride 32, block stride rows * 32)
  BW_CHECK(launch_gemm_plain(H(L.xct), 0, 32, d, H(L.dhst), 32, I(L.gidx_f), 1, Tpad, I(L.offx_f), G, G * f, krc,
                             nullptr, out.dw1_base, d, true, st, (long)d * 32, (long)f * 32));
  BW_CHECK(launch_gemm_plain(H(L.agt), 0, 32, f, H(L.dyct), 32, I(L.gidx_d), 1, Tpad, I(L.offx_d), G, G * d, krc,
                             nullptr, out.dw2_base, f, true, st, (long)f * 32, (long)d * 32));
  // factor gradients: contraction over the pairs of an expert, streamed once
  float* part = F(L.rgpart);
  rankgrad(r, H(L.t1), H(L.dh16), f, offe, permm, k, 0, E, part, out.du1, st);
  rankgrad(r, H(L.qq), x, d, offe, permm, k, 1, E, part, out.dv1, st);
  // the gate of the pair goes into the rank-space rows of the two products of the second matrix
  if (M > 0) {
    hipLaunchKernelGGL(bw_scale_kernel, dim3((M * 4 + 255) / 256), dim3(256), 0, st, H(L.ss), permm, gate, M);
    hipLaunchKernelGGL(bw_scale_kernel, dim3((M * 4 + 255) / 256), dim3(256), 0, st, H(L.uy), permm, gate, M);
  }
  rankgrad(r, H(L.ss), dy, d, offe, permm, k, 1, E, part, out.du2, st);
  rankgrad(r, H(L.uy), H(L.a16), f, offe, permm, k, 0, E, part, out.dv2, st);
#undef BW_GEMM
#undef BW_CHECK
  return hipGetLastError();
}
