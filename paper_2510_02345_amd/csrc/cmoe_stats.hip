// By-products of one routing step: expert loads and their coefficient of variation (the
// load-balance metric of Sec. 4), the EMA activation centroids of the experts (Sec. 3.1,
// Eq. 5) and the per-cluster activity that drives offloading and prefetch (Sec. 3.4).
// All of it is a segmented reduction over the cluster-sorted rows the layer already has:
// the tokens of expert e lie inside the rows of its cluster.
#include "cmoe_internal.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int ST_SEG = 256;      // sorted rows per partial
constexpr int ST_COLS = 2048;    // columns per workgroup: 256 threads x 8

// slot -> (cluster, first row) with slots dealt cluster-major, ceil(n_c / ST_SEG) per cluster
__device__ __forceinline__ bool stats_slot(const int* offsets, int G, int slot, int& c, int& m0, int& m_end) {
  for (c = 0; c < G; ++c) {
    const int lo = offsets[c], hi = offsets[c + 1];
    const int tiles = (hi - lo + ST_SEG - 1) / ST_SEG;
    if (slot < tiles) {
      m0 = lo + slot * ST_SEG;
      m_end = min(hi, m0 + ST_SEG);
      return true;
    }
    slot -= tiles;
  }
  return false;
}

// part[(slot K + j)][d] = sum of x over the rows of the slot whose token selected expert
// c K + j, cnt[slot K + j] = their number.  grid (slots, K, ceil(d / 2048)).
__global__ __launch_bounds__(256) void stats_partial_kernel(const half_t* __restrict__ x,
                                                            const int* __restrict__ perm,
                                                            const int* __restrict__ offsets,
                                                            const int* __restrict__ expert_idx, int G, int K, int k,
                                                            int d, float* __restrict__ part, int* __restrict__ cnt) {
  __shared__ int list[ST_SEG];
  __shared__ int wcnt[4];
  int c, m0, m_end;
  if (!stats_slot(offsets, G, blockIdx.x, c, m0, m_end)) return;
  const int j = blockIdx.y, e = c * K + j;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the slot's rows that selected e, in row order
  const int p = m0 + tid;
  int tok = -1;
  bool hit = false;
  if (p < m_end) {
    tok = perm[p];
    for (int a = 0; a < k; ++a) hit |= expert_idx[(size_t)tok * k + a] == e;
  }
  const unsigned long long m = __ballot(hit);
  if (lane == 0) wcnt[wave] = __popcll(m);
  __syncthreads();
  int before = 0, n = 0;
  for (int w2 = 0; w2 < 4; ++w2) {
    if (w2 < wave) before += wcnt[w2];
    n += wcnt[w2];
  }
  if (hit) list[before + __popcll(m & ((1ull << lane) - 1ull))] = tok;
  __syncthreads();
  const int col = blockIdx.z * ST_COLS + tid * 8;
  const size_t slot_j = (size_t)blockIdx.x * K + j;
  if (blockIdx.z == 0 && tid == 0) cnt[slot_j] = n;
  if (col >= d) return;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int i0 = 0; i0 < n; i0 += 4) {   // four rows per batch of loads, added in row order
    half8 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      v[u] = (i0 + u < n) ? *(const half8*)(x + (size_t)list[i0 + u] * d + col) : half8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += (float)v[u][i];
  }
  float* dst = part + slot_j * d + col;
  *(float4v*)dst = float4v{acc[0], acc[1], acc[2], acc[3]};
  *(float4v*)(dst + 4) = float4v{acc[4], acc[5], acc[6], acc[7]};
}

// Eq. 5 for expert e = blockIdx.x: sums the partials of its cluster's slots in slot order,
// mu_e <- (1 - beta) mu_e + beta sum / n_e when n_e > 0; expert_load[e] = n_e.
__global__ __launch_bounds__(256) void stats_finish_kernel(const float* __restrict__ part,
                                                           const int* __restrict__ cnt,
                                                           const int* __restrict__ offsets, int K, int d, float beta,
                                                           float* __restrict__ mu, int* __restrict__ expert_load) {
  const int e = blockIdx.x, c = e / K, j = e % K;
  int slot0 = 0;
  for (int g = 0; g < c; ++g) slot0 += (offsets[g + 1] - offsets[g] + ST_SEG - 1) / ST_SEG;
  const int tiles = (offsets[c + 1] - offsets[c] + ST_SEG - 1) / ST_SEG;
  int n = 0;
  for (int s = 0; s < tiles; ++s) n += cnt[(size_t)(slot0 + s) * K + j];
  if (blockIdx.y == 0 && threadIdx.x == 0) expert_load[e] = n;
  const int col = blockIdx.y * ST_COLS + threadIdx.x * 8;
  if (col >= d || n == 0) return;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int s = 0; s < tiles; ++s) {
    const float* src = part + ((size_t)(slot0 + s) * K + j) * d + col;
    const float4v a = *(const float4v*)src, b = *(const float4v*)(src + 4);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc[i] += a[i];
      acc[i + 4] += b[i];
    }
  }
  float* m = mu + (size_t)e * d + col;
  const float inv = 1.f / (float)n;
#pragma unroll
  for (int i = 0; i < 8; ++i) m[i] = (1.f - beta) * m[i] + beta * (acc[i] * inv);
}

// One wavefront: cluster loads, activity EMA and idle counters (Sec. 3.4), and the
// coefficient of variation of the expert loads (Sec. 4), in FP64 with a fixed order.
__global__ __launch_bounds__(64) void stats_cluster_kernel(const int* __restrict__ offsets,
                                                          const int* __restrict__ expert_load, int G, int E, float lam,
                                                          float* __restrict__ cluster_act,
                                                          int* __restrict__ cluster_idle,
                                                          int* __restrict__ cluster_load, float* __restrict__ i_load) {
  const int lane = threadIdx.x;
  for (int g = lane; g < G; g += 64) {
    const int n = offsets[g + 1] - offsets[g];
    cluster_load[g] = n;
    cluster_act[g] = (1.f - lam) * cluster_act[g] + lam * (n > 0 ? 1.f : 0.f);
    cluster_idle[g] = n > 0 ? 0 : cluster_idle[g] + 1;
  }
  double sum = 0.0;
  for (int e = lane; e < E; e += 64) sum += (double)expert_load[e];
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
  const double mean = sum / (double)E;
  double var = 0.0;
  for (int e = lane; e < E; e += 64) {
    const double dv = (double)expert_load[e] - mean;
    var += dv * dv;
  }
  for (int off = 32; off > 0; off >>= 1) var += __shfl_xor(var, off, 64);
  if (lane == 0) i_load[0] = mean > 0.0 ? (float)(sqrt(var / (double)E) / mean) : 0.f;
}

}  // namespace

size_t stats_partial_slots(const cmoe_dims& dm, int T) { return (size_t)(T + ST_SEG - 1) / ST_SEG + dm.G; }

hipError_t launch_route_stats(const cmoe_dims& dm, const half_t* x, int T, const int* perm, const int* offsets,
                              const int* expert_idx, float beta, float lam, float* mu, float* cluster_act,
                              int* cluster_idle, int* expert_load, int* cluster_load, float* i_load, float* part,
                              int* cnt, hipStream_t st) {
  const int slots = (int)stats_partial_slots(dm, T), nch = (dm.d + ST_COLS - 1) / ST_COLS;
  if (T > 0)
    hipLaunchKernelGGL(stats_partial_kernel, dim3(slots, dm.K, nch), dim3(256), 0, st, x, perm, offsets, expert_idx,
                       dm.G, dm.K, dm.k, dm.d, part, cnt);
  hipLaunchKernelGGL(stats_finish_kernel, dim3(dm.G * dm.K, nch), dim3(256), 0, st, part, cnt, offsets, dm.K, dm.d,
                     beta, mu, expert_load);
  hipLaunchKernelGGL(stats_cluster_kernel, dim3(1), dim3(64), 0, st, offsets, expert_load, dm.G, dm.G * dm.K, lam,
                     cluster_act, cluster_idle, cluster_load, i_load);
  return hipGetLastError();
}
