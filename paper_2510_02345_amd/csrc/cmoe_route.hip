// Two-stage hierarchical router (Sec. 3.3, Eq. 9 and Eq. 10) and the stable
// token-to-cluster permutation (the single-device part of group-level dispatch).
#include <mutex>

#include "cmoe_internal.h"

namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

__device__ __forceinline__ float dot8(half8 a, half8 b, float acc) {
#pragma unroll
  for (int i = 0; i < 8; ++i) acc = fmaf((float)a[i], (float)b[i], acc);
  return acc;
}

// Ranking key of a logit: a NaN ranks below every number (as -inf), so that the selection
// rounds below always return distinct, valid slots whatever the input holds.
__device__ __forceinline__ float rank_key(float v) { return v == v ? v : -INFINITY; }

// One round of (largest key, lowest lane) over the first n lanes, skipping lanes already
// taken.  Returns the winning lane; marks it taken.
__device__ __forceinline__ int select_round(float key, bool& taken, int lane, int n) {
  float m = (lane < n && !taken) ? key : -INFINITY;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  const unsigned long long who = __ballot(lane < n && !taken && key == m);
  const int j = who ? __ffsll((long long)who) - 1 : 0;   // who is non-empty while fewer than n lanes are taken
  if (lane == j) taken = true;
  return j;
}

constexpr int ROUTE_WAVES = 4;

// One wavefront per token.  The token's row stays in registers for both stages: z_g over
// all G prototypes, then l_j over the K routing vectors of the winning cluster only, so
// the work per token is (G + K) dot products of length d (Sec. 3.3).
template <int MAXC>
__global__ __launch_bounds__(ROUTE_WAVES * 64) void route_kernel(
    const half_t* __restrict__ x, const half_t* __restrict__ rc, const half_t* __restrict__ re,
    const float* __restrict__ bias, int T, int d, int G, int K, int k, int* __restrict__ cluster_id,
    int* __restrict__ expert_idx, float* __restrict__ gate) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * ROUTE_WAVES + (threadIdx.x >> 6);
  if (t >= T) return;
  const int nchunk = d >> 3;
  half8 xv[MAXC];
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    int ch = lane + 64 * i;
    xv[i] = (ch < nchunk) ? *(const half8*)(x + (size_t)t * d + ch * 8) : half8{0, 0, 0, 0, 0, 0, 0, 0};
  }
  // stage 1: the softmax of Eq. 9 is monotone, so the most probable cluster is the
  // largest logit; strict '>' keeps the lowest index on ties
  float best = -INFINITY;
  int c = 0;
  for (int g = 0; g < G; ++g) {
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      int ch = lane + 64 * i;
      if (ch < nchunk) acc = dot8(xv[i], *(const half8*)(rc + (size_t)g * d + ch * 8), acc);
    }
    acc = wave_sum(acc);
    if (bias != nullptr) acc += bias[g];
    if (acc > best) {
      best = acc;
      c = g;
    }
  }
  // stage 2: logits of the K experts of cluster c; lane j keeps l_j
  float mine = -INFINITY;
  for (int j = 0; j < K; ++j) {
    float acc = 0.f;
    const half_t* v = re + (size_t)(c * K + j) * d;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      int ch = lane + 64 * i;
      if (ch < nchunk) acc = dot8(xv[i], *(const half8*)(v + ch * 8), acc);
    }
    acc = wave_sum(acc);
    if (lane == j) mine = acc;
  }
  // top-k by k rounds of (largest value, lowest lane) selection over the wavefront
  float sel_l[8];
  int sel_j[8];
  float lmax = 0.f;
  const float key = rank_key(mine);
  bool taken = false;
#pragma unroll
  for (int a = 0; a < 8; ++a) {
    sel_l[a] = 0.f;
    sel_j[a] = 0;
    if (a < k) {
      const int j = select_round(key, taken, lane, K);
      sel_l[a] = __shfl(mine, j, 64);
      sel_j[a] = j;
      if (a == 0) lmax = sel_l[a];
    }
  }
  if (lane == 0) {
    cluster_id[t] = c;
    float den = 0.f;
    float ex[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) {
      ex[a] = (a < k) ? expf(sel_l[a] - lmax) : 0.f;
      den += ex[a];
    }
#pragma unroll
    for (int a = 0; a < 8; ++a) {
      if (a < k) {
        expert_idx[(size_t)t * k + a] = c * K + sel_j[a];
        gate[(size_t)t * k + a] = ex[a] / den;
      }
    }
  }
}

// ---------------------------------------------------------------- routing variants
// Top-g clusters per token (Sec. 3.3, "Top-g_1 groups"), router temperature (Sec. 3.5) and
// optional scaling by the cluster probability of Eq. 9.  One wavefront per token; lane g
// keeps z_g, lane j keeps l_j.  Outputs are laid out per (token, selected cluster) pair
// a = 0..top_g-1, i.e. as top_g "virtual tokens" per token:
//   cluster_id [T][top_g], expert_idx [T][top_g][k], gate [T][top_g][k]
// gate = w_a * softmax(l_sel / tau), w_a = p_g (scaled) or p_g / sum of the selected p_g.
template <int MAXC>
__global__ __launch_bounds__(ROUTE_WAVES * 64) void route_multi_kernel(
    const half_t* __restrict__ x, const half_t* __restrict__ rc, const half_t* __restrict__ re,
    const float* __restrict__ bias, int T, int d, int G, int K, int k, int top_g, float inv_tau, int scale,
    int* __restrict__ cluster_id, int* __restrict__ expert_idx, float* __restrict__ gate) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * ROUTE_WAVES + (threadIdx.x >> 6);
  if (t >= T) return;
  const int nchunk = d >> 3;
  half8 xv[MAXC];
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    int ch = lane + 64 * i;
    xv[i] = (ch < nchunk) ? *(const half8*)(x + (size_t)t * d + ch * 8) : half8{0, 0, 0, 0, 0, 0, 0, 0};
  }
  auto dot = [&](const half_t* v) {
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      int ch = lane + 64 * i;
      if (ch < nchunk) acc = dot8(xv[i], *(const half8*)(v + ch * 8), acc);
    }
    return wave_sum(acc);
  };
  auto wave_max = [&](float m) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    return m;
  };
  // Eq. 9 with temperature: p_g = softmax(z / tau)
  float zmine = -INFINITY;
  for (int g = 0; g < G; ++g) {
    float z = dot(rc + (size_t)g * d);
    if (bias != nullptr) z += bias[g];
    if (lane == g) zmine = z;
  }
  const float zmax = wave_max(zmine);
  const float ez = (lane < G) ? expf((zmine - zmax) * inv_tau) : 0.f;
  const float pz = ez / wave_sum(ez);
  // the top_g clusters: rounds of (largest logit, lowest lane)
  int sel_c[8];
  float sel_p[8];
  float psum = 0.f;
  const float zkey = rank_key(zmine);
  bool ztaken = false;
#pragma unroll
  for (int a = 0; a < 8; ++a) {
    sel_c[a] = 0;
    sel_p[a] = 0.f;
    if (a < top_g) {
      const int g = select_round(zkey, ztaken, lane, G);
      sel_c[a] = g;
      sel_p[a] = __shfl(pz, g, 64);
      psum += sel_p[a];
    }
  }
#pragma unroll
  for (int a = 0; a < 8; ++a) {
    if (a >= top_g) continue;
    const int c = sel_c[a];
    const float wa = scale ? sel_p[a] : sel_p[a] / psum;
    float mine = -INFINITY;
    for (int j = 0; j < K; ++j) {
      const float l = dot(re + (size_t)(c * K + j) * d);
      if (lane == j) mine = l;
    }
    float sel_l[8];
    int sel_j[8];
    const float key = rank_key(mine);
    bool taken = false;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      sel_l[b] = 0.f;
      sel_j[b] = 0;
      if (b < k) {
        const int j = select_round(key, taken, lane, K);
        sel_l[b] = __shfl(mine, j, 64);
        sel_j[b] = j;
      }
    }
    if (lane == 0) {
      const size_t vt = (size_t)t * top_g + a;
      cluster_id[vt] = c;
      float den = 0.f, ex[8];
#pragma unroll
      for (int b = 0; b < 8; ++b) {
        ex[b] = (b < k) ? expf((sel_l[b] - sel_l[0]) * inv_tau) : 0.f;
        den += ex[b];
      }
#pragma unroll
      for (int b = 0; b < 8; ++b)
        if (b < k) {
          expert_idx[vt * k + b] = c * K + sel_j[b];
          gate[vt * k + b] = wa * (ex[b] / den);
        }
    }
  }
}

// y[t][:] = sum_a yrep[t top_g + a][:] (FP32, a ascending)
__global__ __launch_bounds__(256) void sum_groups_kernel(const half_t* __restrict__ yrep, int top_g, int d,
                                                         half_t* __restrict__ y) {
  const int t = blockIdx.y, col = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (col >= d) return;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int a = 0; a < top_g; ++a) {
    const half8 v = *(const half8*)(yrep + ((size_t)t * top_g + a) * d + col);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] += (float)v[i];
  }
  half8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (half_t)acc[i];
  *(half8*)(y + (size_t)t * d + col) = o;
}

// ---------------------------------------------------------------- permutation
// Pass 1: per-block histogram of cluster ids (LDS integer atomics: order-independent).
__global__ __launch_bounds__(PERMUTE_BLOCK) void permute_hist_kernel(const int* __restrict__ cluster_id, int T, int G,
                                                                     int* __restrict__ blk_counts) {
  __shared__ int hist[64];
  if (threadIdx.x < 64) hist[threadIdx.x] = 0;
  __syncthreads();
  int t = blockIdx.x * PERMUTE_BLOCK + threadIdx.x;
  if (t < T) atomicAdd(&hist[min(max(cluster_id[t], 0), G - 1)], 1);
  __syncthreads();
  if (threadIdx.x < G) blk_counts[(size_t)blockIdx.x * G + threadIdx.x] = hist[threadIdx.x];
}

// Pass 2: one workgroup.  offsets = exclusive scan of the cluster totals; each block's
// count is replaced by the first sorted row that block may write for that cluster.  The
// blocks are cut into SCAN_SEG segments, one wavefront per segment and one lane per cluster:
// segment totals first (independent loads), then the walk inside each segment.
constexpr int SCAN_SEG = 16;
__global__ __launch_bounds__(SCAN_SEG * 64) void permute_scan_kernel(int n_blocks, int G,
                                                                     int* __restrict__ blk_counts,
                                                                     int* __restrict__ offsets) {
  __shared__ int segsum[SCAN_SEG][64];
  __shared__ int total[64];
  const int g = threadIdx.x & 63, seg = threadIdx.x >> 6;
  const int per = (n_blocks + SCAN_SEG - 1) / SCAN_SEG;
  const int b0 = min(seg * per, n_blocks), b1 = min(b0 + per, n_blocks);
  int sum = 0;
  if (g < G)
    for (int b = b0; b < b1; ++b) sum += blk_counts[(size_t)b * G + g];
  segsum[seg][g] = sum;
  __syncthreads();
  if (seg == 0) {
    int run = 0;
    for (int s2 = 0; s2 < SCAN_SEG; ++s2) {   // exclusive over the segments of cluster g
      const int v = segsum[s2][g];
      segsum[s2][g] = run;
      run += v;
    }
    total[g] = g < G ? run : 0;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int c = 0; c < G; ++c) {
      offsets[c] = run;
      const int v = total[c];
      total[c] = run;
      run += v;
    }
    offsets[G] = run;
  }
  __syncthreads();
  if (g < G) {
    int run = total[g] + segsum[seg][g];
    for (int b = b0; b < b1; ++b) {
      const int v = blk_counts[(size_t)b * G + g];
      blk_counts[(size_t)b * G + g] = run;
      run += v;
    }
  }
}

// Pass 3: stable ranks.  Inside a block, a token's rank among equal clusters is the count
// in earlier wavefronts plus the number of lower lanes with the same cluster (ballot).
__global__ __launch_bounds__(PERMUTE_BLOCK) void permute_rank_kernel(const int* __restrict__ cluster_id, int T, int G,
                                                                     const int* __restrict__ blk_base,
                                                                     int* __restrict__ perm,
                                                                     int* __restrict__ inv_perm) {
  constexpr int NW = PERMUTE_BLOCK / 64;
  __shared__ int wcount[NW][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x * PERMUTE_BLOCK + threadIdx.x;
  const int c = (t < T) ? min(max(cluster_id[t], 0), G - 1) : -1;
  int my_rank = 0;
  for (int g = 0; g < G; ++g) {
    unsigned long long m = __ballot(c == g);
    if (lane == 0) wcount[wave][g] = __popcll(m);
    if (c == g) my_rank = __popcll(m & ((1ull << lane) - 1ull));
  }
  __syncthreads();
  if (t < T) {
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wcount[w][c];
    int pos = blk_base[(size_t)blockIdx.x * G + c] + before + my_rank;
    perm[pos] = t;
    inv_perm[t] = pos;
  }
}

// Few tokens: one workgroup (eight wavefronts) per token, the logits of a stage spread over
// the wavefronts so that their dot products run side by side instead of one after another.
constexpr int RS_WAVES = 8;
template <int MAXC>
__global__ __launch_bounds__(RS_WAVES * 64) void route_small_kernel(
    const half_t* __restrict__ x, const half_t* __restrict__ rc, const half_t* __restrict__ re,
    const float* __restrict__ bias, int T, int d, int G, int K, int k, int* __restrict__ cluster_id,
    int* __restrict__ expert_idx, float* __restrict__ gate) {
  __shared__ float zs[64];
  __shared__ float ls[64];
  __shared__ int cs;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = blockIdx.x;
  const int nchunk = d >> 3;
  half8 xv[MAXC];
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    int ch = lane + 64 * i;
    xv[i] = (ch < nchunk) ? *(const half8*)(x + (size_t)t * d + ch * 8) : half8{0, 0, 0, 0, 0, 0, 0, 0};
  }
  auto dot = [&](const half_t* v) {
    float acc = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      int ch = lane + 64 * i;
      if (ch < nchunk) acc = dot8(xv[i], *(const half8*)(v + ch * 8), acc);
    }
    return wave_sum(acc);
  };
  for (int g = wave; g < G; g += RS_WAVES) {
    float z = dot(rc + (size_t)g * d);
    if (bias != nullptr) z += bias[g];
    if (lane == 0) zs[g] = z;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float best = -INFINITY;
    int c = 0;
    for (int g = 0; g < G; ++g)
      if (zs[g] > best) {
        best = zs[g];
        c = g;
      }
    cs = c;
  }
  __syncthreads();
  const int c = cs;
  for (int j = wave; j < K; j += RS_WAVES) {
    float l = dot(re + (size_t)(c * K + j) * d);
    if (lane == 0) ls[j] = l;
  }
  __syncthreads();
  if (wave != 0) return;
  const float mine = (lane < K) ? ls[lane] : -INFINITY;
  float sel_l[8];
  int sel_j[8];
  float lmax = 0.f;
  const float key = rank_key(mine);
  bool taken = false;
#pragma unroll
  for (int a = 0; a < 8; ++a) {
    sel_l[a] = 0.f;
    sel_j[a] = 0;
    if (a < k) {
      const int j = select_round(key, taken, lane, K);
      sel_l[a] = __shfl(mine, j, 64);
      sel_j[a] = j;
      if (a == 0) lmax = sel_l[a];
    }
  }
  if (lane == 0) {
    cluster_id[t] = c;
    float den = 0.f;
    float ex[8];
#pragma unroll
    for (int a = 0; a < 8; ++a) {
      ex[a] = (a < k) ? expf(sel_l[a] - lmax) : 0.f;
      den += ex[a];
    }
#pragma unroll
    for (int a = 0; a < 8; ++a) {
      if (a < k) {
        expert_idx[(size_t)t * k + a] = c * K + sel_j[a];
        gate[(size_t)t * k + a] = ex[a] / den;
      }
    }
  }
}

// T <= 1024: histogram, scan and stable ranks in one workgroup.
__global__ __launch_bounds__(PERMUTE_BLOCK) void permute_small_kernel(const int* __restrict__ cluster_id, int T, int G,
                                                                      int* __restrict__ perm,
                                                                      int* __restrict__ inv_perm,
                                                                      int* __restrict__ offsets) {
  constexpr int NW = PERMUTE_BLOCK / 64;
  __shared__ int wcount[NW][64];
  __shared__ int base[64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int t = threadIdx.x;
  const int c = (t < T) ? min(max(cluster_id[t], 0), G - 1) : -1;
  int my_rank = 0;
  for (int g = 0; g < G; ++g) {
    unsigned long long m = __ballot(c == g);
    if (lane == 0) wcount[wave][g] = __popcll(m);
    if (c == g) my_rank = __popcll(m & ((1ull << lane) - 1ull));
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int g = 0; g < G; ++g) {
      offsets[g] = run;
      base[g] = run;
      for (int w = 0; w < NW; ++w) run += wcount[w][g];
    }
    offsets[G] = run;
  }
  __syncthreads();
  if (t < T) {
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wcount[w][c];
    int pos = base[c] + before + my_rank;
    perm[pos] = t;
    inv_perm[t] = pos;
  }
}

__global__ void zero_offsets_kernel(int G, int* offsets) {
  if ((int)threadIdx.x <= G) offsets[threadIdx.x] = 0;
}

}  // namespace

namespace {
// One workgroup per cluster: a stable counting sort of the cluster's rows by the key
// (first selected expert, second selected expert) taken inside the cluster, or by the
// first expert alone when K * K keys do not fit the 64 bins.
//   rowmap[i] = cluster-sorted row of refined row i,  perm2[i] = its token.
constexpr int PS_THREADS = 1024;
constexpr int PS_KEEP = 8;   // rows per thread whose token and key stay in registers
__global__ __launch_bounds__(PS_THREADS) void pair_sort_kernel(const int* __restrict__ perm,
                                                              const int* __restrict__ offsets,
                                                              const int* __restrict__ expert_idx, int K, int k,
                                                              int two_keys, int* __restrict__ rowmap,
                                                              int* __restrict__ perm2) {
  constexpr int NW = PS_THREADS / 64;
  __shared__ int binbase[64];
  __shared__ int wcount[NW][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.x;
  const int lo = offsets[c], n = offsets[c + 1] - lo;
  if (n <= 0) return;
  auto key_of_tok = [&](int tok) {
    const int* e = expert_idx + (size_t)tok * k;
    // expert slots outside the cluster (inconsistent caller input) are clamped into it
    const int j0 = min(max(e[0] - c * K, 0), K - 1);
    return two_keys ? j0 * K + min(max(e[1] - c * K, 0), K - 1) : j0;
  };
  // The first PS_KEEP rows of a thread (row tid + j * PS_THREADS) are read once, all loads in
  // flight together, and kept in registers for both passes; clusters with more rows take
  // the rest from memory in each pass.
  int tokr[PS_KEEP], keyr[PS_KEEP];
#pragma unroll
  for (int j = 0; j < PS_KEEP; ++j) {
    const int i = tid + j * PS_THREADS;
    tokr[j] = i < n ? perm[lo + i] : 0;
  }
#pragma unroll
  for (int j = 0; j < PS_KEEP; ++j) keyr[j] = tid + j * PS_THREADS < n ? key_of_tok(tokr[j]) : 0;
  if (tid < 64) binbase[tid] = 0;
  __syncthreads();
#pragma unroll
  for (int j = 0; j < PS_KEEP; ++j)
    if (tid + j * PS_THREADS < n) atomicAdd(&binbase[keyr[j]], 1);
  for (int i = tid + PS_KEEP * PS_THREADS; i < n; i += PS_THREADS) atomicAdd(&binbase[key_of_tok(perm[lo + i])], 1);
  __syncthreads();
  if (wave == 0) {   // exclusive scan of the 64 bin counts
    const int cnt = binbase[lane];
    int incl = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, 64);
      if (lane >= off) incl += v;
    }
    binbase[lane] = incl - cnt;
  }
  __syncthreads();
  // one chunk of PS_THREADS rows; chunks in order keep the sort stable
  auto chunk = [&](int i, bool in, int key, int tok) {
    // lanes of this wavefront holding the same key
    unsigned long long same = __ballot(in);
#pragma unroll
    for (int b = 0; b < 6; ++b) {
      const unsigned long long m = __ballot((key >> b) & 1);
      same &= ((key >> b) & 1) ? m : ~m;
    }
    wcount[wave][lane] = 0;
    __syncthreads();
    const int below = __popcll(same & ((1ull << lane) - 1ull));
    if (in && below == 0) wcount[wave][key] = __popcll(same);
    __syncthreads();
    if (in) {
      int before = 0;
      for (int w = 0; w < wave; ++w) before += wcount[w][key];
      const int pos = lo + binbase[key] + before + below;
      rowmap[pos] = lo + i;
      perm2[pos] = tok;
    }
    __syncthreads();
    if (tid < 64) {
      int add = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) add += wcount[w][tid];
      binbase[tid] += add;
    }
    __syncthreads();
  };
#pragma unroll
  for (int j = 0; j < PS_KEEP; ++j) {
    if (j * PS_THREADS >= n) break;   // uniform over the workgroup
    const int i = tid + j * PS_THREADS;
    chunk(i, i < n, keyr[j], tokr[j]);
  }
  for (int i0 = PS_KEEP * PS_THREADS; i0 < n; i0 += PS_THREADS) {
    const int i = i0 + tid;
    const bool in = i < n;
    const int tok = in ? perm[lo + i] : 0;
    chunk(i, in, in ? key_of_tok(tok) : 0, tok);
  }
}
}  // namespace

// Refines the cluster-sorted order: inside every cluster, rows are ordered by (first
// selected expert, second selected expert, original order).  Cluster boundaries (offsets)
// do not move.  Rows of a 16-token block then mostly share their experts, so the fused
// up-projection skips most rank chunks.
hipError_t launch_pair_sort(const cmoe_dims& dm, const int* perm, const int* offsets, const int* expert_idx, int T,
                            int* rowmap, int* perm2, hipStream_t st) {
  (void)T;
  const int two = (dm.k >= 2 && dm.K * dm.K <= 64) ? 1 : 0;
  hipLaunchKernelGGL(pair_sort_kernel, dim3(dm.G), dim3(PS_THREADS), 0, st, perm, offsets, expert_idx, dm.K, dm.k, two,
                     rowmap, perm2);
  return hipGetLastError();
}

hipError_t launch_route(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int* cluster_id,
                        int* expert_idx, float* gate, hipStream_t st) {
  dim3 grid((T + ROUTE_WAVES - 1) / ROUTE_WAVES), block(ROUTE_WAVES * 64);
  const half_t* rc = (const half_t*)w.router_cluster;
  const half_t* re = (const half_t*)w.router_expert;
  int chunks_per_lane = (dm.d / 8 + 63) / 64;
  if (T > SKINNY_T && dm.G + dm.G * dm.K <= 128)
    return launch_route_mfma(dm, w, x, T, cluster_id, expert_idx, gate, st);
  if (T <= SKINNY_T) {
    dim3 g1(T), b1(RS_WAVES * 64);
    if (chunks_per_lane <= 2)
      hipLaunchKernelGGL(route_small_kernel<2>, g1, b1, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k,
                         cluster_id, expert_idx, gate);
    else if (chunks_per_lane <= 4)
      hipLaunchKernelGGL(route_small_kernel<4>, g1, b1, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k,
                         cluster_id, expert_idx, gate);
    else if (chunks_per_lane <= 8)
      hipLaunchKernelGGL(route_small_kernel<8>, g1, b1, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k,
                         cluster_id, expert_idx, gate);
    else
      hipLaunchKernelGGL(route_small_kernel<16>, g1, b1, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K,
                         dm.k, cluster_id, expert_idx, gate);
    return hipGetLastError();
  }
  if (chunks_per_lane <= 2)
    hipLaunchKernelGGL(route_kernel<2>, grid, block, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k,
                       cluster_id, expert_idx, gate);
  else if (chunks_per_lane <= 4)
    hipLaunchKernelGGL(route_kernel<4>, grid, block, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k,
                       cluster_id, expert_idx, gate);
  else if (chunks_per_lane <= 8)
    hipLaunchKernelGGL(route_kernel<8>, grid, block, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k,
                       cluster_id, expert_idx, gate);
  else
    hipLaunchKernelGGL(route_kernel<16>, grid, block, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k,
                       cluster_id, expert_idx, gate);
  return hipGetLastError();
}

hipError_t launch_permute(const cmoe_dims& dm, const int* cluster_id, int T, int* perm, int* inv_perm, int* offsets,
                          int* blk_counts, hipStream_t st) {
  return launch_permute_bins(dm.G, cluster_id, T, perm, inv_perm, offsets, blk_counts, st);
}

hipError_t launch_permute_bins(int bins, const int* cluster_id, int T, int* perm, int* inv_perm, int* offsets,
                               int* blk_counts, hipStream_t st) {
  struct { int G; } dm{bins};
  if (T == 0) {
    hipLaunchKernelGGL(zero_offsets_kernel, dim3(1), dim3(128), 0, st, dm.G, offsets);
    return hipGetLastError();
  }
  if (T <= PERMUTE_BLOCK) {
    hipLaunchKernelGGL(permute_small_kernel, dim3(1), dim3(PERMUTE_BLOCK), 0, st, cluster_id, T, dm.G, perm,
                       inv_perm, offsets);
    return hipGetLastError();
  }
  int n_blocks = (T + PERMUTE_BLOCK - 1) / PERMUTE_BLOCK;
  hipLaunchKernelGGL(permute_hist_kernel, dim3(n_blocks), dim3(PERMUTE_BLOCK), 0, st, cluster_id, T, dm.G,
                     blk_counts);
  hipLaunchKernelGGL(permute_scan_kernel, dim3(1), dim3(SCAN_SEG * 64), 0, st, n_blocks, dm.G, blk_counts, offsets);
  hipLaunchKernelGGL(permute_rank_kernel, dim3(n_blocks), dim3(PERMUTE_BLOCK), 0, st, cluster_id, T, dm.G,
                     blk_counts, perm, inv_perm);
  return hipGetLastError();
}

// ---------------------------------------------------------------- permutation without a workspace argument
// The per-block histogram of the three-pass permutation lives in a file-scope device array
// instead of the caller's workspace, for callers that cannot allocate device memory.  Every
// GPU holds its own copy of the array at its own address; the host resolves that address
// once per device and passes it to the kernels like any other buffer.
static const int kStaticBlocks = CMOE_PERMUTE_STATIC_MAX_TOKENS / PERMUTE_BLOCK;
static __device__ __align__(256) int scratch[(size_t)kStaticBlocks * 64];
static const int kMaxDevices = 64;
static int* g_scratch_ptr[kMaxDevices];
static std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (resolved on the first call per device).
static hipError_t scratch_address(int** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    int* p = nullptr;
    e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

hipError_t launch_permute_static(const cmoe_dims& dm, const int* cluster_id, int T, int* perm, int* inv_perm,
                                 int* offsets, hipStream_t st) {
  int* blk_counts = nullptr;
  // up to PERMUTE_BLOCK tokens run in one workgroup and need no histogram buffer
  if (T > PERMUTE_BLOCK) {
    hipError_t e = scratch_address(&blk_counts);
    if (e != hipSuccess) return e;
  }
  // every entry the later passes read is written by the first pass of the same call: nothing
  // has to start at zero, whatever an earlier call left behind
  return launch_permute_bins(dm.G, cluster_id, T, perm, inv_perm, offsets, blk_counts, st);
}

hipError_t launch_route_multi(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int top_g,
                              float temperature, int scale, int* cluster_id, int* expert_idx, float* gate,
                              hipStream_t st) {
  // many tokens and all router rows in one 128-row tile: matrix-core product, decision in
  // its epilogue (as for the single-cluster router)
  if (T > SKINNY_T && dm.G + dm.G * dm.K <= 128)
    return launch_route_multi_mfma(dm, w, x, T, top_g, temperature, scale, cluster_id, expert_idx, gate, st);
  dim3 grid((T + ROUTE_WAVES - 1) / ROUTE_WAVES), block(ROUTE_WAVES * 64);
  const half_t* rc = (const half_t*)w.router_cluster;
  const half_t* re = (const half_t*)w.router_expert;
  const int chunks_per_lane = (dm.d / 8 + 63) / 64;
  const float inv_tau = 1.f / temperature;
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, grid, block, 0, st, x, rc, re, w.cluster_bias, T, dm.d, dm.G, dm.K, dm.k, top_g, inv_tau,
                       scale, cluster_id, expert_idx, gate);
  };
  if (chunks_per_lane <= 2) go(route_multi_kernel<2>);
  else if (chunks_per_lane <= 4) go(route_multi_kernel<4>);
  else if (chunks_per_lane <= 8) go(route_multi_kernel<8>);
  else go(route_multi_kernel<16>);
  return hipGetLastError();
}

hipError_t launch_sum_groups(const half_t* yrep, int T, int top_g, int d, half_t* y, hipStream_t st) {
  hipLaunchKernelGGL(sum_groups_kernel, dim3((d / 8 + 255) / 256, T), dim3(256), 0, st, yrep, top_g, d, y);
  return hipGetLastError();
}
