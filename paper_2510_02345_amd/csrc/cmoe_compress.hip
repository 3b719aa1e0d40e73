// Construction of the compressed form from dense expert matrices (Sec. 3.2, 3.4):
//   base(c)   = mean of the cluster's K expert matrices                       (Eq. 6)
//   Delta_e   = W_e - base(c), factorised as U_e V_e of rank r                (Eq. 7)
//   U_e, V_e  -> INT4 codes with one FP16 scale per q codes                   (Sec. 3.4)
//   optional gate: an expert whose residual has cosine similarity to the base below a
//   threshold keeps no residual                                              (Sec. 3.4)
// The rank-r factors are the best ones inside the subspace found by a randomised subspace
// iteration (sketch of l >= r rows, Rayleigh-Ritz on the sketch), which for the decaying
// residual spectra of clustered experts is the truncated SVD of Sec. 3.2 to within a
// fraction of a percent of its Frobenius error.  The heavy steps are products of the
// residual (or its transpose) with l sketch rows: weight streams, run by the same kernel
// as the layer's small-T path on a materialised FP16 copy of Delta_e and Delta_e^T.
#include "cmoe_internal.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));

constexpr int CP_LMAX = 48;   // widest sketch

// ---------------------------------------------------------------- base, residuals, their transposes, norms
// One 64 x 64 tile of cluster c: the base tile (Eq. 6: FP32 sum of the K experts in index
// order, divided by K, rounded to FP16), then for each expert e of the cluster
// D = f16(W_e - base), DT = D^T, and the tile's share of sum D^2, sum D base, sum base^2,
// sum W_e^2 (FP32, fixed order), one partial per wavefront -> part[e][tile][wave][4].  The
// tiles of the first CR_KEEP experts stay in registers between the two passes; those of
// further experts are read a second time (from cache).  The transposing LDS tile is double
// buffered: one barrier per expert.
constexpr int CR_KEEP = 8;
__global__ __launch_bounds__(256) void cmp_residual_kernel(const half_t* __restrict__ W, int K, int out_d, int in_d,
                                                           half_t* __restrict__ base, half_t* __restrict__ D,
                                                           half_t* __restrict__ DT, float* __restrict__ part) {
  __shared__ half_t tile[2][64][72];
  const int c = blockIdx.z;
  const int o0 = blockIdx.y * 64, i0 = blockIdx.x * 64;
  const int tid = threadIdx.x;
  const size_t me = (size_t)out_d * in_d;
  const size_t tix = (size_t)blockIdx.y * gridDim.x + blockIdx.x, nt = (size_t)gridDim.x * gridDim.y;
  const int row0 = tid >> 3, ch = tid & 7;   // rows row0 and row0 + 32, 8 columns per thread
  size_t off[2];
  float bsum[2][8];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    off[u] = (size_t)(o0 + row0 + 32 * u) * in_d + i0 + ch * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) bsum[u][i] = 0.f;
  }
  half8 keep[CR_KEEP][2];
#pragma unroll
  for (int j = 0; j < CR_KEEP; ++j)
#pragma unroll
    for (int u = 0; u < 2; ++u)
      keep[j][u] = j < K ? *(const half8*)(W + ((size_t)c * K + j) * me + off[u]) : half8{0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int j = 0; j < CR_KEEP; ++j)
    if (j < K)
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int i = 0; i < 8; ++i) bsum[u][i] += (float)keep[j][u][i];
  for (int j = CR_KEEP; j < K; ++j)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const half8 w8 = *(const half8*)(W + ((size_t)c * K + j) * me + off[u]);
#pragma unroll
      for (int i = 0; i < 8; ++i) bsum[u][i] += (float)w8[i];
    }
  const float kf = (float)K;
  half8 b8[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
#pragma unroll
    for (int i = 0; i < 8; ++i) b8[u][i] = (half_t)(bsum[u][i] / kf);
    *(half8*)(base + (size_t)c * me + off[u]) = b8[u];
  }
  auto one = [&](int j, const half8 (&w)[2]) {
    const int e = c * K + j, buf = j & 1;
    float s_dd = 0.f, s_db = 0.f, s_bb = 0.f, s_ww = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      half8 d8;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float wv = (float)w[u][i], b = (float)b8[u][i];
        d8[i] = (half_t)(wv - b);
        const float dv = (float)d8[i];
        s_dd = fmaf(dv, dv, s_dd);
        s_db = fmaf(dv, b, s_db);
        s_bb = fmaf(b, b, s_bb);
        s_ww = fmaf(wv, wv, s_ww);
      }
      *(half8*)(D + (size_t)e * me + off[u]) = d8;
      *(half8*)(&tile[buf][row0 + 32 * u][ch * 8]) = d8;
    }
    // this barrier also separates the reads of tile[buf] two experts ago from these writes
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int irow = row0 + 32 * u;   // row of the transposed tile
      half8 t8;
#pragma unroll
      for (int i = 0; i < 8; ++i) t8[i] = tile[buf][ch * 8 + i][irow];
      *(half8*)(DT + (size_t)e * me + (size_t)(i0 + irow) * out_d + o0 + ch * 8) = t8;
    }
    // wavefront sums in a fixed order (lanes by halving); the four wavefronts' partials are
    // added, in order, by cmp_stats_kernel
    float v[4] = {s_dd, s_db, s_bb, s_ww};
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int o2 = 32; o2 > 0; o2 >>= 1) v[a] += __shfl_xor(v[a], o2, 64);
    if ((tid & 63) < 4) {
      const int a = tid & 3;
      part[(((size_t)e * nt + tix) * 4 + (tid >> 6)) * 4 + a] = a == 0 ? v[0] : a == 1 ? v[1] : a == 2 ? v[2] : v[3];
    }
  };
#pragma unroll
  for (int j = 0; j < CR_KEEP; ++j)
    if (j < K) one(j, keep[j]);
  for (int j = CR_KEEP; j < K; ++j) {
    half8 w[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) w[u] = *(const half8*)(W + ((size_t)c * K + j) * me + off[u]);
    one(j, w);
  }
}

// stats[e][a] = sum over the n_tiles (tile, wavefront) partials part[e][.][a] (FP64, fixed
// order), a = dd, db, bb, ww.
__global__ __launch_bounds__(256) void cmp_stats_kernel(const float* __restrict__ part, int n_tiles,
                                                        double* __restrict__ stats) {
  __shared__ double red[256];
  const int e = blockIdx.x, a = threadIdx.x & 3, lane4 = threadIdx.x >> 2;   // 64 strided readers per quantity
  const float* src = part + (size_t)e * n_tiles * 4 + a;
  double s = 0.0;
  int t = lane4;
  for (; t + 7 * 64 < n_tiles; t += 8 * 64) {   // eight loads in flight, added in index order
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[(size_t)(t + 64 * u) * 4];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += (double)v[u];
  }
  for (; t < n_tiles; t += 64) s += (double)src[(size_t)t * 4];
  red[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x < 4) {
    double tot = 0.0;
    for (int i = 0; i < 64; ++i) tot += red[i * 4 + threadIdx.x];
    stats[(size_t)e * 4 + threadIdx.x] = tot;
  }
}

// ---------------------------------------------------------------- sketch bookkeeping
__global__ void cmp_offsets_kernel(int E, int l, int* __restrict__ offsets) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i <= E) offsets[i] = i * l;
}
// X[e l + a][:] = omega[a][:] for every expert
__global__ __launch_bounds__(256) void cmp_tile_rows_kernel(const half_t* __restrict__ omega, int l, int n,
                                                            half_t* __restrict__ X) {
  const int row = blockIdx.y, col = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (col >= n) return;
  *(half8*)(X + (size_t)row * n + col) = *(const half8*)(omega + (size_t)(row % l) * n + col);
}

// ---------------------------------------------------------------- Gram matrix of the l sketch rows
// gpart[e][chunk][a][b] = sum over the chunk's 512 columns of X[e l + a][n] X[e l + b][n].
__global__ __launch_bounds__(256) void cmp_gram_kernel(const half_t* __restrict__ X, int l, int n,
                                                       float* __restrict__ gpart) {
  __shared__ half_t xs[CP_LMAX][512 + 8];
  const int e = blockIdx.y, n0 = blockIdx.x * 512, tid = threadIdx.x;
  const int width = min(512, n - n0);
  for (int idx = tid; idx < l * 64; idx += 256) {
    const int a = idx / 64, ch = idx % 64;
    half8 v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (ch * 8 < width) v = *(const half8*)(X + ((size_t)e * l + a) * n + n0 + ch * 8);
    *(half8*)(&xs[a][ch * 8]) = v;
  }
  __syncthreads();
  float* dst = gpart + ((size_t)e * gridDim.x + blockIdx.x) * l * l;
  for (int pr = tid; pr < l * l; pr += 256) {
    const int a = pr / l, b = pr % l;
    if (b > a) continue;   // symmetric: the lower triangle is computed, the upper mirrored
    float s = 0.f;
    for (int i = 0; i < 512; i += 8) {
      const half8 va = *(const half8*)(&xs[a][i]), vb = *(const half8*)(&xs[b][i]);
#pragma unroll
      for (int u = 0; u < 8; ++u) s = fmaf((float)va[u], (float)vb[u], s);
    }
    dst[a * l + b] = s;
    dst[b * l + a] = s;
  }
}

// ---------------------------------------------------------------- small dense steps, one workgroup per expert
// Sums the Gram partials (FP64).  MODE 0: coef = inverse of the Cholesky factor of
// (Gram + shift I), so that coef X has orthonormal rows.  MODE 1: Jacobi eigenvectors of
// the Gram matrix; coef rows = the r eigenvectors of largest eigenvalue (transposed), and
// lam[e] = the sum of those eigenvalues.  The Jacobi sweeps use the round-robin ordering:
// a sweep is l - 1 rounds of l / 2 rotations on disjoint index pairs, which commute, so a
// round applies all of them at once, A <- J^T A J and V <- V J, every element by one thread.
constexpr int CS_THREADS = 256;
constexpr int CS_PER = (CP_LMAX * CP_LMAX + CS_THREADS - 1) / CS_THREADS;   // elements of an l x l matrix per thread
template <int MODE>
__global__ __launch_bounds__(CS_THREADS) void cmp_small_kernel(const float* __restrict__ gpart, int n_chunks, int l,
                                                               int r, float* __restrict__ coef,
                                                               double* __restrict__ lam) {
  __shared__ double A[CP_LMAX][CP_LMAX + 1];
  __shared__ double V[CP_LMAX][CP_LMAX + 1];
  __shared__ double ev[CP_LMAX];
  __shared__ int order[CP_LMAX];
  const int e = blockIdx.x, t = threadIdx.x;
  for (int idx = t; idx < l * l; idx += CS_THREADS) {
    const float* src = gpart + (size_t)e * n_chunks * l * l + idx;
    double s = 0.0;
    int ch = 0;
    for (; ch + 4 <= n_chunks; ch += 4) {   // four loads in flight, summed in chunk order
      const float v0 = src[(size_t)ch * l * l], v1 = src[(size_t)(ch + 1) * l * l];
      const float v2 = src[(size_t)(ch + 2) * l * l], v3 = src[(size_t)(ch + 3) * l * l];
      s += (double)v0;
      s += (double)v1;
      s += (double)v2;
      s += (double)v3;
    }
    for (; ch < n_chunks; ++ch) s += (double)src[(size_t)ch * l * l];
    A[idx / l][idx % l] = s;
  }
  __syncthreads();
  float* cf = coef + (size_t)e * CP_LMAX * CP_LMAX;
  if (MODE == 0) {
    // The sketch may be rank deficient (a residual of rank below l).  A pivot below tau,
    // which is far above the rounding noise of the FP16 rows and their FP32 Gram sums, marks
    // a row the earlier rows already span: it gets a huge pivot, so that its output row is
    // (numerically) zero instead of amplified noise and the rows after it do not see it.
    __shared__ double tau_s;
    if (t == 0) {
      double tr = 0.0;
      for (int i = 0; i < l; ++i) tr += A[i][i];
      tau_s = 1e-5 * tr / l + 1e-290;
    }
    __syncthreads();
    // Cholesky A = L L^T, column by column; the trailing update spread over the workgroup
    for (int j = 0; j < l; ++j) {
      if (t == 0) A[j][j] = A[j][j] > tau_s ? sqrt(A[j][j]) : 1e150;
      __syncthreads();
      if (t > j && t < l) A[t][j] /= A[j][j];
      __syncthreads();
      for (int idx = t; idx < l * l; idx += CS_THREADS) {
        const int i = idx / l, k2 = idx % l;
        if (i > j && k2 > j && k2 <= i) A[i][k2] -= A[i][j] * A[k2][j];
      }
      __syncthreads();
    }
    // V = L^-1 by forward substitution, thread c owns column c
    if (t < l) {
      for (int i = 0; i < l; ++i) {
        double s = (i == t) ? 1.0 : 0.0;
        for (int k2 = t; k2 < i; ++k2) s -= A[i][k2] * V[k2][t];
        V[i][t] = (i < t) ? 0.0 : s / A[i][i];
      }
    }
    __syncthreads();
    for (int idx = t; idx < l * CP_LMAX; idx += CS_THREADS) {
      const int a = idx / CP_LMAX, b = idx % CP_LMAX;
      cf[idx] = b < l ? (float)V[a][b] : 0.f;
    }
  } else {
    // per index k of the current round: its partner and the coefficients of
    // new column k = cc[k] * column k + ss[k] * column partner[k]
    __shared__ int partner[CP_LMAX];
    __shared__ double cc[CP_LMAX], ss[CP_LMAX];
    __shared__ double red[2][CS_THREADS / 64];
    for (int idx = t; idx < l * l; idx += CS_THREADS) V[idx / l][idx % l] = (idx / l == idx % l) ? 1.0 : 0.0;
    __syncthreads();
    const int n2 = (l + 1) / 2 * 2, m = n2 - 1;   // an odd l plays with one idle index
    for (int sweep = 0; sweep < 12; ++sweep) {
      // converged when every off-diagonal element is negligible against the diagonal
      double offmax = 0.0, diagmax = 0.0;
      for (int idx = t; idx < l * l; idx += CS_THREADS) {
        const double a = fabs(A[idx / l][idx % l]);
        if (idx / l == idx % l) diagmax = fmax(diagmax, a); else offmax = fmax(offmax, a);
      }
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) {
        offmax = fmax(offmax, __shfl_xor(offmax, off, 64));
        diagmax = fmax(diagmax, __shfl_xor(diagmax, off, 64));
      }
      if ((t & 63) == 0) {
        red[0][t >> 6] = offmax;
        red[1][t >> 6] = diagmax;
      }
      __syncthreads();
      offmax = 0.0;
      diagmax = 0.0;
      for (int w = 0; w < CS_THREADS / 64; ++w) {
        offmax = fmax(offmax, red[0][w]);
        diagmax = fmax(diagmax, red[1][w]);
      }
      __syncthreads();   // red is rewritten by the next sweep
      if (offmax <= 1e-10 * diagmax) break;   // the same values in every thread
      for (int rr = 0; rr < m; ++rr) {
        if (t < n2 / 2) {
          const int a = t == 0 ? m : (rr + t) % m, b = t == 0 ? rr : (rr - t + m) % m;
          const int p = min(a, b), q2 = max(a, b);
          if (q2 < l) {
            const double apq = A[p][q2], app = A[p][p], aqq = A[q2][q2];
            double c = 1.0, sn = 0.0;
            if (fabs(apq) > 1e-300 && fabs(apq) > 1e-17 * sqrt(fabs(app * aqq))) {
              const double theta = (aqq - app) / (2.0 * apq);
              const double tt = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
              c = 1.0 / sqrt(tt * tt + 1.0);
              sn = tt * c;
            }
            partner[p] = q2;
            cc[p] = c;
            ss[p] = -sn;
            partner[q2] = p;
            cc[q2] = c;
            ss[q2] = sn;
          } else if (p < l) {   // paired with the idle index
            partner[p] = p;
            cc[p] = 1.0;
            ss[p] = 0.0;
          }
        }
        __syncthreads();
        double an[CS_PER], vn[CS_PER];
#pragma unroll
        for (int u = 0; u < CS_PER; ++u) {
          const int idx = t + u * CS_THREADS;
          if (idx < l * l) {
            const int i = idx / l, k2 = idx % l, pi = partner[i], pk = partner[k2];
            const double ci = cc[i], si = ss[i], ck = cc[k2], sk = ss[k2];
            an[u] = ci * (ck * A[i][k2] + sk * A[i][pk]) + si * (ck * A[pi][k2] + sk * A[pi][pk]);
            vn[u] = ck * V[i][k2] + sk * V[i][pk];
          }
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < CS_PER; ++u) {
          const int idx = t + u * CS_THREADS;
          if (idx < l * l) {
            A[idx / l][idx % l] = an[u];
            V[idx / l][idx % l] = vn[u];
          }
        }
        __syncthreads();
      }
    }
    if (t < l) ev[t] = A[t][t];
    __syncthreads();
    if (t < l) {   // rank of eigenvalue t in descending order, ties by index
      int rank = 0;
      for (int i = 0; i < l; ++i) rank += (ev[i] > ev[t]) || (ev[i] == ev[t] && i < t);
      order[rank] = t;
    }
    __syncthreads();
    for (int idx = t; idx < r * CP_LMAX; idx += CS_THREADS) {
      const int rho = idx / CP_LMAX, b = idx % CP_LMAX;
      cf[idx] = b < l ? (float)V[b][order[rho]] : 0.f;
    }
    if (t == 0) {
      double s = 0.0;
      for (int rho = 0; rho < r; ++rho) s += fmax(ev[order[rho]], 0.0);
      lam[e] = s;
    }
  }
}

// ---------------------------------------------------------------- out[e][a][:] = sum_b coef[e][a][b] X[e l + b][:]
template <class OutT>
__global__ __launch_bounds__(256) void cmp_apply_kernel(const float* __restrict__ coef, const half_t* __restrict__ X,
                                                        int l, int ra, int n, OutT* __restrict__ out) {
  __shared__ float cs[CP_LMAX * CP_LMAX];
  const int e = blockIdx.y, tid = threadIdx.x;
  for (int idx = tid; idx < ra * CP_LMAX; idx += 256) cs[idx] = coef[(size_t)e * CP_LMAX * CP_LMAX + idx];
  __syncthreads();
  const int col = blockIdx.x * 256 + tid;
  if (col >= n) return;
  float xv[CP_LMAX];
#pragma unroll
  for (int b = 0; b < CP_LMAX; ++b) xv[b] = (b < l) ? (float)X[((size_t)e * l + b) * n + col] : 0.f;
  for (int a = 0; a < ra; ++a) {
    float s = 0.f;
#pragma unroll
    for (int b = 0; b < CP_LMAX; ++b) s = fmaf(cs[a * CP_LMAX + b], xv[b], s);
    out[((size_t)e * ra + a) * n + col] = (OutT)s;
  }
}

// ---------------------------------------------------------------- Sec. 3.4 quantiser
// One thread per group of q consecutive elements of a row: scale = f16(absmax / 7),
// code = clip(rint(w / scale), -7, 7), codes 0 when the scale rounds to 0 or the row's
// expert is gated off (gate != NULL and gate[row / rows_per_expert] != 0).
__global__ __launch_bounds__(256) void cmp_quantize_kernel(const float* __restrict__ src, long rows, int L, int q,
                                                           const int* __restrict__ gate, int rows_per_expert,
                                                           uint8_t* __restrict__ codes, half_t* __restrict__ scales) {
  const long gidx = (long)blockIdx.x * 256 + threadIdx.x;
  const int gpr = L / q;
  if (gidx >= rows * gpr) return;
  const long row = gidx / gpr;
  const int g = (int)(gidx % gpr);
  const float* s = src + row * L + (long)g * q;
  const bool off = gate != nullptr && gate[row / rows_per_expert] != 0;
  float absmax = 0.f;
  for (int i = 0; i < q; ++i) absmax = fmaxf(absmax, fabsf(s[i]));
  half_t sc = (half_t)(absmax / 7.0f);
  if (off) sc = (half_t)0.f;
  scales[row * gpr + g] = sc;
  const float scf = (float)sc;
  uint8_t* dst = codes + row * (L / 2) + (long)g * (q / 2);
  for (int i = 0; i < q; i += 2) {
    int c0 = 0, c1 = 0;
    if (scf > 0.f) {
      c0 = (int)fminf(fmaxf(rintf(s[i] / scf), -7.f), 7.f);
      c1 = (int)fminf(fmaxf(rintf(s[i + 1] / scf), -7.f), 7.f);
    }
    dst[i / 2] = (uint8_t)((c0 & 0xF) | ((c1 & 0xF) << 4));
  }
}

// gate[e] = 1 when cos(vec Delta_e, vec base_c) < gamma (Sec. 3.4); report[e][2] = cosine,
// report[e][3] = gate, report[e][1] = rank-r error before quantisation
//   sqrt(max(||Delta||^2 - sum of the r largest Ritz values, 0)) / ||W_e||.
__global__ void cmp_gate_kernel(const double* __restrict__ stats, const double* __restrict__ lam, int E, int use_gate,
                                float gamma, int* __restrict__ gate, float* __restrict__ report) {
  const int e = blockIdx.x * 64 + threadIdx.x;
  if (e >= E) return;
  const double dd = stats[e * 4 + 0], db = stats[e * 4 + 1], bb = stats[e * 4 + 2], ww = stats[e * 4 + 3];
  const double den = sqrt(dd) * sqrt(bb);
  const double cosv = den > 0.0 ? db / den : 0.0;
  const int g = (use_gate && cosv < (double)gamma) ? 1 : 0;
  gate[e] = g;
  report[e * 4 + 1] = ww > 0.0 ? (float)(sqrt(fmax(dd - lam[e], 0.0)) / sqrt(ww)) : 0.f;
  report[e * 4 + 2] = (float)cosv;
  report[e * 4 + 3] = (float)g;
}

// ---------------------------------------------------------------- reconstruction error of a stored form
// epart[e][workgroup] = sum over its 64 x 256 elements of (W - base - U V)^2 with U, V dequantised
// (Sec. 3.2's Frobenius error, for what the layer will actually compute); wpart = sum W^2.
__device__ __forceinline__ float cmp_nib(const uint8_t* row, int n) {
  const unsigned b = row[n >> 1];
  return (float)((int)((n & 1 ? b >> 4 : b & 0xF) ^ 8) - 8);
}
// A workgroup takes 64 rows and CE_CT consecutive 64-column tiles of one expert: the U panel
// of its rows is decoded once, the V panel per column tile, all global loads issued before
// the first use; epart has one entry per workgroup.  A one-dimensional grid of
// 8 * ceil(G * tiles / 8) * K workgroups.  The kernel is bound by the vector ALUs, not by
// memory: rebuilding U V costs r FP32 FMAs per element (34 GFLOP for 64 experts of
// 8192 x 2048 at r = 16, about 0.5 ms of issue) next to 2.4 GB of reads.
constexpr int CE_CT = 4;
__global__ __launch_bounds__(256) void cmp_error_kernel(const half_t* __restrict__ W, const half_t* __restrict__ base,
                                                        const uint8_t* __restrict__ u_q,
                                                        const half_t* __restrict__ u_s,
                                                        const uint8_t* __restrict__ v_q,
                                                        const half_t* __restrict__ v_s, int G, int K, int out_d, int in_d,
                                                        int r, int q, int tiles_x, int tiles_y,
                                                        float* __restrict__ epart) {
  __shared__ float us[32][64];                               // U[rho][o0 + 0..63]
  __shared__ __attribute__((aligned(16))) float vs[32][64];  // V[rho][i0 + 0..63]
  __shared__ float red[4][2];
  // Workgroups are dealt round-robin to the 8 XCDs; the K experts of one (cluster, tile) take
  // K consecutive workgroups of ONE XCD, so that the base tile they share is fetched from
  // memory once and found in that XCD's L2 by the others.
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
  const int tc = (local / K) * 8 + xcd, per_c = tiles_x * tiles_y;
  if (tc >= G * per_c) return;
  const int c = tc / per_c, e = c * K + local % K;
  const int tile_y = (tc % per_c) / tiles_x, tile_x = (tc % per_c) % tiles_x;
  const int o0 = tile_y * 64, tid = threadIdx.x;
  const int row0 = tid >> 3, ch = tid & 7;
  const size_t me = (size_t)out_d * in_d;
  // Panels: thread tid < 8 r owns the 8 codes (one 32-bit word) of rank row tid / 8 at columns
  // 8 (tid % 8) .. + 7 of a 64-column tile and their scale (one scale when q is a multiple of
  // 8; other group lengths take the element-wise path).  Every global load of the workgroup -
  // the U words, the V words of all column tiles, the W and base tiles - is issued up front.
  const bool words = (q % 8) == 0;
  const int prho = tid >> 3, pwd = tid & 7;
  const bool powner = words && prho < r;
  const size_t prow = (size_t)e * r + (powner ? prho : 0);
  auto put = [&](float (*dst)[64], unsigned w, float sc) {
#pragma unroll
    for (int b2 = 0; b2 < 4; ++b2) {
      const unsigned byte = (w >> (8 * b2)) & 0xffu;
      dst[prho][pwd * 8 + 2 * b2] = sc * (float)((int)((byte & 0xFu) ^ 8u) - 8);
      dst[prho][pwd * 8 + 2 * b2 + 1] = sc * (float)((int)((byte >> 4) ^ 8u) - 8);
    }
  };
  unsigned uw = 0u, vw[CE_CT];
  float usc = 0.f, vsc[CE_CT];
  half8 w8[CE_CT][2], b8[CE_CT][2];
  if (powner) {
    uw = *(const unsigned*)(u_q + prow * (out_d / 2) + (o0 + pwd * 8) / 2);
    usc = (float)u_s[prow * (out_d / q) + (o0 + pwd * 8) / q];
  }
#pragma unroll
  for (int ct = 0; ct < CE_CT; ++ct) {
    const int i0 = (tile_x * CE_CT + ct) * 64;
    const bool in = i0 < in_d;
    vw[ct] = 0u;
    vsc[ct] = 0.f;
    if (powner && in) {
      vw[ct] = *(const unsigned*)(v_q + prow * (in_d / 2) + (i0 + pwd * 8) / 2);
      vsc[ct] = (float)v_s[prow * (in_d / q) + (i0 + pwd * 8) / q];
    }
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const size_t off = (size_t)(o0 + row0 + 32 * u) * in_d + (in ? i0 : 0) + ch * 8;
      w8[ct][u] = *(const half8*)(W + (size_t)e * me + off);
      b8[ct][u] = *(const half8*)(base + (size_t)c * me + off);
    }
  }
  if (words) {
    if (powner) put(us, uw, usc);
  } else {
    for (int idx = tid; idx < r * 64; idx += 256) {
      const int rho = idx / 64, j = idx % 64;
      const size_t row = (size_t)e * r + rho;
      us[rho][j] = (float)u_s[row * (out_d / q) + (o0 + j) / q] * cmp_nib(u_q + row * (out_d / 2), o0 + j);
    }
  }
  float se = 0.f, sw = 0.f;
#pragma unroll
  for (int ct = 0; ct < CE_CT; ++ct) {
    const int i0 = (tile_x * CE_CT + ct) * 64;
    if (i0 >= in_d) break;   // uniform over the workgroup
    if (ct > 0) __syncthreads();   // the previous column tile has been consumed
    if (words) {
      if (powner) put(vs, vw[ct], vsc[ct]);
    } else {
      for (int idx = tid; idx < r * 64; idx += 256) {
        const int rho = idx / 64, j = idx % 64;
        const size_t row = (size_t)e * r + rho;
        vs[rho][j] = (float)v_s[row * (in_d / q) + (i0 + j) / q] * cmp_nib(v_q + row * (in_d / 2), i0 + j);
      }
    }
    __syncthreads();   // us (first tile) and vs are complete
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      const int row = row0 + 32 * u;
      float uv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) uv[i] = 0.f;
      for (int rho = 0; rho < r; ++rho) {
        const float uo = us[rho][row];
        const float4v va = *(const float4v*)&vs[rho][ch * 8], vb = *(const float4v*)&vs[rho][ch * 8 + 4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          uv[i] = fmaf(uo, va[i], uv[i]);
          uv[4 + i] = fmaf(uo, vb[i], uv[4 + i]);
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float w = (float)w8[ct][u][i];
        const float dv = w - (float)b8[ct][u][i] - uv[i];
        se = fmaf(dv, dv, se);
        sw = fmaf(w, w, sw);
      }
    }
  }
  float v[2] = {se, sw};
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v[a] += __shfl_xor(v[a], off, 64);
  if ((tid & 63) == 0) {
    red[tid >> 6][0] = v[0];
    red[tid >> 6][1] = v[1];
  }
  __syncthreads();
  if (tid < 2)
    epart[((size_t)e * per_c + tc % per_c) * 2 + tid] = ((red[0][tid] + red[1][tid]) + red[2][tid]) + red[3][tid];
}
// err[e * stride] = sqrt(sum epart[..][0]) / sqrt(sum epart[..][1]), FP64, fixed order
__global__ __launch_bounds__(64) void cmp_error_finish_kernel(const float* __restrict__ epart, int n_tiles, int stride,
                                                              float* __restrict__ err) {
  const int e = blockIdx.x, lane = threadIdx.x;
  double se = 0.0, sw = 0.0;
  for (int t = lane; t < n_tiles; t += 64) {
    se += (double)epart[((size_t)e * n_tiles + t) * 2];
    sw += (double)epart[((size_t)e * n_tiles + t) * 2 + 1];
  }
  for (int off = 32; off > 0; off >>= 1) {
    se += __shfl_xor(se, off, 64);
    sw += __shfl_xor(sw, off, 64);
  }
  if (lane == 0) err[(size_t)e * stride] = sw > 0.0 ? (float)(sqrt(se) / sqrt(sw)) : 0.f;
}

struct CompressLayout {
  size_t D, DT, XA, XB, offsets, part, stats, gpart, coef, lam, gate, UF, VF, epart, total;
};
CompressLayout compress_layout(const cmoe_compress_config& c) {
  CompressLayout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = (off + bytes + 255) & ~(size_t)255;
    return at;
  };
  const size_t E = (size_t)c.G * c.K, me = (size_t)c.out_dim * c.in_dim;
  const size_t nmax = c.out_dim > c.in_dim ? c.out_dim : c.in_dim;
  const size_t tiles = (size_t)(c.out_dim / 64) * (c.in_dim / 64);
  L.D = take(E * me * 2);
  L.DT = take(E * me * 2);
  L.XA = take(E * c.sketch * nmax * 2);
  L.XB = take(E * c.sketch * nmax * 2);
  L.offsets = take((E + 1) * 4);
  L.part = take(E * tiles * 4 * 4 * 4);   // four quantities x four wavefront partials per tile
  L.stats = take(E * 4 * 8);
  L.gpart = take(E * ((nmax + 511) / 512) * c.sketch * c.sketch * 4);
  L.coef = take(E * CP_LMAX * CP_LMAX * 4);
  L.lam = take(E * 8);
  L.gate = take(E * 4);
  L.UF = take(E * c.r * (size_t)c.out_dim * 4);
  L.VF = take(E * c.r * (size_t)c.in_dim * 4);
  L.epart = take(E * tiles * 2 * 4);
  L.total = off;
  return L;
}

bool compress_cfg_ok(const cmoe_compress_config* c) {
  if (c == nullptr) return false;
  if (c->out_dim <= 0 || c->in_dim <= 0 || c->out_dim % 64 || c->in_dim % 64) return false;
  if (c->G < 1 || c->K < 1 || c->K > 64 || (long)c->G * c->K > 4096) return false;
  if (c->r < 1 || c->r > 32 || c->sketch < c->r || c->sketch > CP_LMAX) return false;
  if (c->q_group < 2 || c->q_group % 2 || c->out_dim % c->q_group || c->in_dim % c->q_group) return false;
  if (c->n_iter < 0 || c->n_iter > 16) return false;
  return true;
}
bool cptr_ok(const void* p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define CP_CHECK()                         \
  do {                                     \
    hipError_t e_ = hipGetLastError();     \
    if (e_ != hipSuccess) return CMOE_ERR_HIP; \
  } while (0)

// rows of Xin [E l][n] -> orthonormal rows in Xout (Cholesky QR, applied twice by the caller)
int orth_rows(const cmoe_compress_config& c, int E, int n, const half_t* Xin, half_t* Xout, char* ws,
              const CompressLayout& L, hipStream_t st) {
  const int l = c.sketch, nch = (n + 511) / 512;
  hipLaunchKernelGGL(cmp_gram_kernel, dim3(nch, E), dim3(256), 0, st, Xin, l, n, (float*)(ws + L.gpart));
  hipLaunchKernelGGL(cmp_small_kernel<0>, dim3(E), dim3(CS_THREADS), 0, st, (const float*)(ws + L.gpart), nch, l, c.r,
                     (float*)(ws + L.coef), (double*)(ws + L.lam));
  hipLaunchKernelGGL(cmp_apply_kernel<half_t>, dim3((n + 255) / 256, E), dim3(256), 0, st,
                     (const float*)(ws + L.coef), Xin, l, l, n, Xout);
  CP_CHECK();
  return CMOE_OK;
}

}  // namespace

extern "C" size_t cmoe_compress_workspace_bytes(const cmoe_compress_config* cfg) {
  if (!compress_cfg_ok(cfg)) return 0;
  return compress_layout(*cfg).total;
}

extern "C" int cmoe_quantize_int4(const float* src, int64_t rows, int32_t L, int32_t q_group, uint8_t* codes,
                                  cmoe_f16* scales, void* stream) {
  if (rows < 0 || L <= 0 || q_group < 2 || q_group % 2 || L % q_group) return CMOE_ERR_INVALID_ARG;
  if (rows == 0) return CMOE_OK;
  if (!cptr_ok(src) || !cptr_ok(codes) || !cptr_ok(scales)) return CMOE_ERR_INVALID_ARG;
  const long groups = (long)rows * (L / q_group);
  hipLaunchKernelGGL(cmp_quantize_kernel, dim3((unsigned)((groups + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                     src, (long)rows, L, q_group, (const int*)nullptr, 1, codes, (half_t*)scales);
  CP_CHECK();
  return CMOE_OK;
}

extern "C" int cmoe_reconstruction_error(const cmoe_compress_config* cfg, const cmoe_f16* W, const cmoe_f16* base,
                                         const uint8_t* u_q, const cmoe_f16* u_s, const uint8_t* v_q,
                                         const cmoe_f16* v_s, float* err, void* workspace, size_t workspace_bytes,
                                         void* stream) {
  if (!compress_cfg_ok(cfg)) return CMOE_ERR_UNSUPPORTED;
  if (!cptr_ok(W) || !cptr_ok(base) || !cptr_ok(u_q) || !cptr_ok(u_s) || !cptr_ok(v_q) || !cptr_ok(v_s) ||
      !cptr_ok(err) || !cptr_ok(workspace))
    return CMOE_ERR_INVALID_ARG;
  const CompressLayout L = compress_layout(*cfg);
  if (workspace_bytes < L.total) return CMOE_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  const int E = cfg->G * cfg->K, tx = (cfg->in_dim / 64 + CE_CT - 1) / CE_CT, ty = cfg->out_dim / 64;
  hipLaunchKernelGGL(cmp_error_kernel, dim3((unsigned)((cfg->G * tx * ty + 7) / 8 * 8 * cfg->K)), dim3(256), 0, st,
                     (const half_t*)W, (const half_t*)base, u_q, (const half_t*)u_s, v_q, (const half_t*)v_s, cfg->G,
                     cfg->K, cfg->out_dim, cfg->in_dim, cfg->r, cfg->q_group, tx, ty, (float*)(ws + L.epart));
  hipLaunchKernelGGL(cmp_error_finish_kernel, dim3(E), dim3(64), 0, st, (const float*)(ws + L.epart), tx * ty, 1, err);
  CP_CHECK();
  return CMOE_OK;
}

extern "C" int cmoe_compress(const cmoe_compress_config* cfg, const cmoe_f16* W, const cmoe_f16* omega,
                             cmoe_f16* base, uint8_t* u_q, cmoe_f16* u_s, uint8_t* v_q, cmoe_f16* v_s, float* report,
                             void* workspace, size_t workspace_bytes, void* stream) {
  if (!compress_cfg_ok(cfg)) return CMOE_ERR_UNSUPPORTED;
  if (!cptr_ok(W) || !cptr_ok(omega) || !cptr_ok(base) || !cptr_ok(u_q) || !cptr_ok(u_s) || !cptr_ok(v_q) ||
      !cptr_ok(v_s) || !cptr_ok(report) || !cptr_ok(workspace))
    return CMOE_ERR_INVALID_ARG;
  const cmoe_compress_config& c = *cfg;
  const CompressLayout L = compress_layout(c);
  if (workspace_bytes < L.total) return CMOE_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)workspace;
  const int E = c.G * c.K, l = c.sketch, out_d = c.out_dim, in_d = c.in_dim;
  const int tx = in_d / 64, ty = out_d / 64;
  half_t* D = (half_t*)(ws + L.D);
  half_t* DT = (half_t*)(ws + L.DT);
  half_t* XA = (half_t*)(ws + L.XA);
  half_t* XB = (half_t*)(ws + L.XB);
  int* offs = (int*)(ws + L.offsets);
  float* coef = (float*)(ws + L.coef);
  double* stats = (double*)(ws + L.stats);
  double* lam = (double*)(ws + L.lam);
  int* gate = (int*)(ws + L.gate);
  float* UF = (float*)(ws + L.UF);
  float* VF = (float*)(ws + L.VF);

  // Eq. 6 and the residuals (and their transposes) against the stored base
  hipLaunchKernelGGL(cmp_residual_kernel, dim3(tx, ty, c.G), dim3(256), 0, st, (const half_t*)W, c.K, out_d, in_d,
                     (half_t*)base, D, DT, (float*)(ws + L.part));
  hipLaunchKernelGGL(cmp_stats_kernel, dim3(E), dim3(256), 0, st, (const float*)(ws + L.part), tx * ty * 4, stats);
  hipLaunchKernelGGL(cmp_offsets_kernel, dim3((E + 256) / 256), dim3(256), 0, st, E, l, offs);
  hipLaunchKernelGGL(cmp_tile_rows_kernel, dim3((in_d / 8 + 255) / 256, E * l), dim3(256), 0, st, (const half_t*)omega,
                     l, in_d, XA);
  CP_CHECK();
  int rc;
  // Q^T [l][out]: orthonormal rows spanning Delta Omega, refined by n_iter rounds of
  // Z = orth(Delta^T Q), Q = orth(Delta Z)
  if (launch_skinny_rows(XA, D, offs, E, out_d, in_d, l, XB, st) != hipSuccess) return CMOE_ERR_HIP;
  if ((rc = orth_rows(c, E, out_d, XB, XA, ws, L, st)) != CMOE_OK) return rc;
  if ((rc = orth_rows(c, E, out_d, XA, XB, ws, L, st)) != CMOE_OK) return rc;   // Q^T in XB
  for (int it = 0; it < c.n_iter; ++it) {
    if (launch_skinny_rows(XB, DT, offs, E, in_d, out_d, l, XA, st) != hipSuccess) return CMOE_ERR_HIP;
    if ((rc = orth_rows(c, E, in_d, XA, XB, ws, L, st)) != CMOE_OK) return rc;
    if ((rc = orth_rows(c, E, in_d, XB, XA, ws, L, st)) != CMOE_OK) return rc;   // Z^T in XA
    if (launch_skinny_rows(XA, D, offs, E, out_d, in_d, l, XB, st) != hipSuccess) return CMOE_ERR_HIP;
    if ((rc = orth_rows(c, E, out_d, XB, XA, ws, L, st)) != CMOE_OK) return rc;
    if ((rc = orth_rows(c, E, out_d, XA, XB, ws, L, st)) != CMOE_OK) return rc;   // Q^T in XB
  }
  // B = Q^T Delta [l][in] (rows in XA); Rayleigh-Ritz: eigenvectors of B B^T pick the best
  // rank-r pair inside the sketch: U^T = C Q^T, V = C B with C = the r leading eigenvectors
  if (launch_skinny_rows(XB, DT, offs, E, in_d, out_d, l, XA, st) != hipSuccess) return CMOE_ERR_HIP;
  const int nch = (in_d + 511) / 512;
  hipLaunchKernelGGL(cmp_gram_kernel, dim3(nch, E), dim3(256), 0, st, XA, l, in_d, (float*)(ws + L.gpart));
  hipLaunchKernelGGL(cmp_small_kernel<1>, dim3(E), dim3(CS_THREADS), 0, st, (const float*)(ws + L.gpart), nch, l, c.r, coef,
                     lam);
  hipLaunchKernelGGL(cmp_apply_kernel<float>, dim3((out_d + 255) / 256, E), dim3(256), 0, st, (const float*)coef, XB,
                     l, c.r, out_d, UF);
  hipLaunchKernelGGL(cmp_apply_kernel<float>, dim3((in_d + 255) / 256, E), dim3(256), 0, st, (const float*)coef, XA, l,
                     c.r, in_d, VF);
  // gate, quantisation (Sec. 3.4), and the error of the stored form
  hipLaunchKernelGGL(cmp_gate_kernel, dim3((E + 63) / 64), dim3(64), 0, st, (const double*)stats, (const double*)lam,
                     E, c.use_gate, c.gate_gamma, gate, report);
  const long ug = (long)E * c.r * (out_d / c.q_group), vg = (long)E * c.r * (in_d / c.q_group);
  hipLaunchKernelGGL(cmp_quantize_kernel, dim3((unsigned)((ug + 255) / 256)), dim3(256), 0, st, (const float*)UF,
                     (long)E * c.r, out_d, c.q_group, (const int*)gate, c.r, u_q, (half_t*)u_s);
  hipLaunchKernelGGL(cmp_quantize_kernel, dim3((unsigned)((vg + 255) / 256)), dim3(256), 0, st, (const float*)VF,
                     (long)E * c.r, in_d, c.q_group, (const int*)gate, c.r, v_q, (half_t*)v_s);
  const int etx = (tx + CE_CT - 1) / CE_CT;
  hipLaunchKernelGGL(cmp_error_kernel, dim3((unsigned)((c.G * etx * ty + 7) / 8 * 8 * c.K)), dim3(256), 0, st,
                     (const half_t*)W, (const half_t*)base, u_q, (const half_t*)u_s, v_q, (const half_t*)v_s, c.G, c.K,
                     out_d, in_d, c.r, c.q_group, etx, ty, (float*)(ws + L.epart));
  hipLaunchKernelGGL(cmp_error_finish_kernel, dim3(E), dim3(64), 0, st, (const float*)(ws + L.epart), etx * ty, 4,
                     report);
  CP_CHECK();
  return CMOE_OK;
}
