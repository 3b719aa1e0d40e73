// Grouped matrix-core kernels of the expert computation (Sec. 3.2):
//   t1   = V1 x                       (all experts of the token's cluster, then masked)
//   Hb   = W1_base(c) x  -> fused: + U1 t1, GELU, gated sum A, s = V2 a
//   Yb   = W2_base(c) A
//   y    = Yb + sum_j g_j U2 s_j, back in token order
//
// All products are computed "weights x tokens^T": the weight rows are the A operand of
// v_mfma_f32_32x32x16_f16 (rows n of the 32x32 block), the tokens are the B operand
// (columns m).  A lane of a 32x32 accumulator block then holds ONE token (column
// m = lane % 32) and 16 output rows n = 8*(v/4) + 4*(lane/32) + v%4, v = 0..15.  That is
// what lets the per-token quantities (experts, gates) live in per-lane registers, and lets
// an accumulator block be fed back as the B operand of the next product without leaving
// registers (its rows become the contraction index).
#include "cmoe_internal.h"

namespace {

template <int BN_, int BM_, int WAVES_N_, int WAVES_M_>
struct Tile {
  static constexpr int BN = BN_, BM = BM_, WAVES_N = WAVES_N_, WAVES_M = WAVES_M_;
  static constexpr int NT = WAVES_N * WAVES_M * 64;
  static constexpr int WN = BN / WAVES_N, WM = BM / WAVES_M;
  static constexpr int NB = WN / 32, MB = WM / 32;
  static constexpr int BK = 64;        // contraction elements per LDS stage
  static constexpr int LDK = BK + 8;   // padded LDS row (halfs): 144 B, conflict-free b128 reads
  static constexpr int WCH = BN * (BK / 8) / NT, XCH = BM * (BK / 8) / NT;  // 16-B chunks per thread
  static constexpr int SMEM_HALFS = 2 * (BN + BM) * LDK;
  static_assert(BN % (32 * WAVES_N) == 0 && BM % (32 * WAVES_M) == 0, "wave tile");
  static_assert((BN * (BK / 8)) % NT == 0 && (BM * (BK / 8)) % NT == 0, "load split");
};

struct GemmArgs {
  const half_t* W;   // weights of cluster c: W + c * w_cstride, [N][ldw] row-major
  long w_cstride;
  int ldw, N;
  const half_t* X;   // token-side operand, row for sorted row p: X + (gather ? gather[p] : p) * ldx
  int ldx;
  const int* gather;
  int Kc;            // contraction length, multiple of 64
  const int* offsets;
  int G, n_tiles;
};

struct TileCtx {
  int c, n_tile, n0, m0, m_end, wn, wm, lane, tid;
  half_t* smem;
};

__device__ __forceinline__ float16v mfma16(half8 a, half8 b, float16v c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float gelu_erf(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752f)); }

template <class TL, class Epi>
__global__ __launch_bounds__(TL::NT) void gemm_nt_kernel(GemmArgs g, Epi epi) {
  __shared__ __attribute__((aligned(16))) half_t smem[TL::SMEM_HALFS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave % TL::WAVES_N, wm = wave / TL::WAVES_N;

  // which (cluster, row tile, column tile) this workgroup owns: derived on the device
  // from the cluster offsets, so no host round trip sits between routing and the GEMMs
  const int n_tile = blockIdx.x % g.n_tiles;
  int slot = blockIdx.x / g.n_tiles;
  int c = 0, m0 = 0, m_end = 0;
  for (; c < g.G; ++c) {
    int lo = g.offsets[c], hi = g.offsets[c + 1];
    int tiles = (hi - lo + TL::BM - 1) / TL::BM;
    if (slot < tiles) {
      m0 = lo + slot * TL::BM;
      m_end = hi;
      break;
    }
    slot -= tiles;
  }
  if (c == g.G) return;
  const int n0 = n_tile * TL::BN;

  half_t* sW = smem;                               // [2][BN][LDK]
  half_t* sX = smem + 2 * TL::BN * TL::LDK;        // [2][BM][LDK]
  const half_t* Wc = g.W + (size_t)c * g.w_cstride;

  const half_t* gw[TL::WCH];
  const half_t* gx[TL::XCH];
  int lw[TL::WCH], lx[TL::XCH];
#pragma unroll
  for (int i = 0; i < TL::WCH; ++i) {
    int id = tid + i * TL::NT, row = id >> 3, ch = id & 7;
    int n = min(n0 + row, g.N - 1);
    gw[i] = Wc + (size_t)n * g.ldw + ch * 8;
    lw[i] = row * TL::LDK + ch * 8;
  }
#pragma unroll
  for (int i = 0; i < TL::XCH; ++i) {
    int id = tid + i * TL::NT, row = id >> 3, ch = id & 7;
    int p = min(m0 + row, m_end - 1);
    int src = g.gather ? g.gather[p] : p;
    gx[i] = g.X + (size_t)src * g.ldx + ch * 8;
    lx[i] = row * TL::LDK + ch * 8;
  }

  float16v acc[TL::NB][TL::MB];
#pragma unroll
  for (int a = 0; a < TL::NB; ++a)
#pragma unroll
    for (int b = 0; b < TL::MB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  half8 rw[TL::WCH], rx[TL::XCH];
  const int KT = g.Kc / TL::BK;
#pragma unroll
  for (int i = 0; i < TL::WCH; ++i) rw[i] = *(const half8*)(gw[i]);
#pragma unroll
  for (int i = 0; i < TL::XCH; ++i) rx[i] = *(const half8*)(gx[i]);
#pragma unroll
  for (int i = 0; i < TL::WCH; ++i) *(half8*)(sW + lw[i]) = rw[i];
#pragma unroll
  for (int i = 0; i < TL::XCH; ++i) *(half8*)(sX + lx[i]) = rx[i];
  __syncthreads();

  const int frag_row = lane & 31, frag_col = (lane >> 5) * 8;
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
#pragma unroll
      for (int i = 0; i < TL::WCH; ++i) rw[i] = *(const half8*)(gw[i] + (size_t)(kt + 1) * TL::BK);
#pragma unroll
      for (int i = 0; i < TL::XCH; ++i) rx[i] = *(const half8*)(gx[i] + (size_t)(kt + 1) * TL::BK);
    }
    const half_t* cw = sW + cur * TL::BN * TL::LDK + (wn * TL::WN + frag_row) * TL::LDK + frag_col;
    const half_t* cx = sX + cur * TL::BM * TL::LDK + (wm * TL::WM + frag_row) * TL::LDK + frag_col;
#pragma unroll
    for (int ks = 0; ks < TL::BK / 16; ++ks) {
      half8 fa[TL::NB], fb[TL::MB];
#pragma unroll
      for (int a = 0; a < TL::NB; ++a) fa[a] = *(const half8*)(cw + a * 32 * TL::LDK + ks * 16);
#pragma unroll
      for (int b = 0; b < TL::MB; ++b) fb[b] = *(const half8*)(cx + b * 32 * TL::LDK + ks * 16);
#pragma unroll
      for (int a = 0; a < TL::NB; ++a)
#pragma unroll
        for (int b = 0; b < TL::MB; ++b) acc[a][b] = mfma16(fa[a], fb[b], acc[a][b]);
    }
    if (kt + 1 < KT) {
      half_t* nw = sW + (cur ^ 1) * TL::BN * TL::LDK;
      half_t* nx = sX + (cur ^ 1) * TL::BM * TL::LDK;
#pragma unroll
      for (int i = 0; i < TL::WCH; ++i) *(half8*)(nw + lw[i]) = rw[i];
#pragma unroll
      for (int i = 0; i < TL::XCH; ++i) *(half8*)(nx + lx[i]) = rx[i];
    }
    __syncthreads();
  }

  TileCtx ctx{c, n_tile, n0, m0, m_end, wn, wm, lane, tid, smem};
  epi.template run<TL>(ctx, acc);
}

__device__ __forceinline__ half4 to_half4(const float16v& a, int qd) {
  half4 o;
  o[0] = (half_t)a[4 * qd + 0];
  o[1] = (half_t)a[4 * qd + 1];
  o[2] = (half_t)a[4 * qd + 2];
  o[3] = (half_t)a[4 * qd + 3];
  return o;
}

// ---------------------------------------------------------------- epilogue: plain store
// out[p][n] = acc (f16), rows p in cluster-sorted order.
struct EpiStore {
  half_t* out;
  int ldo, N;
  template <class TL>
  __device__ void run(const TileCtx& t, float16v (&acc)[TL::NB][TL::MB]) const {
    const int h = t.lane >> 5;
#pragma unroll
    for (int b = 0; b < TL::MB; ++b) {
      int p = t.m0 + t.wm * TL::WM + b * 32 + (t.lane & 31);
      if (p >= t.m_end) continue;
#pragma unroll
      for (int a = 0; a < TL::NB; ++a) {
        int nb = t.n0 + t.wn * TL::WN + a * 32;
        if (nb >= N) continue;
#pragma unroll
        for (int qd = 0; qd < 4; ++qd)
          *(half4*)(out + (size_t)p * ldo + nb + 8 * qd + 4 * h) = to_half4(acc[a][b], qd);
      }
    }
  }
};

// ---------------------------------------------------------------- epilogue: t1, one-hot expanded
// acc rows are kk = j_local * r + rho over ALL experts of the cluster.  For the token's
// j-th selected expert e_j only the r rows of e_j are kept, the rest written as zero:
//   t1ext[p][j][kk] = (kk / r == e_j - c*K) ? (V1 x)[kk] : 0
// so that U1cat^T (d_ff x K*r) times t1ext[p][j] equals U1_{e_j} (V1_{e_j} x).
struct EpiT1 {
  half_t* t1ext;
  const int* perm;
  const int* expert_idx;
  int k, K, r, KRp;
  template <class TL>
  __device__ void run(const TileCtx& t, float16v (&acc)[TL::NB][TL::MB]) const {
    const int h = t.lane >> 5;
#pragma unroll
    for (int b = 0; b < TL::MB; ++b) {
      int p = t.m0 + t.wm * TL::WM + b * 32 + (t.lane & 31);
      if (p >= t.m_end) continue;
      int tok = perm[p];
      for (int j = 0; j < k; ++j) {
        int e = min(max(expert_idx[(size_t)tok * k + j] - t.c * K, 0), K - 1);
        half_t* row = t1ext + ((size_t)p * k + j) * KRp;
#pragma unroll
        for (int a = 0; a < TL::NB; ++a) {
          int nb = t.n0 + t.wn * TL::WN + a * 32;
          if (nb >= KRp) continue;
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            int kk = nb + 8 * qd + 4 * h;
            half4 v = to_half4(acc[a][b], qd);
            if (kk / r != e) v = half4{0, 0, 0, 0};
            *(half4*)(row + kk) = v;
          }
        }
      }
    }
  }
};

// ---------------------------------------------------------------- epilogue: fused up-projection
// acc = Hb^T block (rows n of d_ff, columns = tokens).  Per token column and selected
// expert j:  h_j = Hb + U1cat^T t1ext_j  (matrix core, contraction over kk, empty 16-chunks
// skipped), a_j = GELU(h_j), A += g_j a_j, and s_j += V2 a_j by feeding the a_j block back
// as B operand (contraction over the block's 32 rows n).  The V2 product runs over
// "passes" of 32 rank rows (32/r experts); a lane contributes to a pass only if its
// token's expert lies in it, so after all passes row (e_j % (32/r))*r + rho of the
// accumulator holds s_j[rho].
template <int KMAX>
struct EpiFusedUp {
  const half_t* u1t;    // [G][d_ff][KRp]
  const half_t* v2p;    // [G][KRp][d_ff], columns permuted inside 16-groups
  const half_t* t1ext;  // [T][k][KRp]
  const int* perm;
  const int* expert_idx;
  const float* gate;
  half_t* A;            // [T][d_ff]
  float* spart;         // [n_tiles][T][k][r]
  int T, k, K, r, KRp, d_ff;

  template <class TL>
  __device__ void run(const TileCtx& t, float16v (&acc)[TL::NB][TL::MB]) const {
    const int h = t.lane >> 5, ml = t.lane & 31;
    const half_t* u1c = u1t + (size_t)t.c * d_ff * KRp;
    const half_t* v2c = v2p + (size_t)t.c * KRp * d_ff;
    const int n_chunks = KRp / 16, n_pass = KRp / 32, epb = 32 / r;
    float* sbuf = (float*)t.smem;  // [WAVES_N][BM][33] floats, reuses the tile buffers
    static_assert(TL::WAVES_N * TL::BM * 33 * 4 <= TL::SMEM_HALFS * 2, "s buffer fits");

#pragma unroll 1
    for (int b = 0; b < TL::MB; ++b) {
      const int p = t.m0 + t.wm * TL::WM + b * 32 + ml;
      const bool valid = p < t.m_end;
      const int pc = valid ? p : t.m_end - 1;
      const int tok = perm[pc];
      int e[KMAX];
      float gj[KMAX];
      unsigned cmask[KMAX], pmask[KMAX];
      const half_t* t1row[KMAX];
      float16v sacc[KMAX];
#pragma unroll
      for (int j = 0; j < KMAX; ++j) {
        e[j] = 0;
        gj[j] = 0.f;
        cmask[j] = 0;
        pmask[j] = 0;
        t1row[j] = t1ext;
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[j][v] = 0.f;
        if (j < k) {
          e[j] = min(max(expert_idx[(size_t)tok * k + j] - t.c * K, 0), K - 1);
          gj[j] = valid ? gate[(size_t)tok * k + j] : 0.f;
          t1row[j] = t1ext + ((size_t)pc * k + j) * KRp;
          int lo = (e[j] * r) >> 4, hi = (e[j] * r + r - 1) >> 4, ps = (e[j] * r) >> 5;
          for (int kc = 0; kc < n_chunks; ++kc)
            if (__ballot(valid && kc >= lo && kc <= hi) != 0ull) cmask[j] |= 1u << kc;
          for (int q = 0; q < n_pass; ++q)
            if (__ballot(valid && q == ps) != 0ull) pmask[j] |= 1u << q;
        }
      }
#pragma unroll
      for (int a = 0; a < TL::NB; ++a) {
        const int nb = t.n0 + t.wn * TL::WN + a * 32;
        if (nb >= d_ff) continue;
        const half_t* u1row = u1c + (size_t)(nb + ml) * KRp + 8 * h;
        float16v o;
#pragma unroll
        for (int v = 0; v < 16; ++v) o[v] = 0.f;
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
          if (j >= k) continue;
          float16v hj = acc[a][b];
          for (int kc = 0; kc < n_chunks; ++kc) {
            if (!((cmask[j] >> kc) & 1u)) continue;
            half8 fa = *(const half8*)(u1row + kc * 16);
            half8 fb = *(const half8*)(t1row[j] + kc * 16 + 8 * h);
            hj = mfma16(fa, fb, hj);
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            hj[v] = gelu_erf(hj[v]);
            o[v] += gj[j] * hj[v];
          }
          const int my_pass = (e[j] * r) >> 5;
          for (int q = 0; q < n_pass; ++q) {
            if (!((pmask[j] >> q) & 1u)) continue;
            const bool on = valid && (q == my_pass);
            const half_t* v2row = v2c + (size_t)(q * 32 + ml) * d_ff + nb + 8 * h;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
              half8 fb;
#pragma unroll
              for (int i = 0; i < 8; ++i) fb[i] = on ? (half_t)hj[8 * s + i] : (half_t)0.f;
              half8 fa = *(const half8*)(v2row + 16 * s);
              sacc[j] = mfma16(fa, fb, sacc[j]);
            }
          }
        }
        if (valid) {
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) *(half4*)(A + (size_t)p * d_ff + nb + 8 * qd + 4 * h) = to_half4(o, qd);
        }
      }
      // s partial of this column block: sum over the wavefronts that split the rows n,
      // in a fixed order, one selected expert at a time through LDS
      for (int j = 0; j < k; ++j) {
        __syncthreads();
        float* mine = sbuf + ((size_t)t.wn * TL::BM + t.wm * TL::WM + b * 32 + ml) * 33;
#pragma unroll
        for (int jj = 0; jj < KMAX; ++jj) {
          if (jj != j) continue;
#pragma unroll
          for (int v = 0; v < 16; ++v) mine[8 * (v >> 2) + 4 * h + (v & 3)] = sacc[jj][v];
        }
        __syncthreads();
        // rows of this b-block only: [wm*WM + b*32, +32) for every wm
        for (int idx = t.tid; idx < TL::WAVES_M * 32 * r; idx += TL::NT) {
          int rho = idx % r, mm = idx / r;
          int m = (mm / 32) * TL::WM + b * 32 + (mm % 32);
          int pp = t.m0 + m;
          if (pp >= t.m_end) continue;
          int tk = perm[pp];
          int ee = min(max(expert_idx[(size_t)tk * k + j] - t.c * K, 0), K - 1);
          int row = (ee % epb) * r + rho;
          float sum = 0.f;
#pragma unroll
          for (int w = 0; w < TL::WAVES_N; ++w) sum += sbuf[((size_t)w * TL::BM + m) * 33 + row];
          spart[(((size_t)t.n_tile * T + pp) * k + j) * r + rho] = sum;
        }
      }
    }
  }
};

// ---------------------------------------------------------------- s partial reduction
__global__ __launch_bounds__(256) void sreduce_kernel(const float* __restrict__ spart, const int* __restrict__ perm,
                                                      int T, int kr, int n_tiles, float* __restrict__ s_down) {
  size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (size_t)T * kr) return;
  size_t p = idx / kr;
  int w = (int)(idx % kr);
  float sum = 0.f;
  for (int nt = 0; nt < n_tiles; ++nt) sum += spart[((size_t)nt * T + p) * kr + w];
  s_down[(size_t)perm[p] * kr + w] = sum;
}

// ---------------------------------------------------------------- combine
// y[perm[p]] = Yb[p] + U2cat^T (d x K*r) . sext[p],   sext[p][e_j*r + rho] = g_j s_j[rho].
// One workgroup: 32 sorted rows x NSPAN blocks of 32 output columns; the expanded,
// gated s vectors of the 32 rows are built once in LDS as f16.
constexpr int CB_WAVES = 4;
constexpr int CB_NPW = 4;  // 32-column blocks per wavefront

__global__ __launch_bounds__(CB_WAVES * 64) void combine_kernel(
    const half_t* __restrict__ u2t, const half_t* __restrict__ yb, const float* __restrict__ s_down,
    const int* __restrict__ perm, const int* __restrict__ offsets, const int* __restrict__ expert_idx,
    const float* __restrict__ gate, int G, int K, int k, int r, int KRp, int d, int n_groups,
    half_t* __restrict__ y) {
  __shared__ __attribute__((aligned(16))) half_t sext[32 * (512 + 8)];
  __shared__ unsigned s_cmask;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, h = lane >> 5, ml = lane & 31;
  const int ngrp = blockIdx.x % n_groups;
  int slot = blockIdx.x / n_groups;
  int c = 0, m0 = 0, m_end = 0;
  for (; c < G; ++c) {
    int lo = offsets[c], hi = offsets[c + 1];
    int tiles = (hi - lo + 31) / 32;
    if (slot < tiles) {
      m0 = lo + slot * 32;
      m_end = hi;
      break;
    }
    slot -= tiles;
  }
  if (c == G) return;
  const int lds = KRp + 8;
  for (int i = tid; i < 32 * lds / 8; i += CB_WAVES * 64) ((half8*)sext)[i] = half8{0, 0, 0, 0, 0, 0, 0, 0};
  if (tid == 0) s_cmask = 0;
  __syncthreads();
  for (int idx = tid; idx < 32 * k * r; idx += CB_WAVES * 64) {
    int rho = idx % r, j = (idx / r) % k, m = idx / (r * k);
    int p = m0 + m;
    if (p >= m_end) continue;
    int tok = perm[p];
    int e = min(max(expert_idx[(size_t)tok * k + j] - c * K, 0), K - 1);
    float v = gate[(size_t)tok * k + j] * s_down[((size_t)tok * k + j) * r + rho];
    sext[m * lds + e * r + rho] = (half_t)v;
    if (rho == 0) atomicOr(&s_cmask, (0xffffffffu >> (31 - (e * r + r - 1) / 16)) & (0xffffffffu << ((e * r) / 16)));
  }
  __syncthreads();
  const unsigned cmask = s_cmask;
  const int p = m0 + ml;
  const bool valid = p < m_end;
  const int tok = valid ? perm[p] : 0;
  const half_t* u2c = u2t + (size_t)c * d * KRp;
  const int n_chunks = KRp / 16;
  for (int i = 0; i < CB_NPW; ++i) {
    int nb = ((ngrp * CB_WAVES + wave) * CB_NPW + i) * 32;
    if (nb >= d) break;
    float16v acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const half_t* u2row = u2c + (size_t)(nb + ml) * KRp + 8 * h;
    for (int kc = 0; kc < n_chunks; ++kc) {
      if (!((cmask >> kc) & 1u)) continue;
      half8 fa = *(const half8*)(u2row + kc * 16);
      half8 fb = *(const half8*)(sext + ml * lds + kc * 16 + 8 * h);
      acc = mfma16(fa, fb, acc);
    }
    if (valid) {
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) {
        int n = nb + 8 * qd + 4 * h;
        half4 b4 = *(const half4*)(yb + (size_t)p * d + n);
        half4 o;
#pragma unroll
        for (int v = 0; v < 4; ++v) o[v] = (half_t)(acc[4 * qd + v] + (float)b4[v]);
        *(half4*)(y + (size_t)tok * d + n) = o;
      }
    }
  }
}

using TileMain = Tile<128, 128, 2, 2>;
static_assert(TileMain::BN == G1_BN, "workspace sizing assumes this column tile");

template <class TL, class Epi>
hipError_t launch_gemm(const GemmArgs& g, int T, const Epi& epi, hipStream_t st) {
  int m_slots = (T + TL::BM - 1) / TL::BM + g.G;
  dim3 grid((unsigned)(g.n_tiles * m_slots)), block(TL::NT);
  hipLaunchKernelGGL((gemm_nt_kernel<TL, Epi>), grid, block, 0, st, g, epi);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_t1(const cmoe_dims& dm, const half_t* x, int T, const int* perm, const int* offsets,
                     const int* expert_idx, const half_t* v1cat, half_t* t1ext, hipStream_t st) {
  using TL = TileMain;
  GemmArgs g{v1cat, (long)dm.KRp * dm.d, dm.d, dm.KRp, x, dm.d, perm, dm.d, offsets, dm.G,
             (dm.KRp + TL::BN - 1) / TL::BN};
  EpiT1 epi{t1ext, perm, expert_idx, dm.k, dm.K, dm.r, dm.KRp};
  return launch_gemm<TL>(g, T, epi, st);
}

hipError_t launch_gemm1(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, const int* perm,
                        const int* offsets, const int* expert_idx, const float* gate, const half_t* u1t,
                        const half_t* v2p, const half_t* t1ext, half_t* a, float* spart, hipStream_t st) {
  using TL = TileMain;
  GemmArgs g{(const half_t*)w.w1_base, (long)dm.d_ff * dm.d, dm.d, dm.d_ff, x, dm.d, perm, dm.d, offsets, dm.G,
             (dm.d_ff + TL::BN - 1) / TL::BN};
  if (dm.k <= 1) {
    EpiFusedUp<1> epi{u1t, v2p, t1ext, perm, expert_idx, gate, a, spart, T, dm.k, dm.K, dm.r, dm.KRp, dm.d_ff};
    return launch_gemm<TL>(g, T, epi, st);
  } else if (dm.k <= 2) {
    EpiFusedUp<2> epi{u1t, v2p, t1ext, perm, expert_idx, gate, a, spart, T, dm.k, dm.K, dm.r, dm.KRp, dm.d_ff};
    return launch_gemm<TL>(g, T, epi, st);
  } else if (dm.k <= 4) {
    EpiFusedUp<4> epi{u1t, v2p, t1ext, perm, expert_idx, gate, a, spart, T, dm.k, dm.K, dm.r, dm.KRp, dm.d_ff};
    return launch_gemm<TL>(g, T, epi, st);
  }
  EpiFusedUp<8> epi{u1t, v2p, t1ext, perm, expert_idx, gate, a, spart, T, dm.k, dm.K, dm.r, dm.KRp, dm.d_ff};
  return launch_gemm<TL>(g, T, epi, st);
}

hipError_t launch_sreduce(const cmoe_dims& dm, int T, const int* perm, const float* spart, float* s_down,
                          hipStream_t st) {
  int kr = dm.k * dm.r;
  size_t n = (size_t)T * kr;
  hipLaunchKernelGGL(sreduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, spart, perm, T, kr,
                     (dm.d_ff + G1_BN - 1) / G1_BN, s_down);
  return hipGetLastError();
}

hipError_t launch_gemm2(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T, const int* offsets,
                        half_t* y_base_sorted, hipStream_t st) {
  using TL = TileMain;
  GemmArgs g{(const half_t*)w.w2_base, (long)dm.d * dm.d_ff, dm.d_ff, dm.d, a, dm.d_ff, nullptr, dm.d_ff, offsets,
             dm.G, (dm.d + TL::BN - 1) / TL::BN};
  EpiStore epi{y_base_sorted, dm.d, dm.d};
  return launch_gemm<TL>(g, T, epi, st);
}

hipError_t launch_combine(const cmoe_dims& dm, const half_t* u2t, const half_t* y_base_sorted, const float* s_down,
                          const int* perm, const int* offsets, const int* expert_idx, const float* gate, int T,
                          half_t* y, hipStream_t st) {
  int n_blocks32 = dm.d / 32;
  int per_wg = CB_WAVES * CB_NPW;
  int n_groups = (n_blocks32 + per_wg - 1) / per_wg;
  int m_slots = (T + 31) / 32 + dm.G;
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)(n_groups * m_slots)), dim3(CB_WAVES * 64), 0, st, u2t,
                     y_base_sorted, s_down, perm, offsets, expert_idx, gate, dm.G, dm.K, dm.k, dm.r, dm.KRp, dm.d,
                     n_groups, y);
  return hipGetLastError();
}
