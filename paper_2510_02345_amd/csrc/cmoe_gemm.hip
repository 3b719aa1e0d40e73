// Grouped matrix-core kernels of the expert computation (Sec. 3.2):
//   t1   = V1 x                       (all experts of the token's cluster, selected rows kept)
//   Hb   = W1_base(c) x  -> fused: + U1 t1, GELU, gated sum A, s = V2 a
//   Yb   = W2_base(c) A
//   y    = Yb + sum_j g_j U2 s_j, back in token order
//
// All products are computed "weights x tokens^T": the weight rows are the A operand of
// v_mfma_f32_32x32x16_f16 (rows n of the 32x32 block), the tokens are the B operand
// (columns m).  A lane of a 32x32 accumulator block then holds ONE token (column
// m = lane % 32) and 16 output rows n = 8*(v/4) + 4*(lane/32) + v%4, v = 0..15.  That is
// what lets the per-token quantities (experts, gates, t1) live in per-lane registers, and
// lets an accumulator block be fed back as the B operand of the next product without
// leaving registers (its rows become the contraction index).
#include "cmoe_internal.h"

namespace {

template <int BN_, int BM_, int WAVES_N_, int WAVES_M_, int OCC_>
struct Tile {
  static constexpr int BN = BN_, BM = BM_, WAVES_N = WAVES_N_, WAVES_M = WAVES_M_, OCC = OCC_;
  static constexpr int NT = WAVES_N * WAVES_M * 64;
  static constexpr int WN = BN / WAVES_N, WM = BM / WAVES_M;
  static constexpr int NB = WN / 32, MB = WM / 32;
  static constexpr int BK = 64;        // contraction elements per LDS stage
  static constexpr int LDK = BK + 8;   // padded LDS row (halfs): 144 B, conflict-free b128 reads
  static constexpr int WCH = BN * (BK / 8) / NT, XCH = BM * (BK / 8) / NT;  // 16-B chunks per thread
  static constexpr int SMEM_HALFS = (BN + BM) * LDK;
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

// GELU(u) = u * Phi(u), Phi by the erf form.  erf(z), z = |u|/sqrt(2), is evaluated with
// the classical five-term rational-exponential formula 1 - (a1 t + ... + a5 t^5) exp(-z^2),
// t = 1/(1 + p z) (absolute error below 1.5e-7), using the hardware exp2 and reciprocal.
__device__ __forceinline__ float gelu_erf(float u) {
  const float z = fabsf(u) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  float poly = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);
  poly = fmaf(t, poly, 0.5f * 1.421413741f);
  poly = fmaf(t, poly, 0.5f * -0.284496736f);
  poly = fmaf(t, poly, 0.5f * 0.254829592f);
  const float ex = __builtin_amdgcn_exp2f(u * u * -0.72134752044448170f);  // exp(-u^2/2)
  const float q = poly * t * ex;                                          // (1 - erf(z)) / 2
  return u * (u > 0.f ? 1.0f - q : q);
}

template <class TL, class Epi>
__global__ __launch_bounds__(TL::NT, TL::OCC) void gemm_nt_kernel(GemmArgs g, Epi epi) {
  __shared__ __attribute__((aligned(16))) half_t smem[Epi::template smem_halfs<TL>()];
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

  half_t* sW = smem;                        // [BN][LDK]
  half_t* sX = smem + TL::BN * TL::LDK;     // [BM][LDK]
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

  const int frag_row = lane & 31, frag_col = (lane >> 5) * 8;
  const half_t* cw = sW + (wn * TL::WN + frag_row) * TL::LDK + frag_col;
  const half_t* cx = sX + (wm * TL::WM + frag_row) * TL::LDK + frag_col;
  for (int kt = 0; kt < KT; ++kt) {
#pragma unroll
    for (int i = 0; i < TL::WCH; ++i) *(half8*)(sW + lw[i]) = rw[i];
#pragma unroll
    for (int i = 0; i < TL::XCH; ++i) *(half8*)(sX + lx[i]) = rx[i];
    __syncthreads();
    if (kt + 1 < KT) {
#pragma unroll
      for (int i = 0; i < TL::WCH; ++i) rw[i] = *(const half8*)(gw[i] + (size_t)(kt + 1) * TL::BK);
#pragma unroll
      for (int i = 0; i < TL::XCH; ++i) rx[i] = *(const half8*)(gx[i] + (size_t)(kt + 1) * TL::BK);
    }
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
  static constexpr int smem_halfs() { return TL::SMEM_HALFS; }
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

// ---------------------------------------------------------------- epilogue: t1 = V1_{e_j} x
// acc rows are kk = j_local * r + rho over ALL experts of the cluster; for the token's
// j-th selected expert only its r rows are kept:  t1[p][j][rho] = acc[(e_j - c*K)*r + rho].
struct EpiT1 {
  half_t* t1;  // [T][k][r], sorted rows
  const int* perm;
  const int* expert_idx;
  int k, K, r, KRp;
  template <class TL>
  static constexpr int smem_halfs() { return TL::SMEM_HALFS; }
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
        half_t* row = t1 + ((size_t)p * k + j) * r;
#pragma unroll
        for (int a = 0; a < TL::NB; ++a) {
          int nb = t.n0 + t.wn * TL::WN + a * 32;
          if (nb >= KRp) continue;
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            int kk = nb + 8 * qd + 4 * h;  // 4 consecutive rank rows, all of one expert (r % 4 == 0)
            if (kk / r == e) *(half4*)(row + (kk - e * r)) = to_half4(acc[a][b], qd);
          }
        }
      }
    }
  }
};

// ---------------------------------------------------------------- epilogue: fused up-projection
// acc = Hb^T block (rows n of d_ff, columns = tokens).  Per token column and selected
// expert j:  h_j = Hb + U1cat^T t1ext_j with t1ext_j the token's t1_j placed at the rank rows
// of expert e_j and zero elsewhere (matrix core, contraction over the cluster's K*r rank
// rows in chunks of 16; a chunk no token of the 32-column block needs is skipped);
// a_j = GELU(h_j); A += g_j a_j; s_j += V2 a_j by feeding the a_j block back as B operand
// (contraction over the block's 32 rows n).  The V2 product runs over "passes" of 32 rank
// rows (32/r experts); a lane contributes to a pass only if its token's expert lies in
// it, so after all passes row (e_j % (32/r))*r + rho of the accumulator holds s_j[rho].
// With STAGE the U1 / V2 panels of the tile are staged through LDS (K*r <= 128);
// otherwise they are read from global memory.
template <int R, int KMAX, bool STAGE>
struct EpiFusedUp {
  const half_t* u1t;  // [G][d_ff][KRp]
  const half_t* v2p;  // [G][KRp][d_ff], columns permuted inside 16-groups
  const half_t* t1;   // [T][k][r], sorted rows
  const int* perm;
  const int* expert_idx;
  const float* gate;
  half_t* A;          // [T][d_ff]
  float* spart;       // [n_tiles][T][k][r]
  int T, k, K, KRp, d_ff;

  static constexpr int EPB = 32 / R;  // experts per 32 rank rows
  static constexpr int NF = (R == 32) ? 2 : 1;

  template <class TL>
  static constexpr int smem_halfs() {
    return STAGE ? (TL::SMEM_HALFS > TL::BN * (128 + 8) + 128 * (TL::BN + 8) ? TL::SMEM_HALFS
                                                                            : TL::BN * (128 + 8) + 128 * (TL::BN + 8))
                 : TL::SMEM_HALFS;
  }

  __device__ static __forceinline__ bool chunk_has(int e, int kc) {
    return R == 32 ? (e == (kc >> 1)) : R == 16 ? (e == kc) : R == 8 ? ((e >> 1) == kc) : ((e >> 2) == kc);
  }
  // B operand of chunk kc for a lane whose token selected expert e with t1 fragments f
  __device__ static __forceinline__ half8 t1_frag(int e, int kc, int h, const half8 (&f)[NF]) {
    const half8 z = {0, 0, 0, 0, 0, 0, 0, 0};
    if (R == 32) return (e == (kc >> 1)) ? ((kc & 1) ? f[NF - 1] : f[0]) : z;
    if (R == 16) return (e == kc) ? f[0] : z;
    if (R == 8) return (e == 2 * kc + h) ? f[0] : z;
    half8 o = z;  // R == 4: slots 0..3 are expert 4kc+2h, slots 4..7 expert 4kc+2h+1
    if (e == 4 * kc + 2 * h) {
      o[0] = f[0][0]; o[1] = f[0][1]; o[2] = f[0][2]; o[3] = f[0][3];
    } else if (e == 4 * kc + 2 * h + 1) {
      o[4] = f[0][0]; o[5] = f[0][1]; o[6] = f[0][2]; o[7] = f[0][3];
    }
    return o;
  }

  template <class TL>
  __device__ void run(const TileCtx& t, float16v (&acc)[TL::NB][TL::MB]) const {
    static_assert(TL::WAVES_N == 1, "one wavefront spans the tile's rows n, so s needs no cross-wave sum");
    const int h = t.lane >> 5, ml = t.lane & 31;
    const half_t* u1c = u1t + (size_t)t.c * d_ff * KRp;
    const half_t* v2c = v2p + (size_t)t.c * KRp * d_ff;
    const int n_chunks = KRp / 16, n_pass = KRp / 32;
    const int ldu = KRp + 8, ldv = TL::BN + 8;
    half_t* sU = t.smem;                 // [BN][KRp + 8]
    half_t* sV = t.smem + TL::BN * ldu;  // [KRp][BN + 8]

    // per-lane token state of every 32-column block this wavefront owns
    int e[TL::MB][KMAX];
    float gj[TL::MB][KMAX];
    half8 f[TL::MB][KMAX][NF];
    int pp[TL::MB];
    bool valid[TL::MB];
#pragma unroll
    for (int b = 0; b < TL::MB; ++b) {
      pp[b] = t.m0 + t.wm * TL::WM + b * 32 + ml;
      valid[b] = pp[b] < t.m_end;
      const int pc = valid[b] ? pp[b] : t.m_end - 1;
      const int tok = perm[pc];
#pragma unroll
      for (int j = 0; j < KMAX; ++j) {
        e[b][j] = 0;
        gj[b][j] = 0.f;
#pragma unroll
        for (int i = 0; i < NF; ++i) f[b][j][i] = half8{0, 0, 0, 0, 0, 0, 0, 0};
        if (j < k) {
          e[b][j] = min(max(expert_idx[(size_t)tok * k + j] - t.c * K, 0), K - 1);
          gj[b][j] = valid[b] ? gate[(size_t)tok * k + j] : 0.f;
          const half_t* tr = t1 + ((size_t)pc * k + j) * R;
          if (R == 32) {
            f[b][j][0] = *(const half8*)(tr + 8 * h);
            f[b][j][NF - 1] = *(const half8*)(tr + 16 + 8 * h);
          } else if (R == 16) {
            f[b][j][0] = *(const half8*)(tr + 8 * h);
          } else if (R == 8) {
            f[b][j][0] = *(const half8*)(tr);
          } else {
            half4 q4 = *(const half4*)(tr);
            f[b][j][0][0] = q4[0]; f[b][j][0][1] = q4[1]; f[b][j][0][2] = q4[2]; f[b][j][0][3] = q4[3];
          }
        }
      }
    }

    if (STAGE) {
      // the main loop ended on a barrier: the tile buffers are free
      constexpr int UB = 4;
      const int u_chunks = TL::BN * (KRp / 8), ucpr = KRp / 8;
      for (int base = t.tid; base < u_chunks; base += UB * TL::NT) {
        half8 tmp[UB];
#pragma unroll
        for (int i = 0; i < UB; ++i) {
          int idx = base + i * TL::NT;
          if (idx < u_chunks) {
            int row = idx / ucpr, ch = idx % ucpr;
            tmp[i] = *(const half8*)(u1c + (size_t)min(t.n0 + row, d_ff - 1) * KRp + ch * 8);
          }
        }
#pragma unroll
        for (int i = 0; i < UB; ++i) {
          int idx = base + i * TL::NT;
          if (idx < u_chunks) *(half8*)(sU + (idx / ucpr) * ldu + (idx % ucpr) * 8) = tmp[i];
        }
      }
      const int v_chunks = KRp * (TL::BN / 8), vcpr = TL::BN / 8;
      for (int base = t.tid; base < v_chunks; base += UB * TL::NT) {
        half8 tmp[UB];
#pragma unroll
        for (int i = 0; i < UB; ++i) {
          int idx = base + i * TL::NT;
          if (idx < v_chunks) {
            int row = idx / vcpr, ch = idx % vcpr;
            tmp[i] = *(const half8*)(v2c + (size_t)row * d_ff + min(t.n0 + ch * 8, d_ff - 8));
          }
        }
#pragma unroll
        for (int i = 0; i < UB; ++i) {
          int idx = base + i * TL::NT;
          if (idx < v_chunks) *(half8*)(sV + (idx / vcpr) * ldv + (idx % vcpr) * 8) = tmp[i];
        }
      }
      __syncthreads();
    }

#pragma unroll
    for (int b = 0; b < TL::MB; ++b) {
      float16v sacc[KMAX];
#pragma unroll
      for (int j = 0; j < KMAX; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[j][v] = 0.f;
#pragma unroll
      for (int a = 0; a < TL::NB; ++a) {
        const int nb = t.n0 + a * 32;
        if (nb >= d_ff) continue;
        float16v o;
#pragma unroll
        for (int v = 0; v < 16; ++v) o[v] = 0.f;
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
          if (j >= k) continue;
          const int ej = e[b][j];
          float16v hj = acc[a][b];
          for (int kc = 0; kc < n_chunks; ++kc) {
            if (__ballot(valid[b] && chunk_has(ej, kc)) == 0ull) continue;
            half8 fa = STAGE ? *(const half8*)(sU + (a * 32 + ml) * ldu + kc * 16 + 8 * h)
                             : *(const half8*)(u1c + (size_t)(nb + ml) * KRp + kc * 16 + 8 * h);
            hj = mfma16(fa, t1_frag(ej, kc, h, f[b][j]), hj);
          }
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            hj[v] = gelu_erf(hj[v]);
            o[v] = fmaf(gj[b][j], hj[v], o[v]);
          }
          for (int q = 0; q < n_pass; ++q) {
            const bool on = valid[b] && (ej / EPB == q);
            if (__ballot(on) == 0ull) continue;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
              half8 fb;
#pragma unroll
              for (int i = 0; i < 8; ++i) fb[i] = on ? (half_t)hj[8 * s + i] : (half_t)0.f;
              half8 fa = STAGE ? *(const half8*)(sV + (q * 32 + ml) * ldv + a * 32 + 16 * s + 8 * h)
                               : *(const half8*)(v2c + (size_t)(q * 32 + ml) * d_ff + nb + 16 * s + 8 * h);
              sacc[j] = mfma16(fa, fb, sacc[j]);
            }
          }
        }
        if (valid[b]) {
#pragma unroll
          for (int qd = 0; qd < 4; ++qd)
            *(half4*)(A + (size_t)pp[b] * d_ff + nb + 8 * qd + 4 * h) = to_half4(o, qd);
        }
      }
      // partial s of this column tile: the lane holds rows 8*qd + 4h + (0..3) of the pass
      // accumulator; those inside [b_e*R, b_e*R + R) are the token's s_j
      if (valid[b]) {
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
          if (j >= k) continue;
          const int be = (e[b][j] % EPB) * R;
          float* dst = spart + (((size_t)t.n_tile * T + pp[b]) * k + j) * R;
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            int row0 = 8 * qd + 4 * h;
            if (row0 >= be && row0 < be + R) {
              float4v v4 = {sacc[j][4 * qd], sacc[j][4 * qd + 1], sacc[j][4 * qd + 2], sacc[j][4 * qd + 3]};
              *(float4v*)(dst + row0 - be) = v4;
            }
          }
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

// 128 weight rows x 256 tokens per workgroup, four wavefronts side by side along the
// tokens (each 128 x 64), two workgroups per CU so that one's epilogue overlaps the
// other's main loop.
using TileMain = Tile<128, 256, 1, 4, 2>;
static_assert(TileMain::BN == G1_BN, "workspace sizing assumes this column tile");

template <class TL, class Epi>
hipError_t launch_gemm(const GemmArgs& g, int T, const Epi& epi, hipStream_t st) {
  int m_slots = (T + TL::BM - 1) / TL::BM + g.G;
  dim3 grid((unsigned)(g.n_tiles * m_slots)), block(TL::NT);
  hipLaunchKernelGGL((gemm_nt_kernel<TL, Epi>), grid, block, 0, st, g, epi);
  return hipGetLastError();
}

template <int R, int KMAX>
hipError_t launch_gemm1_rk(const cmoe_dims& dm, const GemmArgs& g, int T, const int* perm, const int* expert_idx,
                           const float* gate, const half_t* u1t, const half_t* v2p, const half_t* t1, half_t* a,
                           float* spart, hipStream_t st) {
  using TL = TileMain;
  if (dm.KRp <= 128) {
    EpiFusedUp<R, KMAX, true> epi{u1t, v2p, t1, perm, expert_idx, gate, a, spart, T, dm.k, dm.K, dm.KRp, dm.d_ff};
    return launch_gemm<TL>(g, T, epi, st);
  }
  EpiFusedUp<R, KMAX, false> epi{u1t, v2p, t1, perm, expert_idx, gate, a, spart, T, dm.k, dm.K, dm.KRp, dm.d_ff};
  return launch_gemm<TL>(g, T, epi, st);
}

template <int R>
hipError_t launch_gemm1_r(const cmoe_dims& dm, const GemmArgs& g, int T, const int* perm, const int* expert_idx,
                          const float* gate, const half_t* u1t, const half_t* v2p, const half_t* t1, half_t* a,
                          float* spart, hipStream_t st) {
  if (dm.k <= 1) return launch_gemm1_rk<R, 1>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
  if (dm.k <= 2) return launch_gemm1_rk<R, 2>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
  if (dm.k <= 4) return launch_gemm1_rk<R, 4>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
  return launch_gemm1_rk<R, 8>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
}

}  // namespace

hipError_t launch_t1(const cmoe_dims& dm, const half_t* x, int T, const int* perm, const int* offsets,
                     const int* expert_idx, const half_t* v1cat, half_t* t1, hipStream_t st) {
  using TL = TileMain;
  GemmArgs g{v1cat, (long)dm.KRp * dm.d, dm.d, dm.KRp, x, dm.d, perm, dm.d, offsets, dm.G,
             (dm.KRp + TL::BN - 1) / TL::BN};
  EpiT1 epi{t1, perm, expert_idx, dm.k, dm.K, dm.r, dm.KRp};
  return launch_gemm<TL>(g, T, epi, st);
}

hipError_t launch_gemm1(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, const int* perm,
                        const int* offsets, const int* expert_idx, const float* gate, const half_t* u1t,
                        const half_t* v2p, const half_t* t1, half_t* a, float* spart, hipStream_t st) {
  using TL = TileMain;
  GemmArgs g{(const half_t*)w.w1_base, (long)dm.d_ff * dm.d, dm.d, dm.d_ff, x, dm.d, perm, dm.d, offsets, dm.G,
             (dm.d_ff + TL::BN - 1) / TL::BN};
  switch (dm.r) {
    case 4: return launch_gemm1_r<4>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
    case 8: return launch_gemm1_r<8>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
    case 16: return launch_gemm1_r<16>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
    default: return launch_gemm1_r<32>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
  }
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
