// Grouped matrix-core kernels of the expert computation (Sec. 3.2):
//   t1   = V1 x                       (all experts of the token's cluster, selected rows kept)
//   Hb   = W1_base(c) x  -> fused: + U1 t1, GELU, gated sum A, s = V2 a
//   Yb   = W2_base(c) A
//   y    = Yb + sum_j g_j U2 s_j, back in token order
//
// All products are computed "weights x tokens^T": the weight rows are the A operand of
// v_mfma_f32_16x16x32_f16 (rows of the 16x16 block), the tokens are the B operand (columns).
// A lane of an accumulator block then holds ONE token (column lane % 16) and four output
// rows; with the row order of the pair blocks (cmoe_device.h) two blocks give it eight
// consecutive rows.  That is what lets the per-token quantities (experts, gates, t1) live in
// per-lane registers, and lets an accumulator pair be fed back as the B operand of the next
// product without leaving registers (its rows become the contraction index).
#include "cmoe_device.h"

#include <type_traits>

namespace {

// Tile of one workgroup: BN weight rows x BM tokens, WAVES_N x WAVES_M wavefronts, each
// owning (BN/WAVES_N) x (BM/WAVES_M) outputs as 16x16 accumulator blocks.  Operand tiles
// move global -> LDS with direct-to-LDS loads (no register staging) into NS stages of 32
// contraction elements; rows are 64 B, their four 16-B chunks XOR-swizzled with swz(row)
// so that the 16 lanes the LDS serves per cycle hit 64 distinct banks.  The
// weight rows of a tile are stored in MFMA order: tile row rho holds weight row pi_row(rho).
template <int BN_, int BM_, int WAVES_N_, int WAVES_M_, int NS_, int OCC_, bool PINGPONG_, int XSM_, int XSN_>
struct Tile {
  static constexpr int BN = BN_, BM = BM_, WAVES_N = WAVES_N_, WAVES_M = WAVES_M_, NS = NS_, OCC = OCC_;
  static constexpr bool PINGPONG = PINGPONG_;
  static constexpr int XSM = XSM_, XSN = XSN_;  // per-XCD super-tile: XSM row tiles x XSN column tiles
  static constexpr int NWAVES = WAVES_N * WAVES_M, NT = NWAVES * 64;
  static constexpr int WN = BN / WAVES_N, WM = BM / WAVES_M;
  static constexpr int NA = WN / 16, MT = WM / 16;   // 16-row blocks and 16-token blocks of a wavefront
  static constexpr int NP = WN / 32;                 // pair blocks of a wavefront
  static constexpr int BK = 32, ROWB = BK * 2;
  static constexpr int STAGE_BYTES = (BN + BM) * ROWB;
  static constexpr int SMEM_BYTES = NS * STAGE_BYTES;
  static constexpr int PER_WAVE = (BN + BM) / 16 / NWAVES;  // 1-KiB load instructions per wavefront and stage
  static_assert(BN % (32 * WAVES_N) == 0 && BM % (16 * WAVES_M) == 0, "wave tile");
  static_assert(((BN + BM) / 16) % NWAVES == 0, "load split");
  static_assert(!PINGPONG || (NWAVES == 8 && NS >= 3), "ping-pong pairs wavefront w with w + 4");
};

struct GemmArgs {
  const half_t* W;   // weights of cluster c: W + c * w_cstride, [N][ldw] row-major
  long w_cstride;
  int ldw, N;
  const half_t* X;   // token-side operand, row for sorted row p: X + (gather ? gather[p] : p) * ldx
  int ldx;
  const int* gather;
  int Kc;            // contraction length, multiple of 32
  const int* offsets;
  int G, n_tiles, m_slots, spx;
  const half_t* W2;  // optional: rows >= w_split of the weight operand come from W2 (same ldw)
  int w_split;
  int T_all;         // offsets == NULL: one group holding rows [0, T_all)
  // A launch covers the slots rel_lo <= rel < rel_hi of every XCD's range.  Slots are
  // slot_bm rows of one cluster; a tail launch (tail != 0) cuts each of its slots into
  // slot_bm / BM row tiles of a smaller tile shape.
  int slot_bm, rel_lo, rel_hi, tail;
  int x_div;         // row of X = gather[p] / x_div (several sorted rows may share one row of X); 0 = 1
  // optional per-group contraction range: group c contracts columns krange[2c] ..
  // krange[2c] + krange[2c+1] (both multiples of 32) of W and X instead of 0 .. Kc
  const int* krange;
  // elements between consecutive 32-element contraction blocks of a row of W / X; 0 = 32
  // (plain row-major rows).  An operand stored as [K / 32][rows][32] has ld = 32 and a
  // step of rows * 32: the 16 rows of one load instruction are then 1 KiB of contiguous memory.
  long kstep_w, kstep_x;
};

struct TileCtx {
  int c, n_tile, n0, m0, m_end, wn, wm, lane, tid;
  half_t* smem;
};

// One 1-KiB direct-to-LDS load: lane l's 16 bytes land at lds_byte + 16 l.
__device__ __forceinline__ void dma16(const void* g, unsigned lds_byte) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <class TL, class Epi>
__global__ __launch_bounds__(TL::NT, TL::OCC) void gemm_nt_kernel(GemmArgs g, Epi epi) {
  constexpr int SMEM = Epi::template smem_bytes<TL>();
  __shared__ __attribute__((aligned(1024))) char smem[SMEM];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // ping-pong pairs the two wavefronts of a SIMD (w, w + 4); both sets cover the tile
  const int wn = wave % TL::WAVES_N, wm = wave / TL::WAVES_N;

  // Workgroups are dealt round-robin to the 8 XCDs.  XCD x takes the contiguous range of
  // g.spx row-tile slots [x * spx, (x + 1) * spx); inside it, groups of XSM row tiles are
  // walked over the column tiles in blocks of XSN, so the workgroups resident on one XCD
  // share both operands through that XCD's L2.  With few row tiles (spx == 0) the column
  // tiles are simply dealt across the XCDs.
  int n_tile, slot, sub = 0;
  if (g.tail) {
    const int subs = g.slot_bm / TL::BM;
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    n_tile = local % g.n_tiles;
    const int rest = local / g.n_tiles;
    sub = rest % subs;
    const int rel = g.rel_lo + rest / subs;
    slot = xcd * g.spx + rel;
    if (rel >= g.rel_hi || slot >= g.m_slots) return;
  } else if (g.spx == 0) {
    n_tile = blockIdx.x % g.n_tiles;
    slot = blockIdx.x / g.n_tiles;
    if (slot >= g.m_slots) return;
  } else {
    const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
    const int per_group = TL::XSM * g.n_tiles;
    const int vg = local / per_group, rem = local % per_group;
    const int nblk = rem / (TL::XSM * TL::XSN), r2 = rem % (TL::XSM * TL::XSN);
    const int sn = min(TL::XSN, g.n_tiles - nblk * TL::XSN);
    const int rel = vg * TL::XSM + r2 / sn;
    slot = xcd * g.spx + rel;
    n_tile = nblk * TL::XSN + r2 % sn;
    if (r2 / sn >= TL::XSM || rel >= g.rel_hi || slot >= g.m_slots) return;
  }
  // which cluster and row tile the slot is: derived on the device from the cluster
  // offsets, so no host round trip sits between routing and the GEMMs
  int c = 0, m0 = 0, m_end = 0;
  if (g.offsets == nullptr) {
    m0 = slot * TL::BM;
    m_end = g.T_all;
    if (m0 >= m_end) return;
  } else {
    for (; c < g.G; ++c) {
      int lo = g.offsets[c], hi = g.offsets[c + 1];
      int tiles = (hi - lo + g.slot_bm - 1) / g.slot_bm;
      if (slot < tiles) {
        m0 = lo + slot * g.slot_bm + sub * TL::BM;
        m_end = hi;
        break;
      }
      slot -= tiles;
    }
    if (c == g.G || m0 >= m_end) return;
  }
  const int n0 = n_tile * TL::BN;
  const half_t* Wc = g.W + (size_t)c * g.w_cstride;
  const int k_lo = g.krange ? g.krange[2 * c] : 0;
  const long kstep_w = g.kstep_w ? g.kstep_w : TL::BK, kstep_x = g.kstep_x ? g.kstep_x : TL::BK;
  const unsigned smem_base = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;

  // global source of each of this wavefront's load instructions (16 tile rows x 64 B);
  // rows past the end of the matrix / cluster are clamped to the last valid row
  const half_t* gsrc[TL::PER_WAVE];
#pragma unroll
  for (int i = 0; i < TL::PER_WAVE; ++i) {
    const int ii = wave * TL::PER_WAVE + i;
    const int row = ii * 16 + (lane >> 2), pos = lane & 3;
    const int chunk = pos ^ swz(row);
    const half_t* base;
    if (row < TL::BN) {
      const int n = min(n0 + pi_row(row), g.N - 1);
      base = (g.W2 != nullptr && n >= g.w_split) ? g.W2 + (size_t)(n - g.w_split) * g.ldw : Wc + (size_t)n * g.ldw;
    } else {
      const int p = min(m0 + row - TL::BN, m_end - 1);
      base = g.X + (size_t)(g.gather ? (g.x_div > 1 ? g.gather[p] / g.x_div : g.gather[p]) : p) * g.ldx;
    }
    const long step = row < TL::BN ? kstep_w : kstep_x;
    gsrc[i] = base + chunk * 8 + (size_t)(k_lo / TL::BK) * step;
  }
  auto issue = [&](int kt, int stage) {
#pragma unroll
    for (int i = 0; i < TL::PER_WAVE; ++i)
      dma16(gsrc[i] + (size_t)kt * (((wave * TL::PER_WAVE + i) * 16 < TL::BN) ? kstep_w : kstep_x),
            smem_base + stage * TL::STAGE_BYTES + (wave * TL::PER_WAVE + i) * 1024);
  };

  float4v acc[TL::NA][TL::MT];
#pragma unroll
  for (int a = 0; a < TL::NA; ++a)
#pragma unroll
    for (int b = 0; b < TL::MT; ++b) acc[a][b] = float4v{0.f, 0.f, 0.f, 0.f};

  // fragment addresses: lane l reads row (or token) l % 16, 16-byte chunk l / 16 of the 64-byte row
  const int t16 = lane & 15, q = lane >> 4;
  int offa[TL::NA], offb[TL::MT];
#pragma unroll
  for (int a = 0; a < TL::NA; ++a) {
    const int row = wn * TL::WN + a * 16 + t16;
    offa[a] = row * TL::ROWB + ((q ^ swz(row)) << 4);
  }
#pragma unroll
  for (int b = 0; b < TL::MT; ++b) {
    const int row = TL::BN + wm * TL::WM + b * 16 + t16;
    offb[b] = row * TL::ROWB + ((q ^ swz(row)) << 4);
  }

  // 16-token blocks of this wavefront that hold at least one real token (a ragged last
  // row tile of a cluster skips the matrix-core work of the others)
  bool bv[TL::MT];
#pragma unroll
  for (int b = 0; b < TL::MT; ++b) bv[b] = m0 + wm * TL::WM + b * 16 < m_end;

  const int KT = (g.krange ? g.krange[2 * c + 1] : g.Kc) / TL::BK;
#pragma unroll
  for (int s = 0; s < TL::NS - 1; ++s)
    if (s < KT) issue(s, s);
  int stage = 0, nstage = TL::NS - 1;
  if (!TL::PINGPONG) {
    for (int kt = 0; kt < KT; ++kt) {
      // tile kt has landed (own loads), then everyone's; the stage refilled below was
      // read during iteration kt - 1, which every wavefront has left
      if (kt + TL::NS - 2 < KT) wait_vm<(TL::NS - 2) * TL::PER_WAVE>(); else wait_vm<0>();
      __builtin_amdgcn_s_barrier();
      if (kt + TL::NS - 1 < KT) issue(kt + TL::NS - 1, nstage);
      const char* sb = smem + stage * TL::STAGE_BYTES;
      half8 fa[TL::NA], fb[TL::MT];
#pragma unroll
      for (int a = 0; a < TL::NA; ++a) fa[a] = *(const half8*)(sb + offa[a]);
#pragma unroll
      for (int b = 0; b < TL::MT; ++b)
        if (bv[b]) fb[b] = *(const half8*)(sb + offb[b]);
#pragma unroll
      for (int b = 0; b < TL::MT; ++b)
        if (bv[b]) {
#pragma unroll
          for (int a = 0; a < TL::NA; ++a) acc[a][b] = mfma32(fa[a], fb[b], acc[a][b]);
        }
      stage = (stage + 1 == TL::NS) ? 0 : stage + 1;
      nstage = (nstage + 1 == TL::NS) ? 0 : nstage + 1;
    }
  } else {
    // Ping-pong: wavefronts 4..7 run one barrier interval behind wavefronts 0..3, so in
    // every interval one wavefront of each SIMD issues its MFMAs while the other reads
    // fragments from LDS and issues the next loads.  (Issuing the loads from inside the MFMA
    // phase instead, between the 16-cycle MFMAs, measured 5 % slower on the whole layer.)
    const bool set_b = wave >= 4;
    if (KT > 1) wait_vm<(TL::NS - 2) * TL::PER_WAVE>(); else wait_vm<0>();
    if (KT <= TL::NS - 2) wait_vm<0>();
    __builtin_amdgcn_s_barrier();
    if (set_b) __builtin_amdgcn_s_barrier();
    for (int kt = 0; kt < KT; ++kt) {
      const char* sb = smem + stage * TL::STAGE_BYTES;
      half8 fa[TL::NA], fb[TL::MT];
#pragma unroll
      for (int a = 0; a < TL::NA; ++a) fa[a] = *(const half8*)(sb + offa[a]);
#pragma unroll
      for (int b = 0; b < TL::MT; ++b)
        if (bv[b]) fb[b] = *(const half8*)(sb + offb[b]);
      // the stage refilled here held tile kt - 1, which both sets read before the
      // barrier that opened this interval
      if (kt + TL::NS - 1 < KT) {
        issue(kt + TL::NS - 1, nstage);
        wait_vm<(TL::NS - 2) * TL::PER_WAVE>();   // tile kt + 1 (own loads) has landed
      } else {
        wait_vm<0>();
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int b = 0; b < TL::MT; ++b)
        if (bv[b]) {
#pragma unroll
          for (int a = 0; a < TL::NA; ++a) acc[a][b] = mfma32(fa[a], fb[b], acc[a][b]);
        }
      __builtin_amdgcn_s_setprio(0);
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_barrier();
      __builtin_amdgcn_sched_barrier(0);
      stage = (stage + 1 == TL::NS) ? 0 : stage + 1;
      nstage = (nstage + 1 == TL::NS) ? 0 : nstage + 1;
    }
    if (!set_b) __builtin_amdgcn_s_barrier();
  }

  TileCtx ctx{c, n_tile, n0, m0, m_end, wn, wm, lane, tid, (half_t*)smem};
  epi.template run<TL>(ctx, acc);
}

// ---------------------------------------------------------------- epilogue: plain store
// out[p][n] = acc (f16 or f32), rows p in cluster-sorted order.  A lane writes the eight
// consecutive outputs of a pair block for its token in one piece.
template <class OutT>
struct EpiStoreT {
  OutT* out;
  const int* rowmap;  // row p of the tile order is written to out[rowmap[p]] (NULL: identity)
  int ldo, N;
  template <class TL>
  static constexpr int smem_bytes() { return TL::SMEM_BYTES; }
  template <class TL>
  __device__ void run(const TileCtx& t, float4v (&acc)[TL::NA][TL::MT]) const {
    const int t16 = t.lane & 15, q = t.lane >> 4;
#pragma unroll
    for (int b = 0; b < TL::MT; ++b) {
      const int p = t.m0 + t.wm * TL::WM + b * 16 + t16;
      if (p >= t.m_end) continue;
      const size_t orow = rowmap ? rowmap[p] : p;
#pragma unroll
      for (int P = 0; P < TL::NP; ++P) {
        const int nb = t.n0 + t.wn * TL::WN + 32 * P + 8 * q;
        if (nb >= N) continue;   // N is a multiple of 8
        if constexpr (sizeof(OutT) == 2) {
          *(half8*)(out + orow * ldo + nb) = pack_half8(acc[2 * P][b], acc[2 * P + 1][b]);
        } else {
          *(float4v*)(out + orow * ldo + nb) = acc[2 * P][b];
          *(float4v*)(out + orow * ldo + nb + 4) = acc[2 * P + 1][b];
        }
      }
    }
  }
};
using EpiStore = EpiStoreT<half_t>;

// ---------------------------------------------------------------- epilogue: down-projection + combine
// acc = (W2_base A)^T blocks.  Adds the residual of the second matrix as one more
// matrix-core contraction over the cluster's rank rows, y^T += U2cat^T sext^T with
// sext[m][e_j*r + rho] = g_j s_j[rho] (zero elsewhere, chunks of 32 rank rows that no token
// of a 16-token block needs are skipped), and writes the rows straight to token order, 16
// bytes per lane.  K*r <= 128.
struct EpiDownCombine {
  const half_t* u2t;     // [G][d][KRp]
  const float* s_down;   // [T][k][r], token order
  const int* rperm;      // token of tile row p
  const int* expert_idx;
  const float* gate;
  half_t* y;             // [T][d], token order
  int k, K, r, KRp, d;
  template <class TL>
  static constexpr int smem_bytes() {
    return 2 * (TL::BN + TL::BM) * (128 + 8) > TL::SMEM_BYTES ? 2 * (TL::BN + TL::BM) * (128 + 8) : TL::SMEM_BYTES;
  }
  template <class TL>
  __device__ void run(const TileCtx& t, float4v (&acc)[TL::NA][TL::MT]) const {
    const int t16 = t.lane & 15, q = t.lane >> 4;
    const int ldu = KRp + 8, n_chunks = KRp / 32;
    half_t* sU = t.smem;                 // [BN][ldu]  U2 rows of the tile, in MFMA order
    half_t* sS = t.smem + TL::BN * ldu;  // [BM][ldu]  expanded gated s of the tile's tokens
    const half_t* u2c = u2t + (size_t)t.c * d * KRp;
    __syncthreads();  // the stage buffers are free
    {
      constexpr int UB = 4;
      const int u_chunks = TL::BN * (KRp / 8), ucpr = KRp / 8;
      for (int base = t.tid; base < u_chunks; base += UB * TL::NT) {
        half8 tmp[UB];
#pragma unroll
        for (int i = 0; i < UB; ++i) {
          int idx = base + i * TL::NT;
          if (idx < u_chunks)
            tmp[i] = *(const half8*)(u2c + (size_t)min(t.n0 + pi_row(idx / ucpr), d - 1) * KRp + (idx % ucpr) * 8);
        }
#pragma unroll
        for (int i = 0; i < UB; ++i) {
          int idx = base + i * TL::NT;
          if (idx < u_chunks) *(half8*)(sU + (idx / ucpr) * ldu + (idx % ucpr) * 8) = tmp[i];
        }
      }
      for (int i = t.tid; i < TL::BM * ldu / 8; i += TL::NT) ((half8*)sS)[i] = half8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    __syncthreads();
    for (int idx = t.tid; idx < TL::BM * k * r; idx += TL::NT) {
      const int rho = idx % r, j = (idx / r) % k, m = idx / (r * k);
      const int p = t.m0 + m;
      if (p >= t.m_end) continue;
      const int tok = rperm[p];
      const int e = min(max(expert_idx[(size_t)tok * k + j] - t.c * K, 0), K - 1);
      sS[m * ldu + e * r + rho] = (half_t)(gate[(size_t)tok * k + j] * s_down[((size_t)tok * k + j) * r + rho]);
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < TL::MT; ++b) {
      const int ml_t = t.wm * TL::WM + b * 16 + t16;
      const int p = t.m0 + ml_t;
      const bool valid = p < t.m_end;
      const int tok = rperm[valid ? p : t.m_end - 1];
      unsigned mine = 0;
      for (int j = 0; j < k; ++j) {
        const int e = min(max(expert_idx[(size_t)tok * k + j] - t.c * K, 0), K - 1);
        const int lo = (e * r) >> 5, hi = (e * r + r - 1) >> 5;
        mine |= (0xffffffffu >> (31 - hi)) & (0xffffffffu << lo);
      }
      if (!valid) mine = 0;
      unsigned cmask = 0;
      for (int kc = 0; kc < n_chunks; ++kc)
        if (__ballot((mine >> kc) & 1u) != 0ull) cmask |= 1u << kc;
#pragma unroll
      for (int P = 0; P < TL::NP; ++P) {
        const int nl = t.wn * TL::WN + 32 * P;
        if (t.n0 + nl >= d) continue;
        for (int kc = 0; kc < n_chunks; ++kc) {
          if (!((cmask >> kc) & 1u)) continue;
          const half8 fb = *(const half8*)(sS + ml_t * ldu + kc * 32 + 8 * q);
          const half8 fa0 = *(const half8*)(sU + (nl + t16) * ldu + kc * 32 + 8 * q);
          const half8 fa1 = *(const half8*)(sU + (nl + 16 + t16) * ldu + kc * 32 + 8 * q);
          acc[2 * P][b] = mfma32(fa0, fb, acc[2 * P][b]);
          acc[2 * P + 1][b] = mfma32(fa1, fb, acc[2 * P + 1][b]);
        }
        if (valid) *(half8*)(y + (size_t)tok * d + t.n0 + nl + 8 * q) = pack_half8(acc[2 * P][b], acc[2 * P + 1][b]);
      }
    }
  }
};

// ---------------------------------------------------------------- epilogue: two-stage routing
// acc rows are the logits of all G prototypes (rows 0..G-1) and all G*K expert vectors
// (rows G..G+E-1) for the tile's tokens.  The decision is the paper's (Sec. 3.3): the
// cluster with the largest z_g (+ bias) first, then the k largest l_i among that cluster's K
// experts only, lowest index on ties, gates = softmax over the selected logits.  (All E
// expert logits are computed because one matrix-core product over the routers is cheaper
// here than K dot products per token on the vector units; the unselected clusters' logits
// are discarded.)
template <class TL>
__device__ __forceinline__ void stage_logits(const TileCtx& t, float4v (&acc)[TL::NA][TL::MT], float* lg, int LD) {
  const int t16 = t.lane & 15, q = t.lane >> 4;
#pragma unroll
  for (int b = 0; b < TL::MT; ++b) {
    const int m = t.wm * TL::WM + b * 16 + t16;
#pragma unroll
    for (int P = 0; P < TL::NP; ++P)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int n = t.wn * TL::WN + 32 * P + 8 * q;
        lg[m * LD + n + v] = acc[2 * P][b][v];
        lg[m * LD + n + 4 + v] = acc[2 * P + 1][b][v];
      }
  }
}

struct EpiRoute {
  const float* bias;
  int* cluster_id;
  int* expert_idx;
  float* gate;
  int G, K, k;
  template <class TL>
  static constexpr int smem_bytes() {
    return TL::BM * (TL::BN + 1) * 4 > TL::SMEM_BYTES ? TL::BM * (TL::BN + 1) * 4 : TL::SMEM_BYTES;
  }
  template <class TL>
  __device__ void run(const TileCtx& t, float4v (&acc)[TL::NA][TL::MT]) const {
    constexpr int LD = TL::BN + 1;
    float* lg = (float*)t.smem;  // [BM tokens][BN + 1 logits]
    __syncthreads();  // the stage buffers are free
    stage_logits<TL>(t, acc, lg, LD);
    __syncthreads();
    for (int m = t.tid; m < TL::BM; m += TL::NT) {
      const int tok = t.m0 + m;
      if (tok >= t.m_end) continue;
      const float* row = lg + m * LD;
      float best = -INFINITY;
      int c = 0;
      for (int g = 0; g < G; ++g) {
        float z = row[g] + (bias ? bias[g] : 0.f);
        if (z > best) {
          best = z;
          c = g;
        }
      }
      const float* l = row + G + c * K;
      unsigned long long taken = 0ull;  // K <= 32
      float sel[8];
      int selj[8];
      float den = 0.f;
      for (int a = 0; a < k; ++a) {
        // lowest slot not taken yet, replaced by any later slot with a larger logit: a NaN
        // never wins a comparison, so it ranks below every number and the k slots are distinct
        int bj = __ffsll((long long)~taken) - 1;
        float bl = l[bj] == l[bj] ? l[bj] : -INFINITY;
        for (int j = bj + 1; j < K; ++j)
          if (!((taken >> j) & 1ull) && l[j] > bl) {
            bl = l[j];
            bj = j;
          }
        taken |= 1ull << bj;
        sel[a] = l[bj];
        selj[a] = bj;
      }
      const float lmax = sel[0];
      for (int a = 0; a < k; ++a) {
        sel[a] = expf(sel[a] - lmax);
        den += sel[a];
      }
      cluster_id[tok] = c;
      for (int a = 0; a < k; ++a) {
        expert_idx[(size_t)tok * k + a] = c * K + selj[a];
        gate[(size_t)tok * k + a] = sel[a] / den;
      }
    }
  }
};

// The routing variants on the same accumulators: top_g clusters per token (descending
// logit, lowest index on ties), each with its own top-k experts; both softmaxes take
// logits * inv_tau; gate = w_a * softmax(l_sel * inv_tau) with w_a = p_g (scale) or p_g
// renormalised over the selected clusters.  Outputs per virtual token tok * top_g + a.
struct EpiRouteMulti {
  const float* bias;
  int* cluster_id;
  int* expert_idx;
  float* gate;
  int G, K, k, top_g;
  float inv_tau;
  int scale;
  template <class TL>
  static constexpr int smem_bytes() {
    return EpiRoute::smem_bytes<TL>();
  }
  template <class TL>
  __device__ void run(const TileCtx& t, float4v (&acc)[TL::NA][TL::MT]) const {
    constexpr int LD = TL::BN + 1;
    float* lg = (float*)t.smem;  // [BM tokens][BN + 1 logits]
    __syncthreads();  // the stage buffers are free
    stage_logits<TL>(t, acc, lg, LD);
    __syncthreads();
    for (int m = t.tid; m < TL::BM; m += TL::NT) {
      const int tok = t.m0 + m;
      if (tok >= t.m_end) continue;
      float* row = lg + m * LD;
      float zmax = -INFINITY;
      for (int g = 0; g < G; ++g) {
        row[g] += bias ? bias[g] : 0.f;
        zmax = fmaxf(zmax, row[g]);
      }
      float zden = 0.f;
      for (int g = 0; g < G; ++g) zden += expf((row[g] - zmax) * inv_tau);
      unsigned long long ctaken = 0ull;  // G <= 64
      int selc[8];
      float selp[8];
      float psum = 0.f;
      for (int a = 0; a < top_g; ++a) {
        int bg = __ffsll((long long)~ctaken) - 1;
        float bz = row[bg] == row[bg] ? row[bg] : -INFINITY;
        for (int g = bg + 1; g < G; ++g)
          if (!((ctaken >> g) & 1ull) && row[g] > bz) {
            bz = row[g];
            bg = g;
          }
        ctaken |= 1ull << bg;
        selc[a] = bg;
        selp[a] = expf((row[bg] - zmax) * inv_tau) / zden;
        psum += selp[a];
      }
      for (int a = 0; a < top_g; ++a) {
        const int c = selc[a];
        const float wa = scale ? selp[a] : selp[a] / psum;
        const float* l = row + G + c * K;
        unsigned long long taken = 0ull;  // K <= 32
        float sel[8];
        int selj[8];
        for (int b = 0; b < k; ++b) {
          int bj = __ffsll((long long)~taken) - 1;
          float bl = l[bj] == l[bj] ? l[bj] : -INFINITY;
          for (int j = bj + 1; j < K; ++j)
            if (!((taken >> j) & 1ull) && l[j] > bl) {
              bl = l[j];
              bj = j;
            }
          taken |= 1ull << bj;
          sel[b] = l[bj];
          selj[b] = bj;
        }
        const float lmax = sel[0];
        float den = 0.f;
        for (int b = 0; b < k; ++b) {
          sel[b] = expf((sel[b] - lmax) * inv_tau);
          den += sel[b];
        }
        const size_t vt = (size_t)tok * top_g + a;
        cluster_id[vt] = c;
        for (int b = 0; b < k; ++b) {
          expert_idx[vt * k + b] = c * K + selj[b];
          gate[vt * k + b] = wa * (sel[b] / den);
        }
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
  static constexpr int smem_bytes() { return TL::SMEM_BYTES; }
  template <class TL>
  __device__ void run(const TileCtx& t, float4v (&acc)[TL::NA][TL::MT]) const {
    const int t16 = t.lane & 15, q = t.lane >> 4;
#pragma unroll
    for (int b = 0; b < TL::MT; ++b) {
      const int p = t.m0 + t.wm * TL::WM + b * 16 + t16;
      if (p >= t.m_end) continue;
      const int tok = perm[p];
      for (int j = 0; j < k; ++j) {
        const int e = min(max(expert_idx[(size_t)tok * k + j] - t.c * K, 0), K - 1);
        half_t* row = t1 + ((size_t)p * k + j) * r;
#pragma unroll
        for (int P = 0; P < TL::NP; ++P) {
          const int kk = t.n0 + t.wn * TL::WN + 32 * P + 8 * q;   // 8 consecutive rank rows
          if (kk >= KRp) continue;
          if (r >= 8) {           // all of one expert
            if (kk / r == e) *(half8*)(row + (kk - e * r)) = pack_half8(acc[2 * P][b], acc[2 * P + 1][b]);
          } else {                // r == 4: two experts
            const half8 v8 = pack_half8(acc[2 * P][b], acc[2 * P + 1][b]);
            if (kk / 4 == e) *(half4*)row = half4{v8[0], v8[1], v8[2], v8[3]};
            if (kk / 4 + 1 == e) *(half4*)row = half4{v8[4], v8[5], v8[6], v8[7]};
          }
        }
      }
    }
  }
};

// ---------------------------------------------------------------- epilogue: fused up-projection
// acc = Hb^T blocks (rows n of d_ff, columns = tokens).  Per token column and selected
// expert j:  h_j = Hb + U1cat^T t1ext_j with t1ext_j the token's t1_j placed at the rank rows
// of expert e_j and zero elsewhere (matrix core, contraction over the cluster's K*r rank
// rows in chunks of 32; a chunk no token of the 16-token block needs is skipped);
// a_j = GELU(h_j); A += g_j a_j; s_j += V2 a_j by feeding the a_j pair block back as B operand
// (contraction over its 32 rows n).  The V2 product runs over "passes" of 16 rank rows; a
// lane contributes to a pass only if its token's expert lies in it.
// With STAGE the U1 / V2 panels of the tile are staged through LDS (K*r <= 128);
// otherwise they are read from global memory.
template <int R, int KMAX, bool STAGE>
struct EpiFusedUp {
  const half_t* u1t;  // [G][d_ff][KRp]
  const half_t* v2p;  // [G][KRp][d_ff]
  const half_t* t1;   // [T][k][r], sorted rows
  const int* perm;
  const int* expert_idx;
  const float* gate;
  half_t* A;          // [d_ff / 32][T][32]
  float* spart;       // [n_tiles][T][k][r] partials of V2 a over the tile's 256 rows of d_ff, FP32
  int T, k, K, KRp, d_ff;
  using FU = FusedUp<R, KMAX>;

  template <class TL>
  static constexpr int panel_bytes() {
    return (STAGE && 2 * (TL::BN * (128 + 8) + 128 * (TL::BN + 8)) > TL::SMEM_BYTES)
               ? 2 * (TL::BN * (128 + 8) + 128 * (TL::BN + 8))
               : TL::SMEM_BYTES;
  }
  // The two wavefronts that share a token block add their s partials through LDS.  With up
  // to two experts per token the partials of all token blocks are exchanged at the end, in
  // the space of the panels (no longer needed then); otherwise block by block through an
  // area of its own behind the panels.
  static constexpr bool BATCH = KMAX <= 2;
  static constexpr int XS_FLOATS = (BATCH ? 4 * KMAX * FusedUp<R, KMAX>::NSP : 1) * 4 * 64;   // per wavefront column
  template <class TL>
  static constexpr int smem_bytes() {
    static_assert(!BATCH || (TL::MT == 4 && TL::WAVES_M * XS_FLOATS * 4 <= TL::SMEM_BYTES), "exchange area");
    return panel_bytes<TL>() + (BATCH ? 0 : TL::WAVES_M * XS_FLOATS * 4);
  }

  template <class TL>
  __device__ void run(const TileCtx& t, float4v (&acc)[TL::NA][TL::MT]) const {
    static_assert(TL::BN == G1_BN && TL::WAVES_N == 2, "one s partial per tile of G1_BN rows, summed over its two wavefront columns");
    const int t16 = t.lane & 15, q = t.lane >> 4;
    const half_t* u1c = u1t + (size_t)t.c * d_ff * KRp;
    const half_t* v2c = v2p + (size_t)t.c * KRp * d_ff;
    const int n_chunks = KRp / 32, n_pass = KRp / 16;
    const int ldu = KRp + 8, ldv = TL::BN + 8;
    half_t* sU = t.smem;                 // [BN][KRp + 8], rows in MFMA order
    half_t* sV = t.smem + TL::BN * ldu;  // [KRp][BN + 8]

    // per-lane token state of every 16-token block this wavefront owns: loaded up front
    // (behind the panel staging) while it fits the registers, else block by block
    constexpr bool PRELOAD = KMAX <= 2;
    typename FU::Tok tk[PRELOAD ? TL::MT : 1];
    if (PRELOAD) {
#pragma unroll
      for (int b = 0; b < (PRELOAD ? TL::MT : 1); ++b)
        FU::load_tok(tk[b], t.m0 + t.wm * TL::WM + b * 16 + t16, t.m_end, t.c, K, k, perm, expert_idx, gate, t1, q);
    }

    if (STAGE) {
      __syncthreads();  // every wavefront has left the main loop: the stage buffers are free
      constexpr int UB = 4;
      const int u_chunks = TL::BN * (KRp / 8), ucpr = KRp / 8;
      for (int base = t.tid; base < u_chunks; base += UB * TL::NT) {
        half8 tmp[UB];
#pragma unroll
        for (int i = 0; i < UB; ++i) {
          int idx = base + i * TL::NT;
          if (idx < u_chunks) {
            int row = idx / ucpr, ch = idx % ucpr;
            tmp[i] = *(const half8*)(u1c + (size_t)min(t.n0 + pi_row(row), d_ff - 1) * KRp + ch * 8);
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

    // with few experts per token the s partials of all token blocks are kept and exchanged
    // at the end in one go; otherwise block by block
    constexpr int NSB = BATCH ? TL::MT : 1;
    float4v sacc[NSB][KMAX][FU::NSP];
    float* xs = (BATCH ? (float*)t.smem : (float*)((char*)t.smem + panel_bytes<TL>())) + t.wm * XS_FLOATS;
#pragma unroll
    for (int b = 0; b < TL::MT; ++b) {
      const int sb = BATCH ? b : 0;
#pragma unroll
      for (int j = 0; j < KMAX; ++j)
#pragma unroll
        for (int s2 = 0; s2 < FU::NSP; ++s2) sacc[sb][j][s2] = float4v{0.f, 0.f, 0.f, 0.f};
      const int p = t.m0 + t.wm * TL::WM + b * 16 + t16;
      if (!PRELOAD) FU::load_tok(tk[0], p, t.m_end, t.c, K, k, perm, expert_idx, gate, t1, q);
      const typename FU::Tok& tkb = tk[PRELOAD ? b : 0];
      typename FU::Need nd;
      FU::need_of(tkb, k, n_chunks, n_pass, nd);
#pragma unroll
      for (int P = 0; P < TL::NP; ++P) {
        const int nl = t.wn * TL::WN + 32 * P;  // first row of the pair block inside the tile
        const int nb = t.n0 + nl;
        if (nb >= d_ff) continue;
        auto uf = [&](int c, int hh) {
          return STAGE ? *(const half8*)(sU + (nl + 16 * hh + t16) * ldu + c * 32 + 8 * q)
                       : *(const half8*)(u1c + (size_t)(nb + pi_row(16 * hh + t16)) * KRp + c * 32 + 8 * q);
        };
        auto vf = [&](int pp) {
          return STAGE ? *(const half8*)(sV + (pp * 16 + t16) * ldv + nl + 8 * q)
                       : *(const half8*)(v2c + (size_t)(pp * 16 + t16) * d_ff + nb + 8 * q);
        };
        float o[8];
        FU::pair_block(acc[2 * P][b], acc[2 * P + 1][b], tkb, nd, k, q, uf, vf, o, sacc[sb]);
        // A[p][nb + 8q .. nb + 8q + 8) in 32-column blocks ([d_ff / 32][T][32], the operand
        // layout of the down-projection): 16 bytes per lane, four lanes a token's 64 bytes,
        // the block's 16 tokens 1 KiB of contiguous memory
        if (p < t.m_end) {
          half8 o8;
#pragma unroll
          for (int i = 0; i < 8; ++i) o8[i] = (half_t)o[i];
          *(half8*)(A + ((size_t)(nb >> 5) * T + p) * 32 + 8 * q) = o8;
        }
      }
      if (!BATCH) {
        // the two wavefronts that share these tokens (wn = 0, 1) add their partial s through
        // LDS, one accumulator at a time; wn = 0 stores the tile's partial
        __syncthreads();
#pragma unroll
        for (int j = 0; j < KMAX; ++j) {
          if (j >= k) continue;
#pragma unroll
          for (int s2 = 0; s2 < FU::NSP; ++s2) {
            if (t.wn == 1) {
#pragma unroll
              for (int v = 0; v < 4; ++v) xs[v * 64 + t.lane] = sacc[0][j][s2][v];
            }
            __syncthreads();
            if (t.wn == 0) {
#pragma unroll
              for (int v = 0; v < 4; ++v) sacc[0][j][s2][v] += xs[v * 64 + t.lane];
            }
            __syncthreads();
          }
        }
        if (t.wn == 0) FU::store_s(tkb, sacc[0], spart + (size_t)t.n_tile * T * k * R, k, q);
      }
    }
    if (BATCH) {
      // all token blocks at once: wn = 1 writes its partials, wn = 0 adds them and stores
      __syncthreads();
      if (t.wn == 1) {
#pragma unroll
        for (int b = 0; b < NSB; ++b)
#pragma unroll
          for (int j = 0; j < KMAX; ++j)
#pragma unroll
            for (int s2 = 0; s2 < FU::NSP; ++s2)
#pragma unroll
              for (int v = 0; v < 4; ++v) xs[(((b * KMAX + j) * FU::NSP + s2) * 4 + v) * 64 + t.lane] = sacc[b][j][s2][v];
      }
      __syncthreads();
      if (t.wn == 0) {
#pragma unroll
        for (int b = 0; b < NSB; ++b) {
#pragma unroll
          for (int j = 0; j < KMAX; ++j)
#pragma unroll
            for (int s2 = 0; s2 < FU::NSP; ++s2)
#pragma unroll
              for (int v = 0; v < 4; ++v) sacc[b][j][s2][v] += xs[(((b * KMAX + j) * FU::NSP + s2) * 4 + v) * 64 + t.lane];
          FU::store_s(tk[PRELOAD ? b : 0], sacc[b], spart + (size_t)t.n_tile * T * k * R, k, q);
        }
      }
    }
  }
};

// ---------------------------------------------------------------- s partial reduction
// s_down[perm[p]][w] = sum over row tiles of spart[tile][p][w], in a fixed order: a block
// owns 256 consecutive outputs (four per lane, k * r is a multiple of 4 so they belong to one
// token), its NW wavefronts each sum every NW-th tile, and the NW sums are added in
// wavefront order.
template <int NW, class ST>
__global__ __launch_bounds__(64 * NW) void sreduce_kernel(const ST* __restrict__ spart,
                                                          const int* __restrict__ perm, int T, int kr, int n_tiles,
                                                          float* __restrict__ s_down) {
  __shared__ float4v part[NW][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const size_t total = (size_t)T * kr;
  const size_t idx = ((size_t)blockIdx.x * 64 + lane) * 4;
  float4v sum = {0.f, 0.f, 0.f, 0.f};
  if (idx < total) {
#pragma unroll 8
    for (int nt = wave; nt < n_tiles; nt += NW) sum += *(const float4v*)(spart + (size_t)nt * total + idx);
  }
  part[wave][lane] = sum;
  __syncthreads();
  if (wave == 0 && idx < total) {
    float4v s2 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < NW; ++w) s2 += part[w][lane];
    *(float4v*)(s_down + (size_t)perm[idx / kr] * kr + idx % kr) = s2;
  }
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

// Products with at most 128 weight rows (t1 = V1 x over the cluster's rank rows): 128 x 256
// per workgroup, four wavefronts side by side along the tokens (each 128 x 64), two
// workgroups per CU.
using TileMain = Tile<128, 256, 1, 4, 3, 2, false, 8, 8>;
// The router's product (all router rows in one 128-row tile): 128-token tiles, twice the
// workgroups of TileMain for this short, x-streaming launch (64-token tiles measured slower).
using TileRoute = Tile<128, 128, 1, 4, 3, 2, false, 8, 8>;
// The two big products: 256 x 256 per workgroup, eight wavefronts (2 x 4, each 128 x 64) in
// ping-pong, one workgroup per CU: half the operand bytes per flop of the tile above.
using TileBig = Tile<256, 256, 2, 4, 4, 1, true, 4, 8>;
using TileUp = TileBig;  // tile of the fused up-projection
static_assert(TileUp::BN == G1_BN, "workspace sizing assumes one s partial per G1_BN rows");

// Leftover row tiles of the 256 x 256 schedule: 128 x 128, eight wavefronts (2 x 4, each
// 64 x 32).  Four of them replace one big tile, so a last round that would occupy a
// quarter of the CUs fills all of them.
using TileTail = Tile<128, 128, 2, 4, 4, 1, true, 1, 1>;

// TLT = void: one launch.  Otherwise, when the slots of an XCD do not fill whole rounds of
// XSM slots and the leftover would leave at least half of the CUs idle, the leftover slots
// go to a second launch with the smaller tile TLT.
template <class TL, class Epi, class TLT = void>
hipError_t launch_gemm(const GemmArgs& g, int T, const Epi& epi, hipStream_t st) {
  GemmArgs ga = g;
  ga.m_slots = (T + TL::BM - 1) / TL::BM + g.G;
  ga.slot_bm = TL::BM;
  ga.rel_lo = 0;
  ga.tail = 0;
  dim3 block(TL::NT);
  if (ga.m_slots < 32) {
    ga.spx = 0;
    ga.rel_hi = ga.m_slots;
    if constexpr (!std::is_void<TLT>::value) {
      // fewer big tiles than half the CUs: the small tile shape fills the machine better
      if (ga.m_slots * g.n_tiles <= 128) {
        ga.m_slots = (T + TLT::BM - 1) / TLT::BM + g.G;
        ga.slot_bm = TLT::BM;
        ga.rel_hi = ga.m_slots;
        ga.n_tiles = (g.N + TLT::BN - 1) / TLT::BN;
        hipLaunchKernelGGL((gemm_nt_kernel<TLT, Epi>), dim3((unsigned)(ga.m_slots * ga.n_tiles)), dim3(TLT::NT), 0, st,
                           ga, epi);
        return hipGetLastError();
      }
    }
    hipLaunchKernelGGL((gemm_nt_kernel<TL, Epi>), dim3((unsigned)(ga.m_slots * g.n_tiles)), block, 0, st, ga, epi);
    return hipGetLastError();
  }
  ga.spx = (ga.m_slots + 7) / 8;
  ga.rel_hi = ga.spx;
  int tail_slots = 0;
  if constexpr (!std::is_void<TLT>::value) {
    tail_slots = ga.spx % TL::XSM;
    // CUs of an XCD the leftover slots would occupy with the big tile: 32 per XCD
    if (tail_slots * g.n_tiles > 16 || ga.spx < TL::XSM) tail_slots = 0;
  }
  ga.rel_hi = ga.spx - tail_slots;
  const int groups = (ga.rel_hi + TL::XSM - 1) / TL::XSM;
  hipLaunchKernelGGL((gemm_nt_kernel<TL, Epi>), dim3((unsigned)(8 * groups * TL::XSM * g.n_tiles)), block, 0, st, ga,
                     epi);
  hipError_t e = hipGetLastError();
  if constexpr (!std::is_void<TLT>::value) {
    if (e == hipSuccess && tail_slots > 0) {
      GemmArgs gt = ga;
      gt.tail = 1;
      gt.rel_lo = ga.rel_hi;
      gt.rel_hi = ga.spx;
      gt.n_tiles = (g.N + TLT::BN - 1) / TLT::BN;
      const int subs = TL::BM / TLT::BM;
      hipLaunchKernelGGL((gemm_nt_kernel<TLT, Epi>), dim3((unsigned)(8 * tail_slots * subs * gt.n_tiles)),
                         dim3(TLT::NT), 0, st, gt, epi);
      e = hipGetLastError();
    }
  }
  return e;
}

template <int R, int KMAX>
hipError_t launch_gemm1_rk(const cmoe_dims& dm, const GemmArgs& g, int T, const int* perm, const int* expert_idx,
                           const float* gate, const half_t* u1t, const half_t* v2p, const half_t* t1, half_t* a,
                           float* spart, hipStream_t st) {
  using TL = TileUp;
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

hipError_t launch_t1(const cmoe_dims& dm, const half_t* x, int x_div, int T, const int* perm, const int* offsets,
                     const int* expert_idx, const half_t* v1cat, half_t* t1, hipStream_t st) {
  using TL = TileMain;
  GemmArgs g{v1cat, (long)dm.KRp * dm.d, dm.d, dm.KRp, x, dm.d, perm, dm.d, offsets, dm.G,
             (dm.KRp + TL::BN - 1) / TL::BN, 0, 0, nullptr, 0, 0};
  g.x_div = x_div;
  EpiT1 epi{t1, perm, expert_idx, dm.k, dm.K, dm.r, dm.KRp};
  return launch_gemm<TL>(g, T, epi, st);
}

// With a packed copy of the bases (per cluster W1 as [d/32][d_ff][32], then all of W2 as
// [d_ff/32][d][32]) the weight operand is read from it: row stride 32, block stride rows * 32.
static void use_packed_base(GemmArgs& g, const cmoe_dims& dm, const cmoe_weights& w, bool second) {
  if (w.packed == nullptr) return;
  const cmoe_packed_layout PL = cmoe_packed(dm);
  g.W = (const half_t*)((const char*)w.packed + (second ? PL.w2 : PL.w1));
  g.ldw = 32;
  g.kstep_w = (long)(second ? dm.d : dm.d_ff) * 32;
}

hipError_t launch_gemm1(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int x_div, int T,
                        const int* perm,
                        const int* offsets, const int* expert_idx, const float* gate, const half_t* u1t,
                        const half_t* v2p, const half_t* t1, half_t* a, float* spart, hipStream_t st) {
  using TL = TileUp;
  GemmArgs g{(const half_t*)w.w1_base, (long)dm.d_ff * dm.d, dm.d, dm.d_ff, x, dm.d, perm, dm.d, offsets, dm.G,
             (dm.d_ff + TL::BN - 1) / TL::BN, 0, 0, nullptr, 0, 0};
  g.x_div = x_div;
  use_packed_base(g, dm, w, false);
  switch (dm.r) {
    case 4: return launch_gemm1_r<4>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
    case 8: return launch_gemm1_r<8>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
    case 16: return launch_gemm1_r<16>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
    default: return launch_gemm1_r<32>(dm, g, T, perm, expert_idx, gate, u1t, v2p, t1, a, spart, st);
  }
}

hipError_t launch_sreduce(const cmoe_dims& dm, int T, const int* perm, const float* spart, int n_parts,
                          float* s_down, hipStream_t st) {
  int kr = dm.k * dm.r;
  size_t n = (size_t)T * kr;
  const dim3 grid((unsigned)((n + 255) / 256));
  if (n_parts > 128)
    hipLaunchKernelGGL((sreduce_kernel<16, float>), grid, dim3(1024), 0, st, spart, perm, T, kr, n_parts, s_down);
  else
    hipLaunchKernelGGL((sreduce_kernel<4, float>), grid, dim3(256), 0, st, spart, perm, T, kr, n_parts, s_down);
  return hipGetLastError();
}

hipError_t launch_gemm2(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T, const int* offsets,
                        const int* rowmap, half_t* y_base_sorted, hipStream_t st) {
  using TL = TileBig;
  // a is [d_ff / 32][T][32]
  GemmArgs g{(const half_t*)w.w2_base, (long)dm.d * dm.d_ff, dm.d_ff, dm.d, a, 32, nullptr, dm.d_ff, offsets,
             dm.G, (dm.d + TL::BN - 1) / TL::BN, 0, 0, nullptr, 0, 0};
  g.kstep_x = (long)T * 32;
  use_packed_base(g, dm, w, true);
  EpiStore epi{y_base_sorted, rowmap, dm.d, dm.d};
  return launch_gemm<TL, EpiStore, TileTail>(g, T, epi, st);
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

// Matrix-core router for large T (G + G*K logits per token fit one 128-row tile).
hipError_t launch_route_mfma(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int* cluster_id,
                             int* expert_idx, float* gate, hipStream_t st) {
  using TL = TileRoute;
  const int rows = dm.G + dm.G * dm.K;
  GemmArgs g{(const half_t*)w.router_cluster, 0, dm.d, rows, x, dm.d, nullptr, dm.d, nullptr, 1, 1, 0, 0,
             (const half_t*)w.router_expert, dm.G, T};
  EpiRoute epi{w.cluster_bias, cluster_id, expert_idx, gate, dm.G, dm.K, dm.k};
  GemmArgs ga = g;
  ga.m_slots = (T + TL::BM - 1) / TL::BM;
  ga.spx = 0;
  dim3 grid((unsigned)ga.m_slots), block(TL::NT);
  hipLaunchKernelGGL((gemm_nt_kernel<TL, EpiRoute>), grid, block, 0, st, ga, epi);
  return hipGetLastError();
}

// The same product with the routing variants decided in the epilogue.
hipError_t launch_route_multi_mfma(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, int top_g,
                                   float temperature, int scale, int* cluster_id, int* expert_idx, float* gate,
                                   hipStream_t st) {
  using TL = TileRoute;
  const int rows = dm.G + dm.G * dm.K;
  GemmArgs ga{(const half_t*)w.router_cluster, 0, dm.d, rows, x, dm.d, nullptr, dm.d, nullptr, 1, 1, 0, 0,
              (const half_t*)w.router_expert, dm.G, T};
  EpiRouteMulti epi{w.cluster_bias, cluster_id, expert_idx, gate, dm.G, dm.K, dm.k, top_g, 1.f / temperature, scale};
  ga.m_slots = (T + TL::BM - 1) / TL::BM;
  ga.spx = 0;
  dim3 grid((unsigned)ga.m_slots), block(TL::NT);
  hipLaunchKernelGGL((gemm_nt_kernel<TL, EpiRouteMulti>), grid, block, 0, st, ga, epi);
  return hipGetLastError();
}

// Down-projection with the residual of the second matrix and the return to token order
// fused into its epilogue (K*r <= 128).  rperm: token of each row of A.
hipError_t launch_gemm2_combine(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T,
                                const int* offsets, const int* rperm, const half_t* u2t, const float* s_down,
                                const int* expert_idx, const float* gate, half_t* y, hipStream_t st) {
  using TL = TileBig;
  GemmArgs g{(const half_t*)w.w2_base, (long)dm.d * dm.d_ff, dm.d_ff, dm.d, a, 32, nullptr, dm.d_ff, offsets,
             dm.G, (dm.d + TL::BN - 1) / TL::BN, 0, 0, nullptr, 0, 0};
  g.kstep_x = (long)T * 32;
  use_packed_base(g, dm, w, true);
  EpiDownCombine epi{u2t, s_down, rperm, expert_idx, gate, y, dm.k, dm.K, dm.r, dm.KRp, dm.d};
  return launch_gemm<TL, EpiDownCombine, TileTail>(g, T, epi, st);
}

// Grouped product with a plain store, for callers outside the forward path:
//   out[rowmap ? rowmap[p] : p][n] = sum_k X[row(p)][k_g + k] * W_g[n][k_g + k],
// W_g = W + g * w_gstride, row(p) = gather ? gather[p] / x_div : p, rows p of group g in
// [offsets[g], offsets[g+1]); k runs over [0, Kc) or over the group's krange.
hipError_t launch_gemm_plain(const half_t* W, long w_gstride, int ldw, int N, const half_t* X, int ldx,
                             const int* gather, int x_div, int Kc, const int* offsets, int n_groups, int rows,
                             const int* krange, const int* rowmap, void* out, int ldo, bool out_f32,
                             hipStream_t st, long kstep_w, long kstep_x) {
  using TL = TileBig;
  GemmArgs g{W, w_gstride, ldw, N, X, ldx, gather, Kc, offsets, n_groups, (N + TL::BN - 1) / TL::BN, 0, 0, nullptr,
             0, 0};
  g.x_div = x_div;
  g.krange = krange;
  g.kstep_w = kstep_w;
  g.kstep_x = kstep_x;
  if (N <= 64 && !out_f32) {
    // a few output columns per row (products into rank space): one 64-row weight tile, the
    // launch is bound by the stream of X rows
    using TN = Tile<64, 128, 1, 4, 4, 3, false, 8, 1>;
    g.n_tiles = 1;
    EpiStore epi{(half_t*)out, rowmap, ldo, N};
    return launch_gemm<TN, EpiStore>(g, rows, epi, st);
  }
  if (out_f32) {
    EpiStoreT<float> epi{(float*)out, rowmap, ldo, N};
    return launch_gemm<TL, EpiStoreT<float>, TileTail>(g, rows, epi, st);
  }
  EpiStore epi{(half_t*)out, rowmap, ldo, N};
  return launch_gemm<TL, EpiStore, TileTail>(g, rows, epi, st);
}

// packed[c][(k / 32) * N + n][k % 32] = base[c][n][k].  A workgroup takes 64 rows n (four
// threads per row, 16 bytes each) and walks the 32-column blocks of a quarter of K: every
// store instruction of the workgroup writes 4 KiB of contiguous memory.
__global__ __launch_bounds__(256) void pack_base_kernel(const half_t* __restrict__ base, int N, int K,
                                                        half_t* __restrict__ packed) {
  const size_t mat = (size_t)N * K;
  const int n = blockIdx.x * 64 + (threadIdx.x >> 2), c8 = (threadIdx.x & 3) * 8;
  if (n >= N) return;
  const half_t* src = base + blockIdx.z * mat + (size_t)n * K + c8;
  half_t* dst = packed + blockIdx.z * mat + (size_t)n * 32 + c8;
  const int nb = K / 32, per = (nb + 3) / 4, b0 = blockIdx.y * per, b1 = min(nb, b0 + per);
#pragma unroll 4
  for (int kb = b0; kb < b1; ++kb) *(half8*)(dst + (size_t)kb * N * 32) = *(const half8*)(src + kb * 32);
}

hipError_t launch_pack_bases(const cmoe_dims& dm, const cmoe_weights& w, half_t* packed, hipStream_t st) {
  const cmoe_packed_layout PL = cmoe_packed(dm);
  char* pk = (char*)packed;
  hipLaunchKernelGGL(pack_base_kernel, dim3((dm.d_ff + 63) / 64, 4, dm.G), dim3(256), 0, st, (const half_t*)w.w1_base,
                     dm.d_ff, dm.d, (half_t*)(pk + PL.w1));
  hipLaunchKernelGGL(pack_base_kernel, dim3((dm.d + 63) / 64, 4, dm.G), dim3(256), 0, st, (const half_t*)w.w2_base,
                     dm.d, dm.d_ff, (half_t*)(pk + PL.w2));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  // the FP16 panels of all clusters' factors (Sec. 3.4: INT4 is the stored form; the panels are
  // what the matrix cores read)
  return launch_dequant_ffn(dm, w, nullptr, (half_t*)(pk + PL.v1cat), (half_t*)(pk + PL.u1t), (half_t*)(pk + PL.v2p),
                            (half_t*)(pk + PL.u2t), st);
}
