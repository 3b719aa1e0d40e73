// Weight-streaming path of the expert computation for small token counts (Sec. 3.2).
// With only a handful of tokens per cluster the layer is bound by reading every base
// matrix once from HBM, so the two shared-base products are pure streams: a workgroup owns
// 32 weight rows of one cluster and 16 of its tokens, its four wavefronts split the
// contraction dimension, and both operands travel global -> LDS by DMA into per-wavefront
// rings.  The per-expert rank-r terms (INT4 factors dequantised on the fly, Sec. 3.4) are
// small kernels of their own or ride along in the stream launches.
#include "cmoe_device.h"

namespace {

__device__ __forceinline__ float nib_lo(unsigned b) { return (float)((int)(b << 28) >> 28); }
__device__ __forceinline__ float nib_hi(unsigned b) { return (float)((int)(b << 24) >> 28); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

constexpr int SK_ROWS = 32;   // weight rows per workgroup
constexpr int SK_RB = SK_ROWS / 32;  // 32-row blocks per workgroup
constexpr int SK_OCC = 3;     // workgroups per CU the LDS budget is sized for
constexpr int SK_WAVES = 4;   // wavefronts splitting the contraction

// One 1-KiB direct-to-LDS load: lane l's 16 bytes land at lds_byte + 16 l.
__device__ __forceinline__ void dma16(const void* g, unsigned lds_byte) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte) : "memory");
}
// The same with the non-temporal hint: the line is not kept in the caches behind the load.
// For a matrix that is read once per call and is larger than the last-level cache this is
// worth 9 % of the whole weight-streaming path (the two base streams go from 6.0 to 6.5-6.7
// TB/s, and the router, whose rows and tokens are no longer evicted, gets faster too).
__device__ __forceinline__ void dma16_nt(const void* g, unsigned lds_byte) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt" ::"v"(g), "s"(lds_byte) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

constexpr int SK_COLS = 16;                         // tokens per pass over a cluster (layer path)
constexpr int SK_A_BYTES = SK_ROWS * 128;           // weight rows x 64 elements
// Ring geometry of one wavefront for COLS token rows per pass (16, or 32 when the caller
// has more than 16 rows per group: all 32 accumulator columns are then distinct).
template <int COLS>
struct SkRing {
  static constexpr int B_BYTES = COLS * 128;            // token rows x 64 elements
  static constexpr int STAGE = SK_A_BYTES + B_BYTES;    // one wavefront stage
  static constexpr int RING = 2 * STAGE;                // two stages per wavefront
  static constexpr int DMA = (SK_ROWS + COLS) / 8;      // 1-KiB loads per stage (8 rows x 128 B each)
  static constexpr int OCC = COLS == 16 ? SK_OCC : 2;   // workgroups per CU that fit the LDS
};

// acc[rb] += sum_k W[row(rb)][k] X[col][k] over the 64-element steps [it0, it1) of this
// wavefront.  Both operands stream global -> LDS one step ahead of the matrix-core work,
// as whole 128-byte lines per row, into a two-stage ring private to the wavefront (so no
// barrier is needed, only vmcnt), chunks XOR-swizzled with (row >> 1) & 7.
//   wrow / brow: the lane's row (lane / 8) of the first 8-row group of the weight / token
//                tile at step 0, WITHOUT the chunk offset (the swizzle depends on the row);
//                w_stride: elements between 8-row groups; brow[i]: the lane's row of token
//                row group i (rows beyond the pass are clamped by the caller)
//   w_blk:       elements between consecutive 32-element contraction blocks of a weight row:
//                32 for row-major rows, rows * 32 for a matrix stored as [K / 32][rows][32]
//                (the re-tiled copy of the bases); a step of 64 elements is two blocks
// With COLS = 16 accumulator columns 16..31 repeat columns 0..15.  NT: weight loads carry the
// non-temporal hint (the token rows never do: they are re-read by every row block).
template <int COLS, bool NT>
__device__ __forceinline__ void skinny_stream(const half_t* wrow, size_t w_stride, size_t w_blk,
                                              const half_t* const (&brow)[COLS / 8], char* ring, unsigned ring_lds,
                                              int lane, int it0, int it1, float16v (&acc)[SK_RB]) {
  using RG = SkRing<COLS>;
  if (it0 >= it1) return;
  const int fr = lane & 31, h = lane >> 5;
  int offa[SK_RB][4], offb[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
#pragma unroll
    for (int rb = 0; rb < SK_RB; ++rb) {
      const int row = rb * 32 + fr;
      offa[rb][s] = row * 128 + (((2 * s + h) ^ ((row >> 1) & 7)) << 4);
    }
    const int br = fr & (COLS - 1);
    offb[s] = SK_A_BYTES + br * 128 + (((2 * s + h) ^ ((br >> 1) & 7)) << 4);
  }
  // lane l of load i fills row 8i + l/8, chunk position l%8, with source chunk position ^ swizzle(row)
  const int lrow = lane >> 3, lpos = lane & 7;
  const int c0 = (lpos ^ (lrow >> 1)) << 3, c1 = (lpos ^ (lrow >> 1) ^ 4) << 3;  // even / odd groups
  // the same chunks of the weight rows: chunk c = block c / 4 of the step, 8 (c % 4) elements into it
  const size_t wc0 = (size_t)(c0 >> 5) * w_blk + (c0 & 31), wc1 = (size_t)(c1 >> 5) * w_blk + (c1 & 31);
  const size_t w_step = 2 * w_blk;
  auto issue = [&](int it, int stage) {
    const unsigned dst = ring_lds + stage * RG::STAGE;
#pragma unroll
    for (int i = 0; i < SK_ROWS / 8; ++i) {
      const half_t* src = wrow + ((i & 1) ? wc1 : wc0) + (size_t)i * w_stride + (size_t)it * w_step;
      if (NT) dma16_nt(src, dst + i * 1024); else dma16(src, dst + i * 1024);
    }
#pragma unroll
    for (int i = 0; i < COLS / 8; ++i)
      dma16(brow[i] + ((i & 1) ? c1 : c0) + (size_t)it * 64, dst + SK_A_BYTES + i * 1024);
  };
  auto compute = [&](int stage) {
    const char* sb = ring + stage * RG::STAGE;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      half8 fa[SK_RB];
#pragma unroll
      for (int rb = 0; rb < SK_RB; ++rb) fa[rb] = *(const half8*)(sb + offa[rb][s]);
      const half8 fb = *(const half8*)(sb + offb[s]);
#pragma unroll
      for (int rb = 0; rb < SK_RB; ++rb) acc[rb] = mfma16(fa[rb], fb, acc[rb]);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // the stage has been read: it may be refilled
  };
  issue(it0, 0);
  for (int it = it0; it < it1; it += 2) {
    if (it + 1 < it1) {
      issue(it + 1, 1);
      wait_vm<RG::DMA>();
    } else {
      wait_vm<0>();
    }
    compute(0);
    if (it + 1 < it1) {
      if (it + 2 < it1) {
        issue(it + 2, 0);
        wait_vm<RG::DMA>();
      } else {
        wait_vm<0>();
      }
      compute(1);
    }
  }
}

// Sum of the four wavefronts' partial accumulators through LDS; wavefront w < SK_RB returns
// with block w in hb.  red: [SK_WAVES][SK_RB][16][64] floats.
__device__ __forceinline__ void skinny_reduce(float* red, int wave, int lane, const float16v (&acc)[SK_RB],
                                              float16v& hb) {
#pragma unroll
  for (int rb = 0; rb < SK_RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) red[((wave * SK_RB + rb) * 16 + v) * 64 + lane] = acc[rb][v];
  __syncthreads();
  if (wave < SK_RB) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < SK_WAVES; ++w) s += red[((w * SK_RB + wave) * 16 + v) * 64 + lane];
      hb[v] = s;
    }
  }
}

struct SkinnyTile {
  int c, n0, m0, m_end;
};
// Stream workgroup `id` of a launch of nx row blocks x G clusters x passes (row block
// fastest); a pass covers `cols` tokens of the cluster, m_end is the end of the pass.
__device__ __forceinline__ bool skinny_tile(const int* offsets, int id, int nx, int G, int cols, SkinnyTile& t) {
  int xb = id % nx;
  const int yz = id / nx;
  t.c = yz % G;
  const int pass = yz / G;
  // Workgroups are dealt round-robin to the 8 XCDs.  The INT4 factor rows are 128-byte
  // lines shared by 8 neighbouring row blocks, so inside every run of 64 blocks the 8
  // workgroups that land on one XCD take 8 neighbouring row blocks: each line is then
  // fetched into one L2 instead of eight.  (The caller keeps id congruent to the dispatch
  // index modulo 8.)
  if ((nx & 7) == 0 && xb < (nx & ~63)) xb = (xb & ~63) + ((xb & 7) << 3) + ((xb >> 3) & 7);
  t.n0 = xb * SK_ROWS;
  const int lo = offsets[t.c], hi = offsets[t.c + 1];
  t.m0 = lo + pass * cols;
  t.m_end = min(hi, t.m0 + cols);
  return t.m0 < hi;
}

// ---------------------------------------------------------------- t1 = V1_e x
// t1[p][j][:] for sorted row p and its selected expert j, by the calling workgroup: a
// wavefront per rank row, INT4 codes dequantised on the fly (Sec. 3.4).
__device__ __forceinline__ void skinny_t1_job(int p, int j, const half_t* __restrict__ x,
                                              const int* __restrict__ perm, const int* __restrict__ expert_idx,
                                              const uint8_t* __restrict__ v1_q, const half_t* __restrict__ v1_s,
                                              int d, int q, int r, int k, int x_div, int n_exp,
                                              half_t* __restrict__ t1) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  const int tok = perm[p];
  const int e = min(max(expert_idx[(size_t)tok * k + j], 0), n_exp - 1);
  const half_t* xr = x + (size_t)(tok / x_div) * d;
  for (int rho = wave; rho < r; rho += nw) {
    const size_t row = (size_t)e * r + rho;
    const uint8_t* qr = v1_q + row * (d / 2);
    const half_t* sr = v1_s + row * (d / q);
    float acc = 0.f;
    for (int ch0 = lane; ch0 < d / 8; ch0 += 256) {   // 8 elements per chunk: 4 code bytes, one scale
      unsigned bytes[4];
      half8 xv[4];
      float sc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int ch = ch0 + 64 * u;
        const bool in = ch < d / 8;
        bytes[u] = in ? *(const unsigned*)(qr + ch * 4) : 0u;
        xv[u] = in ? *(const half8*)(xr + ch * 8) : half8{0, 0, 0, 0, 0, 0, 0, 0};
        sc[u] = in ? (float)sr[(ch * 8) / q] : 0.f;
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        float part = 0.f;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned b = (bytes[u] >> (8 * i)) & 0xffu;
          part = fmaf(nib_lo(b), (float)xv[u][2 * i], part);
          part = fmaf(nib_hi(b), (float)xv[u][2 * i + 1], part);
        }
        acc = fmaf(sc[u], part, acc);
      }
    }
    acc = wave_sum(acc);
    if (lane == 0) t1[((size_t)p * k + j) * r + rho] = (half_t)acc;
  }
}

// ---------------------------------------------------------------- residual-down
// ures[p][n] = sum_j g_j sum_rho U2_{e_j}[rho][n] s_j[rho] for sorted row p and a chunk of
// 2048 output columns, s_j summed here from its n_parts partials in fixed order.
__device__ __forceinline__ void skinny_ures_job(int p, int chunk, const int* __restrict__ perm,
                                                const int* __restrict__ expert_idx, const float* __restrict__ gate,
                                                const uint8_t* __restrict__ u2_q, const half_t* __restrict__ u2_s,
                                                const float* __restrict__ spart, int n_parts, int T, int d, int q,
                                                int r, int k, int n_exp, float* __restrict__ ures) {
  __shared__ float gs[8 * 32];
  __shared__ int es[8];
  const int tid = threadIdx.x;
  const int tok = perm[p];
  const int kr = k * r;
  if (tid < kr) {
    float sum = 0.f;
    for (int part = 0; part < n_parts; ++part) sum += spart[((size_t)part * T + p) * kr + tid];
    gs[tid] = gate[(size_t)tok * k + tid / r] * sum;
  }
  if (tid < k) es[tid] = min(max(expert_idx[(size_t)tok * k + tid], 0), n_exp - 1);
  __syncthreads();
  const int ch = chunk * 256 + tid;  // 8 output columns
  if (ch >= d / 8) return;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int j = 0; j < k; ++j) {
    const size_t row0 = (size_t)es[j] * r;
    for (int rho0 = 0; rho0 < r; rho0 += 4) {   // r is a multiple of 4: four rows per batch of loads
      unsigned bytes[4];
      float sc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t row = row0 + rho0 + u;
        bytes[u] = *(const unsigned*)(u2_q + row * (d / 2) + ch * 4);
        sc[u] = (float)u2_s[row * (d / q) + (ch * 8) / q] * gs[j * r + rho0 + u];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned b = (bytes[u] >> (8 * i)) & 0xffu;
          acc[2 * i] = fmaf(sc[u], nib_lo(b), acc[2 * i]);
          acc[2 * i + 1] = fmaf(sc[u], nib_hi(b), acc[2 * i + 1]);
        }
    }
  }
  float* dst = ures + (size_t)p * d + ch * 8;
  *(float4v*)dst = float4v{acc[0], acc[1], acc[2], acc[3]};
  *(float4v*)(dst + 4) = float4v{acc[4], acc[5], acc[6], acc[7]};
}

// y[perm[p]] = y_base_sorted[p] + ures[p]
__global__ __launch_bounds__(256) void skinny_add_kernel(const half_t* __restrict__ yb, const float* __restrict__ ures,
                                                         const int* __restrict__ perm, int d,
                                                         half_t* __restrict__ y) {
  const int p = blockIdx.x, ch = blockIdx.y * 256 + threadIdx.x;
  if (ch >= d / 8) return;
  const half8 b8 = *(const half8*)(yb + (size_t)p * d + ch * 8);
  const float* u = ures + (size_t)p * d + ch * 8;
  const float4v u0 = *(const float4v*)u, u1 = *(const float4v*)(u + 4);
  half8 o;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    o[i] = (half_t)((float)b8[i] + u0[i]);
    o[i + 4] = (half_t)((float)b8[i + 4] + u1[i]);
  }
  *(half8*)(y + (size_t)perm[p] * d + ch * 8) = o;
}

// Small jobs that ride along with a weight stream as the first workgroups of its grid:
// they are dispatched first, finish within a few microseconds and leave their slots to
// the stream, instead of costing a launch of their own on the critical path.
enum { SIDE_NONE = 0, SIDE_T1 = 1, SIDE_URES = 2 };
struct SideArgs {
  const half_t* x;
  const int* perm;
  const int* expert_idx;
  const float* gate;
  const uint8_t* fq;     // V1 codes (SIDE_T1) or U2 codes (SIDE_URES)
  const half_t* fs;      // their scales
  const float* spart;
  half_t* t1;
  float* ures;
  int T, d, q, r, k, n_parts, n_jobs;
  int x_div;             // row of x of a token index = index / x_div (>= 1)
  int n_exp;             // G * K: expert slots are clamped to [0, n_exp)
  int n_side;            // workgroups reserved for the jobs (n_jobs rounded up to 8)
};

// ---------------------------------------------------------------- shared-base products
// out[p][n] = sum_k W[c][n][k] X[row(p)][k] for the sorted rows p of cluster c (the product
// the experts of a cluster share, Sec. 3.2): up-projection with W = W1_base, X = x gathered
// through perm, out = Hb; down-projection with W = W2_base, X = A, out = y_base_sorted.
// N: rows of W per cluster, Kc: contraction length, gather: row index of X per sorted row
// or NULL for the identity.  w_blk = 0: W[c] is row-major [N][Kc]; otherwise W[c] is stored
// as [Kc / 32][N][32] and w_blk = N * 32 (the re-tiled copy of the bases): an 8-row load is
// then two contiguous 256-byte pieces instead of eight 128-byte pieces a row apart.
template <int SIDE, int COLS, bool NT>
__global__ __launch_bounds__(256, SkRing<COLS>::OCC) void skinny_base_kernel(const half_t* __restrict__ X,
                                                                  const int* __restrict__ gather,
                                                                  const half_t* __restrict__ W,
                                                                  const int* __restrict__ offsets, int N, int Kc,
                                                                  half_t* __restrict__ out, int nx, int G,
                                                                  long w_blk, SideArgs sa) {
  if (SIDE != SIDE_NONE && (int)blockIdx.x < sa.n_side) {
    const int job = blockIdx.x;
    if (job >= sa.n_jobs) return;
    if (SIDE == SIDE_T1) {
      skinny_t1_job(job / sa.k, job % sa.k, sa.x, sa.perm, sa.expert_idx, sa.fq, sa.fs, sa.d, sa.q, sa.r, sa.k,
                    sa.x_div, sa.n_exp, sa.t1);
    } else {
      const int nch = (sa.d + 2047) / 2048;
      skinny_ures_job(job / nch, job % nch, sa.perm, sa.expert_idx, sa.gate, sa.fq, sa.fs, sa.spart, sa.n_parts, sa.T,
                      sa.d, sa.q, sa.r, sa.k, sa.n_exp, sa.ures);
    }
    return;
  }
  constexpr int RED_BYTES = SK_WAVES * SK_RB * 16 * 64 * 4;
  using RG = SkRing<COLS>;
  constexpr int RINGS = SK_WAVES * RG::RING;
  __shared__ __attribute__((aligned(1024))) char smem[RED_BYTES > RINGS ? RED_BYTES : RINGS];
  float* red = (float*)smem;
  SkinnyTile t;
  if (!skinny_tile(offsets, (int)blockIdx.x - (SIDE != SIDE_NONE ? sa.n_side : 0), nx, G, COLS, t)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, fr = lane & 31, h = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const unsigned smem_lds = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const int lrow = lane >> 3;
  const size_t w_ld = w_blk ? 32 : Kc;   // elements between consecutive weight rows
  const half_t* wrow = W + (size_t)t.c * N * Kc + (size_t)(t.n0 + lrow) * w_ld;
  const int p = t.m0 + fr;
  const half_t* brow[COLS / 8];
#pragma unroll
  for (int i = 0; i < COLS / 8; ++i) {
    int r = min(t.m0 + 8 * i + lrow, t.m_end - 1);
    if (gather != nullptr) r = gather[r] / sa.x_div;
    brow[i] = X + (size_t)r * Kc;
  }
  float16v acc[SK_RB];
#pragma unroll
  for (int rb = 0; rb < SK_RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
  const int iters = Kc / 64;
  skinny_stream<COLS, NT>(wrow, 8 * w_ld, w_blk ? (size_t)w_blk : 32, brow, smem + wv * RG::RING, smem_lds + wv * RG::RING, lane,
                wv * iters / SK_WAVES, (wv + 1) * iters / SK_WAVES, acc);
  __syncthreads();  // every ring has been consumed: its space becomes red
  float16v hb;
  skinny_reduce(red, wave, lane, acc, hb);
  if (wave < SK_RB && fr < COLS && p < t.m_end) {
#pragma unroll
    for (int qd = 0; qd < 4; ++qd)
      *(half4*)(out + (size_t)p * N + t.n0 + wave * 32 + 8 * qd + 4 * h) = to_half4(hb, qd);
  }
}

// ---------------------------------------------------------------- residual-up, GELU, gated sum, V2 product
// In place on A (which holds Hb on entry), for sorted row p and a chunk of RU_CH columns:
//   A[p][n] = sum_j g_j GELU(Hb[p][n] + sum_rho U1_{e_j}[rho][n] t1_j[rho])       (Sec. 3.2)
//   spart[chunk][p][j][rho] = sum_{n in chunk} V2_{e_j}[rho][n] GELU(...)_j[n]
// with the INT4 factors dequantised on the fly (Sec. 3.4).  A thread owns 8 consecutive
// columns (one 32-bit word of codes per rank row); the k*r partial dot products of a thread
// are summed over the wavefront by a halving exchange (64 values on 64 lanes -> lane l ends
// with the total of value l), then over the 4 wavefronts in fixed order.
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
// The 8 INT4 codes c_0..c_7 of one 32-bit word as f16 pairs WITHOUT their offsets removed.
// Flipping bit 3 of every nibble turns a two's-complement code c into c + 8 in [0, 16); a
// nibble masked in place into the mantissa of 1024.0 then reads 1024 + (c + 8) at mantissa
// bit 0 and 1024 + 16 (c + 8) at mantissa bit 4:
//   o[0] = 1032 + (c_0, c_4)        o[1] = 16 (72 + (c_1, c_5))
//   o[2] = 1032 + (c_2, c_6)        o[3] = 16 (72 + (c_3, c_7))
// The users fold the factor 16 into the other operand and subtract the offsets once per
// sum (FP32 accumulation keeps that exact enough: the offsets are < 2^11 times the terms).
constexpr float DQ_OFF_EVEN = 1032.f, DQ_OFF_ODD = 72.f;
__device__ __forceinline__ unsigned and_or(unsigned a, unsigned mask, unsigned bits) {
  unsigned r;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(mask), "v"(bits));
  return r;
}
__device__ __forceinline__ void decode8_raw(unsigned w, half2v (&o)[4]) {
  const unsigned magic = 0x64006400u;
  w ^= 0x88888888u;
  const unsigned w8 = w >> 8;
  o[0] = __builtin_bit_cast(half2v, and_or(w, 0x000f000fu, magic));
  o[1] = __builtin_bit_cast(half2v, and_or(w, 0x00f000f0u, magic));
  o[2] = __builtin_bit_cast(half2v, and_or(w8, 0x000f000fu, magic));
  o[3] = __builtin_bit_cast(half2v, and_or(w8, 0x00f000f0u, magic));
}

// The same with the offsets removed exactly (f16 subtraction of representable values):
// o[0] = (c_0, c_4), o[1] = 16 (c_1, c_5), o[2] = (c_2, c_6), o[3] = 16 (c_3, c_7).
__device__ __forceinline__ void decode8_x16(unsigned w, half2v (&o)[4]) {
  decode8_raw(w, o);
  const half2v even = {(_Float16)1032.f, (_Float16)1032.f}, odd = {(_Float16)1152.f, (_Float16)1152.f};
  o[0] -= even;
  o[1] -= odd;
  o[2] -= even;
  o[3] -= odd;
}

constexpr int RU_N = 8;
constexpr int RU_CH = RU_N * 256;
static_assert(RU_CH == SKINNY_SN, "s partial chunk");

template <int OFF>
__device__ __forceinline__ void halving_step(float (&v)[64], int lane) {
  const bool up = (lane & OFF) != 0;
#pragma unroll
  for (int i = 0; i < OFF; ++i) {
    const float keep = up ? v[i + OFF] : v[i];
    const float send = up ? v[i] : v[i + OFF];
    v[i] = keep + __shfl_xor(send, OFF, 64);
  }
}

template <int R>
__global__ __launch_bounds__(256) void skinny_resid_up_kernel(
    half_t* __restrict__ A, const half_t* __restrict__ t1, const int* __restrict__ perm,
    const int* __restrict__ expert_idx, const float* __restrict__ gate, const uint8_t* __restrict__ u1_q,
    const half_t* __restrict__ u1_s, const uint8_t* __restrict__ v2_q, const half_t* __restrict__ v2_s, int T,
    int d_ff, int k, int q, int n_exp, float* __restrict__ spart) {
  constexpr int EPG = 64 / R;    // experts per group of 64 (expert, rank row) values
  __shared__ int srow[8];        // first factor row e_j R of selected expert j
  __shared__ float st1[256];     // t1_j[rho]
  __shared__ float sg[8];
  __shared__ float red[4][64];
  const int p = blockIdx.x, chunk = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kr = k * R;
  const int tok = perm[p];
  if (tid < kr) st1[tid] = (float)t1[(size_t)p * kr + tid];
  if (tid < k) {
    srow[tid] = min(max(expert_idx[(size_t)tok * k + tid], 0), n_exp - 1) * R;
    sg[tid] = gate[(size_t)tok * k + tid];
  }
  const int n = chunk * RU_CH + tid * RU_N;
  const bool in = n < d_ff;
  const size_t qrow = (size_t)(d_ff / 2), srw = (size_t)(d_ff / q);
  float hbv[8], av[8];
  {
    half8 h8 = {0, 0, 0, 0, 0, 0, 0, 0};
    if (in) h8 = *(const half8*)(A + (size_t)p * d_ff + n);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      hbv[i] = (float)h8[i];
      av[i] = 0.f;
    }
  }
  __syncthreads();
  for (int j0 = 0; j0 < k; j0 += EPG) {
    float part[64];
#pragma unroll
    for (int jj = 0; jj < EPG; ++jj) {
      const int j = j0 + jj;
#pragma unroll
      for (int rho = 0; rho < R; ++rho) part[jj * R + rho] = 0.f;
      if (in && j < k) {
        // the expert's rows are uniform over the workgroup: scalar row bases, one 32-bit
        // lane offset; every code word and scale is requested before the first is used
        const size_t row0 = (size_t)__builtin_amdgcn_readfirstlane(srow[j]);
        const uint8_t* ub = u1_q + row0 * qrow;
        const uint8_t* vb = v2_q + row0 * qrow;
        const half_t* usb = u1_s + row0 * srw;
        const half_t* vsb = v2_s + row0 * srw;
        const unsigned qoff = (unsigned)n / 2, soff = (unsigned)n / (unsigned)q;
        unsigned uw[R], vw[R];
        half_t us[R], vs[R];
#pragma unroll
        for (int rho = 0; rho < R; ++rho) {
          uw[rho] = *(const unsigned*)(ub + rho * qrow + qoff);
          us[rho] = usb[rho * srw + soff];
        }
#pragma unroll
        for (int rho = 0; rho < R; ++rho) {
          vw[rho] = *(const unsigned*)(vb + rho * qrow + qoff);
          vs[rho] = vsb[rho * srw + soff];
        }
        float hj[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) hj[i] = hbv[i];
        float ssum = 0.f;
#pragma unroll
        for (int rho = 0; rho < R; ++rho) {
          const float sc = (float)us[rho] * st1[j * R + rho], sc16 = sc * 0.0625f;
          ssum += sc;
          half2v c[4];
          decode8_raw(uw[rho], c);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float m = (i & 1) ? sc16 : sc;
            hj[i] = fmaf((float)c[i][0], m, hj[i]);
            hj[i + 4] = fmaf((float)c[i][1], m, hj[i + 4]);
          }
        }
        const float g = sg[j];
        half2v g2[4];   // GELU values as f16 pairs (element i, element i + 4), odd i scaled by 1/16
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float off = (i & 1) ? DQ_OFF_ODD : DQ_OFF_EVEN;
          const float lo = gelu_erf(fmaf(-off, ssum, hj[i])), hi = gelu_erf(fmaf(-off, ssum, hj[i + 4]));
          av[i] = fmaf(g, lo, av[i]);
          av[i + 4] = fmaf(g, hi, av[i + 4]);
          const half2v gg = half2v{(_Float16)lo, (_Float16)hi};
          g2[i] = (i & 1) ? gg * half2v{(_Float16)0.0625f, (_Float16)0.0625f} : gg;
        }
        // the two-element dot product instruction is fed exact codes: its accumulation is
        // not a correctly rounded FP32 chain, so large offsets must not pass through it
#pragma unroll
        for (int rho = 0; rho < R; ++rho) {
          half2v c[4];
          decode8_x16(vw[rho], c);
          float dot = 0.f;
#pragma unroll
          for (int i = 0; i < 4; ++i) dot = __builtin_amdgcn_fdot2(c[i], g2[i], dot, false);
          part[jj * R + rho] = (float)vs[rho] * dot;
        }
      }
    }
    halving_step<32>(part, lane);
    halving_step<16>(part, lane);
    halving_step<8>(part, lane);
    halving_step<4>(part, lane);
    halving_step<2>(part, lane);
    halving_step<1>(part, lane);
    red[wave][lane] = part[0];
    __syncthreads();
    if (wave == 0 && j0 * R + lane < kr)
      spart[((size_t)chunk * T + p) * kr + j0 * R + lane] =
          ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
    __syncthreads();
  }
  if (in) {
    half8 o;
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = (half_t)av[i];
    *(half8*)(A + (size_t)p * d_ff + n) = o;
  }
}

// ---------------------------------------------------------------- residual-down + un-permute
// y[t] = y_base_sorted[inv_perm[t]] + sum_j g_j U2_{e_j} s_j with U2 dequantised on the
// fly: one workgroup per token, a thread per 8 output columns.
__global__ __launch_bounds__(256) void skinny_combine_kernel(const half_t* __restrict__ yb,
                                                             const float* __restrict__ s_down,
                                                             const int* __restrict__ inv_perm,
                                                             const int* __restrict__ expert_idx,
                                                             const float* __restrict__ gate,
                                                             const uint8_t* __restrict__ u2_q,
                                                             const half_t* __restrict__ u2_s, int d, int q, int r,
                                                             int k, int n_exp, half_t* __restrict__ y) {
  __shared__ float gs[8 * 32];
  __shared__ int es[8];
  const int t = blockIdx.x, tid = threadIdx.x;
  if (tid < k * r) gs[tid] = gate[(size_t)t * k + tid / r] * s_down[(size_t)t * k * r + tid];
  if (tid < k) es[tid] = min(max(expert_idx[(size_t)t * k + tid], 0), n_exp - 1);
  __syncthreads();
  const int ch = blockIdx.y * 256 + tid;  // 8 output columns
  if (ch >= d / 8) return;
  const half8 b8 = *(const half8*)(yb + (size_t)inv_perm[t] * d + ch * 8);
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = (float)b8[i];
  for (int j = 0; j < k; ++j) {
    const size_t row0 = (size_t)es[j] * r;
    for (int rho0 = 0; rho0 < r; rho0 += 4) {   // r is a multiple of 4: four rows per batch of loads
      unsigned bytes[4];
      float sc[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const size_t row = row0 + rho0 + u;
        bytes[u] = *(const unsigned*)(u2_q + row * (d / 2) + ch * 4);
        sc[u] = (float)u2_s[row * (d / q) + (ch * 8) / q] * gs[j * r + rho0 + u];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned b = (bytes[u] >> (8 * i)) & 0xffu;
          acc[2 * i] = fmaf(sc[u], nib_lo(b), acc[2 * i]);
          acc[2 * i + 1] = fmaf(sc[u], nib_hi(b), acc[2 * i + 1]);
        }
    }
  }
  half8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) o[i] = (half_t)acc[i];
  *(half8*)(y + (size_t)t * d + ch * 8) = o;
}

}  // namespace

// Base matrices larger than this are streamed with the non-temporal hint: they cannot stay in
// the last-level cache (256 MB) from one call to the next anyway, and keeping them out of it
// leaves the routers, the tokens and the factors there.  Smaller layers are left cacheable.
static bool stream_once(const cmoe_dims& dm) {
  return (size_t)dm.G * dm.d * dm.d_ff * sizeof(half_t) > ((size_t)96 << 20);
}

// Hb = W1_base(c) x for every sorted row; with t1 != NULL the t1 = V1 x jobs ride along.
hipError_t launch_skinny_hb(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int x_div, int T,
                            const int* perm, const int* offsets, const int* expert_idx, half_t* t1, half_t* hb,
                            hipStream_t st) {
  const int passes = (T + SK_COLS - 1) / SK_COLS, nx = dm.d_ff / SK_ROWS;
  const unsigned n_stream = (unsigned)nx * dm.G * passes;
  dim3 block(256);
  SideArgs sa{};
  sa.x_div = x_div > 1 ? x_div : 1;
  // the re-tiled copy of W1 when the caller keeps one, else the canonical array
  const half_t* w1 = w.packed ? (const half_t*)((const char*)w.packed + cmoe_packed(dm).w1) : (const half_t*)w.w1_base;
  const long w_blk = w.packed ? (long)dm.d_ff * 32 : 0;
  const bool nt = stream_once(dm);
  if (t1 == nullptr) {
    if (nt)
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, SK_COLS, true>), dim3(n_stream), block, 0, st, x, perm, w1,
                         offsets, dm.d_ff, dm.d, hb, nx, dm.G, w_blk, sa);
    else
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, SK_COLS, false>), dim3(n_stream), block, 0, st, x, perm, w1,
                         offsets, dm.d_ff, dm.d, hb, nx, dm.G, w_blk, sa);
    return hipGetLastError();
  }
  sa.x = x;
  sa.perm = perm;
  sa.expert_idx = expert_idx;
  sa.fq = w.v1_q;
  sa.fs = (const half_t*)w.v1_s;
  sa.t1 = t1;
  sa.T = T;
  sa.d = dm.d;
  sa.q = dm.q;
  sa.r = dm.r;
  sa.k = dm.k;
  sa.n_exp = dm.G * dm.K;
  sa.n_jobs = T * dm.k;
  sa.n_side = (sa.n_jobs + 7) & ~7;
  if (nt)
    hipLaunchKernelGGL((skinny_base_kernel<SIDE_T1, SK_COLS, true>), dim3(n_stream + sa.n_side), block, 0, st, x, perm,
                       w1, offsets, dm.d_ff, dm.d, hb, nx, dm.G, w_blk, sa);
  else
    hipLaunchKernelGGL((skinny_base_kernel<SIDE_T1, SK_COLS, false>), dim3(n_stream + sa.n_side), block, 0, st, x, perm,
                       w1, offsets, dm.d_ff, dm.d, hb, nx, dm.G, w_blk, sa);
  return hipGetLastError();
}

hipError_t launch_skinny_resid_up(const cmoe_dims& dm, const cmoe_weights& w, int T, const int* perm,
                                  const int* expert_idx, const float* gate, const half_t* t1, half_t* a,
                                  float* spart, hipStream_t st) {
  dim3 grid(T, (dm.d_ff + SKINNY_SN - 1) / SKINNY_SN), block(256);
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, grid, block, 0, st, a, t1, perm, expert_idx, gate, w.u1_q, (const half_t*)w.u1_s,
                       w.v2_q, (const half_t*)w.v2_s, T, dm.d_ff, dm.k, dm.q, dm.G * dm.K, spart);
  };
  switch (dm.r) {
    case 4: go(skinny_resid_up_kernel<4>); break;
    case 8: go(skinny_resid_up_kernel<8>); break;
    case 16: go(skinny_resid_up_kernel<16>); break;
    default: go(skinny_resid_up_kernel<32>); break;
  }
  return hipGetLastError();
}

// y_base_sorted = W2_base(c) A; with ures != NULL the residual-down jobs ride along
// (ures[p] = sum_j g_j U2 s_j from the s partials), to be added by launch_skinny_add.
hipError_t launch_skinny_down(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T, const int* offsets,
                              half_t* y_base_sorted, const int* perm, const int* expert_idx, const float* gate,
                              const float* spart, int n_parts, float* ures, hipStream_t st) {
  const int passes = (T + SK_COLS - 1) / SK_COLS, nx = dm.d / SK_ROWS;
  const unsigned n_stream = (unsigned)nx * dm.G * passes;
  dim3 block(256);
  SideArgs sa{};
  sa.x_div = 1;
  const half_t* w2 = w.packed ? (const half_t*)((const char*)w.packed + cmoe_packed(dm).w2) : (const half_t*)w.w2_base;
  const long w_blk = w.packed ? (long)dm.d * 32 : 0;
  const bool nt = stream_once(dm);
  if (ures == nullptr) {
    if (nt)
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, SK_COLS, true>), dim3(n_stream), block, 0, st, a,
                         (const int*)nullptr, w2, offsets, dm.d, dm.d_ff, y_base_sorted, nx, dm.G, w_blk, sa);
    else
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, SK_COLS, false>), dim3(n_stream), block, 0, st, a,
                         (const int*)nullptr, w2, offsets, dm.d, dm.d_ff, y_base_sorted, nx, dm.G, w_blk, sa);
    return hipGetLastError();
  }
  sa.perm = perm;
  sa.expert_idx = expert_idx;
  sa.gate = gate;
  sa.fq = w.u2_q;
  sa.fs = (const half_t*)w.u2_s;
  sa.spart = spart;
  sa.ures = ures;
  sa.T = T;
  sa.d = dm.d;
  sa.q = dm.q;
  sa.r = dm.r;
  sa.k = dm.k;
  sa.n_exp = dm.G * dm.K;
  sa.n_parts = n_parts;
  sa.n_jobs = T * ((dm.d + 2047) / 2048);
  sa.n_side = (sa.n_jobs + 7) & ~7;
  if (nt)
    hipLaunchKernelGGL((skinny_base_kernel<SIDE_URES, SK_COLS, true>), dim3(n_stream + sa.n_side), block, 0, st, a,
                       (const int*)nullptr, w2, offsets, dm.d, dm.d_ff, y_base_sorted, nx, dm.G, w_blk, sa);
  else
    hipLaunchKernelGGL((skinny_base_kernel<SIDE_URES, SK_COLS, false>), dim3(n_stream + sa.n_side), block, 0, st, a,
                       (const int*)nullptr, w2, offsets, dm.d, dm.d_ff, y_base_sorted, nx, dm.G, w_blk, sa);
  return hipGetLastError();
}

// out[p][n] = sum_k W[g][n][k] X[p][k] for the rows p of group g (offsets [n_groups + 1],
// at most max_rows rows per group): the weight stream on its own, for callers outside the
// layer (the compression pipeline streams residual matrices against sketch rows).
hipError_t launch_skinny_rows(const half_t* X, const half_t* W, const int* offsets, int n_groups, int N, int Kc,
                              int max_rows, half_t* out, hipStream_t st) {
  const int nx = N / SK_ROWS;
  SideArgs sa{};
  sa.x_div = 1;
  // a set of matrices far larger than the last-level cache is not worth keeping there
  const bool nt = (size_t)n_groups * N * Kc * sizeof(half_t) > ((size_t)96 << 20);
  if (max_rows > 16) {
    const int passes = (max_rows + 31) / 32;
    if (nt)
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, 32, true>), dim3((unsigned)nx * n_groups * passes), dim3(256), 0,
                         st, X, (const int*)nullptr, W, offsets, N, Kc, out, nx, n_groups, 0L, sa);
    else
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, 32, false>), dim3((unsigned)nx * n_groups * passes), dim3(256), 0,
                         st, X, (const int*)nullptr, W, offsets, N, Kc, out, nx, n_groups, 0L, sa);
  } else {
    if (nt)
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, 16, true>), dim3((unsigned)nx * n_groups), dim3(256), 0, st, X,
                         (const int*)nullptr, W, offsets, N, Kc, out, nx, n_groups, 0L, sa);
    else
      hipLaunchKernelGGL((skinny_base_kernel<SIDE_NONE, 16, false>), dim3((unsigned)nx * n_groups), dim3(256), 0, st, X,
                         (const int*)nullptr, W, offsets, N, Kc, out, nx, n_groups, 0L, sa);
  }
  return hipGetLastError();
}

hipError_t launch_skinny_add(const cmoe_dims& dm, const half_t* y_base_sorted, const float* ures, const int* perm,
                             int T, half_t* y, hipStream_t st) {
  hipLaunchKernelGGL(skinny_add_kernel, dim3(T, (dm.d / 8 + 255) / 256), dim3(256), 0, st, y_base_sorted, ures, perm,
                     dm.d, y);
  return hipGetLastError();
}

hipError_t launch_skinny_combine(const cmoe_dims& dm, const cmoe_weights& w, const half_t* y_base_sorted,
                                 const float* s_down, const int* inv_perm, const int* expert_idx, const float* gate,
                                 int T, half_t* y, hipStream_t st) {
  hipLaunchKernelGGL(skinny_combine_kernel, dim3(T, (dm.d / 8 + 255) / 256), dim3(256), 0, st, y_base_sorted, s_down, inv_perm, expert_idx,
                     gate, w.u2_q, (const half_t*)w.u2_s, dm.d, dm.q, dm.r, dm.k, dm.G * dm.K, y);
  return hipGetLastError();
}
