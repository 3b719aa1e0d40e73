// Weight-streaming path of the expert computation for small token counts (Sec. 3.2).
// With only a handful of tokens per cluster the layer is bound by reading every base
// matrix once from HBM, so these kernels are built around that stream: a workgroup owns 64
// weight rows of one cluster, its four wavefronts split the contraction dimension and read
// their weight fragments straight from global memory in the matrix-core operand layout
// (each lane 16 bytes, four loads covering one 128-byte line per row), with the cluster's
// tokens (at most 32 per pass) as the B operand.  INT4 factors are dequantised on the fly
// (Sec. 3.4); nothing is staged through HBM.
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
constexpr int SK_NCH = SK_ROWS / 8;  // 8-row chunks per workgroup
constexpr int SK_OCC = 3;     // workgroups per CU the LDS budget is sized for
constexpr int SK_WAVES = 4;   // wavefronts splitting the contraction

// One 1-KiB direct-to-LDS load: lane l's 16 bytes land at lds_byte + 16 l.
__device__ __forceinline__ void dma16(const void* g, unsigned lds_byte) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

constexpr int SK_COLS = 16;                         // tokens per pass over a cluster
constexpr int SK_A_BYTES = SK_ROWS * 128;           // 64 weight rows x 64 elements
constexpr int SK_B_BYTES = SK_COLS * 128;           // 16 token rows x 64 elements
constexpr int SK_STAGE = SK_A_BYTES + SK_B_BYTES;   // one wavefront stage
constexpr int SK_RING = 2 * SK_STAGE;               // two stages per wavefront
constexpr int SK_DMA = (SK_ROWS + SK_COLS) / 8;     // 1-KiB loads per stage (8 rows x 128 B each)

// acc[rb] += sum_k W[row(rb)][k] X[col][k] over the 64-element steps [it0, it1) of this
// wavefront.  Both operands stream global -> LDS one step ahead of the matrix-core work,
// as whole 128-byte lines per row, into a two-stage ring private to the wavefront (so no
// barrier is needed, only vmcnt), chunks XOR-swizzled with (row >> 1) & 7.
//   wrow / brow: the lane's row (lane / 8) of the first 8-row group of the weight / token
//                tile at step 0, WITHOUT the chunk offset (the swizzle depends on the row);
//                w_stride / b_stride: elements between 8-row groups (token rows beyond the
//                pass are clamped by the caller through brow1)
// Accumulator columns 16..31 repeat columns 0..15.
__device__ __forceinline__ void skinny_stream(const half_t* wrow, size_t w_stride, const half_t* brow0,
                                              const half_t* brow1, char* ring, unsigned ring_lds, int lane, int it0,
                                              int it1, float16v (&acc)[SK_RB]) {
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
    const int brow = fr & (SK_COLS - 1);
    offb[s] = SK_A_BYTES + brow * 128 + (((2 * s + h) ^ ((brow >> 1) & 7)) << 4);
  }
  // lane l of load i fills row 8i + l/8, chunk position l%8, with source chunk position ^ swizzle(row)
  const int lrow = lane >> 3, lpos = lane & 7;
  const int c0 = (lpos ^ (lrow >> 1)) << 3, c1 = (lpos ^ (lrow >> 1) ^ 4) << 3;  // even / odd groups
  auto issue = [&](int it, int stage) {
    const unsigned dst = ring_lds + stage * SK_STAGE;
#pragma unroll
    for (int i = 0; i < SK_ROWS / 8; ++i)
      dma16(wrow + ((i & 1) ? c1 : c0) + (size_t)i * w_stride + (size_t)it * 64, dst + i * 1024);
    dma16(brow0 + c0 + (size_t)it * 64, dst + SK_A_BYTES);
    dma16(brow1 + c1 + (size_t)it * 64, dst + SK_A_BYTES + 1024);
  };
  auto compute = [&](int stage) {
    const char* sb = ring + stage * SK_STAGE;
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
      wait_vm<SK_DMA>();
    } else {
      wait_vm<0>();
    }
    compute(0);
    if (it + 1 < it1) {
      if (it + 2 < it1) {
        issue(it + 2, 0);
        wait_vm<SK_DMA>();
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
// grid: x = row block, y = cluster, z = pass over the cluster's tokens (SK_COLS per pass);
// m_end is the end of the pass
__device__ __forceinline__ bool skinny_tile(const int* offsets, SkinnyTile& t) {
  t.c = blockIdx.y;
  // Workgroups are dealt round-robin to the 8 XCDs.  The INT4 factor rows are 128-byte
  // lines shared by 8 neighbouring row blocks, so inside every run of 64 blocks the 8
  // workgroups that land on one XCD take 8 neighbouring row blocks: each line is then
  // fetched into one L2 instead of eight.
  int xb = blockIdx.x;
  if ((gridDim.x & 7) == 0 && xb < (int)(gridDim.x & ~63u)) xb = (xb & ~63) + ((xb & 7) << 3) + ((xb >> 3) & 7);
  t.n0 = xb * SK_ROWS;
  const int lo = offsets[t.c], hi = offsets[t.c + 1];
  t.m0 = lo + blockIdx.z * SK_COLS;
  t.m_end = min(hi, t.m0 + SK_COLS);
  return t.m0 < hi;
}

// ---------------------------------------------------------------- t1 = V1_e x
// One workgroup per (sorted row p, selected expert j); a wavefront per rank row.
__global__ __launch_bounds__(1024) void skinny_t1_kernel(const half_t* __restrict__ x, const int* __restrict__ perm,
                                                        const int* __restrict__ expert_idx,
                                                        const uint8_t* __restrict__ v1_q,
                                                        const half_t* __restrict__ v1_s, int d, int q, int r, int k,
                                                        half_t* __restrict__ t1) {
  const int p = blockIdx.x / k, j = blockIdx.x % k;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int tok = perm[p];
  const int e = expert_idx[(size_t)tok * k + j];
  const half_t* xr = x + (size_t)tok * d;
  for (int rho = wave; rho < r; rho += 16) {
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

// ---------------------------------------------------------------- fused up-projection
template <int R, int KMAX, int KRPMAX>
__global__ __launch_bounds__(256, SK_OCC) void skinny_up_kernel(
    const half_t* __restrict__ x, const half_t* __restrict__ w1_base, const uint8_t* __restrict__ u1_q,
    const half_t* __restrict__ u1_s, const uint8_t* __restrict__ v2_q, const half_t* __restrict__ v2_s,
    const half_t* __restrict__ t1, const int* __restrict__ perm, const int* __restrict__ offsets,
    const int* __restrict__ expert_idx, const float* __restrict__ gate, int T, int d, int d_ff, int K, int k, int q,
    int KRp, half_t* __restrict__ A, float* __restrict__ spart) {
  using FU = FusedUp<R, KMAX>;
  constexpr int LDU = KRPMAX + 8, LDV = SK_ROWS + 8;
  constexpr int RED_BYTES = SK_WAVES * SK_RB * 16 * 64 * 4;
  constexpr int SU_BYTES = SK_ROWS * LDU * 2;
  constexpr int R0_BYTES = RED_BYTES > SU_BYTES ? RED_BYTES : SU_BYTES;
  constexpr int EPI_BYTES = R0_BYTES + KRPMAX * LDV * 2;
  constexpr int RINGS = SK_WAVES * SK_RING;
  __shared__ __attribute__((aligned(1024))) char smem[EPI_BYTES > RINGS ? EPI_BYTES : RINGS];
  float* red = (float*)smem;
  half_t* sU = (half_t*)smem;               // [64][LDU]   U1 tile, transposed (after red is dead)
  half_t* sV = (half_t*)(smem + R0_BYTES);  // [KRp][LDV]  V2 tile, columns permuted in 16-groups

  SkinnyTile t;
  if (!skinny_tile(offsets, t)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, fr = lane & 31, h = lane >> 5;

  // ---- per-lane token state of the epilogue, requested before the weight stream starts
  typename FU::Tok tk;
  FU::load_tok(tk, fr < SK_COLS ? t.m0 + fr : t.m_end, t.m_end, t.c, K, k, perm, expert_idx, gate, t1, h);

  // ---- request this thread's share of the cluster's INT4 factor tiles (zero beyond K*r)
  constexpr int FTASKS = KRPMAX * SK_NCH / 256;
  unsigned u_bytes[FTASKS];
  half_t u_sc[FTASKS];
  unsigned short v_bytes[FTASKS][2];
  half_t v_sc[FTASKS][2];
#pragma unroll
  for (int i2 = 0; i2 < FTASKS; ++i2) {
    const int task = tid + i2 * 256;
    const int n8 = task % SK_NCH, kk = task / SK_NCH;
    u_bytes[i2] = 0;
    u_sc[i2] = (half_t)0.f;
    v_bytes[i2][0] = v_bytes[i2][1] = 0;
    v_sc[i2][0] = v_sc[i2][1] = (half_t)0.f;
    if (task < KRp * SK_NCH && kk < K * R) {
      const size_t row = (size_t)t.c * K * R + kk;
      const int n = t.n0 + n8 * 8;
      u_bytes[i2] = *(const unsigned*)(u1_q + row * (d_ff / 2) + n / 2);
      u_sc[i2] = u1_s[row * (d_ff / q) + n / q];
      const int g16 = (n8 * 8) & ~15, hh = n8 & 1;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const int nv = t.n0 + g16 + 8 * a + 4 * hh;
        v_bytes[i2][a] = *(const unsigned short*)(v2_q + row * (d_ff / 2) + nv / 2);
        v_sc[i2][a] = v2_s[row * (d_ff / q) + nv / q];
      }
    }
  }

  // ---- stream W1_base(c) rows [n0, n0 + 64) once; this wavefront's share of d
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const unsigned smem_lds = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const int lrow = lane >> 3;
  const half_t* wrow = w1_base + ((size_t)t.c * d_ff + t.n0 + lrow) * d;
  const half_t* brow0 = x + (size_t)perm[min(t.m0 + lrow, t.m_end - 1)] * d;
  const half_t* brow1 = x + (size_t)perm[min(t.m0 + 8 + lrow, t.m_end - 1)] * d;
  float16v acc[SK_RB];
#pragma unroll
  for (int rb = 0; rb < SK_RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
  const int iters = d / 64;
  skinny_stream(wrow, (size_t)8 * d, brow0, brow1, smem + wv * SK_RING, smem_lds + wv * SK_RING, lane,
                wv * iters / SK_WAVES, (wv + 1) * iters / SK_WAVES, acc);
  __syncthreads();  // every ring has been consumed: its space becomes red

  float16v hb;
  skinny_reduce(red, wave, lane, acc, hb);
  __syncthreads();  // red is dead: its space becomes sU

  // ---- INT4 factors of the cluster for these 64 rows -> LDS as f16 (Sec. 3.4); their
  // code bytes and scales were requested before the weight stream started
  const int KR = K * R;
#pragma unroll
  for (int i2 = 0; i2 < FTASKS; ++i2) {   // U1: 8 consecutive n of one rank row, transposed
    const int task = tid + i2 * 256;
    if (task < KRp * SK_NCH) {
      const int n8 = task % SK_NCH, kk = task / SK_NCH;
      const float sc = (float)u_sc[i2];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const unsigned b = (u_bytes[i2] >> (8 * i)) & 0xffu;
        sU[(n8 * 8 + 2 * i) * LDU + kk] = (half_t)(sc * nib_lo(b));
        sU[(n8 * 8 + 2 * i + 1) * LDU + kk] = (half_t)(sc * nib_hi(b));
      }
    }
  }
#pragma unroll
  for (int i2 = 0; i2 < FTASKS; ++i2) {   // V2: 8 output positions of one rank row
    const int task = tid + i2 * 256;
    if (task < KRp * SK_NCH) {
      const int c8 = task % SK_NCH, kk = task / SK_NCH;
      half8 o;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        const float sc = (float)v_sc[i2][a];
        const unsigned bytes = v_bytes[i2][a];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const unsigned b = (bytes >> (8 * (i >> 1))) & 0xffu;
          o[4 * a + i] = (half_t)(sc * ((i & 1) ? nib_hi(b) : nib_lo(b)));
        }
      }
      *(half8*)(sV + kk * LDV + c8 * 8) = o;
    }
  }
  (void)KR;
  __syncthreads();

  // ---- per-(token, expert) residual, GELU, gated sum, V2 product: one wavefront per block
  if (wave < SK_RB) {
    float16v sacc[KMAX];
#pragma unroll
    for (int j = 0; j < KMAX; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) sacc[j][v] = 0.f;
    float16v o;
    auto uf = [&](int kc) { return *(const half8*)(sU + (wave * 32 + fr) * LDU + kc * 16 + 8 * h); };
    auto vf = [&](int qq, int s2) { return *(const half8*)(sV + (qq * 32 + fr) * LDV + wave * 32 + 16 * s2 + 8 * h); };
    FU::block(hb, tk, k, KRp / 16, KRp / 32, h, uf, vf, o, sacc);
    const int nb = t.n0 + wave * 32;
    if (tk.valid) {
#pragma unroll
      for (int qd = 0; qd < 4; ++qd) *(half4*)(A + (size_t)tk.p * d_ff + nb + 8 * qd + 4 * h) = to_half4(o, qd);
    }
    FU::store_s(tk, sacc, spart + (size_t)(nb / 32) * T * k * R, k, h);
  }
}

// ---------------------------------------------------------------- down-projection
__global__ __launch_bounds__(256, SK_OCC) void skinny_down_kernel(const half_t* __restrict__ A,
                                                             const half_t* __restrict__ w2_base,
                                                             const int* __restrict__ offsets, int d, int d_ff,
                                                             half_t* __restrict__ yb) {
  constexpr int RED_BYTES = SK_WAVES * SK_RB * 16 * 64 * 4;
  constexpr int RINGS = SK_WAVES * SK_RING;
  __shared__ __attribute__((aligned(1024))) char smem[RED_BYTES > RINGS ? RED_BYTES : RINGS];
  float* red = (float*)smem;
  SkinnyTile t;
  if (!skinny_tile(offsets, t)) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, fr = lane & 31, h = lane >> 5;
  const int wv = __builtin_amdgcn_readfirstlane(wave);
  const unsigned smem_lds = (unsigned)(size_t)(__attribute__((address_space(3))) char*)smem;
  const int lrow = lane >> 3;
  const half_t* wrow = w2_base + ((size_t)t.c * d + t.n0 + lrow) * d_ff;
  const int p = t.m0 + fr;
  const half_t* brow0 = A + (size_t)min(t.m0 + lrow, t.m_end - 1) * d_ff;
  const half_t* brow1 = A + (size_t)min(t.m0 + 8 + lrow, t.m_end - 1) * d_ff;
  float16v acc[SK_RB];
#pragma unroll
  for (int rb = 0; rb < SK_RB; ++rb)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[rb][v] = 0.f;
  const int iters = d_ff / 64;
  skinny_stream(wrow, (size_t)8 * d_ff, brow0, brow1, smem + wv * SK_RING, smem_lds + wv * SK_RING, lane,
                wv * iters / SK_WAVES, (wv + 1) * iters / SK_WAVES, acc);
  __syncthreads();  // every ring has been consumed: its space becomes red
  float16v hb;
  skinny_reduce(red, wave, lane, acc, hb);
  if (wave < SK_RB && fr < SK_COLS && p < t.m_end) {
#pragma unroll
    for (int qd = 0; qd < 4; ++qd)
      *(half4*)(yb + (size_t)p * d + t.n0 + wave * 32 + 8 * qd + 4 * h) = to_half4(hb, qd);
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
                                                             int k, half_t* __restrict__ y) {
  __shared__ float gs[8 * 32];
  __shared__ int es[8];
  const int t = blockIdx.x, tid = threadIdx.x;
  if (tid < k * r) gs[tid] = gate[(size_t)t * k + tid / r] * s_down[(size_t)t * k * r + tid];
  if (tid < k) es[tid] = expert_idx[(size_t)t * k + tid];
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

template <int R, int KMAX>
hipError_t launch_up_rk(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, const int* perm,
                        const int* offsets, const int* expert_idx, const float* gate, const half_t* t1, half_t* a,
                        float* spart, hipStream_t st) {
  dim3 grid(dm.d_ff / SK_ROWS, dm.G, (T + SK_COLS - 1) / SK_COLS), block(256);
  if (dm.KRp <= 256)
    hipLaunchKernelGGL((skinny_up_kernel<R, KMAX, 256>), grid, block, 0, st, x, (const half_t*)w.w1_base, w.u1_q,
                       (const half_t*)w.u1_s, w.v2_q, (const half_t*)w.v2_s, t1, perm, offsets, expert_idx, gate, T,
                       dm.d, dm.d_ff, dm.K, dm.k, dm.q, dm.KRp, a, spart);
  else
    hipLaunchKernelGGL((skinny_up_kernel<R, KMAX, 512>), grid, block, 0, st, x, (const half_t*)w.w1_base, w.u1_q,
                       (const half_t*)w.u1_s, w.v2_q, (const half_t*)w.v2_s, t1, perm, offsets, expert_idx, gate, T,
                       dm.d, dm.d_ff, dm.K, dm.k, dm.q, dm.KRp, a, spart);
  return hipGetLastError();
}

template <int R>
hipError_t launch_up_r(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, const int* perm,
                       const int* offsets, const int* expert_idx, const float* gate, const half_t* t1, half_t* a,
                       float* spart, hipStream_t st) {
  if (dm.k <= 1) return launch_up_rk<R, 1>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
  if (dm.k <= 2) return launch_up_rk<R, 2>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
  if (dm.k <= 4) return launch_up_rk<R, 4>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
  return launch_up_rk<R, 8>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
}

}  // namespace

hipError_t launch_skinny_t1(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, const int* perm,
                            const int* expert_idx, half_t* t1, hipStream_t st) {
  hipLaunchKernelGGL(skinny_t1_kernel, dim3(T * dm.k), dim3(1024), 0, st, x, perm, expert_idx, w.v1_q,
                     (const half_t*)w.v1_s, dm.d, dm.q, dm.r, dm.k, t1);
  return hipGetLastError();
}

hipError_t launch_skinny_up(const cmoe_dims& dm, const cmoe_weights& w, const half_t* x, int T, const int* perm,
                            const int* offsets, const int* expert_idx, const float* gate, const half_t* t1,
                            half_t* a, float* spart, hipStream_t st) {
  switch (dm.r) {
    case 4: return launch_up_r<4>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
    case 8: return launch_up_r<8>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
    case 16: return launch_up_r<16>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
    default: return launch_up_r<32>(dm, w, x, T, perm, offsets, expert_idx, gate, t1, a, spart, st);
  }
}

hipError_t launch_skinny_down(const cmoe_dims& dm, const cmoe_weights& w, const half_t* a, int T, const int* offsets,
                              half_t* y_base_sorted, hipStream_t st) {
  dim3 grid(dm.d / SK_ROWS, dm.G, (T + SK_COLS - 1) / SK_COLS), block(256);
  hipLaunchKernelGGL(skinny_down_kernel, grid, block, 0, st, a, (const half_t*)w.w2_base, offsets, dm.d, dm.d_ff,
                     y_base_sorted);
  return hipGetLastError();
}

hipError_t launch_skinny_combine(const cmoe_dims& dm, const cmoe_weights& w, const half_t* y_base_sorted,
                                 const float* s_down, const int* inv_perm, const int* expert_idx, const float* gate,
                                 int T, half_t* y, hipStream_t st) {
  hipLaunchKernelGGL(skinny_combine_kernel, dim3(T, (dm.d / 8 + 255) / 256), dim3(256), 0, st, y_base_sorted, s_down, inv_perm, expert_idx,
                     gate, w.u2_q, (const half_t*)w.u2_s, dm.d, dm.q, dm.r, dm.k, y);
  return hipGetLastError();
}
