// INT4 group-wise factors (Sec. 3.4) -> FP16 operand panels in the layouts the matrix-core
// kernels consume.  value = scale[n / q] * code[n]; code = two's-complement nibble,
// even n in the low nibble of byte n / 2.  Clusters that received no token are skipped,
// so their stored factors are never read (offsets == NULL: every cluster, for the one-time
// packing of the weights).
#include "cmoe_internal.h"

namespace {

__device__ __forceinline__ float nib_lo(unsigned b) { return (float)((int)(b << 28) >> 28); }
__device__ __forceinline__ float nib_hi(unsigned b) { return (float)((int)(b << 24) >> 28); }

// Row-preserving panel: out[c][kk][n] = factor[c*K + kk/r][kk%r][n], rows kk >= K*r zero.
// Block (bx, kk, c) of a grid ((L / 8 + 255) / 256, KRp, G).
__device__ __forceinline__ void dequant_rows(int bx, int kk, int c, const uint8_t* __restrict__ qv,
                                             const half_t* __restrict__ sv, int L, int q, int K, int r, int KRp,
                                             const int* __restrict__ offsets, half_t* __restrict__ out) {
  if (offsets != nullptr && offsets[c + 1] == offsets[c]) return;
  const int n8 = (bx * 256 + threadIdx.x) * 8;  // 8 consecutive output positions
  if (n8 >= L) return;
  half8 o = {0, 0, 0, 0, 0, 0, 0, 0};
  if (kk < K * r) {
    const size_t row = (size_t)(c * K) * r + kk;  // (expert, rho) flattened: e*r + rho
    // q is a multiple of 8, so the 8 aligned elements share one scale
    unsigned bytes = *(const unsigned*)(qv + row * (L / 2) + n8 / 2);
    float sc = (float)sv[row * (L / q) + n8 / q];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      unsigned b = (bytes >> (8 * i)) & 0xffu;
      o[2 * i] = (half_t)(sc * nib_lo(b));
      o[2 * i + 1] = (half_t)(sc * nib_hi(b));
    }
  }
  *(half8*)(out + ((size_t)c * KRp + kk) * L + n8) = o;
}

// Transposed panel: out[c][n][kk] = factor[c*K + kk/r][kk%r][n] (kk >= K*r zero).
// A block takes 64 consecutive n of one cluster and all KRp rank rows: every row's 32 code
// bytes are read as two 16-byte words, dequantised into an LDS tile [64 n][KRp], and the
// tile leaves as whole 16-byte pieces of the n-major rows.  KRp <= 512.
// Block (bx, c) of a grid (L / 64, G).
constexpr int DT_N = 64;
__device__ __forceinline__ void dequant_transpose(int bx, int c, const uint8_t* __restrict__ qv,
                                                  const half_t* __restrict__ sv, int L, int q, int K, int r, int KRp,
                                                  const int* __restrict__ offsets, half_t* __restrict__ out,
                                                  half_t* __restrict__ tile) {
  if (offsets != nullptr && offsets[c + 1] == offsets[c]) return;
  const int n0 = bx * DT_N, ld = KRp + 8, KR = K * r;
  // two threads per rank row: 32 n (16 code bytes) each
  for (int idx = threadIdx.x; idx < KRp * 2; idx += 256) {
    const int kk = idx >> 1, half = idx & 1;
    uint4 w4 = {0u, 0u, 0u, 0u};
    float sc[4] = {0.f, 0.f, 0.f, 0.f};
    if (kk < KR) {
      const size_t row = (size_t)(c * K) * r + kk;
      w4 = *(const uint4*)(qv + row * (L / 2) + (n0 + 32 * half) / 2);
#pragma unroll
      for (int g = 0; g < 4; ++g) sc[g] = (float)sv[row * (L / q) + (n0 + 32 * half + 8 * g) / q];
    }
    const unsigned w[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const unsigned bq = (w[g] >> (8 * i)) & 0xffu;
        const int n = 32 * half + 8 * g + 2 * i;
        tile[n * ld + kk] = (half_t)(sc[g] * nib_lo(bq));
        tile[(n + 1) * ld + kk] = (half_t)(sc[g] * nib_hi(bq));
      }
  }
  __syncthreads();
  const int cpr = KRp / 8;   // 16-byte pieces per output row
  for (int idx = threadIdx.x; idx < DT_N * cpr; idx += 256) {
    const int n = idx / cpr, ch = idx % cpr;
    *(half8*)(out + ((size_t)c * L + n0 + n) * KRp + ch * 8) = *(const half8*)(tile + n * ld + ch * 8);
  }
}

// All panels of a call in ONE launch: the jobs' blocks are laid end to end in a linear grid.
struct DequantJob {
  const uint8_t* qv;
  const half_t* sv;
  half_t* out;
  int L, kind;          // kind 0: rows, 2: transposed
  unsigned nx, first;   // blocks per (kk, c) or per c; first linear block of the job
};
struct DequantJobs {
  DequantJob j[4];
  int n;
};
__global__ __launch_bounds__(256) void dequant_kernel(DequantJobs jobs, int q, int K, int r, int KRp, int G,
                                                      const int* __restrict__ offsets) {
  __shared__ __attribute__((aligned(16))) half_t tile[DT_N * (512 + 8)];
  int ji = 0;
  for (int i = 1; i < jobs.n; ++i)
    if (blockIdx.x >= jobs.j[i].first) ji = i;
  const DequantJob& jb = jobs.j[ji];
  const unsigned local = blockIdx.x - jb.first;
  if (jb.kind == 2) {
    dequant_transpose((int)(local % jb.nx), (int)(local / jb.nx), jb.qv, jb.sv, jb.L, q, K, r, KRp, offsets, jb.out,
                      tile);
  } else {
    const int bx = (int)(local % jb.nx), kk = (int)((local / jb.nx) % KRp), c = (int)(local / jb.nx / KRp);
    dequant_rows(bx, kk, c, jb.qv, jb.sv, jb.L, q, K, r, KRp, offsets, jb.out);
  }
}

void add_job(DequantJobs& js, unsigned& total, const cmoe_dims& dm, const uint8_t* qv, const void* sv, half_t* out,
             int L, int kind) {
  DequantJob& jb = js.j[js.n++];
  jb.qv = qv;
  jb.sv = (const half_t*)sv;
  jb.out = out;
  jb.L = L;
  jb.kind = kind;
  jb.first = total;
  if (kind == 2) {
    jb.nx = (unsigned)(L / DT_N);
    total += jb.nx * dm.G;
  } else {
    jb.nx = (unsigned)((L / 8 + 255) / 256);
    total += jb.nx * dm.KRp * dm.G;
  }
}

}  // namespace

// v1cat, u1t, v2p, and u2t when it is not NULL.
hipError_t launch_dequant_ffn(const cmoe_dims& dm, const cmoe_weights& w, const int* offsets, half_t* v1cat,
                              half_t* u1t, half_t* v2p, half_t* u2t, hipStream_t st) {
  DequantJobs js{};
  unsigned total = 0;
  add_job(js, total, dm, w.u1_q, w.u1_s, u1t, dm.d_ff, 2);
  add_job(js, total, dm, w.v2_q, w.v2_s, v2p, dm.d_ff, 0);
  add_job(js, total, dm, w.v1_q, w.v1_s, v1cat, dm.d, 0);
  if (u2t != nullptr) add_job(js, total, dm, w.u2_q, w.u2_s, u2t, dm.d, 2);
  hipLaunchKernelGGL(dequant_kernel, dim3(total), dim3(256), 0, st, js, dm.q, dm.K, dm.r, dm.KRp, dm.G, offsets);
  return hipGetLastError();
}

hipError_t launch_dequant_u2(const cmoe_dims& dm, const cmoe_weights& w, const int* offsets, half_t* u2t,
                             hipStream_t st) {
  DequantJobs js{};
  unsigned total = 0;
  add_job(js, total, dm, w.u2_q, w.u2_s, u2t, dm.d, 2);
  hipLaunchKernelGGL(dequant_kernel, dim3(total), dim3(256), 0, st, js, dm.q, dm.K, dm.r, dm.KRp, dm.G, offsets);
  return hipGetLastError();
}
