// INT4 group-wise factors (Sec. 3.4) -> FP16 operand panels in the layouts the matrix-core
// kernels consume.  value = scale[n / q] * code[n]; code = two's-complement nibble,
// even n in the low nibble of byte n / 2.  Clusters that received no token are skipped,
// so their stored factors are never read.
#include "cmoe_internal.h"

namespace {

__device__ __forceinline__ float nib_lo(unsigned b) { return (float)((int)(b << 28) >> 28); }
__device__ __forceinline__ float nib_hi(unsigned b) { return (float)((int)(b << 24) >> 28); }

// Row-preserving panel: out[c][kk][pos(n)] = factor[c*K + kk/r][kk%r][n], rows kk >= K*r
// zero.  With PERMUTE16, positions inside every aligned group of 16 are reordered as
// n = 8a + 4h + i  ->  8h + 4a + i, which is the order in which one lane of a 32x32
// accumulator block holds its rows (used for the V2 panel, see the fused up-projection).
template <bool PERMUTE16>
__global__ __launch_bounds__(256) void dequant_rows_kernel(const uint8_t* __restrict__ qv,
                                                           const half_t* __restrict__ sv, int L, int q, int K,
                                                           int r, int KRp, const int* __restrict__ offsets,
                                                           half_t* __restrict__ out) {
  const int c = blockIdx.z;
  if (offsets[c + 1] == offsets[c]) return;
  const int kk = blockIdx.y;
  const int n8 = (blockIdx.x * 256 + threadIdx.x) * 8;  // 8 consecutive output positions
  if (n8 >= L) return;
  half8 o = {0, 0, 0, 0, 0, 0, 0, 0};
  if (kk < K * r) {
    const size_t row = (size_t)(c * K) * r + kk;  // (expert, rho) flattened: e*r + rho
    if (!PERMUTE16) {
      // q is a multiple of 8, so the 8 aligned elements share one scale
      unsigned bytes = *(const unsigned*)(qv + row * (L / 2) + n8 / 2);
      float sc = (float)sv[row * (L / q) + n8 / q];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        unsigned b = (bytes >> (8 * i)) & 0xffu;
        o[2 * i] = (half_t)(sc * nib_lo(b));
        o[2 * i + 1] = (half_t)(sc * nib_hi(b));
      }
    } else {
      // output positions n8..n8+7 of the permuted row = h fixed, a in {0,1}, i in 0..3
      int g16 = n8 & ~15, h = (n8 >> 3) & 1;
#pragma unroll
      for (int a = 0; a < 2; ++a) {
        int n = g16 + 8 * a + 4 * h;  // 4 consecutive source elements = 2 bytes
        unsigned bytes = *(const unsigned short*)(qv + row * (L / 2) + n / 2);
        float sc = (float)sv[row * (L / q) + n / q];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          unsigned b = (bytes >> (8 * (i >> 1))) & 0xffu;
          float code = (i & 1) ? nib_hi(b) : nib_lo(b);
          o[4 * a + i] = (half_t)(sc * code);
        }
      }
    }
  }
  *(half8*)(out + ((size_t)c * KRp + kk) * L + n8) = o;
}

// Transposed panel: out[c][n][kk] = factor[c*K + kk/r][kk%r][n] (kk >= K*r zero).
// A thread produces 8 consecutive kk for two adjacent n (one source byte per kk).
__global__ __launch_bounds__(256) void dequant_transpose_kernel(const uint8_t* __restrict__ qv,
                                                                const half_t* __restrict__ sv, int L, int q, int K,
                                                                int r, int KRp, const int* __restrict__ offsets,
                                                                half_t* __restrict__ out) {
  const int c = blockIdx.y;
  if (offsets[c + 1] == offsets[c]) return;
  const int chunks = KRp / 8;
  const long gid = (long)blockIdx.x * 256 + threadIdx.x;
  const int kc = (int)(gid % chunks);
  const long n2 = gid / chunks;  // pair index: n = 2*n2, 2*n2+1
  if (n2 * 2 >= L) return;
  half8 o0 = {0, 0, 0, 0, 0, 0, 0, 0}, o1 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    int kk = kc * 8 + i;
    if (kk < K * r) {
      const size_t row = (size_t)(c * K) * r + kk;
      unsigned b = qv[row * (L / 2) + n2];
      float s = (float)sv[row * (L / q) + (2 * n2) / q];  // q even: both nibbles share the group
      o0[i] = (half_t)(s * nib_lo(b));
      o1[i] = (half_t)(s * nib_hi(b));
    }
  }
  half_t* dst = out + ((size_t)c * L + 2 * n2) * KRp + kc * 8;
  *(half8*)dst = o0;
  *(half8*)(dst + KRp) = o1;
}

}  // namespace

hipError_t launch_dequant_ffn(const cmoe_dims& dm, const cmoe_weights& w, const int* offsets, half_t* v1cat,
                              half_t* u1t, half_t* v2p, hipStream_t st) {
  {
    dim3 grid((dm.d / 8 + 255) / 256, dm.KRp, dm.G);
    hipLaunchKernelGGL(dequant_rows_kernel<false>, grid, dim3(256), 0, st, w.v1_q, (const half_t*)w.v1_s, dm.d,
                       dm.q, dm.K, dm.r, dm.KRp, offsets, v1cat);
  }
  {
    dim3 grid((dm.d_ff / 8 + 255) / 256, dm.KRp, dm.G);
    hipLaunchKernelGGL(dequant_rows_kernel<true>, grid, dim3(256), 0, st, w.v2_q, (const half_t*)w.v2_s, dm.d_ff,
                       dm.q, dm.K, dm.r, dm.KRp, offsets, v2p);
  }
  {
    long threads = (long)(dm.d_ff / 2) * (dm.KRp / 8);
    dim3 grid((unsigned)((threads + 255) / 256), dm.G);
    hipLaunchKernelGGL(dequant_transpose_kernel, grid, dim3(256), 0, st, w.u1_q, (const half_t*)w.u1_s, dm.d_ff,
                       dm.q, dm.K, dm.r, dm.KRp, offsets, u1t);
  }
  return hipGetLastError();
}

hipError_t launch_dequant_u2(const cmoe_dims& dm, const cmoe_weights& w, const int* offsets, half_t* u2t,
                             hipStream_t st) {
  long threads = (long)(dm.d / 2) * (dm.KRp / 8);
  dim3 grid((unsigned)((threads + 255) / 256), dm.G);
  hipLaunchKernelGGL(dequant_transpose_kernel, grid, dim3(256), 0, st, w.u2_q, (const half_t*)w.u2_s, dm.d, dm.q,
                     dm.K, dm.r, dm.KRp, offsets, u2t);
  return hipGetLastError();
}
