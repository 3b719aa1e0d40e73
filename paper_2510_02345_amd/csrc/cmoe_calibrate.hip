// Calibration kernel for the benchmark: what rate do the FP16 matrix cores sustain on this
// machine when they are never kept waiting?  The loop is the inner schedule of the grouped
// products (eight wavefronts per workgroup in two sets that alternate LDS fragment reads and
// v_mfma_f32_16x16x32_f16 issue, one barrier apart) with operands of random mantissas read
// from LDS, but with no global memory traffic, no epilogue and one workgroup per compute
// unit.  Every matrix-core issue slot is used (1024 cycles per iteration and SIMD for 64
// instructions of 16 cycles, the 8 x 4 accumulator blocks of a 128 x 64 wavefront tile
// twice), so the rate that comes out is set by the clock the power
// management grants under this load and nothing else.  With zero_operands every operand is
// 0.0: same instructions, same issue rate, far less switching in the multipliers - the
// difference between the two rates is the share of the published peak that the power limit,
// not the kernel, takes away on real data.
#include "cmoe_internal.h"

namespace {

__global__ __launch_bounds__(512, 1) void calibrate_mfma_kernel(int iters, int zero_operands,
                                                                unsigned long long* __restrict__ ticks,
                                                                float* __restrict__ sink) {
  __shared__ __attribute__((aligned(1024))) char smem[2 * 32768];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < 2 * 32768 / 2; i += 512) {
    unsigned x = (unsigned)i * 2654435761u + blockIdx.x * 97u;
    x ^= x >> 15;
    x *= 2246822519u;
    x ^= x >> 13;
    // unit-scale values with random mantissas (sum of two uniforms)
    const float v = (((x & 0xffff) / 65536.f - 0.5f) + (((x >> 16) & 0xffff) / 65536.f - 0.5f)) * 1.7f;
    ((half_t*)smem)[i] = zero_operands ? (half_t)0.f : (half_t)v;
  }
  __syncthreads();
  int off[12];
#pragma unroll
  for (int i = 0; i < 12; ++i) off[i] = ((wave * 12 + i) * 1024 + lane * 16) & 32767;   // conflict-free 1-KiB reads
  float4v acc[8][4];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = float4v{0.f, 0.f, 0.f, 0.f};
  half8 f[12];
#pragma unroll
  for (int i = 0; i < 12; ++i) f[i] = *(const half8*)(smem + off[i]);
  const bool set_b = wave >= 4;
  const unsigned long long c0 = clock64(), w0 = wall_clock64();
  __builtin_amdgcn_s_barrier();
  if (set_b) __builtin_amdgcn_s_barrier();
  int stage = 0;
  for (int it = 0; it < iters; ++it) {
    const char* sb = smem + stage * 32768;
#pragma unroll
    for (int i = 0; i < 12; ++i) f[i] = *(const half8*)(sb + off[i]);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int a = 0; a < 8; ++a)
        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_f16(f[a], f[8 + b], acc[a][b], 0, 0, 0);
    __builtin_amdgcn_s_setprio(0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    stage ^= 1;
  }
  if (!set_b) __builtin_amdgcn_s_barrier();
  if (tid == 0) {
    atomicAdd(&ticks[0], clock64() - c0);         // shader clock cycles
    atomicAdd(&ticks[1], wall_clock64() - w0);    // constant-rate counter
  }
  float s = 0.f;
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) s += acc[a][b][0] + acc[a][b][1] + acc[a][b][2] + acc[a][b][3];
  sink[(size_t)blockIdx.x * 512 + tid] = s;
}

}  // namespace

extern "C" int cmoe_calibrate_mfma(int32_t n_workgroups, int32_t iters, int32_t zero_operands, uint64_t* ticks,
                                   float* sink, void* stream) {
  if (n_workgroups <= 0 || n_workgroups > 4096 || iters <= 0 || ticks == nullptr || sink == nullptr)
    return CMOE_ERR_INVALID_ARG;
  hipLaunchKernelGGL(calibrate_mfma_kernel, dim3((unsigned)n_workgroups), dim3(512), 0, (hipStream_t)stream, iters,
                     zero_operands != 0 ? 1 : 0, (unsigned long long*)ticks, sink);
  return hipGetLastError() == hipSuccess ? CMOE_OK : CMOE_ERR_HIP;
}
