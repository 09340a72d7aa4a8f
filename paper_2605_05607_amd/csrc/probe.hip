// moe_probe_mfma_rate: what the matrix cores of this device sustain with operands already in registers, the
// reference point for the MFMA fractions that the GEMM kernels are priced against (a figure for the measurement
// harness; nothing on the layer's path calls it).
#define MOE355_BENCH  // the declaration of the probe sits in the bench section of the public header
#include "forward_types.h"

namespace moe355 {

// Every wave runs `iters` rounds of 8 independent 32x32x16 bf16 instructions (8 accumulators, as the GEMM tile
// keeps) on pseudo-random operands (toggling inputs draw the power that real data draws) and stores one value so
// that nothing is optimised away.
__global__ __launch_bounds__(512, 1) void mfma_rate_kernel(int iters, float *__restrict__ sink) {
  const int tid = blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t s = 0x9E3779B9u * (uint32_t)(tid + 1);
  bf16x8 a[4], b[2];
#pragma unroll
  for (int i = 0; i < 6; ++i) {
    u32x4 v;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      s = s * 1664525u + 1013904223u;
      // two bf16 values in [-2, 2): sign and mantissa random, exponent 0 or -1 .. small numbers that stay finite
      v[q] = (s & 0x807F807Fu) | 0x3F003F00u;
    }
    if (i < 4) a[i] = __builtin_bit_cast(bf16x8, v); else b[i - 4] = __builtin_bit_cast(bf16x8, v);
  }
  f32x16 acc[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[0], acc[mi][0], 0, 0, 0);
      acc[mi][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], b[1], acc[mi][1], 0, 0, 0);
    }
  }
  float t = 0.f;
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) t += acc[mi][j][r];
  sink[tid] = t;
}

}  // namespace moe355

using namespace moe355;

extern "C" int moe_probe_mfma_rate(int workgroups, int iters, float *sink, size_t sink_floats, double *flops,
                                   void *stream) {
  if (workgroups < 1 || workgroups > 65535 || iters < 1 || !sink || !flops) return MOE_ERR_INVALID_ARG;
  if (sink_floats < (size_t)workgroups * 512) return MOE_ERR_WORKSPACE;
  begin_launches();
  hipLaunchKernelGGL(mfma_rate_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, iters, sink);
  // 8 waves x 8 instructions x 2 * 32 * 32 * 16 flop per round and workgroup
  *flops = (double)workgroups * 8.0 * 8.0 * 2.0 * 32 * 32 * 16 * (double)iters;
  return launch_status();
}
