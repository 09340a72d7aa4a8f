// Small kernels of the backward pass (the GEMMs are in gemm_bf16.h and wgrad_bf16.h).
#pragma once
#include "forward_types.h"

namespace moe355 {

__global__ void fill_f32_kernel(float *__restrict__ dst, size_t n, float v) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) dst[i] = v;
}

// Gradient of the gate weights: for local row r (token t, pair p = perm[base + r], weight w) the forward kept the
// weighted expert output o_w[r] = w o, so d_topk_w[p] = <o, dy_t> = <o_w[r], dy_t> / w.  One wave per row; the
// sum runs lane-strided, then over the lanes in a fixed butterfly: the same bits on every run.
__global__ __launch_bounds__(256) void gate_weight_grad_kernel(const float *__restrict__ o_w,
                                                               const bf16_t *__restrict__ dy,
                                                               const int32_t *__restrict__ header,
                                                               const int32_t *__restrict__ row_tok,
                                                               const float *__restrict__ row_w,
                                                               const int32_t *__restrict__ perm, int d,
                                                               float *__restrict__ d_topk_w) {
  const int P = header[1], base = header[2];
  const int lane = threadIdx.x & 63;
  for (int r = blockIdx.x * 4 + (threadIdx.x >> 6); r < P; r += gridDim.x * 4) {
    const float *orow = o_w + (size_t)r * d;
    const bf16_t *grow = dy + (size_t)row_tok[r] * d;
    float acc = 0.f;
#pragma unroll 4
    for (int c = lane * 4; c < d; c += 256) {  // d % 8 == 0: groups of 4 stay inside the row
      const f32x4 ov = *reinterpret_cast<const f32x4 *>(orow + c);
      const bf16x4 gv = *reinterpret_cast<const bf16x4 *>(grow + c);
#pragma unroll
      for (int q = 0; q < 4; ++q) acc = fmaf(ov[q], (float)gv[q], acc);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off);
    // (a weight that underflowed to zero leaves nothing of o in o_w: its gradient is reported as zero)
    if (lane == 0) d_topk_w[perm[base + r]] = row_w[r] != 0.f ? acc / row_w[r] : 0.f;
  }
}

}  // namespace moe355
