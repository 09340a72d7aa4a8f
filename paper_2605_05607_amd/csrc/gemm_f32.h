// Grouped fp32 GEMMs on the vector ALU (fp32 layers).
#pragma once
#include "forward_types.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Plain fp32 grouped GEMM (vector ALU) for fp32 layers: 64 x 64 tile, 16-wide k slab, 4 x 4 per thread.
// Weights are the unpacked "input x output" matrices.
// ------------------------------------------------------------------------------------------------
template <bool GATED>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs g) {
  __shared__ float sA[kFBM][kFBK + 1];
  __shared__ float sB[GATED ? 2 : 1][kFBK][kFBN];
  const int q = chunked_item(blockIdx.x, *g.n_items);
  if (q < 0) return;
  const int4 item = g.work[q];
  const int le = item.x, m0 = item.y, rows = item.z & kItemRowsMask, nt = item.w & ((1 << kTileShift) - 1);
  const int tid = threadIdx.x;
  const int ty = tid >> 4, tx = tid & 15;
  const float *A = static_cast<const float *>(g.A);
  const size_t wsz = (size_t)g.K * g.N;
  const float *W0 = static_cast<const float *>(g.Bp) + (size_t)le * wsz;
  // gate matrices of all local experts come first, then the up matrices
  const float *W1 = GATED ? W0 + (size_t)g.n_ktiles * wsz : nullptr;  // n_ktiles carries E_loc for this kernel

  const int ar = tid >> 2, akq = (tid & 3) * 4;
  const int arc = ar < rows ? ar : rows - 1;
  const int a_row = g.row_map ? g.row_map[m0 + arc] : m0 + arc;
  const float *a_src = A + (size_t)a_row * g.lda + akq;
  const int bk = tid >> 4, bn4 = (tid & 15) * 4;
  const int n0 = nt * kFBN;

  float accg[4][4] = {}, accu[4][4] = {};
  for (int k0 = 0; k0 < g.K; k0 += kFBK) {
    float4 av = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k0 + akq < g.K) av = *reinterpret_cast<const float4 *>(a_src + k0);
    sA[ar][akq + 0] = av.x; sA[ar][akq + 1] = av.y; sA[ar][akq + 2] = av.z; sA[ar][akq + 3] = av.w;
    float4 bv = make_float4(0.f, 0.f, 0.f, 0.f), bv1 = bv;
    if (k0 + bk < g.K && n0 + bn4 < g.N) {
      bv = *reinterpret_cast<const float4 *>(W0 + (size_t)(k0 + bk) * g.N + n0 + bn4);
      if (GATED) bv1 = *reinterpret_cast<const float4 *>(W1 + (size_t)(k0 + bk) * g.N + n0 + bn4);
    }
    *reinterpret_cast<float4 *>(&sB[0][bk][bn4]) = bv;
    if (GATED) *reinterpret_cast<float4 *>(&sB[GATED ? 1 : 0][bk][bn4]) = bv1;
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kFBK; ++kk) {
      float a[4], b0[4], b1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sA[ty * 4 + i][kk];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        b0[j] = sB[0][kk][tx + 16 * j];
        if (GATED) b1[j] = sB[GATED ? 1 : 0][kk][tx + 16 * j];
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          accg[i][j] = fmaf(a[i], b0[j], accg[i][j]);
          if (GATED) accu[i][j] = fmaf(a[i], b1[j], accu[i][j]);
        }
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row_l = ty * 4 + i;
    if (row_l >= rows) continue;
    const size_t grow = (size_t)(m0 + row_l);
    float *out = static_cast<float *>(g.out) + grow * g.ldo;
    const float w = GATED ? 1.f : g.row_w[grow];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx + 16 * j;
      if (col >= g.N) continue;
      if (GATED) {
        const float gv = accg[i][j];
        out[col] = (gv / (1.0f + expf(-gv))) * accu[i][j];
      } else {
        out[col] = accg[i][j] * w;
      }
    }
  }
}

}  // namespace moe355
