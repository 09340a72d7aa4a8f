// Combine, the phase-split Dispatch copy and the pieces of the unfused comparison path.
#pragma once
#include "forward_types.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Combine: one workgroup per token sums the gate-weighted rows of the token's local slots in slot order
// (fp32) and writes the y row once; tokens without a local slot get zeros.
// ------------------------------------------------------------------------------------------------
template <typename OutT>
__device__ __forceinline__ void store8(OutT *dst, const float (&v)[8]);
template <>
__device__ __forceinline__ void store8<float>(float *dst, const float (&v)[8]) {
  *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4 *>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
template <>
__device__ __forceinline__ void store8<bf16_t>(bf16_t *dst, const float (&v)[8]) {
  bf16x8 o;
#pragma unroll
  for (int q = 0; q < 8; ++q) o[q] = (bf16_t)v[q];
  *reinterpret_cast<bf16x8 *>(dst) = o;
}

template <typename OutT>
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ rows,
                                                      const int32_t *__restrict__ topk_idx,
                                                      const int32_t *__restrict__ inv_perm,
                                                      const int32_t *__restrict__ offsets, int k, int d, int e_lo,
                                                      int E_loc, int P_cap, int skip_sole,
                                                      OutT *__restrict__ y) {
  __shared__ int srow[kMaxTopK];
  __shared__ int snum;
  const int t = blockIdx.x;
  if (threadIdx.x == 0) {
    const int base = offsets[e_lo];
    int n = 0;
    for (int j = 0; j < k; ++j) {
      const int e = topk_idx[(size_t)t * k + j];
      if (e < e_lo || e >= e_lo + E_loc) continue;
      const int row = inv_perm[(size_t)t * k + j] - base;
      if (row >= 0 && row < P_cap) srow[n++] = row;
    }
    snum = n;
  }
  __syncthreads();
  const int n = snum;
  if (n == 1 && skip_sole) return;  // GEMM-2 has written this token's row
  for (int c = threadIdx.x * 8; c < d; c += blockDim.x * 8) {
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int i = 0; i < n; ++i) {
      const float *src = rows + (size_t)srow[i] * d + c;
      const float4 lo = *reinterpret_cast<const float4 *>(src);
      const float4 hi = *reinterpret_cast<const float4 *>(src + 4);
      acc[0] += lo.x; acc[1] += lo.y; acc[2] += lo.z; acc[3] += lo.w;
      acc[4] += hi.x; acc[5] += hi.y; acc[6] += hi.z; acc[7] += hi.w;
    }
    store8<OutT>(y + (size_t)t * d + c, acc);
  }
}

// ------------------------------------------------------------------------------------------------
// Dispatch as a materialised copy (phase-split entry point): one workgroup per local dedup entry reads the
// token row once and writes it to the layout row of every slot in the entry's mask.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void dispatch_gather_kernel(const uint4 *__restrict__ x,
                                                              const int32_t *__restrict__ rank_offsets,
                                                              const int32_t *__restrict__ dedup_tok,
                                                              const uint32_t *__restrict__ dedup_mask,
                                                              const int32_t *__restrict__ inv_perm,
                                                              const int32_t *__restrict__ offsets, int T, int k,
                                                              int lrb, int lre, int e_lo, int P_cap, int row_chunks,
                                                              uint4 *__restrict__ xs) {
  const int u0 = rank_offsets[lrb];
  const int u = u0 + blockIdx.x;
  if (u >= rank_offsets[lre]) return;
  const int t = dedup_tok[u];
  uint32_t mask = dedup_mask[u];
  if (t < 0 || t >= T) return;
  const int base = offsets[e_lo];
  for (int c = threadIdx.x; c < row_chunks; c += blockDim.x) {
    const uint4 v = x[(size_t)t * row_chunks + c];
    uint32_t m = mask;
    while (m) {
      const int j = __builtin_ctz(m);
      m &= m - 1;
      if (j >= k) break;
      const int row = inv_perm[(size_t)t * k + j] - base;
      if (row >= 0 && row < P_cap) xs[(size_t)row * row_chunks + c] = v;
    }
  }
}

// ---- pieces of the unfused comparison path ----
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4 *__restrict__ x,
                                                          const int32_t *__restrict__ header,
                                                          const int32_t *__restrict__ row_tok, int row_chunks,
                                                          uint4 *__restrict__ xs) {
  const int r = blockIdx.x;
  if (r >= header[1]) return;
  const int t = row_tok[r];
  for (int c = threadIdx.x; c < row_chunks; c += blockDim.x)
    xs[(size_t)r * row_chunks + c] = x[(size_t)t * row_chunks + c];
}

__global__ void fill_zero_kernel(float4 *__restrict__ p, size_t n4) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x)
    p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

__global__ __launch_bounds__(256) void scatter_add_kernel(const float *__restrict__ rows,
                                                          const int32_t *__restrict__ header,
                                                          const int32_t *__restrict__ row_tok, int d,
                                                          float *__restrict__ y32) {
  const int r = blockIdx.x;
  if (r >= header[1]) return;
  const int t = row_tok[r];
  for (int c = threadIdx.x; c < d; c += blockDim.x) atomicAdd(&y32[(size_t)t * d + c], rows[(size_t)r * d + c]);
}

template <typename OutT>
__global__ __launch_bounds__(256) void cast_rows_kernel(const float *__restrict__ y32, OutT *__restrict__ y,
                                                        size_t n8) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n8; i += (size_t)gridDim.x * blockDim.x) {
    float v[8];
    const float4 lo = *reinterpret_cast<const float4 *>(y32 + i * 8);
    const float4 hi = *reinterpret_cast<const float4 *>(y32 + i * 8 + 4);
    v[0] = lo.x; v[1] = lo.y; v[2] = lo.z; v[3] = lo.w; v[4] = hi.x; v[5] = hi.y; v[6] = hi.z; v[7] = hi.w;
    store8<OutT>(y + i * 8, v);
  }
}

}  // namespace moe355
