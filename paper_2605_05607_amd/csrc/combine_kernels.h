// Combine, the phase-split Dispatch copy and the pieces of the unfused comparison path.
#pragma once
#include "forward_types.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Combine: one wave per token sums the gate-weighted rows of the token's local slots in slot order (fp32) and
// writes the y row once; tokens without a local slot get zeros.  The slots are resolved by the lanes of the wave
// (one slot each), not serially.  (Measured against the earlier form, one workgroup per token with the slots resolved
// by its first thread: the same 5.0-5.2 TB/s from HBM, i.e. the rate this machine copies at; loading the rows with
// the non-temporal hint was 10 % slower.)
// ------------------------------------------------------------------------------------------------
// Eight consecutive outputs.  STREAM: with the non-temporal hint (a y row inside the fused call: nothing of the call
// reads it again, and the next call's operands keep their place in the caches).
template <typename OutT, bool STREAM = false>
__device__ __forceinline__ void store8(OutT *dst, const float (&v)[8]) {
  if constexpr (sizeof(OutT) == 4) {
    *reinterpret_cast<float4 *>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
  } else {
    bf16x8 o;
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = (bf16_t)v[q];
    if constexpr (STREAM)
      __builtin_nontemporal_store(o, reinterpret_cast<bf16x8 *>(dst));
    else
      *reinterpret_cast<bf16x8 *>(dst) = o;
  }
}

// The sum of one token's rows by one wave.  `row` holds, in the lanes named by `slots`, the layout rows of the token's
// local slots (lane = slot index); the rows are added in slot order, starting from zero, in fp32.  Four pieces of 512
// columns at a time (8 per lane each) and the loads of two slots in flight together.  poison: write NaN instead.
template <typename OutT, bool STREAM = false>
__device__ __forceinline__ void combine_token_rows(const float *__restrict__ rows, int row, uint64_t slots, int d,
                                                   OutT *__restrict__ yrow, int lane, int poison) {
  for (int c0 = lane * 8; c0 < d; c0 += 4 * 512) {
    float acc[4][8];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int q = 0; q < 8; ++q) acc[u][q] = 0.f;
    uint64_t s = slots;
    while (s) {
      const int j0 = __builtin_ctzll(s);
      s &= s - 1;
      const float *src0 = rows + (size_t)__builtin_amdgcn_readlane(row, j0) * d;
      const bool two = s != 0;
      const int j1 = two ? __builtin_ctzll(s) : j0;
      s &= s - 1;  // (0 stays 0)
      const float *src1 = rows + (size_t)__builtin_amdgcn_readlane(row, j1) * d;
      f32x4 a[4][2], b[4][2];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int c = c0 + u * 512;
        if (c < d) {
          a[u][0] = *reinterpret_cast<const f32x4 *>(src0 + c);
          a[u][1] = *reinterpret_cast<const f32x4 *>(src0 + c + 4);
          if (two) {
            b[u][0] = *reinterpret_cast<const f32x4 *>(src1 + c);
            b[u][1] = *reinterpret_cast<const f32x4 *>(src1 + c + 4);
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (c0 + u * 512 < d) {
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[u][q] += a[u][q >> 2][q & 3];
          if (two) {
#pragma unroll
            for (int q = 0; q < 8; ++q) acc[u][q] += b[u][q >> 2][q & 3];
          }
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int c = c0 + u * 512;
      if (c < d) {
        if (poison) {
#pragma unroll
          for (int q = 0; q < 8; ++q) acc[u][q] = __builtin_nanf("");
        }
        store8<OutT, STREAM>(yrow + c, acc[u]);
      }
    }
  }
}

// Layout row of slot `lane` of token t if that slot is local (else -1): one lane per slot.
__device__ __forceinline__ int combine_slot_row(const int32_t *__restrict__ topk_idx,
                                                const int32_t *__restrict__ inv_perm, int t, int k, int lane,
                                                int e_lo, int E_loc, int base, int row_limit) {
  if (lane >= k) return -1;
  const int e = topk_idx[(size_t)t * k + lane];
  if (e < e_lo || e >= e_lo + E_loc) return -1;
  const int r = inv_perm[(size_t)t * k + lane] - base;
  return r >= 0 && r < row_limit ? r : -1;
}

constexpr int kCombineWaves = 4;  // tokens per workgroup of combine_kernel: one per wave

// FUSED (inside the fused calls): tokens with one local slot are skipped, GEMM-2 has written their rows, and the y rows
// leave with the non-temporal hint; the stand-alone Combine writes every row with plain stores (measured from HBM on
// rotated buffers it is 5 % slower with the hint, while the fused forward on the DeepSeek-shaped layer gains 1.3 %).
template <typename OutT, bool FUSED>
__global__ __launch_bounds__(kCombineWaves * 64) void combine_kernel(const float *__restrict__ rows,
                                                                     const int32_t *__restrict__ topk_idx,
                                                                     const int32_t *__restrict__ inv_perm,
                                                                     const int32_t *__restrict__ offsets, int T, int k,
                                                                     int d, int e_lo, int E_loc, int P_cap,
                                                                     OutT *__restrict__ y) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * kCombineWaves + (threadIdx.x >> 6);  // wave-uniform
  if (t >= T) return;
  const int row = combine_slot_row(topk_idx, inv_perm, t, k, lane, e_lo, E_loc, offsets[e_lo], P_cap);
  const uint64_t slots = __ballot(row >= 0);
  if (FUSED && __popcll(slots) == 1) return;  // GEMM-2 has written this token's row
  combine_token_rows<OutT, FUSED>(rows, row, slots, d, y + (size_t)t * d, lane, 0);
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
