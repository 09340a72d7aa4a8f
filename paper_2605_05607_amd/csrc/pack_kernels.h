// One-off re-tiling of the expert weights into the layout the GEMM kernels stream.
#pragma once
#include "forward_types.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Weight packing (one-off).  Output tile (le, nt, kt) covers kBN output columns x kBK reduction indices (32 KiB)
// and is stored in the order the matrix-core instruction consumes it: for every block cb of 32 columns and every
// 16-wide reduction step kk, the 64 lanes' B operands of v_mfma_f32_32x32x16_bf16 lie next to each other, lane l
// holding the 8 values B[column cb*32 + l%32][k = kk*16 + (l/32)*8 .. +8] at byte ((cb*4 + kk)*64 + l)*16.
// The GEMM kernels copy a tile linearly into the LDS (16 bytes per lane, fully coalesced) and a wave reads an
// operand as one contiguous KiB (no bank conflicts); a wave can equally load an operand straight from global
// memory with one coalesced 1 KiB access.  Zero-padded outside the matrix.
// GATED tiles pair gate and up columns inside one wave column: blocks cb = 2 wn and 2 wn + 1 are the gate and the
// up columns nt*128 + wn*32 + 0..31 of the same h columns.
// ------------------------------------------------------------------------------------------------
template <bool GATED>
__global__ __launch_bounds__(256) void pack_bf16_kernel(const bf16_t *__restrict__ W0, const bf16_t *__restrict__ W1,
                                                        bf16_t *__restrict__ out, int K, int N, int n_ntiles,
                                                        int n_ktiles) {
  // grid: x = kt, y = nt, z = le;   256 threads: thread = tile row n_l, loops over the 8 chunks
  const int kt = blockIdx.x, nt = blockIdx.y, le = blockIdx.z;
  const int n_l = threadIdx.x;
  const int wn = n_l >> 6, j = (n_l >> 5) & 1, i = n_l & 31;
  const bf16_t *W = (GATED && j == 1) ? W1 : W0;
  const int col = GATED ? nt * (kBN / 2) + wn * 32 + i : nt * kBN + n_l;
  const size_t wbase = (size_t)le * K * N;
  bf16_t *tile = out + ((size_t)(le * n_ntiles + nt) * n_ktiles + kt) * (kBN * kBK);
  for (int c = 0; c < 8; ++c) {
    bf16x8 v;
    for (int q = 0; q < 8; ++q) {
      const int kk = kt * kBK + c * 8 + q;
      v[q] = (col < N && kk < K) ? W[wbase + (size_t)kk * N + col] : (bf16_t)0.0f;
    }
    // chunk c = 2 kk + k-half; column block cb = n_l >> 5
    *reinterpret_cast<bf16x8 *>(tile + ((((n_l >> 5) * 4 + (c >> 1)) * 64 + (c & 1) * 32 + (n_l & 31)) << 3)) = v;
  }
}

// The same tile image from a source whose rows are the OUTPUT columns (the transposed use of a weight matrix in the
// backward pass): B[k][n] = W[n][k], W = [E_loc][N][K] with K contiguous, so a thread's 8 values are one 16-byte
// load.  The tiles go to reduction tiles kt_offset + kt of n_ktiles_total (two sources can share one reduction
// range: the gate weights, then the up weights).
__global__ __launch_bounds__(256) void pack_bf16_transposed_kernel(const bf16_t *__restrict__ W,
                                                                   bf16_t *__restrict__ out, int K, int N,
                                                                   int n_ntiles, int n_ktiles_total, int kt_offset) {
  const int kt = blockIdx.x, nt = blockIdx.y, le = blockIdx.z;
  const int n_l = threadIdx.x;
  const int col = nt * kBN + n_l;
  const bf16_t *src = W + ((size_t)le * N + (col < N ? col : 0)) * K;
  bf16_t *tile = out + ((size_t)(le * n_ntiles + nt) * n_ktiles_total + kt_offset + kt) * (kBN * kBK);
  for (int c = 0; c < 8; ++c) {
    const int kk = kt * kBK + c * 8;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (col < N && kk < K) v = *reinterpret_cast<const u32x4 *>(src + kk);  // K % 8 == 0: the chunk is inside the row
    *reinterpret_cast<u32x4 *>(tile + ((((n_l >> 5) * 4 + (c >> 1)) * 64 + (c & 1) * 32 + (n_l & 31)) << 3)) = v;
  }
}

__global__ void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

}  // namespace moe355
