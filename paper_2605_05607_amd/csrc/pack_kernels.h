// One-off re-tiling of the expert weights into the layout the GEMM kernels stream.
#pragma once
#include "forward_types.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Weight packing (one-off).  Output tile (le, nt, kt) covers kBN output columns x kBK reduction indices and is
// the byte image of the LDS stage the GEMM kernel reads, so the kernel copies it linearly (16 bytes per lane,
// fully coalesced):  row n_l of the tile is the 128-byte run of its 64 k values, cut into eight 16-byte
// chunks; chunk c of row n_l sits at slot c ^ ((n_l >> 1) & 7).  The LDS of gfx950 has 64 four-byte banks, so
// a 128-bit operand read is served 16 lanes at a time; with this swizzle the 16 rows such a group touches
// fall on 16 different bank groups (measured: zero bank-conflict cycles).  Zero-padded outside the matrix.
// GATED tiles pair gate and up columns inside one wave column: tile rows [wn*64, wn*64+32) are the gate
// columns nt*128 + wn*32 + 0..31 and rows [wn*64+32, wn*64+64) the up columns of the same h columns.
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
    *reinterpret_cast<bf16x8 *>(tile + (size_t)n_l * kBK + ((c ^ ((n_l >> 1) & 7)) << 3)) = v;
  }
}

__global__ void copy_f32_kernel(const float *__restrict__ src, float *__restrict__ dst, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

}  // namespace moe355
