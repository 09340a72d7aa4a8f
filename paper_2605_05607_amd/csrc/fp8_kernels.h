// Quantisation to E4M3 for the FP8 form of the expert GEMMs (Sec. V-A runs the DeepSeek-V3 GEMMs in FP8 and gives
// no scheme; the one used: a scale per token for x, per expert and output column for the weights, a given static
// scale per expert for h; scale = largest magnitude of the group / 448, 1 for an all-zero group; code =
// convert(value / scale) with an fp32 division).
#pragma once
#include "forward_types.h"

namespace moe355 {

constexpr int kFp8KStep = 128;  // reduction indices per packed tile and k-step (128 bytes per row, as for bf16)

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// One workgroup per row of x [rows, cols] (bf16, cols % 8 == 0): codes [rows, cols], scales [rows].
__global__ __launch_bounds__(256) void fp8_quantize_rows_kernel(const uint4 *__restrict__ x, int cols,
                                                                uint8_t *__restrict__ codes,
                                                                float *__restrict__ scales) {
  __shared__ float wave_max[4];
  const size_t row = blockIdx.x;
  const int chunks = cols / 8;
  const uint4 *src = x + row * chunks;
  float amax = 0.f;
  for (int c = threadIdx.x; c < chunks; c += 256) {
    const uint4 v = src[c];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      amax = fmaxf(amax, fabsf(bf16_bits_to_f32(w[q] & 0xFFFFu)));
      amax = fmaxf(amax, fabsf(bf16_bits_to_f32(w[q] >> 16)));
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = amax;
  __syncthreads();
  amax = fmaxf(fmaxf(wave_max[0], wave_max[1]), fmaxf(wave_max[2], wave_max[3]));
  const float scale = amax > 0.f ? amax / 448.0f : 1.0f;
  if (threadIdx.x == 0) scales[row] = scale;
  uint2 *dst = reinterpret_cast<uint2 *>(codes + row * (size_t)cols);
  for (int c = threadIdx.x; c < chunks; c += 256) {
    const uint4 v = src[c];  // second read of the row: served by the caches
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t out[2] = {0u, 0u};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint32_t lo = to_e4m3(bf16_bits_to_f32(w[q] & 0xFFFFu) / scale);
      const uint32_t hi = to_e4m3(bf16_bits_to_f32(w[q] >> 16) / scale);
      out[q >> 1] |= (lo | (hi << 8)) << ((q & 1) * 16);
    }
    dst[c] = make_uint2(out[0], out[1]);
  }
}

// Largest magnitude of every output column of W [E_loc][K][N] (bf16) over one slice of the reduction index
// (blockIdx.z of gridDim.z slices), folded into amax [E_loc][pitch] with an integer atomic max (bit patterns of
// non-negative floats order like the floats, and a maximum does not depend on the order of its operands).  amax
// must be zero on entry.  grid (ceil(N / 256), E_loc, slices).
__global__ __launch_bounds__(256) void fp8_column_amax_kernel(const bf16_t *__restrict__ W, int K, int N,
                                                              uint32_t *__restrict__ amax, int pitch) {
  const int col = blockIdx.x * 256 + threadIdx.x, le = blockIdx.y;
  if (col >= N) return;
  const int per = (K + gridDim.z - 1) / gridDim.z;
  const int k0 = blockIdx.z * per, k1 = min(K, k0 + per);
  const bf16_t *w = W + (size_t)le * K * N + col;
  float m = 0.f;
#pragma unroll 8
  for (int kk = k0; kk < k1; ++kk) m = fmaxf(m, fabsf((float)w[(size_t)kk * N]));
  atomicMax(&amax[(size_t)le * pitch + col], __float_as_uint(m));
}

// amax -> scale in place: largest magnitude / 448, 1 for an all-zero column.
__global__ void fp8_scales_from_amax_kernel(float *__restrict__ s, size_t n) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const float a = s[i];
    s[i] = a > 0.f ? a / 448.0f : 1.0f;
  }
}

// Quantise and re-tile the weights (one-off).  The tile image is that of pack_bf16_kernel with 16 codes in every
// 16-byte operand: tile (le, nt, kt) covers kBN output columns x 128 reduction indices; for column block cb, step kk
// and lane l the 16 bytes at ((cb*4 + kk)*64 + l)*16 hold B[column cb*32 + l%32][k = kt*128 + (2 kk + l/32)*16 .. +16].
// GATED tiles pair gate and up columns as in the bf16 layout; s0 / s1 are the column scales of W0 / W1.
template <bool GATED>
__global__ __launch_bounds__(256) void pack_fp8_kernel(const bf16_t *__restrict__ W0, const bf16_t *__restrict__ W1,
                                                       const float *__restrict__ s0, const float *__restrict__ s1,
                                                       int scale_pitch, uint8_t *__restrict__ out, int K, int N,
                                                       int n_ntiles, int n_ktiles) {
  const int kt = blockIdx.x, nt = blockIdx.y, le = blockIdx.z;
  const int n_l = threadIdx.x;
  const int wn = n_l >> 6, j = (n_l >> 5) & 1, i = n_l & 31;
  const bf16_t *W = (GATED && j == 1) ? W1 : W0;
  const float *sc = (GATED && j == 1) ? s1 : s0;
  const int col = GATED ? nt * (kBN / 2) + wn * 32 + i : nt * kBN + n_l;
  const float scale = col < N ? sc[(size_t)le * scale_pitch + col] : 1.0f;
  const size_t wbase = (size_t)le * K * N;
  uint8_t *tile = out + ((size_t)(le * n_ntiles + nt) * n_ktiles + kt) * (size_t)kTileBytes;
  for (int c = 0; c < 8; ++c) {
    uint32_t v[4] = {0u, 0u, 0u, 0u};
    for (int q = 0; q < 16; ++q) {
      const int kk = kt * kFp8KStep + c * 16 + q;
      const uint32_t code = (col < N && kk < K) ? to_e4m3((float)W[wbase + (size_t)kk * N + col] / scale) : 0u;
      v[q >> 2] |= code << ((q & 3) * 8);
    }
    *reinterpret_cast<uint4 *>(tile + ((((n_l >> 5) * 4 + (c >> 1)) * 64 + (c & 1) * 32 + (n_l & 31)) << 4)) =
        make_uint4(v[0], v[1], v[2], v[3]);
  }
}

}  // namespace moe355
