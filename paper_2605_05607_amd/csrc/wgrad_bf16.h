// Weight gradients of the expert FFN on the matrix cores: for every local expert, C = A^T B summed over the expert's
// rows (dW_gate = x^T dg, dW_up = x^T du, dW_down = (w h)^T dy).  The reduction index is the row, which is the slow
// index of both operands in memory, while a matrix-core operand wants 8 consecutive reduction indices per lane; so
// the operands are first transposed (and gathered: x and dy rows are fetched by token) into [column][row] buffers
// in which every expert's rows start at a multiple of 64 and are zero-padded to a multiple of 64.  The GEMM then is
// the forward tile's main loop with both operands staged like its A operand.
#pragma once
#include "gemm_bf16.h"

namespace moe355 {

// kb[le] = first 64-row block of local expert le in the padded row order, kb[E_loc] = number of blocks.
__global__ __launch_bounds__(256) void wgrad_blocks_kernel(const int32_t *__restrict__ offsets,
                                                           const int32_t *__restrict__ header, int e_lo, int E_loc,
                                                           int32_t *__restrict__ kb) {
  __shared__ int scratch[17];
  const int P = header[1], base = header[2];
  const int ipt = (E_loc + 255) / 256;
  const int lo = min(E_loc, (int)threadIdx.x * ipt), hi = min(E_loc, lo + ipt);
  int mine = 0;
  for (int le = lo; le < hi; ++le) {
    const int cnt = max(0, min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base));
    mine += (cnt + 63) >> 6;
  }
  int total;
  int run = block_exclusive_scan(mine, scratch, &total);
  for (int le = lo; le < hi; ++le) {
    const int cnt = max(0, min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base));
    kb[le] = run;
    run += (cnt + 63) >> 6;
  }
  if (threadIdx.x == 0) kb[E_loc] = total;
}

// dst[c][64 b + i] = src[row(r)][c0 + c] for the i-th row r of padded block b (zero where the block is padded),
// c < C.  src rows have pitch ld; row(r) = row_map[r] or r.  dst has pitch kpad.  grid (ceil(C / 64), block cap).
__global__ __launch_bounds__(256) void gather_transpose_kernel(const bf16_t *__restrict__ src,
                                                               const int32_t *__restrict__ row_map, int ld, int c0,
                                                               int C, const int32_t *__restrict__ offsets,
                                                               const int32_t *__restrict__ header,
                                                               const int32_t *__restrict__ kb, int e_lo, int E_loc,
                                                               bf16_t *__restrict__ dst, size_t kpad) {
  __shared__ uint16_t tile[64][66];  // [row][column], 33 words per row: column reads hit distinct banks
  const int b = blockIdx.y;
  if (b >= kb[E_loc]) return;
  int lo = 0, hi = E_loc;  // expert that owns block b: largest le with kb[le] <= b (empty experts own no block)
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (kb[mid] <= b) lo = mid; else hi = mid;
  }
  const int le = lo;
  const int P = header[1], base = header[2];
  const int start = min(P, offsets[e_lo + le] - base);
  const int cnt = max(0, min(P, offsets[e_lo + le + 1] - base) - start);
  const int r_first = (b - kb[le]) * 64;  // first row of this block inside the expert
  const int cblk = blockIdx.x * 64;
  // load: thread t -> rows (t >> 3) and (t >> 3) + 32, 16-byte chunk t & 7
  for (int i = 0; i < 2; ++i) {
    const int rl = (threadIdx.x >> 3) + 32 * i, ch = threadIdx.x & 7;
    u32x4 v = {0u, 0u, 0u, 0u};
    const int c = cblk + ch * 8;
    if (r_first + rl < cnt && c < C) {
      const int r = start + r_first + rl;
      const size_t row = row_map ? (size_t)row_map[r] : (size_t)r;
      v = *reinterpret_cast<const u32x4 *>(src + row * ld + c0 + c);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      tile[rl][ch * 8 + 2 * q] = (uint16_t)(v[q] & 0xFFFFu);
      tile[rl][ch * 8 + 2 * q + 1] = (uint16_t)(v[q] >> 16);
    }
  }
  __syncthreads();
  // store: thread t -> columns (t >> 3) and (t >> 3) + 32, rows 8 (t & 7) .. + 8 as one 16-byte chunk
  for (int i = 0; i < 2; ++i) {
    const int cl = (threadIdx.x >> 3) + 32 * i, ch = threadIdx.x & 7;
    if (cblk + cl >= C) continue;
    u32x4 v;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      v[q] = (uint32_t)tile[ch * 8 + 2 * q][cl] | ((uint32_t)tile[ch * 8 + 2 * q + 1][cl] << 16);
    *reinterpret_cast<u32x4 *>(dst + (size_t)(cblk + cl) * kpad + (size_t)b * 64 + ch * 8) = v;
  }
}

struct WgradArgs {
  const bf16_t *AT;   // [M][kpad]  transposed left operand (rows = columns of the original row-major operand)
  const bf16_t *BT;   // [N][kpad]
  bf16_t *C;          // [E_loc][M][N]
  const int32_t *kb;  // [E_loc + 1]
  size_t kpad;
  int M, N, n_mt, n_nt;
};

// One workgroup per (local expert, 256 x 256 output tile); 8 waves = 2 x 4, each 128 x 64 as 4 x 2 accumulators.
// LDS: two stages of (A 256 x 64, B 256 x 64), rows of 128 bytes with the forward tile's chunk swizzle.
__global__ __launch_bounds__(kGemmThreads, 1) void wgrad_bf16_kernel(const WgradArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, w8 = tid >> 6;
  const int wm = w8 >> 2, wn = w8 & 3;
  const int le = blockIdx.y;
  const int mt = blockIdx.x / a.n_nt, nt = blockIdx.x % a.n_nt;
  const int m0 = mt * kBM, n0 = nt * kBN;
  const int kb0 = a.kb[le], KT = a.kb[le + 1] - kb0;

  const int chunk = tid & 7, row0 = tid >> 3;  // rows row0 + 64 i
  const bf16_t *ap[4], *bp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ap[i] = a.AT + (size_t)min(m0 + row0 + 64 * i, a.M - 1) * a.kpad + (size_t)kb0 * 64 + chunk * 8;
    bp[i] = a.BT + (size_t)min(n0 + row0 + 64 * i, a.N - 1) * a.kpad + (size_t)kb0 * 64 + chunk * 8;
  }
  const int dst = (row0 * 8 + (chunk ^ ((row0 >> 1) & 7))) * 16;  // + 8192 per 64 rows; B stage 32768 further
  u32x4 ra[4], rb[4];

  f32x16 acc[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][j][r] = 0.f;

  const int l31 = lane & 31, khalf = lane >> 5, sw = (lane >> 1) & 7;
  if (KT > 0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ra[i] = *reinterpret_cast<const u32x4 *>(ap[i]);
      rb[i] = *reinterpret_cast<const u32x4 *>(bp[i]);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<u32x4 *>(smem + dst + 8192 * i) = ra[i];
      *reinterpret_cast<u32x4 *>(smem + 32768 + dst + 8192 * i) = rb[i];
    }
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
      const unsigned char *st = smem + (kt & 1) * kStageBytes;
      if (kt + 1 < KT) {  // uniform
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          ra[i] = *reinterpret_cast<const u32x4 *>(ap[i] + (size_t)(kt + 1) * 64);
          rb[i] = *reinterpret_cast<const u32x4 *>(bp[i] + (size_t)(kt + 1) * 64);
        }
      }
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int slot = ((kk * 2 + khalf) ^ sw) * 16;
        bf16x8 fa[4], fb[2];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
          fa[mi] = *reinterpret_cast<const bf16x8 *>(st + (wm * 128 + mi * 32 + l31) * 128 + slot);
#pragma unroll
        for (int j = 0; j < 2; ++j)
          fb[j] = *reinterpret_cast<const bf16x8 *>(st + 32768 + (wn * 64 + j * 32 + l31) * 128 + slot);
#pragma unroll
        for (int mi = 0; mi < 4; ++mi) {
          acc[mi][0] = mfma_bf16(fa[mi], fb[0], acc[mi][0]);
          acc[mi][1] = mfma_bf16(fa[mi], fb[1], acc[mi][1]);
        }
      }
      if (kt + 1 < KT) {
        unsigned char *nx = smem + ((kt + 1) & 1) * kStageBytes;  // last read before the previous barrier
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          *reinterpret_cast<u32x4 *>(nx + dst + 8192 * i) = ra[i];
          *reinterpret_cast<u32x4 *>(nx + 32768 + dst + 8192 * i) = rb[i];
        }
      }
      __syncthreads();
    }
  }
  // epilogue: each wave turns its 32 x 64 blocks around through a private LDS patch (fp32, row pitch 288 bytes) so
  // that a row leaves as contiguous bf16
  __syncthreads();
  unsigned char *patch = smem + w8 * kPatchBytes;
  bf16_t *C = a.C + (size_t)le * a.M * a.N;
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
      *reinterpret_cast<float *>(patch + rl * 288 + l31 * 4) = acc[mi][0][r];
      *reinterpret_cast<float *>(patch + rl * 288 + 128 + l31 * 4) = acc[mi][1][r];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const int rl = it * 4 + (lane >> 4), cc = lane & 15;  // 16 groups of 4 columns per row
      const int m = m0 + wm * 128 + mi * 32 + rl, n = n0 + wn * 64 + cc * 4;
      const f32x4 v = *reinterpret_cast<const f32x4 *>(patch + rl * 288 + cc * 16);
      if (m < a.M && n < a.N) {  // N % 8 == 0: the four columns are inside together
        bf16x4 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = (bf16_t)v[q];
        *reinterpret_cast<bf16x4 *>(C + (size_t)m * a.N + n) = o;
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace moe355
