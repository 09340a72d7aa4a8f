// Weight gradients of the expert FFN on the matrix cores: for every local expert, C = A^T B summed over the expert's
// rows (dW_gate = x^T dg, dW_up = x^T du, dW_down = (w h)^T dy).  The reduction index is the row, which is the slow
// index of both operands in memory, while a matrix-core operand wants 8 consecutive reduction indices per lane; so
// the operands are first transposed (and gathered: x and dy rows are fetched by token) into buffers of 64-row blocks,
// [block][column][64 rows], in which every expert's rows start at a block boundary and are zero-padded to one: what
// a workgroup stages per k-step is then one contiguous piece of memory per operand.  The GEMM is the forward tile's
// main loop with both operands staged like its A operand.
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

// dst[b][c][i] = src[row(r)][c0 + c] for the i-th row r of padded block b (zero where the block is padded), c < C,
// i < 64.  src rows have pitch ld; row(r) = row_map[r] or r.  grid (ceil(C / 64), block cap).
__global__ __launch_bounds__(256) void gather_transpose_kernel(const bf16_t *__restrict__ src,
                                                               const int32_t *__restrict__ row_map, int ld, int c0,
                                                               int C, const int32_t *__restrict__ offsets,
                                                               const int32_t *__restrict__ header,
                                                               const int32_t *__restrict__ kb, int e_lo, int E_loc,
                                                               bf16_t *__restrict__ dst) {
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
    *reinterpret_cast<u32x4 *>(dst + ((size_t)b * C + cblk + cl) * 64 + ch * 8) = v;
  }
}

struct WgradArgs {
  const bf16_t *AT;   // [block][lda][64]: rows a0 .. a0 + M of every block are the left operand's columns
  const bf16_t *BT;   // [block][ldb][64]: rows b0 .. b0 + N
  bf16_t *C;          // [E_loc][M][N]
  const int32_t *kb;  // [E_loc + 1]
  int lda, ldb, a0, b0;
  int M, N, n_mt, n_nt;
};

// Experts with at most kThinSteps blocks of 64 rows are left to wgrad_thin_bf16_kernel (those without rows to
// wgrad_zero_empty_kernel): their cost is writing the output, and that kernel's small workgroups overlap the stores of
// one tile with the loads of the next on the same CU.
constexpr int kThinSteps = 2;
constexpr int kThinTiles = 4;  // output tiles per workgroup of wgrad_thin_bf16_kernel

// Zero gradients of the local experts without rows: grid (shares, E_loc, 3 matrices), each workgroup clears one
// contiguous share of `units` 16-byte units.  Few registers and no LDS on purpose: its waves fit beside a GEMM
// workgroup on the same CU.
__global__ __launch_bounds__(256) void wgrad_zero_empty_kernel(const int32_t *__restrict__ kb, u32x4 *c0, u32x4 *c1,
                                                               u32x4 *c2, size_t units) {
  const int le = blockIdx.y;
  if (kb[le + 1] != kb[le]) return;
  u32x4 *C = (blockIdx.z == 0 ? c0 : blockIdx.z == 1 ? c1 : c2) + (size_t)le * units;
  const size_t share = (units + gridDim.x - 1) / gridDim.x;
  const size_t u0 = blockIdx.x * share, u1 = u0 + share < units ? u0 + share : units;
  const u32x4 zero = {0u, 0u, 0u, 0u};
  for (size_t u = u0 + threadIdx.x; u < u1; u += 256) __builtin_nontemporal_store(zero, &C[u]);
}

// The gradients are written once and not read again by this library: all three kernels below store them with the
// non-temporal hint, so that 0.9 GB of output per product does not push the operands, which every tile of an expert
// shares, out of the L2s (measured: -9 % of the weight-gradient time on the GPT-OSS-shaped layer, -6.5 % on the
// Mixtral-shaped one, -9 % on the Qwen3-shaped one, -2 % on the DeepSeek-shaped one).
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
  if (KT <= kThinSteps) return;  // whole workgroup: the thin kernel owns this expert

  const int chunk = tid & 7, row0 = tid >> 3;  // rows row0 + 64 i
  const bf16_t *ap[4], *bp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    ap[i] = a.AT + ((size_t)kb0 * a.lda + a.a0 + min(m0 + row0 + 64 * i, a.M - 1)) * 64 + chunk * 8;
    bp[i] = a.BT + ((size_t)kb0 * a.ldb + a.b0 + min(n0 + row0 + 64 * i, a.N - 1)) * 64 + chunk * 8;
  }
  const int dst = (row0 * 8 + (chunk ^ ((row0 >> 1) & 7))) * 16;  // + 8192 per 64 rows; B stage 32768 further
  const size_t a_step = (size_t)a.lda * 64, b_step = (size_t)a.ldb * 64;  // elements from one block to the next
  u32x4 ra[4], rb[4];

  f32x16 acc[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][j][r] = 0.f;

  const int l31 = lane & 31, khalf = lane >> 5, sw = (lane >> 1) & 7;
  const int a_rd = (wm * 128 + l31) * 128;            // + mi * 4096
  const int b_rd = 32768 + (wn * 64 + l31) * 128;     // + j * 4096
  bf16x8 fa0[4], fb0[2], fa1[4], fb1[2];  // operand fragments of two consecutive substeps
#define MOE355_W_READ(FA, FB, STAGE, KK)                                                           \
  do {                                                                                             \
    const int slot_ = (((KK) * 2 + khalf) ^ sw) * 16;                                              \
    _Pragma("unroll") for (int mi = 0; mi < 4; ++mi) FA[mi] =                                      \
        *reinterpret_cast<const bf16x8 *>((STAGE) + a_rd + mi * 4096 + slot_);                     \
    FB[0] = *reinterpret_cast<const bf16x8 *>((STAGE) + b_rd + slot_);                             \
    FB[1] = *reinterpret_cast<const bf16x8 *>((STAGE) + b_rd + 4096 + slot_);                      \
  } while (0)
#define MOE355_W_MFMAS(FA, FB)                                                                     \
  do {                                                                                             \
    _Pragma("unroll") for (int mi = 0; mi < 4; ++mi) {                                             \
      acc[mi][0] = mfma_bf16(FA[mi], FB[0], acc[mi][0]);                                           \
      acc[mi][1] = mfma_bf16(FA[mi], FB[1], acc[mi][1]);                                           \
    }                                                                                              \
  } while (0)
  // the slab in flight moves in three portions {a0, a1, b0}, {a2, a3, b1}, {b2, b3}: stored into the other stage and
  // reloaded for the slab after it, spread under the matrix instructions as in the forward tile
#define MOE355_W_STORE(NX, I0, I1, J0, J1)                                                         \
  do {                                                                                             \
    if ((I0) >= 0) *reinterpret_cast<u32x4 *>((NX) + dst + 8192 * (I0)) = ra[(I0) < 0 ? 0 : (I0)]; \
    if ((I1) >= 0) *reinterpret_cast<u32x4 *>((NX) + dst + 8192 * (I1)) = ra[(I1) < 0 ? 0 : (I1)]; \
    *reinterpret_cast<u32x4 *>((NX) + 32768 + dst + 8192 * (J0)) = rb[(J0)];                       \
    if ((J1) >= 0) *reinterpret_cast<u32x4 *>((NX) + 32768 + dst + 8192 * (J1)) = rb[(J1) < 0 ? 0 : (J1)]; \
  } while (0)
#define MOE355_W_LOAD(KP, I0, I1, J0, J1)                                                          \
  do {                                                                                             \
    if ((I0) >= 0) ra[(I0) < 0 ? 0 : (I0)] = *reinterpret_cast<const u32x4 *>(ap[(I0) < 0 ? 0 : (I0)] + (size_t)(KP) * a_step); \
    if ((I1) >= 0) ra[(I1) < 0 ? 0 : (I1)] = *reinterpret_cast<const u32x4 *>(ap[(I1) < 0 ? 0 : (I1)] + (size_t)(KP) * a_step); \
    rb[(J0)] = *reinterpret_cast<const u32x4 *>(bp[(J0)] + (size_t)(KP) * b_step);                 \
    if ((J1) >= 0) rb[(J1) < 0 ? 0 : (J1)] = *reinterpret_cast<const u32x4 *>(bp[(J1) < 0 ? 0 : (J1)] + (size_t)(KP) * b_step); \
  } while (0)
  /* order as in the forward tile: reads two behind each of the first three MFMAs, a store and a load behind each of
     the next NW, the remaining MFMAs last */
#define MOE355_W_ORDER(NW)                                                                         \
  do {                                                                                             \
    _Pragma("unroll") for (int i_ = 0; i_ < 3; ++i_) {                                             \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                           \
      __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);                                           \
    }                                                                                              \
    _Pragma("unroll") for (int i_ = 0; i_ < (NW); ++i_) {                                          \
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                           \
      __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                                           \
      __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                           \
    }                                                                                              \
    __builtin_amdgcn_sched_group_barrier(0x008, 5 - (NW), 0);                                      \
  } while (0)
  {
    const int kt_last = KT - 1;  // KT > kThinSteps >= 1
    MOE355_W_LOAD(0, 0, 1, 0, -1); MOE355_W_LOAD(0, 2, 3, 1, -1); MOE355_W_LOAD(0, -1, -1, 2, 3);
    MOE355_W_STORE(smem, 0, 1, 0, -1); MOE355_W_STORE(smem, 2, 3, 1, -1); MOE355_W_STORE(smem, -1, -1, 2, 3);
    {
      const int k1 = min(1, kt_last);
      MOE355_W_LOAD(k1, 0, 1, 0, -1); MOE355_W_LOAD(k1, 2, 3, 1, -1); MOE355_W_LOAD(k1, -1, -1, 2, 3);
    }
    __syncthreads();
    MOE355_W_READ(fa0, fb0, smem, 0);
    for (int kt = 0; kt < KT; ++kt) {
      const unsigned char *cur = smem + (kt & 1) * kStageBytes;
      unsigned char *nx = smem + ((kt & 1) ^ 1) * kStageBytes;
      const int kp = min(kt + 2, kt_last);  // past the end: the last slab again (in bounds, never used)
      MOE355_W_READ(fa1, fb1, cur, 1);
      MOE355_W_MFMAS(fa0, fb0);
      MOE355_W_STORE(nx, 0, 1, 0, -1);
      MOE355_W_LOAD(kp, 0, 1, 0, -1);
      MOE355_W_READ(fa0, fb0, cur, 2);
      MOE355_W_MFMAS(fa1, fb1);
      MOE355_W_STORE(nx, 2, 3, 1, -1);
      MOE355_W_LOAD(kp, 2, 3, 1, -1);
      MOE355_W_READ(fa1, fb1, cur, 3);
      MOE355_W_MFMAS(fa0, fb0);
      MOE355_W_STORE(nx, -1, -1, 2, 3);
      MOE355_W_LOAD(kp, -1, -1, 2, 3);
      MOE355_W_ORDER(3);
      MOE355_W_ORDER(3);
      MOE355_W_ORDER(2);
      __syncthreads();
      MOE355_W_READ(fa0, fb0, nx, 0);
      MOE355_W_MFMAS(fa1, fb1);
      MOE355_W_ORDER(0);
    }
  }
#undef MOE355_W_READ
#undef MOE355_W_MFMAS
#undef MOE355_W_STORE
#undef MOE355_W_LOAD
#undef MOE355_W_ORDER
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
    for (int it = 0; it < 4; ++it) {
      const int rl = it * 8 + (lane >> 3), cc = lane & 7;  // 8 groups of 8 columns per row: 16-byte stores
      const int m = m0 + wm * 128 + mi * 32 + rl, n = n0 + wn * 64 + cc * 8;
      const f32x4 v0 = *reinterpret_cast<const f32x4 *>(patch + rl * 288 + cc * 32);
      const f32x4 v1 = *reinterpret_cast<const f32x4 *>(patch + rl * 288 + cc * 32 + 16);
      if (m < a.M && n < a.N) {  // N % 8 == 0: the eight columns are inside together
        bf16x8 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          o[q] = (bf16_t)v0[q];
          o[4 + q] = (bf16_t)v1[q];
        }
        __builtin_nontemporal_store(o, reinterpret_cast<bf16x8 *>(C + (size_t)m * a.N + n));
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// Experts with 0 .. kThinSteps blocks of rows: 128 x 128 output tiles, 4 waves = 2 x 2, each 64 x 64; one LDS stage of
// (A 128 x 64, B 128 x 64) = 32 KiB (the epilogue patches reuse it) and at most 128 registers, so that four workgroups
// share a CU.  (Measured on the DeepSeek-shaped layer: four workgroups per CU instead of three -2.5 %, four tiles per
// workgroup -1.5 % of the weight-gradient time; requesting the next tile's operands ahead of the epilogue needs 150
// registers, i.e. three workgroups per CU, and comes out the same.)
// grid (ceil(n_mt * n_nt / kThinTiles), E_loc); a.n_mt / a.n_nt count 128-tiles here.
__global__ __launch_bounds__(256, 4) void wgrad_thin_bf16_kernel(const WgradArgs a) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * kPatchBytes];  // 36 KiB >= one 32 KiB stage
  const int tid = threadIdx.x, lane = tid & 63, w4 = tid >> 6;
  const int wm = w4 >> 1, wn = w4 & 1;
  const int le = blockIdx.y;
  const int kb0 = a.kb[le], KT = a.kb[le + 1] - kb0;
  if (KT > kThinSteps || KT == 0) return;  // whole workgroup: wgrad_bf16_kernel / wgrad_zero_empty_kernel own this expert
  const int chunk = tid & 7, row0 = tid >> 3;  // rows row0 + 32 i
  const int l31 = lane & 31, khalf = lane >> 5, sw = (lane >> 1) & 7;
  // kThinTiles consecutive tiles per workgroup (a tile is a few microseconds of dependent latencies: load, LDS,
  // matrix instructions, LDS, store; what hides them is the number of workgroups a CU holds, four here, and not
  // having to start a new workgroup for every tile)
  for (int rep = 0; rep < kThinTiles; ++rep) {
  const int tile_id = blockIdx.x * kThinTiles + rep;
  if (tile_id >= a.n_mt * a.n_nt) break;  // (uniform)
  const int mt = tile_id / a.n_nt, nt = tile_id % a.n_nt;
  const int m0 = mt * 128, n0 = nt * 128;
  if (rep > 0) __syncthreads();  // the previous tile's patches are done with the LDS
  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][j][r] = 0.f;
  for (int kt = 0; kt < KT; ++kt) {
    u32x4 ra[4], rb[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const size_t blk = (size_t)(kb0 + kt);
      ra[i] = *reinterpret_cast<const u32x4 *>(
          a.AT + (blk * a.lda + a.a0 + min(m0 + row0 + 32 * i, a.M - 1)) * 64 + chunk * 8);
      rb[i] = *reinterpret_cast<const u32x4 *>(
          a.BT + (blk * a.ldb + a.b0 + min(n0 + row0 + 32 * i, a.N - 1)) * 64 + chunk * 8);
    }
    if (kt > 0) __syncthreads();  // the previous step's fragment reads are done
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = row0 + 32 * i;
      const int dst = (row * 8 + (chunk ^ ((row >> 1) & 7))) * 16;
      *reinterpret_cast<u32x4 *>(smem + dst) = ra[i];
      *reinterpret_cast<u32x4 *>(smem + 16384 + dst) = rb[i];
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const int slot = ((kk * 2 + khalf) ^ sw) * 16;
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int q = 0; q < 2; ++q) {
        fa[q] = *reinterpret_cast<const bf16x8 *>(smem + (wm * 64 + q * 32 + l31) * 128 + slot);
        fb[q] = *reinterpret_cast<const bf16x8 *>(smem + 16384 + (wn * 64 + q * 32 + l31) * 128 + slot);
      }
#pragma unroll
      for (int mi = 0; mi < 2; ++mi) {
        acc[mi][0] = mfma_bf16(fa[mi], fb[0], acc[mi][0]);
        acc[mi][1] = mfma_bf16(fa[mi], fb[1], acc[mi][1]);
      }
    }
  }
  __syncthreads();  // the stage is dead: every wave takes a private patch
  unsigned char *patch = smem + w4 * kPatchBytes;
  bf16_t *C = a.C + (size_t)le * a.M * a.N;
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
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
    for (int it = 0; it < 4; ++it) {
      const int rl = it * 8 + (lane >> 3), cc = lane & 7;  // 8 groups of 8 columns per row: 16-byte stores
      const int m = m0 + wm * 64 + mi * 32 + rl, n = n0 + wn * 64 + cc * 8;
      const f32x4 v0 = *reinterpret_cast<const f32x4 *>(patch + rl * 288 + cc * 32);
      const f32x4 v1 = *reinterpret_cast<const f32x4 *>(patch + rl * 288 + cc * 32 + 16);
      if (m < a.M && n < a.N) {  // N % 8 == 0: the eight columns are inside together
        bf16x8 o;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          o[q] = (bf16_t)v0[q];
          o[4 + q] = (bf16_t)v1[q];
        }
        __builtin_nontemporal_store(o, reinterpret_cast<bf16x8 *>(C + (size_t)m * a.N + n));
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  }  // tiles of this workgroup
}

}  // namespace moe355
