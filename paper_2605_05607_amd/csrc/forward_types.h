// Types, constants and small device helpers shared by the kernels of the forward path.
#pragma once
#include "common.h"

namespace moe355 {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));

// fp32 -> E4M3 code (OCP 8-bit floating point, the format the matrix cores read): round to nearest even,
// saturating at +-448; finite input.
__device__ __forceinline__ uint8_t to_e4m3(float v) {
  v = __builtin_amdgcn_fmed3f(v, 448.0f, -448.0f);
  return (uint8_t)(__builtin_amdgcn_cvt_pk_fp8_f32(v, v, 0, false) & 0xFF);
}

constexpr int kTileBytes = kBN * kBK * 2;  // one packed weight tile = one LDS stage image of B (32 KiB)

constexpr int kTileShift = 12;  // work item .w = N tile | M-tile id << kTileShift
// work item .z = rows of the tile | kItemLone if the tile is its expert's only M tile (its weights are read once)
constexpr int kItemRowsMask = 0xFFFF;
constexpr int kItemLone = 1 << 16;
constexpr int kChunk = 32;  // work items that are resident on one XCD at a time (one per CU)
constexpr int kChunkM = 8;  // M tiles per chunk (at most)

// List position of workgroup `block` (or -1): XCD x = block % 8 takes whole 32-item chunks x, x + 8, ... while
// complete rounds of 8 chunks last; the remaining items (fewer than 256) are cut into 8 equal contiguous pieces so
// that every XCD gets the same number of items to within one.
__device__ __forceinline__ int chunked_item(int block, int n_items) {
  const int xcd = block & 7, j = block >> 3;
  const int full_rows = n_items / (8 * kChunk);
  if (j < full_rows * kChunk) return ((j / kChunk) * 8 + xcd) * kChunk + (j % kChunk);
  const int rem = n_items - full_rows * 8 * kChunk;
  const int jj = j - full_rows * kChunk;
  const int piece = rem / 8, extra = rem % 8;
  const int size = piece + (xcd < extra);
  if (jj >= size) return -1;
  return full_rows * 8 * kChunk + xcd * piece + min(xcd, extra) + jj;
}

// Arguments of one grouped GEMM (see gemm_bf16.h for the meaning of the operands).
struct GemmArgs {
  const void *A;
  const int32_t *row_map;
  const void *Bp;
  void *out;
  const float *row_w;
  const int32_t *row_sole;  // GEMM-2 only, may be null: token of a row that is the token's only local slot, else -1
  void *y;                  // GEMM-2 only: layer output, target of the sole rows
  const int32_t *n_items;  // device: number of work items of this GEMM
  const int4 *work;        // device: work list
  int K, N, lda, ldo, n_ntiles, n_ktiles;
  // training path only (null otherwise): kept g and u (written by GEMM-1, read by the first backward GEMM) and the
  // weighted h the first backward GEMM writes
  void *aux;
  void *aux2;
  // FP8 operands only (null otherwise)
  const float *a_scale;  // GEMM-1: scale of every token's row of x (indexed like A's rows)
  const float *b_scale;  // scales of the output columns: GEMM-1 [E_loc][2][N] (gate, up), GEMM-2 [E_loc][N]
  const float *h_scale;  // [E_loc] scale of h: GEMM-1 divides by it, GEMM-2 multiplies
};

}  // namespace moe355
