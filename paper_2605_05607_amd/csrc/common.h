// Internal helpers shared by the moe355 translation units (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "moe355.h"

namespace moe355 {

constexpr int kWave = 64;
constexpr int kMaxExperts = 4096;
constexpr int kMaxTopK = 32;

// GEMM macro-tile of the bf16 MFMA kernels.  The paper's tile is 128 tokens (GEMM tile = synchronisation
// granularity, Sec. VII-C); here the M tile is 256 rows so that one pass over a weight panel does twice the
// math per byte that has to cross the L2 -> CU path, which is what bounds the matrix cores on gfx950.
constexpr int kBM = 256;
constexpr int kBN = 256;
constexpr int kBK = 64;
// Tile of the plain fp32 kernels (small reference-grade path for fp32 layers).
constexpr int kFBM = 64;
constexpr int kFBN = 64;
constexpr int kFBK = 16;

struct Derived {
  int epr;         // experts per rank
  int E_loc;       // local experts
  int e_lo;        // first local expert
  int64_t pairs;   // T * k
  int64_t P_cap;   // upper bound on local pairs: T * min(k, E_loc)
  int bm;          // M tile of the dtype's GEMM kernels
  int max_mtiles;  // upper bound on M tiles: ceil(P_cap / bm) + E_loc
  int nt1, nt2;    // N tiles of GEMM-1 (over f) and GEMM-2 (over d)
  int elt;         // bytes per element of x / weights / y
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Shape checks common to all entry points.  Returns MOE_OK or the error to hand back.
int check_shape(const moe_shape *s, Derived *out);

// hipGetLastError() reports (and clears) the last error of ANY earlier runtime call on this thread, including
// the caller's own; every entry point therefore drops a stale error before its first launch and reads the
// status after each launch.
inline void begin_launches() { (void)hipGetLastError(); }
inline int launch_status() { return hipGetLastError() == hipSuccess ? MOE_OK : MOE_ERR_HIP; }

// Raises a kernel's dynamic-LDS limit, once per device (the attribute belongs to the function on one device).
// `done` is the call site's bit mask of devices already served.
inline bool allow_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false;
  const uint64_t bit = uint64_t(1) << dev;
  if (done.load(std::memory_order_acquire) & bit) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return false;
  done.fetch_or(bit, std::memory_order_release);
  return true;
}

// ---- layout of the forward workspace (offsets in bytes, 256-byte aligned) ----
struct FwdLayout {
  size_t header;    // int32[32]: [0] work items of GEMM-1, [1] P, [2] first layout row of the local segment,
                    //            [3] work items of GEMM-2, [4] M tiles, [8..23] queue tickets and [24] error flag
                    //            of the resident GEMM kernel
  size_t work1;     // int4[max_mtiles * nt1]  (local expert, first local row, valid rows, N tile) per work item
  size_t work2;     // int4[max_mtiles * nt2]
  size_t row_tok;   // int32[P_cap]       token of each local row
  size_t row_w;     // float[P_cap]       gate weight of each local row
  size_t row_sole;  // int32[P_cap]       the row's token if it is that token's only local slot, else -1
  size_t tile_ready;  // int32[max_mtiles] GEMM-1 items finished per M tile (hand-over inside the resident kernel)
  size_t row_tile;    // int32[P_cap]      M tile of each local row        } resident kernel that also runs
  size_t tile_done;   // int32[max_mtiles] GEMM-2 items finished per M tile } Combine
  size_t h;         // elt  [P_cap, f]
  size_t o;         // float[P_cap, d]
  size_t total;
};
FwdLayout forward_layout(const moe_shape *s, const Derived &dv);

// ---- packed weight geometry ----
// bf16: gate/up as [E_loc][ceil(f/128)][ceil(d/64)] tiles of 256 x 64 elements (128 gate + 128 up columns
// of the same 128 h columns), down as [E_loc][ceil(d/256)][ceil(f/64)] tiles of 256 x 64; inside a tile the
// values are stored in matrix-core operand order (see pack_kernels.h), zero-padded.
// fp32: plain copies (gate then up, then down).
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace moe355

#ifdef __HIPCC__
namespace moe355 {

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Inclusive scan over the 64 lanes of a wave.
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  const int lane = lane_id();
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int n = __shfl_up(v, off, 64);
    if (lane >= off) v += n;
  }
  return v;
}

// Exclusive scan over a block of up to 1024 threads (blockDim.x multiple of 64).  `scratch` holds 17 ints.
// Returns the exclusive prefix of v; *total receives the block sum.  All threads must call.
__device__ __forceinline__ int block_exclusive_scan(int v, int *scratch, int *total) {
  const int lane = lane_id();
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  const int inc = wave_inclusive_scan(v);
  __syncthreads();
  if (lane == 63) scratch[wave] = inc;
  __syncthreads();
  if (wave == 0) {
    int w = lane < nwaves ? scratch[lane] : 0;
    int winc = wave_inclusive_scan(w);
    if (lane < nwaves) scratch[lane] = winc - w;
    if (lane == 63) scratch[16] = winc;
  }
  __syncthreads();
  const int base = scratch[wave];
  *total = scratch[16];
  return base + inc - v;
}

}  // namespace moe355
#endif
