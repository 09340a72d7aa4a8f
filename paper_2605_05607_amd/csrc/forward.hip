// moe_fused_forward and its building blocks: weight packing, tile table, grouped SwiGLU GEMMs (GEMM-1 and
// GEMM-2 of Sec. II-A) with the token gather fused into GEMM-1's operand load (Dispatch of Sec. II-A without a
// materialised copy), the gate weight applied in GEMM-2's epilogue (Sec. III-C), and the per-token reduction
// with a single write-back (Combine; the one-GPU form of the in-switch reduction of Sec. II-C).
#include <algorithm>

#include "common.h"

namespace moe355 {

typedef __bf16 bf16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));

constexpr int kTileBytes = kBN * kBK * 2;  // one packed weight tile = one LDS stage image of B (32 KiB)

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

// ------------------------------------------------------------------------------------------------
// Work lists and per-row metadata of the local layout segment.
// header[0] = work items of GEMM-1, header[1] = P (local rows), header[2] = first layout row of the segment,
// header[3] = work items of GEMM-2, header[4] = M tiles; header[8..15] / [16..23] = ticket counters of the GEMM-1 /
// GEMM-2 queues and header[24] = error flag of the resident GEMM kernel (all cleared here).
//
// A work item is one output tile (expert, M tile, N tile): int4 (local expert, first local row, valid rows,
// N tile | M-tile id << 12).  Full M tiles come first and the partial tile of each
// expert (its last rows) afterwards, largest first, so that the launch ends with its shortest items; partial
// tiles of at most 64 rows (pure weight streaming) are mixed into the full tiles (see the list order below).
// The order of the list is also what keeps the L2 useful:
// the chip has 8 XCDs with a private 4 MiB L2 each and workgroup i runs on XCD i % 8, so every GEMM workgroup
// maps its index to a list position such that XCD x works through the 32-item chunks x, x + 8, x + 16, ...;
// and a chunk is a block of (up to 8 M tiles) x (32 / that many N tiles) of ONE expert, so the 32 workgroups
// that are resident on an XCD at the same time share a few A slabs and a few weight panels instead of
// streaming 32 different ones through the L2.
// ------------------------------------------------------------------------------------------------
constexpr int kTileShift = 12;  // work item .w = N tile | M-tile id << kTileShift
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

// Rows up to which a partial tile counts as "streaming": its cost is reading the expert's weights from HBM, not
// the matrix cores.
constexpr int kStreamRows = 64;

__global__ __launch_bounds__(256) void fwd_prep_kernel(const int32_t *__restrict__ offsets,
                                                       const int32_t *__restrict__ perm,
                                                       const float *__restrict__ topk_w, int T, int k, int e_lo,
                                                       int E_loc, int bm, int P_cap, int max_mtiles, int nt1, int nt2,
                                                       int32_t *__restrict__ header, int4 *__restrict__ work1,
                                                       int4 *__restrict__ work2, int32_t *__restrict__ row_tok,
                                                       float *__restrict__ row_w,
                                                       const int32_t *__restrict__ topk_idx,
                                                       int32_t *__restrict__ row_sole,
                                                       int32_t *__restrict__ tile_ready) {
  // LDS: full0[E_loc + 1] first full M tile of each expert | part[E_loc] rows of its partial tile (0 = none) |
  //      order[E_loc] partial tiles: first the large ones (> kStreamRows rows), largest first, then the
  //      streaming ones, largest first | 17 ints of scan scratch
  extern __shared__ int lds[];
  int *full0 = lds;
  int *part = full0 + E_loc + 1;
  int *order = part + E_loc;
  int *scratch = order + E_loc;
  const int base = offsets[e_lo];
  const int P = max(0, min(P_cap, offsets[e_lo + E_loc] - base));
  const long long npairs = (long long)T * k;
  for (int r = blockIdx.x * blockDim.x + threadIdx.x; r < P; r += gridDim.x * blockDim.x) {
    int p = perm[base + r];
    p = p < 0 ? 0 : (p >= npairs ? (int)(npairs - 1) : p);
    const int t = p / k;
    row_tok[r] = t;
    row_w[r] = topk_w[p];
    if (row_sole) {
      // a row that is its token's only local slot needs no reduction: GEMM-2 writes it straight to y
      int n_local = 0;
      for (int j = 0; j < k; ++j) {
        const int e = topk_idx[(size_t)t * k + j];
        n_local += e >= e_lo && e < e_lo + E_loc;
      }
      row_sole[r] = n_local == 1 ? t : -1;
    }
  }
  // Every block rebuilds the small per-expert tables (cheap) so that the lists can be written grid-wide.
  // An expert with cnt rows has cnt / bm full tiles and, if cnt % bm != 0, one partial tile.
  const int ipt = (E_loc + blockDim.x - 1) / blockDim.x;
  const int lo = min(E_loc, (int)threadIdx.x * ipt);
  const int hi = min(E_loc, lo + ipt);
  int local_full = 0, local_big = 0, local_small = 0;
  for (int le = lo; le < hi; ++le) {
    const int cnt = max(0, min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base));
    part[le] = cnt % bm;
    local_full += cnt / bm;
    local_big += (cnt % bm) > kStreamRows;
    local_small += (cnt % bm) != 0 && (cnt % bm) <= kStreamRows;
  }
  int n_full, n_big, n_small;
  int run = block_exclusive_scan(local_full, scratch, &n_full);
  for (int le = lo; le < hi; ++le) {
    const int cnt = max(0, min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base));
    full0[le] = run;
    run += cnt / bm;
  }
  if (threadIdx.x == 0) full0[E_loc] = n_full;
  (void)block_exclusive_scan(local_big, scratch, &n_big);
  (void)block_exclusive_scan(local_small, scratch, &n_small);
  __syncthreads();
  // rank sort inside the two classes of partial tiles (for very many experts keep the expert order)
  for (int le = lo; le < hi; ++le) {
    const int mine = part[le];
    if (mine == 0) continue;
    const bool small = mine <= kStreamRows;
    int rank = 0;
    for (int o = 0; o < E_loc; ++o) {
      const int po = part[o];
      if (po == 0 || (po <= kStreamRows) != small) continue;
      rank += E_loc <= 1024 ? (po > mine || (po == mine && o < le)) : (o < le);
    }
    order[(small ? n_big : 0) + rank] = le;
  }
  __syncthreads();
  n_full = min(n_full, max_mtiles);
  n_big = min(n_big, max_mtiles - n_full);
  n_small = min(n_small, max_mtiles - n_full - n_big);
  const int n_tiles = n_full + n_big + n_small;
  const int n1 = n_tiles * nt1, n2 = n_tiles * nt2;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    header[0] = n1;
    header[1] = P;
    header[2] = base;
    header[3] = n2;
    header[4] = n_tiles;
    for (int i = 8; i <= 24; ++i) header[i] = 0;
  }
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_tiles; i += gridDim.x * blockDim.x) tile_ready[i] = 0;
  for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < n1 + n2; q += gridDim.x * blockDim.x) {
    const bool second = q >= n1;
    const int Nt = second ? nt2 : nt1;
    const int qq = second ? q - n1 : q;
    // List order.  Classes: F = full tiles, B = big partial tiles, S = streaming partial tiles.
    //   [ mixed chunks: each 32-item chunk holds 8 items of S, then 24 items of F, so that some CUs of every XCD
    //     stream weights from HBM while the others multiply; only when S is at least half as large as F,
    //     otherwise the few S items would just push full tiles into an extra round ]
    //   [ rest of F ] [ B, largest first ] [ rest of S ]          -- the launch ends with its shortest items
    const int nF = n_full * Nt, nS = n_small * Nt, nB = n_big * Nt;
    constexpr int nsc = 8, nfc = kChunk - nsc;
    const int n_mix = (nF > 0 && 2 * nS >= nF) ? min(nF / nfc, nS / nsc) : 0;
    // F items that share operands form groups of gsz consecutive list positions; gsz follows the F share of a chunk
    const int gsz = n_mix > 0 ? nfc : kChunk;
    int cls, idx;  // class 0 = F, 1 = B, 2 = S; idx = position inside the class list
    if (qq < n_mix * kChunk) {
      const int c = qq / kChunk, sl = qq % kChunk;
      if (sl < nsc) { cls = 2; idx = c * nsc + sl; } else { cls = 0; idx = c * nfc + (sl - nsc); }
    } else {
      int r = qq - n_mix * kChunk;
      const int f_rem = nF - n_mix * nfc;
      if (r < f_rem) { cls = 0; idx = n_mix * nfc + r; }
      else if ((r -= f_rem) < nB) { cls = 1; idx = r; }
      else { cls = 2; idx = n_mix * nsc + (r - nB); }
    }
    int le, mt, nt, rows, tile;
    if (cls == 0) {
      // expert that owns F position idx: largest le with full0[le] * Nt <= idx
      int a = 0, b = E_loc;
      while (b - a > 1) {
        const int mid = (a + b) >> 1;
        if (full0[mid] * Nt <= idx) a = mid; else b = mid;
      }
      le = a;
      const int Mt = full0[le + 1] - full0[le];
      int r = idx - full0[le] * Nt;
      // inside the expert: M groups of up to 8 tiles; inside an M group: N groups of gsz / (M tiles) tiles.
      // (A slab and B panel of a tile are equally large, so the bytes a chunk pulls into its L2 are smallest
      // when the chunk is close to square: 8 x 4 rather than 32 x 1.)
      const int Mg = min(Mt, kChunkM);
      const int mg = r / (Mg * Nt);
      r -= mg * Mg * Nt;
      const int Mcur = min(Mg, Mt - mg * Mg);
      const int G = max(1, gsz / Mcur);
      const int ng = r / (Mcur * G);
      r -= ng * Mcur * G;
      const int Gcur = min(G, Nt - ng * G);
      mt = mg * Mg + r / Gcur;
      nt = ng * G + r % Gcur;
      rows = bm;
      tile = full0[le] + mt;
    } else {
      le = order[(cls == 2 ? n_big : 0) + idx / Nt];
      tile = n_full + (cls == 2 ? n_big : 0) + idx / Nt;
      nt = idx % Nt;
      const int cnt = min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base);
      mt = cnt / bm;
      rows = part[le];
    }
    const int start = min(P, offsets[e_lo + le] - base);
    const int4 item = make_int4(le, start + mt * bm, rows, nt | (tile << kTileShift));
    if (second) work2[qq] = item; else work1[qq] = item;
  }
}

// ------------------------------------------------------------------------------------------------
// Grouped bf16 GEMM on the matrix cores.  C[rows of one expert tile, kBN/2 or kBN columns] = A * W_e.
//   A rows   : row_map == nullptr -> A[m0 + r, :]; else A[row_map[m0 + r], :] (token gather of Dispatch).
//   B tiles  : packed LDS images streamed linearly.
//   GATED    : epilogue h = silu(g) * u, written as bf16   (GEMM-1)
//   !GATED   : epilogue o = acc * row_w[row], written fp32 (GEMM-2, gate weight of Sec. III-C)
// Tile 256 x 256 x 64, one workgroup of 512 threads per CU.  Every operand byte enters the CU once (global ->
// registers -> LDS) because the L2 -> CU path, not the matrix core, is what saturates first on this chip;
// sharing goes through the LDS, which has bandwidth to spare.  8 waves = 2 (rows) x 4 (columns), each wave
// owns 128 x 64 as 4 x 2 MFMA 32x32x16 accumulators; two waves per SIMD cover each other's LDS latency.
// LDS is double buffered (2 x 64 KiB) with one barrier per k-step; the next slab is in flight in registers
// while the current one is multiplied.  NB = number of 32-row blocks of this wave that hold valid rows (the
// others are skipped: small experts are weight-streaming bound and need no padding math).
// ------------------------------------------------------------------------------------------------
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
};

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

constexpr int kGemmThreads = 512;
constexpr int kAStageBytes = kBM * kBK * 2;               // 32 KiB
constexpr int kStageBytes = kAStageBytes + kTileBytes;    // 64 KiB: A slab then B slab
constexpr int kPatchBytes = 32 * 288;                     // per-wave epilogue patch (fits 8 x in the stages)

template <bool GATED, bool RESIDENT, int NB, int NA, int DEPTH>
__device__ __forceinline__ void gemm_bf16_tile(const GemmArgs &g, unsigned char *smem, int nt, int le, int m0,
                                               int rows, int nblk_total) {
  // RESIDENT (the kernel that loops over items): the thread index goes through an empty asm so that nothing
  // derived from it counts as loop invariant; hoisting those values across items costs more registers than the
  // tile has to spare.
  int tid = threadIdx.x;
  if (RESIDENT) asm volatile("" : "+v"(tid));
  const int lane = tid & 63;
  const int w8 = tid >> 6;
  const int wm = w8 >> 2, wn = w8 & 3;

  // ---- global -> register staging (scalars, not arrays, so nothing lands in scratch) ----
  // A: thread t stages chunk t & 7 (8 reduction indices) of rows (t >> 3) + 64 i; B: chunks t + 512 i
  const int a_chunk = tid & 7;
  const int a_row0 = tid >> 3;  // 0..63
  const bf16_t *a_base = static_cast<const bf16_t *>(g.A) + a_chunk * 8;
#define MOE355_A_ROW(i)                                                                          \
  const int a_rc##i = a_row0 + 64 * i < rows ? a_row0 + 64 * i : rows - 1; /* padding: a valid row */ \
  const uint32_t a_off##i =                                                                      \
      (uint32_t)(g.row_map ? g.row_map[m0 + a_rc##i] : m0 + a_rc##i) * (uint32_t)g.lda;
  MOE355_A_ROW(0) MOE355_A_ROW(1) MOE355_A_ROW(2) MOE355_A_ROW(3)
#undef MOE355_A_ROW
  // LDS destination of row a_row0; row + 64 i lies 8192 bytes further (64 i keeps the swizzle bits)
  const int a_dst = (a_row0 * 8 + (a_chunk ^ ((a_row0 >> 1) & 7))) * 16;
  const unsigned char *b_src =
      static_cast<const unsigned char *>(g.Bp) + ((size_t)(le * g.n_ntiles + nt) * g.n_ktiles) * kTileBytes + tid * 16;

  // Register slab sets.  Set x always exists; set y is used when DEPTH == 2 (two slabs in flight: tiles with at
  // most 64 rows are pure weight streaming, their accumulators are small, and what limits them is the number of
  // bytes a CU keeps in flight towards HBM).
  u32x4 ra0x, ra1x, ra2x, ra3x, rb0x, rb1x, rb2x, rb3x;
  u32x4 ra0y, ra1y, ra2y, ra3y, rb0y, rb1y, rb2y, rb3y;
  // A slab is moved in three portions: {ra0, ra1, rb0}, {ra2, ra3, rb1}, {rb2, rb3}
  // k tail: a chunk past K is replaced by chunk 0 of the same row (valid memory, finite data); the packed B
  // tile is zero there, so it contributes nothing and no select has to wait on the load
#define MOE355_A_OFF(KT) ((KT) * kBK + a_chunk * 8 < g.K ? (KT) * kBK : -a_chunk * 8)
  // NA = row loads per thread that reach valid rows (1: rows < 64, 2: rows < 128, 4: all); the others are skipped
#define MOE355_LOAD_P0(S, KT)                                                                       \
  do {                                                                                              \
    ra0##S = *reinterpret_cast<const u32x4 *>(a_base + a_off0 + MOE355_A_OFF(KT));                  \
    if (NA > 1) ra1##S = *reinterpret_cast<const u32x4 *>(a_base + a_off1 + MOE355_A_OFF(KT));      \
    rb0##S = *reinterpret_cast<const u32x4 *>(b_src + (size_t)(KT) * kTileBytes);                   \
  } while (0)
#define MOE355_LOAD_P1(S, KT)                                                                       \
  do {                                                                                              \
    if (NA > 2) ra2##S = *reinterpret_cast<const u32x4 *>(a_base + a_off2 + MOE355_A_OFF(KT));      \
    if (NA > 2) ra3##S = *reinterpret_cast<const u32x4 *>(a_base + a_off3 + MOE355_A_OFF(KT));      \
    rb1##S = *reinterpret_cast<const u32x4 *>(b_src + (size_t)(KT) * kTileBytes + 8192);            \
  } while (0)
#define MOE355_LOAD_P2(S, KT)                                                                       \
  do {                                                                                              \
    rb2##S = *reinterpret_cast<const u32x4 *>(b_src + (size_t)(KT) * kTileBytes + 16384);           \
    rb3##S = *reinterpret_cast<const u32x4 *>(b_src + (size_t)(KT) * kTileBytes + 24576);           \
  } while (0)
#define MOE355_STORE_P0(S, BUF)                                                                     \
  do {                                                                                              \
    unsigned char *s_ = smem + (BUF) * kStageBytes;                                                 \
    *reinterpret_cast<u32x4 *>(s_ + a_dst) = ra0##S;                                                \
    if (NA > 1) *reinterpret_cast<u32x4 *>(s_ + a_dst + 8192) = ra1##S;                             \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16) = rb0##S;                              \
  } while (0)
#define MOE355_STORE_P1(S, BUF)                                                                     \
  do {                                                                                              \
    unsigned char *s_ = smem + (BUF) * kStageBytes;                                                 \
    if (NA > 2) *reinterpret_cast<u32x4 *>(s_ + a_dst + 16384) = ra2##S;                            \
    if (NA > 2) *reinterpret_cast<u32x4 *>(s_ + a_dst + 24576) = ra3##S;                            \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16 + 8192) = rb1##S;                       \
  } while (0)
#define MOE355_STORE_P2(S, BUF)                                                                     \
  do {                                                                                              \
    unsigned char *s_ = smem + (BUF) * kStageBytes;                                                 \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16 + 16384) = rb2##S;                      \
    *reinterpret_cast<u32x4 *>(s_ + kAStageBytes + tid * 16 + 24576) = rb3##S;                      \
  } while (0)

  f32x16 acc[NB > 0 ? NB : 1][2];
#pragma unroll
  for (int mi = 0; mi < NB; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][j][r] = 0.f;

  // ---- LDS -> MFMA operand addressing: lane l reads row l & 31 of a 32-row block, k half l >> 5 ----
  const int l31 = lane & 31, khalf = lane >> 5, sw = (lane >> 1) & 7;
  const int a_rd = (wm * 128 + l31) * 128;                  // + mi * 4096
  const int b_rd = kAStageBytes + (wn * 64 + l31) * 128;    // + j * 4096

  constexpr int NF = NB > 0 ? NB : 1;
  bf16x8 fa0[NF], fb0[2], fa1[NF], fb1[2];  // operand fragments of two consecutive k-substeps
#define MOE355_READ_FRAGS(FA, FB, STAGE, KK)                                                           \
  do {                                                                                                 \
    const int slot_ = (((KK) * 2 + khalf) ^ sw) * 16;                                                  \
    _Pragma("unroll") for (int mi = 0; mi < NB; ++mi) FA[mi] =                                         \
        *reinterpret_cast<const bf16x8 *>((STAGE) + a_rd + mi * 4096 + slot_);                         \
    if (NB > 0) {                                                                                      \
      FB[0] = *reinterpret_cast<const bf16x8 *>((STAGE) + b_rd + slot_);                               \
      FB[1] = *reinterpret_cast<const bf16x8 *>((STAGE) + b_rd + 4096 + slot_);                        \
    }                                                                                                  \
  } while (0)
#define MOE355_MFMAS(FA, FB)                                                                           \
  do {                                                                                                 \
    _Pragma("unroll") for (int mi = 0; mi < NB; ++mi) {                                                \
      acc[mi][0] = mfma_bf16(FA[mi], FB[0], acc[mi][0]);                                               \
      acc[mi][1] = mfma_bf16(FA[mi], FB[1], acc[mi][1]);                                               \
    }                                                                                                  \
  } while (0)

  // Pipeline.  At the top of k-step kt: LDS stage kt & 1 holds slab kt, a register set holds slab kt + 1 (its
  // loads were issued DEPTH k-steps ago, in three portions), and fa0 / fb0 hold the operands of substep 0.
  // Substeps 0..2 each multiply, fetch the next substep's operands, move one portion of the register set into the
  // other stage and reissue that portion's loads for slab kt + 1 + DEPTH, so the global loads, the LDS stores and
  // the LDS reads are all spread under the MFMAs instead of forming a burst around the barrier.  The single
  // barrier sits before substep 3, whose operands are already in registers; substep 3 also fetches substep 0 of
  // the next slab.  Reloads past the last k-step repeat the last slab: in bounds, never used.
  // Requested instruction order (sched_group_barrier masks: 0x008 MFMA, 0x020 VMEM read, 0x100 DS read,
  // 0x200 DS write).
#define MOE355_ORDER(NW)                                                                                \
  do {                                                                                                 \
    if (NB > 0) {                                                                                      \
      __builtin_amdgcn_sched_group_barrier(0x100, NB + 2, 0);                                          \
      __builtin_amdgcn_sched_group_barrier(0x008, 2 * NB, 0);                                          \
    }                                                                                                  \
    if ((NW) > 0) {                                                                                    \
      __builtin_amdgcn_sched_group_barrier(0x200, (NW), 0);                                            \
      __builtin_amdgcn_sched_group_barrier(0x020, (NW), 0);                                            \
    }                                                                                                  \
  } while (0)
#define MOE355_KSTEP(S, KT_, KPRE)                                                                      \
  do {                                                                                                 \
    const unsigned char *sCur = smem + ((KT_) & 1) * kStageBytes;                                      \
    const int nxt = ((KT_) & 1) ^ 1;                                                                   \
    const int kp_ = min((KPRE), kt_last);                                                              \
    MOE355_READ_FRAGS(fa1, fb1, sCur, 1);                                                              \
    MOE355_MFMAS(fa0, fb0);                                                                            \
    MOE355_STORE_P0(S, nxt);                                                                           \
    MOE355_LOAD_P0(S, kp_);                                                                            \
    MOE355_READ_FRAGS(fa0, fb0, sCur, 2);                                                              \
    MOE355_MFMAS(fa1, fb1);                                                                            \
    MOE355_STORE_P1(S, nxt);                                                                           \
    MOE355_LOAD_P1(S, kp_);                                                                            \
    MOE355_READ_FRAGS(fa1, fb1, sCur, 3);                                                              \
    MOE355_MFMAS(fa0, fb0);                                                                            \
    MOE355_STORE_P2(S, nxt);                                                                           \
    MOE355_LOAD_P2(S, kp_);                                                                            \
    MOE355_ORDER(NA > 1 ? 3 : 2);                                                                      \
    MOE355_ORDER(NA > 2 ? 3 : 1);                                                                      \
    MOE355_ORDER(2);                                                                                   \
    __syncthreads();                                                                                   \
    MOE355_READ_FRAGS(fa0, fb0, smem + nxt * kStageBytes, 0);                                          \
    MOE355_MFMAS(fa1, fb1);                                                                            \
    MOE355_ORDER(0);                                                                                   \
  } while (0)

  const int KT = g.n_ktiles;
  const int kt_last = KT - 1;
  MOE355_LOAD_P0(x, 0); MOE355_LOAD_P1(x, 0); MOE355_LOAD_P2(x, 0);
  MOE355_STORE_P0(x, 0); MOE355_STORE_P1(x, 0); MOE355_STORE_P2(x, 0);
  {
    const int k1 = min(1, kt_last);
    MOE355_LOAD_P0(x, k1); MOE355_LOAD_P1(x, k1); MOE355_LOAD_P2(x, k1);
    if (DEPTH == 2) {
      const int k2 = min(2, kt_last);
      MOE355_LOAD_P0(y, k2); MOE355_LOAD_P1(y, k2); MOE355_LOAD_P2(y, k2);
    }
  }
  __syncthreads();
  MOE355_READ_FRAGS(fa0, fb0, smem, 0);

  if (DEPTH == 1) {
    for (int kt = 0; kt < KT; ++kt) MOE355_KSTEP(x, kt, kt + 2);
  } else {
    // set x carries the odd slabs, set y the even ones
    for (int kt = 0; kt < KT; kt += 2) {
      MOE355_KSTEP(x, kt, kt + 3);
      if (kt + 1 < KT) MOE355_KSTEP(y, kt + 1, kt + 4);
    }
  }
#undef MOE355_KSTEP
#undef MOE355_ORDER
#undef MOE355_READ_FRAGS
#undef MOE355_MFMAS
#undef MOE355_LOAD_P0
#undef MOE355_LOAD_P1
#undef MOE355_LOAD_P2
#undef MOE355_STORE_P0
#undef MOE355_STORE_P1
#undef MOE355_STORE_P2
#undef MOE355_A_OFF

  // ---- epilogue ----
  // Accumulator register r of lane l holds C[8*(r/4) + 4*(l/32) + r%4][l%32] of its 32x32 block, i.e. a lane
  // owns one column.  Each wave turns its blocks around through a private LDS patch (the stages are dead now)
  // so that the global stores are 16 bytes per lane along a row instead of one element per lane.
  __syncthreads();  // every wave has finished reading the stages
  unsigned char *patch = smem + w8 * kPatchBytes;
#pragma unroll
  for (int mi = 0; mi < NB; ++mi) {
    const int blk_row0 = wm * 128 + mi * 32;  // first tile row of this 32-row block
    if (GATED) {
      // h block: 32 rows x 32 columns bf16, row pitch 80 bytes (keeps the two half-waves on different banks)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
        const float gv = acc[mi][0][r], uv = acc[mi][1][r];
        *reinterpret_cast<bf16_t *>(patch + rl * 80 + l31 * 2) = (bf16_t)((gv / (1.0f + __expf(-gv))) * uv);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int c = it * 64 + lane;        // 16-byte chunk: 4 chunks per row
        const int rl = c >> 2, cc = c & 3;
        const int row_l = blk_row0 + rl;
        const int col = nt * (kBN / 2) + wn * 32 + cc * 8;
        const u32x4 v = *reinterpret_cast<const u32x4 *>(patch + rl * 80 + cc * 16);
        if (row_l < rows && col < g.N)
          *reinterpret_cast<u32x4 *>(static_cast<bf16_t *>(g.out) + (size_t)(m0 + row_l) * g.ldo + col) = v;
      }
    } else {
      // o block: 32 rows x 64 columns fp32, row pitch 288 bytes.  A row whose token has no other local slot
      // is final already (the Combine sum would have one term): it goes to y in the output type, skipping o.
      int sole[8];
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int row_l = blk_row0 + it * 4 + (lane >> 4);
        sole[it] = (g.row_sole && row_l < rows) ? g.row_sole[m0 + row_l] : -1;
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rl = (r >> 2) * 8 + khalf * 4 + (r & 3);
        const int row_l = blk_row0 + rl;
        const float wgt = row_l < rows ? g.row_w[m0 + row_l] : 0.f;
        *reinterpret_cast<float *>(patch + rl * 288 + l31 * 4) = acc[mi][0][r] * wgt;
        *reinterpret_cast<float *>(patch + rl * 288 + 128 + l31 * 4) = acc[mi][1][r] * wgt;
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int rl = it * 4 + (lane >> 4), cc = lane & 15;  // 16 chunks of 16 bytes per row
        const int row_l = blk_row0 + rl;
        const int col = nt * kBN + wn * 64 + cc * 4;
        const f32x4 v = *reinterpret_cast<const f32x4 *>(patch + rl * 288 + cc * 16);
        if (row_l < rows && col < g.N) {
          if (sole[it] >= 0) {
            bf16x4 b;
#pragma unroll
            for (int q = 0; q < 4; ++q) b[q] = (bf16_t)(v[q] + 0.0f);  // + 0 as in the sum that starts from zero
            *reinterpret_cast<bf16x4 *>(static_cast<bf16_t *>(g.y) + (size_t)sole[it] * g.ldo + col) = b;
          } else {
            *reinterpret_cast<f32x4 *>(static_cast<float *>(g.out) + (size_t)(m0 + row_l) * g.ldo + col) = v;
          }
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();  // the patch is reused by the next block
  }
}

// One work item on the matrix cores.  Wave-uniform dispatch on the number of valid 32-row blocks: every variant
// executes the same sequence of barriers.
template <bool GATED, bool RESIDENT>
__device__ __forceinline__ void gemm_bf16_item(const GemmArgs &g, unsigned char *smem, const int4 item) {
  const int le = item.x, m0 = item.y, rows = item.z, nt = item.w & ((1 << kTileShift) - 1);
  const int nblk_total = (rows + 31) >> 5;                        // 1..8
  const int wm = threadIdx.x >> 8;                                // wave row (wave-uniform)
  const int nb = max(0, min(4, nblk_total - 4 * wm));             // valid 32-row blocks of this wave
#define MOE355_TILE(NB_, NA_) \
  gemm_bf16_tile<GATED, RESIDENT, NB_, NA_, (NA_ == 1 ? 2 : 1)>(g, smem, nt, le, m0, rows, nblk_total)
  if (nblk_total <= 2) {
    if (nb == 2) MOE355_TILE(2, 1); else if (nb == 1) MOE355_TILE(1, 1); else MOE355_TILE(0, 1);
  } else if (nblk_total <= 4) {
    if (nb == 4) MOE355_TILE(4, 2); else if (nb == 3) MOE355_TILE(3, 2); else MOE355_TILE(0, 2);
  } else {
    if (nb == 4) MOE355_TILE(4, 4); else if (nb == 3) MOE355_TILE(3, 4); else if (nb == 2) MOE355_TILE(2, 4);
    else MOE355_TILE(1, 4);
  }
#undef MOE355_TILE
}

// One workgroup per work item; workgroup -> item by chunked_item.
template <bool GATED>
__global__ __launch_bounds__(kGemmThreads, 1) void gemm_bf16_kernel(const GemmArgs g) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages x 64 KiB
  const int q = chunked_item(blockIdx.x, *g.n_items);
  if (q < 0) return;
  gemm_bf16_item<GATED, false>(g, smem, g.work[q]);
}

// ------------------------------------------------------------------------------------------------
// GEMM-1 and GEMM-2 of a layer in ONE launch of resident workgroups (one per CU), the one-GPU form of the
// tile-granular GEMM-1 => GEMM-2 hand-over of the fused kernel (Sec. IV-A, IV-B): a GEMM-2 tile starts as soon
// as the h rows of its M tile are complete, so the CUs that run out of GEMM-1 work (a launch of a few hundred
// tiles of ~100 us ends with many CUs idle) continue with GEMM-2 instead of waiting for a kernel boundary.
// moe_fused_forward uses it for bf16 layers whose experts get less than one full M tile of rows on average (the
// launches are then dominated by partial tiles and by the tail of the few large experts; measured 5 % faster on the
// DeepSeek-shaped load); with fuller experts the ticket, fence and poll per item cost 2-6 % more than the idle
// tail they remove, and the kernel boundary of moe_fused_forward_two_launch is used instead.
//
// Work distribution: both lists are cut into 8 queues exactly as a plain launch would spread them over the XCDs
// (queue x = virtual blocks x, x + 8, ...; see chunked_item); a workgroup draws tickets from its home queue
// (blockIdx % 8, the XCD it runs on) and, when that is empty, from the others.  It moves on to GEMM-2 only after
// it has seen every GEMM-1 queue empty, i.e. when every GEMM-1 item is already in the hands of a running
// workgroup; GEMM-1 items never wait, so the counter a GEMM-2 item polls is always completed by workgroups that
// make progress: no deadlock for any number of resident workgroups and any placement.
// Hand-over: the producers of an M tile store h, fence at device scope, and count themselves in tile_ready;
// the consumer polls the counter, then fences before it loads h (the L2s of the XCDs are not coherent with
// each other, the device-scope fences write back / invalidate them).
// ------------------------------------------------------------------------------------------------
struct PipelineArgs {
  GemmArgs g1, g2;
  int32_t *tickets;     // [16]: queues of GEMM-1, then of GEMM-2
  int32_t *tile_ready;  // [M tiles] GEMM-1 items finished per M tile
  int32_t *error;       // set if a wait gave up (cannot happen unless the lists are corrupt)
  int nt1;              // GEMM-1 items per M tile
};

constexpr int kMaxPolls = 1 << 22;  // x ~1 us: a bound so that no wave can wait forever

// All items of one GEMM that this workgroup can get hold of: home queue first, then the other queues.
template <bool GATED>
__device__ __forceinline__ void gemm_bf16_drain(const GemmArgs &g, unsigned char *smem, int *s_item,
                                                int32_t *__restrict__ tickets, int32_t *__restrict__ tile_ready,
                                                int32_t *__restrict__ error, int nt1) {
  const int home = blockIdx.x & 7;
  const int n_items = *g.n_items;
  const int n_virtual = (n_items + 8 * kChunk - 1) / (8 * kChunk) * (8 * kChunk);
  int qsel = 0;
  while (qsel < 8) {
    const int queue = (home + qsel) & 7;
    __syncthreads();  // the previous item is done with the LDS (and with *s_item)
    if (threadIdx.x == 0) {
      const int v = queue + 8 * atomicAdd(&tickets[queue], 1);
      *s_item = v < n_virtual ? chunked_item(v, n_items) : -2;
    }
    __syncthreads();
    const int q = *s_item;
    if (q == -2) {  // queue exhausted
      ++qsel;
      continue;
    }
    if (q < 0) continue;  // a virtual block without an item
    const int4 item = g.work[q];
    const int tile = item.w >> kTileShift;
    if (GATED) {
      gemm_bf16_item<true, true>(g, smem, item);
      __syncthreads();  // every thread's h stores happen before thread 0's release ...
      if (threadIdx.x == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");  // ... which makes them visible device-wide ...
        atomicAdd(&tile_ready[tile], 1);                     // ... before the item is counted
      }
    } else {
      if (threadIdx.x == 0) {
        int polls = 0;
        while (__hip_atomic_load(&tile_ready[tile], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < nt1) {
          __builtin_amdgcn_s_sleep(32);
          if (++polls > kMaxPolls) {
            *error = 1;
            break;
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");  // order the loads of h after the counter
      }
      __syncthreads();
      gemm_bf16_item<false, true>(g, smem, item);
    }
  }
}

__global__ __launch_bounds__(kGemmThreads, 1) void gemm_bf16_pipeline_kernel(const PipelineArgs p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages x 64 KiB
  __shared__ int s_item;
  gemm_bf16_drain<true>(p.g1, smem, &s_item, p.tickets, p.tile_ready, p.error, p.nt1);
  gemm_bf16_drain<false>(p.g2, smem, &s_item, p.tickets + 8, p.tile_ready, p.error, p.nt1);
}

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
  const int le = item.x, m0 = item.y, rows = item.z, nt = item.w & ((1 << kTileShift) - 1);
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

// ------------------------------------------------------------------------------------------------
// Host-side launch helpers
// ------------------------------------------------------------------------------------------------
struct Ws {
  int32_t *header, *row_tok, *row_sole, *tile_ready;
  int4 *work1, *work2;
  float *row_w;
  void *h;
  float *o;
};

static Ws carve(void *workspace, const FwdLayout &L) {
  unsigned char *b = static_cast<unsigned char *>(workspace);
  Ws w;
  w.header = reinterpret_cast<int32_t *>(b + L.header);
  w.work1 = reinterpret_cast<int4 *>(b + L.work1);
  w.work2 = reinterpret_cast<int4 *>(b + L.work2);
  w.row_tok = reinterpret_cast<int32_t *>(b + L.row_tok);
  w.row_w = reinterpret_cast<float *>(b + L.row_w);
  w.row_sole = reinterpret_cast<int32_t *>(b + L.row_sole);
  w.tile_ready = reinterpret_cast<int32_t *>(b + L.tile_ready);
  w.h = b + L.h;
  w.o = reinterpret_cast<float *>(b + L.o);
  return w;
}

// sole != nullptr: also mark the rows GEMM-2 may write straight to y (see the GEMM-2 epilogue)
static int launch_prep(const moe_shape *s, const Derived &dv, const moe_dispatch *tb, const int32_t *topk_idx,
                       const float *topk_w, const Ws &w, int32_t *sole, hipStream_t st) {
  const int blocks = (int)std::min<int64_t>(1024, std::max<int64_t>(1, (dv.P_cap + 255) / 256));
  hipLaunchKernelGGL(fwd_prep_kernel, dim3(blocks), dim3(256), (size_t)(3 * dv.E_loc + 1 + 17) * sizeof(int), st,
                     tb->offsets, tb->perm, topk_w, s->T, s->k, dv.e_lo, dv.E_loc, dv.bm, (int)dv.P_cap, dv.max_mtiles,
                     dv.nt1, dv.nt2, w.header, w.work1, w.work2, w.row_tok, w.row_w, topk_idx, sole, w.tile_ready);
  return launch_status();
}

// GEMM-1 (gated) then GEMM-2 on the rows described by the tile table.  a1 / a1_map select the A operand of
// GEMM-1: the token matrix with the row -> token map (fused gather) or a materialised copy (map == nullptr).
static int launch_gemms(const moe_shape *s, const Derived &dv, const void *a1, const int32_t *a1_map, int a1_ld,
                        const void *packed_gu, const void *packed_down, const Ws &w, const int32_t *sole, void *y,
                        hipStream_t st, void *const *events = nullptr, bool pipelined = false) {
  auto mark = [&](int i) {
    if (events && events[i]) (void)hipEventRecord((hipEvent_t)events[i], st);
  };
  GemmArgs g1{};
  g1.A = a1; g1.row_map = a1_map; g1.Bp = packed_gu; g1.out = w.h; g1.row_w = nullptr;
  g1.row_sole = nullptr; g1.y = nullptr;
  g1.n_items = w.header + 0; g1.work = w.work1;
  g1.K = s->d; g1.N = s->f; g1.lda = a1_ld; g1.ldo = s->f;
  GemmArgs g2 = g1;
  g2.A = w.h; g2.row_map = nullptr; g2.Bp = packed_down; g2.out = w.o; g2.row_w = w.row_w;
  g2.row_sole = sole; g2.y = y;
  g2.K = s->f; g2.N = s->d; g2.lda = s->f; g2.ldo = s->d;
  g2.n_items = w.header + 3; g2.work = w.work2;
  const auto grid_of = [&](int nt) { return dim3((unsigned)(((size_t)dv.max_mtiles * nt + 255) / 256 * 256)); };
  if (s->dtype == MOE_BF16) {
    // the two LDS stages (128 KiB) exceed the default dynamic limit; raising it is a per-function attribute
    static const bool lds_ok = [] {
      const hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_bf16_kernel<true>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStageBytes);
      const hipError_t e2 = hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_bf16_kernel<false>),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStageBytes);
      return e1 == hipSuccess && e2 == hipSuccess;
    }();
    if (!lds_ok) return MOE_ERR_HIP;
    g1.n_ntiles = ceil_div(s->f, kBN / 2); g1.n_ktiles = ceil_div(s->d, kBK);
    g2.n_ntiles = ceil_div(s->d, kBN);     g2.n_ktiles = ceil_div(s->f, kBK);
    if (pipelined) {
      static const bool pipe_ok =
          hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_bf16_pipeline_kernel),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 2 * kStageBytes) == hipSuccess;
      // one resident workgroup per CU (each takes most of a CU's LDS)
      int dev = 0, n_cu = 0;
      if (!pipe_ok || hipGetDevice(&dev) != hipSuccess ||
          hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu < 1)
        return MOE_ERR_HIP;
      PipelineArgs pa;
      pa.g1 = g1; pa.g2 = g2;
      pa.tickets = w.header + 8; pa.tile_ready = w.tile_ready; pa.error = w.header + 24; pa.nt1 = dv.nt1;
      hipLaunchKernelGGL(gemm_bf16_pipeline_kernel, dim3((unsigned)n_cu), dim3(kGemmThreads), 2 * kStageBytes, st,
                         pa);
      mark(2);
      mark(3);
      return launch_status();
    }
    hipLaunchKernelGGL(gemm_bf16_kernel<true>, grid_of(dv.nt1), dim3(kGemmThreads), 2 * kStageBytes, st,
                       g1);
    int rc = launch_status();
    mark(2);
    if (rc != MOE_OK) return rc;
    hipLaunchKernelGGL(gemm_bf16_kernel<false>, grid_of(dv.nt2), dim3(kGemmThreads), 2 * kStageBytes, st,
                       g2);
    mark(3);
    return launch_status();
  }
  g1.n_ntiles = ceil_div(s->f, kFBN); g1.n_ktiles = dv.E_loc;
  g2.n_ntiles = ceil_div(s->d, kFBN); g2.n_ktiles = dv.E_loc;
  hipLaunchKernelGGL(gemm_f32_kernel<true>, grid_of(dv.nt1), dim3(256), 0, st, g1);
  int rc = launch_status();
  mark(2);
  if (rc != MOE_OK) return rc;
  hipLaunchKernelGGL(gemm_f32_kernel<false>, grid_of(dv.nt2), dim3(256), 0, st, g2);
  mark(3);
  return launch_status();
}

static int launch_combine(const moe_shape *s, const Derived &dv, const float *rows, const int32_t *topk_idx,
                          const moe_dispatch *tb, void *y, bool skip_sole, hipStream_t st) {
  if (s->dtype == MOE_BF16)
    hipLaunchKernelGGL(combine_kernel<bf16_t>, dim3(s->T), dim3(256), 0, st, rows, topk_idx, tb->inv_perm,
                       tb->offsets, s->k, s->d, dv.e_lo, dv.E_loc, (int)dv.P_cap, (int)skip_sole, static_cast<bf16_t *>(y));
  else
    hipLaunchKernelGGL(combine_kernel<float>, dim3(s->T), dim3(256), 0, st, rows, topk_idx, tb->inv_perm,
                       tb->offsets, s->k, s->d, dv.e_lo, dv.E_loc, (int)dv.P_cap, (int)skip_sole, static_cast<float *>(y));
  return launch_status();
}

static bool tables_ok(const moe_dispatch *t) {
  return t && t->counts && t->offsets && t->perm && t->inv_perm && t->rank_counts && t->rank_offsets &&
         t->dedup_tok && t->dedup_mask && t->pair_to_dedup;
}

}  // namespace moe355

using namespace moe355;

extern "C" int moe_pack_weights(const moe_shape *shape, const void *W_gate, const void *W_up, const void *W_down,
                                void *packed_gate_up, void *packed_down, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!W_gate || !W_up || !W_down || !packed_gate_up || !packed_down) return MOE_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  begin_launches();
  const int d = shape->d, f = shape->f;
  if (shape->dtype == MOE_F32) {
    const size_t one = (size_t)dv.E_loc * d * f;
    float *gu = static_cast<float *>(packed_gate_up);
    hipLaunchKernelGGL(copy_f32_kernel, dim3(1024), dim3(256), 0, st, static_cast<const float *>(W_gate), gu, one);
    hipLaunchKernelGGL(copy_f32_kernel, dim3(1024), dim3(256), 0, st, static_cast<const float *>(W_up), gu + one, one);
    hipLaunchKernelGGL(copy_f32_kernel, dim3(1024), dim3(256), 0, st, static_cast<const float *>(W_down),
                       static_cast<float *>(packed_down), one);
    return launch_status();
  }
  const int nt1 = ceil_div(f, kBN / 2), kt1 = ceil_div(d, kBK);
  const int nt2 = ceil_div(d, kBN), kt2 = ceil_div(f, kBK);
  if (nt1 > 65535 || nt2 > 65535 || dv.E_loc > 65535) return MOE_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(pack_bf16_kernel<true>, dim3(kt1, nt1, dv.E_loc), dim3(256), 0, st,
                     static_cast<const bf16_t *>(W_gate), static_cast<const bf16_t *>(W_up),
                     static_cast<bf16_t *>(packed_gate_up), d, f, nt1, kt1);
  if ((rc = launch_status()) != MOE_OK) return rc;
  hipLaunchKernelGGL(pack_bf16_kernel<false>, dim3(kt2, nt2, dv.E_loc), dim3(256), 0, st,
                     static_cast<const bf16_t *>(W_down), static_cast<const bf16_t *>(nullptr),
                     static_cast<bf16_t *>(packed_down), f, d, nt2, kt2);
  return launch_status();
}

static int forward_common(const moe_shape *shape, const void *x, const int32_t *topk_idx, const float *topk_w,
                          const moe_dispatch *tables, const void *packed_gate_up, const void *packed_down, void *y,
                          void *workspace, size_t workspace_bytes, void *stream, bool fused,
                          void *const *events = nullptr, int gemm_launches = 0) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!x || !topk_idx || !topk_w || !packed_gate_up || !packed_down || !y || !tables_ok(tables))
    return MOE_ERR_INVALID_ARG;
  const size_t need = fused ? moe_forward_workspace_bytes(shape) : moe_unfused_workspace_bytes(shape);
  if (!workspace || workspace_bytes < need) return MOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return MOE_ERR_INVALID_ARG;
  if ((int64_t)dv.max_mtiles * std::max(dv.nt1, dv.nt2) > (int64_t)1 << 30) return MOE_ERR_UNSUPPORTED;
  // gemm_launches: 0 = by shape, 1 = resident kernel with the tile-level hand-over (bf16 only), 2 = two launches
  if (gemm_launches == 1 && shape->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  const bool pipelined = (gemm_launches ? gemm_launches : moe_forward_gemm_launches(shape)) == 1;
  // a work item packs its N tile and its M-tile id into one word
  if (std::max(dv.nt1, dv.nt2) >= 1 << kTileShift || dv.max_mtiles >= 1 << (31 - kTileShift)) return MOE_ERR_UNSUPPORTED;
  // the GEMM kernels address A rows with 32-bit element offsets (row * row length)
  if (std::max<int64_t>(shape->T, dv.P_cap) * std::max(shape->d, shape->f) >= (int64_t)1 << 32) return MOE_ERR_UNSUPPORTED;
  if (shape->T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  begin_launches();
  const FwdLayout L = forward_layout(shape, dv);
  const Ws w = carve(workspace, L);
  auto mark = [&](int i) {
    if (events && events[i]) (void)hipEventRecord((hipEvent_t)events[i], st);
  };
  // fused bf16 layers: GEMM-2 writes the rows that need no reduction straight to y and Combine skips them
  int32_t *sole = fused && shape->dtype == MOE_BF16 ? w.row_sole : nullptr;
  mark(0);
  if ((rc = launch_prep(shape, dv, tables, topk_idx, topk_w, w, sole, st)) != MOE_OK) return rc;
  mark(1);
  if (fused) {
    if ((rc = launch_gemms(shape, dv, x, w.row_tok, shape->d, packed_gate_up, packed_down, w, sole, y, st,
                           events, pipelined)) != MOE_OK)
      return rc;
    rc = launch_combine(shape, dv, w.o, topk_idx, tables, y, sole != nullptr, st);
    mark(4);
    return rc;
  }
  // unfused: gather copy -> GEMMs on the copy -> zero -> atomic scatter-add -> cast
  unsigned char *b = static_cast<unsigned char *>(workspace);
  const size_t rows = (size_t)(dv.P_cap > 0 ? dv.P_cap : 1);
  void *xs = b + L.total;
  float *y32 = reinterpret_cast<float *>(b + L.total + align_up(rows * (size_t)shape->d * dv.elt, 256));
  const int row_chunks = shape->d * dv.elt / 16;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)rows), dim3(256), 0, st, static_cast<const uint4 *>(x),
                     w.header, w.row_tok, row_chunks, static_cast<uint4 *>(xs));
  if ((rc = launch_status()) != MOE_OK) return rc;
  if ((rc = launch_gemms(shape, dv, xs, nullptr, shape->d, packed_gate_up, packed_down, w, nullptr, nullptr, st, nullptr,
                         pipelined)) != MOE_OK) return rc;
  const size_t n = (size_t)shape->T * shape->d;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, st, reinterpret_cast<float4 *>(y32), n / 4);
  hipLaunchKernelGGL(scatter_add_kernel, dim3((unsigned)rows), dim3(256), 0, st, w.o, w.header, w.row_tok, shape->d,
                     y32);
  if (shape->dtype == MOE_BF16)
    hipLaunchKernelGGL(cast_rows_kernel<bf16_t>, dim3(2048), dim3(256), 0, st, y32, static_cast<bf16_t *>(y), n / 8);
  else
    hipLaunchKernelGGL(cast_rows_kernel<float>, dim3(2048), dim3(256), 0, st, y32, static_cast<float *>(y), n / 8);
  return launch_status();
}

extern "C" int moe_fused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx, const float *topk_w,
                                 const moe_dispatch *tables, const void *packed_gate_up, const void *packed_down,
                                 void *y, void *workspace, size_t workspace_bytes, void *stream) {
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true);
}

extern "C" int moe_fused_forward_timed(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                       const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                       const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                       void *stream, void *const *events) {
  if (!events) return MOE_ERR_INVALID_ARG;
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true, events);
}

extern "C" int moe_fused_forward_two_launch(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                            const float *topk_w, const moe_dispatch *tables,
                                            const void *packed_gate_up, const void *packed_down, void *y,
                                            void *workspace, size_t workspace_bytes, void *stream,
                                            void *const *events) {
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true, events, 2);
}

extern "C" int moe_fused_forward_one_launch(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                            const float *topk_w, const moe_dispatch *tables,
                                            const void *packed_gate_up, const void *packed_down, void *y,
                                            void *workspace, size_t workspace_bytes, void *stream,
                                            void *const *events) {
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true, events, 1);
}

extern "C" int moe_unfused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                   const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                   const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                   void *stream) {
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, false);
}

extern "C" int moe_dispatch_gather(const moe_shape *shape, const void *x, const moe_dispatch *tables, void *xs,
                                   void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!x || !xs || !tables_ok(tables)) return MOE_ERR_INVALID_ARG;
  if (shape->T == 0) return MOE_OK;
  const int nlr = shape->local_rank_end - shape->local_rank_begin;
  const int64_t max_entries = (int64_t)shape->T * (shape->k < nlr ? shape->k : nlr);
  begin_launches();
  hipLaunchKernelGGL(dispatch_gather_kernel, dim3((unsigned)max_entries), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const uint4 *>(x), tables->rank_offsets, tables->dedup_tok, tables->dedup_mask,
                     tables->inv_perm, tables->offsets, shape->T, shape->k, shape->local_rank_begin,
                     shape->local_rank_end, dv.e_lo, (int)dv.P_cap, shape->d * dv.elt / 16, static_cast<uint4 *>(xs));
  return launch_status();
}

extern "C" int moe_combine_reduce(const moe_shape *shape, const float *rows, const int32_t *topk_idx,
                                  const moe_dispatch *tables, void *y, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!rows || !topk_idx || !y || !tables_ok(tables)) return MOE_ERR_INVALID_ARG;
  if (shape->T == 0) return MOE_OK;
  begin_launches();
  return launch_combine(shape, dv, rows, topk_idx, tables, y, false, (hipStream_t)stream);
}
