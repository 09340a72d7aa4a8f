// Tile table: work lists of the two GEMMs and per-row metadata of the local layout segment.
#pragma once
#include "forward_types.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Work lists and per-row metadata of the local layout segment.
// header[0] = work items of GEMM-1, header[1] = P (local rows), header[2] = first layout row of the segment,
// header[3] = work items of GEMM-2, header[4] = M tiles; header[8..15] / [16..23] = ticket counters of the GEMM-1 /
// GEMM-2 queues and header[24] = error flag of the resident GEMM kernel (all cleared here).  row_tile / tile_done
// (both may be null): M tile of every local row and the per-tile counter of finished GEMM-2 items, for the resident
// kernel that also runs Combine.
//
// A work item is one output tile (expert, M tile, N tile): int4 (local expert, first local row, valid rows,
// N tile | M-tile id << 12).  An expert's partial tile (its last rows) walks with the expert's full tiles when it has
// more than 64 rows: it needs the same weight panels, and running it in the same chunks fetches them once instead of
// twice (measured on layers whose experts hold one or two full tiles and a partial one: the L2 fills of GEMM-1 were
// twice the weights).  Partial tiles of at most 64 rows (pure weight streaming) are mixed into those chunks or
// trail them (see the list order below).
// The order of the list is also what keeps the L2 useful:
// the chip has 8 XCDs with a private 4 MiB L2 each and workgroup i runs on XCD i % 8, so every GEMM workgroup
// maps its index to a list position such that XCD x works through the 32-item chunks x, x + 8, x + 16, ...;
// and a chunk is a block of (up to 8 M tiles) x (32 / that many N tiles) of ONE expert, so the 32 workgroups
// that are resident on an XCD at the same time share a few A slabs and a few weight panels instead of
// streaming 32 different ones through the L2.
// ------------------------------------------------------------------------------------------------

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
                                                       int32_t *__restrict__ tile_ready,
                                                       int32_t *__restrict__ row_tile,
                                                       int32_t *__restrict__ tile_done) {
  // LDS: full0[E_loc + 1] first full M tile of each expert | part[E_loc] rows of its partial tile (0 = none) |
  //      order[E_loc] partial tiles: first the large ones (> kStreamRows rows), largest first, then the
  //      streaming ones, largest first | only with row_tile: pos[E_loc] place of each expert's partial tile in
  //      `order` | 17 ints of scan scratch
  extern __shared__ int lds[];
  int *full0 = lds;
  int *part = full0 + E_loc + 1;
  int *order = part + E_loc;
  int *pos = order + E_loc;
  int *scratch = row_tile ? pos + E_loc : pos;
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
  int local_full = 0, local_small = 0;
  for (int le = lo; le < hi; ++le) {
    const int cnt = max(0, min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base));
    part[le] = cnt % bm;
    local_full += cnt / bm + ((cnt % bm) > kStreamRows);  // a large partial tile walks with the expert's full tiles
    local_small += (cnt % bm) != 0 && (cnt % bm) <= kStreamRows;
  }
  int n_full, n_big, n_small;
  int run = block_exclusive_scan(local_full, scratch, &n_full);
  for (int le = lo; le < hi; ++le) {
    const int cnt = max(0, min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base));
    full0[le] = run;
    run += cnt / bm + ((cnt % bm) > kStreamRows);
  }
  if (threadIdx.x == 0) full0[E_loc] = n_full;
  n_big = 0;  // (no separate class any more: see the list order below)
  (void)block_exclusive_scan(local_small, scratch, &n_small);
  __syncthreads();
  // rank sort of the streaming partial tiles (for very many experts keep the expert order)
  for (int le = lo; le < hi; ++le) {
    const int mine = part[le];
    if (mine == 0 || mine > kStreamRows) continue;
    int rank = 0;
    for (int o = 0; o < E_loc; ++o) {
      const int po = part[o];
      if (po == 0 || po > kStreamRows) continue;
      rank += E_loc <= 1024 ? (po > mine || (po == mine && o < le)) : (o < le);
    }
    order[rank] = le;
    if (row_tile) pos[le] = rank;
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
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_tiles; i += gridDim.x * blockDim.x) {
    tile_ready[i] = 0;
    if (tile_done) tile_done[i] = 0;
  }
  // M tile of every local row (the resident kernel's Combine stage looks up the tile whose GEMM-2 items it waits for)
  if (row_tile) {
    for (int r = blockIdx.x * blockDim.x + threadIdx.x; r < P; r += gridDim.x * blockDim.x) {
      // expert of row r: largest le whose first row is <= r
      int a = 0, b = E_loc;
      while (b - a > 1) {
        const int mid = (a + b) >> 1;
        if (min(P, offsets[e_lo + mid] - base) <= r) a = mid; else b = mid;
      }
      const int start = min(P, offsets[e_lo + a] - base);
      const int cnt = min(P, offsets[e_lo + a + 1] - base) - start;
      const int mt = (r - start) / bm;
      const int tile = (mt < cnt / bm || part[a] > kStreamRows) ? full0[a] + mt : n_full + pos[a];
      row_tile[r] = min(tile, max(n_tiles - 1, 0));
    }
  }
  for (int q = blockIdx.x * blockDim.x + threadIdx.x; q < n1 + n2; q += gridDim.x * blockDim.x) {
    const bool second = q >= n1;
    const int Nt = second ? nt2 : nt1;
    const int qq = second ? q - n1 : q;
    // List order.  Classes: F = full tiles and partial tiles of more than kStreamRows rows, S = streaming partial
    // tiles (class B, partial tiles as a list of their own, is empty: n_big = 0).
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
      // Inside the group the shorter side runs fastest.  The workgroups of an XCD start a few microseconds apart
      // (one whenever a CU becomes free), and the L2 keeps only the last few k-steps of what they stream; two items
      // share a panel through it only if they sit within a few list positions of each other, and with the shorter
      // side innermost both the A sharers and the B sharers do.
      if (Gcur <= Mcur) {
        mt = mg * Mg + r / Gcur;
        nt = ng * G + r % Gcur;
      } else {
        mt = mg * Mg + r % Mcur;
        nt = ng * G + r / Mcur;
      }
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
    if (cls == 0) {
      // the expert's last tile of this class may be its large partial tile
      const int cnt = min(P, offsets[e_lo + le + 1] - base) - min(P, offsets[e_lo + le] - base);
      if (mt >= cnt / bm) rows = part[le];
    }
    const int start = min(P, offsets[e_lo + le] - base);
    const int cnt_le = min(P, offsets[e_lo + le + 1] - base) - start;
    const int4 item = make_int4(le, start + mt * bm, rows | (cnt_le <= bm ? kItemLone : 0), nt | (tile << kTileShift));
    if (second) work2[qq] = item; else work1[qq] = item;
  }
}

}  // namespace moe355
