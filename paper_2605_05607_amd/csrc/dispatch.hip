// moe_build_dispatch: per-expert counts and offsets (the nactive[expert] of Sec. III-E), the stable
// algebraic<->layout row maps (AL Table of Sec. III-D; token id list per tile of Sec. IV-B) and the table of
// distinct (token, rank) pairs (the redundancy of Sec. II-B; rank(e) = e / experts_per_rank, Sec. III-D).
//
// Two small kernels, no atomics on device memory, so the result does not depend on scheduling:
//   1. hist : the token range is cut into <= 64 chunks, one block per chunk counts its pairs per expert and
//             its first-of-rank pairs per rank (LDS counters);
//   2. place: every block first sums the chunk histograms (all chunks -> counts, earlier chunks -> its own
//             starting cursors) and scans the counts across experts into offsets (block 0 writes them out).
//             The chunk is cut once more into one contiguous token range per wave; a count of those ranges
//             (LDS) turns the chunk cursors into per-wave cursors, and every wave then walks its range in pair
//             order: lanes holding the same expert are found with one ballot per bit of the expert id, the
//             popcount of the lower lanes is the rank inside the group, and the highest lane of the group
//             advances the wave's LDS cursor.
#include <algorithm>

#include "common.h"

namespace moe355 {

constexpr int kMaxChunks = 64;

struct PairLane {
  int t, j, e, r;
  bool active, valid;
};

// Lane -> pair assignment of one iteration: floor(64 / k) whole tokens, slot-major inside a token.
__device__ __forceinline__ int ceil_div_dev(int a, int b) { return (a + b - 1) / b; }

__device__ __forceinline__ int load_expert(const int32_t *__restrict__ topk_idx, int t0, int t_end, int k, int tpi) {
  const int lane = lane_id();
  const int tl = lane / k;
  const int t = t0 + tl;
  return (tl < tpi && t < t_end) ? topk_idx[(size_t)t * k + (lane - tl * k)] : -1;
}

// `e` is this lane's expert id as returned by load_expert for the same t0 (fetched one iteration ahead so that
// the walk does not wait on global memory every 64 pairs).
__device__ __forceinline__ PairLane make_pair(int e, int t0, int t_end, int k, int tpi, int E, int epr) {
  PairLane p;
  const int lane = lane_id();
  const int tl = lane / k;
  p.j = lane - tl * k;
  p.t = t0 + tl;
  p.active = tl < tpi && p.t < t_end;
  p.e = p.active ? e : -1;
  p.valid = p.active && p.e >= 0 && p.e < E;
  p.r = p.valid ? p.e / epr : -1;
  return p;
}

// Slots of the same token that lie on the same rank as this lane's slot (bit jj per slot).
__device__ __forceinline__ uint32_t same_rank_slots(const PairLane &p, int k) {
  const int lane = lane_id();
  uint32_t m = 0;
  for (int jj = 0; jj < k; ++jj) {
    const int rr = __shfl(p.r, (lane - p.j + jj) & 63, 64);
    if (p.valid && rr == p.r) m |= 1u << jj;
  }
  return m;
}

// Lanes among `pred` lanes whose `key` equals this lane's key (bits = number of significant key bits).
__device__ __forceinline__ unsigned long long match_lanes(bool pred, int key, int bits) {
  unsigned long long m = __ballot(pred);
  for (int b = 0; b < bits; ++b) {
    const bool bit = (key >> b) & 1;
    const unsigned long long bal = __ballot(pred && bit);
    m &= bit ? bal : ~bal;
  }
  return m;
}

// Adds the pairs of tokens [t_begin, t_end) to the LDS counters cnt[E] / rcnt[R] (one wave; the counters may
// be shared with other waves).
__device__ __forceinline__ void count_range(const int32_t *__restrict__ topk_idx, int t_begin, int t_end, int k,
                                            int E, int epr, int *cnt, int *rcnt) {
  const int tpi = kWave / k;
  int e_next = load_expert(topk_idx, t_begin, t_end, k, tpi);
  for (int t0 = t_begin; t0 < t_end; t0 += tpi) {
    const PairLane p = make_pair(e_next, t0, t_end, k, tpi, E, epr);
    e_next = load_expert(topk_idx, t0 + tpi, t_end, k, tpi);
    const uint32_t slots = same_rank_slots(p, k);
    if (p.valid) {
      atomicAdd(&cnt[p.e], 1);
      if ((slots & ((1u << p.j) - 1u)) == 0) atomicAdd(&rcnt[p.r], 1);  // first slot of its (token, rank)
    }
  }
}

constexpr int kTableThreads = 512;  // block size of both kernels

__global__ __launch_bounds__(kTableThreads) void dispatch_hist_kernel(const int32_t *__restrict__ topk_idx, int T,
                                                                      int E, int k, int R, int tpc,
                                                                      int32_t *__restrict__ chunk_cnt,
                                                                      int32_t *__restrict__ chunk_rcnt) {
  extern __shared__ int sm[];
  int *cnt = sm;
  int *rcnt = sm + E;
  const int c = blockIdx.x;
  const int wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
  for (int i = threadIdx.x; i < E + R; i += blockDim.x) sm[i] = 0;
  __syncthreads();
  const int t_begin = c * tpc;
  const int t_end = min(T, t_begin + tpc);
  const int tpw = ceil_div_dev(tpc, nwaves);
  count_range(topk_idx, min(t_end, t_begin + wave * tpw), min(t_end, t_begin + (wave + 1) * tpw), k, E, E / R, cnt,
              rcnt);
  __syncthreads();
  // histograms are stored expert-major ([expert][chunk]) so that the placement kernel reads one expert's 64
  // chunk counts as one contiguous 256-byte run
  for (int i = threadIdx.x; i < E; i += blockDim.x) chunk_cnt[(size_t)i * kMaxChunks + c] = cnt[i];
  for (int i = threadIdx.x; i < R; i += blockDim.x) chunk_rcnt[(size_t)i * kMaxChunks + c] = rcnt[i];
}

__global__ __launch_bounds__(kTableThreads) void dispatch_place_kernel(
    const int32_t *__restrict__ topk_idx, int T, int E, int k, int R, int tpc, int nch, int ebits, int rbits, int nwalk,
    const int32_t *__restrict__ chunk_cnt, const int32_t *__restrict__ chunk_rcnt, int32_t *__restrict__ counts,
    int32_t *__restrict__ offsets, int32_t *__restrict__ rank_counts, int32_t *__restrict__ rank_offsets,
    int32_t *__restrict__ perm, int32_t *__restrict__ inv_perm, int32_t *__restrict__ dedup_tok,
    uint32_t *__restrict__ dedup_mask, int32_t *__restrict__ pair_to_dedup) {
  extern __shared__ int sm[];
  int *cursor = sm;            // [E] next free layout row of each expert for this chunk
  int *rcursor = sm + E;       // [R] next free dedup entry of each rank for this chunk
  int *tot = rcursor + R;      // [E + R] totals over all chunks
  int *scratch = tot + E + R;  // [17]
  int *sub = scratch + 17;     // [nwalk][E + R] per walking wave: pair counts of its token range, then its cursors
  const int lane = lane_id();
  const int wave = threadIdx.x >> 6;
  const int c = blockIdx.x;
  const int epr = E / R;
  // token range of this wave inside the chunk (waves >= nwalk only help with the tables)
  const int chunk_begin = c * tpc;
  const int chunk_end = min(T, chunk_begin + tpc);
  const int tpw = ceil_div_dev(tpc, nwalk);
  const int t_begin = min(chunk_end, chunk_begin + min(wave, nwalk) * tpw);
  const int t_end = wave < nwalk ? min(chunk_end, t_begin + tpw) : t_begin;
  for (int i = threadIdx.x; i < nwalk * (E + R); i += blockDim.x) sub[i] = 0;
  __syncthreads();
  if (wave < nwalk) count_range(topk_idx, t_begin, t_end, k, E, epr, sub + wave * (E + R), sub + wave * (E + R) + E);
  // per expert / rank: total over all chunks and the part that belongs to earlier chunks
  for (int i = threadIdx.x; i < E + R; i += blockDim.x) {
    const int4 *row = reinterpret_cast<const int4 *>(i < E ? chunk_cnt + (size_t)i * kMaxChunks
                                                           : chunk_rcnt + (size_t)(i - E) * kMaxChunks);
    int4 v[kMaxChunks / 4];
#pragma unroll
    for (int q = 0; q < kMaxChunks / 4; ++q) v[q] = row[q];  // 16 independent 16-byte loads
    int total = 0, before = 0;
#pragma unroll
    for (int q = 0; q < kMaxChunks / 4; ++q) {
      const int vals[4] = {v[q].x, v[q].y, v[q].z, v[q].w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int cc = q * 4 + u;
        const int val = cc < nch ? vals[u] : 0;  // slots of chunks that do not exist hold stale workspace bytes
        total += val;
        before += cc < c ? val : 0;
      }
    }
    tot[i] = total;
    sm[i] = before;
  }
  __syncthreads();
  // exclusive scan of the totals across experts, then across ranks: each thread owns a run of consecutive items
  for (int pass = 0; pass < 2; ++pass) {
    const int n = pass == 0 ? E : R;
    const int *src = pass == 0 ? tot : tot + E;
    int *cur = pass == 0 ? cursor : rcursor;
    int32_t *cnt_out = pass == 0 ? counts : rank_counts;
    int32_t *off_out = pass == 0 ? offsets : rank_offsets;
    const int ipt = (n + blockDim.x - 1) / blockDim.x;
    const int lo = min(n, (int)threadIdx.x * ipt);
    const int hi = min(n, lo + ipt);
    int local = 0;
    for (int i = lo; i < hi; ++i) local += src[i];
    int total;
    int run = block_exclusive_scan(local, scratch, &total);
    for (int i = lo; i < hi; ++i) {
      const int v = src[i];
      if (c == 0) {
        cnt_out[i] = v;
        off_out[i] = run;
      }
      cur[i] += run;
      run += v;
    }
    if (c == 0 && threadIdx.x == 0) off_out[n] = total;
    __syncthreads();
  }
  // chunk cursors -> per-wave cursors: wave w starts where the waves before it end
  for (int i = threadIdx.x; i < E + R; i += blockDim.x) {
    int run = sm[i];
    for (int w = 0; w < nwalk; ++w) {
      const int v = sub[w * (E + R) + i];
      sub[w * (E + R) + i] = run;
      run += v;
    }
  }
  __syncthreads();
  if (wave >= nwalk) return;  // each walk is a single-wave job; no block barrier below
  cursor = sub + wave * (E + R);
  rcursor = cursor + E;
  const int tpi = kWave / k;
  const unsigned long long lower = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  const long long npairs = (long long)T * k;
  const long long ndedup = (long long)T * min(k, R);
  int e_next = load_expert(topk_idx, t_begin, t_end, k, tpi);
  for (int t0 = t_begin; t0 < t_end; t0 += tpi) {
    const PairLane p = make_pair(e_next, t0, t_end, k, tpi, E, epr);
    e_next = load_expert(topk_idx, t0 + tpi, t_end, k, tpi);
    const size_t pid = (size_t)p.t * k + p.j;

    // ---- layout row of every pair (stable: lower lanes are earlier pairs) ----
    const unsigned long long grp = match_lanes(p.valid, p.e, ebits);
    int row = -1;
    if (p.valid) row = cursor[p.e] + __popcll(grp & lower);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (p.valid && (lane == 63 || (grp >> (lane + 1)) == 0)) cursor[p.e] = row + 1;
    if (p.active) inv_perm[pid] = row;
    if (p.valid && row >= 0 && row < npairs) perm[row] = (int32_t)pid;

    // ---- distinct (token, rank) entries ----
    const uint32_t slots = same_rank_slots(p, k);
    const bool first = p.valid && (slots & ((1u << p.j) - 1u)) == 0;
    const unsigned long long rgrp = match_lanes(first, p.r, rbits);
    int pos = -1;
    if (first) pos = rcursor[p.r] + __popcll(rgrp & lower);
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (first && (lane == 63 || (rgrp >> (lane + 1)) == 0)) rcursor[p.r] = pos + 1;
    if (first && pos >= 0 && pos < ndedup) {
      dedup_tok[pos] = p.t;
      dedup_mask[pos] = slots;
    }
    const int first_slot = slots ? __builtin_ctz(slots) : 0;
    const int pos_of_first = __shfl(pos, (lane - p.j + first_slot) & 63, 64);
    if (p.active) pair_to_dedup[pid] = p.valid ? pos_of_first : -1;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

}  // namespace moe355

using namespace moe355;

static int chunking(int T, int *tpc) {
  if (T <= 0) {
    *tpc = 1;
    return 0;
  }
  *tpc = ceil_div(T, kMaxChunks);
  return ceil_div(T, *tpc);
}

extern "C" size_t moe_dispatch_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  return align_up((size_t)kMaxChunks * (shape->E + shape->R) * sizeof(int32_t), 256);
}

// Both forms of the call: the chunk histograms live in `chunk_ws` (kMaxChunks * (E + R) int32).
static int build_dispatch_launches(const moe_shape *shape, const int32_t *topk_idx, const moe_dispatch *out,
                                   int32_t *chunk_ws, hipStream_t st) {
  const int T = shape->T, E = shape->E, k = shape->k, R = shape->R;
  int tpc;
  const int nch = chunking(T, &tpc);
  int32_t *chunk_cnt = chunk_ws;
  int32_t *chunk_rcnt = chunk_cnt + (size_t)kMaxChunks * E;
  int rc;
  begin_launches();
  const size_t sm_wave = (size_t)(E + R) * sizeof(int);
  if (nch > 0) {
    hipLaunchKernelGGL(dispatch_hist_kernel, dim3(nch), dim3(kTableThreads), sm_wave, st, topk_idx, T, E, k, R, tpc,
                       chunk_cnt, chunk_rcnt);
    if ((rc = launch_status()) != MOE_OK) return rc;
  }
  int ebits = 0, rbits = 0;
  while ((1 << ebits) < E) ++ebits;
  while ((1 << rbits) < R) ++rbits;
  // The placement kernel keeps (2 + walking waves) arrays of E + R counters in LDS; with the largest E and R even
  // one walking wave needs more than the default 64 KiB of dynamic LDS, so the limit is raised (once per device).
  constexpr size_t kPlaceLds = 144 * 1024;
  static std::atomic<uint64_t> done{0};
  if (!allow_dynamic_lds(reinterpret_cast<const void *>(&dispatch_place_kernel), (int)kPlaceLds, done))
    return MOE_ERR_HIP;
  const size_t fit = (kPlaceLds - 1024) / sm_wave;  // arrays that fit; at least 3 for E + R <= 8192
  const int nwalk = (int)std::max<size_t>(1, std::min<size_t>(kTableThreads / kWave, fit > 2 ? fit - 2 : 1));
  // with T == 0 a single block still writes the all-zero counts and offsets
  hipLaunchKernelGGL(dispatch_place_kernel, dim3(nch > 0 ? nch : 1), dim3(kTableThreads),
                     (size_t)((2 + nwalk) * (E + R) + 17) * sizeof(int), st, topk_idx, T, E, k, R, tpc, nch, ebits, rbits,
                     nwalk, chunk_cnt,
                     chunk_rcnt, out->counts, out->offsets, out->rank_counts, out->rank_offsets, out->perm,
                     out->inv_perm, out->dedup_tok, out->dedup_mask, out->pair_to_dedup);
  return launch_status();
}

static bool dispatch_outputs_ok(const moe_dispatch *out) {
  return out && out->counts && out->offsets && out->perm && out->inv_perm && out->rank_counts && out->rank_offsets &&
         out->dedup_tok && out->dedup_mask && out->pair_to_dedup;
}

extern "C" int moe_build_dispatch(const moe_shape *shape, const int32_t *topk_idx, const moe_dispatch *out,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!topk_idx || !dispatch_outputs_ok(out)) return MOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < moe_dispatch_workspace_bytes(shape)) return MOE_ERR_WORKSPACE;
  return build_dispatch_launches(shape, topk_idx, out, static_cast<int32_t *>(workspace), (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------------
// The same call for callers that cannot allocate device memory (code under HIP graph capture, serving loops,
// harnesses that forbid hipMalloc): the chunk histograms live in a file-scope device array instead of a caller
// workspace.  Every GPU holds its own copy of the array at its own address; the address is looked up once per device
// (hipGetSymbolAddress with that device current) and kept.  In host code the array's name is only a handle for that
// lookup: kernels and copies always get the looked-up pointer.
// ------------------------------------------------------------------------------------------------
namespace moe355 {
constexpr int kStaticMaxCounters = MOE_NOALLOC_MAX_COUNTERS;  // limit on E + R
static __device__ __align__(256) unsigned char scratch[(size_t)kMaxChunks * kStaticMaxCounters * sizeof(int32_t)];
constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];  // zero-initialised: not looked up yet

// Device address of `scratch` on the current device (nullptr on failure).  Allocates nothing.
static void *scratch_on_current_device() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
    (void)hipGetLastError();
    return nullptr;
  }
  g_scratch_ptr[dev].store(p, std::memory_order_release);  // every thread looks up the same address
  return p;
}
}  // namespace moe355

extern "C" int moe_build_dispatch_noalloc(const moe_shape *shape, const int32_t *topk_idx, const moe_dispatch *out,
                                          void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!topk_idx || !dispatch_outputs_ok(out)) return MOE_ERR_INVALID_ARG;
  if (shape->E + shape->R > kStaticMaxCounters) return MOE_ERR_UNSUPPORTED;  // beyond the static scratch
  void *ws = scratch_on_current_device();
  if (!ws) return MOE_ERR_HIP;
  // Nothing has to start at zero: the histogram kernel overwrites the rows of every chunk that exists and the
  // placement kernel ignores the others.
  return build_dispatch_launches(shape, topk_idx, out, static_cast<int32_t *>(ws), (hipStream_t)stream);
}
