// moe_fused_forward and its building blocks: weight packing, tile table, grouped SwiGLU GEMMs (GEMM-1 and
// GEMM-2 of Sec. II-A) with the token gather fused into GEMM-1's operand load (Dispatch of Sec. II-A without a
// materialised copy), the gate weight applied in GEMM-2's epilogue (Sec. III-C), and the per-token reduction
// with a single write-back (Combine; the one-GPU form of the in-switch reduction of Sec. II-C).
#include <algorithm>
#include <atomic>
#include <mutex>

#include "backward_kernels.h"
#include "combine_kernels.h"
#include "fp8_kernels.h"
#include "gemm_bf16.h"
#include "gemm_f32.h"
#include "pack_kernels.h"
#include "prep_kernel.h"
#include "wgrad_bf16.h"

namespace moe355 {

// ------------------------------------------------------------------------------------------------
// Host-side launch helpers
// ------------------------------------------------------------------------------------------------
struct Ws {
  int32_t *header, *row_tok, *row_sole, *tile_ready, *row_tile, *tile_done;
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
  w.row_tile = reinterpret_cast<int32_t *>(b + L.row_tile);
  w.tile_done = reinterpret_cast<int32_t *>(b + L.tile_done);
  w.h = b + L.h;
  w.o = reinterpret_cast<float *>(b + L.o);
  return w;
}

// LDS of the tile-table kernel: three (with the row -> tile map: four) per-expert arrays and the scan scratch.
static size_t prep_lds_bytes(const Derived &dv, bool combine_tables) {
  return (size_t)((combine_tables ? 4 : 3) * dv.E_loc + 1 + 17) * sizeof(int);
}

// sole != nullptr: also mark the rows GEMM-2 may write straight to y (see the GEMM-2 epilogue);
// combine_tables: also the row -> M tile map and the cleared GEMM-2 counters of the resident kernel's Combine stage
static int launch_prep(const moe_shape *s, const Derived &dv, const moe_dispatch *tb, const int32_t *topk_idx,
                       const float *topk_w, const Ws &w, int32_t *sole, hipStream_t st,
                       bool combine_tables = false) {
  const int blocks = (int)std::min<int64_t>(1024, std::max<int64_t>(1, (dv.P_cap + 255) / 256));
  hipLaunchKernelGGL(fwd_prep_kernel, dim3(blocks), dim3(256), prep_lds_bytes(dv, combine_tables), st,
                     tb->offsets, tb->perm, topk_w, s->T, s->k, dv.e_lo, dv.E_loc, dv.bm, (int)dv.P_cap, dv.max_mtiles,
                     dv.nt1, dv.nt2, w.header, w.work1, w.work2, w.row_tok, w.row_w, topk_idx, sole, w.tile_ready,
                     combine_tables ? w.row_tile : nullptr, combine_tables ? w.tile_done : nullptr);
  return launch_status();
}

// Compute units of the current device, looked up once per device (0 on failure).
static int compute_units() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n > 0) return n;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return 0;
  cached[dev].store(n, std::memory_order_relaxed);
  return n;
}

// FP8 form of the GEMMs: quantised x with its per-token scales, the column scales that follow the packed tiles,
// and the per-expert scale of h.
struct Fp8Operands {
  const uint8_t *xq;
  const float *x_scale, *gu_scale, *down_scale, *h_scale;
};

static size_t fp8_tile_bytes(const moe_shape *s, const Derived &dv, int which) {
  if (which == 0) return (size_t)dv.E_loc * ceil_div(s->f, kBN / 2) * ceil_div(s->d, kFp8KStep) * kTileBytes;
  return (size_t)dv.E_loc * ceil_div(s->d, kBN) * ceil_div(s->f, kFp8KStep) * kTileBytes;
}

// GEMM-1 (gated) then GEMM-2 on the rows described by the tile table.  a1 / a1_map select the A operand of
// GEMM-1: the token matrix with the row -> token map (fused gather) or a materialised copy (map == nullptr).
static int launch_gemms(const moe_shape *s, const Derived &dv, const void *a1, const int32_t *a1_map, int a1_ld,
                        const void *packed_gu, const void *packed_down, const Ws &w, const int32_t *sole, void *y,
                        hipStream_t st, void *const *events = nullptr, bool pipelined = false,
                        const Fp8Operands *q = nullptr, void *keep_gu = nullptr, float *keep_o = nullptr,
                        int max_polls = kMaxPolls, int wait_extra = 0, const moe_dispatch *combine_tb = nullptr,
                        const int32_t *topk_idx = nullptr) {
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
  if (keep_gu) {  // training forward: g and u are kept, and every weighted row goes to the kept o
    g1.aux = keep_gu;
    g2.out = keep_o;
  }
  const auto grid_of = [&](int nt) { return dim3((unsigned)(((size_t)dv.max_mtiles * nt + 255) / 256 * 256)); };
  if (q) {
    static std::atomic<uint64_t> done1{0}, done2{0}, done_pipe{0};
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_kernel<true, true>), 2 * kStageBytes, done1) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_kernel<false, true>), 2 * kStageBytes, done2) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_fp8_pipeline_kernel), 2 * kStageBytes, done_pipe))
      return MOE_ERR_HIP;
    g1.A = q->xq; g1.a_scale = q->x_scale; g1.b_scale = q->gu_scale; g1.h_scale = q->h_scale;
    g2.b_scale = q->down_scale; g2.h_scale = q->h_scale;
    g1.n_ntiles = ceil_div(s->f, kBN / 2); g1.n_ktiles = ceil_div(s->d, kFp8KStep);
    g2.n_ntiles = ceil_div(s->d, kBN);     g2.n_ktiles = ceil_div(s->f, kFp8KStep);
    if (pipelined) {
      const int n_cu = compute_units();
      if (n_cu < 1) return MOE_ERR_HIP;
      PipelineArgs pa;
      pa.g1 = g1; pa.g2 = g2;
      pa.tickets = w.header + 8; pa.tile_ready = w.tile_ready; pa.error = w.header + 24; pa.nt1 = dv.nt1 + wait_extra;
      pa.max_polls = max_polls;
      hipLaunchKernelGGL(gemm_fp8_pipeline_kernel, dim3((unsigned)n_cu), dim3(kGemmThreads), 2 * kStageBytes, st, pa);
      mark(2);
      mark(3);
      return launch_status();
    }
    hipLaunchKernelGGL((gemm_bf16_kernel<true, true>), grid_of(dv.nt1), dim3(kGemmThreads), 2 * kStageBytes, st, g1);
    int rc = launch_status();
    mark(2);
    if (rc != MOE_OK) return rc;
    hipLaunchKernelGGL((gemm_bf16_kernel<false, true>), grid_of(dv.nt2), dim3(kGemmThreads), 2 * kStageBytes, st, g2);
    mark(3);
    return launch_status();
  }
  if (s->dtype == MOE_BF16) {
    // the two LDS stages (128 KiB) exceed the default dynamic limit; raising it is a per-function attribute
    static std::atomic<uint64_t> done1{0}, done2{0}, done_pipe{0};
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_kernel<true>), 2 * kStageBytes, done1) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_kernel<false>), 2 * kStageBytes, done2) ||
        !allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_pipeline_kernel), 2 * kStageBytes, done_pipe))
      return MOE_ERR_HIP;
    g1.n_ntiles = ceil_div(s->f, kBN / 2); g1.n_ktiles = ceil_div(s->d, kBK);
    g2.n_ntiles = ceil_div(s->d, kBN);     g2.n_ktiles = ceil_div(s->f, kBK);
    if (pipelined) {
      // one resident workgroup per CU (each takes most of a CU's LDS)
      const int n_cu = compute_units();
      if (n_cu < 1) return MOE_ERR_HIP;
      PipelineArgs pa;
      pa.g1 = g1; pa.g2 = g2;
      pa.tickets = w.header + 8; pa.tile_ready = w.tile_ready; pa.error = w.header + 24; pa.nt1 = dv.nt1 + wait_extra;
      pa.max_polls = max_polls;
      if (keep_gu) {
        static std::atomic<uint64_t> done_tp{0};
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_train_pipeline_kernel), 2 * kStageBytes, done_tp))
          return MOE_ERR_HIP;
        hipLaunchKernelGGL(gemm_train_pipeline_kernel, dim3((unsigned)n_cu), dim3(kGemmThreads), 2 * kStageBytes, st,
                           pa);
      } else if (combine_tb) {
        // Combine as the third stage of the same launch (wait_extra also raises its target, for the give-up test)
        static std::atomic<uint64_t> done_c{0};
        if (!allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_combine_kernel), 2 * kStageBytes, done_c))
          return MOE_ERR_HIP;
        pa.tile_done = w.tile_done; pa.row_tile = w.row_tile;
        pa.topk_idx = topk_idx; pa.inv_perm = combine_tb->inv_perm; pa.offsets = combine_tb->offsets;
        pa.header = w.header;
        pa.T = s->T; pa.k = s->k; pa.e_lo = dv.e_lo; pa.E_loc = dv.E_loc; pa.P_cap = (int)dv.P_cap;
        pa.nt2 = dv.nt2 + wait_extra; pa.n_mtiles_cap = dv.max_mtiles;
        hipLaunchKernelGGL(gemm_bf16_combine_kernel, dim3((unsigned)n_cu), dim3(kGemmThreads), 2 * kStageBytes, st,
                           pa);
      } else {
        hipLaunchKernelGGL(gemm_bf16_pipeline_kernel, dim3((unsigned)n_cu), dim3(kGemmThreads), 2 * kStageBytes, st,
                           pa);
      }
      mark(2);
      mark(3);
      return launch_status();
    }
    if (keep_gu) {
      static std::atomic<uint64_t> done_t{0};
      if (!allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_kernel<true, false, true>), 2 * kStageBytes,
                             done_t))
        return MOE_ERR_HIP;
      hipLaunchKernelGGL((gemm_bf16_kernel<true, false, true>), grid_of(dv.nt1), dim3(kGemmThreads), 2 * kStageBytes,
                         st, g1);
    } else {
      hipLaunchKernelGGL(gemm_bf16_kernel<true>, grid_of(dv.nt1), dim3(kGemmThreads), 2 * kStageBytes, st, g1);
    }
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
  const dim3 grid((unsigned)ceil_div(s->T, kCombineWaves)), block(kCombineWaves * 64);
#define MOE355_COMBINE(T_, FUSED_)                                                                             \
  hipLaunchKernelGGL((combine_kernel<T_, FUSED_>), grid, block, 0, st, rows, topk_idx, tb->inv_perm, tb->offsets, \
                     s->T, s->k, s->d, dv.e_lo, dv.E_loc, (int)dv.P_cap, static_cast<T_ *>(y))
  if (s->dtype == MOE_BF16) {
    if (skip_sole) MOE355_COMBINE(bf16_t, true); else MOE355_COMBINE(bf16_t, false);
  } else {
    if (skip_sole) MOE355_COMBINE(float, true); else MOE355_COMBINE(float, false);
  }
#undef MOE355_COMBINE
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
                          void *const *events = nullptr, int gemm_launches = 0, const float *h_scale = nullptr,
                          void *keep = nullptr, int max_polls = kMaxPolls, int wait_extra = 0) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!x || !topk_idx || !topk_w || !packed_gate_up || !packed_down || !y || !tables_ok(tables))
    return MOE_ERR_INVALID_ARG;
  const bool fp8 = h_scale != nullptr;  // FP8 GEMMs: bf16 layers whose rows are whole 16-code chunks
  if (fp8 && (shape->dtype != MOE_BF16 || shape->d % 16 != 0 || shape->f % 16 != 0)) return MOE_ERR_UNSUPPORTED;
  const size_t need = fp8     ? moe_fp8_forward_workspace_bytes(shape)
                      : fused ? moe_forward_workspace_bytes(shape)
                              : moe_unfused_workspace_bytes(shape);
  if (!workspace || workspace_bytes < need) return MOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return MOE_ERR_INVALID_ARG;
  // rows are moved 16 bytes at a time
  if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(y) | reinterpret_cast<uintptr_t>(packed_gate_up) |
       reinterpret_cast<uintptr_t>(packed_down)) % 16 != 0)
    return MOE_ERR_INVALID_ARG;
  if ((int64_t)dv.max_mtiles * std::max(dv.nt1, dv.nt2) > (int64_t)1 << 30) return MOE_ERR_UNSUPPORTED;
  // gemm_launches: 0 = by shape, 1 = resident kernel with the tile-level hand-over (bf16 only), 2 = two launches,
  // 3 = resident kernel that also runs Combine (bf16 inference forward only)
  if ((gemm_launches == 1 || gemm_launches == 3) && shape->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  const bool with_combine = gemm_launches == 3;
  if (with_combine && (!fused || fp8 || keep)) return MOE_ERR_UNSUPPORTED;
  if (with_combine && prep_lds_bytes(dv, true) > 64 * 1024) return MOE_ERR_UNSUPPORTED;  // the tile table's LDS
  const bool pipelined = with_combine || (gemm_launches ? gemm_launches : moe_forward_gemm_launches(shape)) == 1;
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
  // (not in the training forward, which keeps every weighted row for the backward pass)
  int32_t *sole = fused && shape->dtype == MOE_BF16 && !keep ? w.row_sole : nullptr;
  void *keep_gu = nullptr;
  float *keep_o = nullptr;
  if (keep) {
    const size_t rows = (size_t)(dv.P_cap > 0 ? dv.P_cap : 1);
    keep_gu = keep;
    keep_o = reinterpret_cast<float *>(static_cast<unsigned char *>(keep) + align_up(rows * 2 * shape->f * 2, 256));
  }
  mark(0);
  Fp8Operands q{};
  if (fp8) {
    // x as codes with one scale per token, behind the tile-table part of the workspace
    unsigned char *b = static_cast<unsigned char *>(workspace);
    uint8_t *xq = b + L.total;
    float *x_scale = reinterpret_cast<float *>(b + L.total + align_up((size_t)shape->T * shape->d, 256));
    hipLaunchKernelGGL(fp8_quantize_rows_kernel, dim3((unsigned)shape->T), dim3(256), 0, st,
                       static_cast<const uint4 *>(x), shape->d, xq, x_scale);
    if ((rc = launch_status()) != MOE_OK) return rc;
    q.xq = xq;
    q.x_scale = x_scale;
    q.gu_scale = reinterpret_cast<const float *>(static_cast<const unsigned char *>(packed_gate_up) +
                                                 align_up(fp8_tile_bytes(shape, dv, 0), 256));
    q.down_scale = reinterpret_cast<const float *>(static_cast<const unsigned char *>(packed_down) +
                                                   align_up(fp8_tile_bytes(shape, dv, 1), 256));
    q.h_scale = h_scale;
  }
  if ((rc = launch_prep(shape, dv, tables, topk_idx, topk_w, w, sole, st, with_combine)) != MOE_OK) return rc;
  mark(1);
  if (fused) {
    if ((rc = launch_gemms(shape, dv, x, w.row_tok, shape->d, packed_gate_up, packed_down, w, sole, y, st,
                           events, pipelined, fp8 ? &q : nullptr, keep_gu, keep_o, max_polls, wait_extra,
                           with_combine ? tables : nullptr, topk_idx)) != MOE_OK)
      return rc;
    if (!with_combine) rc = launch_combine(shape, dv, keep ? keep_o : w.o, topk_idx, tables, y, sole != nullptr, st);
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

extern "C" size_t moe_fp8_packed_weight_bytes(const moe_shape *shape, int which) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK || (which != 0 && which != 1)) return 0;
  const size_t scales = (size_t)dv.E_loc * (which == 0 ? 2 * (size_t)shape->f : (size_t)shape->d) * sizeof(float);
  return align_up(fp8_tile_bytes(shape, dv, which), 256) + align_up(scales, 256);
}

extern "C" size_t moe_fp8_forward_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  const size_t T = (size_t)(shape->T > 0 ? shape->T : 1);
  return forward_layout(shape, dv).total + align_up(T * shape->d, 256) + align_up(T * sizeof(float), 256);
}

extern "C" int moe_fp8_pack_weights(const moe_shape *shape, const void *W_gate, const void *W_up, const void *W_down,
                                    void *packed_gate_up, void *packed_down, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!W_gate || !W_up || !W_down || !packed_gate_up || !packed_down) return MOE_ERR_INVALID_ARG;
  if (shape->dtype != MOE_BF16 || shape->d % 16 != 0 || shape->f % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(packed_gate_up) | reinterpret_cast<uintptr_t>(packed_down)) % 16 != 0)
    return MOE_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  begin_launches();
  const int d = shape->d, f = shape->f;
  const int nt1 = ceil_div(f, kBN / 2), kt1 = ceil_div(d, kFp8KStep);
  const int nt2 = ceil_div(d, kBN), kt2 = ceil_div(f, kFp8KStep);
  if (nt1 > 65535 || nt2 > 65535 || dv.E_loc > 65535) return MOE_ERR_UNSUPPORTED;
  uint8_t *gu = static_cast<uint8_t *>(packed_gate_up), *dn = static_cast<uint8_t *>(packed_down);
  float *s_gu = reinterpret_cast<float *>(gu + align_up(fp8_tile_bytes(shape, dv, 0), 256));  // [E_loc][2][f]
  float *s_dn = reinterpret_cast<float *>(dn + align_up(fp8_tile_bytes(shape, dv, 1), 256));  // [E_loc][d]
  const bf16_t *Wg = static_cast<const bf16_t *>(W_gate), *Wu = static_cast<const bf16_t *>(W_up);
  const bf16_t *Wd = static_cast<const bf16_t *>(W_down);
  // column maxima (the reduction range cut into slices for enough workgroups), then scales in place
  const size_t n_gu = (size_t)dv.E_loc * 2 * f, n_dn = (size_t)dv.E_loc * d;
  hipLaunchKernelGGL(fill_f32_kernel, dim3(256), dim3(256), 0, st, s_gu, n_gu, 0.0f);
  hipLaunchKernelGGL(fill_f32_kernel, dim3(256), dim3(256), 0, st, s_dn, n_dn, 0.0f);
  const int slices_d = std::max(1, std::min(32, d / 64)), slices_f = std::max(1, std::min(32, f / 64));
  hipLaunchKernelGGL(fp8_column_amax_kernel, dim3(ceil_div(f, 256), dv.E_loc, slices_d), dim3(256), 0, st, Wg, d, f,
                     reinterpret_cast<uint32_t *>(s_gu), 2 * f);
  hipLaunchKernelGGL(fp8_column_amax_kernel, dim3(ceil_div(f, 256), dv.E_loc, slices_d), dim3(256), 0, st, Wu, d, f,
                     reinterpret_cast<uint32_t *>(s_gu + f), 2 * f);
  hipLaunchKernelGGL(fp8_column_amax_kernel, dim3(ceil_div(d, 256), dv.E_loc, slices_f), dim3(256), 0, st, Wd, f, d,
                     reinterpret_cast<uint32_t *>(s_dn), d);
  hipLaunchKernelGGL(fp8_scales_from_amax_kernel, dim3(256), dim3(256), 0, st, s_gu, n_gu);
  hipLaunchKernelGGL(fp8_scales_from_amax_kernel, dim3(256), dim3(256), 0, st, s_dn, n_dn);
  if ((rc = launch_status()) != MOE_OK) return rc;
  hipLaunchKernelGGL(pack_fp8_kernel<true>, dim3(kt1, nt1, dv.E_loc), dim3(256), 0, st, Wg, Wu, s_gu, s_gu + f, 2 * f,
                     gu, d, f, nt1, kt1);
  if ((rc = launch_status()) != MOE_OK) return rc;
  hipLaunchKernelGGL(pack_fp8_kernel<false>, dim3(kt2, nt2, dv.E_loc), dim3(256), 0, st, Wd,
                     static_cast<const bf16_t *>(nullptr), s_dn, static_cast<const float *>(nullptr), d, dn, f, d, nt2,
                     kt2);
  return launch_status();
}

extern "C" int moe_fp8_quantize_rows(int64_t rows, int cols, const void *x, void *codes, float *scales,
                                     void *stream) {
  if (rows < 0 || rows > 0x7FFFFFFF || cols < 8 || cols % 8 != 0) return MOE_ERR_INVALID_ARG;
  if (!x || !codes || !scales) return MOE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(x) % 16) != 0 || (reinterpret_cast<uintptr_t>(codes) % 8) != 0)
    return MOE_ERR_INVALID_ARG;
  if (rows == 0) return MOE_OK;
  begin_launches();
  hipLaunchKernelGGL(fp8_quantize_rows_kernel, dim3((unsigned)rows), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const uint4 *>(x), cols, static_cast<uint8_t *>(codes), scales);
  return launch_status();
}

extern "C" int moe_fp8_fused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                     const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                     const void *packed_down, const float *h_scale, void *y, void *workspace,
                                     size_t workspace_bytes, void *stream, void *const *events) {
  if (!h_scale) return MOE_ERR_INVALID_ARG;
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true, events, 0, h_scale);
}

extern "C" int moe_fused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx, const float *topk_w,
                                 const moe_dispatch *tables, const void *packed_gate_up, const void *packed_down,
                                 void *y, void *workspace, size_t workspace_bytes, void *stream) {
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true);
}

extern "C" int moe_fused_forward_bounded(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                         const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                         const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                         void *stream, int max_polls, int wait_extra) {
  if (max_polls < 1 || wait_extra < 0) return MOE_ERR_INVALID_ARG;
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true, nullptr, 1, nullptr, nullptr, max_polls, wait_extra);
}

extern "C" int moe_forward_status(const void *workspace, int32_t *flag, void *stream) {
  if (!workspace || !flag) return MOE_ERR_INVALID_ARG;
  // header word 24 of the forward workspace (see FwdLayout): raised by a wait of the resident kernel that gave up
  const int32_t *word = static_cast<const int32_t *>(workspace) + 24;
  hipStream_t st = (hipStream_t)stream;
  if (hipMemcpyAsync(flag, word, sizeof(int32_t), hipMemcpyDeviceToHost, st) != hipSuccess ||
      hipStreamSynchronize(st) != hipSuccess) {
    (void)hipGetLastError();
    return MOE_ERR_HIP;
  }
  return MOE_OK;
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

extern "C" int moe_fused_forward_resident(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                          const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                          const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                          void *stream, void *const *events, int max_polls, int wait_extra) {
  if (max_polls < 0 || wait_extra < 0) return MOE_ERR_INVALID_ARG;
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true, events, 3, nullptr, nullptr, max_polls ? max_polls : kMaxPolls,
                        wait_extra);
}

extern "C" int moe_unfused_forward(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                   const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                   const void *packed_down, void *y, void *workspace, size_t workspace_bytes,
                                   void *stream) {
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, false);
}

// ------------------------------------------------------------------------------------------------
// Training path: forward that keeps what the backward pass needs, and the backward pass.
// ------------------------------------------------------------------------------------------------
namespace moe355 {

// Backward workspace: the tile table (lists for the two backward GEMMs), the per-row metadata and the intermediates.
struct BwdLayout {
  FwdLayout t;   // header .. tile_ready as in the forward layout (h and o unused)
  size_t dgu;    // bf16 [P_cap, 2 f]  dg, then du
  size_t hw;     // bf16 [P_cap, f]    w silu(g) u
  size_t dxr;    // float[P_cap, d]    rows of dx before the per-token sum
  // weight gradients: operands transposed to [64-row block][column][64 rows], every expert's rows padded to blocks
  size_t kb;     // int32[E_loc + 1]   first block of every local expert in the padded row order
  size_t xT, dyT;  // bf16 [blocks][d][64]   gathered x rows, gathered dy rows
  size_t hwT;    // bf16 [blocks][f][64]
  size_t dguT;   // bf16 [blocks][2 f][64]
  size_t kpad;   // padded row capacity: 64 (ceil(P_cap / 64) + E_loc)
  size_t total;
};

static Derived backward_derived(const moe_shape *s, const Derived &dv) {
  Derived b = dv;
  b.nt1 = ceil_div(s->f, kBN);  // first backward GEMM: dh over f in plain 256-column tiles
  return b;
}

static BwdLayout backward_layout(const moe_shape *s, const Derived &dvb) {
  BwdLayout L;
  size_t off = 0;
  auto take = [&off](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  const size_t rows = (size_t)(dvb.P_cap > 0 ? dvb.P_cap : 1);
  L.t.header = take(32 * sizeof(int32_t));
  L.t.work1 = take((size_t)dvb.max_mtiles * dvb.nt1 * 4 * sizeof(int32_t));
  L.t.work2 = take((size_t)dvb.max_mtiles * dvb.nt2 * 4 * sizeof(int32_t));
  L.t.row_tok = take(rows * sizeof(int32_t));
  L.t.row_w = take(rows * sizeof(float));
  L.t.row_sole = take(rows * sizeof(int32_t));
  L.t.tile_ready = take((size_t)dvb.max_mtiles * sizeof(int32_t));
  L.t.row_tile = L.t.tile_done = 0;  // forward only
  L.t.h = L.t.o = 0;
  L.dgu = take(rows * 2 * (size_t)s->f * 2);
  L.hw = take(rows * (size_t)s->f * 2);
  L.dxr = take(rows * (size_t)s->d * sizeof(float));
  L.kpad = 64 * ((rows + 63) / 64 + (size_t)dvb.E_loc);
  L.kb = take((size_t)(dvb.E_loc + 1) * sizeof(int32_t));
  L.xT = take((size_t)s->d * L.kpad * 2);
  L.dyT = take((size_t)s->d * L.kpad * 2);
  L.hwT = take((size_t)s->f * L.kpad * 2);
  L.dguT = take(2 * (size_t)s->f * L.kpad * 2);
  L.t.total = L.total = off;
  return L;
}

static bool backward_supported(const moe_shape *s) { return s->dtype == MOE_BF16 && s->f % kBK == 0; }

}  // namespace moe355

extern "C" size_t moe_train_kept_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  const size_t rows = (size_t)(dv.P_cap > 0 ? dv.P_cap : 1);
  return align_up(rows * 2 * shape->f * 2, 256) + align_up(rows * (size_t)shape->d * sizeof(float), 256);
}

extern "C" size_t moe_backward_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  return backward_layout(shape, backward_derived(shape, dv)).total;
}

extern "C" size_t moe_backward_packed_weight_bytes(const moe_shape *shape, int which) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK || (which != 0 && which != 1)) return 0;
  if (which == 0) return (size_t)dv.E_loc * ceil_div(shape->f, kBN) * ceil_div(shape->d, kBK) * kTileBytes;  // Wd^T
  return (size_t)dv.E_loc * ceil_div(shape->d, kBN) * (2 * ceil_div(shape->f, kBK)) * kTileBytes;  // [Wg^T; Wu^T]
}

extern "C" int moe_pack_weights_backward(const moe_shape *shape, const void *W_gate, const void *W_up,
                                         const void *W_down, void *packed_down_t, void *packed_gate_up_t,
                                         void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!W_gate || !W_up || !W_down || !packed_down_t || !packed_gate_up_t) return MOE_ERR_INVALID_ARG;
  if (!backward_supported(shape)) return MOE_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(W_gate) | reinterpret_cast<uintptr_t>(W_up) | reinterpret_cast<uintptr_t>(W_down) |
       reinterpret_cast<uintptr_t>(packed_down_t) | reinterpret_cast<uintptr_t>(packed_gate_up_t)) % 16 != 0)
    return MOE_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  begin_launches();
  const int d = shape->d, f = shape->f;
  const int ntf = ceil_div(f, kBN), ktd = ceil_div(d, kBK), ntd = ceil_div(d, kBN), ktf = f / kBK;
  if (ntf > 65535 || ntd > 65535 || dv.E_loc > 65535) return MOE_ERR_UNSUPPORTED;
  // B[k = model index][n = hidden index] = W_down[n][k]
  hipLaunchKernelGGL(pack_bf16_transposed_kernel, dim3(ktd, ntf, dv.E_loc), dim3(256), 0, st,
                     static_cast<const bf16_t *>(W_down), static_cast<bf16_t *>(packed_down_t), d, f, ntf, ktd, 0);
  // B[k = hidden index, gate then up][n = model index] = W_gate[n][k], W_up[n][k]
  hipLaunchKernelGGL(pack_bf16_transposed_kernel, dim3(ktf, ntd, dv.E_loc), dim3(256), 0, st,
                     static_cast<const bf16_t *>(W_gate), static_cast<bf16_t *>(packed_gate_up_t), f, d, ntd, 2 * ktf, 0);
  hipLaunchKernelGGL(pack_bf16_transposed_kernel, dim3(ktf, ntd, dv.E_loc), dim3(256), 0, st,
                     static_cast<const bf16_t *>(W_up), static_cast<bf16_t *>(packed_gate_up_t), f, d, ntd, 2 * ktf, ktf);
  return launch_status();
}

extern "C" int moe_fused_forward_train(const moe_shape *shape, const void *x, const int32_t *topk_idx,
                                       const float *topk_w, const moe_dispatch *tables, const void *packed_gate_up,
                                       const void *packed_down, void *y, void *kept, size_t kept_bytes,
                                       void *workspace, size_t workspace_bytes, void *stream) {
  if (!shape) return MOE_ERR_INVALID_ARG;
  if (shape->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (!kept || kept_bytes < moe_train_kept_bytes(shape)) return MOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(kept) % 256 != 0) return MOE_ERR_INVALID_ARG;
  return forward_common(shape, x, topk_idx, topk_w, tables, packed_gate_up, packed_down, y, workspace,
                        workspace_bytes, stream, true, nullptr, 0, nullptr, kept);
}

// The backward pass runs its memory-bound preparation for the weight gradients (zero gradients of experts without
// rows, transposed operands) beside its compute-bound GEMMs: those kernels need at most 16 registers and little or no
// LDS, so their waves fit on a CU next to a GEMM workgroup.  They go to a stream of the library's own (one per device,
// default priority, created on first use and kept), forked from and joined to the caller's stream by events.
struct SideStream {
  hipStream_t stream;
  hipEvent_t fork, mid, join;
  std::mutex enqueue;  // held by a call from its fork to its join: the events are re-recorded by every call
};
static SideStream *side_stream() {
  static SideStream made[64];  // (the mutex makes the struct non-trivial: default-constructed once)
  static std::atomic<int> state[64];  // 0 none, 1 being made, 2 ready
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
  if (state[dev].load(std::memory_order_acquire) == 2) return &made[dev];
  int expect = 0;
  if (state[dev].compare_exchange_strong(expect, 1)) {
    SideStream &m = made[dev];
    if (hipStreamCreateWithFlags(&m.stream, hipStreamNonBlocking) != hipSuccess ||
        hipEventCreateWithFlags(&m.fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m.mid, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&m.join, hipEventDisableTiming) != hipSuccess) {
      state[dev].store(0);
      return nullptr;
    }
    state[dev].store(2, std::memory_order_release);
    return &m;
  }
  while (state[dev].load(std::memory_order_acquire) == 1) {
  }
  return state[dev].load(std::memory_order_acquire) == 2 ? &made[dev] : nullptr;
}

extern "C" int moe_fused_backward(const moe_shape *shape, const void *x, const void *dy, const int32_t *topk_idx,
                                  const float *topk_w, const moe_dispatch *tables, const void *packed_down_t,
                                  const void *packed_gate_up_t, const void *kept, size_t kept_bytes, void *dx,
                                  float *d_topk_w, void *dW_gate, void *dW_up, void *dW_down, void *workspace,
                                  size_t workspace_bytes, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!x || !dy || !topk_idx || !topk_w || !packed_down_t || !packed_gate_up_t || !dx || !d_topk_w ||
      !tables_ok(tables))
    return MOE_ERR_INVALID_ARG;
  const bool wgrad = dW_gate || dW_up || dW_down;
  if (wgrad && !(dW_gate && dW_up && dW_down)) return MOE_ERR_INVALID_ARG;  // all three or none
  if (!backward_supported(shape)) return MOE_ERR_UNSUPPORTED;
  if (!kept || kept_bytes < moe_train_kept_bytes(shape)) return MOE_ERR_WORKSPACE;
  if (!workspace || workspace_bytes < moe_backward_workspace_bytes(shape)) return MOE_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(kept)) % 256 != 0)
    return MOE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(dy) | reinterpret_cast<uintptr_t>(dx) |
       reinterpret_cast<uintptr_t>(packed_down_t) | reinterpret_cast<uintptr_t>(packed_gate_up_t)) % 16 != 0)
    return MOE_ERR_INVALID_ARG;
  const Derived dvb = backward_derived(shape, dv);
  if ((int64_t)dvb.max_mtiles * std::max(dvb.nt1, dvb.nt2) > (int64_t)1 << 30) return MOE_ERR_UNSUPPORTED;
  if (std::max(dvb.nt1, dvb.nt2) >= 1 << kTileShift || dvb.max_mtiles >= 1 << (31 - kTileShift)) return MOE_ERR_UNSUPPORTED;
  if (std::max<int64_t>(shape->T, dv.P_cap) * std::max(shape->d, 2 * shape->f) >= (int64_t)1 << 32) return MOE_ERR_UNSUPPORTED;
  if (wgrad && (reinterpret_cast<uintptr_t>(dW_gate) | reinterpret_cast<uintptr_t>(dW_up) |
                reinterpret_cast<uintptr_t>(dW_down)) % 16 != 0)
    return MOE_ERR_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  begin_launches();
  const size_t n_pairs = (size_t)shape->T * shape->k;
  if (shape->T == 0) {
    if (wgrad) {  // no rows: every weight gradient is zero (bf16 zeros are zero words)
      const size_t words = (size_t)dv.E_loc * shape->d * shape->f / 2;
      for (void *p : {dW_gate, dW_up, dW_down})
        hipLaunchKernelGGL(fill_f32_kernel, dim3(1024), dim3(256), 0, st, static_cast<float *>(p), words, 0.0f);
    }
    return launch_status();
  }
  const BwdLayout L = backward_layout(shape, dvb);
  const Ws w = carve(workspace, L.t);
  unsigned char *b = static_cast<unsigned char *>(workspace);
  bf16_t *dgu = reinterpret_cast<bf16_t *>(b + L.dgu), *hw = reinterpret_cast<bf16_t *>(b + L.hw);
  float *dxr = reinterpret_cast<float *>(b + L.dxr);
  const size_t rows = (size_t)(dv.P_cap > 0 ? dv.P_cap : 1);
  const bf16_t *kept_gu = static_cast<const bf16_t *>(kept);
  const float *kept_o = reinterpret_cast<const float *>(static_cast<const unsigned char *>(kept) +
                                                        align_up(rows * 2 * shape->f * 2, 256));
  if ((rc = launch_prep(shape, dvb, tables, topk_idx, topk_w, w, w.row_sole, st)) != MOE_OK) return rc;
  // side stream: what the weight gradients need besides the products (nothing of it reads a GEMM's output before `mid`)
  SideStream *side = nullptr;
  std::unique_lock<std::mutex> side_lock;  // (released when the call returns)
  int32_t *kb = reinterpret_cast<int32_t *>(b + L.kb);
  bf16_t *xT = reinterpret_cast<bf16_t *>(b + L.xT), *dyT = reinterpret_cast<bf16_t *>(b + L.dyT);
  bf16_t *hwT = reinterpret_cast<bf16_t *>(b + L.hwT), *dguT = reinterpret_cast<bf16_t *>(b + L.dguT);
  const int kblocks = (int)(L.kpad / 64);
  const auto transpose = [&](const bf16_t *src, const int32_t *map, int ld, int C, bf16_t *dst) {
    hipLaunchKernelGGL(gather_transpose_kernel, dim3(ceil_div(C, 64), kblocks), dim3(256), 0, side->stream, src, map,
                       ld, 0, C, tables->offsets, w.header, kb, dv.e_lo, dv.E_loc, dst);
  };
  // from the fork on, every return first makes the caller's stream wait for the side stream
  const auto join = [&](int code) {
    if (!side) return code;
    if (hipEventRecord(side->join, side->stream) != hipSuccess || hipStreamWaitEvent(st, side->join, 0) != hipSuccess)
      return code != MOE_OK ? code : (int)MOE_ERR_HIP;
    return code;
  };
  if (wgrad) {
    if (kblocks > 65535) return MOE_ERR_UNSUPPORTED;
    if (!(side = side_stream())) return MOE_ERR_HIP;
    side_lock = std::unique_lock<std::mutex>(side->enqueue);
    if (hipEventRecord(side->fork, st) != hipSuccess || hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess) {
      side = nullptr;
      return MOE_ERR_HIP;
    }
    hipLaunchKernelGGL(wgrad_blocks_kernel, dim3(1), dim3(256), 0, side->stream, tables->offsets, w.header, dv.e_lo,
                       dv.E_loc, kb);
    transpose(static_cast<const bf16_t *>(x), w.row_tok, shape->d, shape->d, xT);
    transpose(static_cast<const bf16_t *>(dy), w.row_tok, shape->d, shape->d, dyT);
    if ((rc = launch_status()) != MOE_OK) return join(rc);
  }
  // gradient of the gate weights (zero for the slots whose expert is not local)
  hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)std::min<size_t>(1024, (n_pairs + 255) / 256)), dim3(256), 0, st,
                     d_topk_w, n_pairs, 0.0f);
  hipLaunchKernelGGL(gate_weight_grad_kernel, dim3((unsigned)std::min<size_t>(4096, (rows + 3) / 4)), dim3(256), 0, st,
                     kept_o, static_cast<const bf16_t *>(dy), w.header, w.row_tok, w.row_w, tables->perm, shape->d,
                     d_topk_w);
  if ((rc = launch_status()) != MOE_OK) return join(rc);
  static std::atomic<uint64_t> done_b1{0}, done_b2{0};
  if (!allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_kernel<false, false, true>), 2 * kStageBytes,
                         done_b1) ||
      !allow_dynamic_lds(reinterpret_cast<const void *>(&gemm_bf16_kernel<false>), 2 * kStageBytes, done_b2))
    return join(MOE_ERR_HIP);
  const auto grid_of = [&](int nt) { return dim3((unsigned)(((size_t)dvb.max_mtiles * nt + 255) / 256 * 256)); };
  // dh_raw = dy[token of the row] Wd^T, then the SwiGLU derivative with the kept g and u
  GemmArgs g1{};
  g1.A = dy; g1.row_map = w.row_tok; g1.Bp = packed_down_t; g1.out = dgu; g1.row_w = w.row_w;
  g1.aux = const_cast<bf16_t *>(kept_gu); g1.aux2 = hw;
  g1.n_items = w.header + 0; g1.work = w.work1;
  g1.K = shape->d; g1.N = shape->f; g1.lda = shape->d; g1.ldo = 2 * shape->f;
  g1.n_ntiles = dvb.nt1; g1.n_ktiles = ceil_div(shape->d, kBK);
  hipLaunchKernelGGL((gemm_bf16_kernel<false, false, true>), grid_of(dvb.nt1), dim3(kGemmThreads), 2 * kStageBytes, st,
                     g1);
  if ((rc = launch_status()) != MOE_OK) return join(rc);
  if (wgrad) {  // dg, du and w h are there: their transposes run beside the second GEMM
    if (hipEventRecord(side->mid, st) != hipSuccess || hipStreamWaitEvent(side->stream, side->mid, 0) != hipSuccess)
      return join(MOE_ERR_HIP);
    transpose(hw, nullptr, shape->f, shape->f, hwT);
    transpose(dgu, nullptr, 2 * shape->f, 2 * shape->f, dguT);
    if ((rc = launch_status()) != MOE_OK) return join(rc);
  }
  // rows of dx = [dg | du] [Wg^T ; Wu^T]; a row that is its token's only local slot goes straight to dx
  GemmArgs g2{};
  g2.A = dgu; g2.row_map = nullptr; g2.Bp = packed_gate_up_t; g2.out = dxr; g2.row_w = nullptr;
  g2.row_sole = w.row_sole; g2.y = dx;
  g2.n_items = w.header + 3; g2.work = w.work2;
  g2.K = 2 * shape->f; g2.N = shape->d; g2.lda = 2 * shape->f; g2.ldo = shape->d;
  g2.n_ntiles = dvb.nt2; g2.n_ktiles = 2 * (shape->f / kBK);
  hipLaunchKernelGGL(gemm_bf16_kernel<false>, grid_of(dvb.nt2), dim3(kGemmThreads), 2 * kStageBytes, st, g2);
  if ((rc = launch_status()) != MOE_OK) return join(rc);
  if ((rc = launch_combine(shape, dv, dxr, topk_idx, tables, dx, true, st)) != MOE_OK || !wgrad) return join(rc);
  // weight gradients: one grouped product per weight matrix, over the transposed operands
  static std::atomic<uint64_t> done_w{0};
  if (!allow_dynamic_lds(reinterpret_cast<const void *>(&wgrad_bf16_kernel), 2 * kStageBytes, done_w))
    return join(MOE_ERR_HIP);
  if ((rc = join(MOE_OK)) != MOE_OK) return rc;
  const size_t units = (size_t)shape->d * shape->f / 8;  // 16-byte units of one expert's gradient
  hipLaunchKernelGGL(wgrad_zero_empty_kernel,
                     dim3((unsigned)std::min<size_t>(1024, ceil_div(units, (size_t)8192)), dv.E_loc, 3), dim3(256), 0,
                     st, kb, static_cast<u32x4 *>(dW_gate), static_cast<u32x4 *>(dW_up), static_cast<u32x4 *>(dW_down),
                     units);
  const auto product = [&](const bf16_t *AT, int lda, const bf16_t *BT, int ldb, int b0, int M, int N, void *C) {
    WgradArgs a;
    a.AT = AT; a.BT = BT; a.C = static_cast<bf16_t *>(C); a.kb = kb;
    a.lda = lda; a.ldb = ldb; a.a0 = 0; a.b0 = b0;
    a.M = M; a.N = N; a.n_mt = ceil_div(M, kBM); a.n_nt = ceil_div(N, kBN);
    hipLaunchKernelGGL(wgrad_bf16_kernel, dim3(a.n_mt * a.n_nt, dv.E_loc), dim3(kGemmThreads), 2 * kStageBytes, st, a);
    a.n_mt = ceil_div(M, 128); a.n_nt = ceil_div(N, 128);  // experts with few or no rows: small tiles
    hipLaunchKernelGGL(wgrad_thin_bf16_kernel, dim3(ceil_div(a.n_mt * a.n_nt, kThinTiles), dv.E_loc), dim3(256), 0, st,
                       a);
  };
  product(xT, shape->d, dguT, 2 * shape->f, 0, shape->d, shape->f, dW_gate);         // x^T dg
  product(xT, shape->d, dguT, 2 * shape->f, shape->f, shape->d, shape->f, dW_up);    // x^T du
  product(hwT, shape->f, dyT, shape->d, 0, shape->f, shape->d, dW_down);             // (w h)^T dy
  return launch_status();
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
