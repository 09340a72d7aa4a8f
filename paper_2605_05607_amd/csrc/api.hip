// Host-side pieces of the C ABI that touch no device: shape validation, workspace geometry, status strings.
#include <algorithm>

#include "common.h"

namespace moe355 {

int check_shape(const moe_shape *s, Derived *out) {
  if (!s) return MOE_ERR_INVALID_ARG;
  if (s->T < 0 || s->d < 1 || s->f < 1 || s->E < 1 || s->R < 1 || s->k < 1) return MOE_ERR_INVALID_ARG;
  if (s->E % s->R != 0) return MOE_ERR_INVALID_ARG;
  if (s->k > s->E || s->k > kMaxTopK) return MOE_ERR_INVALID_ARG;
  if (s->local_rank_begin < 0 || s->local_rank_end <= s->local_rank_begin || s->local_rank_end > s->R)
    return MOE_ERR_INVALID_ARG;
  if (s->d % 8 != 0 || s->f % 8 != 0) return MOE_ERR_INVALID_ARG;
  if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (s->E > kMaxExperts) return MOE_ERR_UNSUPPORTED;
  if ((int64_t)s->T * s->k > (int64_t)1 << 30) return MOE_ERR_UNSUPPORTED;  // pair ids and rows are int32
  Derived d;
  d.epr = s->E / s->R;
  d.E_loc = (s->local_rank_end - s->local_rank_begin) * d.epr;
  d.e_lo = s->local_rank_begin * d.epr;
  d.pairs = (int64_t)s->T * s->k;
  d.P_cap = (int64_t)s->T * (s->k < d.E_loc ? s->k : d.E_loc);
  d.bm = s->dtype == MOE_BF16 ? kBM : kFBM;
  d.max_mtiles = (int)((d.P_cap + d.bm - 1) / d.bm) + d.E_loc;
  d.elt = s->dtype == MOE_BF16 ? 2 : 4;
  d.nt1 = s->dtype == MOE_BF16 ? ceil_div(s->f, kBN / 2) : ceil_div(s->f, kFBN);
  d.nt2 = s->dtype == MOE_BF16 ? ceil_div(s->d, kBN) : ceil_div(s->d, kFBN);
  if (out) *out = d;
  return MOE_OK;
}

FwdLayout forward_layout(const moe_shape *s, const Derived &dv) {
  FwdLayout L;
  size_t off = 0;
  auto take = [&off](size_t bytes) {
    const size_t at = off;
    off = align_up(off + bytes, 256);
    return at;
  };
  const size_t rows = (size_t)(dv.P_cap > 0 ? dv.P_cap : 1);
  L.header = take(32 * sizeof(int32_t));
  L.work1 = take((size_t)dv.max_mtiles * dv.nt1 * 4 * sizeof(int32_t));
  L.work2 = take((size_t)dv.max_mtiles * dv.nt2 * 4 * sizeof(int32_t));
  L.row_tok = take(rows * sizeof(int32_t));
  L.row_w = take(rows * sizeof(float));
  L.row_sole = take(rows * sizeof(int32_t));
  L.tile_ready = take((size_t)dv.max_mtiles * sizeof(int32_t));
  L.row_tile = take(rows * sizeof(int32_t));
  L.tile_done = take((size_t)dv.max_mtiles * sizeof(int32_t));
  L.h = take(rows * (size_t)s->f * dv.elt);
  L.o = take(rows * (size_t)s->d * sizeof(float));
  L.total = off;
  return L;
}

}  // namespace moe355

using namespace moe355;

extern "C" size_t moe_forward_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  return forward_layout(shape, dv).total;
}

extern "C" size_t moe_workspace_bytes(const moe_shape *shape) {
  // one buffer for both calls of a step: the dispatch scratch is dead once moe_build_dispatch's kernels have run
  return std::max(moe_dispatch_workspace_bytes(shape), moe_forward_workspace_bytes(shape));
}

extern "C" int moe_forward_gemm_launches(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  // one resident launch with the tile-level hand-over when the mean number of rows per expert, T k / E, is below
  // one M tile; a kernel boundary between the GEMMs otherwise (and always for fp32 layers)
  return shape->dtype == MOE_BF16 && (int64_t)shape->T * shape->k < (int64_t)shape->E * kBM ? 1 : 2;
}

extern "C" size_t moe_unfused_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  const size_t rows = (size_t)(dv.P_cap > 0 ? dv.P_cap : 1);
  // fused layout + gathered copy of x [P_cap, d] + fp32 scatter target [T, d]
  return forward_layout(shape, dv).total + align_up(rows * (size_t)shape->d * dv.elt, 256) +
         align_up((size_t)(shape->T > 0 ? shape->T : 1) * shape->d * sizeof(float), 256);
}

extern "C" size_t moe_packed_weight_bytes(const moe_shape *shape, int which) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  if (which != 0 && which != 1) return 0;
  if (shape->dtype == MOE_F32) {
    const size_t one = (size_t)dv.E_loc * shape->d * shape->f * sizeof(float);
    return align_up(which == 0 ? 2 * one : one, 256);
  }
  const size_t tile = (size_t)kBN * kBK * 2;
  if (which == 0) return (size_t)dv.E_loc * ceil_div(shape->f, kBN / 2) * ceil_div(shape->d, kBK) * tile;
  return (size_t)dv.E_loc * ceil_div(shape->d, kBN) * ceil_div(shape->f, kBK) * tile;
}

extern "C" const char *moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID_ARG: return "invalid argument";
    case MOE_ERR_UNSUPPORTED: return "unsupported dtype or extent";
    case MOE_ERR_WORKSPACE: return "workspace missing or too small";
    case MOE_ERR_HIP: return "kernel launch failed";
    default: return "unknown status";
  }
}
