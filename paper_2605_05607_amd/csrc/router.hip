// moe_router_logits: the gate network ahead of the routing (Sec. II-A: the experts of a token are "selected by
// the gate network"; reading: a bias-free linear map, one row of W_r per expert).  logits[T,E] = x[T,d] * W_r[E,d]^T
// in fp32, summed in a fixed order, so that the routing built on it is reproducible.
#include <algorithm>

#include "route_pick.h"

namespace moe355 {

typedef __bf16 rbf16_t;
typedef rbf16_t rbf16x8 __attribute__((ext_vector_type(8)));
typedef float rf32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t ru32x4 __attribute__((ext_vector_type(4)));

constexpr int kRouterBN = 256;      // experts per workgroup
constexpr int kRouterBK = 64;       // reduction indices per k-step
constexpr int kRouterThreads = 512; // 8 waves = 2 (token blocks) x 4 (expert blocks of 64)
constexpr int kRouterMaxSplit = 8;
// LDS bytes of one stage for a tile of BM tokens: A slab then B slab
constexpr int router_stage_bytes(int BM) { return (BM + kRouterBN) * kRouterBK * 2; }

// One workgroup owns BM (64 or 128) tokens x 256 experts x one contiguous part of the reduction range (blockIdx.z): the
// product is skinny (a few hundred experts), so its cost is reading x once, and cutting the reduction range is
// what gives the chip enough workgroups.  Both operands have the reduction index contiguous in memory; a k-step
// moves BM x 64 of x and 256 x 64 of W_r through the LDS (16 bytes per lane, coalesced along the rows, chunks
// XOR-swizzled by (row >> 1) & 7 as in the expert GEMMs), double buffered, with the next four slabs in flight in
// registers.  A part's block is written as fp32 to partial[part][T][E]; router_reduce_kernel adds the parts in
// the order 0, 1, 2, ... so that the logits, and the routing built on them, are reproducible.  Every workgroup
// streams its whole W_r part from the L2, so the 128-token tile halves the bytes that cross the L2 -> CU path (the
// cost of this skinny product next to reading x once); the 64-token tile is for layers with too few tokens to
// give every CU a workgroup otherwise.
template <int BM>
__global__ __launch_bounds__(kRouterThreads) void router_logits_bf16_kernel(const rbf16_t *__restrict__ x,
                                                                            const rbf16_t *__restrict__ W,
                                                                            float *__restrict__ partial, int T, int d,
                                                                            int E, int steps_per_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int l31 = lane & 31, khalf = lane >> 5, sw = (lane >> 1) & 7;
  constexpr int kStage = router_stage_bytes(BM);
  constexpr int MB = BM / 64;  // 32-row token blocks per wave, and x rows staged per thread
  const int t0 = blockIdx.y * BM, e0 = blockIdx.x * kRouterBN;
  const int KT = (d + kRouterBK - 1) / kRouterBK;
  const int kt_begin = min(KT, (int)blockIdx.z * steps_per_part), kt_end = min(KT, kt_begin + steps_per_part);

  // staging: thread t moves 16-byte chunk t & 7 of x row t >> 3 and of W_r rows (t >> 3) + 64 i
  const int chunk = tid & 7, row = tid >> 3;
  const rbf16_t *xa0 = x + (size_t)min(t0 + row, T - 1) * d + chunk * 8;  // rows past the end: the last row, unused
  const rbf16_t *xa1 = x + (size_t)min(t0 + row + 64, T - 1) * d + chunk * 8;
  const rbf16_t *wb0 = W + (size_t)min(e0 + row, E - 1) * d + chunk * 8;
  const rbf16_t *wb1 = W + (size_t)min(e0 + row + 64, E - 1) * d + chunk * 8;
  const rbf16_t *wb2 = W + (size_t)min(e0 + row + 128, E - 1) * d + chunk * 8;
  const rbf16_t *wb3 = W + (size_t)min(e0 + row + 192, E - 1) * d + chunk * 8;
  const int dst = (row * 8 + (chunk ^ ((row >> 1) & 7))) * 16;  // + 8192 per 64 rows
  // Register ring of kRing slabs: the slab of k-step kt is requested four steps before it moves to the LDS, so that
  // the latency of the loads (x comes from HBM) is covered by four steps of work instead of one.  Every load is
  // unconditional (past the end it repeats the last k-step) and a slab past the end of this part, or a chunk past d,
  // is replaced by zeros in x when it is stored: the loop then has no data-dependent branch and a fixed number of
  // loads between a load and its use.
  constexpr int kRing = 4;
  ru32x4 ra0[kRing], ra1[kRing], rb0[kRing], rb1[kRing], rb2[kRing], rb3[kRing];
  const ru32x4 zero4 = {0u, 0u, 0u, 0u};
#define MOE355_ROUTER_LOAD(S_, KT_)                                                 \
  do {                                                                              \
    const int kc_ = min((KT_), KT - 1);                                             \
    const int off_ = kc_ * kRouterBK + chunk * 8 < d ? kc_ * kRouterBK : -chunk * 8; /* past d: chunk 0, valid */ \
    ra0[S_] = *reinterpret_cast<const ru32x4 *>(xa0 + off_);                        \
    if (MB > 1) ra1[S_] = *reinterpret_cast<const ru32x4 *>(xa1 + off_);            \
    rb0[S_] = *reinterpret_cast<const ru32x4 *>(wb0 + off_);                        \
    rb1[S_] = *reinterpret_cast<const ru32x4 *>(wb1 + off_);                        \
    rb2[S_] = *reinterpret_cast<const ru32x4 *>(wb2 + off_);                        \
    rb3[S_] = *reinterpret_cast<const ru32x4 *>(wb3 + off_);                        \
  } while (0)
#define MOE355_ROUTER_STORE(S_, STAGE, KT_)                                         \
  do {                                                                              \
    const bool live_ = (KT_) < kt_end && (KT_) * kRouterBK + chunk * 8 < d;         \
    unsigned char *s_ = smem + (STAGE) * kStage;                                    \
    *reinterpret_cast<ru32x4 *>(s_ + dst) = live_ ? ra0[S_] : zero4;                \
    if (MB > 1) *reinterpret_cast<ru32x4 *>(s_ + 8192 + dst) = live_ ? ra1[S_] : zero4; \
    *reinterpret_cast<ru32x4 *>(s_ + BM * 128 + dst) = rb0[S_];                     \
    *reinterpret_cast<ru32x4 *>(s_ + BM * 128 + 8192 + dst) = rb1[S_];              \
    *reinterpret_cast<ru32x4 *>(s_ + BM * 128 + 16384 + dst) = rb2[S_];             \
    *reinterpret_cast<ru32x4 *>(s_ + BM * 128 + 24576 + dst) = rb3[S_];             \
  } while (0)

  rf32x16 acc[MB][2];
#pragma unroll
  for (int mi = 0; mi < MB; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][j][r] = 0.f;

  // Step I_ of a round of four (k-step KT_): multiply the slab in stage I_ & 1, move the next slab from its ring slot
  // to the other stage (last read before the previous barrier) and request that slot again five k-steps ahead.
#define MOE355_ROUTER_STEP(I_, KT_)                                                                     \
  do {                                                                                                  \
    const unsigned char *sA = smem + ((I_) & 1) * kStage + (wm * (BM / 2) + l31) * 128;                 \
    const unsigned char *sB = smem + ((I_) & 1) * kStage + BM * 128 + (wn * 64 + l31) * 128;            \
    _Pragma("unroll") for (int kk = 0; kk < 4; ++kk) {                                                  \
      const int slot = ((kk * 2 + khalf) ^ sw) * 16;                                                    \
      const rbf16x8 fb0 = *reinterpret_cast<const rbf16x8 *>(sB + slot);                                \
      const rbf16x8 fb1 = *reinterpret_cast<const rbf16x8 *>(sB + 4096 + slot);                         \
      _Pragma("unroll") for (int mi = 0; mi < MB; ++mi) {                                               \
        const rbf16x8 fa = *reinterpret_cast<const rbf16x8 *>(sA + mi * 4096 + slot);                   \
        acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb0, acc[mi][0], 0, 0, 0);             \
        acc[mi][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb1, acc[mi][1], 0, 0, 0);             \
      }                                                                                                 \
    }                                                                                                   \
    MOE355_ROUTER_STORE(((I_) + 1) % kRing, ((I_) + 1) & 1, (KT_) + 1);                                 \
    MOE355_ROUTER_LOAD(((I_) + 1) % kRing, (KT_) + 1 + kRing);                                          \
    __syncthreads();                                                                                    \
  } while (0)
  if (kt_begin < kt_end) {
    MOE355_ROUTER_LOAD(0, kt_begin);
    MOE355_ROUTER_LOAD(1, kt_begin + 1);
    MOE355_ROUTER_LOAD(2, kt_begin + 2);
    MOE355_ROUTER_LOAD(3, kt_begin + 3);
    MOE355_ROUTER_STORE(0, 0, kt_begin);
    MOE355_ROUTER_LOAD(0, kt_begin + kRing);
    __syncthreads();
    // whole rounds: a k-step past the end multiplies zeros
    for (int kt = kt_begin; kt < kt_end; kt += kRing) {
      MOE355_ROUTER_STEP(0, kt);
      MOE355_ROUTER_STEP(1, kt + 1);
      MOE355_ROUTER_STEP(2, kt + 2);
      MOE355_ROUTER_STEP(3, kt + 3);
    }
  }
#undef MOE355_ROUTER_STEP
#undef MOE355_ROUTER_LOAD
#undef MOE355_ROUTER_STORE
  // accumulator register r of lane l is C[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32] of its 32 x 32 block
  float *out = partial + (size_t)blockIdx.z * T * E;
#pragma unroll
  for (int mi = 0; mi < MB; ++mi)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int t = t0 + wm * (BM / 2) + mi * 32 + 8 * (r >> 2) + 4 * khalf + (r & 3), e = e0 + wn * 64 + j * 32 + l31;
        if (t < T && e < E) out[(size_t)t * E + e] = acc[mi][j][r];
      }
}

// The routing straight from the partial sums: one wave per token adds the parts of its row in the order 0, 1, 2, ...
// (the logits of router_reduce_kernel, bit for bit), keeps them in registers, lane l owning experts
// [l * PER, l * PER + PER), and picks (route_pick_registers).  The logits themselves are stored only on request.
template <int PER>
__global__ __launch_bounds__(256) void router_reduce_topk_kernel(const float *__restrict__ partial, size_t n,
                                                                 int parts, float *__restrict__ logits,
                                                                 int32_t *__restrict__ topk_idx,
                                                                 float *__restrict__ topk_w, int T, int E, int k) {
  const int lane = lane_id();
  const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= T) return;  // whole wave leaves together
  const float *row = partial + (size_t)t * E;
  uint32_t key[PER];
  float val[PER];
  if (PER % 4 == 0 && (E & 3) == 0) {
#pragma unroll
    for (int q = 0; q < PER / 4; ++q) {
      const int e0 = lane * PER + q * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e0 < E) {  // E % 4 == 0: the four are inside together
        v = *reinterpret_cast<const float4 *>(row + e0);
        for (int p = 1; p < parts; ++p) {
          const float4 a = *reinterpret_cast<const float4 *>(row + (size_t)p * n + e0);
          v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
        }
        if (logits) *reinterpret_cast<float4 *>(logits + (size_t)t * E + e0) = v;
      }
      const float vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        val[q * 4 + u] = vv[u];
        key[q * 4 + u] = e0 < E ? ordered_key(vv[u]) : 0u;
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int e = lane * PER + i;
      float v = 0.f;
      if (e < E) {
        v = row[e];
        for (int p = 1; p < parts; ++p) v += row[(size_t)p * n + e];
        if (logits) logits[(size_t)t * E + e] = v;
      }
      val[i] = v;
      key[i] = e < E ? ordered_key(v) : 0u;
    }
  }
  route_pick_registers<PER>(val, key, E, k, t, topk_idx, topk_w);
}

// logits = partial[0] + partial[1] + ... in that order.
// (`logits` may be part 0 itself: every element is read before it is written, by the thread that writes it.)
__global__ __launch_bounds__(256) void router_reduce_kernel(const float *partial, float *logits, size_t n, int parts) {
  for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    float v = partial[i];
    for (int q = 1; q < parts; ++q) v += partial[(size_t)q * n + i];
    logits[i] = v;
  }
}

// fp32 layers: one thread per logit, fp32 fused multiply-adds in ascending reduction order (reference-grade path).
__global__ __launch_bounds__(256) void router_logits_f32_kernel(const float *__restrict__ x,
                                                                const float *__restrict__ W,
                                                                float *__restrict__ logits, int T, int d, int E) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i >= (size_t)T * E) return;
  const int t = (int)(i / E), e = (int)(i % E);
  const float *xr = x + (size_t)t * d, *wr = W + (size_t)e * d;
  float sum = 0.f;
  for (int c = 0; c < d; ++c) sum = fmaf(xr[c], wr[c], sum);
  logits[i] = sum;
}

}  // namespace moe355

using namespace moe355;

// Token tile of the bf16 kernel: 128 where that still gives every CU a workgroup, else 64.
static int router_tile(const moe_shape *s) {
  const int kt = ceil_div(s->d, kRouterBK);
  const int wgs128 = ceil_div(s->E, kRouterBN) * ceil_div(s->T > 0 ? s->T : 1, 128) * std::min(kRouterMaxSplit, kt);
  return wgs128 >= 512 ? 128 : 64;
}

// Parts the reduction range is cut into: enough to give every CU a workgroup, at most kRouterMaxSplit, and never
// more than there are k-steps.
static int router_split(const moe_shape *s) {
  const int tiles = ceil_div(s->E, kRouterBN) * ceil_div(s->T > 0 ? s->T : 1, router_tile(s));
  const int kt = ceil_div(s->d, kRouterBK);
  return std::max(1, std::min(std::min(kRouterMaxSplit, kt), ceil_div(256, tiles)));
}

extern "C" size_t moe_router_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  if (shape->dtype != MOE_BF16) return 256;
  const int parts = router_split(shape);
  return align_up((parts > 1 ? (size_t)parts : 0) * (size_t)(shape->T > 0 ? shape->T : 1) * shape->E * sizeof(float) + 1,
                  256);
}

extern "C" size_t moe_route_from_x_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  // the partial sums of every part (one part at least: the logits need not be stored anywhere else)
  const int parts = shape->dtype == MOE_BF16 ? router_split(shape) : 1;
  return align_up((size_t)parts * (size_t)(shape->T > 0 ? shape->T : 1) * shape->E * sizeof(float), 256);
}

// The product into `partial` (parts > 1) or straight into `direct` (one part).
static int launch_router_gemm(const moe_shape *shape, const void *x, const void *W_r, float *partial, float *direct,
                              int *parts_out, hipStream_t st) {
  const int parts = router_split(shape);
  *parts_out = parts;
  const int bm = router_tile(shape);
  const int steps_per_part = ceil_div(ceil_div(shape->d, kRouterBK), parts);
  const dim3 grid(ceil_div(shape->E, kRouterBN), ceil_div(shape->T, bm), parts);
  if (grid.y > 65535) return MOE_ERR_UNSUPPORTED;
  float *out = parts > 1 ? partial : direct;
  static std::atomic<uint64_t> done64{0}, done128{0};
  if (bm == 128) {
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&router_logits_bf16_kernel<128>), 2 * router_stage_bytes(128),
                           done128))
      return MOE_ERR_HIP;
    hipLaunchKernelGGL(router_logits_bf16_kernel<128>, grid, dim3(kRouterThreads), 2 * router_stage_bytes(128), st,
                       static_cast<const rbf16_t *>(x), static_cast<const rbf16_t *>(W_r), out, shape->T, shape->d,
                       shape->E, steps_per_part);
  } else {
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&router_logits_bf16_kernel<64>), 2 * router_stage_bytes(64),
                           done64))
      return MOE_ERR_HIP;
    hipLaunchKernelGGL(router_logits_bf16_kernel<64>, grid, dim3(kRouterThreads), 2 * router_stage_bytes(64), st,
                       static_cast<const rbf16_t *>(x), static_cast<const rbf16_t *>(W_r), out, shape->T, shape->d,
                       shape->E, steps_per_part);
  }
  return launch_status();
}

extern "C" int moe_router_logits(const moe_shape *shape, const void *x, const void *W_r, float *logits,
                                 void *workspace, size_t workspace_bytes, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!x || !W_r || !logits) return MOE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(W_r)) % 16 != 0) return MOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < moe_router_workspace_bytes(shape)) return MOE_ERR_WORKSPACE;
  if (shape->T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  begin_launches();
  if (shape->dtype == MOE_BF16) {
    int parts = 1;
    if ((rc = launch_router_gemm(shape, x, W_r, static_cast<float *>(workspace), logits, &parts, st)) != MOE_OK)
      return rc;
    if (parts > 1) {
      const size_t n = (size_t)shape->T * shape->E;
      hipLaunchKernelGGL(router_reduce_kernel, dim3((unsigned)std::min<size_t>(2048, (n + 255) / 256)), dim3(256), 0,
                         st, static_cast<const float *>(workspace), logits, n, parts);
    }
  } else {
    const size_t n = (size_t)shape->T * shape->E;
    hipLaunchKernelGGL(router_logits_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float *>(x), static_cast<const float *>(W_r), logits, shape->T, shape->d,
                       shape->E);
  }
  return launch_status();
}

// Gate network and routing in one call: the logits are summed from the partial products inside the kernel that picks,
// and reach memory only if the caller asks for them.
extern "C" int moe_route_from_x(const moe_shape *shape, const void *x, const void *W_r, float *logits,
                                int32_t *topk_idx, float *topk_w, void *workspace, size_t workspace_bytes,
                                void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!x || !W_r || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(W_r)) % 16 != 0) return MOE_ERR_INVALID_ARG;
  if (!workspace || workspace_bytes < moe_route_from_x_workspace_bytes(shape)) return MOE_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return MOE_ERR_INVALID_ARG;
  if (shape->T == 0) return MOE_OK;
  hipStream_t st = (hipStream_t)stream;
  begin_launches();
  float *partial = static_cast<float *>(workspace);
  const size_t n = (size_t)shape->T * shape->E;
  int parts = 1;
  if (shape->dtype == MOE_BF16) {
    if ((rc = launch_router_gemm(shape, x, W_r, partial, partial, &parts, st)) != MOE_OK) return rc;
  } else {
    hipLaunchKernelGGL(router_logits_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float *>(x), static_cast<const float *>(W_r), partial, shape->T, shape->d,
                       shape->E);
    if ((rc = launch_status()) != MOE_OK) return rc;
  }
  if (shape->E <= 512) {
    const dim3 grid(ceil_div(shape->T, 4)), block(256);
#define MOE355_ROUTE_X(PER_)                                                                                          \
  hipLaunchKernelGGL(router_reduce_topk_kernel<PER_>, grid, block, 0, st, partial, n, parts, logits, topk_idx, topk_w, \
                     shape->T, shape->E, shape->k)
    if (shape->E <= 64) MOE355_ROUTE_X(1);
    else if (shape->E <= 128) MOE355_ROUTE_X(2);
    else if (shape->E <= 256) MOE355_ROUTE_X(4);
    else MOE355_ROUTE_X(8);
#undef MOE355_ROUTE_X
    return launch_status();
  }
  // more experts than a wave keeps in registers: add the parts in place (part 0 becomes the logits), then the routing
  // kernel that keeps its keys in the LDS
  if (parts > 1) {
    hipLaunchKernelGGL(router_reduce_kernel, dim3((unsigned)std::min<size_t>(2048, (n + 255) / 256)), dim3(256), 0, st,
                       partial, partial, n, parts);
    if ((rc = launch_status()) != MOE_OK) return rc;
  }
  if (logits) {
    if (hipMemcpyAsync(logits, partial, n * sizeof(float), hipMemcpyDeviceToDevice, st) != hipSuccess) {
      (void)hipGetLastError();
      return MOE_ERR_HIP;
    }
  }
  return moe_route_topk(shape, partial, topk_idx, topk_w, stream);
}
