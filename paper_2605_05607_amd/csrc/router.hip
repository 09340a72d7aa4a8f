// moe_router_logits: the gate network ahead of the routing (Sec. II-A: the experts of a token are "selected by
// the gate network"; reading: a bias-free linear map, one row of W_r per expert).  logits[T,E] = x[T,d] * W_r[E,d]^T
// in fp32, summed in a fixed order, so that the routing built on it is reproducible.
#include <algorithm>

#include "common.h"

namespace moe355 {

typedef __bf16 rbf16_t;
typedef rbf16_t rbf16x8 __attribute__((ext_vector_type(8)));
typedef float rf32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t ru32x4 __attribute__((ext_vector_type(4)));

constexpr int kRouterBM = 64;       // tokens per workgroup
constexpr int kRouterBN = 256;      // experts per workgroup
constexpr int kRouterBK = 64;       // reduction indices per k-step
constexpr int kRouterThreads = 512; // 8 waves = 2 (token blocks of 32) x 4 (expert blocks of 64)
constexpr int kRouterStage = (kRouterBM + kRouterBN) * kRouterBK * 2;  // 40 KiB: A slab then B slab
constexpr int kRouterMaxSplit = 8;

// One workgroup owns 64 tokens x 256 experts x one contiguous part of the reduction range (blockIdx.z): the
// product is skinny (a few hundred experts), so its cost is reading x once, and cutting the reduction range is
// what gives the chip enough workgroups.  Both operands have the reduction index contiguous in memory; a k-step
// moves 64 x 64 of x and 256 x 64 of W_r through the LDS (16 bytes per lane, coalesced along the rows, chunks
// XOR-swizzled by (row >> 1) & 7 as in the expert GEMMs), double buffered with the next slab in flight in
// registers.  A part's block is written as fp32 to partial[part][T][E]; router_reduce_kernel adds the parts in
// the order 0, 1, 2, ... so that the logits, and the routing built on them, are reproducible.
__global__ __launch_bounds__(kRouterThreads) void router_logits_bf16_kernel(const rbf16_t *__restrict__ x,
                                                                            const rbf16_t *__restrict__ W,
                                                                            float *__restrict__ partial, int T, int d,
                                                                            int E, int steps_per_part) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];  // 2 stages
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;
  const int l31 = lane & 31, khalf = lane >> 5, sw = (lane >> 1) & 7;
  const int t0 = blockIdx.y * kRouterBM, e0 = blockIdx.x * kRouterBN;
  const int KT = (d + kRouterBK - 1) / kRouterBK;
  const int kt_begin = min(KT, (int)blockIdx.z * steps_per_part), kt_end = min(KT, kt_begin + steps_per_part);

  // staging: thread t moves 16-byte chunk t & 7 of x row t >> 3 and of W_r rows (t >> 3) + 64 i
  const int chunk = tid & 7, row = tid >> 3;
  const rbf16_t *xa = x + (size_t)min(t0 + row, T - 1) * d + chunk * 8;  // rows past the end: the last row, unused
  const rbf16_t *wb0 = W + (size_t)min(e0 + row, E - 1) * d + chunk * 8;
  const rbf16_t *wb1 = W + (size_t)min(e0 + row + 64, E - 1) * d + chunk * 8;
  const rbf16_t *wb2 = W + (size_t)min(e0 + row + 128, E - 1) * d + chunk * 8;
  const rbf16_t *wb3 = W + (size_t)min(e0 + row + 192, E - 1) * d + chunk * 8;
  const int dst = (row * 8 + (chunk ^ ((row >> 1) & 7))) * 16;  // + 8192 per 64 rows
  ru32x4 ra, rb0, rb1, rb2, rb3;
  // a chunk past d is read from the start of the row (valid) and replaced by zeros in x: it then adds nothing
#define MOE355_ROUTER_LOAD(KT_)                                                     \
  do {                                                                              \
    const bool in_ = (KT_) * kRouterBK + chunk * 8 < d;                             \
    const int off_ = in_ ? (KT_) * kRouterBK : -chunk * 8;                          \
    ra = *reinterpret_cast<const ru32x4 *>(xa + off_);                              \
    rb0 = *reinterpret_cast<const ru32x4 *>(wb0 + off_);                            \
    rb1 = *reinterpret_cast<const ru32x4 *>(wb1 + off_);                            \
    rb2 = *reinterpret_cast<const ru32x4 *>(wb2 + off_);                            \
    rb3 = *reinterpret_cast<const ru32x4 *>(wb3 + off_);                            \
    if (!in_) ra = ru32x4{0u, 0u, 0u, 0u};                                          \
  } while (0)
#define MOE355_ROUTER_STORE(STAGE)                                                  \
  do {                                                                              \
    unsigned char *s_ = smem + (STAGE) * kRouterStage;                              \
    *reinterpret_cast<ru32x4 *>(s_ + dst) = ra;                                     \
    *reinterpret_cast<ru32x4 *>(s_ + 8192 + dst) = rb0;                             \
    *reinterpret_cast<ru32x4 *>(s_ + 16384 + dst) = rb1;                            \
    *reinterpret_cast<ru32x4 *>(s_ + 24576 + dst) = rb2;                            \
    *reinterpret_cast<ru32x4 *>(s_ + 32768 + dst) = rb3;                            \
  } while (0)

  rf32x16 acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

  if (kt_begin < kt_end) {
    MOE355_ROUTER_LOAD(kt_begin);
    MOE355_ROUTER_STORE(0);
    __syncthreads();
    for (int kt = kt_begin; kt < kt_end; ++kt) {
      const int cur = (kt - kt_begin) & 1;
      if (kt + 1 < kt_end) MOE355_ROUTER_LOAD(kt + 1);  // uniform branch
      const unsigned char *sA = smem + cur * kRouterStage + (wm * 32 + l31) * 128;
      const unsigned char *sB = smem + cur * kRouterStage + 8192 + (wn * 64 + l31) * 128;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int slot = ((kk * 2 + khalf) ^ sw) * 16;
        const rbf16x8 fa = *reinterpret_cast<const rbf16x8 *>(sA + slot);
        const rbf16x8 fb0 = *reinterpret_cast<const rbf16x8 *>(sB + slot);
        const rbf16x8 fb1 = *reinterpret_cast<const rbf16x8 *>(sB + 4096 + slot);
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb0, acc[0], 0, 0, 0);
        acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb1, acc[1], 0, 0, 0);
      }
      if (kt + 1 < kt_end) MOE355_ROUTER_STORE(cur ^ 1);  // that stage was last read before the previous barrier
      __syncthreads();
    }
  }
#undef MOE355_ROUTER_LOAD
#undef MOE355_ROUTER_STORE
  // accumulator register r of lane l is C[8 * (r / 4) + 4 * (l / 32) + r % 4][l % 32] of its 32 x 32 block
  float *out = partial + (size_t)blockIdx.z * T * E;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int t = t0 + wm * 32 + 8 * (r >> 2) + 4 * khalf + (r & 3), e = e0 + wn * 64 + j * 32 + l31;
      if (t < T && e < E) out[(size_t)t * E + e] = acc[j][r];
    }
}

// logits = partial[0] + partial[1] + ... in that order.
__global__ __launch_bounds__(256) void router_reduce_kernel(const float *__restrict__ partial,
                                                            float *__restrict__ logits, size_t n, int parts) {
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

// Parts the reduction range is cut into: enough to give every CU a workgroup, at most kRouterMaxSplit, and never
// more than there are k-steps.
static int router_split(const moe_shape *s) {
  const int tiles = ceil_div(s->E, kRouterBN) * ceil_div(s->T > 0 ? s->T : 1, kRouterBM);
  const int kt = ceil_div(s->d, kRouterBK);
  return std::max(1, std::min(std::min(kRouterMaxSplit, kt), ceil_div(512, tiles)));
}

extern "C" size_t moe_router_workspace_bytes(const moe_shape *shape) {
  Derived dv;
  if (check_shape(shape, &dv) != MOE_OK) return 0;
  if (shape->dtype != MOE_BF16) return 256;
  const int parts = router_split(shape);
  return align_up((parts > 1 ? (size_t)parts : 0) * (size_t)(shape->T > 0 ? shape->T : 1) * shape->E * sizeof(float) + 1,
                  256);
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
    static std::atomic<uint64_t> done{0};
    if (!allow_dynamic_lds(reinterpret_cast<const void *>(&router_logits_bf16_kernel), 2 * kRouterStage, done))
      return MOE_ERR_HIP;
    const int parts = router_split(shape);
    const int steps_per_part = ceil_div(ceil_div(shape->d, kRouterBK), parts);
    const dim3 grid(ceil_div(shape->E, kRouterBN), ceil_div(shape->T, kRouterBM), parts);
    if (grid.y > 65535) return MOE_ERR_UNSUPPORTED;
    float *partial = parts > 1 ? static_cast<float *>(workspace) : logits;
    hipLaunchKernelGGL(router_logits_bf16_kernel, grid, dim3(kRouterThreads), 2 * kRouterStage, st,
                       static_cast<const rbf16_t *>(x), static_cast<const rbf16_t *>(W_r), partial, shape->T, shape->d,
                       shape->E, steps_per_part);
    if ((rc = launch_status()) != MOE_OK) return rc;
    if (parts > 1) {
      const size_t n = (size_t)shape->T * shape->E;
      hipLaunchKernelGGL(router_reduce_kernel, dim3((unsigned)std::min<size_t>(2048, (n + 255) / 256)), dim3(256), 0,
                         st, partial, logits, n, parts);
    }
  } else {
    const size_t n = (size_t)shape->T * shape->E;
    hipLaunchKernelGGL(router_logits_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                       static_cast<const float *>(x), static_cast<const float *>(W_r), logits, shape->T, shape->d,
                       shape->E);
  }
  return launch_status();
}
