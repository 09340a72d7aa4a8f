// moe_route_topk: softmax top-k routing with renormalised weights (gate of Sec. II-A; the routing is
// produced before Dispatch, Sec. III-E).  One 64-lane wave owns one token row.
#include "common.h"

namespace moe355 {

// Order-preserving map from finite fp32 to uint32 (larger float <=> larger key); -0 and +0 map to the same
// key so that they tie, as they do under a float comparison.  Key 0 is never produced by a finite value and
// marks an expert that has already been picked.
__device__ __forceinline__ uint32_t ordered_key(float v) {
  const uint32_t b = __float_as_uint(v + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

constexpr int kRouteWaves = 4;  // waves (token rows) per block; fewer when E is large enough to crowd the LDS

__global__ __launch_bounds__(kRouteWaves * kWave) void route_topk_kernel(const float *__restrict__ logits,
                                                                         int32_t *__restrict__ topk_idx,
                                                                         float *__restrict__ topk_w, int T, int E,
                                                                         int k) {
  extern __shared__ uint32_t smem[];  // per wave: E keys, then 32 floats for the picked logits
  const int wave = threadIdx.x >> 6;
  const int lane = lane_id();
  const int t = blockIdx.x * (blockDim.x >> 6) + wave;
  if (t >= T) return;  // whole wave leaves together; no block-wide barrier is used below
  uint32_t *keys = smem + (size_t)wave * (E + kMaxTopK);
  float *picked = reinterpret_cast<float *>(keys + E);
  const float *row = logits + (size_t)t * E;
  for (int e = lane; e < E; e += kWave) keys[e] = ordered_key(row[e]);
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");

  for (int j = 0; j < k; ++j) {
    // best (key, lowest index) among this lane's strided experts
    uint32_t bk = 0;
    uint32_t bi = 0xFFFFFFFFu;
    for (int e = lane; e < E; e += kWave) {
      const uint32_t key = keys[e];
      if (key > bk) {
        bk = key;
        bi = (uint32_t)e;
      }
    }
    // wave-wide maximum of (key, -index): ties go to the lower index
    unsigned long long best = ((unsigned long long)bk << 32) | (unsigned long long)(0xFFFFFFFFu - bi);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const unsigned long long other = __shfl_xor(best, off, 64);
      best = other > best ? other : best;
    }
    const int e_best = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
    if (lane == 0) {
      // k <= E, so an unpicked expert always exists; the clamp only guards against non-finite input
      const int e_ok = e_best >= 0 && e_best < E ? e_best : 0;
      topk_idx[(size_t)t * k + j] = e_ok;
      picked[j] = row[e_ok];
      keys[e_ok] = 0u;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  if (lane < k) {
    const float m = picked[0];
    float sum = 0.f;
    for (int i = 0; i < k; ++i) sum += expf(picked[i] - m);  // slot order
    topk_w[(size_t)t * k + lane] = expf(picked[lane] - m) / sum;
  }
}

}  // namespace moe355

using namespace moe355;

extern "C" int moe_route_topk(const moe_shape *shape, const float *logits, int32_t *topk_idx, float *topk_w,
                              void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!logits || !topk_idx || !topk_w) return MOE_ERR_INVALID_ARG;
  if (shape->T == 0) return MOE_OK;
  begin_launches();
  const size_t per_wave = (size_t)(shape->E + kMaxTopK) * sizeof(uint32_t);
  int waves = kRouteWaves;
  while (waves > 1 && waves * per_wave > 48 * 1024) waves >>= 1;
  const int blocks = ceil_div(shape->T, waves);
  const size_t smem = waves * per_wave;
  hipLaunchKernelGGL(route_topk_kernel, dim3(blocks), dim3(waves * kWave), smem, (hipStream_t)stream, logits,
                     topk_idx, topk_w, shape->T, shape->E, shape->k);
  return launch_status();
}
