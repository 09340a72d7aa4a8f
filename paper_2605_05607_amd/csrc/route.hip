// moe_route_topk: softmax top-k routing with renormalised weights (gate of Sec. II-A; the routing is
// produced before Dispatch, Sec. III-E).  One 64-lane wave owns one token row.  Up to 512 experts the row
// lives in registers (a contiguous run of experts per lane) and a pick costs a handful of cross-lane
// operations; beyond that the keys go through the LDS.
#include "route_pick.h"

namespace moe355 {

// Register variant for E <= 64 * PER: lane l owns experts [l * PER, l * PER + PER) (see route_pick_registers).
template <int PER>
__global__ __launch_bounds__(256) void route_topk_reg_kernel(const float *__restrict__ logits,
                                                             int32_t *__restrict__ topk_idx,
                                                             float *__restrict__ topk_w, int T, int E, int k) {
  const int wave = threadIdx.x >> 6;
  const int lane = lane_id();
  const int t = blockIdx.x * (blockDim.x >> 6) + wave;
  if (t >= T) return;  // whole wave leaves together
  const float *row = logits + (size_t)t * E;
  uint32_t key[PER];
  float val[PER];
  if (PER % 4 == 0 && (E & 3) == 0) {
#pragma unroll
    for (int q = 0; q < PER / 4; ++q) {
      const int e0 = lane * PER + q * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (e0 < E) v = *reinterpret_cast<const float4 *>(row + e0);  // E % 4 == 0: the four are inside together
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
      val[i] = e < E ? row[e] : 0.f;
      key[i] = e < E ? ordered_key(val[i]) : 0u;
    }
  }
  route_pick_registers<PER>(val, key, E, k, t, topk_idx, topk_w);
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

// Routing with a softmax (gate 0) or sigmoid (gate 1) gate and an optional per-expert bias that steers the
// selection only (the gate of DeepSeek-V3-style models; the paper leaves the gate open, Sec. II-A).  Selection
// value: logit + bias, or 1 / (1 + exp(-logit)) + bias, in fp32; k largest, lowest index on ties; weights from the
// logits alone: softmax over the picks, or the picked sigmoids divided by their sum.  Same structure as
// route_topk_kernel: one wave per token, keys in the LDS.
__global__ __launch_bounds__(kRouteWaves * kWave) void route_topk_gate_kernel(const float *__restrict__ logits,
                                                                              const float *__restrict__ bias,
                                                                              int gate,
                                                                              int32_t *__restrict__ topk_idx,
                                                                              float *__restrict__ topk_w, int T,
                                                                              int E, int k) {
  extern __shared__ uint32_t smem[];  // per wave: E keys, then 32 floats for the picked logits
  const int wave = threadIdx.x >> 6;
  const int lane = lane_id();
  const int t = blockIdx.x * (blockDim.x >> 6) + wave;
  if (t >= T) return;  // whole wave leaves together; no block-wide barrier is used below
  uint32_t *keys = smem + (size_t)wave * (E + kMaxTopK);
  float *picked = reinterpret_cast<float *>(keys + E);
  const float *row = logits + (size_t)t * E;
  for (int e = lane; e < E; e += kWave) {
    const float l = row[e];
    const float base = gate == 0 ? l : 1.0f / (1.0f + expf(-l));
    keys[e] = ordered_key(base + (bias ? bias[e] : 0.0f));
  }
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  for (int j = 0; j < k; ++j) {
    uint32_t bk = 0;
    uint32_t bi = 0xFFFFFFFFu;
    for (int e = lane; e < E; e += kWave) {
      const uint32_t key = keys[e];
      if (key > bk) {
        bk = key;
        bi = (uint32_t)e;
      }
    }
    unsigned long long best = ((unsigned long long)bk << 32) | (unsigned long long)(0xFFFFFFFFu - bi);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
      const unsigned long long other = __shfl_xor(best, off, 64);
      best = other > best ? other : best;
    }
    const int e_best = (int)(0xFFFFFFFFu - (uint32_t)(best & 0xFFFFFFFFull));
    if (lane == 0) {
      const int e_ok = e_best >= 0 && e_best < E ? e_best : 0;  // guards against non-finite input only
      topk_idx[(size_t)t * k + j] = e_ok;
      picked[j] = row[e_ok];
      keys[e_ok] = 0u;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
  if (lane < k) {
    float m = picked[0];
    for (int i = 1; i < k; ++i) m = fmaxf(m, picked[i]);
    float sum = 0.f;
    for (int i = 0; i < k; ++i) sum += gate == 0 ? expf(picked[i] - m) : 1.0f / (1.0f + expf(-picked[i]));
    const float mine = gate == 0 ? expf(picked[lane] - m) : 1.0f / (1.0f + expf(-picked[lane]));
    topk_w[(size_t)t * k + lane] = mine / sum;
  }
}

// Backward of moe_route_topk's weights: they are a softmax over the k picked logits, so for token t
//   dlogits[t][e_j] = w_j (dw_j - sum_i w_i dw_i),  0 for the experts that were not picked.
// One wave per token; the row of dlogits is zeroed by the wave, then the k lanes that hold a pick write theirs.
__global__ __launch_bounds__(256) void route_backward_kernel(const int32_t *__restrict__ topk_idx,
                                                             const float *__restrict__ topk_w,
                                                             const float *__restrict__ d_topk_w,
                                                             float *__restrict__ dlogits, int T, int E, int k) {
  const int lane = lane_id();
  const int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (t >= T) return;  // whole wave
  float *row = dlogits + (size_t)t * E;
  for (int e = lane; e < E; e += kWave) row[e] = 0.f;
  const float w = lane < k ? topk_w[(size_t)t * k + lane] : 0.f;
  const float dw = lane < k ? d_topk_w[(size_t)t * k + lane] : 0.f;
  float dot = 0.f;
  for (int j = 0; j < k; ++j)  // slot order, the same sum in every lane
    dot = fmaf(__shfl(w, j), __shfl(dw, j), dot);
  // the zeros above and the values below come from different lanes of this wave: order them
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  __builtin_amdgcn_s_waitcnt(0x0F70);  // the zero stores have been acknowledged (vmcnt(0))
  if (lane < k) {
    const int e = topk_idx[(size_t)t * k + lane];
    if (e >= 0 && e < E) row[e] = w * (dw - dot);
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
  if (shape->E <= 512) {
    const dim3 grid(ceil_div(shape->T, 4)), block(256);
    hipStream_t st = (hipStream_t)stream;
#define MOE355_ROUTE(PER_) \
  hipLaunchKernelGGL(route_topk_reg_kernel<PER_>, grid, block, 0, st, logits, topk_idx, topk_w, shape->T, shape->E, shape->k)
    if (shape->E <= 64) MOE355_ROUTE(1);
    else if (shape->E <= 128) MOE355_ROUTE(2);
    else if (shape->E <= 256) MOE355_ROUTE(4);
    else MOE355_ROUTE(8);
#undef MOE355_ROUTE
    return launch_status();
  }
  const size_t per_wave = (size_t)(shape->E + kMaxTopK) * sizeof(uint32_t);
  int waves = kRouteWaves;
  while (waves > 1 && waves * per_wave > 48 * 1024) waves >>= 1;
  const int blocks = ceil_div(shape->T, waves);
  const size_t smem = waves * per_wave;
  hipLaunchKernelGGL(route_topk_kernel, dim3(blocks), dim3(waves * kWave), smem, (hipStream_t)stream, logits,
                     topk_idx, topk_w, shape->T, shape->E, shape->k);
  return launch_status();
}

extern "C" int moe_route_topk_gate(const moe_shape *shape, const float *logits, const float *bias, int gate,
                                   int32_t *topk_idx, float *topk_w, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!logits || !topk_idx || !topk_w || (gate != MOE_GATE_SOFTMAX && gate != MOE_GATE_SIGMOID))
    return MOE_ERR_INVALID_ARG;
  if (shape->T == 0) return MOE_OK;
  begin_launches();
  const size_t per_wave = (size_t)(shape->E + kMaxTopK) * sizeof(uint32_t);
  int waves = kRouteWaves;
  while (waves > 1 && waves * per_wave > 48 * 1024) waves >>= 1;
  hipLaunchKernelGGL(route_topk_gate_kernel, dim3(ceil_div(shape->T, waves)), dim3(waves * kWave), waves * per_wave,
                     (hipStream_t)stream, logits, bias, gate, topk_idx, topk_w, shape->T, shape->E, shape->k);
  return launch_status();
}

extern "C" int moe_route_backward(const moe_shape *shape, const int32_t *topk_idx, const float *topk_w,
                                  const float *d_topk_w, float *dlogits, void *stream) {
  Derived dv;
  int rc = check_shape(shape, &dv);
  if (rc != MOE_OK) return rc;
  if (!topk_idx || !topk_w || !d_topk_w || !dlogits) return MOE_ERR_INVALID_ARG;
  if (shape->T == 0) return MOE_OK;
  begin_launches();
  hipLaunchKernelGGL(route_backward_kernel, dim3(ceil_div(shape->T, 4)), dim3(256), 0, (hipStream_t)stream, topk_idx,
                     topk_w, d_topk_w, dlogits, shape->T, shape->E, shape->k);
  return launch_status();
}
