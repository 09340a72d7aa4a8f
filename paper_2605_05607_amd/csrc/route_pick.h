// Top-k selection of one token row held in registers: shared by the routing kernel and by the gate-network kernel
// that routes straight from its partial sums.
#pragma once
#include "common.h"

namespace moe355 {

// Order-preserving map from finite fp32 to uint32 (larger float <=> larger key); -0 and +0 map to the same
// key so that they tie, as they do under a float comparison.  Key 0 is never produced by a finite value and
// marks an expert that has already been picked.
__device__ __forceinline__ uint32_t ordered_key(float v) {
  const uint32_t b = __float_as_uint(v + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Maximum over the wave, returned in every lane: butterfly inside the rows of 16 lanes with data-parallel
// primitives (lane ^ 1, lane ^ 2, mirrored halves, mirrored row), then the four row results are combined.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  auto step = [](uint32_t x, uint32_t y) { return x > y ? x : y; };
  v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));   // quad_perm [1,0,3,2]
  v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));   // quad_perm [2,3,0,1]
  v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, false));  // row_half_mirror
  v = step(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, false));  // row_mirror
  const uint32_t a = (uint32_t)__builtin_amdgcn_readlane((int)v, 0), b = (uint32_t)__builtin_amdgcn_readlane((int)v, 16);
  const uint32_t c = (uint32_t)__builtin_amdgcn_readlane((int)v, 32), d = (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
  return step(step(a, b), step(c, d));
}

// The k picks of one token whose logits sit in registers, lane l owning experts [l * PER, l * PER + PER) (val = logit,
// key = ordered_key(logit), 0 for experts past E).  Ties resolve to the lower expert index because a lane scans its
// run upwards with a strict comparison and, across lanes, the lowest lane holding the wave maximum wins.  Lanes
// 0..k-1 write the picks (slot order = pick order) and their softmax weights renormalised over the picks.
template <int PER>
__device__ __forceinline__ void route_pick_registers(float (&val)[PER], uint32_t (&key)[PER], int E, int k, int t,
                                                     int32_t *__restrict__ topk_idx, float *__restrict__ topk_w) {
  const int lane = lane_id();
  int my_e = 0;
  float my_x = 0.f, first = 0.f, sum = 0.f;
  for (int j = 0; j < k; ++j) {
    uint32_t bk = 0;
    int bs = 0;
    float bv = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      if (key[i] > bk) {
        bk = key[i];
        bs = i;
        bv = val[i];
      }
    }
    const uint32_t top = wave_max_u32(bk);
    const unsigned long long holders = __ballot(bk == top);
    const int win = holders ? __builtin_ctzll(holders) : 0;
    const int slot = __builtin_amdgcn_readlane(bs, win);
    const float v_best = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bv), win));
    // k <= E, so an unpicked expert always exists; the clamp only guards against non-finite input
    int e_best = win * PER + slot;
    e_best = e_best < E ? e_best : 0;
#pragma unroll
    for (int i = 0; i < PER; ++i)
      if (lane == win && i == slot) key[i] = 0u;  // picked
    if (j == 0) first = v_best;                    // the largest logit: softmax shift
    const float x = expf(v_best - first);
    sum += x;                                      // slot order
    if (lane == j) {
      my_e = e_best;
      my_x = x;
    }
  }
  if (lane < k) {
    topk_idx[(size_t)t * k + lane] = my_e;
    topk_w[(size_t)t * k + lane] = my_x / sum;
  }
}

}  // namespace moe355
