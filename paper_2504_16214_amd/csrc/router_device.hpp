// Per-token routing by one wavefront, shared by the stand-alone router kernel and the fused
// router + bucketing kernel: top-k of a row of logits (+ optional per-expert bias) in descending
// order, ties to the lower expert index, and the softmax over the selected values.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace moe {

constexpr int kRouterMaxPerLane = 16;   // E <= 64 * 16

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) {
    const unsigned long long o = __shfl_xor(v, off, 64);
    v = o > v ? o : v;
  }
  return v;
}

__device__ __forceinline__ float wave_sum_f32_lanes_below(float v, int n) {
  // sum of lanes [0, n) in lane order 0, 1, 2, ... (sequential: k is small and the order is fixed)
  float s = 0.f;
#pragma unroll 1
  for (int j = 0; j < n; ++j) s += __shfl(v, j, 64);
  return s;
}

// One wave routes token `row`: the E logits live in the wave's registers (E <= 1024: at most 16
// per lane), selection is topk rounds of a wave-wide arg-max on a 64-bit key (order-preserving
// image of the float in the high word, inverted index in the low word).  Lanes [0, topk) write
// ids_out[lane] and w_out[lane].
__device__ __forceinline__ void route_token(const float* __restrict__ row, const float* __restrict__ bias, int E,
                                            int topk, int lane, int32_t* ids_out, float* w_out) {
  // key of element e = lane + 64 i: ordered(float) << 32 | ~e ; 0 marks "absent or taken"
  unsigned long long key[kRouterMaxPerLane];
#pragma unroll
  for (int i = 0; i < kRouterMaxPerLane; ++i) {
    const int e = lane + 64 * i;
    key[i] = 0ull;
    if (e < E) {
      float v = row[e];
      if (bias) v = v + bias[e];            // one float32 rounding, as the definition states
      v = v + 0.0f;                         // -0.0 -> +0.0: signed zeros compare equal
      uint32_t u = __float_as_uint(v);
      u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      key[i] = ((unsigned long long)u << 32) | (unsigned long long)(0xffffffffu - (uint32_t)e);
    }
  }
  float my_val = 0.f;                       // lane j keeps the j-th selected logit (j < topk <= 64)
  int my_id = 0;
#pragma unroll 1
  for (int j = 0; j < topk; ++j) {      // (not unrolled: topk is a run-time value up to 64 and the body holds all 16 keys)
    unsigned long long best = 0ull;
#pragma unroll
    for (int i = 0; i < kRouterMaxPerLane; ++i) best = key[i] > best ? key[i] : best;
    best = wave_max_u64(best);
    const uint32_t e = 0xffffffffu - (uint32_t)(best & 0xffffffffull);
    uint32_t u = (uint32_t)(best >> 32);
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    my_val = lane == j ? __uint_as_float(u) : my_val;
    my_id = lane == j ? (int)e : my_id;
    // the owner lane retires the element (selects, not branches: with branches the compiler keeps a
    // copy of all sixteen keys per path)
#pragma unroll
    for (int i = 0; i < kRouterMaxPerLane; ++i) key[i] = ((int)e == lane + 64 * i) ? 0ull : key[i];
  }
  // softmax over the k selected logits; the first selected one is the maximum
  const float m = __shfl(my_val, 0, 64);
  const float p = lane < topk ? expf(my_val - m) : 0.f;
  const float denom = wave_sum_f32_lanes_below(p, topk);
  if (lane < topk) {
    ids_out[lane] = my_id;
    w_out[lane] = p / denom;
  }
}


// ---- the same routing by a group of 16 lanes (one DPP row), four tokens per wave ---------------
// For E <= 256 and topk <= 16: a lane holds at most 16 keys (element e = lane16 + 16 i), the
// group-wide arg-max is four DPP steps inside the row (no LDS permutes), and the arithmetic of the
// weights is the one of route_token, operation for operation (same bits).
template <int CTRL>
__device__ __forceinline__ unsigned long long dpp_u64(unsigned long long v) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, CTRL, 0xf, 0xf, true);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(v >> 32), CTRL, 0xf, 0xf, true);
  return ((unsigned long long)hi << 32) | lo;
}

__device__ __forceinline__ unsigned long long row_max_u64(unsigned long long v) {
  unsigned long long o;
  o = dpp_u64<0xB1>(v);  v = o > v ? o : v;      // quad_perm [1,0,3,2]: lane ^ 1
  o = dpp_u64<0x4E>(v);  v = o > v ? o : v;      // quad_perm [2,3,0,1]: lane ^ 2
  o = dpp_u64<0x141>(v); v = o > v ? o : v;      // row_half_mirror: the other quad of each 8 lanes
  o = dpp_u64<0x140>(v); v = o > v ? o : v;      // row_mirror: the other half of the row
  return v;
}

constexpr int kRouter16MaxE = 256, kRouter16MaxTopk = 16;

__device__ __forceinline__ void route_token_row16(const float* __restrict__ row, const float* __restrict__ bias, int E,
                                                  int topk, int lane, int32_t* ids_out, float* w_out) {
  const int l16 = lane & 15;
  unsigned long long key[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int e = l16 + 16 * i;
    key[i] = 0ull;
    if (e < E) {
      float v = row[e];
      if (bias) v = v + bias[e];
      v = v + 0.0f;
      uint32_t u = __float_as_uint(v);
      u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
      key[i] = ((unsigned long long)u << 32) | (unsigned long long)(0xffffffffu - (uint32_t)e);
    }
  }
  float my_val = 0.f;
  int my_id = 0;
#pragma unroll 1
  for (int j = 0; j < topk; ++j) {
    unsigned long long best = 0ull;
#pragma unroll
    for (int i = 0; i < 16; ++i) best = key[i] > best ? key[i] : best;
    best = row_max_u64(best);
    const uint32_t e = 0xffffffffu - (uint32_t)(best & 0xffffffffull);
    uint32_t u = (uint32_t)(best >> 32);
    u = (u & 0x80000000u) ? (u & 0x7fffffffu) : ~u;
    my_val = l16 == j ? __uint_as_float(u) : my_val;
    my_id = l16 == j ? (int)e : my_id;
#pragma unroll
    for (int i = 0; i < 16; ++i) key[i] = ((int)e == l16 + 16 * i) ? 0ull : key[i];
  }
  const float m = __shfl(my_val, 0, 16);
  const float p = l16 < topk ? expf(my_val - m) : 0.f;
  float denom = 0.f;
#pragma unroll 1
  for (int j = 0; j < topk; ++j) denom += __shfl(p, j, 16);      // lane order, as in route_token
  if (l16 < topk) {
    ids_out[l16] = my_id;
    w_out[l16] = p / denom;
  }
}

}  // namespace moe
