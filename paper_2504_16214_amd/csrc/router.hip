// Router: logits [T, E] (+ optional per-expert bias) -> top-k expert ids and the softmax over the
// selected logits.  One wave per token; the E logits of a token live in the wave's registers
// (E <= 1024: at most 16 per lane), selection is k rounds of a wave-wide arg-max on a 64-bit key
// (order-preserving image of the float in the high word, inverted index in the low word), so ties
// go to the lower expert index by construction.  Also holds the two "achievable roof" probes the
// benchmark reports beside the nominal peaks.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "router_device.hpp"

namespace moe {

// grid: ceil(T / 4) workgroups of 256 threads (4 waves = 4 tokens)
__global__ void __launch_bounds__(256)
route_topk_kernel(const float* __restrict__ logits, const float* __restrict__ bias, int T, int E, int topk,
                  int32_t* __restrict__ ids, float* __restrict__ weights) {
  const int lane = threadIdx.x & 63;
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (t >= T) return;                       // whole wave exits together
  route_token(logits + (size_t)t * E, bias, E, topk, lane, ids + (size_t)t * topk, weights + (size_t)t * topk);
}

int launch_route_topk(const float* logits, const float* bias, int T, int E, int topk, int32_t* ids,
                      float* weights, hipStream_t stream) {
  if (T == 0) return 0;
  hipLaunchKernelGGL(route_topk_kernel, dim3((T + 3) / 4), dim3(256), 0, stream, logits, bias, T, E, topk, ids,
                     weights);
  return (int)hipGetLastError();
}

// ---- achievable-roof probes ---------------------------------------------------------------
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Streaming read of `n16` 16-byte words with non-temporal 128-bit loads, the way the GEMM streams
// weights: every workgroup walks its own contiguous slice with eight loads in flight per lane.
// The XOR of everything read goes to sink[workgroup] so nothing is optimised away.
__global__ void __launch_bounds__(256)
stream_read_kernel(const u32x4_t* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
  constexpr int UNR = 8;
  const size_t per_wg = n16 / gridDim.x;                   // the remainder (< gridDim.x words) is not read
  const u32x4_t* p = src + per_wg * blockIdx.x;
  u32x4_t acc = {0u, 0u, 0u, 0u};
  size_t i = threadIdx.x;
  for (; i + (UNR - 1) * 256 < per_wg; i += 256 * UNR) {
    u32x4_t v[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
    for (int u = 0; u < UNR; ++u) acc ^= v[u];
  }
  for (; i < per_wg; i += 256) acc ^= __builtin_nontemporal_load(p + i);
  uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) r ^= __shfl_xor(r, off, 64);
  if ((threadIdx.x & 63) == 0) atomicXor(sink + blockIdx.x, r);
}

// Register-resident MFMA loop: every wave issues `iters` x 16 independent
// v_mfma_f32_16x16x32_f16 (4 accumulators round-robin); 2 workgroups of 4 waves per CU.
__global__ void __launch_bounds__(256)
mfma_loop_kernel(float* __restrict__ sink, int iters) {
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  h8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(1.0f + (threadIdx.x & 3)); b[i] = (_Float16)0.5f; }
  f32x4_t c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      c0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c1, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c2, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c3, 0, 0, 0);
    }
  }
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

int launch_stream_read(const void* src, size_t bytes, uint32_t* sink, int grid, hipStream_t stream) {
  hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(256), 0, stream, (const u32x4_t*)src, bytes / 16, sink);
  return (int)hipGetLastError();
}
int launch_mfma_loop(float* sink, int grid, int iters, hipStream_t stream) {
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(grid), dim3(256), 0, stream, sink, iters);
  return (int)hipGetLastError();
}

}  // namespace moe
