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

// Issue-mix probe: what one SIMD sustains when matrix instructions share it with VALU work and LDS
// fragment reads, the three things the mixed-type GEMM's inner loop is made of.  Per 8 independent
// v_mfma_f32_16x16x32_f16 a wave issues 8 * NV independent VALU operations and ND ds_read_b128 in
// the GEMM's fragment-read pattern (row pitch 18 chunks).  256 workgroups of 8 waves = two waves
// per SIMD on every CU.  The instruction order is fixed by inline assembly; results are not
// meaningful numbers (nothing waits for a matrix result before it is overwritten by a later one
// of the same chain, and the LDS is never initialised): the probe measures issue rates only.
template <int NV, int ND>
__global__ void __launch_bounds__(512)
issue_mix_kernel(float* __restrict__ sink, int iters) {
  extern __shared__ __align__(16) unsigned char mix_lds[];
  f32x4_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = f32x4_t{0, 0, 0, 0};
  u32x4_t a = {0x3c003c00u + threadIdx.x, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u}, b = a;
  uint32_t x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = threadIdx.x * 7 + i;
  uint32_t m1 = 0x000F000Fu, o1 = 0x64006400u;
  asm volatile("" : "+v"(m1), "+v"(o1));
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t addr = wave * 8192 + ((lane & 15) * 18 + (lane >> 4)) * 16;
  u32x4_t r[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) r[i] = a;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+v"(acc[u]) : "v"(r[u]), "v"(b));
#pragma unroll
      for (int v = 0; v < NV; ++v)
        asm volatile("v_and_or_b32 %0, %0, %1, %2" : "+v"(x[(u * NV + v) % 8]) : "v"(m1), "v"(o1));
      if (u < ND) asm volatile("ds_read_b128 %0, %1" : "=v"(r[(u + 4) % 8]) : "v"(addr));
    }
    if (ND > 0) asm volatile("s_waitcnt lgkmcnt(0)");
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += acc[i][0] + (float)x[i] + (float)r[i].x;
  sink[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

template <int NV, int ND>
static int launch_issue_mix_t(float* sink, int iters, hipStream_t stream) {
  hipLaunchKernelGGL((issue_mix_kernel<NV, ND>), dim3(256), dim3(512), 64 * 1024, stream, sink, iters);
  return (int)hipGetLastError();
}

// NV in {0, 1, 2, 3, 4, 6}, ND in {0, 2, 4, 8}; -1 for any other combination
int launch_issue_mix(float* sink, int iters, int nv, int nd, hipStream_t stream) {
#define MOE_MIX(NV, ND) if (nv == NV && nd == ND) return launch_issue_mix_t<NV, ND>(sink, iters, stream);
#define MOE_MIX_ROW(NV) MOE_MIX(NV, 0) MOE_MIX(NV, 2) MOE_MIX(NV, 4) MOE_MIX(NV, 8)
  MOE_MIX_ROW(0) MOE_MIX_ROW(1) MOE_MIX_ROW(2) MOE_MIX_ROW(3) MOE_MIX_ROW(4) MOE_MIX_ROW(6)
#undef MOE_MIX_ROW
#undef MOE_MIX
  return -1;
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
