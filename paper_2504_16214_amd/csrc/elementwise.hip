// SiLU-and-multiply between the two expert projections and the top-k weighted combine.
// Both are pure streaming kernels: 128-bit loads/stores, fp32 math, one rounding.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"   // 16-bit conversions and silu_f32 only

namespace moe {

template <int DT>
__global__ void __launch_bounds__(256)
silu_mul_kernel(const uint16_t* __restrict__ H, uint16_t* __restrict__ act, long long S, int N) {
  // one thread = 8 consecutive columns when N % 8 == 0, else one column
  const bool vec = (N & 7) == 0;
  const long long per_row = vec ? (N >> 3) : N;
  const long long total = S * per_row;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long s = i / per_row;
    const int c = (int)(i - s * per_row);
    const uint16_t* hrow = H + s * 2 * (long long)N;
    uint16_t* arow = act + s * (long long)N;
    if (vec) {
      const uint4 g = *reinterpret_cast<const uint4*>(hrow + c * 8);
      const uint4 u = *reinterpret_cast<const uint4*>(hrow + N + c * 8);
      const uint32_t gw[4] = {g.x, g.y, g.z, g.w}, uw[4] = {u.x, u.y, u.z, u.w};
      uint32_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const float g0 = from_bits16<DT>((uint16_t)gw[k]), g1 = from_bits16<DT>((uint16_t)(gw[k] >> 16));
        const float u0 = from_bits16<DT>((uint16_t)uw[k]), u1 = from_bits16<DT>((uint16_t)(uw[k] >> 16));
        o[k] = (uint32_t)to_bits16<DT>(silu_f32(g0) * u0) | ((uint32_t)to_bits16<DT>(silu_f32(g1) * u1) << 16);
      }
      *reinterpret_cast<uint4*>(arow + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
      arow[c] = to_bits16<DT>(silu_f32(from_bits16<DT>(hrow[c])) * from_bits16<DT>(hrow[N + c]));
    }
  }
}

// ids == nullptr: every slot contributes.  Otherwise slots whose expert id lies outside
// [0, E) contribute zero (their Y rows were never written).
// YF32 = 1: Y holds float32 (the fused layer keeps the down projection unrounded until here).
template <int DT, int YF32>
__global__ void __launch_bounds__(256)
combine_kernel(const void* __restrict__ Yv, const float* __restrict__ w, const int32_t* __restrict__ ids,
               int E, uint16_t* __restrict__ out, long long T, int topk, int K, int planes, long long plane) {
  const uint16_t* Y = reinterpret_cast<const uint16_t*>(Yv);
  const float* Yf = reinterpret_cast<const float*>(Yv);
  const bool vec = (K & 7) == 0;
  const long long per_row = vec ? (K >> 3) : K;
  const long long total = T * per_row;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const long long t = i / per_row;
    const int c = (int)(i - t * per_row);
    if (vec) {
      float acc[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) acc[k] = 0.f;
      for (int j = 0; j < topk; ++j) {
        const long long slot = t * topk + j;
        if (ids) { const int e = ids[slot]; if (e < 0 || e >= E) continue; }
        const float wj = w[slot];
        if constexpr (YF32) {
          const float4 y0 = *reinterpret_cast<const float4*>(Yf + slot * (long long)K + c * 8);
          const float4 y1 = *reinterpret_cast<const float4*>(Yf + slot * (long long)K + c * 8 + 4);
          float yv[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
          // a split reduction left one partial sum per plane: add them in plane order
          for (int pl = 1; pl < planes; ++pl) {
            const float* yp = Yf + pl * plane + slot * (long long)K + c * 8;
            const float4 a0 = *reinterpret_cast<const float4*>(yp);
            const float4 a1 = *reinterpret_cast<const float4*>(yp + 4);
            yv[0] += a0.x; yv[1] += a0.y; yv[2] += a0.z; yv[3] += a0.w;
            yv[4] += a1.x; yv[5] += a1.y; yv[6] += a1.z; yv[7] += a1.w;
          }
#pragma unroll
          for (int k = 0; k < 8; ++k) acc[k] = __builtin_fmaf(wj, yv[k], acc[k]);
        } else {
          const uint4 y = *reinterpret_cast<const uint4*>(Y + slot * (long long)K + c * 8);
          const uint32_t yw[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            acc[2 * k] = __builtin_fmaf(wj, from_bits16<DT>((uint16_t)yw[k]), acc[2 * k]);
            acc[2 * k + 1] = __builtin_fmaf(wj, from_bits16<DT>((uint16_t)(yw[k] >> 16)), acc[2 * k + 1]);
          }
        }
      }
      uint32_t o[4];
#pragma unroll
      for (int k = 0; k < 4; ++k)
        o[k] = (uint32_t)to_bits16<DT>(acc[2 * k]) | ((uint32_t)to_bits16<DT>(acc[2 * k + 1]) << 16);
      *reinterpret_cast<uint4*>(out + t * (long long)K + c * 8) = make_uint4(o[0], o[1], o[2], o[3]);
    } else {
      float acc = 0.f;
      for (int j = 0; j < topk; ++j) {
        const long long slot = t * topk + j;
        if (ids) { const int e = ids[slot]; if (e < 0 || e >= E) continue; }
        float yv = YF32 ? Yf[slot * (long long)K + c] : from_bits16<DT>(Y[slot * (long long)K + c]);
        if constexpr (YF32) for (int pl = 1; pl < planes; ++pl) yv += Yf[pl * plane + slot * (long long)K + c];
        acc = __builtin_fmaf(w[slot], yv, acc);
      }
      out[t * (long long)K + c] = to_bits16<DT>(acc);
    }
  }
}

static int grid_for(long long work_items) {
  long long blocks = (work_items + 255) / 256;
  const long long cap = 256LL * 32;      // 256 CUs, grid-stride beyond that
  if (blocks > cap) blocks = cap;
  if (blocks < 1) blocks = 1;
  return (int)blocks;
}

// Offline repack of packed weights into operand order: a permutation of 16-byte chunks.
// Output chunk (((e*NB + b)*NC + c)*64 + 16*j + n) = bytes [64c + 16j, +16) of row r(b, n) of
// expert e; r = 16b + n, or (paired) 32*(b/2) + 2n + (b&1).
typedef uint32_t rp_u32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256)
repack_qweight_kernel(const rp_u32x4* __restrict__ in, rp_u32x4* __restrict__ out, long long total,
                      int N_out, int NB, int NC, int paired) {
  for (long long o = (long long)blockIdx.x * 256 + threadIdx.x; o < total; o += (long long)gridDim.x * 256) {
    const int l = (int)(o & 63);
    long long t = o >> 6;
    const int c = (int)(t % NC); t /= NC;
    const int b = (int)(t % NB);
    const long long e = t / NB;
    const int n = l & 15, j = l >> 4;
    const int row = paired ? 32 * (b >> 1) + 2 * n + (b & 1) : 16 * b + n;
    out[o] = in[(e * N_out + row) * (long long)(4 * NC) + 4 * c + j];
  }
}

int launch_repack(const int32_t* q, int E, int N_out, int K_in, int paired, int32_t* out, hipStream_t stream) {
  const int NB = N_out / 16, NC = K_in / 128;
  const long long total = (long long)E * NB * NC * 64;
  hipLaunchKernelGGL(repack_qweight_kernel, dim3(grid_for(total)), dim3(256), 0, stream,
                     (const rp_u32x4*)q, (rp_u32x4*)out, total, N_out, NB, NC, paired);
  return (int)hipGetLastError();
}

// Import of AWQ-packed tensors: qweight [E, K_in, N_out/8] words hold eight neighbouring output
// columns each, column 8c + n' at bits [4 r(n'), 4 r(n') + 4) with r = (0, 4, 1, 5, 2, 6, 3, 7); the
// result is this library's [E, N_out, K_in/8] words, sequential along the reduction.  A wave
// covers 64 output columns (so the eight lanes of a column group read the same word and a row's
// reads are contiguous); a lane gathers 32 reduction rows into four output words (16 bytes).
__device__ __forceinline__ uint32_t awq_nibble(uint32_t word, int col_in_word) {
  const int pos = ((col_in_word & 1) << 2) | (col_in_word >> 1);      // 0,4,1,5,2,6,3,7
  return (word >> (4 * pos)) & 0xFu;
}

__global__ void __launch_bounds__(256)
awq_import_qweight_kernel(const uint32_t* __restrict__ in, uint32_t* __restrict__ out, int K_in, int N_out,
                          int vec_ok) {
  const int NW = N_out >> 3, KW = K_in >> 3;
  const int n = blockIdx.x * 64 + (threadIdx.x & 63);
  const int kj0 = blockIdx.y * 16 + (threadIdx.x >> 6) * 4;
  const long long e = blockIdx.z;
  if (n >= N_out || kj0 >= KW) return;
  const uint32_t* src = in + e * (long long)K_in * NW + (n >> 3);
  uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (kj0 + j < KW) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t word = src[(long long)(8 * (kj0 + j) + i) * NW];
        w[j] |= awq_nibble(word, n & 7) << (4 * i);
      }
    }
  }
  uint32_t* dst = out + (e * N_out + n) * (long long)KW + kj0;
  if (vec_ok && kj0 + 3 < KW) {
    rp_u32x4 v = {w[0], w[1], w[2], w[3]};
    *reinterpret_cast<rp_u32x4*>(dst) = v;
  } else {
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (kj0 + j < KW) dst[j] = w[j];
  }
}

// scales [E, G, N_out] 16-bit -> [E, N_out, G]; qzeros [E, G, N_out/8] words -> zeros [E, N_out, G] bytes
__global__ void __launch_bounds__(256)
awq_import_scale_zero_kernel(const uint32_t* __restrict__ qzeros, const uint16_t* __restrict__ scales_in,
                             uint16_t* __restrict__ scales_out, uint8_t* __restrict__ zeros_out, long long total,
                             int G, int N_out) {
  for (long long o = (long long)blockIdx.x * 256 + threadIdx.x; o < total; o += (long long)gridDim.x * 256) {
    const int n = (int)(o % N_out);
    long long t = o / N_out;
    const int gi = (int)(t % G);
    const long long e = t / G;
    const long long dst = (e * N_out + n) * (long long)G + gi;
    scales_out[dst] = scales_in[o];
    zeros_out[dst] = (uint8_t)awq_nibble(qzeros[(e * G + gi) * (long long)(N_out >> 3) + (n >> 3)], n & 7);
  }
}

int launch_awq_import(const int32_t* aq, const int32_t* az, const void* as, int E, int K_in, int N_out, int group,
                      int32_t* q, void* s, uint8_t* z, hipStream_t stream) {
  const int KW = K_in / 8, G = K_in / group;
  const int vec_ok = (KW % 4 == 0 && ((uintptr_t)q % 16) == 0) ? 1 : 0;
  hipLaunchKernelGGL(awq_import_qweight_kernel, dim3((N_out + 63) / 64, (KW + 15) / 16, E), dim3(256), 0, stream,
                     (const uint32_t*)aq, (uint32_t*)q, K_in, N_out, vec_ok);
  int err = (int)hipGetLastError();
  if (err != 0) return err;
  const long long total = (long long)E * G * N_out;
  hipLaunchKernelGGL(awq_import_scale_zero_kernel, dim3(grid_for(total)), dim3(256), 0, stream,
                     (const uint32_t*)az, (const uint16_t*)as, (uint16_t*)s, z, total, G, N_out);
  return (int)hipGetLastError();
}

int launch_silu_mul(const void* H, void* act, long long S, int N, int dt, hipStream_t stream) {
  const long long items = S * (((N & 7) == 0) ? (N >> 3) : N);
  if (items == 0) return 0;
  if (dt == kF16)
    hipLaunchKernelGGL(silu_mul_kernel<kF16>, dim3(grid_for(items)), dim3(256), 0, stream,
                       (const uint16_t*)H, (uint16_t*)act, S, N);
  else
    hipLaunchKernelGGL(silu_mul_kernel<kBF16>, dim3(grid_for(items)), dim3(256), 0, stream,
                       (const uint16_t*)H, (uint16_t*)act, S, N);
  return (int)hipGetLastError();
}

int launch_combine(const void* Y, int y_f32, int planes, const float* w, const int32_t* ids, int E, void* out,
                   long long T, int topk, int K, int dt, hipStream_t stream) {
  const long long plane = T * topk * (long long)K;      // elements per partial-sum plane
  const long long items = T * (((K & 7) == 0) ? (K >> 3) : K);
  if (items == 0) return 0;
  const dim3 grid(grid_for(items)), block(256);
#define MOE_LAUNCH_COMBINE(DT, F) \
  hipLaunchKernelGGL((combine_kernel<DT, F>), grid, block, 0, stream, Y, w, ids, E, (uint16_t*)out, T, topk, K, planes, plane)
  if (dt == kF16) { if (y_f32) MOE_LAUNCH_COMBINE(kF16, 1); else MOE_LAUNCH_COMBINE(kF16, 0); }
  else { if (y_f32) MOE_LAUNCH_COMBINE(kBF16, 1); else MOE_LAUNCH_COMBINE(kBF16, 0); }
#undef MOE_LAUNCH_COMBINE
  return (int)hipGetLastError();
}

}  // namespace moe
