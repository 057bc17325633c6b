// On-the-fly FP8 quantisation of activations for the FP8 mixture-of-experts layer: one float32
// scale per row and per 128 reduction indices (1 x 128 tiles), codes in OCP e4m3.  Float32
// arithmetic in exactly these steps, because the steps decide integer codes:
//     m = max(max |x| over the tile, 1e-4);  scale = m / 448;  code = e4m3(x * (448 / m))
// (the published fine-grained FP8 recipe of the model family the paper serves; Section VII-D names
// the workload, Table II the kernel).  The second kernel applies SiLU-and-multiply to the gate/up
// product first, rounds the activation to the 16-bit type (it is a 16-bit tensor by the layer's
// definition) and quantises that, so the activation never goes to memory in 16 bits.
//
// Mapping: a tile of 128 elements is handled by 16 lanes with 8 consecutive elements each
// (16-byte loads, 8-byte code stores); a wave covers four tiles; the tile maximum is a four-step
// butterfly inside the 16 lanes.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"   // 16-bit conversions and silu_f32 only

namespace fp8 {

typedef uint32_t q_u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t q_u32x2 __attribute__((ext_vector_type(2)));

// two float32 -> two e4m3 codes in the low or high half of a word (round to nearest even; the
// matrix unit's own converter, OCP flavour on this chip)
__device__ __forceinline__ uint32_t pack_e4m3(float a, float b, uint32_t old, bool high) {
  return high ? (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, true)
              : (uint32_t)__builtin_amdgcn_cvt_pk_fp8_f32(a, b, (int)old, false);
}

// FUSE = 0: X [rows, K] -> codes [rows, K], scales [rows, K / 128]
// FUSE = 1: H [rows, 2K] (columns [0, K) gate, [K, 2K) up) -> the same for act = rnd(silu(gate) * up)
template <int DT, int FUSE>
__global__ void __launch_bounds__(256)
quantize_rows_kernel(const uint16_t* __restrict__ X, long long rows, int K, uint8_t* __restrict__ codes,
                     float* __restrict__ scales) {
  const int KB = K >> 7;
  const long long tiles = rows * KB;
  const int lane16 = threadIdx.x & 15;
  const long long group0 = ((long long)blockIdx.x * 256 + threadIdx.x) >> 4;      // 16-lane group index
  const long long ngroups = ((long long)gridDim.x * 256) >> 4;
  for (long long t = group0; t < tiles; t += ngroups) {                           // uniform per 16-lane group
    const long long row = t / KB;
    const int kb = (int)(t - row * KB);
    const int col = kb * 128 + lane16 * 8;
    float x[8];
    if constexpr (FUSE) {
      const uint16_t* hrow = X + row * 2 * (long long)K;
      const q_u32x4 g = *reinterpret_cast<const q_u32x4*>(hrow + col);
      const q_u32x4 u = *reinterpret_cast<const q_u32x4*>(hrow + K + col);
      const uint32_t gw[4] = {g.x, g.y, g.z, g.w}, uw[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float g0 = moe::from_bits16<DT>((uint16_t)gw[i]), g1 = moe::from_bits16<DT>((uint16_t)(gw[i] >> 16));
        const float u0 = moe::from_bits16<DT>((uint16_t)uw[i]), u1 = moe::from_bits16<DT>((uint16_t)(uw[i] >> 16));
        // the activation is a 16-bit tensor: round it before it is quantised
        x[2 * i] = moe::from_bits16<DT>(moe::to_bits16<DT>(moe::silu_f32(g0) * u0));
        x[2 * i + 1] = moe::from_bits16<DT>(moe::to_bits16<DT>(moe::silu_f32(g1) * u1));
      }
    } else {
      const q_u32x4 v = *reinterpret_cast<const q_u32x4*>(X + row * (long long)K + col);
      const uint32_t vw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[2 * i] = moe::from_bits16<DT>((uint16_t)vw[i]);
        x[2 * i + 1] = moe::from_bits16<DT>((uint16_t)(vw[i] >> 16));
      }
    }
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(x[i]));
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 16));
    m = fmaxf(m, 1e-4f);
    const float ratio = 448.0f / m;          // correctly rounded float32 division
    uint32_t lo = 0u, hi = 0u;
    lo = pack_e4m3(x[0] * ratio, x[1] * ratio, lo, false);
    lo = pack_e4m3(x[2] * ratio, x[3] * ratio, lo, true);
    hi = pack_e4m3(x[4] * ratio, x[5] * ratio, hi, false);
    hi = pack_e4m3(x[6] * ratio, x[7] * ratio, hi, true);
    *reinterpret_cast<q_u32x2*>(codes + row * (long long)K + col) = q_u32x2{lo, hi};
    if (lane16 == 0) scales[t] = m / 448.0f;
  }
}

// rows * K / 128 tiles, 16 per workgroup; returns a hipError_t
int launch_fp8_quantize(const void* X, long long rows, int K, int dt, int fuse_silu, uint8_t* codes, float* scales,
                        hipStream_t stream) {
  const long long tiles = rows * (K >> 7);
  if (tiles == 0) return 0;
  long long blocks = (tiles + 15) / 16;
  const long long cap = 256LL * 32;
  if (blocks > cap) blocks = cap;
  const dim3 grid((unsigned)blocks), block(256);
  const uint16_t* x = (const uint16_t*)X;
#define FP8_LAUNCH_Q(DT, F) hipLaunchKernelGGL((quantize_rows_kernel<DT, F>), grid, block, 0, stream, x, rows, K, codes, scales)
  if (dt == moe::kF16) { if (fuse_silu) FP8_LAUNCH_Q(moe::kF16, 1); else FP8_LAUNCH_Q(moe::kF16, 0); }
  else { if (fuse_silu) FP8_LAUNCH_Q(moe::kBF16, 1); else FP8_LAUNCH_Q(moe::kBF16, 0); }
#undef FP8_LAUNCH_Q
  return (int)hipGetLastError();
}

}  // namespace fp8
