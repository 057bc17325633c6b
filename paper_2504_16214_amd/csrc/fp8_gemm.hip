// Blockwise-scaled FP8 GEMM for gfx950:
//   C[m, n] = sum_kb a_scale[m, kb] * b_scale[n / 128, kb] * sum_{k in block kb} A[m, k] * B[n, k]
// A [M, K], B [N, K] e4m3 codes (OCP), scales float32, one reduction block = 128 = the depth of one
// v_mfma_f32_16x16x128_f8f6f4, so every matrix instruction starts from a zero accumulator and its
// result is folded into the float32 accumulator with one scaled FMA per register.
//
// Mapping.  A workgroup of four waves owns BM = 16 MT rows of A ("tokens") and BN = 4 * 16 NT rows
// of B ("features"); wave w owns features [16 NT w, 16 NT (w + 1)) of the tile.  The features are
// the matrix instruction's row operand and the tokens its column operand, so a lane ends up with
// one token and 4 NT consecutive features: 16-byte stores, and one activation scale per lane.
//   * B is never shared inside a workgroup: every wave streams its own rows straight from global
//     memory in operand order (lane (n, j) reads bytes [16 j, 16 j + 16) and [64 + 16 j, +16) of its
//     row's 128-byte block: full lines per row), one reduction block ahead, in registers.
//   * A is shared by the four waves: global -> registers -> LDS (two buffers, one barrier per
//     block), read back with the same byte permutation.  The order of the 128 reduction indices
//     inside an instruction is free as long as both operands use the same one.
//   * Split reduction: blockIdx also selects a range of reduction blocks; split i writes plane i
//     of a float32 buffer and a second kernel adds the planes in order and rounds once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "fp8_gemm.hpp"

namespace fp8 {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kPitch = 160;   // LDS bytes per activation row: 128 + 32 (10 chunks: conflict-free operand reads)

__device__ __forceinline__ uint32_t to_bf16_bits(float x) {
  uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ uint32_t to_f16_bits(float x) {
  const _Float16 h = (_Float16)x;                 // round to nearest even
  return (uint32_t)__builtin_bit_cast(uint16_t, h);
}
template <int BF16>
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return BF16 ? (to_bf16_bits(lo) | (to_bf16_bits(hi) << 16)) : (to_f16_bits(lo) | (to_f16_bits(hi) << 16));
}

// NTL: weights are read once per launch (one row block): non-temporal loads
template <int MT, int NT, int NTL>
__global__ void __launch_bounds__(256)
fp8_blockwise_gemm_kernel(const GemmParams p) {
  constexpr int BM = 16 * MT, WN = 16 * NT, BN = 4 * WN;
  constexpr int ACH = (BM * 8 + 255) / 256;             // 16-byte chunks of the activation tile per thread
  __shared__ __attribute__((aligned(16))) unsigned char xs[2][BM * kPitch];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ln = lane & 15, lj = lane >> 4;

  // hardware block id -> logical tile: consecutive ids go round the 8 XCDs, so give every XCD a
  // contiguous range of tiles; inside a range the row blocks of one feature block are neighbours
  // (they share the weight rows through that XCD's L2)
  const int total = gridDim.x;
  int L;
  {
    const int id = blockIdx.x, q = total >> 3, r = total & 7, x = id & 7;
    L = x * q + (x < r ? x : r) + (id >> 3);
  }
  const int m_blocks = (p.M + BM - 1) / BM, n_blocks = p.N / BN;
  const int split = L / (m_blocks * n_blocks);
  L -= split * (m_blocks * n_blocks);
  const int nb = L / m_blocks, mb = L - nb * m_blocks;
  const int row0 = mb * BM;                       // first token of the tile
  const int n0w = nb * BN + wave * WN;            // first feature of this wave
  const int KB = p.K >> 7;
  const int kb0 = split * p.kb_per_split;
  int kb1 = kb0 + p.kb_per_split;
  if (kb1 > KB) kb1 = KB;
  const int nkb = kb1 - kb0;                      // >= 1 by construction of the grid

  // ---- per-lane source addresses ----
  const uint8_t* bsrc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int wrow = n0w + 4 * NT * (ln >> 2) + 4 * nt + (ln & 3);     // operand row ln of sub-tile nt
    bsrc[nt] = p.B + (size_t)wrow * p.K + 16 * lj;
  }
  const uint8_t* asrc[ACH];
  int adst[ACH];
#pragma unroll
  for (int i = 0; i < ACH; ++i) {
    const int c = tid + 256 * i;
    int r = c >> 3;
    if (r >= BM) r = BM - 1;                      // threads beyond the tile repeat its last row (not stored)
    int g = row0 + r;
    if (g >= p.M) g = p.M - 1;
    asrc[i] = p.A + (size_t)g * p.K + 16 * (c & 7);
    adst[i] = r * kPitch + 16 * (c & 7);
  }
  const float* assrc[MT];                         // activation scale of the lane's token in row block mt
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int g = row0 + 16 * mt + ln;
    if (g >= p.M) g = p.M - 1;
    assrc[mt] = p.a_scale + (size_t)g * KB;
  }
  const float* bssrc = p.b_scale + (size_t)(n0w >> 7) * KB;      // wave-uniform

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  i32x4 bw[2][NT][2];          // weight operands, ring of two reduction blocks
  i32x4 ar[ACH];               // activation chunks on their way to LDS
  float sa[2][MT], sb[2];

  auto load_block = [&](int ring, int kb) __attribute__((always_inline)) {
    const size_t off = (size_t)kb * 128;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const i32x4* s = reinterpret_cast<const i32x4*>(bsrc[nt] + off);
      if (NTL) {
        bw[ring][nt][0] = __builtin_nontemporal_load(s);
        bw[ring][nt][1] = __builtin_nontemporal_load(s + 4);
      } else {
        bw[ring][nt][0] = s[0];
        bw[ring][nt][1] = s[4];
      }
    }
#pragma unroll
    for (int i = 0; i < ACH; ++i) ar[i] = *reinterpret_cast<const i32x4*>(asrc[i] + off);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) sa[ring][mt] = assrc[mt][kb];
    sb[ring] = bssrc[kb];
  };
  auto store_a = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < ACH; ++i)
      if (tid + 256 * i < BM * 8) *reinterpret_cast<i32x4*>(&xs[buf][adst[i]]) = ar[i];
  };
  auto compute = [&](int ring) __attribute__((always_inline)) {
    const float bs = sb[ring];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const unsigned char* xp = &xs[ring][(16 * mt + ln) * kPitch + 16 * lj];
      const i32x4 lo = *reinterpret_cast<const i32x4*>(xp);
      const i32x4 hi = *reinterpret_cast<const i32x4*>(xp + 64);
      const i32x8 xa = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      const float sp = sa[ring][mt] * bs;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const i32x4 w0 = bw[ring][nt][0], w1 = bw[ring][nt][1];
        const i32x8 wa = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
        const f32x4 part = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
            wa, xa, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);       // e4m3 x e4m3, no block exponents
        acc[mt][nt] += part * sp;
      }
    }
  };

  // ---- pipeline: block i + 1 is in flight while block i is multiplied ----
  load_block(0, kb0);
  store_a(0);
  __syncthreads();
  for (int it = 0; it < nkb; it += 2) {
    {
      const int nx = it + 1 < nkb ? it + 1 : nkb - 1;      // past the end: a valid block, never consumed
      load_block(1, kb0 + nx);
      compute(0);
      store_a(1);
      __syncthreads();
    }
    if (it + 1 < nkb) {
      const int nx = it + 2 < nkb ? it + 2 : nkb - 1;
      load_block(0, kb0 + nx);
      compute(1);
      store_a(0);
      __syncthreads();
    }
  }

  // ---- epilogue: the lane's token, 4 NT consecutive features ----
  const int f0 = n0w + 4 * NT * lj;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int t = row0 + 16 * mt + ln;
    if (t >= p.M) continue;
    if (p.k_splits > 1) {
      float* dst = reinterpret_cast<float*>(p.C) + ((size_t)split * p.M + t) * p.N + f0;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) *reinterpret_cast<f32x4*>(dst + 4 * nt) = acc[mt][nt];
    } else {
      uint16_t* dst = reinterpret_cast<uint16_t*>(p.C) + (size_t)t * p.N + f0;
      uint32_t w[2 * NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if (p.out_bf16) {
          w[2 * nt] = pack2<1>(acc[mt][nt][0], acc[mt][nt][1]);
          w[2 * nt + 1] = pack2<1>(acc[mt][nt][2], acc[mt][nt][3]);
        } else {
          w[2 * nt] = pack2<0>(acc[mt][nt][0], acc[mt][nt][1]);
          w[2 * nt + 1] = pack2<0>(acc[mt][nt][2], acc[mt][nt][3]);
        }
      }
      if constexpr (NT == 1) {
        *reinterpret_cast<u32x2*>(dst) = u32x2{w[0], w[1]};
      } else {
#pragma unroll
        for (int h = 0; h < NT / 2; ++h)
          *reinterpret_cast<u32x4*>(dst + 8 * h) = u32x4{w[4 * h], w[4 * h + 1], w[4 * h + 2], w[4 * h + 3]};
      }
    }
  }
}

// Sum of the float32 planes in plane order, one rounding.  n4 = M * N / 4.
__global__ void __launch_bounds__(256)
fp8_split_reduce_kernel(const f32x4* __restrict__ planes, int k_splits, long long n4, u32x2* __restrict__ C,
                        int out_bf16) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long long)gridDim.x * 256) {
    f32x4 s = planes[i];
    for (int k = 1; k < k_splits; ++k) s += planes[(long long)k * n4 + i];
    C[i] = out_bf16 ? u32x2{pack2<1>(s[0], s[1]), pack2<1>(s[2], s[3])}
                    : u32x2{pack2<0>(s[0], s[1]), pack2<0>(s[2], s[3])};
  }
}

template <int MT, int NT, int NTL>
static int launch_one(const GemmParams& p, hipStream_t stream) {
  constexpr int BM = 16 * MT, BN = 64 * NT;
  const int grid = ((p.M + BM - 1) / BM) * (p.N / BN) * p.k_splits;
  hipLaunchKernelGGL((fp8_blockwise_gemm_kernel<MT, NT, NTL>), dim3(grid), dim3(256), 0, stream, p);
  return (int)hipGetLastError();
}

template <int MT>
static int launch_mt(const GemmParams& p, int nt, int ntl, hipStream_t stream) {
  if (MT <= 4 && ntl) {
    constexpr int NTLv = MT <= 4 ? 1 : 0;
    switch (nt) {
      case 1: return launch_one<MT, 1, NTLv>(p, stream);
      case 2: return launch_one<MT, 2, NTLv>(p, stream);
      case 4: return launch_one<MT, 4, NTLv>(p, stream);
    }
  } else {
    switch (nt) {
      case 1: return launch_one<MT, 1, 0>(p, stream);
      case 2: return launch_one<MT, 2, 0>(p, stream);
      case 4: return launch_one<MT, 4, 0>(p, stream);
    }
  }
  return -1;
}

// mt in {1, 2, 4, 8}, nt in {1, 2, 4}; -1: no such variant
int launch_fp8_gemm(const GemmParams& p, int mt, int nt, int ntl, hipStream_t stream) {
  switch (mt) {
    case 1: return launch_mt<1>(p, nt, ntl, stream);
    case 2: return launch_mt<2>(p, nt, ntl, stream);
    case 4: return launch_mt<4>(p, nt, ntl, stream);
    case 8: return launch_mt<8>(p, nt, ntl, stream);
  }
  return -1;
}

// Register-resident loop of the FP8 matrix instruction (the achievable matrix-unit roof).
__global__ void __launch_bounds__(256)
fp8_mfma_loop_kernel(float* __restrict__ sink, int iters) {
  i32x8 a, b;
#pragma unroll
  for (int i = 0; i < 8; ++i) { a[i] = 0x38383838; b[i] = 0x30303030 + (int)(threadIdx.x & 1); }
  f32x4 c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      c0 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c0, 0, 0, 0, 0, 0, 0);
      c1 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c1, 0, 0, 0, 0, 0, 0);
      c2 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c2, 0, 0, 0, 0, 0, 0);
      c3 = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c3, 0, 0, 0, 0, 0, 0);
    }
  }
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
}

int launch_fp8_mfma_loop(float* sink, int grid, int iters, hipStream_t stream) {
  hipLaunchKernelGGL(fp8_mfma_loop_kernel, dim3(grid), dim3(256), 0, stream, sink, iters);
  return (int)hipGetLastError();
}

int launch_fp8_split_reduce(const float* planes, int k_splits, long long mn, void* C, int out_bf16,
                            hipStream_t stream) {
  const long long n4 = mn / 4;
  long long blocks = (n4 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(fp8_split_reduce_kernel, dim3((int)blocks), dim3(256), 0, stream, (const f32x4*)planes,
                     k_splits, n4, (u32x2*)C, out_bf16);
  return (int)hipGetLastError();
}

}  // namespace fp8
