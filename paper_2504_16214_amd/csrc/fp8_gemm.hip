// Blockwise-scaled FP8 GEMM for gfx950:
//   C[m, n] = sum_kb a_scale[m, kb] * b_scale[n / 128, kb] * sum_{k in block kb} A[m, k] * B[n, k]
// A [M, K], B [N, K] e4m3 codes (OCP), scales float32, one reduction block = 128 = the depth of one
// v_mfma_f32_16x16x128_f8f6f4, so every matrix instruction starts from a zero accumulator and its
// result is folded into the float32 accumulator with one scaled FMA per register.
//
// Mapping.  A workgroup of WM x WN waves owns BM rows of A ("tokens") and BN rows of B ("features").
// The features are the matrix instruction's row operand and the tokens its column operand, so a
// lane ends up with one token and 4 NT consecutive features: 16-byte stores, one activation scale
// per lane and row block.
//   * Both operands go global -> LDS with direct-to-LDS loads (global_load_lds_dwordx4: no staging
//     registers, no ds_write) -> operand registers.  The global side is fully coalesced (eight lanes
//     per 128-byte row block); operand-order loads straight from global memory (one row per lane)
//     cost the texture path four times the cycles and were the bottleneck of a first version.  LDS
//     rows are 128 bytes with their 16-byte chunks XOR-swizzled by the row index (the swizzle is
//     applied on the global side: which chunk a lane fetches), a ring of NS buffers (two in every
//     compiled variant), one barrier per reduction block; every wave waits for its own loads of the
//     next block (vmcnt) before that barrier.
//   * The order of the 128 reduction indices inside an instruction is free as long as both
//     operands use the same one: lane group j takes bytes [16 j, +16) and [64 + 16 j, +16) of a row.
//   * The activation scales of a block travel through LDS with the tile (one 4-byte direct-to-LDS
//     load per token).
//   * Split reduction: blockIdx also selects a range of reduction blocks; split i writes plane i
//     of a float32 buffer and a second kernel adds the planes in order and rounds once.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "fp8_gemm.hpp"

namespace fp8 {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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

// Workgroup = WM x WN waves; wave (wm, wn) owns tokens [16 MT wm, 16 MT (wm + 1)) and features
// [16 NT wn, 16 NT (wn + 1)) of the BM x BN tile (BM = 16 MT WM, BN = 16 NT WN).
template <int WM, int WN, int MT, int NT, int NS>
struct Geom {
  static constexpr int T = 64 * WM * WN;                 // threads
  static constexpr int BM = 16 * MT * WM, BN = 16 * NT * WN;
  static constexpr int RPP = T / 8;                      // tile rows one pass of the workgroup loads
  static constexpr int AROWS = (BM + RPP - 1) / RPP * RPP;   // activation rows held in LDS (padded to whole passes)
  static constexpr int CHA = AROWS / RPP, CHB = BN / RPP;    // 16-byte chunks per thread and block
  static constexpr int SCALES = T;                          // activation-scale slots: one per thread (slots past BM repeat the last row)
  static constexpr int STAGE = (AROWS + BN) * 128 + SCALES * 4;  // bytes: A rows, B rows, activation scales
  static constexpr int LDS = NS * STAGE;                    // NS buffers: NS - 1 blocks in flight
  static constexpr int LPB = CHA + CHB + 1;                 // vector-memory loads per wave and block
  static_assert(BM <= T, "one activation scale per thread");
  static_assert(LPB * (NS - 2) <= 63, "vmcnt is six bits");
  static_assert(BN % RPP == 0, "feature tile must be whole passes");
};

template <int WM, int WN, int MT, int NT, int NS>
__global__ void __launch_bounds__(64 * WM * WN, (WM * WN == 4 && MT * NT <= 16 ? 2 : 1))
fp8_blockwise_gemm_kernel(const GemmParams p) {
  using G = Geom<WM, WN, MT, NT, NS>;
  constexpr int T = G::T, BM = G::BM, BN = G::BN, RPP = G::RPP, AROWS = G::AROWS, CHA = G::CHA, CHB = G::CHB;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave - wm * WN;
  const int ln = lane & 15, lj = lane >> 4;

  // hardware block id -> logical tile: consecutive ids go round the 8 XCDs, so give every XCD a
  // contiguous range of tiles.  The grouped launch is sized for the bucketing capacity; its ranges
  // are cut over the row blocks that really exist (num_padded), so the unused capacity does not
  // leave the last XCDs without work, and the surplus workgroups exit here.
  const bool grouped = p.sorted_slot_ids != nullptr;
  const int n_blocks = p.N / BN;
  const int m_blocks = grouped ? *p.num_padded / BM : (p.M + BM - 1) / BM;
  const int total = grouped ? m_blocks * n_blocks : (int)gridDim.x;
  int L;
  {
    const int id = blockIdx.x, q = total >> 3, r = total & 7, x = id & 7, idx = id >> 3;
    if (idx >= q + (x < r ? 1 : 0)) return;       // (uniform over the workgroup: nobody reaches a barrier)
    L = x * q + (x < r ? x : r) + idx;
  }
  const int split = L / (m_blocks * n_blocks);
  L -= split * (m_blocks * n_blocks);
  // inside a split, tiles are walked in groups of group_m row blocks: feature block by feature block
  // inside a group, so the workgroups that run together share both their A rows and their B rows
  const int per_group = p.group_m * n_blocks;
  const int grp = L / per_group;
  const int rem = L - grp * per_group;
  int m_in = m_blocks - grp * p.group_m;
  if (m_in > p.group_m) m_in = p.group_m;
  const int nb = rem / m_in, mb = grp * p.group_m + (rem - nb * m_in);
  const int row0 = mb * BM;                       // first token of the tile
  const int n0 = nb * BN;                         // first feature of the tile
  const int KB = p.K >> 7;
  const int kb0 = split * p.kb_per_split;
  int kb1 = kb0 + p.kb_per_split;
  if (kb1 > KB) kb1 = KB;
  const int nkb = kb1 - kb0;                      // >= 1 by construction of the grid

  // ---- global -> LDS: direct-to-LDS loads (no staging registers, no ds_write) ----
  // LDS row r keeps its chunk c at position c ^ (r & 7): the operand reads below (16 rows, one
  // chunk position per lane group) then touch every bank group once.  One load instruction of a
  // wave fills 1 KiB of LDS in lane order = 8 rows x 8 positions; the lane at position s of row r
  // therefore fetches chunk s ^ (r & 7) of that row.  Pass i of the workgroup covers tile rows
  // [RPP i, RPP (i + 1)), wave w rows 8 w .. 8 w + 7 of the pass.
  const int srow = tid >> 3, sc = tid & 7;
  const uint8_t* Bmat = p.B;
  const float* bsmat = p.b_scale;
  if (grouped) {
    // row blocks past the bucketed slots, and blocks without an expert, have nothing to do
    // (uniform over the workgroup: nobody reaches a barrier)
    if (row0 >= *p.num_padded) return;
    const int e = p.block_expert_ids[mb];
    if (e < 0) return;
    Bmat += (size_t)e * p.b_expert_stride;
    bsmat += (size_t)e * p.bs_expert_stride;
  }
  // A row behind a tile row: dense = the row itself (rows past the matrix repeat its last row and
  // are never stored); grouped = slot / row_div (padding rows read row 0)
  auto a_row_of = [&](int r) __attribute__((always_inline)) -> int {
    if (grouped) {
      const int slot = p.sorted_slot_ids[row0 + r];
      return (slot >= 0 && slot < p.num_slots) ? slot / p.row_div : 0;
    }
    const int g = row0 + r;
    return g >= p.M ? p.M - 1 : g;
  };
  uint32_t aoff[CHA], boff[CHB];                  // byte offsets from A / B (host checks they fit 32 bits)
#pragma unroll
  for (int i = 0; i < CHA; ++i) {
    int r = srow + RPP * i;
    if (r >= BM) r = BM - 1;                      // LDS rows past the token tile (padding of the pass) repeat its last row
    aoff[i] = (uint32_t)a_row_of(r) * (uint32_t)p.K + 16u * (sc ^ (srow & 7));
  }
#pragma unroll
  for (int i = 0; i < CHB; ++i) boff[i] = (uint32_t)(n0 + srow + RPP * i) * (uint32_t)p.K + 16u * (sc ^ (srow & 7));
  // activation scale of tile row tid (threads past BM repeat the last row)
  const float* assrc = p.a_scale + (size_t)a_row_of(tid < BM ? tid : BM - 1) * KB;
  const float* bssrc = bsmat + (size_t)((n0 + wn * 16 * NT) >> 7) * KB;      // wave-uniform

  // ---- operand read positions ----
  // features: operand row ln of sub-tile nt is feature 4 NT (ln >> 2) + 4 nt + (ln & 3) of the wave's
  // range, so that a lane ends up with 4 NT consecutive features of its token
  const int xrow = wm * 16 * MT + ln;             // + 16 mt
  const int xpos = 16 * (lj ^ (ln & 7));          // tile rows are multiples of 16 apart: (row & 7) == (ln & 7)
  // sub-tile nt: rows 4 nt further down; (row & 7) changes by 4 (nt & 1), i.e. the position flips by 64
  const int wr0 = wn * 16 * NT + 4 * NT * (ln >> 2) + (ln & 3);
  const int wpos0 = (AROWS + wr0) * 128 + 16 * (lj ^ (wr0 & 7));
  static_assert(NT == 1 || (4 * NT) % 8 == 0, "the swizzle of the feature rows assumes 4 NT % 8 == 0");

  f32x4 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

  float sb[NS];               // weight-block scale of the block in each LDS buffer

  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  auto dma_block = [&](int buf, int kb) __attribute__((always_inline)) {
    const uint8_t* ab = p.A + (size_t)kb * 128;
    const uint8_t* bb = Bmat + (size_t)kb * 128;
    unsigned char* st = lds + buf * G::STAGE + 1024 * wave;            // this wave's 8 rows of every pass
#pragma unroll
    for (int i = 0; i < CHB; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(bb + boff[i]), (lptr_t)(st + (AROWS + RPP * i) * 128), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < CHA; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(ab + aoff[i]), (lptr_t)(st + RPP * i * 128), 16, 0, 0);
    __builtin_amdgcn_global_load_lds((gptr_t)(assrc + kb),
                                     (lptr_t)(lds + buf * G::STAGE + (AROWS + BN) * 128 + 256 * wave), 4, 0, 0);
    sb[buf] = bssrc[kb];
  };
  auto read_op = [&](const unsigned char* st, int off) __attribute__((always_inline)) -> i32x8 {
    // chunk positions c and c ^ 4 of the row: reduction indices [16 lj, +16) and [64 + 16 lj, +16)
    const i32x4 lo = *reinterpret_cast<const i32x4*>(st + off);
    const i32x4 hi = *reinterpret_cast<const i32x4*>(st + (off ^ 64));
    return i32x8{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
  };
  i32x8 wa[NT];
  float sp[MT];                // a_scale * b_scale of the lane's token in every row block
  auto read_w = [&](int ring) __attribute__((always_inline)) {
    const unsigned char* st = lds + ring * G::STAGE;
    const float* ss = reinterpret_cast<const float*>(st + (AROWS + BN) * 128) + xrow;
    const float bs = sb[ring];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) sp[mt] = ss[16 * mt] * bs;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) wa[nt] = read_op(st, (wpos0 + 512 * nt) ^ (64 * (nt & 1)));
  };
  // row blocks [MLO, MHI) of the tile against the wave's NT weight operands
  auto compute = [&](int ring, auto mlo, auto mhi) __attribute__((always_inline)) {
    constexpr int MLO = decltype(mlo)::value, MHI = decltype(mhi)::value;
    const unsigned char* st = lds + ring * G::STAGE;
    // software pipeline: the activation operand of row block mt + 1 is read from LDS, and the
    // partial sums of row block mt - 1 are folded into the accumulators, while row block mt is
    // in the matrix unit
    i32x8 xa = read_op(st, (xrow + 16 * MLO) * 128 + xpos);
    f32x4 pprev[NT];
#pragma unroll
    for (int mt = MLO; mt < MHI; ++mt) {
      i32x8 xn = xa;
      if (mt + 1 < MHI) xn = read_op(st, (xrow + 16 * (mt + 1)) * 128 + xpos);
      f32x4 part[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        part[nt] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
            wa[nt], xa, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);   // e4m3 x e4m3, no block exponents
      if (mt > MLO) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt - 1][nt] += pprev[nt] * sp[mt - 1];
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) pprev[nt] = part[nt];
      xa = xn;
      // Instruction order.  Left to itself the scheduler gathers every FMA of the block at its
      // end, which keeps all partial sums alive.  An empty asm that takes the accumulators just
      // updated and the next activation operand ties them together: the matrix instructions of
      // row block mt + 1 cannot start before the FMAs of row block mt - 1 are done.
      if (mt > MLO) {
        if constexpr (NT == 4)
          asm volatile("" : "+v"(acc[mt - 1][0]), "+v"(acc[mt - 1][1]), "+v"(acc[mt - 1][2]), "+v"(acc[mt - 1][3]), "+v"(xa));
        else if constexpr (NT == 2)
          asm volatile("" : "+v"(acc[mt - 1][0]), "+v"(acc[mt - 1][1]), "+v"(xa));
        else
          asm volatile("" : "+v"(acc[mt - 1][0]), "+v"(xa));
      }
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[MHI - 1][nt] += pprev[nt] * sp[MHI - 1];
  };
  using std::integral_constant;
  // vmcnt(n): at most n of this wave's vector-memory loads still in flight (six bits, split 4 + 2)
  constexpr int kLanded = ((G::LPB * (NS - 2)) & 15) | (((G::LPB * (NS - 2)) >> 4) << 14) | 0x0F70;
  // One block.  Buffer cur is multiplied; the block NS - 1 ahead is sent to the buffer that was
  // multiplied last (every wave is past the barrier that followed it); before the closing barrier
  // each wave waits until its own part of the NEXT block has landed.
  auto stage = [&](auto cur_c, int kb_far) __attribute__((always_inline)) {
    constexpr int cur = decltype(cur_c)::value;
    read_w(cur);
    __builtin_amdgcn_sched_barrier(0);       // the LDS reads above are issued before the far block's loads
    dma_block((cur + NS - 1) % NS, kb_far);
    __builtin_amdgcn_sched_barrier(0);
    compute(cur, integral_constant<int, 0>{}, integral_constant<int, MT>{});
    __builtin_amdgcn_s_waitcnt(kLanded);
    __syncthreads();
  };

  // ---- pipeline: NS - 1 blocks in flight while one is multiplied ----
  // (block indices past the end are clamped: a valid block is loaded and never consumed, so every
  // wave issues the same number of loads per stage and the vmcnt arithmetic holds)
  auto clampk = [&](int i) __attribute__((always_inline)) { return kb0 + (i < nkb ? i : nkb - 1); };
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) dma_block(s, clampk(s));
  __builtin_amdgcn_s_waitcnt(kLanded);
  __syncthreads();
  for (int it = 0; it < nkb; it += NS) {
    stage(integral_constant<int, 0>{}, clampk(it + NS - 1));
    if constexpr (NS >= 2) { if (it + 1 < nkb) stage(integral_constant<int, 1>{}, clampk(it + NS)); }
    if constexpr (NS >= 3) { if (it + 2 < nkb) stage(integral_constant<int, 2>{}, clampk(it + NS + 1)); }
    if constexpr (NS >= 4) { if (it + 3 < nkb) stage(integral_constant<int, 3>{}, clampk(it + NS + 2)); }
  }

  // ---- epilogue: the lane's token, 4 NT consecutive features ----
  const int f0 = n0 + wn * 16 * NT + 4 * NT * lj;
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    int t = row0 + xrow + 16 * mt;               // dense: the token; grouped: the slot behind the tile row
    if (grouped) {
      t = p.sorted_slot_ids[t];
      if (t < 0 || t >= p.num_slots) continue;   // padding row
    } else if (t >= p.M) {
      continue;
    }
    if (p.k_splits > 1 || p.out_bf16 == 2) {     // float32: a partial plane, or the result itself
      float* dst = reinterpret_cast<float*>(p.C) + ((size_t)split * p.M + t) * p.N + f0;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) *reinterpret_cast<f32x4*>(dst + 4 * nt) = acc[mt][nt];
    } else {
      uint16_t* dst = reinterpret_cast<uint16_t*>(p.C) + (size_t)t * p.N + f0;
      uint32_t w[2 * NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        if (p.out_bf16 == 1) {
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
fp8_split_reduce_kernel(const f32x4* __restrict__ planes, int k_splits, long long n4, void* __restrict__ C,
                        int out_type) {
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n4; i += (long long)gridDim.x * 256) {
    f32x4 s = planes[i];
    for (int k = 1; k < k_splits; ++k) s += planes[(long long)k * n4 + i];
    if (out_type == 2) reinterpret_cast<f32x4*>(C)[i] = s;
    else
      reinterpret_cast<u32x2*>(C)[i] = out_type == 1 ? u32x2{pack2<1>(s[0], s[1]), pack2<1>(s[2], s[3])}
                                                     : u32x2{pack2<0>(s[0], s[1]), pack2<0>(s[2], s[3])};
  }
}

template <int WM, int WN, int MT, int NT, int NS>
static int launch_one(const GemmParams& p, hipStream_t stream) {
  using G = Geom<WM, WN, MT, NT, NS>;
  auto kern = fp8_blockwise_gemm_kernel<WM, WN, MT, NT, NS>;
  if (G::LDS > 64 * 1024) {
    // raise the dynamic LDS limit of this kernel once per device
    constexpr int kMaxDev = 64;
    static bool allowed[kMaxDev] = {};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return (int)err;
    if (dev < 0 || dev >= kMaxDev || !allowed[dev]) {
      err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                G::LDS);
      if (err != hipSuccess) return (int)err;
      if (dev >= 0 && dev < kMaxDev) allowed[dev] = true;
    }
  }
  const int grid = ((p.M + G::BM - 1) / G::BM) * (p.N / G::BN) * p.k_splits;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(G::T), G::LDS, stream, p);
  return (int)hipGetLastError();
}

// Tiles.  bm = tokens per workgroup in {16, 32, 64, 128, 256}, bn = features per workgroup in
// {64, 128, 256}; bm = 256 runs eight waves (2 x 4), everything else four (1 x 4).  Returns a
// hipError_t, or -1 for an unknown tile.  Measured and not compiled in: three LDS buffers (two
// blocks in flight: no gain on the small tiles, -30 % on 128 x 128 where it costs the second
// workgroup per CU) and the non-temporal cache policy on the weight loads (-18 % on streaming
// shapes).
int launch_fp8_gemm(const GemmParams& p, int bm, int bn, hipStream_t stream) {
#define FP8_TILE(BMv, BNv, WMv, WNv, MTv, NTv, NSv)                                   \
  if (bm == BMv && bn == BNv) return launch_one<WMv, WNv, MTv, NTv, NSv>(p, stream);
  FP8_TILE(16, 64, 1, 4, 1, 1, 2)   FP8_TILE(16, 128, 1, 4, 1, 2, 2)   FP8_TILE(16, 256, 1, 4, 1, 4, 2)
  FP8_TILE(32, 64, 1, 4, 2, 1, 2)   FP8_TILE(32, 128, 1, 4, 2, 2, 2)   FP8_TILE(32, 256, 1, 4, 2, 4, 2)
  FP8_TILE(64, 64, 1, 4, 4, 1, 2)   FP8_TILE(64, 128, 1, 4, 4, 2, 2)   FP8_TILE(64, 256, 1, 4, 4, 4, 2)
  FP8_TILE(128, 64, 1, 4, 8, 1, 2)  FP8_TILE(128, 128, 1, 4, 8, 2, 2)  FP8_TILE(128, 256, 1, 4, 8, 4, 2)
  FP8_TILE(256, 256, 2, 4, 8, 4, 2) FP8_TILE(256, 128, 2, 4, 8, 2, 2)
#undef FP8_TILE
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
                     k_splits, n4, C, out_bf16);
  return (int)hipGetLastError();
}

}  // namespace fp8
