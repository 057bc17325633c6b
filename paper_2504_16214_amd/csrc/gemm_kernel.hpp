// Grouped W4A16 GEMM for gfx950 (MI355X): C[s, :] = A[s / row_div, :] . dequant(W[expert(s)])^T
//
// Dataflow (the efficient one of the paper's Fig. 4(b), Section II-C, re-cut for CDNA4):
//   packed int4 weights  : global --128-bit coalesced loads--> VGPR --> wave-private LDS tile
//                          --ds_read (one lane = one MFMA operand column)--> VGPR
//                          --in-register nibble unpack to the exact integers q - z--> MFMA B operand
//                          (the group scale multiplies the fp32 partial sum of each chunk-step)
//   activations          : global --128-bit loads--> VGPR --> shared LDS tile (padded rows)
//                          --ds_read_b128--> MFMA A operand
//   scales / zero points : staged once per workgroup into LDS, one 32-bit entry per (group, row)
// Weights never travel register -> LDS -> register after the cast; every hop of A, B, scale
// and zp is a wide vector access (Table III).
//
// Work decomposition.  A workgroup (256 threads = 4 wavefronts of 64) owns a tile of
// M_T = 16*MT bucketed slots of one expert and N_T = 64*NT output features.  Wave w owns
// features [w*16*NT, (w+1)*16*NT) of the tile for all M_T slots, so each packed weight is
// unpacked exactly once per workgroup and the wave's weight tile in LDS is private to it
// (no barrier on the weight path).  The activation tile is shared by the four waves.
//
// MFMA mapping (v_mfma_f32_16x16x32_{f16,bf16}): tokens on the M side, output features on
// the N side.  Lane l holds for A: row l%16, k-slots 8*(l/16)..+7; for B: column l%16, same
// k-slots; for the 16x16 result: rows 4*(l/16)..+3, column l%16.
//
// Reduction-index permutation.  Summation order over k is free, so one chunk-step of
// CK = 32*KW reduction indices feeds KW MFMAs like this: lane (n, j) reads KW consecutive
// packed words (8*KW k's starting at CK*u + 8*KW*j); word i goes to MFMA i.  MFMA i thus
// contracts k = CK*u + 8*KW*j + 8*i + e (j = 0..3, e = 0..7); the A operand is read at the
// same k's.  Inside a word the nibble pairs come out as (e, e+4), so the A tile is stored in
// LDS with each run of 8 elements reordered to 0,4,1,5,2,6,3,7.  KW is chosen so that one
// chunk-step never straddles a quantisation group (group % CK == 0).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

namespace moe {

struct GemmParams {
  const void* A;
  int row_div;
  const int32_t* qweight;
  const void* scales;
  const uint8_t* zeros;
  const int32_t* sorted_slot_ids;
  const int32_t* block_expert_ids;
  const int32_t* num_padded;
  int num_slots, E, N_out, K_in, group, block_m;
  void* C;
  int ldc;
  int n_tiles;    // workgroups along the feature dimension
  int G;          // K_in / group
  int cpg;        // chunk-steps per quantisation group = group / (32*KW)
  int half_n;     // fused SiLU-and-multiply: N (weight rows [0,N) gate, [N,2N) up); else 0
  int sz_vec;     // 1 if scale rows are 16-byte aligned (G % 8 == 0 and aligned base pointers)
  int out_f32;    // 1: C is float32 (the layer's down projection feeds the combine unrounded)
  int k_splits;   // > 1: the reduction is cut into k_splits ranges of k_span indices, one workgroup each;
  int k_span;     //      split i writes its partial sums to the float32 plane C + i * split_stride
  long long split_stride;   // elements between planes (register-scale kernels with out_f32 only)
  int dense;      // 1: no routing tables (all three pointers null): one expert, slot s = row s of A and C
  int tiles_per_wg;  // consecutive feature tiles one workgroup walks (1 unless SZR)
};

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx4_t __attribute__((ext_vector_type(4)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));
// native 128-bit / 64-bit register vectors (not HIP's struct-based u32x4: these stay in VGPRs)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kF16 = 0, kBF16 = 1;

template <int DT>
__device__ __forceinline__ floatx4_t mfma16x16x32(const u32x4& a, const u32x4& b, floatx4_t c) {
  if constexpr (DT == kF16) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a),
                                                  __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
  }
}

// ---- int4 -> 16-bit float, in registers ---------------------------------------------------
// The MFMA never sees a rounded weight.  Two ways of removing the zero point, chosen by ZM:
//
//   ZM = 1 (bf16, which has no packed arithmetic): the B operand holds the BIASED integers
//     bias + q, produced by one AND-OR per nibble pair; a second MFMA with the constant operand
//     -(bias + z) subtracts bias and zero point inside the fp32 accumulation.
//   ZM = 0 (fp16): one packed subtract per nibble pair yields the exact integers q - z.
// Either way the group scale is applied in fp32 (to the partial sum of a chunk-step, or by
// keeping the accumulator in units of the current group's scale: see RS in the kernel).
//
// fp16: nibbles 0/4 of a word are ORed into the mantissa of 1024.0 (ulp 1: value 1024 + q);
//       nibbles 1/5 sit four bits higher and are ORed into the mantissa of 64.0 (ulp 1/16,
//       value 64 + q), which saves the shift.  One shift by 8 brings nibbles 2/6 and 3/7 into
//       the same two positions.  5 VALU ops per 8 weights.
// bf16: 7 mantissa bits only: every pair is shifted down and ORed into 128.0 (value 128 + q).
//
// LDS entry per (group, feature row): fp16: hi = fp16 bits of 1024 + z (sign set when ZM),
// lo = scale bits.  bf16: hi = scale bits, lo = z.
// (a & mask) | orv in one VALU op.  v_and_or_b32 is a VOP3 instruction and on gfx9-class
// encodings VOP3 takes no literal and only one scalar operand, so the compiler only selects it
// when one of the two constants already lives in a VGPR.  The OR patterns are therefore handed
// in as VGPR values made opaque once at kernel start (vgpr_const); the selection and all MFMA
// hazard bookkeeping stay with the compiler (no inline asm near the MFMAs).
__device__ __forceinline__ uint32_t vgpr_const(uint32_t v) {
  uint32_t d;
  asm volatile("v_mov_b32 %0, %1" : "=v"(d) : "s"(v));
  return d;
}
struct UnpackConsts {
  uint32_t or_hi;   // fp16: 0x64006400 (1024.0 pair)   bf16: 0x43004300 (128.0 pair)
  uint32_t or_lo;   // fp16: 0x54005400 (64.0 pair)     bf16: 0xC300C300 (-128.0 pair, zero-point operand)
};

template <int DT, int ZM>
__device__ __forceinline__ uint32_t pack_sz_entry(uint16_t scale_bits, uint8_t z) {
  if constexpr (DT == kF16) return (((ZM ? 0xE400u : 0x6400u) | (uint32_t)z) << 16) | (uint32_t)scale_bits;
  else return ((uint32_t)scale_bits << 16) | (uint32_t)z;
}

template <int DT, int ZM>
struct DeqCtx;
template <int ZM>
struct DeqCtx<kF16, ZM> {
  uint32_t zA, zB;   // packed pairs: (-)(1024 + z) and (-)(64 + z)
  float s;
  DeqCtx() = default;
  // Straight from the register-resident panel: zreg holds the zero points of four groups (one
  // per byte), z4reg the same shifted left by four, sreg two fp16 scales.  One byte permute per
  // constant: byte gq of zreg under the exponent byte of 1024.0 (or of 64.0, mantissa bits 4..7).
  // (gp is a constant after unrolling, so the selector is a scalar literal.)
  __device__ __forceinline__ static DeqCtx from_panel(int gp, uint32_t sreg, uint32_t zreg, uint32_t z4reg,
                                                      const UnpackConsts& k) {
    static_assert(ZM == 0, "fp16 uses the packed subtract");
    const uint32_t sel = 0x05000500u | ((uint32_t)(gp & 3) << 16) | (uint32_t)(gp & 3);
    DeqCtx c;
    c.zA = __builtin_amdgcn_perm(k.or_hi, zreg, sel);
    c.zB = __builtin_amdgcn_perm(k.or_lo, z4reg, sel);
    c.s = (float)__builtin_bit_cast(_Float16, (uint16_t)((gp & 1) ? (sreg >> 16) : (sreg & 0xffffu)));
    return c;
  }
  __device__ __forceinline__ uint32_t zero_point() const { return zA & 0xfu; }
  __device__ __forceinline__ explicit DeqCtx(uint32_t e) {
    zA = __builtin_amdgcn_perm(e, e, 0x07060706u);                       // (hi16, hi16)
    zB = ((zA & 0x000F000Fu) << 4) | (ZM ? 0xD400D400u : 0x54005400u);   // z moved to mantissa bits 4..7
    s = (float)__builtin_bit_cast(_Float16, (uint16_t)(e & 0xffffu));
  }
  // constant B operand of the zero-point MFMA (ZM only)
  __device__ __forceinline__ u32x4 zoperand() const { return u32x4{zA, zB, zA, zB}; }
};
template <int ZM>
struct DeqCtx<kBF16, ZM> {
  uint32_t zA;       // ZM: packed pair -(128 + z) as bf16
  float zc, s;
  DeqCtx() = default;
  __device__ __forceinline__ static DeqCtx from_panel(int gp, uint32_t sreg, uint32_t zreg, uint32_t /*z4reg*/,
                                                      const UnpackConsts& k) {
    const uint32_t sel = 0x05000500u | ((uint32_t)(gp & 3) << 16) | (uint32_t)(gp & 3);
    DeqCtx c;
    c.zA = __builtin_amdgcn_perm(k.or_lo, zreg, sel);       // or_lo = 0xC300C300: -(128 + z) pairs
    c.zc = 128.0f + (float)((zreg >> (8 * (gp & 3))) & 0xffu);
    c.s = __builtin_bit_cast(float, (gp & 1) ? (sreg & 0xffff0000u) : (sreg << 16));
    return c;
  }
  __device__ __forceinline__ uint32_t zero_point() const { return zA & 0xfu; }
  __device__ __forceinline__ explicit DeqCtx(uint32_t e) {
    s = __builtin_bit_cast(float, e & 0xffff0000u);
    zc = 128.0f + (float)(e & 0xffu);
    zA = ((e & 0xffu) * 0x10001u) | 0xC300C300u;
  }
  __device__ __forceinline__ u32x4 zoperand() const { return u32x4{zA, zA, zA, zA}; }
};

// One packed word (8 nibbles) -> 8 sixteen-bit floats in the order 0,4,1,5,2,6,3,7:
// biased integers (ZM) or exact q - z (not ZM).
template <int DT, int ZM>
__device__ __forceinline__ u32x4 dequant_word(uint32_t w, const DeqCtx<DT, ZM>& c, const UnpackConsts& k) {
  uint32_t r[4];
  if constexpr (DT == kF16) {
    const uint32_t w8 = w >> 8;
    r[0] = (w & 0x000F000Fu) | k.or_hi;
    r[1] = (w & 0x00F000F0u) | k.or_lo;
    r[2] = (w8 & 0x000F000Fu) | k.or_hi;
    r[3] = (w8 & 0x00F000F0u) | k.or_lo;
    if constexpr (!ZM) {
      const half2_t zA = __builtin_bit_cast(half2_t, c.zA), zB = __builtin_bit_cast(half2_t, c.zB);
      r[0] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, r[0]) - zA);
      r[1] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, r[1]) - zB);
      r[2] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, r[2]) - zA);
      r[3] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, r[3]) - zB);
    }
  } else {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const uint32_t t = ((w >> (4 * p)) & 0x000F000Fu) | k.or_hi;
      if constexpr (ZM) {
        r[p] = t;
      } else {
        const float lo = __builtin_bit_cast(float, t << 16);
        const float hi = __builtin_bit_cast(float, t & 0xffff0000u);
        floatx2_t f = {lo - c.zc, hi - c.zc};
        r[p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
      }
    }
  }
  return u32x4{r[0], r[1], r[2], r[3]};
}

template <int DT>
__device__ __forceinline__ uint16_t to_bits16(float v) {
  if constexpr (DT == kF16) return __builtin_bit_cast(uint16_t, (_Float16)v);
  else return __builtin_bit_cast(uint16_t, (__bf16)v);
}
template <int DT>
__device__ __forceinline__ float from_bits16(uint16_t b) {
  if constexpr (DT == kF16) return (float)__builtin_bit_cast(_Float16, b);
  else return __builtin_bit_cast(float, (uint32_t)b << 16);
}

__device__ __forceinline__ float silu_f32(float x) { return x / (1.0f + __expf(-x)); }

// 8 consecutive 16-bit elements x0..x7 -> order x0,x4,x1,x5,x2,x6,x3,x7
__device__ __forceinline__ u32x4 interleave8(const u32x4& a) {
  u32x4 o;
  o.x = __builtin_amdgcn_perm(a.z, a.x, 0x05040100u);  // (x0, x4)
  o.y = __builtin_amdgcn_perm(a.z, a.x, 0x07060302u);  // (x1, x5)
  o.z = __builtin_amdgcn_perm(a.w, a.y, 0x05040100u);  // (x2, x6)
  o.w = __builtin_amdgcn_perm(a.w, a.y, 0x07060302u);  // (x3, x7)
  return o;
}

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Map the hardware
// block id to a logical tile index so that every XCD walks a contiguous range of tiles:
// tiles that share an activation tile (same slot block, neighbouring feature tiles) or the
// same expert's weights (neighbouring slot blocks) then meet in one L2.  `total` is the number
// of tiles that really exist (known on the device only: it follows from num_padded); the
// launch grid covers the worst case.  Returns -1 for a workgroup with nothing to do.  Every
// XCD gets total/8 tiles (+1 for the first total%8), so unused block capacity does not idle
// whole XCDs.
__device__ __forceinline__ int xcd_contiguous_index(int pid, int total) {
  const int xcd = pid & 7, idx = pid >> 3;
  const int per = total >> 3, rem = total & 7;
  if (idx >= per + (xcd < rem ? 1 : 0)) return -1;
  return xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
}

// Packed weights: streamed once per launch in the small-token regime (non-temporal, so they
// do not displace the activation tiles in L2); with large token tiles the same expert rows are
// read again by the neighbouring slot blocks and should stay cached.
template <bool STREAM>
__device__ __forceinline__ u32x4 load_weights(const unsigned char* p) {
  if constexpr (STREAM) return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  else return *reinterpret_cast<const u32x4*>(p);
}

template <int KW>
struct WordVec;
template <>
struct WordVec<1> { uint32_t w[1]; };
template <>
struct WordVec<2> { uint32_t w[2]; };
template <>
struct WordVec<4> { uint32_t w[4]; };

template <int KW>
__device__ __forceinline__ WordVec<KW> lds_read_words(const unsigned char* p) {
  WordVec<KW> v;
  if constexpr (KW == 4) {
    u32x4 t = *reinterpret_cast<const u32x4*>(p);
    v.w[0] = t.x; v.w[1] = t.y; v.w[2] = t.z; v.w[3] = t.w;
  } else if constexpr (KW == 2) {
    u32x2 t = *reinterpret_cast<const u32x2*>(p);
    v.w[0] = t.x; v.w[1] = t.y;
  } else {
    v.w[0] = *reinterpret_cast<const uint32_t*>(p);
  }
  return v;
}

// LDS row padding.  Measured with a 128-bit read microbenchmark: a lane (n, j) reading row n at
// 16-byte chunk j runs at full rate when the row pitch is 2 mod 4 chunks (6, 10) and 1.35x slower
// at the odd pitches 5 and 9.  The activation tile is read the same way (row n, chunk j + 4i for
// the i-th MFMA of a chunk-step), which is why its chunks are stored transposed inside each
// chunk-step (chunk KW*j + i at position j + 4*i): with the natural order (chunk 4j + i) no
// pitch gets rid of the 1.35x.  (End to end the effect is within run-to-run noise: LDS time is a
// few percent of the kernel.)
constexpr int kXRowPad = 32;
constexpr int kWRowPad(int ks) { return ks >= 512 ? 16 : 32; }   // 512-k stages: LDS room for three workgroups
// activation tile buffers in LDS per token-tile size (see TileGeom::XBUFS)
constexpr int kXBufs(int mt, int ks, int wv = 4) { return wv == 8 ? 3 : (mt == 2 || ks >= 512) ? 1 : 2; }

template <int MT, int NT, int KS, int WV = 4>
struct TileGeom {
  static constexpr int THREADS = 64 * WV;    // WV wavefronts per workgroup (4, or 8 for the widest tiles)
  static constexpr int M_T = 16 * MT;        // slots per workgroup tile
  static constexpr int NW = 16 * NT;         // features per wave
  static constexpr int N_T = WV * NW;        // features per workgroup
  static constexpr int XP = KS * 2 + kXRowPad;   // LDS bytes per activation row (padded)
  static constexpr int WP = KS / 2 + kWRowPad(KS);   // LDS bytes per packed weight row (padded)
  static constexpr int CPR = KS / 8;         // 16-byte chunks per activation row
  static constexpr int RPP = THREADS / CPR;  // activation rows per cooperative pass
  static constexpr int XPASS = M_T / RPP;    // passes per stage
  static constexpr int LPR = KS / 32;        // lanes covering one weight row (16 B each)
  static constexpr int RPI = 64 / LPR;       // weight rows per wave load instruction
  static constexpr int WPASS = NW / RPI;     // weight load instructions per stage per wave
  static_assert(XPASS >= 1 && WPASS >= 1, "tile too small for the load mapping");
  // Activation tile buffers: two (one barrier per stage) except for 32-slot tiles, where a single
  // buffer (two barriers per stage) is what lets a third workgroup fit on a CU, and for the
  // eight-wave tile, whose skewed pipeline rotates three.
  static constexpr int XBUFS = kXBufs(MT, KS, WV);
  static size_t lds_bytes(int G, int szr, int pre = 0) {
    return (size_t)XBUFS * M_T * XP + (pre ? 0 : (size_t)WV * NW * WP) + (szr ? 0 : (size_t)G * N_T * 4) +
           (size_t)M_T * 4;
  }
};

// Local feature index of a workgroup tile -> weight row / output column.
//   plain : weight row = output column = feature f of the tile.  A wave's sub-tiles are
//           interleaved in pairs (sub-tile 2p takes the even, 2p+1 the odd features of a run of
//           32), so a lane owns two ADJACENT output columns per pair and stores them with one
//           instruction: full 128-byte lines per row for float32 output.
//   fused SiLU-and-multiply: wave-local sub-tiles alternate gate, up; the pair (2p, 2p+1)
//   covers act columns c..c+15 with weight rows c (gate) and N + c (up).
template <int NT, int FUSE, int WV = 4>
__device__ __forceinline__ void feature_of(int n_tile, int wave, int sub, int n, const GemmParams& p,
                                           int& wrow, int& ocol, bool& valid) {
  constexpr int NW = 16 * NT, N_T = WV * NW;
  if constexpr (FUSE == 0) {
    const int f = NT == 1 ? n_tile * N_T + wave * NW + n
                          : n_tile * N_T + wave * NW + (sub >> 1) * 32 + 2 * n + (sub & 1);
    wrow = f; ocol = f; valid = f < p.N_out;
  } else {
    const int c = n_tile * (N_T / 2) + wave * (NW / 2) + (sub >> 1) * 16 + n;
    wrow = (sub & 1) * p.half_n + c; ocol = c; valid = c < p.half_n;
  }
}

// SZR = 1: scales and zero points are not staged in LDS; every lane fetches the groups of the
// current panel (4 pipeline stages: 8 groups for KS = 256, 4 for KS = 128) of its own feature
// rows straight into registers, prefetched one panel ahead.  Needs group == 128 (one group per
// chunk-step, KW == 4) and 16-byte aligned scale rows (G % 8 == 0).
// It frees the largest LDS consumer of the bandwidth-bound shapes, which is what bounds the
// number of resident workgroups per CU there.
//
// PRE = 1: `qweight` is in the operand-order layout (blocks of 16 rows x 128 k stored as the 64
// lanes' 16-byte operand chunks, blocks of a row set consecutive along the reduction; row sets
// contiguous for the fused gate/up GEMM, even/odd pairs of 32 rows otherwise).  A wave then loads
// its operand words fully coalesced straight into registers: no weight tile in LDS, one per-lane
// offset (lane * 16) for every weight load.  Register-scale kernels only.
//
// PRE = 2: `qweight` is in the stated row-major layout, but a wave still loads its operand words
// straight into registers (a load instruction covers 16 rows x 64 bytes): no weight tile in LDS.
// Only for large token tiles, whose weights mostly come from L2 (the row blocks of an expert
// re-read them); from HBM this access shape is slower than 128-byte row segments.
//
// WV = 8: eight wavefronts per workgroup (two per SIMD) share one activation tile; wave w owns
// features [w*16*NT, (w+1)*16*NT) of a tile of 128*NT features.
template <int DT, int MT, int NT, int KS, int KW, int FUSE, int SZR, int PRE = 0, int WV = 4>
// Minimum workgroups per CU: two wherever the tile's registers fit 256 per lane.  Besides the
// occupancy this decides where the accumulators live: with a budget above 256 registers the
// compiler keeps them in accumulation registers, which VALU instructions cannot address, and
// every rescale of an accumulator becomes read + multiply + write back (the 64-row tile without
// register scales spent a quarter of its VALU instructions on those copies).
__global__ void __launch_bounds__(64 * WV, (WV == 8 ? 1 : ((MT * NT <= 4 || (MT * NT <= 8 && MT <= 4) || (SZR && MT <= 4) || (PRE == 2 && NT <= 2)) ? 2 : 1)))
w4a16_gemm_kernel(const GemmParams p) {
  static_assert(SZR == 0 || KW == 4, "register-resident scales need 128-k chunk-steps (group 128)");
  static_assert(PRE == 0 || (SZR == 1 && (FUSE == 1 || NT >= 2)), "operand-order weights: register-scale, paired tiles");
  static_assert(WV == 4 || (WV == 8 && SZR == 1), "eight-wave workgroups: register-scale kernels only");
  using G_ = TileGeom<MT, NT, KS, WV>;
  constexpr int THREADS = G_::THREADS;
  constexpr int M_T = G_::M_T, NW = G_::NW, N_T = G_::N_T, XP = G_::XP, WP = G_::WP;
  constexpr int CPR = G_::CPR, RPP = G_::RPP, XPASS = G_::XPASS;
  constexpr int LPR = G_::LPR, RPI = G_::RPI, WPASS = G_::WPASS;
  constexpr int CK = 32 * KW, UCH = KS / CK;
  static_assert(FUSE == 0 || NT % 2 == 0, "fused SiLU needs gate/up sub-tile pairs");
  // Zero point: fp16 subtracts bias + z with one packed op per pair (exact: integers below 2048).
  // bf16 has no packed arithmetic, the per-pair subtract would cost four times the VALU work, so
  // there the biased integers go to the MFMA and bias + z is subtracted by a second MFMA against a
  // constant operand.  (VALU and MFMA instructions of one SIMD largely serialise on this chip --
  // measured -- so for fp16 four packed ops are cheaper than one more 16-cycle MFMA.)
  constexpr int ZM = DT == kBF16 ? 1 : 0;
  // RS = 1 (large token tiles): no separate partial-sum registers.  The accumulator of feature
  // row n is kept in units of the scale of the group being processed: on entering a group with
  // scale s it is multiplied by unit/s (unit := s), the MFMAs then add the exact integer products
  // straight into it, and the epilogue multiplies by the last unit.  Costs the same one VALU op
  // per accumulator element and group as the fused multiply-add on partial sums, but halves the
  // accumulator registers, which is what lets 64x256 tiles run two workgroups per CU.  Each
  // rescale is one fp32 rounding (and a 1-ulp reciprocal): about 1e-6 relative over a row.
  // A zero scale keeps the unit and zeroes the group's operand instead.
  constexpr int RS = MT >= 4 ? 1 : 0;

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* xs = smem;                                        // [2][M_T][XP]
  constexpr int XBUFS = G_::XBUFS;
  unsigned char* ws_all = xs + XBUFS * M_T * XP;                   // [WV][NW][WP] (absent when PRE)
  uint32_t* sz = reinterpret_cast<uint32_t*>(ws_all + (PRE ? 0 : WV * NW * WP));  // [G][N_T] (absent when SZR)
  int* slot_s = reinterpret_cast<int*>(sz + (SZR ? 0 : p.G * N_T));  // [M_T]

  // A workgroup owns one block of M_T slots and `tiles_per_wg` consecutive feature tiles; it
  // walks them with one continuous load pipeline (no drain between tiles), so the fixed cost of
  // starting a workgroup is paid once per several tiles when the reduction is short.
  const int tpw = SZR ? p.tiles_per_wg : 1;
  const int tgroups = (p.n_tiles + tpw - 1) / tpw;
  const int ksp = SZR ? p.k_splits : 1;
  const int rows_padded = p.dense ? (p.num_slots + M_T - 1) / M_T * M_T : *p.num_padded;
  int L = xcd_contiguous_index(blockIdx.x, (rows_padded / M_T) * tgroups * ksp);
  if (L < 0) return;
  const int split = L % ksp;        // neighbouring workgroups take the ranges of one tile
  L /= ksp;
  const int tile0 = (L % tgroups) * tpw;
  const int ntl = p.n_tiles - tile0 < tpw ? p.n_tiles - tile0 : tpw;     // tiles this workgroup walks
  const int row0 = (L / tgroups) * M_T;
  const int e = p.dense ? 0 : p.block_expert_ids[row0 / p.block_m];
  // slot id of a tile row: from the bucketing table, or the row itself for the plain GEMM
  auto slot_at = [&](int r) __attribute__((always_inline)) { return p.dense ? (r < p.num_slots ? r : p.num_slots) : p.sorted_slot_ids[r]; };
  if (e < 0 || e >= p.E) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ln = lane & 15, lj = lane >> 4;
  UnpackConsts uk;
  uk.or_hi = vgpr_const(DT == kF16 ? 0x64006400u : 0x43004300u);
  uk.or_lo = vgpr_const(DT == kF16 ? 0x54005400u : 0xC300C300u);
  unsigned char* wsw = ws_all + wave * NW * WP;
  const int K_in = p.K_in;                          // row stride of A and of the packed weights
  // reduction range of this workgroup: [k0, k0 + K_ext); the whole row unless the launch splits it
  const int k0 = ksp > 1 ? split * p.k_span : 0;
  const int K_ext = ksp > 1 ? (K_in - k0 < p.k_span ? K_in - k0 : p.k_span) : K_in;

  // ---- per-thread global addresses ------------------------------------------------
  // Every load address is (workgroup-uniform 64-bit base) + (32-bit per-lane byte offset): the
  // stage advance is scalar arithmetic on the base and costs no VALU, and the per-lane part is
  // a single register per load.  Loads are never predicated: padding rows, feature rows past
  // N_out and reduction chunks past K_in are redirected to a valid address; what they fetch
  // only ever reaches output rows / columns that are not stored, or chunk-steps that are not
  // executed.  (The host checks that one expert's weights and the A matrix stay below 2 GiB.)
  const unsigned char* const xbase = reinterpret_cast<const unsigned char*>(p.A) + (size_t)k0 * 2;
  uint32_t xoff[XPASS];
  const int xr_row = tid / CPR, xr_chunk = tid % CPR;
  // LDS position of the thread's 16-byte chunk: transposed inside its chunk-step (4*KW chunks)
  const int xw_pos = (xr_chunk / (4 * KW)) * (4 * KW) + (xr_chunk % (4 * KW)) / KW + 4 * (xr_chunk % KW);
#pragma unroll
  for (int ps = 0; ps < XPASS; ++ps) {
    const int slot = slot_at(row0 + ps * RPP + xr_row);
    const uint32_t arow = (slot >= 0 && slot < p.num_slots) ? (uint32_t)(slot / p.row_div) : 0u;
    xoff[ps] = arow * (uint32_t)(K_in * 2) + (uint32_t)(xr_chunk * 16);
  }
  // (operand-order layout: the k0 / 128 leading blocks of a row set are 1 KiB each)
  const unsigned char* const wbase = reinterpret_cast<const unsigned char*>(p.qweight) +
                                     (size_t)e * p.N_out * (size_t)(K_in >> 1) +
                                     (PRE == 1 ? (size_t)(k0 >> 7) * 1024 : (size_t)(k0 >> 1));
  uint32_t woff[WPASS];      // rows of the tile the LOAD cursor is in
  const int wl_row = lane / LPR, wl_chunk = lane % LPR;
  auto set_w_rows = [&](int tile) __attribute__((always_inline)) {
    if constexpr (PRE == 1) {
      // load q = s * UCH + u fetches chunk-step u of the stage for sub-tile s: block of the
      // sub-tile's row set, 1 KiB per chunk-step, the lane's own 16 bytes
#pragma unroll
      for (int q = 0; q < WPASS; ++q) {
        const int sub = q / UCH;
        int wrow, ocol;
        bool ok;
        feature_of<NT, FUSE, WV>(tile, wave, sub, 0, p, wrow, ocol, ok);
        if (!ok) wrow = 0;
        const uint32_t blk = FUSE ? (uint32_t)wrow >> 4 : (((uint32_t)wrow >> 5) << 1) | (uint32_t)(sub & 1);
        woff[q] = (blk * (uint32_t)(K_in >> 7) + (uint32_t)(q % UCH)) * 1024u + (uint32_t)(lane * 16);
      }
    } else if constexpr (PRE == 2) {
      // row-major weights in operand order: lane (n, j) fetches bytes [64u + 16j, +16) of row n of sub-tile s
#pragma unroll
      for (int q = 0; q < WPASS; ++q) {
        int wrow, ocol;
        bool ok;
        feature_of<NT, FUSE, WV>(tile, wave, q / UCH, ln, p, wrow, ocol, ok);
        if (!ok) wrow = 0;
        woff[q] = (uint32_t)wrow * (uint32_t)(K_in >> 1) + (uint32_t)((q % UCH) * 64 + lj * 16);
      }
    } else {
#pragma unroll
      for (int q = 0; q < WPASS; ++q) {
        const int rw = q * RPI + wl_row;
        int wrow, ocol;
        bool ok;
        feature_of<NT, FUSE, WV>(tile, wave, rw >> 4, rw & 15, p, wrow, ocol, ok);
        if (!ok) wrow = 0;
        woff[q] = (uint32_t)wrow * (uint32_t)(K_in >> 1) + (uint32_t)(wl_chunk * 16);
      }
    }
  };
  set_w_rows(tile0);
  // K tail (K_in % KS != 0): in the last stage, chunks past K_in step back onto the row's last
  // valid 16 bytes.  wback / xback are the per-lane byte distances; zero when there is no tail.
  const int nst = (K_ext + KS - 1) / KS;
  // (register-scale kernels only run on reductions of whole 4-stage panels: never a tail)
  const bool has_tail = SZR ? false : (K_ext % KS) != 0;
  uint32_t wback = 0, xback = 0;
  if (has_tail) {
    const int tail_k = K_ext - (nst - 1) * KS;           // valid reduction indices of the last stage
    const int wmax = tail_k / 2 - 16, xmax = tail_k * 2 - 16;
    wback = wl_chunk * 16 > wmax ? (uint32_t)(wl_chunk * 16 - wmax) : 0u;
    xback = xr_chunk * 16 > xmax ? (uint32_t)(xr_chunk * 16 - xmax) : 0u;
  }

  // Register prefetch rings (all slot indices are compile-time constants after unrolling, so the
  // rings stay in VGPRs).  Weights come from HBM: their loads are issued PDW stages ahead.
  // Activations come from L2 (every feature tile of a block re-reads them): PDX stages ahead.
  // Small token tiles: two stages ahead.  Four-deep weight rings (with two- or four-deep
  // activation rings) were measured 4-8 % slower on the decode shapes: the extra 32-48 registers
  // cost a workgroup per CU at 16x128 tiles and buy nothing at 32x128, where occupancy is the same.
  // Large token tiles spend several microseconds per stage, one stage of flight time is enough
  // and the registers are worth more to the compiler (no spills at 64x256).
  // steps per loop trip; with register scales one scale panel: 1024 k (512 k for 128-k stages)
  constexpr int UNR = SZR ? (KS >= 256 ? 1024 / KS : 4) : 2;
  // (512-k stages -- 256-byte row segments, one stage ahead, single activation buffer, three
  // workgroups per CU -- were measured 3-5 % slower than 256-k stages on the decode shapes; the
  // geometry below still covers them)
  // (two stages ahead for the large tiles as well was measured 1-2 % slower: their stalls are not load latency)
  constexpr int PDW = (MT >= 4 || KS >= 512) ? 1 : 2;
  constexpr int PDX = (MT >= 4 || XBUFS == 1) ? 1 : 2;
  static_assert(UNR % PDW == 0 && UNR % PDX == 0, "ring slots must repeat with the unrolled trip");
  u32x4 xr[PDX][XPASS], wr[PDW][WPASS];
  // activation passes that carry live rows: all of them here; the main loop of the 128-slot
  // eight-wave tile is specialised on its live 16-row sub-tiles and shadows this constant
  constexpr int XLIVE = XPASS;
  // A stage past the end still issues its loads (onto the last stage, which was just fetched) so
  // the loop body is branch-free and the compiler can count the outstanding loads exactly.
  // The per-lane offsets pass through an empty asm so that they stay opaque 32-bit VGPR values:
  // the loads then take the scalar-base + 32-bit-offset form instead of 64-bit per-lane addresses
  // (which cost two registers per load and VALU adds per stage).
#define MOE_LOAD_W(ST, WV)                                                                      \
  {                                                                                             \
    const int stc_ = (ST) < nst ? (ST) : nst - 1;                                               \
    const unsigned char* wb_ = wbase + (size_t)stc_ * (PRE == 1 ? UCH * 1024 : KS / 2);         \
    uint32_t wsub_ = 0;                                                                         \
    if (has_tail && stc_ == nst - 1) wsub_ = wback;                                             \
    _Pragma("unroll") for (int q = 0; q < WPASS; ++q) {                                         \
      asm("" : "+v"(woff[q]));                                                                  \
      WV[q] = load_weights<(MT <= 2)>(wb_ + (woff[q] - wsub_));                                 \
    }                                                                                           \
  }
#define MOE_LOAD_X(ST, XV)                                                                      \
  {                                                                                             \
    const int stc_ = (ST) < nst ? (ST) : nst - 1;                                               \
    const unsigned char* xb_ = xbase + (size_t)stc_ * (KS * 2);                                 \
    uint32_t xsub_ = 0;                                                                         \
    if (has_tail && stc_ == nst - 1) xsub_ = xback;                                             \
    _Pragma("unroll") for (int ps = 0; ps < XLIVE; ++ps) {                                      \
      asm("" : "+v"(xoff[ps]));                                                                 \
      XV[ps] = *reinterpret_cast<const u32x4*>(xb_ + (xoff[ps] - xsub_));                       \
    }                                                                                           \
  }
#define MOE_STORE_STAGE(XV, WV, XBUF)                                                           \
  {                                                                                             \
    if constexpr (!PRE) {                                                                       \
      _Pragma("unroll") for (int q = 0; q < WPASS; ++q) {                                       \
        const u32x4 t_ = WV[q];                                                                 \
        *reinterpret_cast<u32x4*>(wsw + (q * RPI + wl_row) * WP + wl_chunk * 16) =              \
            t_;                                                                                 \
      }                                                                                         \
    }                                                                                           \
    _Pragma("unroll") for (int ps = 0; ps < XLIVE; ++ps)                                        \
        *reinterpret_cast<u32x4*>((XBUF) + (ps * RPP + xr_row) * XP + xw_pos * 16) =            \
            interleave8(XV[ps]);                                                                \
  }

  // Flattened step index over (tile, stage).  nst_pad rounds the stages of a tile up to whole
  // trips; stages in [nst, nst_pad) are dead (clamped loads, no compute).
  const int nst_pad = (nst + UNR - 1) / UNR * UNR;
  int ld_t = 0, ld_st = 0;          // weight LOAD cursor: tile (local) and stage of the next stage to fetch
  int lx_st = 0;                    // activation LOAD cursor: stage only (every tile reads the same rows)
#define MOE_ADVANCE_W_CURSOR()                                      \
  {                                                                 \
    if (__builtin_expect(++ld_st == nst_pad, 0)) {                  \
      /* once per tile: the empty asm keeps this a real (scalar) branch; if-converted it     */ \
      /* costs ~24 VALU instructions in every stage                                          */ \
      asm volatile("");                                             \
      ld_st = 0;                                                    \
      if (++ld_t < ntl) {                                           \
        set_w_rows(tile0 + ld_t);                                   \
      } else { /* past the last tile: re-read row 0 of the expert; the lane keeps its own  */ \
               /* chunk offset so that subtracting wback (<= wl_chunk*16) cannot underflow  */ \
        _Pragma("unroll") for (int q = 0; q < WPASS; ++q)                                   \
            woff[q] = PRE == 1 ? (uint32_t)((q % UCH) * 1024 + lane * 16)                   \
                      : PRE == 2 ? (uint32_t)((q % UCH) * 64 + lj * 16) : (uint32_t)(wl_chunk * 16); \
      }                                                             \
    }                                                               \
  }
#define MOE_ADVANCE_X_CURSOR() { if (++lx_st == nst_pad) lx_st = 0; }
#pragma unroll
  for (int r = 0; r < (PDW > PDX ? PDW : PDX); ++r) {
    if (r < PDX) {
      MOE_LOAD_X(lx_st, xr[r])
      MOE_ADVANCE_X_CURSOR()
    }
    if (r < PDW) {
      MOE_LOAD_W(ld_st, wr[r])
      MOE_ADVANCE_W_CURSOR()
    }
  }

  // ---- register-resident scales / zero points (SZR) -----------------------------------
  // s_cur/s_nxt: fp16/bf16 scales (two per register) and zero-point bytes (four per register)
  // of the current / next panel, per sub-tile.
  constexpr int PG = SZR ? UNR * UCH : 8;          // groups per panel
  uint32_t s_cur[NT][PG / 2], s_nxt[NT][PG / 2];
  uint32_t z_cur[NT][(PG + 3) / 4], z_nxt[NT][(PG + 3) / 4];
  uint32_t z4_cur[NT][(PG + 3) / 4];               // z_cur with every byte shifted left by four
  auto adopt_zero_points = [&](const uint32_t(&zv)[NT][(PG + 3) / 4]) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < NT; ++s)
#pragma unroll
      for (int i = 0; i < (PG + 3) / 4; ++i) {
        z_cur[s][i] = zv[s][i] & 0x0f0f0f0fu;      // zero points are 4-bit by contract
        z4_cur[s][i] = z_cur[s][i] << 4;
      }
  };
  uint32_t sz_row[NT];                             // element offset of the lane's row (host checks the range)
  const int G_ext = ksp > 1 ? K_ext / 128 : p.G;   // groups in the reduction range (SZR: group 128)
  auto load_sz = [&](int g0, uint32_t(&sv)[NT][PG / 2], uint32_t(&zv)[NT][(PG + 3) / 4]) __attribute__((always_inline)) {
    if (g0 > G_ext - PG) g0 = G_ext - PG;           // clamp onto the last panel of the range
#pragma unroll
    for (int s = 0; s < NT; ++s) {
      const uint16_t* sp = reinterpret_cast<const uint16_t*>(p.scales) + sz_row[s] + g0;
      const uint8_t* zp = p.zeros + sz_row[s] + g0;
      if constexpr (PG == 8) {
        const u32x4 a = *reinterpret_cast<const u32x4*>(sp);
        const u32x2 b = *reinterpret_cast<const u32x2*>(zp);
        sv[s][0] = a.x; sv[s][1] = a.y; sv[s][2] = a.z; sv[s][3] = a.w;
        zv[s][0] = b.x; zv[s][1] = b.y;
      } else {
        const u32x2 a = *reinterpret_cast<const u32x2*>(sp);
        sv[s][0] = a.x; sv[s][1] = a.y;
        zv[s][0] = *reinterpret_cast<const uint32_t*>(zp);
      }
    }
  };
  auto set_sz_rows = [&](int tile) __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < NT; ++s) {
      int wrow, ocol;
      bool ok;
      feature_of<NT, FUSE, WV>(tile, wave, s, ln, p, wrow, ocol, ok);
      if (!ok) wrow = 0;
      sz_row[s] = ((uint32_t)e * (uint32_t)p.N_out + (uint32_t)wrow) * (uint32_t)p.G + (uint32_t)(k0 / 128);
    }
  };
  int sp_t = 0, sp_pan = 1;          // panel cursor: tile (local) and panel of the next prefetch
  const int npan = nst_pad / UNR;
  if constexpr (SZR) {
    set_sz_rows(tile0);
    load_sz(0, s_cur, z_nxt);
    adopt_zero_points(z_nxt);
    if (npan == 1) { sp_pan = 0; sp_t = 1; if (sp_t < ntl) set_sz_rows(tile0 + sp_t); }
  }

  // ---- stage scales / zero points of this tile's rows into LDS ---------------------
  if (tid < M_T) slot_s[tid] = slot_at(row0 + tid);
  if constexpr (!SZR) {
    const uint16_t* sc = reinterpret_cast<const uint16_t*>(p.scales);
    const int G = p.G, G8 = (G + 7) >> 3;
    for (int idx = tid; idx < N_T * G8; idx += THREADS) {
      const int lf = idx % N_T, gb = (idx / N_T) * 8;
      int wrow, ocol;
      bool ok;
      feature_of<NT, FUSE, WV>(tile0, lf / NW, (lf % NW) >> 4, lf & 15, p, wrow, ocol, ok);
      uint16_t sv[8];
      uint8_t zv[8];
      if (!ok) wrow = 0;      // fetched but never used: the row's outputs are not stored
      const size_t rbase = ((size_t)e * p.N_out + wrow) * G;
      if (p.sz_vec) {
        const u32x4 s4 = *reinterpret_cast<const u32x4*>(sc + rbase + gb);
        const u32x2 z2 = *reinterpret_cast<const u32x2*>(p.zeros + rbase + gb);
        const uint32_t sw[4] = {s4.x, s4.y, s4.z, s4.w};
        const uint32_t zw[2] = {z2.x, z2.y};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          sv[i] = (uint16_t)(sw[i >> 1] >> (16 * (i & 1)));
          zv[i] = (uint8_t)(zw[i >> 2] >> (8 * (i & 3)));
        }
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int gi = gb + i < G ? gb + i : G - 1;
          sv[i] = sc[rbase + gi];
          zv[i] = p.zeros[rbase + gi];
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if (gb + i < G) sz[(gb + i) * N_T + lf] = pack_sz_entry<DT, ZM>(sv[i], zv[i]);
    }
  }

  // Live 16-row sub-tiles of this tile.  The slots of a block are packed at its front, so the
  // count follows from the first row of every sub-tile (workgroup-uniform scalar loads).  The
  // eight-wave tile runs a main loop compiled for exactly that many sub-tiles: padding sub-tiles
  // cost no matrix instruction, no rescale, no LDS traffic (the weights' unpack is shared by all
  // live sub-tiles and is what the large tile amortises).
  constexpr bool SPEC = PRE == 2 && MT == 8;
  int live = MT;
  if constexpr (SPEC) {
    live = 0;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int sl = slot_at(row0 + 16 * mt);
      live += (sl >= 0 && sl < p.num_slots) ? 1 : 0;
    }
    live = __builtin_amdgcn_readfirstlane(live);      // uniform by construction: keep the dispatch a scalar branch
  }

  auto tile_body = [&](auto mlc) __attribute__((always_inline)) {
  constexpr int ML = decltype(mlc)::value;               // live sub-tiles this instance computes
  constexpr int XLIVE = (16 * ML + RPP - 1) / RPP;       // activation passes that hold them
  floatx4_t acc[ML][NT];
#pragma unroll
  for (int mt = 0; mt < ML; ++mt)
#pragma unroll
    for (int s = 0; s < NT; ++s) acc[mt][s] = floatx4_t{0.f, 0.f, 0.f, 0.f};
  float unit[NT];      // RS: scale the accumulator of each sub-tile is currently expressed in
#pragma unroll
  for (int s = 0; s < NT; ++s) unit[s] = 1.f;

  u32x4 wcur[WPASS];      // PRE: the weight words of the stage being computed (copied out of the ring)
  auto compute_stage = [&](int st, const unsigned char* xbuf, auto rc) __attribute__((always_inline)) {
    constexpr int R = decltype(rc)::value;       // step index inside the unrolled trip
    const int left = (K_ext - st * KS) / CK;     // <= 0 for a stage past the end
    // (the run-time bound also keeps the chunk-steps apart for the scheduler: with a constant bound
    // it interleaves them and needs ~40 more registers, which costs a workgroup per CU)
    const int nu = left < UCH ? left : UCH;   // SZR: whole panels, no partial or dead stage
#pragma unroll
    for (int u = 0; u < UCH; ++u) {
      if (u >= nu) break;
      const int cc = st * UCH + u;
      const int gi = p.cpg == 1 ? cc : cc / p.cpg;
      WordVec<KW> wv[NT];
      DeqCtx<DT, ZM> ctx[NT];
#pragma unroll
      for (int s = 0; s < NT; ++s) {
        if constexpr (SZR) {
          const int gp = (UCH * R + u) % PG;   // group inside the panel: constant after unrolling
          ctx[s] = DeqCtx<DT, ZM>::from_panel(gp, s_cur[s][gp >> 1], z_cur[s][gp >> 2], z4_cur[s][gp >> 2], uk);
        } else {
          ctx[s] = DeqCtx<DT, ZM>(sz[gi * N_T + wave * NW + s * 16 + ln]);
        }
        if constexpr (PRE) {
          const u32x4 t = wcur[s * UCH + u];      // the lane's four operand words, straight from the ring
          wv[s].w[0] = t.x; wv[s].w[1] = t.y; wv[s].w[2] = t.z; wv[s].w[3] = t.w;
        } else {
          wv[s] = lds_read_words<KW>(wsw + (s * 16 + ln) * WP + 16 * KW * u + 4 * KW * lj);
        }
      }
      u32x4 zop[NT];
      float scl[NT];
#pragma unroll
      for (int s = 0; s < NT; ++s) {
        scl[s] = ctx[s].s;
        if constexpr (ZM) zop[s] = ctx[s].zoperand();
      }
      if constexpr (RS) {
        bool zero_scale[NT];
        bool any_zero = false;
        float rs[NT];
#pragma unroll
        for (int s = 0; s < NT; ++s) {
          zero_scale[s] = scl[s] == 0.f;
          any_zero |= zero_scale[s];
          rs[s] = zero_scale[s] ? 1.f : unit[s] * __builtin_amdgcn_rcpf(scl[s]);
          unit[s] = zero_scale[s] ? unit[s] : scl[s];
        }
        if (__builtin_expect(__ballot(any_zero) != 0ull, 0)) {
          // Rare: a group with scale 0 contributes nothing.  Replace its packed words by q == z
          // (exact zero after the subtract).  The empty asm keeps this a real branch.
          asm volatile("" ::: "memory");
#pragma unroll
          for (int s = 0; s < NT; ++s) {
            // q == z everywhere: the subtract (or the zero-point MFMA) cancels it exactly
            const uint32_t zword = ctx[s].zero_point() * 0x11111111u;
#pragma unroll
            for (int i = 0; i < KW; ++i) wv[s].w[i] = zero_scale[s] ? zword : wv[s].w[i];
          }
        }
        // activation fragments one packed word ahead of the MFMAs that use them (the reads of
        // word i+1 are in flight while word i multiplies), so the LDS latency is not exposed
        // MT times per word
        u32x4 a_nxt[ML];
#define MOE_AREAD(MT_, OFF_) *reinterpret_cast<const u32x4*>(xbuf + ((MT_) * 16 + ln) * XP + 16 * (OFF_))
#pragma unroll
        for (int mt = 0; mt < ML; ++mt)
          a_nxt[mt] = MOE_AREAD(mt, 4 * KW * u + lj);
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          u32x4 a_cur[ML];
#pragma unroll
          for (int mt = 0; mt < ML; ++mt) a_cur[mt] = a_nxt[mt];
          if (i + 1 < KW) {
#pragma unroll
            for (int mt = 0; mt < ML; ++mt)
              a_nxt[mt] = MOE_AREAD(mt, 4 * KW * u + lj + 4 * (i + 1));
          }
          u32x4 b[NT];
#pragma unroll
          for (int s = 0; s < NT; ++s) b[s] = dequant_word<DT, ZM>(wv[s].w[i], ctx[s], uk);
#pragma unroll
          for (int mt = 0; mt < ML; ++mt) {
            const u32x4 a = a_cur[mt];
#pragma unroll
            for (int s = 0; s < NT; ++s) {
              // the rescale of each accumulator tile sits right before its first MFMA of the
              // group, so it overlaps with the MFMAs of the neighbouring tiles
              if (i == 0) {
#pragma unroll
                for (int c = 0; c < 4; ++c) acc[mt][s][c] *= rs[s];
              }
              acc[mt][s] = mfma16x16x32<DT>(a, b[s], acc[mt][s]);
            }
            if constexpr (ZM) {
#pragma unroll
              for (int s = 0; s < NT; ++s) acc[mt][s] = mfma16x16x32<DT>(a, zop[s], acc[mt][s]);
            }
          }
        }
      } else {
        floatx4_t part[ML][NT];
#pragma unroll
        for (int i = 0; i < KW; ++i) {
          u32x4 b[NT];
#pragma unroll
          for (int s = 0; s < NT; ++s) b[s] = dequant_word<DT, ZM>(wv[s].w[i], ctx[s], uk);
#pragma unroll
          for (int mt = 0; mt < ML; ++mt) {
            const u32x4 a = *reinterpret_cast<const u32x4*>(
                xbuf + (mt * 16 + ln) * XP + 16 * (4 * KW * u + lj + 4 * i));
#pragma unroll
            for (int s = 0; s < NT; ++s)
              part[mt][s] = mfma16x16x32<DT>(a, b[s], i == 0 ? floatx4_t{0.f, 0.f, 0.f, 0.f} : part[mt][s]);
            if constexpr (ZM) {
#pragma unroll
              for (int s = 0; s < NT; ++s) part[mt][s] = mfma16x16x32<DT>(a, zop[s], part[mt][s]);
            }
          }
        }
#pragma unroll
        for (int s = 0; s < NT; ++s) {
#pragma unroll
          for (int mt = 0; mt < ML; ++mt)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[mt][s][i] = __builtin_fmaf(scl[s], part[mt][s][i], acc[mt][s][i]);
        }
      }
    }
  };

  MOE_STORE_STAGE(xr[0], wr[0], xs)
  __syncthreads();

  // ---- store one finished feature tile: one rounding to the 16-bit type, rows by slot id ----
  auto store_tile = [&](int tile) __attribute__((always_inline)) {
    if constexpr (RS) {
#pragma unroll
      for (int mt = 0; mt < ML; ++mt)
#pragma unroll
        for (int s = 0; s < NT; ++s)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[mt][s][i] *= unit[s];
    }
    uint16_t* C16 = reinterpret_cast<uint16_t*>(p.C);
#pragma unroll
    for (int mt = 0; mt < ML; ++mt) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int slot = slot_s[mt * 16 + lj * 4 + i];
        if (slot < 0 || slot >= p.num_slots) continue;
        uint16_t* crow = C16 + (size_t)slot * p.ldc;
        if constexpr (FUSE == 0 && NT == 1) {
          int wrow, ocol; bool ok;
          feature_of<NT, FUSE, WV>(tile, wave, 0, ln, p, wrow, ocol, ok);
          if (ok) {
            if (p.out_f32) (reinterpret_cast<float*>(p.C) + (size_t)split * p.split_stride)[(size_t)slot * p.ldc + ocol] = acc[mt][0][i];
            else crow[ocol] = to_bits16<DT>(acc[mt][0][i]);
          }
        } else if constexpr (FUSE == 0) {
#pragma unroll
          for (int s = 0; s < NT; s += 2) {
            // columns ocol (even) and ocol + 1 belong to this lane: one 8-byte / 4-byte store
            int wrow, ocol; bool ok;
            feature_of<NT, FUSE, WV>(tile, wave, s, ln, p, wrow, ocol, ok);
            if (ok) {
              if (p.out_f32) {
                float* dst = reinterpret_cast<float*>(p.C) + (size_t)split * p.split_stride + (size_t)slot * p.ldc + ocol;
                *reinterpret_cast<floatx2_t*>(dst) = floatx2_t{acc[mt][s][i], acc[mt][s + 1][i]};
              } else {
                *reinterpret_cast<uint32_t*>(crow + ocol) =
                    (uint32_t)to_bits16<DT>(acc[mt][s][i]) | ((uint32_t)to_bits16<DT>(acc[mt][s + 1][i]) << 16);
              }
            }
          }
        } else {
#pragma unroll
          for (int s = 0; s < NT; s += 2) {
            int wrow, ocol; bool ok;
            feature_of<NT, FUSE, WV>(tile, wave, s, ln, p, wrow, ocol, ok);
            if (ok) {
              // round gate/up to the storage type first so the fused path equals the staged one
              const float g = from_bits16<DT>(to_bits16<DT>(acc[mt][s][i]));
              const float u = from_bits16<DT>(to_bits16<DT>(acc[mt][s + 1][i]));
              crow[ocol] = to_bits16<DT>(silu_f32(g) * u);
            }
          }
        }
      }
    }
#pragma unroll
    for (int mt = 0; mt < ML; ++mt)
#pragma unroll
      for (int s = 0; s < NT; ++s) acc[mt][s] = floatx4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < NT; ++s) unit[s] = 1.f;
  };

  if constexpr (WV == 8) {
    // ---- skewed pipeline of the eight-wave tile --------------------------------------------
    // All eight waves of the workgroup run in step, so whatever one wave waits for, the whole CU
    // waits for.  Three activation buffers take every wait off the critical path:
    //   step g:  store stage g+1 (fetched during step g-1) into its buffer; fetch stage g+2 (X) and
    //            g+1 (weights); multiply words 0 and 1 of stage g; BARRIER; multiply words 2 and 3,
    //            and while word 3 multiplies read the first fragments of stage g+1.
    // The barrier sits in the middle of a stage's matrix work: the stores it publishes were issued
    // half a stage earlier, the fragments read after it are needed half a stage later, and the
    // buffer a step writes was last read two steps before (its readers passed the previous
    // barrier), so nothing waits on LDS latency, on the store, or on the global loads.
    static_assert(PRE == 2 && SZR == 1 && KS == 128 && KW == 4 && UCH == 1 && UNR == 4 && PDW == 1 && PDX == 1 &&
                  RS == 1 && XBUFS == 3 && WPASS == NT, "the skewed pipeline is written for the 128-k register-scale tile");
    constexpr int XBYTES = M_T * XP;
    MOE_LOAD_X(lx_st, xr[0])          // stage 1 (stage 0 is in buffer 0 already)
    MOE_ADVANCE_X_CURSOR()
    unsigned char* xb_cur = xs;
    unsigned char* xb_nxt = xs + XBYTES;
    unsigned char* xb_fre = xs + 2 * XBYTES;
    u32x4 a_pf[ML];                   // activation fragments of the next word, one word ahead
#pragma unroll
    for (int mt = 0; mt < ML; ++mt)
      a_pf[mt] = *reinterpret_cast<const u32x4*>(xb_cur + (mt * 16 + ln) * XP + 16 * lj);
    DeqCtx<DT, ZM> ctx[NT];
    float rs[NT];
    u32x4 zop[NT];
    // word i of the stage: its fragments are in a_pf; start the reads of the following word (word 0
    // of the next stage after word 3) from rd_buf, unpack, multiply.
    auto word = [&](auto ic, auto rc, const unsigned char* rd_buf) __attribute__((always_inline)) {
      constexpr int i = decltype(ic)::value;
      constexpr int R = decltype(rc)::value;
      u32x4 a_cur[ML];
#pragma unroll
      for (int mt = 0; mt < ML; ++mt) a_cur[mt] = a_pf[mt];
#pragma unroll
      for (int mt = 0; mt < ML; ++mt)
        a_pf[mt] = *reinterpret_cast<const u32x4*>(rd_buf + (mt * 16 + ln) * XP + 16 * (lj + 4 * ((i + 1) & 3)));
      if constexpr (i == 0) {
        bool zero_scale[NT];
        bool any_zero = false;
#pragma unroll
        for (int s = 0; s < NT; ++s) {
          constexpr int gp = R % PG;
          ctx[s] = DeqCtx<DT, ZM>::from_panel(gp, s_cur[s][gp >> 1], z_cur[s][gp >> 2], z4_cur[s][gp >> 2], uk);
          if constexpr (ZM) zop[s] = ctx[s].zoperand();
          zero_scale[s] = ctx[s].s == 0.f;
          any_zero |= zero_scale[s];
          rs[s] = zero_scale[s] ? 1.f : unit[s] * __builtin_amdgcn_rcpf(ctx[s].s);
          unit[s] = zero_scale[s] ? unit[s] : ctx[s].s;
        }
        if (__builtin_expect(__ballot(any_zero) != 0ull, 0)) {
          asm volatile("" ::: "memory");      // rare: a real branch (see the four-wave path)
#pragma unroll
          for (int s = 0; s < NT; ++s) {
            const uint32_t zword = ctx[s].zero_point() * 0x11111111u;
            if (zero_scale[s]) wcur[s] = u32x4{zword, zword, zword, zword};
          }
        }
      }
      u32x4 b[NT];
#pragma unroll
      for (int s = 0; s < NT; ++s) {
        const uint32_t w = i == 0 ? wcur[s].x : i == 1 ? wcur[s].y : i == 2 ? wcur[s].z : wcur[s].w;
        b[s] = dequant_word<DT, ZM>(w, ctx[s], uk);
      }
#pragma unroll
      for (int mt = 0; mt < ML; ++mt) {
#pragma unroll
        for (int s = 0; s < NT; ++s) {
          if constexpr (i == 0) {
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[mt][s][c] *= rs[s];
          }
          acc[mt][s] = mfma16x16x32<DT>(a_cur[mt], b[s], acc[mt][s]);
        }
        if constexpr (ZM) {
#pragma unroll
          for (int s = 0; s < NT; ++s) acc[mt][s] = mfma16x16x32<DT>(a_cur[mt], zop[s], acc[mt][s]);
        }
      }
    };
    int c_t = 0, c_st = 0;
    const int trips = ntl * npan;
    for (int trip = 0; trip < trips; ++trip) {
      load_sz(sp_pan * PG, s_nxt, z_nxt);
      if (__builtin_expect(++sp_pan == npan, 0)) {
        asm volatile("");
        sp_pan = 0;
        if (++sp_t < ntl) set_sz_rows(tile0 + sp_t);
      }
      [&]<int... Rs>(std::integer_sequence<int, Rs...>) {
        (([&] {
           constexpr int r = Rs;
           // the stage fetched during the previous step goes to the buffer nobody reads any more
#pragma unroll
           for (int ps = 0; ps < XLIVE; ++ps)
             *reinterpret_cast<u32x4*>(xb_nxt + (ps * RPP + xr_row) * XP + xw_pos * 16) = interleave8(xr[0][ps]);
#pragma unroll
           for (int q = 0; q < WPASS; ++q) wcur[q] = wr[0][q];
           MOE_LOAD_X(lx_st, xr[0])
           MOE_ADVANCE_X_CURSOR()
           MOE_LOAD_W(ld_st, wr[0])
           MOE_ADVANCE_W_CURSOR()
           word(std::integral_constant<int, 0>{}, std::integral_constant<int, r>{}, xb_cur);
           word(std::integral_constant<int, 1>{}, std::integral_constant<int, r>{}, xb_cur);
           __syncthreads();
           word(std::integral_constant<int, 2>{}, std::integral_constant<int, r>{}, xb_cur);
           word(std::integral_constant<int, 3>{}, std::integral_constant<int, r>{}, xb_nxt);
           unsigned char* const t_ = xb_cur;
           xb_cur = xb_nxt; xb_nxt = xb_fre; xb_fre = t_;
         }()),
         ...);
      }(std::make_integer_sequence<int, UNR>{});
#pragma unroll
      for (int s = 0; s < NT; ++s) {
#pragma unroll
        for (int i = 0; i < PG / 2; ++i) s_cur[s][i] = s_nxt[s][i];
      }
      adopt_zero_points(z_nxt);
      c_st += UNR;
      if (c_st == nst_pad) {
        store_tile(tile0 + c_t);
        c_st = 0;
        ++c_t;
      }
    }
  } else {
  // Step: issue the loads PD stages ahead into the ring slot whose stage went to LDS in the
  // previous step, compute the current stage from LDS, move the next stage from its ring slot
  // into LDS, barrier.  UNR steps per trip so ring slots, activation buffers and (SZR) the scale
  // registers are indexed statically.  Dead stages compute nothing (their loads are clamped onto
  // valid addresses, their LDS stores are never read).  A trip never straddles two tiles.
  int c_t = 0, c_st = 0;             // compute cursor
  const int trips = ntl * npan;
  for (int trip = 0; trip < trips; ++trip) {
    if constexpr (SZR) {
      // prefetch the scales / zero points of the next panel (possibly of the next tile)
      load_sz(sp_pan * PG, s_nxt, z_nxt);
      if (__builtin_expect(++sp_pan == npan, 0)) {
        asm volatile("");      // a real branch, taken once per tile
        sp_pan = 0;
        if (++sp_t < ntl) set_sz_rows(tile0 + sp_t);
      }
    }
    [&]<int... Rs>(std::integer_sequence<int, Rs...>) {
      (([&] {
         constexpr int r = Rs;
         // activations first: the wait for them (loads complete in issue order) then leaves the
         // younger weight loads of PDW - PDX + 1 stages in flight
         if constexpr (PRE) {
           // the ring slot about to be refilled holds the stage computed in this step
#pragma unroll
           for (int q = 0; q < WPASS; ++q) wcur[q] = wr[r % PDW][q];
         }
         MOE_LOAD_X(lx_st, xr[r % PDX])
         MOE_ADVANCE_X_CURSOR()
         MOE_LOAD_W(ld_st, wr[r % PDW])
         MOE_ADVANCE_W_CURSOR()
         compute_stage(c_st + r, xs + (r % XBUFS) * (M_T * XP), std::integral_constant<int, r>{});
         if constexpr (XBUFS == 1) __syncthreads();      // everyone is done reading the single buffer
         MOE_STORE_STAGE(xr[(r + 1) % PDX], wr[(r + 1) % PDW], xs + ((r + 1) % XBUFS) * (M_T * XP))
         __syncthreads();
       }()),
       ...);
    }(std::make_integer_sequence<int, UNR>{});
    if constexpr (SZR) {
#pragma unroll
      for (int s = 0; s < NT; ++s) {
#pragma unroll
        for (int i = 0; i < PG / 2; ++i) s_cur[s][i] = s_nxt[s][i];
      }
      adopt_zero_points(z_nxt);
    }
    c_st += UNR;
    if (c_st == nst_pad) {
      store_tile(tile0 + c_t);
      c_st = 0;
      ++c_t;
    }
  }
  }    // four-wave pipeline
  };   // tile_body

  if constexpr (SPEC) {
    static_assert(MT == 8, "the live-sub-tile dispatch is written for 128-slot tiles");
    switch (live) {      // workgroup-uniform
      case 1: tile_body(std::integral_constant<int, 1>{}); break;
      case 2: tile_body(std::integral_constant<int, 2>{}); break;
      case 3: tile_body(std::integral_constant<int, 3>{}); break;
      case 4: tile_body(std::integral_constant<int, 4>{}); break;
      case 5: tile_body(std::integral_constant<int, 5>{}); break;
      case 6: tile_body(std::integral_constant<int, 6>{}); break;
      case 7: tile_body(std::integral_constant<int, 7>{}); break;
      case 8: tile_body(std::integral_constant<int, 8>{}); break;
      default: break;    // no live row (second half of a 256-slot block): nothing to do
    }
  } else {
    tile_body(std::integral_constant<int, MT>{});
  }
#undef MOE_LOAD_W
#undef MOE_AREAD
#undef MOE_LOAD_X
#undef MOE_STORE_STAGE
#undef MOE_ADVANCE_W_CURSOR
#undef MOE_ADVANCE_X_CURSOR
}

// Host-side launcher, one per instantiation.  Returns hipError_t as int.
template <int DT, int MT, int NT, int KS, int KW, int FUSE, int SZR, int PRE = 0, int WV = 4>
int launch_w4a16_gemm(const GemmParams& p, int grid, hipStream_t stream);

}  // namespace moe
