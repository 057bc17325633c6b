// Host side of the C ABI declared in include/moe_w4a16.h: argument validation, tile choice,
// workspace carving and kernel launches.  No allocation, no synchronisation, caller's stream.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/fp8_blockwise_gemm.h"
#include "../../include/moe_w4a16.h"
#include "fp8_gemm.hpp"
#include "gemm_kernel.hpp"


namespace moe {

int launch_align(const int32_t*, int, int, int, int, int32_t*, int32_t*, int32_t*, int32_t*, int32_t*,
                 hipStream_t);
int launch_silu_mul(const void*, void*, long long, int, int, hipStream_t);
int launch_repack(const int32_t*, int, int, int, int, int32_t*, hipStream_t);
int launch_awq_import(const int32_t*, const int32_t*, const void*, int, int, int, int, int32_t*, void*, uint8_t*,
                      hipStream_t);
int launch_route_topk(const float*, const float*, int, int, int, int32_t*, float*, hipStream_t);
int launch_route_align(const float*, const float*, int, int, int, int32_t*, float*, int, int, int32_t*, int32_t*,
                       int32_t*, int32_t*, int32_t*, hipStream_t);
int launch_stream_read(const void*, size_t, uint32_t*, int, hipStream_t);
int launch_mfma_loop(float*, int, int, hipStream_t);
int launch_issue_mix(float*, int, int, int, hipStream_t);
int launch_combine(const void*, int, int, const float*, const int32_t*, int, void*, long long, int, int, int,
                   hipStream_t);
}  // namespace moe
namespace fp8 {
int launch_fp8_quantize(const void*, long long, int, int, int, uint8_t*, float*, hipStream_t);
}
namespace moe {

// ---- table of compiled GEMM variants ------------------------------------------------------
#define MOE_DECL(DT, MT, NT, KS, KW, F, Z) \
  extern template int launch_w4a16_gemm<DT, MT, NT, KS, KW, F, Z, 0, 4>(const GemmParams&, int, hipStream_t);
#define MOE_DECL_PRE(DT, MT, NT, KS, F) \
  extern template int launch_w4a16_gemm<DT, MT, NT, KS, 4, F, 1, 1, 4>(const GemmParams&, int, hipStream_t);
#define MOE_DECL_WIDE(DT, MT, NT, KS, F, WV) \
  extern template int launch_w4a16_gemm<DT, MT, NT, KS, 4, F, 1, 2, WV>(const GemmParams&, int, hipStream_t);
#define MOE_ALL_DT_KW(M, MT, NT, KS, F) \
  M(0, MT, NT, KS, 1, F, 0) M(0, MT, NT, KS, 2, F, 0) M(0, MT, NT, KS, 4, F, 0) \
  M(1, MT, NT, KS, 1, F, 0) M(1, MT, NT, KS, 2, F, 0) M(1, MT, NT, KS, 4, F, 0)
#define MOE_TILE(MT, NT, KS) MOE_ALL_DT_KW(MOE_DECL, MT, NT, KS, 0)
#define MOE_TILE_FUSE(MT, NT, KS) MOE_ALL_DT_KW(MOE_DECL, MT, NT, KS, 1)
#include "gemm_variants.def"
#define MOE_TILE_SZR(MT, NT, KS) MOE_DECL(0, MT, NT, KS, 4, 0, 1) MOE_DECL(1, MT, NT, KS, 4, 0, 1)
#define MOE_TILE_SZR_FUSE(MT, NT, KS) MOE_DECL(0, MT, NT, KS, 4, 1, 1) MOE_DECL(1, MT, NT, KS, 4, 1, 1)
#include "gemm_variants_szr.def"
#define MOE_TILE_PRE(MT, NT, KS) MOE_DECL_PRE(0, MT, NT, KS, 0) MOE_DECL_PRE(1, MT, NT, KS, 0)
#define MOE_TILE_PRE_FUSE(MT, NT, KS) MOE_DECL_PRE(0, MT, NT, KS, 1) MOE_DECL_PRE(1, MT, NT, KS, 1)
#include "gemm_variants_pre.def"
#define MOE_TILE_WIDE(MT, NT, KS, WV) MOE_DECL_WIDE(0, MT, NT, KS, 0, WV) MOE_DECL_WIDE(1, MT, NT, KS, 0, WV)
#define MOE_TILE_WIDE_FUSE(MT, NT, KS, WV) MOE_DECL_WIDE(0, MT, NT, KS, 1, WV) MOE_DECL_WIDE(1, MT, NT, KS, 1, WV)
#include "gemm_variants_wide.def"

typedef int (*GemmLaunchFn)(const GemmParams&, int, hipStream_t);
// pre: 0 = weight tile staged in LDS, 1 = operand-order (repacked) weights, 2 = row-major weights
// loaded in operand order; wv = wavefronts per workgroup
struct GemmVariant { int dt, mt, nt, ks, kw, fuse, szr, pre, wv; GemmLaunchFn fn; };
#define MOE_ENTRY(DT, MT, NT, KS, KW, F, Z) {DT, MT, NT, KS, KW, F, Z, 0, 4, &launch_w4a16_gemm<DT, MT, NT, KS, KW, F, Z, 0, 4>},
#define MOE_ENTRY_PRE(DT, MT, NT, KS, F) {DT, MT, NT, KS, 4, F, 1, 1, 4, &launch_w4a16_gemm<DT, MT, NT, KS, 4, F, 1, 1, 4>},
#define MOE_ENTRY_WIDE(DT, MT, NT, KS, F, WV) {DT, MT, NT, KS, 4, F, 1, 2, WV, &launch_w4a16_gemm<DT, MT, NT, KS, 4, F, 1, 2, WV>},
static const GemmVariant kVariants[] = {
#define MOE_TILE(MT, NT, KS) MOE_ALL_DT_KW(MOE_ENTRY, MT, NT, KS, 0)
#define MOE_TILE_FUSE(MT, NT, KS) MOE_ALL_DT_KW(MOE_ENTRY, MT, NT, KS, 1)
#include "gemm_variants.def"
#define MOE_TILE_SZR(MT, NT, KS) MOE_ENTRY(0, MT, NT, KS, 4, 0, 1) MOE_ENTRY(1, MT, NT, KS, 4, 0, 1)
#define MOE_TILE_SZR_FUSE(MT, NT, KS) MOE_ENTRY(0, MT, NT, KS, 4, 1, 1) MOE_ENTRY(1, MT, NT, KS, 4, 1, 1)
#include "gemm_variants_szr.def"
#define MOE_TILE_PRE(MT, NT, KS) MOE_ENTRY_PRE(0, MT, NT, KS, 0) MOE_ENTRY_PRE(1, MT, NT, KS, 0)
#define MOE_TILE_PRE_FUSE(MT, NT, KS) MOE_ENTRY_PRE(0, MT, NT, KS, 1) MOE_ENTRY_PRE(1, MT, NT, KS, 1)
#include "gemm_variants_pre.def"
#define MOE_TILE_WIDE(MT, NT, KS, WV) MOE_ENTRY_WIDE(0, MT, NT, KS, 0, WV) MOE_ENTRY_WIDE(1, MT, NT, KS, 0, WV)
#define MOE_TILE_WIDE_FUSE(MT, NT, KS, WV) MOE_ENTRY_WIDE(0, MT, NT, KS, 1, WV) MOE_ENTRY_WIDE(1, MT, NT, KS, 1, WV)
#include "gemm_variants_wide.def"
};

static const GemmVariant* find_variant(int dt, int mt, int nt, int kw, int fuse, int szr, int pre = 0, int wv = 4) {
  for (const GemmVariant& v : kVariants)
    if (v.dt == dt && v.mt == mt && v.nt == nt && v.kw == kw && v.fuse == fuse && v.szr == szr && v.pre == pre &&
        v.wv == wv)
      return &v;
  return nullptr;
}

// ---- thread-local state -----------------------------------------------------------------
static thread_local char g_err[512] = "";
static thread_local void* g_events[7] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
static thread_local int g_nevents = 0;
static thread_local int g_force_mt = 0, g_force_nt = 0;
static thread_local int g_scale_path = 0;   // 0 auto, 1 LDS table, 2 registers
static thread_local int g_force_tpw = 0;    // feature tiles per workgroup (register-scale kernels), 0 = auto
static thread_local int g_force_ksplit = 0; // reduction splits of the layer's down projection, 0 = auto
static thread_local int g_force_block_m = 0; // bucketing block of the layer, 0 = auto
static thread_local int g_wide_mode = 0;     // eight-wave 128-token tiles: 0 = when the shape allows, 1 = never
static thread_local int g_last_plan[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};   // what the last grouped GEMM launch used

static int fail(int status, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return status;
}
static int hip_fail(int err, const char* what) {
  return fail(MOE_HIP_ERROR, "%s: %s", what, hipGetErrorString((hipError_t)err));
}

static bool valid_block_m(int b) { return b == 16 || b == 32 || b == 64 || b == 128 || b == 256; }
static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static size_t align_capacity(long long S, int E, int block_m) {
  const long long worst = S + (S < E ? S : E) * (long long)(block_m - 1);
  return (size_t)((worst + block_m - 1) / block_m * block_m);
}
constexpr size_t kLdsLimit = 160 * 1024;
constexpr int kMaxGroups = 512;

static size_t gemm_lds_bytes(int mt, int nt, int ks, int G, int szr) {
  const size_t M_T = 16 * mt, NW = 16 * nt;
  return kXBufs(mt, ks) * M_T * (ks * 2 + kXRowPad) + 4 * NW * (ks / 2 + kWRowPad(ks)) + (szr ? 0 : (size_t)G * 64 * nt * 4) + M_T * 4;
}

// The eight-wave 128-token tile serves 128-slot blocks of register-scale shapes in the stated
// weight layout (group 128, 16-byte aligned scale rows).
static bool wide_tile_usable(int block_m, int szr_ok, int pre) {
  return block_m >= 128 && szr_ok && !pre && g_wide_mode != 1 && g_force_mt == 0 && g_force_nt == 0;
}

// Tile choice.  Tokens per tile follow the bucketing block; the feature width per workgroup is
// as wide as LDS allows while still giving every CU a couple of workgroups (256 CUs).
static int choose_tile(int num_slots, int E, int feat, int G, int block_m, int fuse, int szr_ok, int dt, int pre,
                       int& mt, int& nt, int& ks, int& szr) {
  mt = block_m / 16;
  if (mt > 8) mt = 8;
  if (g_force_mt > 0) {
    if ((block_m / 16) % g_force_mt != 0) return -1;
    mt = g_force_mt;
  }
  ks = mt >= 4 ? 128 : 256;
  const int min_nt = (fuse || mt >= 4) ? 2 : 1;
  // register-resident scales when the shape allows it and such a variant is compiled
  auto pick_szr = [&](int nt_) {
    if ((g_scale_path == 1 && !pre) || !szr_ok) return 0;
    return find_variant(dt, mt, nt_, 4, fuse, 1, pre) ? 1 : 0;
  };
  if (g_force_nt > 0) {
    nt = g_force_nt;
    szr = pick_szr(nt);
    if ((g_scale_path == 2 || pre) && !szr) return -1;
    return (nt >= min_nt && (nt == 1 || nt == 2 || nt == 4) && gemm_lds_bytes(mt, nt, ks, G, szr) <= kLdsLimit) ? 0 : -1;
  }
  const long long est_blocks = (num_slots + 16 * mt - 1) / (16 * mt) + (num_slots < E ? num_slots : E) / 2;
  // 256-feature tiles only pay off with register-resident scales (two workgroups per CU)
  nt = (mt >= 4 && pick_szr(4)) ? 4 : 2;
  for (;;) {
    const int fpw = fuse ? 32 * nt : 64 * nt;
    const long long wgs = est_blocks * ((feat + fpw - 1) / fpw);
    szr = pick_szr(nt);
    if ((g_scale_path == 2 || pre) && !szr) { if (nt == min_nt) return -1; nt >>= 1; continue; }
    const bool fits = gemm_lds_bytes(mt, nt, ks, G, szr) <= kLdsLimit;
    // 128-feature tiles stay even when they leave fewer than two workgroups per CU: measured
    // faster than twice as many 64-feature tiles (same bytes in flight, less activation staging)
    if (fits && (wgs >= 512 || nt <= 2 || nt == min_nt)) return 0;
    if (nt == min_nt) return -1;
    nt >>= 1;
  }
}

struct GemmArgs {
  const void* A; int row_div;
  const int32_t* qweight; const void* scales; const uint8_t* zeros;
  const int32_t* sorted_slot_ids; const int32_t* block_expert_ids; const int32_t* num_padded;
  int num_slots, E, N_out, K_in, group, block_m, dt;
  void* C; int ldc; int fuse_half_n; int out_f32;
  int dense = 0;             // 1: plain GEMM, no routing tables (the three table pointers are null)
  int pre = 0;               // 1: qweight is in the operand-order layout of moe_repack_qweight
  int k_splits = 1;          // wanted reduction splits (float32 output planes num_slots*ldc apart)
  int* used_splits = nullptr;  // out: the number of planes the launch really wrote
};

static int run_gemm(const GemmArgs& a, hipStream_t stream) {
  if (a.dt != MOE_F16 && a.dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (a.num_slots < 0 || a.E < 1 || a.row_div < 1 || a.N_out < 1 || a.K_in < 1 || a.group < 1)
    return fail(MOE_INVALID_ARGUMENT, "sizes must be positive (num_slots >= 0)");
  if (!valid_block_m(a.block_m)) return fail(MOE_INVALID_ARGUMENT, "block_m must be 16, 32, 64, 128 or 256");
  if (a.group % 32 != 0) return fail(MOE_UNSUPPORTED_SHAPE, "group_size %d is not a multiple of 32", a.group);
  if (a.K_in % a.group != 0) return fail(MOE_UNSUPPORTED_SHAPE, "K_in %d is not a multiple of group_size %d", a.K_in, a.group);
  if (a.N_out % 16 != 0) return fail(MOE_UNSUPPORTED_SHAPE, "N_out %d is not a multiple of 16", a.N_out);
  const int G = a.K_in / a.group;
  if (G > kMaxGroups) return fail(MOE_UNSUPPORTED_SHAPE, "K_in/group_size = %d exceeds %d", G, kMaxGroups);
  if (a.num_slots == 0) return MOE_OK;
  if (!a.A || !a.qweight || !a.scales || !a.zeros || !a.C ||
      (!a.dense && (!a.sorted_slot_ids || !a.block_expert_ids || !a.num_padded)))
    return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (((uintptr_t)a.A | (uintptr_t)a.qweight) % 16 != 0)
    return fail(MOE_INVALID_ARGUMENT, "A and qweight must be 16-byte aligned");
  if ((uintptr_t)a.scales % 2 != 0 || (uintptr_t)a.C % (a.out_f32 ? 8 : 4) != 0)
    return fail(MOE_INVALID_ARGUMENT, "scales must be 2-byte aligned and C 4-byte aligned");

  // kernels address with 32-bit per-lane byte offsets from a per-expert / per-matrix base
  if ((long long)a.N_out * (a.K_in / 2) >= (1LL << 31))
    return fail(MOE_UNSUPPORTED_SHAPE, "one expert's packed weights must stay below 2 GiB");
  if (((long long)(a.num_slots + a.row_div - 1) / a.row_div) * a.K_in * 2 >= (1LL << 31))
    return fail(MOE_UNSUPPORTED_SHAPE, "the A matrix must stay below 2 GiB");
  const int fuse = a.fuse_half_n > 0 ? 1 : 0;
  const int feat = fuse ? a.fuse_half_n : a.N_out;
  const int kw = a.group % 128 == 0 ? 4 : (a.group % 64 == 0 ? 2 : 1);
  int mt, nt, ks, szr;
  const int sz_vec = (G % 8 == 0 && (uintptr_t)a.scales % 16 == 0 && (uintptr_t)a.zeros % 8 == 0) ? 1 : 0;
  const int szr_ok = sz_vec && a.group == 128 && (long long)a.E * a.N_out * G < (1LL << 31);
  if (a.pre && (!szr_ok || (!fuse && a.N_out % 32 != 0)))
    return fail(MOE_UNSUPPORTED_SHAPE, "operand-order weights need group_size 128, K_in %% 1024 == 0, 16-byte aligned "
                "scale rows and (down projection) N_out %% 32 == 0");
  int wv = 4, pre = a.pre;
  if (wide_tile_usable(a.block_m, szr_ok, a.pre) && find_variant(a.dt, 8, 2, 4, fuse, 1, 2, 8)) {
    mt = 8; nt = 2; ks = 128; szr = 1; wv = 8; pre = 2;
  } else if (choose_tile(a.num_slots, a.E, feat, G, a.block_m, fuse, szr_ok, a.dt, a.pre, mt, nt, ks, szr) != 0) {
    return fail(MOE_UNSUPPORTED_SHAPE, "no GEMM tile fits (K_in/group_size = %d, block_m = %d, override %d/%d)",
                G, a.block_m, g_force_mt, g_force_nt);
  }
  const GemmVariant* v = find_variant(a.dt, mt, nt, kw, fuse, szr, pre, wv);
  if (!v) return fail(MOE_UNSUPPORTED_SHAPE, "GEMM variant mt=%d nt=%d kw=%d fuse=%d szr=%d is not compiled", mt, nt, kw, fuse, szr);

  GemmParams p;
  p.A = a.A; p.row_div = a.row_div;
  p.qweight = a.qweight; p.scales = a.scales; p.zeros = a.zeros;
  p.sorted_slot_ids = a.sorted_slot_ids; p.block_expert_ids = a.block_expert_ids; p.num_padded = a.num_padded;
  p.num_slots = a.num_slots; p.E = a.E; p.N_out = a.N_out; p.K_in = a.K_in; p.group = a.group;
  p.block_m = a.block_m; p.C = a.C; p.ldc = a.ldc;
  const int fpw = (fuse ? 8 : 16) * nt * wv;     // features (act columns when fused) per workgroup tile
  p.n_tiles = (feat + fpw - 1) / fpw;
  p.G = G;
  p.cpg = a.group / (32 * kw);
  p.half_n = a.fuse_half_n;
  p.out_f32 = a.out_f32;
  p.sz_vec = sz_vec;
  p.dense = a.dense;
  // Split reduction: whole scale panels (4 pipeline stages) per range, every range non-empty.
  int ksp = 1, kspan = a.K_in;
  if (a.k_splits > 1 && szr && a.out_f32 && !fuse) {
    const int pan = ks >= 256 ? 1024 : 512, npan = a.K_in / pan;   // one scale panel of the kernel
    const int pps = (npan + a.k_splits - 1) / a.k_splits;
    ksp = (npan + pps - 1) / pps;
    kspan = pps * pan;
  }
  p.k_splits = ksp; p.k_span = kspan; p.split_stride = (long long)a.num_slots * a.ldc;
  if (a.used_splits) *a.used_splits = ksp;
  const size_t cap = align_capacity(a.num_slots, a.E, a.block_m);
  // Register-scale kernels can walk several feature tiles per workgroup: aim for about 48
  // pipeline stages per workgroup at small token tiles (the start-up of a workgroup costs about
  // as much as ten of their stages) while keeping a few thousand workgroups in the launch.
  int tpw = 1;
  if (szr) {
    const int nst = kspan / ks;
    const int target = mt <= 2 ? 48 : 24;       // large token tiles: stages are long, start-up matters less
    tpw = (target + nst - 1) / nst;
    if (tpw > 8) tpw = 8;
    if (tpw > p.n_tiles) tpw = p.n_tiles;
    // prefer a count that divides the tiles of a block evenly (no short last group)
    for (int t = tpw; t <= tpw + 2 && t <= 8 && t <= p.n_tiles; ++t)
      if (p.n_tiles % t == 0) { tpw = t; break; }
    const long long est_blocks = (a.num_slots + 16 * mt - 1) / (16 * mt) + (a.num_slots < a.E ? a.num_slots : a.E) / 2;
    // (measured on the 256-expert decode shape: seven or eight 8-stage tiles per workgroup beat five,
    // as long as about 1500 workgroups remain)
    while (tpw > 1 && est_blocks * ((p.n_tiles + tpw - 1) / tpw) * ksp < 1536) --tpw;
  }
  if (g_force_tpw > 0) tpw = szr ? (g_force_tpw < p.n_tiles ? g_force_tpw : p.n_tiles) : 1;
  p.tiles_per_wg = tpw;
  const long long grid = (long long)(cap / (16 * mt)) * ((p.n_tiles + tpw - 1) / tpw) * ksp;
  if (grid > 0x7fffffffLL) return fail(MOE_UNSUPPORTED_SHAPE, "grid too large");
  g_last_plan[0] = mt; g_last_plan[1] = nt; g_last_plan[2] = ks; g_last_plan[3] = szr;
  g_last_plan[4] = tpw; g_last_plan[5] = ksp; g_last_plan[6] = kspan; g_last_plan[7] = fuse;
  g_last_plan[8] = wv;
  const int err = v->fn(p, (int)grid, stream);
  if (err != 0) return hip_fail(err, "grouped GEMM launch");
  return MOE_OK;
}

// wide_shape: the layer's shapes admit the eight-wave tile; wide_tile: it will be used (not with
// operand-order weights, which only the four-wave tiles read)
static int pick_block_m(long long S, int E, bool wide_shape = false, bool wide_tile = false) {
  const long long avg = S / (E > 0 ? E : 1);
  if (avg <= 8) return 16;
  if (avg <= (wide_shape ? 28 : 24)) return 32;
  // 128-slot blocks only for the eight-wave tile (every unpacked weight feeds up to eight matrix
  // instructions and its main loop skips the block's empty 16-row sub-tiles, so a block that is a
  // quarter full costs a quarter of the matrix work); the four-wave 128-slot tiles run one
  // workgroup per CU and lose to 64-slot ones.  Measured on the 256-expert layer shape: 32 rows per
  // expert 1.73 against 1.88 ms, 48 rows a tie, 64 rows 2.40 against 2.90 ms; up to 28 rows the
  // 32-slot tile wins (28 rows: 1.65 ms for both, 64-slot blocks 1.86).
  if (wide_tile) return 128;
  return 64;
}

// Can both projections of a layer run on the eight-wave tile?  (group 128, whole 8-group scale
// panels in K and N; pointer alignment is checked again at launch)
static bool layer_wide_ok(int K, int N, int group_size) {
  return group_size == 128 && K % 1024 == 0 && N % 1024 == 0 && g_wide_mode != 1 && g_force_mt == 0 && g_force_nt == 0;
}

// Reduction splits of the layer's down projection.  With few experts and few rows the launch has
// too few workgroups to keep enough loads in flight; cutting the reduction multiplies them (the
// combine adds the partial planes).  Only for small token tiles: large ones have rows to spare.
static int pick_k_splits(long long S, int E, int K, int N, int block_m) {
  if (block_m > 32) return 1;
  const long long est_blocks = (S + block_m - 1) / block_m + (S < E ? S : E) / 2;
  const long long wgs = est_blocks * ((K + 127) / 128);
  if (wgs <= 0 || wgs >= 768) return 1;
  long long want = (768 + wgs - 1) / wgs;      // about one workgroup per resident slot (3 per CU)
  const int npan = N / 1024;
  if (want > npan) want = npan;
  if (want > 8) want = 8;
  return want < 1 ? 1 : (int)want;
}

struct Workspace {
  size_t counts, offsets, num_padded, sorted, blocks, act, Y, total;
};
static Workspace carve(long long T, int K, int N, int E, int topk) {
  const long long S = T * topk;
  Workspace w;
  size_t o = 0;
  w.counts = o;      o += round_up((size_t)E * 4, 256);
  w.offsets = o;     o += round_up((size_t)(E + 1) * 4, 256);
  w.num_padded = o;  o += 256;
  w.sorted = o;      o += round_up(align_capacity(S, E, 256) * 4, 256);   // the largest block any caller can force
  w.blocks = o;      o += round_up((align_capacity(S, E, 16) / 16 + 1) * 4, 256);
  w.act = o;         o += round_up((size_t)S * N * 2, 256);
  // float32 (combined unrounded); one plane per reduction split (at most 8, small batches only)
  w.Y = o;           o += round_up((size_t)S * K * 4 * std::max(pick_k_splits(S, E, K, N, pick_block_m(S, E)),
                                                            pick_k_splits(S, E, K, N, pick_block_m(S, E, true))), 256);
  w.total = o;
  return w;
}

}  // namespace moe

using namespace moe;

// ---- blockwise-scaled FP8 GEMM: tile and split choice --------------------------------------
static thread_local int g_fp8_mt = 0, g_fp8_nt = 0, g_fp8_splits = 0, g_fp8_group_m = 0;

struct Fp8Plan { int bm, bn, splits, kb_per_split; };

// false: the (forced) plan does not fit the shape
static bool fp8_plan(int M, int N, int K, Fp8Plan& pl) {
  const int KB = K / 128;
  int bm = M <= 16 ? 16 : M <= 32 ? 32 : M <= 64 ? 64 : 128;
  // 128 features per workgroup measured fastest at every token-tile height up to 128 (two or
  // more workgroups per CU; 256 wide costs occupancy, 64 wide LDS traffic per matrix
  // instruction).  Large problems take the 256 x 256 eight-wave tile (fewest LDS bytes per
  // matrix instruction: 1.65-1.8 against 1.4-1.5 PFLOP/s) when it still yields two workgroups per CU.
  int bn = 128;
  if (M > 128 && N % 256 == 0 && (long long)((M + 255) / 256) * (N / 256) >= 512) { bm = 256; bn = 256; }
  // a few hundred rows: 64-token tiles when 128-token tiles would leave CUs without a second workgroup
  else if (M > 128 && N % 128 == 0 && (long long)((M + 127) / 128) * (N / 128) < 512) bm = 64;
  if (g_fp8_mt) { bm = 16 * g_fp8_mt; bn = 128; }
  if (bm != 16 && bm != 32 && bm != 64 && bm != 128 && bm != 256) return false;
  const long long m_blocks = (M + bm - 1) / bm;
  while (bn > 64 && N % bn != 0) bn >>= 1;
  // small problems: narrower feature tiles first (more workgroups streaming weights) ...
  while (bn > 64 && m_blocks * (N / bn) < 256) bn >>= 1;
  if (g_fp8_nt) bn = 64 * g_fp8_nt;
  if ((bn != 64 && bn != 128 && bn != 256) || N % bn != 0 || (bm == 256 && bn == 64)) return false;
  const long long wgs = m_blocks * (N / bn);
  // ... then a split of the reduction, each split at least four blocks long
  int splits = 1;
  if (wgs < 256) {
    splits = (int)((768 + wgs - 1) / wgs);
    if (splits > KB / 4) splits = KB / 4;
    if (splits > 16) splits = 16;
    if (splits < 1) splits = 1;
  }
  if (g_fp8_splits) splits = g_fp8_splits;
  if (splits < 1 || splits > KB) return false;
  const int per = (KB + splits - 1) / splits;
  splits = (KB + per - 1) / per;                       // no empty split
  pl = Fp8Plan{bm, bn, splits, per};
  return true;
}

extern "C" {

const char* moe_last_error(void) { return g_err; }

size_t moe_align_capacity(int T, int topk, int E, int block_m) {
  if (T < 0 || topk < 1 || E < 1 || !valid_block_m(block_m)) return 0;
  return align_capacity((long long)T * topk, E, block_m);
}

int moe_align_by_expert(const int32_t* topk_ids, int T, int topk, int E, int block_m,
                        int32_t* expert_counts, int32_t* expert_offsets, int32_t* sorted_slot_ids,
                        int32_t* block_expert_ids, int32_t* num_padded, void* stream) {
  if (T < 0 || topk < 1 || E < 1) return fail(MOE_INVALID_ARGUMENT, "need T >= 0, topk >= 1, E >= 1");
  if (!valid_block_m(block_m)) return fail(MOE_INVALID_ARGUMENT, "block_m must be 16, 32, 64, 128 or 256");
  if (E > 1024) return fail(MOE_UNSUPPORTED_SHAPE, "E = %d exceeds 1024", E);
  const long long S = (long long)T * topk;
  if (S > 0x7fffffffLL / 2) return fail(MOE_UNSUPPORTED_SHAPE, "T*topk too large");
  if (!expert_counts || !expert_offsets || !num_padded || (S > 0 && (!topk_ids || !sorted_slot_ids || !block_expert_ids)))
    return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  const size_t cap = align_capacity(S, E, block_m);
  const int err = launch_align(topk_ids, (int)S, E, block_m, (int)cap, expert_counts, expert_offsets,
                               sorted_slot_ids, block_expert_ids, num_padded, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "align launch");
  return MOE_OK;
}

int moe_w4a16_grouped_gemm(const void* A, int row_div, const int32_t* qweight, const void* scales,
                           const uint8_t* zeros, const int32_t* sorted_slot_ids,
                           const int32_t* block_expert_ids, const int32_t* num_padded, int num_slots,
                           int E, int N_out, int K_in, int group_size, int block_m, moe_dtype dt,
                           void* C, void* stream) {
  GemmArgs a{A, row_div, qweight, scales, zeros, sorted_slot_ids, block_expert_ids, num_padded,
             num_slots, E, N_out, K_in, group_size, block_m, (int)dt, C, N_out, 0, 0};
  return run_gemm(a, (hipStream_t)stream);
}

int moe_w4a16_dense_gemm(const void* A, const int32_t* qweight, const void* scales, const uint8_t* zeros,
                         int M, int N_out, int K_in, int group_size, moe_dtype dt, void* C, void* stream) {
  if (M < 0) return fail(MOE_INVALID_ARGUMENT, "need M >= 0");
  const int block_m = M <= 16 ? 16 : (M <= 32 ? 32 : 64);
  GemmArgs a{A, 1, qweight, scales, zeros, nullptr, nullptr, nullptr,
             M, 1, N_out, K_in, group_size, block_m, (int)dt, C, N_out, 0, 0};
  a.dense = 1;
  return run_gemm(a, (hipStream_t)stream);
}

int moe_route_topk(const float* logits, const float* bias, int T, int E, int topk,
                   int32_t* topk_ids, float* topk_weights, void* stream) {
  if (T < 0 || E < 1 || topk < 1) return fail(MOE_INVALID_ARGUMENT, "need T >= 0, E >= 1, topk >= 1");
  if (E > 1024) return fail(MOE_UNSUPPORTED_SHAPE, "E = %d exceeds 1024", E);
  if (topk > E || topk > 64) return fail(MOE_UNSUPPORTED_SHAPE, "topk = %d exceeds min(E, 64)", topk);
  if (T == 0) return MOE_OK;
  if (!logits || !topk_ids || !topk_weights) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  const int err = launch_route_topk(logits, bias, T, E, topk, topk_ids, topk_weights, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "router launch");
  return MOE_OK;
}

int moe_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes < 16 || ((uintptr_t)src % 16) != 0)
    return fail(MOE_INVALID_ARGUMENT, "probe needs a 16-byte aligned source of at least 16 bytes and a sink");
  const int err = launch_stream_read(src, bytes, (uint32_t*)sink, 256 * 16, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "stream-read probe launch");
  return MOE_OK;
}

int moe_probe_mfma(void* sink, int iters, void* stream) {
  if (!sink || iters < 1) return fail(MOE_INVALID_ARGUMENT, "probe needs a sink and iters >= 1");
  const int err = launch_mfma_loop((float*)sink, 512, iters, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "MFMA probe launch");
  return MOE_OK;
}

int moe_probe_issue_mix(void* sink, int iters, int valu_per_mfma, int lds_reads_per_8_mfma, void* stream) {
  if (!sink || iters < 1) return fail(MOE_INVALID_ARGUMENT, "probe needs a sink and iters >= 1");
  const int err = launch_issue_mix((float*)sink, iters, valu_per_mfma, lds_reads_per_8_mfma, (hipStream_t)stream);
  if (err == -1)
    return fail(MOE_UNSUPPORTED_SHAPE, "issue-mix probe: valu_per_mfma must be 0, 1, 2, 3, 4 or 6 and "
                "lds_reads_per_8_mfma 0, 2, 4 or 8");
  if (err != 0) return hip_fail(err, "issue-mix probe launch");
  return MOE_OK;
}

int moe_silu_mul(const void* H, void* act, int S, int N, moe_dtype dt, void* stream) {
  if (S < 0 || N < 1) return fail(MOE_INVALID_ARGUMENT, "need S >= 0 and N >= 1");
  if (dt != MOE_F16 && dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (S == 0) return MOE_OK;
  if (!H || !act) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (N % 8 == 0 && ((uintptr_t)H | (uintptr_t)act) % 16 != 0)
    return fail(MOE_INVALID_ARGUMENT, "H and act must be 16-byte aligned");
  const int err = launch_silu_mul(H, act, S, N, (int)dt, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "silu_mul launch");
  return MOE_OK;
}

int moe_combine(const void* Y, const float* topk_weights, void* out, int T, int topk, int K, moe_dtype dt,
                void* stream) {
  if (T < 0 || topk < 1 || K < 1) return fail(MOE_INVALID_ARGUMENT, "need T >= 0, topk >= 1, K >= 1");
  if (dt != MOE_F16 && dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (T == 0) return MOE_OK;
  if (!Y || !topk_weights || !out) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (K % 8 == 0 && ((uintptr_t)Y | (uintptr_t)out) % 16 != 0)
    return fail(MOE_INVALID_ARGUMENT, "Y and out must be 16-byte aligned");
  const int err = launch_combine(Y, 0, 1, topk_weights, nullptr, 0, out, T, topk, K, (int)dt, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "combine launch");
  return MOE_OK;
}

int moe_combine_masked(const void* Y, const float* topk_weights, const int32_t* topk_ids, int E, void* out, int T,
                       int topk, int K, moe_dtype dt, void* stream) {
  if (T < 0 || topk < 1 || K < 1 || E < 1) return fail(MOE_INVALID_ARGUMENT, "need T >= 0, topk >= 1, K >= 1, E >= 1");
  if (dt != MOE_F16 && dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (T == 0) return MOE_OK;
  if (!Y || !topk_weights || !topk_ids || !out) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (K % 8 == 0 && ((uintptr_t)Y | (uintptr_t)out) % 16 != 0)
    return fail(MOE_INVALID_ARGUMENT, "Y and out must be 16-byte aligned");
  const int err = launch_combine(Y, 0, 1, topk_weights, topk_ids, E, out, T, topk, K, (int)dt, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "combine launch");
  return MOE_OK;
}

size_t moe_w4a16_layer_workspace_bytes(int T, int K, int N, int E, int topk, moe_dtype dt) {
  (void)dt;
  if (T < 0 || K < 1 || N < 1 || E < 1 || topk < 1) return 0;
  return carve(T, K, N, E, topk).total;
}

int moe_layer_block_m(int T, int E, int topk) {
  if (T < 0 || E < 1 || topk < 1) return 0;
  return pick_block_m((long long)T * topk, E);
}

int moe_layer_block_m_for(int T, int K, int N, int E, int topk, int group_size) {
  if (T < 0 || K < 1 || N < 1 || E < 1 || topk < 1 || group_size < 1) return 0;
  if (g_force_block_m > 0) return g_force_block_m;
  return pick_block_m((long long)T * topk, E, layer_wide_ok(K, N, group_size), layer_wide_ok(K, N, group_size));
}

}  // extern "C"

// Up to this many tokens the router runs inside the bucketing workgroup (one launch); beyond it the
// many-workgroup router kernel plus the bucketing kernel are faster than one CU routing everything
// (measured, 256 experts, top-8: fused 10.6 / 15.0 / 23.4 us at 16 / 64 / 128 tokens against
// 15.1 us for the two launches).
constexpr int kFusedRouteMaxTokens = 64;

struct RouteArgs {            // routed layer: the layer's first step computes ids / weights itself
  const float* logits = nullptr;
  const float* bias = nullptr;
  int32_t* ids = nullptr;     // [T, topk] tables to fill (inside the caller's workspace)
  float* weights = nullptr;
};

// router (+ bucketing): one launch for small batches, two otherwise
static int route_and_align(const RouteArgs& r, int T, int E, int topk, int block_m, int32_t* counts, int32_t* offsets,
                           int32_t* sorted, int32_t* blocks, int32_t* num_padded, hipStream_t stream) {
  const long long S = (long long)T * topk;
  const int cap = (int)align_capacity(S, E, block_m);
  int err;
  if (T <= kFusedRouteMaxTokens) {
    err = launch_route_align(r.logits, r.bias, T, E, topk, r.ids, r.weights, block_m, cap, counts, offsets, sorted,
                             blocks, num_padded, stream);
    if (err != 0) return hip_fail(err, "router + align launch");
    return MOE_OK;
  }
  err = launch_route_topk(r.logits, r.bias, T, E, topk, r.ids, r.weights, stream);
  if (err != 0) return hip_fail(err, "router launch");
  err = launch_align(r.ids, (int)S, E, block_m, cap, counts, offsets, sorted, blocks, num_padded, stream);
  if (err != 0) return hip_fail(err, "align launch");
  return MOE_OK;
}

static int layer_impl(const void* X, const int32_t* topk_ids, const float* topk_weights,
                      const int32_t* qw1, const void* s1, const uint8_t* z1,
                      const int32_t* qw2, const void* s2, const uint8_t* z2,
                      void* out, int T, int K, int N, int E, int topk, int group_size, moe_dtype dt,
                      void* workspace, size_t workspace_bytes, void* stream_v, int pre,
                      const RouteArgs* route = nullptr) {
  hipStream_t stream = (hipStream_t)stream_v;
  if (T < 0 || K < 1 || N < 1 || E < 1 || topk < 1 || group_size < 1)
    return fail(MOE_INVALID_ARGUMENT, "need T >= 0 and positive K, N, E, topk, group_size");
  if (dt != MOE_F16 && dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (E > 1024) return fail(MOE_UNSUPPORTED_SHAPE, "E = %d exceeds 1024", E);
  if (group_size % 32 != 0 || K % group_size != 0 || N % group_size != 0)
    return fail(MOE_UNSUPPORTED_SHAPE, "group_size %d must be a multiple of 32 dividing K=%d and N=%d", group_size, K, N);
  if (K % 16 != 0 || N % 16 != 0) return fail(MOE_UNSUPPORTED_SHAPE, "K and N must be multiples of 16");
  if (K / group_size > kMaxGroups || N / group_size > kMaxGroups)
    return fail(MOE_UNSUPPORTED_SHAPE, "more than %d quantisation groups per row", kMaxGroups);
  if (T == 0) return MOE_OK;
  if (!X || !topk_ids || !topk_weights || !qw1 || !s1 || !z1 || !qw2 || !s2 || !z2 || !out || !workspace)
    return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (((uintptr_t)workspace % 256) != 0) return fail(MOE_INVALID_ARGUMENT, "workspace must be 256-byte aligned");
  if (((uintptr_t)out % 16) != 0) return fail(MOE_INVALID_ARGUMENT, "out must be 16-byte aligned");
  const Workspace w = carve(T, K, N, E, topk);
  if (workspace_bytes < w.total)
    return fail(MOE_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  const long long S = (long long)T * topk;
  if (S > 0x7fffffffLL / 2) return fail(MOE_UNSUPPORTED_SHAPE, "T*topk too large");

  unsigned char* base = (unsigned char*)workspace;
  int32_t* counts = (int32_t*)(base + w.counts);
  int32_t* offsets = (int32_t*)(base + w.offsets);
  int32_t* num_padded = (int32_t*)(base + w.num_padded);
  int32_t* sorted = (int32_t*)(base + w.sorted);
  int32_t* blocks = (int32_t*)(base + w.blocks);
  void* act = base + w.act;
  void* Y = base + w.Y;
  // a forced bucketing block wins; a forced token tile (tuning hook) also fixes the block
  const int block_m = g_force_block_m > 0 ? g_force_block_m
                      : (g_force_mt == 1 || g_force_mt == 2 || g_force_mt == 4 || g_force_mt == 8)
                          ? 16 * g_force_mt : pick_block_m(S, E, layer_wide_ok(K, N, group_size), !pre && layer_wide_ok(K, N, group_size));
  const bool ev = g_nevents == 5;

  if (ev) (void)hipEventRecord((hipEvent_t)g_events[0], stream);
  int err;
  if (route) {
    const int rst = route_and_align(*route, T, E, topk, block_m, counts, offsets, sorted, blocks, num_padded, stream);
    if (rst != MOE_OK) return rst;
  } else {
    err = launch_align(topk_ids, (int)S, E, block_m, (int)align_capacity(S, E, block_m), counts, offsets,
                       sorted, blocks, num_padded, stream);
    if (err != 0) return hip_fail(err, "align launch");
  }

  if (ev) (void)hipEventRecord((hipEvent_t)g_events[1], stream);
  GemmArgs g1{X, topk, qw1, s1, z1, sorted, blocks, num_padded, (int)S, E, 2 * N, K, group_size, block_m,
              (int)dt, act, N, N, 0};
  g1.pre = pre;
  int st = run_gemm(g1, stream);
  if (st != MOE_OK) return st;

  if (ev) (void)hipEventRecord((hipEvent_t)g_events[2], stream);
  GemmArgs g2{act, 1, qw2, s2, z2, sorted, blocks, num_padded, (int)S, E, K, N, group_size, block_m,
              (int)dt, Y, K, 0, 1};
  // reduction splits: as many partial planes as the caller's workspace holds
  int want = g_force_ksplit > 0 ? g_force_ksplit : pick_k_splits(S, E, K, N, block_m);
  const size_t planes_fit = (workspace_bytes - w.Y) / ((size_t)S * K * 4);
  if ((size_t)want > planes_fit) want = (int)planes_fit;
  int planes = 1;
  g2.k_splits = want;
  g2.used_splits = &planes;
  g2.pre = pre;
  st = run_gemm(g2, stream);
  if (st != MOE_OK) return st;

  if (ev) (void)hipEventRecord((hipEvent_t)g_events[3], stream);
  err = launch_combine(Y, 1, planes, topk_weights, topk_ids, E, out, T, topk, K, (int)dt, stream);
  if (err != 0) return hip_fail(err, "combine launch");
  if (ev) (void)hipEventRecord((hipEvent_t)g_events[4], stream);
  return MOE_OK;
}

extern "C" {

int moe_w4a16_layer(const void* X, const int32_t* topk_ids, const float* topk_weights,
                    const int32_t* qw1, const void* s1, const uint8_t* z1,
                    const int32_t* qw2, const void* s2, const uint8_t* z2,
                    void* out, int T, int K, int N, int E, int topk, int group_size, moe_dtype dt,
                    void* workspace, size_t workspace_bytes, void* stream) {
  return layer_impl(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, out, T, K, N, E, topk, group_size, dt,
                    workspace, workspace_bytes, stream, 0);
}

int moe_w4a16_layer_prepacked(const void* X, const int32_t* topk_ids, const float* topk_weights,
                              const int32_t* qw1p, const void* s1, const uint8_t* z1,
                              const int32_t* qw2p, const void* s2, const uint8_t* z2,
                              void* out, int T, int K, int N, int E, int topk, int group_size, moe_dtype dt,
                              void* workspace, size_t workspace_bytes, void* stream) {
  return layer_impl(X, topk_ids, topk_weights, qw1p, s1, z1, qw2p, s2, z2, out, T, K, N, E, topk, group_size, dt,
                    workspace, workspace_bytes, stream, 1);
}

// ---- the layer for callers that cannot allocate ---------------------------------------------
// Same kernels as moe_w4a16_layer; the bucketing tables, `act` and the float32 down-projection
// planes live in a fixed device array of this module instead of a caller workspace.  Every GPU
// the library runs on holds its own copy of the array (at its own address) until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device, resolved once per device.  (In host code the
// array's name is only a handle for hipGetSymbolAddress, never an address to hand to a kernel.)
static int static_scratch(void** ptr) {
  constexpr int kMaxDev = 64;
  static void* ptrs[kMaxDev] = {};
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return hip_fail((int)err, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDev) return fail(MOE_UNSUPPORTED_SHAPE, "device index %d outside [0, %d)", dev, kMaxDev);
  void* p = __atomic_load_n(&ptrs[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess || !p) return hip_fail((int)err, "hipGetSymbolAddress(scratch)");
    __atomic_store_n(&ptrs[dev], p, __ATOMIC_RELEASE);      // racing first calls resolve the same address
  }
  *ptr = p;
  return MOE_OK;
}

int moe_w4a16_layer_noalloc(const void* X, const int32_t* topk_ids, const float* topk_weights,
                            const int32_t* qw1, const void* s1, const uint8_t* z1,
                            const int32_t* qw2, const void* s2, const uint8_t* z2,
                            void* out, int T, int K, int N, int E, int topk, int group_size, moe_dtype dt,
                            void* stream) {
  if (T < 0 || K < 1 || N < 1 || E < 1 || topk < 1)
    return fail(MOE_INVALID_ARGUMENT, "need T >= 0 and positive K, N, E, topk, group_size");
  const size_t need = carve(T, K, N, E, topk).total;
  if (need > kStaticScratchBytes)
    return fail(MOE_WORKSPACE_TOO_SMALL,
                "moe_w4a16_layer_noalloc: these sizes need %zu bytes of scratch, the built-in array holds %zu; "
                "use moe_w4a16_layer with a caller workspace", need, kStaticScratchBytes);
  void* ptr = nullptr;
  const int st = static_scratch(&ptr);
  if (st != MOE_OK) return st;
  // nothing in the array has to start at zero: the bucketing kernel writes every table entry it or
  // the GEMMs read, and act / Y rows are read only for slots whose rows this call wrote
  return layer_impl(X, topk_ids, topk_weights, qw1, s1, z1, qw2, s2, z2, out, T, K, N, E, topk, group_size, dt,
                    ptr, kStaticScratchBytes, stream, 0);
}

int moe_repack_qweight(const int32_t* qweight, int E, int N_out, int K_in, int paired, int32_t* out, void* stream) {
  if (E < 1 || N_out < 1 || K_in < 1) return fail(MOE_INVALID_ARGUMENT, "need positive E, N_out, K_in");
  if (K_in % 128 != 0 || N_out % (paired ? 32 : 16) != 0)
    return fail(MOE_UNSUPPORTED_SHAPE, "repack needs K_in %% 128 == 0 and N_out %% %d == 0", paired ? 32 : 16);
  if (!qweight || !out || qweight == out) return fail(MOE_INVALID_ARGUMENT, "null or aliased pointer argument");
  if ((((uintptr_t)qweight | (uintptr_t)out) % 16) != 0)
    return fail(MOE_INVALID_ARGUMENT, "qweight and out must be 16-byte aligned");
  const int err = launch_repack(qweight, E, N_out, K_in, paired ? 1 : 0, out, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "repack launch");
  return MOE_OK;
}

int moe_import_awq(const int32_t* awq_qweight, const int32_t* awq_qzeros, const void* awq_scales, int E, int K_in,
                   int N_out, int group_size, int32_t* qweight, void* scales, uint8_t* zeros, void* stream) {
  if (E < 1 || K_in < 1 || N_out < 1 || group_size < 1)
    return fail(MOE_INVALID_ARGUMENT, "need positive E, K_in, N_out, group_size");
  if (E > 65535) return fail(MOE_UNSUPPORTED_SHAPE, "import handles at most 65535 experts per call");
  if (K_in % 8 != 0 || N_out % 8 != 0 || K_in % group_size != 0)
    return fail(MOE_UNSUPPORTED_SHAPE, "import needs K_in %% 8 == 0, N_out %% 8 == 0, K_in %% group_size == 0");
  if (!awq_qweight || !awq_qzeros || !awq_scales || !qweight || !scales || !zeros)
    return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if ((const void*)awq_qweight == (const void*)qweight || awq_scales == (const void*)scales)
    return fail(MOE_INVALID_ARGUMENT, "the import does not work in place");
  if (((uintptr_t)awq_qweight | (uintptr_t)awq_qzeros | (uintptr_t)qweight) % 4 != 0 ||
      ((uintptr_t)awq_scales | (uintptr_t)scales) % 2 != 0)
    return fail(MOE_INVALID_ARGUMENT, "word tensors must be 4-byte, scale tensors 2-byte aligned");
  const int err = launch_awq_import(awq_qweight, awq_qzeros, awq_scales, E, K_in, N_out, group_size, qweight, scales,
                                    zeros, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "AWQ import launch");
  return MOE_OK;
}

size_t moe_w4a16_routed_layer_workspace_bytes(int T, int K, int N, int E, int topk, moe_dtype dt) {
  const size_t layer = moe_w4a16_layer_workspace_bytes(T, K, N, E, topk, dt);
  if (layer == 0 && T != 0) return 0;
  if (T < 0 || topk < 1) return 0;
  // routing tables in front of the layer's own workspace: ids int32 [S], weights float32 [S]
  return 2 * round_up((size_t)T * topk * 4, 256) + layer;
}

int moe_w4a16_routed_layer(const void* X, const float* logits, const float* bias,
                           const int32_t* qw1, const void* s1, const uint8_t* z1,
                           const int32_t* qw2, const void* s2, const uint8_t* z2,
                           void* out, int T, int K, int N, int E, int topk, int group_size, moe_dtype dt,
                           void* workspace, size_t workspace_bytes, void* stream) {
  if (T < 0 || topk < 1 || E < 1) return fail(MOE_INVALID_ARGUMENT, "need T >= 0, topk >= 1, E >= 1");
  if (T == 0) return MOE_OK;
  if (!workspace) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (((uintptr_t)workspace % 256) != 0) return fail(MOE_INVALID_ARGUMENT, "workspace must be 256-byte aligned");
  const size_t table = round_up((size_t)T * topk * 4, 256);
  if (workspace_bytes < 2 * table)
    return fail(MOE_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes,
                moe_w4a16_routed_layer_workspace_bytes(T, K, N, E, topk, dt));
  if (E > 1024) return fail(MOE_UNSUPPORTED_SHAPE, "E = %d exceeds 1024", E);
  if (topk > E || topk > 64) return fail(MOE_UNSUPPORTED_SHAPE, "topk = %d exceeds min(E, 64)", topk);
  if (!logits) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  unsigned char* base = (unsigned char*)workspace;
  RouteArgs r;
  r.logits = logits; r.bias = bias;
  r.ids = (int32_t*)base;
  r.weights = (float*)(base + table);
  return layer_impl(X, r.ids, r.weights, qw1, s1, z1, qw2, s2, z2, out, T, K, N, E, topk, group_size, dt,
                    base + 2 * table, workspace_bytes - 2 * table, stream, 0, &r);
}

int moe_route_align(const float* logits, const float* bias, int T, int E, int topk, int block_m,
                    int32_t* topk_ids, float* topk_weights, int32_t* expert_counts, int32_t* expert_offsets,
                    int32_t* sorted_slot_ids, int32_t* block_expert_ids, int32_t* num_padded, void* stream) {
  if (T < 0 || E < 1 || topk < 1) return fail(MOE_INVALID_ARGUMENT, "need T >= 0, E >= 1, topk >= 1");
  if (!valid_block_m(block_m)) return fail(MOE_INVALID_ARGUMENT, "block_m must be 16, 32, 64, 128 or 256");
  if (E > 1024) return fail(MOE_UNSUPPORTED_SHAPE, "E = %d exceeds 1024", E);
  if (topk > E || topk > 64) return fail(MOE_UNSUPPORTED_SHAPE, "topk = %d exceeds min(E, 64)", topk);
  const long long S = (long long)T * topk;
  if (S > 0x7fffffffLL / 2) return fail(MOE_UNSUPPORTED_SHAPE, "T*topk too large");
  if (!expert_counts || !expert_offsets || !num_padded ||
      (S > 0 && (!logits || !topk_ids || !topk_weights || !sorted_slot_ids || !block_expert_ids)))
    return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  RouteArgs r;
  r.logits = logits; r.bias = bias; r.ids = topk_ids; r.weights = topk_weights;
  return route_and_align(r, T, E, topk, block_m, expert_counts, expert_offsets, sorted_slot_ids, block_expert_ids,
                         num_padded, (hipStream_t)stream);
}

int moe_set_stage_events(void* const* events, int n) {
  if (n == 0 || events == nullptr) { g_nevents = 0; return MOE_OK; }
  if (n != 5 && n != 7) return fail(MOE_INVALID_ARGUMENT, "expected 5 events (16-bit layer) or 7 (FP8 layer)");
  for (int i = 0; i < n; ++i) g_events[i] = events[i];
  g_nevents = n;
  return MOE_OK;
}

int moe_set_scale_path(int mode) {
  if (mode < 0 || mode > 2) return fail(MOE_INVALID_ARGUMENT, "scale path mode must be 0, 1 or 2");
  g_scale_path = mode;
  return MOE_OK;
}

int moe_set_tiles_per_workgroup(int n) {
  if (n < 0 || n > 64) return fail(MOE_INVALID_ARGUMENT, "tiles per workgroup must be in 0..64");
  g_force_tpw = n;
  return MOE_OK;
}

int moe_set_reduction_splits(int n) {
  if (n < 0 || n > 64) return fail(MOE_INVALID_ARGUMENT, "reduction splits must be in 0..64");
  g_force_ksplit = n;
  return MOE_OK;
}

int moe_set_block_m_override(int block_m) {
  if (block_m != 0 && !valid_block_m(block_m))
    return fail(MOE_INVALID_ARGUMENT, "block_m override must be 0, 16, 32, 64, 128 or 256");
  g_force_block_m = block_m;
  return MOE_OK;
}

int moe_last_gemm_plan(int* plan9) {
  if (!plan9) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  for (int i = 0; i < 9; ++i) plan9[i] = g_last_plan[i];
  return MOE_OK;
}

int moe_set_wide_tiles(int mode) {
  if (mode < 0 || mode > 1) return fail(MOE_INVALID_ARGUMENT, "wide tile mode must be 0 (when usable) or 1 (never)");
  g_wide_mode = mode;
  return MOE_OK;
}

int moe_set_tile_override(int mt, int nt) {
  if (mt < 0 || nt < 0) return fail(MOE_INVALID_ARGUMENT, "negative tile override");
  g_force_mt = mt; g_force_nt = nt;
  return MOE_OK;
}

// ---- blockwise-scaled FP8 GEMM (include/fp8_blockwise_gemm.h) -------------------------------
size_t fp8_blockwise_gemm_workspace_bytes(int M, int N, int K) {
  if (M < 1 || N < 64 || K < 128 || K % 128 != 0 || N % 64 != 0) return 0;
  Fp8Plan pl;
  if (!fp8_plan(M, N, K, pl)) return 0;
  return pl.splits > 1 ? round_up((size_t)pl.splits * (size_t)M * (size_t)N * sizeof(float), 256) : 0;
}

int fp8_blockwise_gemm(const uint8_t* A, const float* a_scale, const uint8_t* B, const float* b_scale, void* C,
                       int M, int N, int K, int out_dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (M < 0 || N < 1 || K < 1) return fail(MOE_INVALID_ARGUMENT, "need M >= 0, N >= 1, K >= 1");
  if (out_dtype < 0 || out_dtype > 2)
    return fail(MOE_INVALID_ARGUMENT, "out_dtype must be 0 (fp16), 1 (bf16) or 2 (float32)");
  if (K % 128 != 0 || N % 64 != 0)
    return fail(MOE_UNSUPPORTED_SHAPE, "the FP8 GEMM needs K %% 128 == 0 and N %% 64 == 0 (got N=%d K=%d)", N, K);
  if (M == 0) return MOE_OK;
  if (!A || !a_scale || !B || !b_scale || !C) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) % 16 != 0 || ((uintptr_t)a_scale | (uintptr_t)b_scale) % 4 != 0)
    return fail(MOE_INVALID_ARGUMENT, "A, B, C must be 16-byte aligned, the scales 4-byte aligned");
  if (C == (const void*)A || C == (const void*)B) return fail(MOE_INVALID_ARGUMENT, "C must not alias an input");
  Fp8Plan pl;
  if (!fp8_plan(M, N, K, pl)) return fail(MOE_UNSUPPORTED_SHAPE, "the forced FP8 plan does not fit M=%d N=%d K=%d", M, N, K);
  if ((unsigned long long)M * (unsigned long long)K >= (1ull << 32) ||
      (unsigned long long)N * (unsigned long long)K >= (1ull << 32))
    return fail(MOE_UNSUPPORTED_SHAPE, "the FP8 GEMM addresses A and B with 32-bit offsets: M * K and N * K must be below 2^32");
  const long long m_blocks = (M + pl.bm - 1) / pl.bm;
  const long long grid = m_blocks * (N / pl.bn) * pl.splits;
  if (grid > 0x7fffffffLL) return fail(MOE_UNSUPPORTED_SHAPE, "too many workgroups");
  fp8::GemmParams p = {};
  p.A = A; p.a_scale = a_scale; p.B = B; p.b_scale = b_scale;
  p.M = M; p.N = N; p.K = K;
  p.k_splits = pl.splits; p.kb_per_split = pl.kb_per_split; p.out_bf16 = out_dtype;
  p.group_m = g_fp8_group_m ? g_fp8_group_m : 8;     // row blocks per tile group (4 ... 16 measured alike)
  if (pl.splits > 1) {
    const size_t need = round_up((size_t)pl.splits * (size_t)M * (size_t)N * sizeof(float), 256);
    if (!workspace || workspace_bytes < need)
      return fail(MOE_WORKSPACE_TOO_SMALL, "FP8 GEMM workspace: need %zu bytes, got %zu", need, workspace_bytes);
    if ((uintptr_t)workspace % 256 != 0) return fail(MOE_INVALID_ARGUMENT, "workspace must be 256-byte aligned");
    p.C = workspace;
  } else {
    p.C = C;
  }
  int err = fp8::launch_fp8_gemm(p, pl.bm, pl.bn, (hipStream_t)stream);
  if (err == -1) return fail(MOE_UNSUPPORTED_SHAPE, "no FP8 GEMM variant for tile %d x %d", pl.bm, pl.bn);
  if (err != 0) return hip_fail(err, "FP8 GEMM launch");
  if (pl.splits > 1) {
    err = fp8::launch_fp8_split_reduce((const float*)workspace, pl.splits, (long long)M * N, C, out_dtype,
                                       (hipStream_t)stream);
    if (err != 0) return hip_fail(err, "FP8 split reduction launch");
  }
  return MOE_OK;
}

int fp8_moe_grouped_gemm(const uint8_t* A, const float* a_scale, int row_div, const uint8_t* B,
                         const float* b_scale, const int32_t* sorted_slot_ids, const int32_t* block_expert_ids,
                         const int32_t* num_padded, int num_slots, int E, int N, int K, int block_m, int out_dtype,
                         void* C, void* stream) {
  if (num_slots < 0 || E < 1 || E > 1024 || N < 1 || K < 1 || row_div < 1)
    return fail(MOE_INVALID_ARGUMENT, "need num_slots >= 0, 1 <= E <= 1024, N >= 1, K >= 1, row_div >= 1");
  if (out_dtype < 0 || out_dtype > 2)
    return fail(MOE_INVALID_ARGUMENT, "out_dtype must be 0 (fp16), 1 (bf16) or 2 (float32)");
  if (!valid_block_m(block_m)) return fail(MOE_INVALID_ARGUMENT, "block_m must be 16, 32, 64, 128 or 256");
  if (K % 128 != 0 || N % 64 != 0 || (block_m == 256 && N % 128 != 0))
    return fail(MOE_UNSUPPORTED_SHAPE,
                "the grouped FP8 GEMM needs K %% 128 == 0 and N %% 64 == 0 (N %% 128 == 0 at block_m 256); got N=%d K=%d",
                N, K);
  if (num_slots == 0) return MOE_OK;
  if (!A || !a_scale || !B || !b_scale || !sorted_slot_ids || !block_expert_ids || !num_padded || !C)
    return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (((uintptr_t)A | (uintptr_t)B | (uintptr_t)C) % 16 != 0 || ((uintptr_t)a_scale | (uintptr_t)b_scale) % 4 != 0)
    return fail(MOE_INVALID_ARGUMENT, "A, B, C must be 16-byte aligned, the scales 4-byte aligned");
  if (C == (const void*)A || C == (const void*)B) return fail(MOE_INVALID_ARGUMENT, "C must not alias an input");
  const unsigned long long rows_a = ((unsigned long long)num_slots + row_div - 1) / row_div;
  if (rows_a * (unsigned long long)K >= (1ull << 32) || (unsigned long long)N * (unsigned long long)K >= (1ull << 32))
    return fail(MOE_UNSUPPORTED_SHAPE, "32-bit operand offsets: rows(A) * K and N * K must be below 2^32");
  const size_t cap = align_capacity(num_slots, E, block_m);
  const int bn = N % 128 == 0 ? 128 : 64;
  const long long grid = (long long)(cap / block_m) * (N / bn);
  if (cap > 0x7fffffffULL || grid > 0x7fffffffLL) return fail(MOE_UNSUPPORTED_SHAPE, "too many workgroups");
  fp8::GemmParams p = {};
  p.A = A; p.a_scale = a_scale; p.B = B; p.b_scale = b_scale; p.C = C;
  p.M = (int)cap; p.N = N; p.K = K;
  p.k_splits = 1; p.kb_per_split = K / 128; p.out_bf16 = out_dtype;
  p.group_m = g_fp8_group_m ? g_fp8_group_m : 8;
  p.sorted_slot_ids = sorted_slot_ids; p.block_expert_ids = block_expert_ids; p.num_padded = num_padded;
  p.num_slots = num_slots; p.row_div = row_div;
  p.b_expert_stride = (size_t)N * (size_t)K;
  p.bs_expert_stride = (size_t)((N + 127) / 128) * (size_t)(K / 128);
  const int err = fp8::launch_fp8_gemm(p, block_m, bn, (hipStream_t)stream);
  if (err == -1) return fail(MOE_UNSUPPORTED_SHAPE, "no FP8 GEMM variant for tile %d x %d", block_m, bn);
  if (err != 0) return hip_fail(err, "grouped FP8 GEMM launch");
  return MOE_OK;
}

// ---- FP8 mixture-of-experts layer ------------------------------------------------------------
int fp8_quantize_rows(const void* X, int rows, int K, int dt, uint8_t* codes, float* scales, void* stream) {
  if (rows < 0 || K < 1) return fail(MOE_INVALID_ARGUMENT, "need rows >= 0 and K >= 1");
  if (dt != MOE_F16 && dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (K % 128 != 0) return fail(MOE_UNSUPPORTED_SHAPE, "the activation quantiser needs K %% 128 == 0 (got %d)", K);
  if (rows == 0) return MOE_OK;
  if (!X || !codes || !scales) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if ((uintptr_t)X % 16 != 0 || (uintptr_t)codes % 8 != 0 || (uintptr_t)scales % 4 != 0)
    return fail(MOE_INVALID_ARGUMENT, "X must be 16-byte, codes 8-byte, scales 4-byte aligned");
  const int err = fp8::launch_fp8_quantize(X, rows, K, (int)dt, 0, codes, scales, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "activation quantiser launch");
  return MOE_OK;
}

int fp8_silu_mul_quantize(const void* H, int S, int N, int dt, uint8_t* codes, float* scales, void* stream) {
  if (S < 0 || N < 1) return fail(MOE_INVALID_ARGUMENT, "need S >= 0 and N >= 1");
  if (dt != MOE_F16 && dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (N % 128 != 0) return fail(MOE_UNSUPPORTED_SHAPE, "the activation quantiser needs N %% 128 == 0 (got %d)", N);
  if (S == 0) return MOE_OK;
  if (!H || !codes || !scales) return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if ((uintptr_t)H % 16 != 0 || (uintptr_t)codes % 8 != 0 || (uintptr_t)scales % 4 != 0)
    return fail(MOE_INVALID_ARGUMENT, "H must be 16-byte, codes 8-byte, scales 4-byte aligned");
  const int err = fp8::launch_fp8_quantize(H, S, N, (int)dt, 1, codes, scales, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "SiLU-and-multiply quantiser launch");
  return MOE_OK;
}

static thread_local int g_fp8_layer_block_m = 0;

static int fp8_pick_block_m(long long S, int E) {
  if (g_fp8_layer_block_m > 0) return g_fp8_layer_block_m;
  const long long avg = S / (E > 0 ? E : 1);
  if (avg <= 32) return 32;      // measured: 32-token tiles stream the weights fastest at a few rows per expert
  if (avg >= 96) return 128;     // about one row block per expert: its weights are fetched once (measured +2 %)
  return 64;
}

struct Fp8Workspace { size_t counts, offsets, num_padded, sorted, blocks, xq, sx, H, aq, sa, Y, total; };
static Fp8Workspace fp8_carve(long long T, int K, int N, int E, int topk) {
  const long long S = T * topk;
  Fp8Workspace w;
  size_t o = 0;
  w.counts = o;      o += round_up((size_t)E * 4, 256);
  w.offsets = o;     o += round_up((size_t)(E + 1) * 4, 256);
  w.num_padded = o;  o += 256;
  w.sorted = o;      o += round_up(align_capacity(S, E, 256) * 4, 256);
  w.blocks = o;      o += round_up((align_capacity(S, E, 16) / 16 + 1) * 4, 256);
  w.xq = o;          o += round_up((size_t)T * K, 256);
  w.sx = o;          o += round_up((size_t)T * (K / 128) * 4, 256);
  w.H = o;           o += round_up((size_t)S * 2 * N * 2, 256);
  w.aq = o;          o += round_up((size_t)S * N, 256);
  w.sa = o;          o += round_up((size_t)S * (N / 128) * 4, 256);
  w.Y = o;           o += round_up((size_t)S * K * 4, 256);
  w.total = o;
  return w;
}

size_t fp8_moe_layer_workspace_bytes(int T, int K, int N, int E, int topk) {
  if (T < 0 || K < 128 || N < 128 || E < 1 || topk < 1 || K % 128 != 0 || N % 128 != 0) return 0;
  return fp8_carve(T, K, N, E, topk).total;
}

int fp8_set_layer_block_m(int block_m) {
  if (block_m != 0 && !valid_block_m(block_m))
    return fail(MOE_INVALID_ARGUMENT, "block_m override must be 0, 16, 32, 64, 128 or 256");
  g_fp8_layer_block_m = block_m;
  return MOE_OK;
}

int fp8_moe_layer(const void* X, const int32_t* topk_ids, const float* topk_weights,
                  const uint8_t* w1, const float* w1_scale, const uint8_t* w2, const float* w2_scale,
                  void* out, int T, int K, int N, int E, int topk, int dt,
                  void* workspace, size_t workspace_bytes, void* stream_v) {
  hipStream_t stream = (hipStream_t)stream_v;
  if (T < 0 || K < 1 || N < 1 || E < 1 || topk < 1)
    return fail(MOE_INVALID_ARGUMENT, "need T >= 0 and positive K, N, E, topk");
  if (dt != MOE_F16 && dt != MOE_BF16) return fail(MOE_INVALID_ARGUMENT, "dt must be MOE_F16 or MOE_BF16");
  if (E > 1024) return fail(MOE_UNSUPPORTED_SHAPE, "E = %d exceeds 1024", E);
  if (K % 128 != 0 || N % 128 != 0)
    return fail(MOE_UNSUPPORTED_SHAPE, "the FP8 layer needs K %% 128 == 0 and N %% 128 == 0 (got K=%d N=%d)", K, N);
  if (T == 0) return MOE_OK;
  if (!X || !topk_ids || !topk_weights || !w1 || !w1_scale || !w2 || !w2_scale || !out || !workspace)
    return fail(MOE_INVALID_ARGUMENT, "null pointer argument");
  if (((uintptr_t)workspace % 256) != 0) return fail(MOE_INVALID_ARGUMENT, "workspace must be 256-byte aligned");
  if (((uintptr_t)X | (uintptr_t)out | (uintptr_t)w1 | (uintptr_t)w2) % 16 != 0)
    return fail(MOE_INVALID_ARGUMENT, "X, out and the weight tensors must be 16-byte aligned");
  const long long S = (long long)T * topk;
  if (S > 0x7fffffffLL / 2) return fail(MOE_UNSUPPORTED_SHAPE, "T*topk too large");
  const Fp8Workspace w = fp8_carve(T, K, N, E, topk);
  if (workspace_bytes < w.total)
    return fail(MOE_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  unsigned char* base = (unsigned char*)workspace;
  int32_t* counts = (int32_t*)(base + w.counts);
  int32_t* offsets = (int32_t*)(base + w.offsets);
  int32_t* num_padded = (int32_t*)(base + w.num_padded);
  int32_t* sorted = (int32_t*)(base + w.sorted);
  int32_t* blocks = (int32_t*)(base + w.blocks);
  uint8_t* xq = base + w.xq;
  float* sx = (float*)(base + w.sx);
  void* H = base + w.H;
  uint8_t* aq = base + w.aq;
  float* sa = (float*)(base + w.sa);
  float* Y = (float*)(base + w.Y);
  const int block_m = fp8_pick_block_m(S, E);
  const bool ev = g_nevents == 7;
  auto mark = [&](int i) { if (ev) (void)hipEventRecord((hipEvent_t)g_events[i], stream); };

  mark(0);
  int err = launch_align(topk_ids, (int)S, E, block_m, (int)align_capacity(S, E, block_m), counts, offsets, sorted,
                         blocks, num_padded, stream);
  if (err != 0) return hip_fail(err, "align launch");
  mark(1);
  err = fp8::launch_fp8_quantize(X, T, K, (int)dt, 0, xq, sx, stream);
  if (err != 0) return hip_fail(err, "activation quantiser launch");
  mark(2);
  int st = fp8_moe_grouped_gemm(xq, sx, topk, w1, w1_scale, sorted, blocks, num_padded, (int)S, E, 2 * N, K, block_m,
                                (int)dt, H, stream);
  if (st != MOE_OK) return st;
  mark(3);
  // rows of slots that were not bucketed hold stale bytes: they are quantised like any other row
  // and never read again (the second product only gathers bucketed slots)
  err = fp8::launch_fp8_quantize(H, S, N, (int)dt, 1, aq, sa, stream);
  if (err != 0) return hip_fail(err, "SiLU-and-multiply quantiser launch");
  mark(4);
  st = fp8_moe_grouped_gemm(aq, sa, 1, w2, w2_scale, sorted, blocks, num_padded, (int)S, E, K, N, block_m, 2, Y, stream);
  if (st != MOE_OK) return st;
  mark(5);
  err = launch_combine(Y, 1, 1, topk_weights, topk_ids, E, out, T, topk, K, (int)dt, stream);
  if (err != 0) return hip_fail(err, "combine launch");
  mark(6);
  return MOE_OK;
}

int fp8_set_plan_override(int mt, int nt, int k_splits, int group_m) {
  if (mt < 0 || nt < 0 || k_splits < 0 || group_m < 0) return fail(MOE_INVALID_ARGUMENT, "negative plan override");
  g_fp8_mt = mt; g_fp8_nt = nt; g_fp8_splits = k_splits; g_fp8_group_m = group_m;
  return MOE_OK;
}

int fp8_probe_mfma(void* sink, int iters, void* stream) {
  if (!sink || iters < 1) return fail(MOE_INVALID_ARGUMENT, "probe needs a sink and iters >= 1");
  const int err = fp8::launch_fp8_mfma_loop((float*)sink, 512, iters, (hipStream_t)stream);
  if (err != 0) return hip_fail(err, "FP8 MFMA probe launch");
  return MOE_OK;
}

}  // extern "C"
