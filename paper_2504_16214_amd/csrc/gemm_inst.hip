// Explicit instantiations of the grouped W4A16 GEMM for one (dtype, KW) pair.
// Compiled several times with -DMOE_DT={0,1} -DMOE_KW={1,2,4} so the variants build in parallel.
#include "gemm_kernel.hpp"

#ifndef MOE_DT
#error "compile with -DMOE_DT=0|1"
#endif
#ifndef MOE_KW
#error "compile with -DMOE_KW=1|2|4"
#endif

namespace moe {

template <int DT, int MT, int NT, int KS, int KW, int FUSE, int SZR, int PRE, int WV>
int launch_w4a16_gemm(const GemmParams& p, int grid, hipStream_t stream) {
  auto kern = w4a16_gemm_kernel<DT, MT, NT, KS, KW, FUSE, SZR, PRE, WV>;
  const size_t lds = TileGeom<MT, NT, KS, WV>::lds_bytes(p.G, SZR, PRE);
  if (lds > 64 * 1024) {
    // Raise the dynamic LDS limit of this kernel, once per device and size (the attribute is
    // per device; remembering it per device keeps a second GPU of the process correct).
    constexpr int kMaxDev = 64;
    static size_t lds_allowed[kMaxDev] = {};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return (int)err;
    if (dev < 0 || dev >= kMaxDev || lds > lds_allowed[dev]) {
      err = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (err != hipSuccess) return (int)err;
      if (dev >= 0 && dev < kMaxDev) lds_allowed[dev] = lds;
    }
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * WV), lds, stream, p);
  return (int)hipGetLastError();
}

#if !defined(MOE_PRE) && !defined(MOE_WIDE)
#define MOE_TILE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, MOE_KW, 0, 0, 0, 4>(const GemmParams&, int, hipStream_t);
#define MOE_TILE_FUSE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, MOE_KW, 1, 0, 0, 4>(const GemmParams&, int, hipStream_t);
#include "gemm_variants.def"

// register-resident scale variants: group 128 only (KW == 4), small token tiles
#if MOE_KW == 4
#define MOE_TILE_SZR(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 0, 1, 0, 4>(const GemmParams&, int, hipStream_t);
#define MOE_TILE_SZR_FUSE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 1, 1, 0, 4>(const GemmParams&, int, hipStream_t);
#include "gemm_variants_szr.def"
#endif
#endif  // !MOE_PRE && !MOE_WIDE

// operand-order (prepacked) weights: own translation unit (-DMOE_PRE) so it builds in parallel
#if defined(MOE_PRE) && MOE_KW == 4
#define MOE_TILE_PRE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 0, 1, 1, 4>(const GemmParams&, int, hipStream_t);
#define MOE_TILE_PRE_FUSE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 1, 1, 1, 4>(const GemmParams&, int, hipStream_t);
#include "gemm_variants_pre.def"
#endif

// eight-wave workgroups on row-major weights loaded in operand order (large token tiles, group 128):
// own translation unit (-DMOE_WIDE)
#if defined(MOE_WIDE) && MOE_KW == 4
#define MOE_TILE_WIDE(MT, NT, KS, WV) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 0, 1, 2, WV>(const GemmParams&, int, hipStream_t);
#define MOE_TILE_WIDE_FUSE(MT, NT, KS, WV) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 1, 1, 2, WV>(const GemmParams&, int, hipStream_t);
#include "gemm_variants_wide.def"
#endif

}  // namespace moe
