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

template <int DT, int MT, int NT, int KS, int KW, int FUSE, int SZR, int PRE>
int launch_w4a16_gemm(const GemmParams& p, int grid, hipStream_t stream) {
  auto kern = w4a16_gemm_kernel<DT, MT, NT, KS, KW, FUSE, SZR, PRE>;
  const size_t lds = TileGeom<MT, NT, KS>::lds_bytes(p.G, SZR, PRE);
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
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), lds, stream, p);
  return (int)hipGetLastError();
}

#ifndef MOE_PRE
#define MOE_TILE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, MOE_KW, 0, 0, 0>(const GemmParams&, int, hipStream_t);
#define MOE_TILE_FUSE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, MOE_KW, 1, 0, 0>(const GemmParams&, int, hipStream_t);
#include "gemm_variants.def"

// register-resident scale variants: group 128 only (KW == 4), small token tiles
#if MOE_KW == 4
#define MOE_TILE_SZR(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 0, 1, 0>(const GemmParams&, int, hipStream_t);
#define MOE_TILE_SZR_FUSE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 1, 1, 0>(const GemmParams&, int, hipStream_t);
#include "gemm_variants_szr.def"
#endif
#endif  // !MOE_PRE

// operand-order (prepacked) weights: own translation unit (-DMOE_PRE) so it builds in parallel
#if defined(MOE_PRE) && MOE_KW == 4
#define MOE_TILE_PRE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 0, 1, 1>(const GemmParams&, int, hipStream_t);
#define MOE_TILE_PRE_FUSE(MT, NT, KS) \
  template int launch_w4a16_gemm<MOE_DT, MT, NT, KS, 4, 1, 1, 1>(const GemmParams&, int, hipStream_t);
#include "gemm_variants_pre.def"
#endif

}  // namespace moe
