// Launch interface of the blockwise-scaled FP8 GEMM kernels (fp8_gemm.hip), used by the C ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fp8 {

struct GemmParams {
  const uint8_t* A;
  const float* a_scale;
  const uint8_t* B;
  const float* b_scale;
  void* C;             // k_splits == 1: 16-bit [M, N]; otherwise float32 planes [k_splits, M, N]
  int M, N, K;
  int k_splits;        // >= 1
  int kb_per_split;    // reduction blocks per split (the last split may be shorter)
  int out_bf16;        // 16-bit output type when k_splits == 1: 1 bf16, 0 fp16
};

// mt in {1, 2, 4, 8} (16 mt rows of A per workgroup), nt in {1, 2, 4} (64 nt rows of B per workgroup),
// ntl: non-temporal weight loads (mt <= 4 only).  Returns a hipError_t, or -1 for an unknown variant.
int launch_fp8_gemm(const GemmParams& p, int mt, int nt, int ntl, hipStream_t stream);
int launch_fp8_split_reduce(const float* planes, int k_splits, long long mn, void* C, int out_bf16,
                            hipStream_t stream);

int launch_fp8_mfma_loop(float* sink, int grid, int iters, hipStream_t stream);

}  // namespace fp8
