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
  void* C;             // k_splits == 1: the result [M, N]; otherwise float32 planes [k_splits, M, N]
  int M, N, K;
  int k_splits;        // >= 1
  int kb_per_split;    // reduction blocks per split (the last split may be shorter)
  int out_bf16;        // output type of the result: 0 fp16, 1 bf16, 2 float32
  int group_m;         // row blocks per tile group (>= 1): the order in which tiles are handed out
  // Grouped (one weight matrix per expert) mode, sorted_slot_ids != nullptr: M is the capacity of
  // the slot table (a multiple of the token tile), tile row r of row block mb is slot
  // sorted_slot_ids[mb * BM + r] (>= num_slots: padding), its A row is slot / row_div, its C row is
  // slot; row block mb belongs to expert block_expert_ids[mb] (blocks at or past *num_padded do
  // nothing); B and b_scale advance by b_expert_stride / bs_expert_stride elements per expert.
  const int32_t* sorted_slot_ids;
  const int32_t* block_expert_ids;
  const int32_t* num_padded;
  int num_slots, row_div;
  size_t b_expert_stride, bs_expert_stride;
};

// bm = tokens per workgroup in {16, 32, 64, 128, 256}, bn = features per workgroup in {64, 128, 256}
// (bm = 256 with bn in {128, 256}, bm <= 128 with any bn).
// A and B are addressed with
// 32-bit byte offsets: M * K and N * K must be below 2^32.  Returns a hipError_t, or -1 for an
// unknown tile.
int launch_fp8_gemm(const GemmParams& p, int bm, int bn, hipStream_t stream);
int launch_fp8_split_reduce(const float* planes, int k_splits, long long mn, void* C, int out_bf16,
                            hipStream_t stream);

int launch_fp8_mfma_loop(float* sink, int grid, int iters, hipStream_t stream);

}  // namespace fp8
