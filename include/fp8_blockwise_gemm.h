/*
 * C ABI of the blockwise-scaled FP8 GEMM for MI355X (gfx950), exported by the same shared
 * library as the W4A16 mixture-of-experts layer.
 *
 * The operator is the "blockwise scaled FP8 GEMM" of the paper's kernel table (Table II, H100
 * rows) and serving evaluation (Section VII-D).  The paper names it without writing it down; the
 * definition used is the published fine-grained FP8 scheme of the model family it serves
 * (1 x 128 activation tiles, 128 x 128 weight blocks):
 *
 *   C[m, n] = sum over kb of a_scale[m, kb] * b_scale[n / 128, kb] *
 *                 sum_{k in [128 kb, 128 kb + 128)} A[m, k] * B[n, k]
 *
 *   A       [M, K] 8-bit floats, OCP e4m3 (1-4-3, bias 7, no infinities, 0x7f / 0xff = NaN, max 448)
 *   a_scale [M, K/128] float32
 *   B       [N, K] e4m3 (the weight: one row per output feature)
 *   b_scale [ceil(N/128), K/128] float32
 *   C       [M, N] out_dtype: 0 = fp16, 1 = bf16 (rounded once from float32), 2 = float32 (the
 *           accumulator as it is).
 *
 * Arithmetic: the 128 products of a block are summed by one matrix instruction (exact products,
 * the instruction's own internal alignment of the sum), every block's sum is scaled by
 * float32(a_scale * b_scale) and accumulated in float32.
 *
 * All pointers are caller-owned DEVICE memory; A, B and C 16-byte aligned, scales 4-byte
 * aligned; C must not alias an input.  K % 128 == 0, N % 64 == 0, M >= 0 (M == 0 is a no-op),
 * M * K and N * K below 2^32.
 * Nothing is allocated and nothing synchronises with the host: kernels go to `stream`
 * (a hipStream_t; NULL = the default stream).  `workspace`: at least
 * fp8_blockwise_gemm_workspace_bytes(M, N, K) bytes, 256-byte aligned (float32 partial planes
 * when the reduction is split over workgroups; may be NULL when that size is 0).
 * Returns a moe_status value (0 = ok, 1 = invalid argument, 2 = unsupported shape,
 * 3 = workspace too small, 4 = HIP error); the message is read with moe_last_error().
 */
#ifndef FP8_BLOCKWISE_GEMM_H
#define FP8_BLOCKWISE_GEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

size_t fp8_blockwise_gemm_workspace_bytes(int M, int N, int K);

int fp8_blockwise_gemm(const uint8_t* A, const float* a_scale, const uint8_t* B, const float* b_scale,
                       void* C, int M, int N, int K, int out_dtype,
                       void* workspace, size_t workspace_bytes, void* stream);

/*
 * Grouped form: one weight matrix per expert, one launch over all experts (the structure of the
 * paper's mixture-of-experts kernel, Section VII-B, with the FP8 operands above):
 *   C[s, :] = the blockwise-scaled product of row s / row_div of A with B[e_s]  for every
 *   bucketed slot s, e_s being the expert whose segment of sorted_slot_ids contains s.
 *   A [rows_A, K] e4m3, a_scale [rows_A, K/128] float32, rows_A >= ceil(num_slots / row_div);
 *   B [E, N, K] e4m3, b_scale [E, ceil(N/128), K/128] float32;
 *   sorted_slot_ids / block_expert_ids / num_padded: as produced by moe_align_by_expert
 *   (include/moe_w4a16.h) with the same block_m, E and num_slots = T * topk;
 *   C [num_slots, N] 16-bit, written at row = slot id; rows of slots that were not bucketed are
 *   left untouched.
 * Same arithmetic, alignment and size rules as fp8_blockwise_gemm; block_m in
 * {16, 32, 64, 128, 256} is the token tile of the kernel (N % 128 == 0 at 256); the reduction is
 * never split, so no workspace.  num_slots == 0 is a no-op.
 */
int fp8_moe_grouped_gemm(const uint8_t* A, const float* a_scale, int row_div,
                         const uint8_t* B, const float* b_scale,
                         const int32_t* sorted_slot_ids, const int32_t* block_expert_ids,
                         const int32_t* num_padded, int num_slots, int E, int N, int K, int block_m,
                         int out_dtype, void* C, void* stream);

/*
 * Tuning hook (thread-local, not part of the operator): force the tile (mt in {1,2,4,8,16} = rows
 * of A per workgroup / 16, nt in {1,2,4} = rows of B per workgroup / 64; mt = 16 not with nt = 1)
 * and the number of
 * reduction splits, and group_m = how many row blocks form a group in the order tiles are handed
 * to the XCDs (L2 reuse); zeros restore the automatic choice.  A forced plan that does not fit the
 * shape makes fp8_blockwise_gemm return "unsupported shape".  The workspace size query follows
 * the forced plan.
 */
int fp8_set_plan_override(int mt, int nt, int k_splits, int group_m);

/*
 * Achievable-roof probe for the benchmark: a register-resident loop of the FP8 matrix
 * instruction (iters x 16 per wave, 512 workgroups of four waves = 2 per CU).  sink: device
 * memory for 512 * 256 floats.  2 * 16 * 16 * 128 flop per instruction.
 */
int fp8_probe_mfma(void* sink, int iters, void* stream);

#ifdef __cplusplus
}
#endif
#endif
