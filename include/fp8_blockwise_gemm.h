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
 * FP8 mixture-of-experts layer: the gated expert MLP of the 16-bit layer (include/moe_w4a16.h)
 * with e4m3 weights (128 x 128 block scales) and activations quantised on the fly, the FP8
 * workload family of the paper's serving evaluation (Section VII-D; the grouped kernel structure
 * is that of Section VII-B).  The paper does not write the operator down; the quantisation rule
 * is the published fine-grained FP8 recipe:
 *
 *   quantise (fp8_quantize_rows): per row and per 128 reduction indices, in float32,
 *       m = max(max |x|, 1e-4);  scale = m / 448;  code = e4m3(x * (448 / m))   (round to nearest even)
 *   X [rows, K] dt -> codes [rows, K] uint8, scales [rows, K/128] float32; K % 128 == 0.
 *
 *   fp8_silu_mul_quantize: act = round_dt(silu(H[:, :N]) * H[:, N:]) quantised the same way,
 *       H [S, 2N] dt -> codes [S, N], scales [S, N/128]; N % 128 == 0.  The 16-bit activation never
 *       goes to memory.
 *
 *   fp8_moe_layer: bucketing -> quantise X -> grouped FP8 product with W1 [E, 2N, K] (rows [0, N)
 *       gate, [N, 2N) up; w1_scale [E, 2N/128, K/128]) rounded to dt -> SiLU-and-multiply + quantise
 *       -> grouped FP8 product with W2 [E, K, N] (w2_scale [E, K/128, N/128]) kept in float32 ->
 *       weighted combine in j order, one rounding to dt.  X [T, K] dt, topk_ids [T, topk] int32,
 *       topk_weights [T, topk] float32, out [T, K] dt.  Slots with an expert id outside [0, E)
 *       contribute zero.  K % 128 == 0, N % 128 == 0, E <= 1024.  Six launches on `stream`, no
 *       allocation; `workspace`: at least fp8_moe_layer_workspace_bytes(...) bytes, 256-byte aligned.
 *
 * All pointers are caller-owned device memory; X, H, out and the weight tensors 16-byte aligned.
 * dt is a moe_dtype (0 = fp16, 1 = bf16).  Each returns a moe_status.
 * fp8_set_layer_block_m: force the token tile of the layer's two grouped products (0 = choose);
 * thread-local tuning hook.  With moe_set_stage_events(events, 7) the layer records seven events:
 * before the bucketing, the quantiser, the first product, the SiLU quantiser, the second
 * product, the combine, and after it.
 */
int fp8_quantize_rows(const void* X, int rows, int K, int dt, uint8_t* codes, float* scales, void* stream);
int fp8_silu_mul_quantize(const void* H, int S, int N, int dt, uint8_t* codes, float* scales, void* stream);
size_t fp8_moe_layer_workspace_bytes(int T, int K, int N, int E, int topk);
int fp8_moe_layer(const void* X, const int32_t* topk_ids, const float* topk_weights,
                  const uint8_t* w1, const float* w1_scale, const uint8_t* w2, const float* w2_scale,
                  void* out, int T, int K, int N, int E, int topk, int dt,
                  void* workspace, size_t workspace_bytes, void* stream);
int fp8_set_layer_block_m(int block_m);

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
