/*
 * moe_w4a16.h -- C ABI of the MI355X (gfx950) W4A16 mixture-of-experts layer.
 *
 * The operator is the FP16xINT4 "mixed-type MoE" layer of the paper's
 * evaluation (Section VII-B "Mixed-type MoE", Fig. 10, Table III): fp16/bf16
 * activations A, int4 weights B with per-group scale and zero-point tensors,
 * weights cast to the activation type in registers and contracted on the
 * matrix units (Section II-C, Fig. 4(b)), all experts served by one launch.
 *
 * Conventions shared by every entry point
 *   - Plain C, no exceptions.  Every function that can fail returns a
 *     moe_status; moe_last_error() gives a thread-local message for the last
 *     non-OK status returned on the calling thread.
 *   - EVERY pointer argument is a DEVICE pointer owned by the caller (for
 *     example a PyTorch allocation).  The library never allocates, frees or
 *     keeps them, never synchronises with the host, and enqueues work only on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *   - Row-major tensors, innermost dimension contiguous, no strides.
 *   - dt selects the 16-bit activation/scale/output type (moe_dtype).
 *   - Shapes are validated on the host before any launch; data-dependent
 *     problems (an expert id outside [0, E)) cannot be reported synchronously:
 *     such slots are ignored (not bucketed, contribute zero to the output).
 *   - T == 0 is a successful no-op.
 *
 * Quantised weight format (per expert e, output row n, reduction index k)
 *   qweight [E, N_out, K_in/8] int32: element k = 8j+i of a row is the unsigned
 *           nibble in bits [4i, 4i+4) of word j.
 *   scales  [E, N_out, K_in/g] dt, zeros [E, N_out, K_in/g] uint8 in 0..15:
 *           W[e,n,k] = (q - zeros[e,n,k/g]) * scales[e,n,k/g].
 *   Requirements: g % 32 == 0, K_in % g == 0, N_out % 16 == 0,
 *   K_in / g <= 512 (group tables are staged in LDS).
 */
#ifndef MOE_W4A16_H
#define MOE_W4A16_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_INVALID_ARGUMENT = 1,
  MOE_UNSUPPORTED_SHAPE = 2,
  MOE_WORKSPACE_TOO_SMALL = 3,
  MOE_HIP_ERROR = 4
} moe_status;

/* Any int may arrive here from a C caller (the entry points answer MOE_INVALID_ARGUMENT to values
 * other than these two); for a C++ translation unit the enumeration therefore has int as its fixed
 * underlying type, so that reading such a value is defined. */
#ifdef __cplusplus
typedef enum moe_dtype : int { MOE_F16 = 0, MOE_BF16 = 1 } moe_dtype;
#else
typedef enum moe_dtype { MOE_F16 = 0, MOE_BF16 = 1 } moe_dtype;
#endif

/* Message for the last non-OK status returned on this thread ("" if none). */
const char* moe_last_error(void);

/*
 * Number of int32 rows sorted_slot_ids must hold:
 * roundup(S + min(E, S) * (block_m - 1), block_m) with S = T * topk.
 * Returns 0 for invalid arguments.
 */
size_t moe_align_capacity(int T, int topk, int E, int block_m);

/*
 * Expert bucketing: stable counting sort of the S = T*topk routed slots
 * (slot s = t*topk + j goes to expert topk_ids[s]) with every non-empty
 * expert padded to a multiple of block_m.  The paper treats the MoE layer as
 * one kernel over all experts (Section VII-B); this is the indexing that
 * makes a single grouped launch possible.  Integer outputs, fully
 * deterministic:
 *   expert_counts    [E]        slots per expert, unpadded
 *   expert_offsets   [E+1]      exclusive prefix sum of the padded counts
 *   sorted_slot_ids  [capacity] segment e = its slots in ascending slot order,
 *                               then the sentinel S; all of [num_padded,
 *                               capacity) is S
 *   block_expert_ids [capacity/block_m] owning expert per block, -1 past the end
 *   num_padded       [1]        = expert_offsets[E]
 * block_m in {16, 32, 64, 128, 256}; 1 <= E <= 1024.
 */
int moe_align_by_expert(const int32_t* topk_ids, int T, int topk, int E, int block_m,
                        int32_t* expert_counts, int32_t* expert_offsets,
                        int32_t* sorted_slot_ids, int32_t* block_expert_ids,
                        int32_t* num_padded, void* stream);

/*
 * Grouped W4A16 GEMM (Section II-C / Fig. 4(b) dataflow, Table III operands):
 *   C[s, n] = sum_k A[s / row_div, k] * W[e_s, n, k]     for every bucketed slot s,
 * e_s being the expert whose segment of sorted_slot_ids contains s.
 * fp32 accumulation, one round-to-nearest-even to dt.
 *   A   [rows_A, K_in] dt; rows_A >= ceil(num_slots / row_div).
 *       row_div = topk for the gate/up projection (A = token activations),
 *       1 for the down projection (A is already per slot).
 *   C   [num_slots, N_out] dt, 4-byte aligned, written at row = slot id.  Rows of
 *       slots that were not bucketed are left untouched.
 *   sorted_slot_ids / block_expert_ids / num_padded: as produced by
 *       moe_align_by_expert with the same block_m and num_slots = T*topk.
 */
int moe_w4a16_grouped_gemm(const void* A, int row_div,
                           const int32_t* qweight, const void* scales, const uint8_t* zeros,
                           const int32_t* sorted_slot_ids, const int32_t* block_expert_ids,
                           const int32_t* num_padded,
                           int num_slots, int E, int N_out, int K_in, int group_size, int block_m,
                           moe_dtype dt, void* C, void* stream);

/*
 * The plain FP16xINT4 GEMM the paper's mixed-type dataflow is introduced with (Section II-C,
 * Fig. 4(b)): C[m, n] = sum_k A[m, k] * W[n, k], one weight matrix, no routing.
 *   A [M, K_in] dt, qweight [N_out, K_in/8], scales / zeros [N_out, K_in/g], C [M, N_out] dt.
 * Same kernels, requirements and rounding as moe_w4a16_grouped_gemm (it is that product with
 * one expert and slot m = row m).
 */
int moe_w4a16_dense_gemm(const void* A, const int32_t* qweight, const void* scales, const uint8_t* zeros,
                         int M, int N_out, int K_in, int group_size, moe_dtype dt, void* C, void* stream);

/*
 * Router in front of the layer (the benchmark statement's routing rule; the paper is silent):
 * for every token the topk largest of logits[t, :] + bias[:], in descending order, ties to
 * the lower expert index, and the softmax over those topk values.
 *   logits [T, E] float32; bias [E] float32 or NULL (added in float32, one rounding);
 *   topk_ids [T, topk] int32; topk_weights [T, topk] float32 (float32 arithmetic).
 * 1 <= topk <= min(E, 64), E <= 1024.  Logits must be finite (-inf is allowed for all but the
 * largest of a row).
 */
int moe_route_topk(const float* logits, const float* bias, int T, int E, int topk,
                   int32_t* topk_ids, float* topk_weights, void* stream);

/*
 * act[s, n] = silu(H[s, n]) * H[s, N + n],  silu(x) = x / (1 + exp(-x)).
 * H [S, 2N] dt (columns [0,N) gate, [N,2N) up), act [S, N] dt; fp32 math, one rounding.
 * The gated activation between the two projections of each expert.  The paper is silent on it
 * (it times the layer as a whole, Section VII-B / Fig. 10); the definition is the benchmark
 * statement's "SiLU-and-multiply".
 */
int moe_silu_mul(const void* H, void* act, int S, int N, moe_dtype dt, void* stream);

/*
 * out[t, c] = sum_{j<topk} topk_weights[t, j] * Y[t*topk + j, c]
 * Y [T*topk, K] dt, topk_weights [T, topk] float32, out [T, K] dt;
 * fp32 accumulation in j order, one rounding.  The paper is silent on this step as well (the
 * benchmark statement's "top-k-weighted combine").
 * moe_combine reads every row of Y: in a staged chain with expert ids outside [0, E) the rows
 * of those slots were never written by moe_w4a16_grouped_gemm, so either clear Y first or use
 * moe_combine_masked, which takes the ids and lets such slots contribute zero (what the fused
 * layer does).
 */
int moe_combine(const void* Y, const float* topk_weights, void* out,
                int T, int topk, int K, moe_dtype dt, void* stream);
int moe_combine_masked(const void* Y, const float* topk_weights, const int32_t* topk_ids, int E, void* out,
                       int T, int topk, int K, moe_dtype dt, void* stream);

/* Bytes of workspace moe_w4a16_layer needs for these sizes (0 if invalid). */
size_t moe_w4a16_layer_workspace_bytes(int T, int K, int N, int E, int topk, moe_dtype dt);

/*
 * The whole layer on one stream (the unit the paper times in Fig. 10):
 * bucketing -> grouped GEMM with W1 [E, 2N, K] (rows [0,N) gate, [N,2N) up)
 * fused with SiLU-and-multiply -> grouped GEMM with W2 [E, K, N] -> weighted
 * combine.  X [T, K] dt, topk_ids [T, topk] int32, topk_weights [T, topk]
 * float32, out [T, K] dt.  `workspace` is caller-owned device memory of at
 * least moe_w4a16_layer_workspace_bytes(...) bytes, 256-byte aligned; its
 * contents are scratch.  Slots with an expert id outside [0, E) contribute
 * zero.
 */
int moe_w4a16_layer(const void* X, const int32_t* topk_ids, const float* topk_weights,
                    const int32_t* qw1, const void* s1, const uint8_t* z1,
                    const int32_t* qw2, const void* s2, const uint8_t* z2,
                    void* out, int T, int K, int N, int E, int topk, int group_size,
                    moe_dtype dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * moe_w4a16_layer for callers that cannot allocate device memory or carry a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * (minus the workspace), same kernels and same results bit for bit.  The bucketing tables, the
 * activation between the two GEMMs and the float32 down-projection planes live in a fixed
 * 64 MiB device array inside the library (one copy per GPU, held until the process ends); the
 * call performs no allocation of any kind.  Sizes for which
 * moe_w4a16_layer_workspace_bytes(...) exceeds 64 MiB return MOE_WORKSPACE_TOO_SMALL (the
 * DeepSeek-shaped decode batch of 128 tokens needs 33 MiB).  The array's address is resolved on
 * the first call on each device (make that call outside a graph capture).  All calls on one GPU
 * share the array: calls that overlap on one GPU (different streams or threads) race; calls
 * ordered on one stream, or serialised by the caller, are safe.
 */
int moe_w4a16_layer_noalloc(const void* X, const int32_t* topk_ids, const float* topk_weights,
                            const int32_t* qw1, const void* s1, const uint8_t* z1,
                            const int32_t* qw2, const void* s2, const uint8_t* z2,
                            void* out, int T, int K, int N, int E, int topk, int group_size,
                            moe_dtype dt, void* stream);

/*
 * Offline weight repack and the layer on repacked weights (the "offline repack into the matrix
 * unit's operand order" that weight-only kernels of this kind use; the paper's kernels move packed
 * weights in their consumption order as well, Fig. 5 / Table III).
 *
 * moe_repack_qweight: qweight [E, N_out, K_in/8] -> out (same size, must not alias): blocks of
 * 16 rows x 128 reduction indices stored as 64 consecutive 16-byte chunks, chunk 16*j + n =
 * bytes [64c + 16j, 64c + 16j + 16) of the block's row n; blocks of a row set consecutive along
 * the reduction.  paired = 0: row set b = rows 16b .. 16b+15 (use for W1).  paired = 1: row sets
 * 2q / 2q+1 = even / odd rows of rows 32q .. 32q+31 (use for W2).  K_in % 128 == 0,
 * N_out % 16 == 0 (32 if paired), both pointers 16-byte aligned.  A pure permutation.
 *
 * moe_w4a16_layer_prepacked: moe_w4a16_layer with qw1p = repack(W1, paired 0) and
 * qw2p = repack(W2, paired 1); scales and zero points stay in their original layout.
 * Needs group_size == 128, K % 1024 == 0, N % 1024 == 0.  Same results bit for bit.
 */
int moe_repack_qweight(const int32_t* qweight, int E, int N_out, int K_in, int paired, int32_t* out, void* stream);
int moe_w4a16_layer_prepacked(const void* X, const int32_t* topk_ids, const float* topk_weights,
                              const int32_t* qw1p, const void* s1, const uint8_t* z1,
                              const int32_t* qw2p, const void* s2, const uint8_t* z2,
                              void* out, int T, int K, int N, int E, int topk, int group_size,
                              moe_dtype dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Import of AWQ-packed checkpoints (the paper's layer comes from an AWQ checkpoint, Section
 * VII-B / VII-D; the tensor format is the publicly documented AWQ "GEMM" one).  For E linear
 * layers y = x W, W [K_in, N_out]:
 *   awq_qweight [E, K_in, N_out/8] int32, awq_qzeros [E, K_in/g, N_out/8] int32: each word holds
 *       eight neighbouring OUTPUT columns, bits [4p, 4p+4) = column 8c + (0,2,4,6,1,3,5,7)[p];
 *   awq_scales  [E, K_in/g, N_out] 16-bit floats (either type; moved unchanged);
 *   W[k, n] = (q[k, n] - z[k/g, n]) * s[k/g, n].
 * Writes the same q, z, s in this library's layout: qweight [E, N_out, K_in/8] (sequential
 * nibbles along the reduction), scales [E, N_out, K_in/g], zeros [E, N_out, K_in/g] bytes.
 * For the layer, W1 = the gate projection's columns followed by the up projection's (concatenate
 * the two checkpoints' tensors along N_out before or after the import), W2 = the down projection.
 * All pointers device memory, caller-owned; outputs must not alias inputs; words 4-byte,
 * scales 2-byte aligned; K_in % 8 == 0, N_out % 8 == 0, K_in % group_size == 0, E <= 65535.
 * Two kernels on `stream`, no allocation.  Returns a moe_status.
 */
int moe_import_awq(const int32_t* awq_qweight, const int32_t* awq_qzeros, const void* awq_scales,
                   int E, int K_in, int N_out, int group_size,
                   int32_t* qweight, void* scales, uint8_t* zeros, void* stream);

/*
 * Router fused with the expert bucketing: moe_route_topk followed by moe_align_by_expert with the
 * ids staying on the device, as ONE launch for batches of up to 64 tokens (the 16 waves of the
 * bucketing workgroup route the tokens first, four tokens per wave when E <= 256 and topk <= 16),
 * as the two kernels back to back beyond that (one compute unit routing more tokens is slower
 * than the extra launch).  Outputs
 * are those of the two calls, bit for bit: topk_ids / topk_weights [T, topk] and the five tables
 * of moe_align_by_expert.  Same limits as the two.
 */
int moe_route_align(const float* logits, const float* bias, int T, int E, int topk, int block_m,
                    int32_t* topk_ids, float* topk_weights, int32_t* expert_counts, int32_t* expert_offsets,
                    int32_t* sorted_slot_ids, int32_t* block_expert_ids, int32_t* num_padded, void* stream);

/*
 * Router + layer on one stream: moe_route_align into tables held in the workspace, then the two
 * grouped GEMMs and the combine of moe_w4a16_layer (four launches up to 64 tokens, five beyond).
 * Arguments as for the two; `workspace` of at least moe_w4a16_routed_layer_workspace_bytes(...)
 * bytes, 256-byte aligned.
 */
size_t moe_w4a16_routed_layer_workspace_bytes(int T, int K, int N, int E, int topk, moe_dtype dt);
int moe_w4a16_routed_layer(const void* X, const float* logits, const float* bias,
                           const int32_t* qw1, const void* s1, const uint8_t* z1,
                           const int32_t* qw2, const void* s2, const uint8_t* z2,
                           void* out, int T, int K, int N, int E, int topk, int group_size,
                           moe_dtype dt, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Measurement hooks (not part of the operator).
 *
 * moe_set_stage_events: while set (n == 5), moe_w4a16_layer records the given
 * hipEvent_t handles on its stream: events[0] before bucketing, [1] before the
 * first grouped GEMM, [2] before the second, [3] before the combine, [4] after
 * it.  Pass (NULL, 0) to clear.  Thread-local.
 *
 * moe_set_tile_override: force the grouped GEMM tile (tokens per tile =
 * 16*mt, output features per workgroup = 64*nt) instead of the built-in
 * heuristic; (0, 0) restores it.  Unsupported combinations make the GEMM
 * return MOE_UNSUPPORTED_SHAPE.  Thread-local.
 *
 * moe_set_scale_path: where the grouped GEMM keeps scales / zero points: 0 = choose
 * (registers when group_size == 128, the scale rows are 16-byte aligned and the token tile is
 * small; an LDS table otherwise), 1 = always the LDS table, 2 = registers or
 * MOE_UNSUPPORTED_SHAPE.  Thread-local.
 *
 * moe_set_tiles_per_workgroup: how many consecutive feature tiles one workgroup of the
 * register-scale GEMM walks with a continuous load pipeline; 0 = choose.  Thread-local.
 *
 * moe_set_reduction_splits: into how many ranges moe_w4a16_layer cuts the reduction of its down
 * projection (one workgroup per range, float32 partial planes in the workspace, added by the
 * combine); 0 = choose (more than one only for small batches on few experts, where the launch
 * would otherwise have too few workgroups).  Limited by the planes the workspace holds and by the
 * number of 1024-index scale panels; ignored by kernels without register-resident scales.
 * Thread-local.
 *
 * moe_layer_block_m: the bucketing block size the layer picks for these sizes.
 *
 * moe_set_block_m_override: force the bucketing block of moe_w4a16_layer (16 ... 256) instead of
 * the built-in choice; 0 restores it.  Thread-local.
 *
 * moe_layer_block_m_for: the same with the layer's shapes known (group-128 layers with
 * K % 1024 == 0 and N % 1024 == 0 and more than 28 rows per expert take 128-slot blocks for
 * the eight-wave tile); honours moe_set_block_m_override.
 *
 * moe_set_wide_tiles: 0 = use the eight-wave 128-token tile whenever block_m >= 128 and the shape
 * allows it (default), 1 = never (the four-wave tiles serve every block size).  Thread-local.
 *
 * moe_last_gemm_plan: what the last grouped / dense GEMM launch issued from this thread used:
 * plan9 (HOST pointer to 9 ints) = {mt, nt, ks, register_scales, tiles_per_workgroup,
 * reduction_splits, reduction_indices_per_split, fused_silu, waves}.  A workgroup covers 16*mt
 * rows and tiles_per_workgroup consecutive tiles of 16*nt*waves features (half as many act
 * columns when fused).  Tests use it to aim samples at tile and tile-group borders.
 */
int moe_set_stage_events(void* const* events, int n);

/*
 * Achievable-roof probes for the benchmark (not part of the operator): what this chip sustains
 * on the two resources the layer is priced against, measured by the caller with events around
 * the call.
 *
 * moe_probe_stream_read: reads `bytes` (multiple of 16) from src once with the same
 * non-temporal 128-bit loads the GEMM streams weights with.  sink: >= 16 KiB of device scratch.
 *
 * moe_probe_mfma: 512 workgroups x 4 waves each issue iters x 16 register-resident
 * v_mfma_f32_16x16x32_f16 (16384 flop each).  sink: >= 512 KiB of device scratch.
 *
 * moe_probe_issue_mix: 256 workgroups x 8 waves (two waves per SIMD) each issue iters x 8
 * v_mfma_f32_16x16x32_f16 with valu_per_mfma independent VALU operations after every one and
 * lds_reads_per_8_mfma ds_read_b128 (the GEMM's fragment-read pattern) per eight: the instruction
 * mix of the mixed-type GEMM's inner loop without its memory traffic.  valu_per_mfma in
 * {0, 1, 2, 3, 4, 6}, lds_reads_per_8_mfma in {0, 2, 4, 8}.  sink: >= 512 KiB of device scratch.
 * `bench.py --issue-model` times the grid of combinations; the cost model the design notes use
 * (time per matrix instruction = max(16, 8 + 4 x VALU) SIMD cycles, plus 0.5 to 7 cycles for the
 * LDS reads) is fitted to its output.
 */
int moe_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream);
int moe_probe_mfma(void* sink, int iters, void* stream);
int moe_probe_issue_mix(void* sink, int iters, int valu_per_mfma, int lds_reads_per_8_mfma, void* stream);
int moe_set_tile_override(int mt, int nt);
int moe_set_scale_path(int mode);
int moe_set_tiles_per_workgroup(int n);
int moe_set_reduction_splits(int n);
int moe_layer_block_m(int T, int E, int topk);
int moe_set_block_m_override(int block_m);
int moe_last_gemm_plan(int* plan9);
int moe_layer_block_m_for(int T, int K, int N, int E, int topk, int group_size);
int moe_set_wide_tiles(int mode);

#ifdef __cplusplus
}
#endif
#endif /* MOE_W4A16_H */
