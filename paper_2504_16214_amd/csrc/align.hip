// Expert bucketing for the grouped MoE launch: a stable counting sort of the routed slots by
// expert, every non-empty expert padded to a multiple of block_m, plus the block -> expert
// table.  The paper serves all experts from one launch (Section VII-B); this is the index
// structure that makes that possible.  Integer work only, bit-exact and order-deterministic.
//
// One workgroup of 16 wavefronts:
//   1. each wave histograms a contiguous range of slots into its own LDS row (integer LDS
//      atomics: the counts do not depend on arrival order);
//   2. per expert, the 16 partial counts are turned into exclusive bases on top of the
//      padded expert offsets (wave-level prefix scan over experts with __shfl_up);
//   3. each wave walks its range again in slot order, 64 slots at a time: a ballot per id
//      bit yields the mask of lanes holding the same expert, popcount of the lower lanes is
//      the rank inside the tile, the LDS counter supplies the running base.  Ascending slot
//      order inside every expert segment follows by construction.
//
// route_align_kernel is the same workgroup with the router in front (small batches): each of the
// 16 waves first routes its share of the tokens (top-k ids and softmax weights, written for the
// later steps of the layer), then the bucketing runs on the ids the workgroup has just written.
// One launch instead of two; the ids and tables are bit for bit those of the separate kernels.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "router_device.hpp"

namespace moe {

constexpr int kAlignWaves = 16;
constexpr int kAlignThreads = 64 * kAlignWaves;
constexpr int kAlignBatch = 8;      // tiles of 64 slot ids a wave fetches before it processes them

// The bucketing proper; every thread of the (single) workgroup calls it.  `topk_ids` is not
// restrict-qualified: in the fused kernel the same workgroup wrote it just before.
__device__ __forceinline__ void
align_body(const int32_t* topk_ids, int S, int E, int block_m, int capacity, int id_bits,
           int32_t* __restrict__ expert_counts, int32_t* __restrict__ expert_offsets,
           int32_t* __restrict__ sorted_slot_ids, int32_t* __restrict__ block_expert_ids,
           int32_t* __restrict__ num_padded) {
  extern __shared__ int lds[];
  int* hist = lds;                         // [kAlignWaves][E]
  int* off = lds + kAlignWaves * E;        // [E + 1] padded exclusive offsets
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  for (int i = tid; i < kAlignWaves * E; i += kAlignThreads) hist[i] = 0;
  for (int i = tid; i < capacity; i += kAlignThreads) sorted_slot_ids[i] = S;
  __syncthreads();

  // contiguous slot range of this wave, a multiple of 64 long
  const int per_wave = ((S + kAlignWaves - 1) / kAlignWaves + 63) & ~63;
  const int begin = wave * per_wave;
  const int end = begin + per_wave < S ? begin + per_wave : S;

  // (both walks fetch kAlignBatch tiles of 64 ids ahead of using them: with one load per trip the
  // walk of a large batch is a chain of memory latencies)
  for (int s0 = begin; s0 < end; s0 += 64 * kAlignBatch) {
    int ev[kAlignBatch];
#pragma unroll
    for (int u = 0; u < kAlignBatch; ++u) {
      const int s = s0 + 64 * u + lane;
      ev[u] = s < end ? topk_ids[s] : -1;
    }
#pragma unroll
    for (int u = 0; u < kAlignBatch; ++u)
      if (ev[u] >= 0 && ev[u] < E) atomicAdd(&hist[wave * E + ev[u]], 1);
  }
  __syncthreads();

  // padded exclusive prefix over experts (wave 0), E <= 1024
  if (wave == 0) {
    int carry = 0;
    for (int e0 = 0; e0 < E; e0 += 64) {
      const int e = e0 + lane;
      int total = 0;
      if (e < E)
        for (int w = 0; w < kAlignWaves; ++w) total += hist[w * E + e];
      if (e < E) expert_counts[e] = total;
      const int padded = (total + block_m - 1) / block_m * block_m;
      int incl = padded;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d, 64);
        if (lane >= d) incl += up;
      }
      if (e < E) off[e] = carry + incl - padded;
      carry += __shfl(incl, 63, 64);
    }
    if (lane == 0) off[E] = carry;
  }
  __syncthreads();

  // per-wave running bases: hist[w][e] <- off[e] + sum_{w' < w} hist[w'][e]
  for (int e = tid; e < E; e += kAlignThreads) {
    int run = off[e];
    for (int w = 0; w < kAlignWaves; ++w) {
      const int c = hist[w * E + e];
      hist[w * E + e] = run;
      run += c;
    }
  }
  for (int e = tid; e <= E; e += kAlignThreads) expert_offsets[e] = off[e];
  if (tid == 0) num_padded[0] = off[E];
  __syncthreads();

  // scatter in slot order
  for (int s0 = begin; s0 < end; s0 += 64 * kAlignBatch) {
    int ev[kAlignBatch];
#pragma unroll
    for (int u = 0; u < kAlignBatch; ++u) {
      const int s = s0 + 64 * u + lane;
      ev[u] = s < end ? topk_ids[s] : -1;
    }
#pragma unroll
    for (int u = 0; u < kAlignBatch; ++u) {      // tiles in slot order
      if (s0 + 64 * u >= end) break;             // (wave-uniform)
      const int s = s0 + 64 * u + lane;
      int e = ev[u];
      if (e < 0 || e >= E) e = -1;
      const bool valid = e >= 0;
      unsigned long long same = __ballot(valid);
      for (int b = 0; b < id_bits; ++b) {
        const bool bit = (e >> b) & 1;
        const unsigned long long m = __ballot(valid && bit);
        same &= bit ? m : ~m;
      }
      if (valid) {
        const unsigned long long below = same & ((1ull << lane) - 1ull);
        const int rank = __popcll(below);
        int* ctr = &hist[wave * E + e];
        const int base = *ctr;
        sorted_slot_ids[base + rank] = s;
        if (rank == 0) *ctr = base + __popcll(same);   // after every lane of the group has read it
      }
    }
  }

  // block -> expert: upper bound of the block's first row among the padded offsets
  const int nblocks = capacity / block_m;
  const int total_rows = off[E];
  for (int b = tid; b < nblocks; b += kAlignThreads) {
    const int row = b * block_m;
    int ex = -1;
    if (row < total_rows) {
      int lo = 0, hi = E;             // find the smallest e with off[e + 1] > row
      while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (off[mid + 1] > row) hi = mid; else lo = mid + 1;
      }
      ex = lo;
    }
    block_expert_ids[b] = ex;
  }
}

__global__ void __launch_bounds__(kAlignThreads)
align_kernel(const int32_t* __restrict__ topk_ids, int S, int E, int block_m, int capacity, int id_bits,
             int32_t* __restrict__ expert_counts, int32_t* __restrict__ expert_offsets,
             int32_t* __restrict__ sorted_slot_ids, int32_t* __restrict__ block_expert_ids,
             int32_t* __restrict__ num_padded) {
  align_body(topk_ids, S, E, block_m, capacity, id_bits, expert_counts, expert_offsets, sorted_slot_ids,
             block_expert_ids, num_padded);
}

__global__ void __launch_bounds__(kAlignThreads)
route_align_kernel(const float* __restrict__ logits, const float* __restrict__ bias, int T, int E, int topk,
                   int32_t* topk_ids, float* __restrict__ topk_weights, int block_m, int capacity, int id_bits,
                   int32_t* __restrict__ expert_counts, int32_t* __restrict__ expert_offsets,
                   int32_t* __restrict__ sorted_slot_ids, int32_t* __restrict__ block_expert_ids,
                   int32_t* __restrict__ num_padded) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (E <= kRouter16MaxE && topk <= kRouter16MaxTopk) {
    // one token per 16-lane row: 64 tokens of the workgroup in flight at a time
    for (int t = wave * 4 + (lane >> 4); t < T; t += kAlignWaves * 4)      // uniform inside a row
      route_token_row16(logits + (size_t)t * E, bias, E, topk, lane, topk_ids + (size_t)t * topk,
                        topk_weights + (size_t)t * topk);
  } else {
    for (int t = wave; t < T; t += kAlignWaves)      // wave-uniform trip count
      route_token(logits + (size_t)t * E, bias, E, topk, lane, topk_ids + (size_t)t * topk,
                  topk_weights + (size_t)t * topk);
  }
  // the ids go to memory for the combine and are read back by this same workgroup: make the
  // writes visible to its other waves before anyone reads them
  __threadfence_block();
  __syncthreads();
  align_body(topk_ids, T * topk, E, block_m, capacity, id_bits, expert_counts, expert_offsets, sorted_slot_ids,
             block_expert_ids, num_padded);
}

static int raise_align_lds(const void* kern, size_t lds, size_t& allowed) {
  if (lds > allowed) {
    hipError_t err = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (err != hipSuccess) return (int)err;
    allowed = lds;
  }
  return 0;
}

// Dynamic LDS beyond 64 KiB needs the per-kernel attribute, remembered per device (the attribute
// is per device; a process may drive several GPUs).
constexpr int kAlignMaxDev = 64;
static size_t g_align_lds[2][kAlignMaxDev];

static int prepare_align_lds(int which, const void* kern, size_t lds) {
  if (lds <= 64 * 1024) return 0;
  int dev = 0;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return (int)err;
  if (dev < 0 || dev >= kAlignMaxDev) {
    size_t none = 0;
    return raise_align_lds(kern, lds, none);
  }
  return raise_align_lds(kern, lds, g_align_lds[which][dev]);
}

int launch_route_align(const float* logits, const float* bias, int T, int E, int topk, int32_t* topk_ids,
                       float* topk_weights, int block_m, int capacity, int32_t* expert_counts,
                       int32_t* expert_offsets, int32_t* sorted_slot_ids, int32_t* block_expert_ids,
                       int32_t* num_padded, hipStream_t stream) {
  int id_bits = 0;
  while ((1 << id_bits) < E) ++id_bits;
  const size_t lds = (size_t)(kAlignWaves * E + E + 1) * sizeof(int);
  const int perr = prepare_align_lds(1, reinterpret_cast<const void*>(route_align_kernel), lds);
  if (perr != 0) return perr;
  hipLaunchKernelGGL(route_align_kernel, dim3(1), dim3(kAlignThreads), lds, stream, logits, bias, T, E, topk,
                     topk_ids, topk_weights, block_m, capacity, id_bits, expert_counts, expert_offsets,
                     sorted_slot_ids, block_expert_ids, num_padded);
  return (int)hipGetLastError();
}

int launch_align(const int32_t* topk_ids, int S, int E, int block_m, int capacity,
                 int32_t* expert_counts, int32_t* expert_offsets, int32_t* sorted_slot_ids,
                 int32_t* block_expert_ids, int32_t* num_padded, hipStream_t stream) {
  int id_bits = 0;
  while ((1 << id_bits) < E) ++id_bits;
  const size_t lds = (size_t)(kAlignWaves * E + E + 1) * sizeof(int);
  const int perr = prepare_align_lds(0, reinterpret_cast<const void*>(align_kernel), lds);
  if (perr != 0) return perr;
  hipLaunchKernelGGL(align_kernel, dim3(1), dim3(kAlignThreads), lds, stream, topk_ids, S, E, block_m,
                     capacity, id_bits, expert_counts, expert_offsets, sorted_slot_ids,
                     block_expert_ids, num_padded);
  return (int)hipGetLastError();
}

}  // namespace moe
