// Device prepass: the varlen tile scheduler.  Builds, from cu_seqlens alone, the list of work
// items the attention kernel consumes, ordered longest first so that the hardware's in-order
// workgroup dispatch acts as a longest-processing-time scheduler over the 256 CUs.
//
// The paper's Request Processor prepares such per-batch "control parameters" ahead of the GPU
// work (Section 4.1); here it is a single small kernel on the same stream, so no host
// synchronisation is needed and ragged batches cost the host nothing.
//
// Item = up to 4 consecutive wave tiles of one (sequence, KV head), in the flattened order
// f = token_tile * group + head_in_group.  Cost = number of 64-key tiles its last wave tile reads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_fwd.hpp"

namespace hydra {

constexpr int kCostBuckets = 1024;
constexpr int kPrepassThreads = 1024;

// Workspace layout (all int32 unless noted):
//   [0]            n_items
//   [4 .. 4+B]     item_offset[b]  exclusive prefix of items per sequence (per KV head), B+1 entries
//   then, 16-byte aligned, WorkItem[capacity]
//   then int32 redo_flags[capacity]: all zero between calls; the fast attention kernel sets the
//   flag of an item it cannot finish exactly, the careful kernel redoes the item and clears it
struct WorkspaceLayout {
  size_t offsets_at;  // bytes
  size_t items_at;    // bytes
  size_t flags_at;    // bytes
  size_t capacity;    // items
  size_t total;       // bytes
};

inline size_t item_capacity(int64_t batch, int64_t total_tokens, int64_t n_q_heads, int64_t n_kv_heads) {
  const int64_t group = n_q_heads / n_kv_heads;
  // sum_b ceil(L_b/64) <= N/64 + B ; items per sequence <= wave_tiles/4 + 1
  const int64_t wave_tiles = group * (total_tokens / kWaveTileRows + batch);
  return (size_t)(n_kv_heads * (wave_tiles / kWavesPerItem + batch + 1));
}

inline WorkspaceLayout workspace_layout(int64_t batch, int64_t total_tokens, int64_t n_q_heads, int64_t n_kv_heads) {
  WorkspaceLayout w;
  w.offsets_at = 16;
  size_t end = w.offsets_at + (size_t)(batch + 1) * 4;
  w.items_at = (end + 15) & ~(size_t)15;
  w.capacity = item_capacity(batch, total_tokens, n_q_heads, n_kv_heads);
  w.flags_at = w.items_at + w.capacity * sizeof(WorkItem);
  w.total = w.flags_at + w.capacity * sizeof(int32_t);
  return w;
}

__device__ __forceinline__ int items_of_sequence(int len, int group) {
  const int tok_tiles = (len + kWaveTileRows - 1) / kWaveTileRows;
  return (tok_tiles * group + kWavesPerItem - 1) / kWavesPerItem;
}

template <bool CAUSAL>
__global__ __launch_bounds__(kPrepassThreads) void build_worklist_kernel(const int32_t* __restrict__ cu, int batch, int n_kv_heads, int group,
                                                                         int32_t* __restrict__ n_items_out, int32_t* __restrict__ item_offset,
                                                                         WorkItem* __restrict__ items, int32_t* __restrict__ redo_flags, int capacity) {
  __shared__ int partial[kPrepassThreads];
  __shared__ int hist[kCostBuckets];
  __shared__ int cursor[kCostBuckets];
  const int tid = threadIdx.x;
  for (int i = tid; i < capacity; i += kPrepassThreads) redo_flags[i] = 0;

  // 1. items per sequence -> exclusive prefix (each thread owns a contiguous run of sequences)
  const int per_thread = (batch + kPrepassThreads - 1) / kPrepassThreads;
  const int b_lo = tid * per_thread;
  const int b_hi = b_lo + per_thread < batch ? b_lo + per_thread : batch;
  int mine = 0;
  for (int b = b_lo; b < b_hi; ++b) mine += items_of_sequence(cu[b + 1] - cu[b], group);
  partial[tid] = mine;
  for (int i = tid; i < kCostBuckets; i += kPrepassThreads) {
    hist[i] = 0;
    cursor[i] = 0;
  }
  __syncthreads();
  // Hillis-Steele inclusive scan over the per-thread partial sums
  for (int d = 1; d < kPrepassThreads; d <<= 1) {
    const int add = tid >= d ? partial[tid - d] : 0;
    __syncthreads();
    partial[tid] += add;
    __syncthreads();
  }
  int run = partial[tid] - mine;
  for (int b = b_lo; b < b_hi; ++b) {
    item_offset[b] = run;
    run += items_of_sequence(cu[b + 1] - cu[b], group);
  }
  const int per_head = partial[kPrepassThreads - 1];
  if (tid == 0) item_offset[batch] = per_head;
  __threadfence_block();
  __syncthreads();

  int total = per_head * n_kv_heads;
  if (total > capacity) total = capacity;  // cannot happen for valid cu_seqlens; keeps stores in bounds
  if (tid == 0) *n_items_out = total;
  // entries past the end of the list are marked empty (length 0): the attention kernel is launched
  // over the whole capacity and recognises them without reading the item count
  for (int i = total + tid; i < capacity; i += kPrepassThreads) items[i] = make_int4(0, 0, 0, 0);

  // 2. histogram of costs, 3. descending bucket starts, 4. scatter
  for (int pass = 0; pass < 2; ++pass) {
    for (int idx = tid; idx < total; idx += kPrepassThreads) {
      const int kv_head = idx / per_head;
      const int r = idx - kv_head * per_head;
      // largest b with item_offset[b] <= r (offsets are non-decreasing; empty sequences repeat)
      int lo = 0, hi = batch;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (item_offset[mid] <= r) lo = mid; else hi = mid;
      }
      const int b = lo;
      const int len = cu[b + 1] - cu[b];
      const int tok_tiles = (len + kWaveTileRows - 1) / kWaveTileRows;
      const int wave_tiles = tok_tiles * group;
      const int f0 = (r - item_offset[b]) * kWavesPerItem;
      const int f_last = f0 + kWavesPerItem - 1 < wave_tiles ? f0 + kWavesPerItem - 1 : wave_tiles - 1;
      const int cost = CAUSAL ? f_last / group + 1 : tok_tiles;
      const int bucket = cost < kCostBuckets ? cost : kCostBuckets - 1;
      if (pass == 0) {
        atomicAdd(&hist[bucket], 1);
      } else {
        const int pos = hist[bucket] + atomicAdd(&cursor[bucket], 1);
        items[pos] = make_int4(cu[b], len, f0, kv_head);
      }
    }
    __syncthreads();
    if (pass == 0) {
      // counts -> start positions, largest cost first: exclusive scan over reversed buckets
      static_assert(kCostBuckets == kPrepassThreads, "one bucket per thread");
      const int n = hist[kCostBuckets - 1 - tid];
      partial[tid] = n;
      __syncthreads();
      for (int d = 1; d < kPrepassThreads; d <<= 1) {
        const int add = tid >= d ? partial[tid - d] : 0;
        __syncthreads();
        partial[tid] += add;
        __syncthreads();
      }
      hist[kCostBuckets - 1 - tid] = partial[tid] - n;
      __syncthreads();
    }
  }
}

}  // namespace hydra
