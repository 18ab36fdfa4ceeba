// Device prepass: the varlen tile scheduler.  Builds, from cu_seqlens alone, the work list the
// attention kernel consumes.
//
// The paper's Request Processor prepares such per-batch "control parameters" ahead of the GPU
// work (Section 4.1); here it is a single small kernel on the same stream, so no host
// synchronisation is needed and ragged batches cost the host nothing.
//
// Item = up to 4 consecutive wave tiles of one (sequence, KV head), in the flattened order
// f = token_tile * group + head_in_group.  Cost = number of 64-key tiles its last wave tile reads.
//
// Order of the list.  The chip has 8 dies, each with its own L2 and 32 compute units, and the
// attention kernel keeps one queue per die.  All items of one (sequence, KV head) pair read the same
// K/V rows, so a pair goes to ONE queue as a contiguous run (most expensive item first): the
// workgroups of that die pick the run up together and the rows come from memory once per die
// instead of once per item.  Pairs are ranked by sequence length, longest first, and dealt to the
// queues in serpentine order (0..7, 7..0, ...), which keeps the queues' total work level and puts
// the short sequences at the end of every queue; the last kTailSort items of a queue are then
// re-ordered by descending cost, so that the items claimed last are the cheapest and the
// workgroups finish close together.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_fwd.hpp"

namespace hydra {

constexpr int kPrepassThreads = 1024;
constexpr int kPrepassLdsSeqs = 4096;    // sequence lengths kept in LDS for the ranking
constexpr int kPrepassLdsPrefix = 8192;  // queue prefix entries kept in LDS
constexpr int kTailSort = 256;          // at most this many items at the end of every queue are ordered by cost

// Items at the end of a queue that step 4 of the prepass sorts.  An item covers 128 query rows of one head, so
// the pairs that a tail of T items touches hold about T * 128 / group tokens of K and V: the tail is as long as
// 3 MB of such rows allow (a die's L2 has 4 MB), at most kTailSort.
inline int tail_sort_items(int group, int head_dim) {
  const int64_t bytes_per_item = (int64_t)kWavesPerItem * kWaveTileRows * head_dim * 4 / group;
  const int64_t fit = ((int64_t)3 << 20) / (bytes_per_item > 0 ? bytes_per_item : 1);
  return (int)(fit < kTailSort ? fit : kTailSort);
}

// Workspace layout:
//   WorkControl                          (counts, queue starts, one cache line per queue head)
//   int32 sorted_seq[B]                  sequences by descending length
//   int32 queue_prefix[kXcds][rows]      rows = ceil(B * Hkv / 8): items before the pair of (row, queue) in its queue
//   WorkItem items[capacity]             16-byte aligned
//   int32 redo_flags[capacity]           all zero between calls; the fast attention kernel sets the flag
//                                        of an item it cannot finish exactly, the careful kernel redoes
//                                        the item and clears it
struct WorkspaceLayout {
  size_t sorted_at;  // bytes
  size_t prefix_at;  // bytes
  size_t items_at;   // bytes
  size_t flags_at;   // bytes
  size_t rows;       // pair rows
  size_t capacity;   // items
  size_t total;      // bytes
};

inline size_t item_capacity(int64_t batch, int64_t total_tokens, int64_t n_q_heads, int64_t n_kv_heads) {
  const int64_t group = n_q_heads / n_kv_heads;
  // sum_b ceil(L_b/64) <= N/64 + B ; items per sequence <= wave_tiles/4 + 1
  const int64_t wave_tiles = group * (total_tokens / kWaveTileRows + batch);
  return (size_t)(n_kv_heads * (wave_tiles / kWavesPerItem + batch + 1));
}

inline WorkspaceLayout workspace_layout(int64_t batch, int64_t total_tokens, int64_t n_q_heads, int64_t n_kv_heads) {
  WorkspaceLayout w;
  w.rows = (size_t)((batch * n_kv_heads + kXcds - 1) / kXcds);
  w.sorted_at = sizeof(WorkControl);
  w.prefix_at = w.sorted_at + (size_t)batch * 4;
  const size_t end = w.prefix_at + w.rows * kXcds * 4;
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

// queue of the pair with rank r (row r / 8): serpentine dealing
__device__ __forceinline__ int pair_rank(int row, int queue) { return row * kXcds + ((row & 1) ? kXcds - 1 - queue : queue); }

template <bool CAUSAL>
__global__ __launch_bounds__(kPrepassThreads) void build_worklist_kernel(const int32_t* __restrict__ cu, int batch, int n_kv_heads, int group,
                                                                         WorkControl* __restrict__ ctrl, int32_t* __restrict__ sorted_seq,
                                                                         int32_t* __restrict__ queue_prefix_global, int rows,
                                                                         WorkItem* __restrict__ items, int32_t* __restrict__ redo_flags,
                                                                         int capacity, int tail_items) {
  __shared__ int s_len[kPrepassLdsSeqs];
  __shared__ int s_start[kPrepassLdsSeqs];
  __shared__ int s_sorted[kPrepassLdsSeqs];
  __shared__ int s_prefix[kPrepassLdsPrefix];
  __shared__ int s_queue_len[kXcds];
  __shared__ int s_queue_start[kXcds + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < capacity; i += kPrepassThreads) redo_flags[i] = 0;
  if (tid < kXcds) ctrl->queue_head[tid * kHeadStride] = 0;
  if (tid == 0) {
    ctrl->redo_any = 0;
    ctrl->careful_done = 0;
  }

  // Small batches (the normal case) are handled entirely in LDS after one read of cu_seqlens;
  // the global arrays are only used for what does not fit.
  const bool in_lds = batch <= kPrepassLdsSeqs;
  int* sorted = in_lds ? s_sorted : sorted_seq;
  for (int b = tid; b < batch && b < kPrepassLdsSeqs; b += kPrepassThreads) {
    const int start = cu[b];
    s_start[b] = start;
    s_len[b] = cu[b + 1] - start;
  }
  __syncthreads();
  auto length_of = [&](int b) { return b < kPrepassLdsSeqs ? s_len[b] : cu[b + 1] - cu[b]; };
  auto start_of = [&](int b) { return b < kPrepassLdsSeqs ? s_start[b] : cu[b]; };

  // 1. rank the sequences by descending length (ties by index): each thread counts who precedes its sequence
  for (int b = tid; b < batch; b += kPrepassThreads) {
    const int mine = length_of(b);
    int rank = 0;
    for (int o = 0; o < batch; ++o) {
      const int other = length_of(o);
      rank += (other > mine || (other == mine && o < b)) ? 1 : 0;
    }
    sorted[rank] = b;
  }
  __threadfence_block();
  __syncthreads();

  // 2. per queue, the running item count over its pairs (one pair per row): wave x scans queue x
  int* queue_prefix = rows * kXcds <= kPrepassLdsPrefix ? s_prefix : queue_prefix_global;
  const int n_pairs = batch * n_kv_heads;
  if (wave < kXcds) {
    int carry = 0;
    for (int row0 = 0; row0 < rows; row0 += 64) {
      const int row = row0 + lane;
      const int r = pair_rank(row, wave);
      int n = 0;
      if (row < rows && r < n_pairs) n = items_of_sequence(length_of(sorted[r / n_kv_heads]), group);
      int incl = n;
#pragma unroll
      for (int d = 1; d < 64; d <<= 1) {
        const int up = __shfl_up(incl, d);
        if (lane >= d) incl += up;
      }
      if (row < rows) queue_prefix[wave * rows + row] = carry + incl - n;
      carry += __shfl(incl, 63);
    }
    if (lane == 0) s_queue_len[wave] = carry;
  }
  __threadfence_block();
  __syncthreads();
  {
    // every thread computes the queue starts for itself; threads 0 .. 8 publish them
    int run = 0, mine = 0;
#pragma unroll
    for (int x = 0; x < kXcds; ++x) {
      if (tid == x) mine = run;
      run += s_queue_len[x];
    }
    if (run > capacity) run = capacity;  // cannot happen for valid cu_seqlens; keeps stores in bounds
    if (tid == kXcds) mine = run;
    if (tid <= kXcds) {
      if (mine > run) mine = run;
      s_queue_start[tid] = mine;
      ctrl->xcd_start[tid] = mine;
    }
    if (tid == 0) ctrl->n_items = run;
  }
  __syncthreads();

  // 3. four threads per pair write the pair's items (thread k takes items k, k + 4, ...): the pair's place in
  // its queue is known from step 2, so an item costs a few instructions
  const int total = s_queue_start[kXcds];
  constexpr int kThreadsPerPair = 4;
  for (int slot = tid / kThreadsPerPair; slot < rows * kXcds; slot += kPrepassThreads / kThreadsPerPair) {
    const int x = slot / rows, row = slot - x * rows;
    const int r = pair_rank(row, x);
    if (r >= n_pairs) continue;
    const int b = sorted[r / n_kv_heads];
    const int kv_head = r % n_kv_heads;
    const int start = start_of(b), len = length_of(b);
    const int n = items_of_sequence(len, group);
    const int base = s_queue_start[x] + queue_prefix[slot];
    for (int j = tid % kThreadsPerPair; j < n; j += kThreadsPerPair) {
      // most expensive first: under the causal mask the cost grows with the item's position in the sequence
      const int i = CAUSAL ? n - 1 - j : j;
      if (base + j < total) items[base + j] = make_int4(start, len, i * kWavesPerItem, kv_head);
    }
  }

  // 4. the last tail_items (<= kTailSort) items of every queue are put in order of descending cost (ties keep
  // their order).  Workgroups finish within about one item of each other, and an item is claimed one round
  // before it runs: what matters for the end of the kernel is that the items claimed last are the cheap ones.
  // The runs of step 3 end with the shortest sequences, but every run still goes from its dearest item to its
  // cheapest.  (Only a tail, sized by the caller so that the K/V rows of the pairs in it fit the die's L2
  // together: sorted, the items of one pair run apart in time, and rows that have left the L2 in between come
  // from memory once per item instead of once per die.)
  __threadfence_block();
  __syncthreads();
  int* s_cost = s_prefix;  // step 3 was the last reader of the queue prefixes
  static_assert(kXcds * kTailSort <= kPrepassLdsPrefix && (kXcds * kTailSort) % kPrepassThreads == 0, "tail entries per thread");
  constexpr int kPerThread = kXcds * kTailSort / kPrepassThreads;
  WorkItem held[kPerThread];
  int place[kPerThread];
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    const int e = tid + k * kPrepassThreads;
    const int x = e / kTailSort, o = e % kTailSort;
    const int q_begin = s_queue_start[x], q_end = s_queue_start[x + 1];
    const int tail = q_end - tail_items > q_begin ? q_end - tail_items : q_begin;
    place[k] = -1;
    int cost = -1;
    if (o < tail_items && tail + o < q_end) {
      held[k] = items[tail + o];
      place[k] = tail;
      const int len = held[k].y;
      cost = (len + kKvTileRows - 1) / kKvTileRows;
      if (CAUSAL) {
        const int wave_tiles = ((len + kWaveTileRows - 1) / kWaveTileRows) * group;
        const int f_last = held[k].z + kWavesPerItem - 1 < wave_tiles ? held[k].z + kWavesPerItem - 1 : wave_tiles - 1;
        const int keys = (f_last / group + 1) * kWaveTileRows;  // keys visible to the item's last query tile
        if (keys < len) cost = (keys + kKvTileRows - 1) / kKvTileRows;
      }
    }
    s_cost[e] = cost;
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < kPerThread; ++k) {
    if (place[k] < 0) continue;
    const int e = tid + k * kPrepassThreads;
    const int x = e / kTailSort, o = e % kTailSort;
    const int mine = s_cost[e];
    int rank = 0;
    for (int other = 0; other < kTailSort; ++other) {
      const int c = s_cost[x * kTailSort + other];  // (-1 past the end of a short queue: never ahead of a real item)
      rank += (c > mine || (c == mine && other < o)) ? 1 : 0;
    }
    place[k] += rank;
  }
  __syncthreads();  // every thread holds its items: the tail can be overwritten
#pragma unroll
  for (int k = 0; k < kPerThread; ++k)
    if (place[k] >= 0) items[place[k]] = held[k];
}

}  // namespace hydra
