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
constexpr int kTailSort = 128;          // at most this many items at the end of every queue are ordered by cost

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
struct WorkspaceLayout {
  size_t sorted_at;  // bytes
  size_t prefix_at;  // bytes
  size_t items_at;   // bytes
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
  w.total = w.items_at + w.capacity * sizeof(WorkItem);
  return w;
}

__device__ __forceinline__ int items_of_sequence(int len, int group) {
  const int tok_tiles = (len + kWaveTileRows - 1) / kWaveTileRows;
  return (tok_tiles * group + kWavesPerItem - 1) / kWavesPerItem;
}

// Workgroups of the prepass: one per 1024 places of the list, at least one per queue (its tail), at most 64.
inline unsigned prepass_workgroups(size_t capacity) {
  const size_t g = (capacity + kPrepassThreads - 1) / kPrepassThreads;
  return (unsigned)(g < (size_t)kXcds ? (size_t)kXcds : g > 64 ? 64 : g);
}

// queue of the pair with rank r (row r / 8): serpentine dealing
__device__ __forceinline__ int pair_rank(int row, int queue) { return row * kXcds + ((row & 1) ? kXcds - 1 - queue : queue); }

template <bool CAUSAL>
__global__ __launch_bounds__(kPrepassThreads) void build_worklist_kernel(const int32_t* __restrict__ cu, int batch, int n_kv_heads, int group,
                                                                         WorkControl* __restrict__ ctrl, int32_t* __restrict__ sorted_seq,
                                                                         int32_t* __restrict__ queue_prefix_global, int rows,
                                                                         WorkItem* __restrict__ items,
                                                                         int capacity, int tail_items) {
  __shared__ int s_len[kPrepassLdsSeqs];
  __shared__ int s_start[kPrepassLdsSeqs];
  __shared__ int s_sorted[kPrepassLdsSeqs];
  __shared__ int s_prefix[kPrepassLdsPrefix];
  __shared__ __attribute__((aligned(16))) int s_key[kPrepassThreads / 2];  // step 1: rank counters; step 4: sort keys (kTailSort of them)
  __shared__ __attribute__((aligned(16))) WorkItem s_tail[kTailSort];
  __shared__ int s_queue_len[kXcds];
  __shared__ int s_queue_start[kXcds + 1];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // Every workgroup of the grid derives the ranking and the queue layout for itself (steps 1 and 2: a few
  // microseconds, and no synchronisation between workgroups is needed); the places of the list are then shared
  // out over the grid (step 3), and workgroup x < 8 also orders the tail of queue x (step 4).  Workgroup 0
  // writes the control block.
  const bool leader = blockIdx.x == 0;
  if (leader && tid < kXcds) ctrl->queue_head[tid * kHeadStride] = 0;

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

  // 1. rank the sequences by descending length (ties by index): count who precedes each sequence.  Batches of
  // up to half the workgroup have several threads per sequence, each counting a share of the others.
  if (batch <= kPrepassThreads / 2) {
    int* s_rank = s_key;  // (unused until step 3)
    const int parts = kPrepassThreads / batch;
    if (tid < batch) s_rank[tid] = 0;
    __syncthreads();
    const int b = tid / parts, part = tid - b * parts;
    if (b < batch) {
      const int mine = s_len[b];
      int count = 0;
      for (int o = part; o < batch; o += parts) {
        const int other = s_len[o];
        count += (other > mine || (other == mine && o < b)) ? 1 : 0;
      }
      if (count) atomicAdd(&s_rank[b], count);
    }
    __syncthreads();
    if (tid < batch) s_sorted[s_rank[tid]] = tid;
  } else {
    for (int b = tid; b < batch; b += kPrepassThreads) {
      const int mine = length_of(b);
      int rank = 0;
#pragma unroll 8
      for (int o = 0; o < batch; ++o) {
        const int other = length_of(o);
        rank += (other > mine || (other == mine && o < b)) ? 1 : 0;
      }
      sorted[rank] = b;
    }
  }
  if (!in_lds) __threadfence_block();  // (a fence also waits for every store this thread has in flight)
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
  if (queue_prefix != s_prefix) __threadfence_block();
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
      if (leader) ctrl->xcd_start[tid] = mine;
    }
    if (leader && tid == 0) ctrl->n_items = run;
  }
  __syncthreads();

  // 3. one thread per place of the list (consecutive threads write consecutive items).  The queue of a place
  // follows from the queue starts, its pair from a binary search over the queue's prefix (step 2), and the
  // item from the distance to the pair's first place.
  const int total = s_queue_start[kXcds];
  // item of place p, which lies in queue x; cost = 64-key tiles the item streams (those visible to its last query tile)
  auto item_at = [&](int p, int x, int& cost) -> WorkItem {
    const int local = p - s_queue_start[x];
    // the last row that starts at or before this place (a row without items starts where the next one does;
    // rows past the last pair start at the end of the queue)
    const int* prefix = queue_prefix + x * rows;
    int lo = 0, hi = rows - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (prefix[mid] <= local) lo = mid; else hi = mid - 1;
    }
    int r = pair_rank(lo, x);
    if (r >= n_pairs) r = n_pairs - 1;  // cannot happen for valid cu_seqlens
    const int seq_rank = r / n_kv_heads;
    const int b = sorted[seq_rank];
    const int kv_head = r - seq_rank * n_kv_heads;
    const int start = start_of(b), len = length_of(b);
    const int n = items_of_sequence(len, group);
    int j = local - prefix[lo];
    if (j >= n) j = n - 1;  // (same remark)
    // most expensive first: under the causal mask the cost grows with the item's position in the sequence
    const int i = CAUSAL ? n - 1 - j : j;
    cost = (len + kKvTileRows - 1) / kKvTileRows;
    if (CAUSAL) {
      const int wave_tiles = ((len + kWaveTileRows - 1) / kWaveTileRows) * group;
      const int f_last = i * kWavesPerItem + kWavesPerItem - 1 < wave_tiles ? i * kWavesPerItem + kWavesPerItem - 1 : wave_tiles - 1;
      const int keys = (f_last / group + 1) * kWaveTileRows;
      if (keys < len) cost = (keys + kKvTileRows - 1) / kKvTileRows;
    }
    return make_int4(start, len, i * kWavesPerItem, kv_head);
  };
  auto tail_of = [&](int x) {  // first place of queue x that step 4 orders
    const int q_begin = s_queue_start[x], q_end = s_queue_start[x + 1];
    return q_end - tail_items > q_begin ? q_end - tail_items : q_begin;
  };
  for (int p = blockIdx.x * kPrepassThreads + tid; p < total; p += gridDim.x * kPrepassThreads) {
    int x = 0;
#pragma unroll
    for (int q = 1; q < kXcds; ++q) x += p >= s_queue_start[q] ? 1 : 0;
    if (p >= tail_of(x)) continue;  // step 4
    int cost;
    items[p] = item_at(p, x, cost);
  }

  // 4. the last tail_items (<= kTailSort) places of every queue in order of descending cost.  Workgroups finish
  // within about one item of each other, and an item is claimed one round before it runs: what matters for the
  // end of the kernel is that the items claimed last are the cheap ones.  The runs of step 3 end with the
  // shortest sequences, but every run still goes from its dearest item to its cheapest.  (Only a tail, sized by
  // the caller so that the K/V rows of the pairs in it fit the die's L2 together: sorted, the items of one pair
  // run apart in time, and rows that have left the L2 in between come from memory once per item instead of
  // once per die.)  Workgroup x takes queue x: its items go to LDS with a sort key, and wave 0 sorts the keys
  if (blockIdx.x >= kXcds) return;
  const int tail_x = tail_of(blockIdx.x), tail_n = s_queue_start[blockIdx.x + 1] - tail_x;
  __syncthreads();  // (s_key held the rank counters of step 1)
  if (tid < kTailSort) {
    int key = -1;
    if (tid < tail_n) {
      int cost;
      s_tail[tid] = item_at(tail_x + tid, blockIdx.x, cost);
      key = cost * kTailSort + (kTailSort - 1 - tid);  // distinct keys; equal costs keep their order
    }
    s_key[tid] = key;
  }
  __syncthreads();
  // (distinct by construction, -1 = no item) with a bitonic network held in registers: lane l has the keys of
  // places l, l + 64, ...
  constexpr int kKeysPerLane = kTailSort / 64;
  static_assert(kTailSort % 64 == 0 && (kTailSort & (kTailSort - 1)) == 0, "a power of two, whole registers");
  if (wave == 0) {
    int key[kKeysPerLane];
#pragma unroll
    for (int r = 0; r < kKeysPerLane; ++r) key[r] = s_key[r * 64 + lane];
#pragma unroll
    for (int size = 2; size <= kTailSort; size <<= 1) {
#pragma unroll
      for (int stride = size >> 1; stride > 0; stride >>= 1) {
        if (stride >= 64) {
          const int rs = stride / 64;  // the partner sits in another register of the same lane
#pragma unroll
          for (int r = 0; r < kKeysPerLane; ++r) {
            if (r & rs) continue;
            const bool descending = ((r * 64) & size) == 0;
            const int a = key[r], b = key[r | rs];
            const bool swap = descending ? a < b : a > b;
            key[r] = swap ? b : a;
            key[r | rs] = swap ? a : b;
          }
        } else {
#pragma unroll
          for (int r = 0; r < kKeysPerLane; ++r) {
            const int other = __shfl_xor(key[r], stride);
            const bool descending = (((r * 64 + lane) & size) == 0);
            const bool first = (lane & stride) == 0;  // the earlier place of the pair
            const int hi = key[r] > other ? key[r] : other, lo = key[r] > other ? other : key[r];
            key[r] = (first == descending) ? hi : lo;
          }
        }
      }
    }
#pragma unroll
    for (int r = 0; r < kKeysPerLane; ++r)
      if (key[r] >= 0) items[tail_x + r * 64 + lane] = s_tail[kTailSort - 1 - (key[r] & (kTailSort - 1))];
  }
}

}  // namespace hydra
