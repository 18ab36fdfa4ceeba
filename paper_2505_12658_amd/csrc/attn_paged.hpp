// Attention of a hybrid batch over the paged KV cache (gfx950).
//
// The paper's batch scheduler (Algorithm 1) fills one batch, under a token budget, with the decode
// requests (one new token each) and with chunks of prefill requests (get_chunked_size new tokens
// each); all of them attend to their request's KV cache, which is paged (Section 4.5; block size 16 in Section 5.1).
// Request b brings q_len new tokens and has kv_len tokens of context in the cache, the new ones
// included (written beforehand by the paged KV write).  New token i sees keys 0 .. kv_len - q_len + i:
// the causal mask aligned to the END of the context.  q_len == kv_len is an ordinary prefill,
// q_len == 1 a decode step.
//
// Decomposition: a workgroup of 4 waves takes up to four consecutive wave tiles of one (request, KV
// head); a wave tile is 32 new tokens of one query head, flattened as f = token_tile * group +
// head_in_group, so with grouped queries the waves share every K/V tile.  In the plain form K/V tiles of
// 64 keys are gathered row by row from the pages (a lane looks its row's page up in the block table, then
// the 16-byte pieces travel global -> LDS with direct-to-LDS loads) into two stages: tile t + 1 is
// fetched while tile t is used.  Scores are kept transposed (S^T = K Q^T, O^T += V^T P^T, as in the
// packed kernel) and the softmax is the textbook online one: running maximum and rescaling at every
// tile.  Two workgroups per compute unit.
// Requests with few new tokens (decode steps above all) take a second form, in which the rows of ALL the
// query heads of a KV head share one tile and the four waves split the keys: see run_packed_rows.
// When the batch is small for the chip or its contexts are long, the packed-rows form also splits a context
// over several workgroups and a second, small kernel merges their partial results (see n_splits).
// Groups of wave tiles run on the packed kernel's software pipeline where the cache layout allows (PagedSource);
// the loop at the end of attn_paged_kernel is the plain form of the same computation (no pipelining inside the
// wave, online softmax), which the other layouts and the groups that leave the pipeline's range take.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_fwd.hpp"
#include "attn_tiles.hpp"

namespace hydra {
namespace paged {

constexpr int kRows = 32;          // new tokens (or packed rows) per wave tile
constexpr int kWavesPerGroup = 4;  // wave tiles per workgroup

struct PagedArgs {
  const uint16_t* q;        // [total_q, n_q_heads, D] with token stride
  uint16_t* out;            // [total_q, n_q_heads, D] contiguous
  int64_t q_stride;         // elements per token
  const uint16_t* k_cache;  // [num_blocks, block_size, n_kv_heads, D]
  const uint16_t* v_cache;
  const int32_t* block_tables;  // [batch, max_blocks_per_seq]
  const int32_t* cu_seqlens_q;  // [batch + 1]
  const int32_t* kv_lens;       // [batch]
  int32_t max_blocks_per_seq;
  int32_t num_blocks;
  int32_t block_shift;  // log2(block_size)
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t group;     // n_q_heads / n_kv_heads
  float scale_log2;  // softmax_scale * log2(e)
  // Packed-rows form, long contexts split over workgroups: a context of more than halves_per_split half tiles
  // (32 keys each) is cut into the fewest shares that fit that size, all of (nearly) the same length (share_plan);
  // n_splits workgroups per (request, KV head), one per share.  A context that fits one share is done by its first
  // workgroup, which writes `out` itself (the others leave at once); of a longer one every share leaves a partial
  // result in `partials`, and the combine kernel merges them.  n_splits == 1: never split.
  int32_t n_splits;
  int32_t halves_per_split;
  float* partials;  // [batch, n_kv_heads, n_splits] records of kPartialFloats<D> floats
  int32_t batch;
  int32_t n_tile_wgs;  // workgroups of the wave-tile form at the end of the grid (an upper bound from the host)
};

// One partial result of the packed-rows form: per row (32 rows) the maximum and the sum, then the
// unnormalised output rows [32][D] (only the first q_len * group rows are written and read).
template <int D>
constexpr int kPartialFloats = 2 * kRows + kRows * D;

// How a context of n_halves half tiles is cut: `shares` shares of `per` half tiles (the last one may be shorter);
// one share when it fits halves_per_split.
__device__ __forceinline__ void share_plan(int n_halves, int halves_per_split, int& per, int& shares) {
  const int k = (n_halves + halves_per_split - 1) / halves_per_split;
  per = k > 1 ? (n_halves + k - 1) / k : n_halves;
  shares = per > 0 ? (n_halves + per - 1) / per : 0;
}
// half tiles [begin, end) of share s (empty past the last share)
__device__ __forceinline__ void split_range(int n_halves, int per, int s, int& begin, int& end) {
  begin = s * per < n_halves ? s * per : n_halves;
  end = begin + per < n_halves ? begin + per : n_halves;
}

template <int D>
struct StageGeom : RowGeom<D> {
  using RowGeom<D>::kTileBytes;
  using RowGeom<D>::kPvChunks;
  static constexpr int kStageBytes = 2 * kTileBytes;  // K then V
  // A wave's slot in the packed-rows form: a stage of a HALF tile (32 keys of K, then of V) during the loop,
  // its unnormalised output (kPvChunks * 16 registers x 64 lanes x 4 bytes) for the merge.  Four slots; the
  // wave-tile form uses the same memory as its two 64-key stages.
  static constexpr int kHalfStageBytes = kStageBytes / 2;
  static constexpr int kPartialBytes = kPvChunks * 16 * 64 * 4;
  static constexpr int kSlotBytes = kHalfStageBytes > kPartialBytes ? kHalfStageBytes : kPartialBytes;
  static constexpr int kLdsBytes = (4 * kSlotBytes > 2 * kStageBytes ? 4 * kSlotBytes : 2 * kStageBytes) + 64;  // slack: D=80 reads V columns 80..95
};

#if defined(__HIP_DEVICE_COMPILE__)
// The K/V tiles are gathered from the pages in two moves, so that the block-table lookup of a tile is in
// flight while the tile before it is fetched and used (done in one move, every tile would pay the lookup's
// round trip before its loads can even be issued):
//   fetch_tile_slots: per load instruction of this wave, the cache row ("slot" = block * block_size + offset)
//     of this lane's key.  Load instructions first, first + step, ... (a workgroup's four waves share a tile
//     with first = wave, step = 4; a wave that owns a whole tile uses first = 0, step = 1).  Keys past the end
//     of the context re-read the last valid key (always masked later).  Block ids are clamped to the cache,
//     so a corrupt table cannot make the loads leave it.
//   issue_tile_loads: the direct-to-LDS loads of the K rows and V rows of those slots (KEYS keys: 64, or 32
//     for a half tile; K rows first, then V rows).
template <int D, int KEYS, int STEP>
struct TileSlots {
  static constexpr int kLoadInstr = KEYS * StageGeom<D>::kRowBytes / 1024;
  static constexpr int kCount = (kLoadInstr + STEP - 1) / STEP;
  int32_t slot[kCount];  // (the host refuses caches of 2^31 rows or more)
};

// (in two steps for callers that keep other loads in flight across the look-up: the table entries are requested
// by request_tile_blocks and only touched, which is what the compiler waits for, by slots_from_blocks)
template <int D, int KEYS, int STEP>
__device__ __forceinline__ void request_tile_blocks(TileSlots<D, KEYS, STEP>& ts, const PagedArgs& a, const int32_t* table, int first, int lane,
                                                    int kv_len, int kv0) {
  using G = StageGeom<D>;
#pragma unroll
  for (int u = 0; u < TileSlots<D, KEYS, STEP>::kCount; ++u) {
    const int instr = first + STEP * u;
    const int row = (instr * 64 + lane) / G::kChunks;
    int tok = kv0 + row;
    tok = tok < kv_len ? tok : kv_len - 1;
    ts.slot[u] = table[tok >> a.block_shift];
  }
}
template <int D, int KEYS, int STEP>
__device__ __forceinline__ void slots_from_blocks(TileSlots<D, KEYS, STEP>& ts, const PagedArgs& a, int first, int lane, int kv_len, int kv0) {
  using G = StageGeom<D>;
  const int in_block = (1 << a.block_shift) - 1;
#pragma unroll
  for (int u = 0; u < TileSlots<D, KEYS, STEP>::kCount; ++u) {
    const int instr = first + STEP * u;
    const int row = (instr * 64 + lane) / G::kChunks;
    int tok = kv0 + row;
    tok = tok < kv_len ? tok : kv_len - 1;
    int block = ts.slot[u];
    block = block < 0 ? 0 : (block >= a.num_blocks ? a.num_blocks - 1 : block);
    ts.slot[u] = (block << a.block_shift) + (tok & in_block);
  }
}
template <int D, int KEYS, int STEP>
__device__ __forceinline__ void fetch_tile_slots(TileSlots<D, KEYS, STEP>& ts, const PagedArgs& a, const int32_t* table, int first, int lane,
                                                 int kv_len, int kv0) {
  request_tile_blocks(ts, a, table, first, lane, kv_len, kv0);
  slots_from_blocks(ts, a, first, lane, kv_len, kv0);
}

// CPOL: cache-policy bits of the load instructions (2 = nt: lines marked for early replacement, for rows that no
// other workgroup reads again).
template <int CPOL = 0, int D, int KEYS, int STEP>
__device__ __forceinline__ void issue_tile_loads(const TileSlots<D, KEYS, STEP>& ts, const PagedArgs& a, unsigned char* stage, int first, int lane,
                                                 int kv_head) {
  using G = StageGeom<D>;
  constexpr int kTileBytes = KEYS * G::kRowBytes;
  const int64_t row_elems = (int64_t)a.n_kv_heads * D;
#pragma unroll
  for (int u = 0; u < TileSlots<D, KEYS, STEP>::kCount; ++u) {
    const int instr = first + STEP * u;
    if (instr < TileSlots<D, KEYS, STEP>::kLoadInstr) {
      const int flat = instr * 64 + lane;
      const int row = flat / G::kChunks;
      const int phys = flat % G::kChunks;
      const uint16_t* kp = a.k_cache + ts.slot[u] * row_elems + kv_head * D + k_swizzle<D>(row, phys) * 8;
      const uint16_t* vp = a.v_cache + ts.slot[u] * row_elems + kv_head * D + v_swizzle<D>(row, phys) * 8;
      __builtin_amdgcn_global_load_lds(HYDRA_GLOBAL_PTR(kp), HYDRA_LDS_PTR(stage + instr * 1024), 16, 0, CPOL);
      __builtin_amdgcn_global_load_lds(HYDRA_GLOBAL_PTR(vp), HYDRA_LDS_PTR(stage + kTileBytes + instr * 1024), 16, 0, CPOL);
    }
  }
}

// ---- the wave-tile form on the packed kernel's pipeline --------------------------------------------------
// A prefill chunk is causal attention whose queries are the LAST q_len positions of a context of kv_len keys,
// so a group of four wave tiles runs through the packed kernel's item loop (attn_fwd.hpp: software-pipelined
// key-block steps, fixed softmax reference with a row-sum check) with this source: one item, its K/V tiles
// gathered from the pages.
//
// The gatherer relies on a load instruction's rows (1024 bytes: 4 rows at head_dim 128, 8 at 64) lying in ONE
// cache block, which holds when the block size is at least that many rows (tiles start at multiples of 64 keys):
// the block is then the same for all lanes, the load goes through a buffer descriptor that starts at the group's
// first row and ends with its last valid row (rows past the end of the context arrive as zeros, as in the packed
// kernel), and a tile needs one table entry per load instruction of the wave.  Those entries are looked up one
// tile ahead: lane u of the wave fetches the entry of the wave's load u, the iteration-end wait for all loads
// covers it, and the next iteration's issue reads it lane by lane into scalar registers.  The V tile of an
// iteration comes from the blocks its K tile came from one iteration earlier, so they are kept.
// head_dim 80 (a row is not a whole fraction of 1024 bytes) and smaller blocks take the plain loop further down.
struct PagedSource {
  static constexpr bool kPaged = true;
  const PagedArgs* args;
  const int32_t* table;  // the request's row of the block table
  int64_t q_start;       // first new token of the request in the packed q / out
  int q_len, kv_len;     // new tokens, context (new tokens included)
  int f0, kv_head;       // first flattened wave tile of the group, KV head

  template <int D>
  struct Gather {
    using G = TileGeom<D>;
    static constexpr int kPerWave = G::kLoadInstr / 4;          // load instructions per wave and tile
    static constexpr int kRowsPerInstr = 1024 / G::kRowBytes;   // rows one load instruction covers
    static_assert(G::kLoadInstr % 4 == 0 && 1024 % G::kRowBytes == 0 && TileLoader<D>::kUniformStep, "whole rows per instruction");
    uint32_t k_lo, k_hi, v_lo, v_hi;  // byte address of this KV head's part of cache row 0 (uniform)
    uint32_t row_bytes;               // bytes between cache rows (uniform)
    uint32_t k_lane_off, v_lane_off;  // this lane's 16 bytes inside a load instruction's rows
    const int32_t* table;
    int kv_len, block_shift, last_block, last_entry, wave;
    int next_tile;              // the next K tile to issue, whose table entries `pending` holds
    int32_t pending;            // lane u < kPerWave: table entry of this wave's load u of tile next_tile
    int32_t v_block[kPerWave];  // blocks of the next V tile to issue (uniform)

    // (first key of the rows of this wave's load u of a tile)
    __device__ __forceinline__ int first_key(int tile, int u) const { return tile * kKvTileRows + kRowsPerInstr * (wave + 4 * u); }

    __device__ __forceinline__ void lookup(int tile) {
      // (the lane number is formed here, two instructions, instead of living in a register through the hot loop)
      const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
      pending = 0;
      if (lane < kPerWave) {
        int entry = first_key(tile, lane) >> block_shift;
        entry = entry < last_entry ? entry : last_entry;  // (tiles past the context are looked up but never loaded)
        pending = table[entry];
      }
    }
    __device__ __forceinline__ void take(int32_t (&block)[kPerWave]) const {
#pragma unroll
      for (int u = 0; u < kPerWave; ++u) {
        const int b = __builtin_amdgcn_readlane(pending, u);
        block[u] = b < 0 ? 0 : (b > last_block ? last_block : b);  // a corrupt table cannot make the loads leave the cache
      }
    }
    __device__ __forceinline__ void issue_tile(int tile, const int32_t (&block)[kPerWave], uint32_t lo, uint32_t hi, uint32_t lane_off,
                                               uint32_t lds_dst) const {
#pragma unroll
      for (int u = 0; u < kPerWave; ++u) {
        const int key = first_key(tile, u);
        const uint32_t slot = ((uint32_t)block[u] << block_shift) + ((uint32_t)key & ((1u << block_shift) - 1u));
        const uint64_t base = (((uint64_t)hi << 32) | lo) + (uint64_t)slot * row_bytes;
        int valid = kv_len - key;
        valid = valid > kRowsPerInstr ? kRowsPerInstr : valid;
        u32x4_t rsrc;
        rsrc[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
        rsrc[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
        rsrc[2] = __builtin_amdgcn_readfirstlane(valid > 0 ? (uint32_t)(valid - 1) * row_bytes + D * 2 : 0u);
        rsrc[3] = 0x00020000u;
        const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_dst + (wave + 4 * u) * 1024);
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" : : "s"(m0), "v"(lane_off), "s"(rsrc));
      }
    }

    __device__ __forceinline__ void init(const PagedSource& src, int kv_head, int wave_, int lane) {
      const PagedArgs& a = *src.args;
      wave = wave_;
      __builtin_assume(wave >= 0 && wave < kWavesPerItem);
      table = src.table;
      kv_len = src.kv_len;
      block_shift = a.block_shift;
      last_block = a.num_blocks - 1;
      last_entry = a.max_blocks_per_seq - 1;
      row_bytes = __builtin_amdgcn_readfirstlane((uint32_t)a.n_kv_heads * (D * 2));
      const uint64_t kb = (uint64_t)(uintptr_t)(a.k_cache + (int64_t)kv_head * D), vb = (uint64_t)(uintptr_t)(a.v_cache + (int64_t)kv_head * D);
      k_lo = __builtin_amdgcn_readfirstlane((uint32_t)kb);
      k_hi = __builtin_amdgcn_readfirstlane((uint32_t)(kb >> 32));
      v_lo = __builtin_amdgcn_readfirstlane((uint32_t)vb);
      v_hi = __builtin_amdgcn_readfirstlane((uint32_t)(vb >> 32));
      // (the swizzles repeat from one load instruction of the wave to its next, 16 or 32 rows further on)
      const int in_instr = lane / G::kChunks, phys = lane % G::kChunks, row = kRowsPerInstr * wave + in_instr;
      k_lane_off = (uint32_t)in_instr * row_bytes + k_swizzle<D>(row, phys) * 16;
      v_lane_off = (uint32_t)in_instr * row_bytes + v_swizzle<D>(row, phys) * 16;
      next_tile = 0;
      lookup(0);
    }
    // K tile 0
    __device__ __forceinline__ void issue_first(uint32_t k_dst) {
      take(v_block);
      issue_tile(0, v_block, k_lo, k_hi, k_lane_off, k_dst);
      next_tile = 1;
      lookup(1);
    }
    // The V tile that goes with the K tile issued last (if has_v) and the next K tile (if has_k).  Both sets of
    // table entries are in scalar registers before the first load goes out: the compiler waits for the look-up
    // where its result is first read, and a wait placed behind tile loads would wait for those as well.
    __device__ __forceinline__ void issue(bool has_v, uint32_t v_dst, bool has_k, uint32_t k_dst) {
      if (!has_v && !has_k) return;
      int32_t k_block[kPerWave];
      take(k_block);
      if (has_v) issue_tile(next_tile - 1, v_block, v_lo, v_hi, v_lane_off, v_dst);
      if (has_k) issue_tile(next_tile, k_block, k_lo, k_hi, k_lane_off, k_dst);
#pragma unroll
      for (int u = 0; u < kPerWave; ++u) v_block[u] = k_block[u];
      ++next_tile;
      lookup(next_tile);
    }
  };
};

// The same rows on their way through registers: ordinary loads, which complete in the order they were issued and
// can be counted, so that a wave can have the NEXT tile's rows in flight while it computes on the current one
// (direct-to-LDS loads land in no particular order: a wave that uses them can only wait for all of its loads).
// The rows are written to the stage, in the layout the direct loads would have produced, when their turn comes.
template <int D, int KEYS>
struct TileRegs {
  static constexpr int kLoadInstr = KEYS * StageGeom<D>::kRowBytes / 1024;
  u32x4_t k[kLoadInstr], v[kLoadInstr];
};
template <int D, int KEYS>
__device__ __forceinline__ void load_tile_regs(TileRegs<D, KEYS>& regs, const TileSlots<D, KEYS, 1>& ts, const PagedArgs& a, int lane, int kv_head) {
  using G = StageGeom<D>;
  const int64_t row_elems = (int64_t)a.n_kv_heads * D;
#pragma unroll
  for (int u = 0; u < TileRegs<D, KEYS>::kLoadInstr; ++u) {
    const int flat = u * 64 + lane;
    const int row = flat / G::kChunks, phys = flat % G::kChunks;
    const uint16_t* kp = a.k_cache + ts.slot[u] * row_elems + kv_head * D + k_swizzle<D>(row, phys) * 8;
    const uint16_t* vp = a.v_cache + ts.slot[u] * row_elems + kv_head * D + v_swizzle<D>(row, phys) * 8;
    // (nt: each key of the context is read by exactly one wave of one workgroup)
    regs.k[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(kp));
    regs.v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(vp));
  }
}
template <int D, int KEYS>
__device__ __forceinline__ void store_tile_regs(const TileRegs<D, KEYS>& regs, unsigned char* stage, int lane) {
  constexpr int kTileBytes = KEYS * StageGeom<D>::kRowBytes;
#pragma unroll
  for (int u = 0; u < TileRegs<D, KEYS>::kLoadInstr; ++u) {
    *reinterpret_cast<u32x4_t*>(stage + u * 1024 + lane * 16) = regs.k[u];
    *reinterpret_cast<u32x4_t*>(stage + kTileBytes + u * 1024 + lane * 16) = regs.v[u];
  }
}

// A wave's state for 32 * QS query rows (QS sub-tiles of 32) and the arithmetic of one 64-key tile:
// S^T = K Q^T, mask, online softmax (running maximum, rescaling), O^T += V^T P^T.
template <int D, int QS>
struct WaveTile {
  using G = StageGeom<D>;
  static constexpr int KS = G::kQkSteps;
  static constexpr int CC = G::kPvChunks;
  static constexpr int ROWB = G::kRowBytes;
  bf16x8_t qf[QS][KS];  // B operand: lane (m, hf) holds its row's columns hf*D/2 + 8*s .. +7
  int q_lim[QS];        // largest visible key index of this lane's row in sub-tile qs
  uint32_t k_off[KS], v_off[CC];
  f32x16_t o_acc[QS][CC];
  float row_max[QS], row_sum[QS];
  float c;  // softmax_scale * log2(e)
  int hf;

  __device__ __forceinline__ void init(int lane, float scale_log2) {
    const int m = lane & 31, sl = lane & 15, grp = (lane >> 4) & 1;
    hf = lane >> 5;
    c = scale_log2;
#pragma unroll
    for (int s = 0; s < KS; ++s) k_off[s] = m * ROWB + k_swizzle<D>(m, KS * hf + s) * 16;
    const int r = 4 * hf + (sl >> 2);
#pragma unroll
    for (int cc = 0; cc < CC; ++cc) {
      const int chunk = 4 * cc + 2 * grp + ((sl & 3) >> 1);
      v_off[cc] = r * ROWB + v_swizzle<D>(r, chunk) * 16 + 8 * (sl & 1);  // inside the V rows of a stage
    }
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
      row_max[qs] = -3.0e38f;
      row_sum[qs] = 0.f;
#pragma unroll
      for (int cc = 0; cc < CC; ++cc)
#pragma unroll
        for (int r2 = 0; r2 < 16; ++r2) o_acc[qs][cc][r2] = 0.f;
    }
  }
  // row pointer: this lane's query row of sub-tile qs (columns 0 .. D-1 contiguous)
  __device__ __forceinline__ void load_q(int qs, const uint16_t* row_ptr, int limit) {
    q_lim[qs] = limit;
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[qs][s] = *reinterpret_cast<const bf16x8_t*>(row_ptr + hf * (D / 2) + 8 * s);
  }

  // one K/V tile of 32 * RBN keys whose first key is kv0, already complete in `stage` (K rows, then V rows);
  // need_mask: some key of the tile lies past some row's limit
  template <int RBN = 2>
  __device__ __forceinline__ void tile(const unsigned char* stage, int kv0, bool need_mask) {
    // ---- S^T = K Q^T ----
    f32x16_t s_acc[RBN][QS];  // [rb][qs]
    // (consecutive matrix instructions go to different accumulators wherever there are several: one that
    // continues the accumulator of the instruction right before it waits for that one to finish)
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb)
#pragma unroll
      for (int qs = 0; qs < QS; ++qs)
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[rb][qs][r] = 0.f;
#pragma unroll
    for (int s = 0; s < KS; ++s)
#pragma unroll
      for (int rb = 0; rb < RBN; ++rb) {
        const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(stage + rb * 32 * ROWB + k_off[s]);
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) s_acc[rb][qs] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qs][s], s_acc[rb][qs], 0, 0, 0);
      }
    if (need_mask) {
#pragma unroll
      for (int rb = 0; rb < RBN; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv0 + 32 * rb + 8 * (r >> 2) + 4 * hf + (r & 3);
#pragma unroll
          for (int qs = 0; qs < QS; ++qs)
            if (key > q_lim[qs]) s_acc[rb][qs][r] = -__builtin_inff();
        }
    }
    // ---- online softmax, P in bf16 ----
    bf16x8_t p_frag[QS][RBN][2];  // [qs][rb][s2]
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
      float tmax = s_acc[0][qs][0];
#pragma unroll
      for (int rb = 0; rb < RBN; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s_acc[rb][qs][r]);
      tmax = max_with_other_half(tmax);
      // (a row whose keys are all masked so far keeps the initial, very negative maximum: every
      // exponential below is then exp2(-inf) = 0)
      const float m_new = fmaxf(row_max[qs], tmax);
      const float alpha = fast_exp2((row_max[qs] - m_new) * c);
      row_max[qs] = m_new;
      const float mc = m_new * c;
      float psum = 0.f;
#pragma unroll
      for (int rb = 0; rb < RBN; ++rb) {
        float p[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) p[r] = fast_exp2(__builtin_fmaf(s_acc[rb][qs][r], c, -mc));
        if (need_mask) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kv0 + 32 * rb + 8 * (r >> 2) + 4 * hf + (r & 3);
            if (key > q_lim[qs]) p[r] = 0.f;
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) psum += p[r];
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
          for (int e = 0; e < 8; e += 2) {
            f32x2_t pr = {p[8 * s2 + e], p[8 * s2 + e + 1]};
            bf16x2_t pb = __builtin_convertvector(pr, bf16x2_t);
            p_frag[qs][rb][s2][e] = pb[0];
            p_frag[qs][rb][s2][e + 1] = pb[1];
          }
      }
      row_sum[qs] = row_sum[qs] * alpha + psum;
#pragma unroll
      for (int cc = 0; cc < CC; ++cc)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_acc[qs][cc][r] *= alpha;
    }
    // ---- O^T += V^T P^T ----
#pragma unroll
    for (int rb = 0; rb < RBN; ++rb)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) {
          const unsigned char* vp = stage + RBN * 32 * ROWB + v_off[cc] + (32 * rb + 16 * s2) * ROWB;
          const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_PTR(vp));
          const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_PTR(vp + 8 * ROWB));
          typedef __attribute__((ext_vector_type(8))) short s16x8_t;
          const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, both);
#pragma unroll
          for (int qs = 0; qs < QS; ++qs) o_acc[qs][cc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p_frag[qs][rb][s2], o_acc[qs][cc], 0, 0, 0);
        }
  }

  // normalise this lane's row of sub-tile qs, round to bf16 and store it at out_row (D contiguous elements)
  __device__ __forceinline__ void store_row(int qs, uint16_t* out_row) {
    const float total = sum_with_other_half(row_sum[qs]);
    const float inv = 1.0f / total;
    if (out_row == nullptr) return;  // (every lane takes part in the exchange above)
#pragma unroll
    for (int cc = 0; cc < CC; ++cc)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = 32 * cc + 8 * g4 + 4 * hf;
        if (col < D) {
          f32x2_t a0 = {o_acc[qs][cc][4 * g4] * inv, o_acc[qs][cc][4 * g4 + 1] * inv};
          f32x2_t a1 = {o_acc[qs][cc][4 * g4 + 2] * inv, o_acc[qs][cc][4 * g4 + 3] * inv};
          const bf16x2_t b0 = __builtin_convertvector(a0, bf16x2_t);
          const bf16x2_t b1 = __builtin_convertvector(a1, bf16x2_t);
          u32x2_t pk = {__builtin_bit_cast(uint32_t, b0), __builtin_bit_cast(uint32_t, b1)};
          *reinterpret_cast<u32x2_t*>(out_row + col) = pk;
        }
      }
  }
};

// Few new tokens (q_len * group <= 32: decode steps above all): ALL (token, head) pairs of one (request, KV
// head) form one tile of rows, row = token * group + head_in_group, and the four waves split the KEYS
// instead of the rows: wave w takes the half tiles (32 keys) w, w + 4, ... into a stage of its own (no
// workgroup barrier inside the loop; a wave's next half tile travels through registers while it computes on
// the current one, see TileRegs), and the four partial results (maximum, sum, unnormalised output per row)
// are merged through LDS at the end.
template <int D>
__device__ __forceinline__ void run_packed_rows(const PagedArgs& a, unsigned char* smem, float* s_stats, const int32_t* table, int64_t q_start,
                                                int q_len, int kv_len, int kv_head, int request, int split) {
  using G = StageGeom<D>;
  using W = WaveTile<D, 1>;
  constexpr int kHalfKeys = kKvTileRows / 2;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 31;
  const int shift = kv_len - q_len;
  const int n_rows = q_len * a.group;

  W w;
  w.init(lane, a.scale_log2);
  int r = m;
  const bool valid = r < n_rows;
  r = valid ? r : n_rows - 1;
  const int token = r / a.group;
  const int head = kv_head * a.group + (r - token * a.group);
  w.load_q(0, a.q + (q_start + token) * a.q_stride + head * D, shift + token);

  unsigned char* stage = smem + wave * G::kSlotBytes;
  const int n_halves = (kv_len + kHalfKeys - 1) / kHalfKeys;
  int h_begin, h_end;
  int per_share, n_shares;
  share_plan(n_halves, a.halves_per_split, per_share, n_shares);
  split_range(n_halves, per_share, split, h_begin, h_end);
  if (h_begin >= h_end) return;  // past the context's last share: the combine kernel knows and skips it
  const bool whole = n_halves <= a.halves_per_split;  // the context fits one share: this workgroup writes the output
  // The rows of half tile h + 4 travel (into registers) while half tile h is computed on, and the block-table
  // look-up of half tile h + 8 travels behind them; its entries are not touched before the top of the next round.
  TileSlots<D, kHalfKeys, 1> slots;
  TileRegs<D, kHalfKeys> regs;
  if (h_begin + wave < h_end) {
    fetch_tile_slots(slots, a, table, 0, lane, kv_len, (h_begin + wave) * kHalfKeys);
    load_tile_regs(regs, slots, a, lane, kv_head);
    if (h_begin + wave + kWavesPerGroup < h_end) request_tile_blocks(slots, a, table, 0, lane, kv_len, (h_begin + wave + kWavesPerGroup) * kHalfKeys);
  }
  for (int h = h_begin + wave; h < h_end; h += kWavesPerGroup) {
    const int kv0 = h * kHalfKeys;
    store_tile_regs(regs, stage, lane);
    if (h + kWavesPerGroup < h_end) {
      slots_from_blocks(slots, a, 0, lane, kv_len, (h + kWavesPerGroup) * kHalfKeys);
      load_tile_regs(regs, slots, a, lane, kv_head);
      if (h + 2 * kWavesPerGroup < h_end) request_tile_blocks(slots, a, table, 0, lane, kv_len, (h + 2 * kWavesPerGroup) * kHalfKeys);
    }
    __builtin_amdgcn_sched_barrier(0);  // (the loads go out before the arithmetic, not wherever the scheduler finds room)
    w.template tile<1>(stage, kv0, kv0 + kHalfKeys - 1 > shift);
  }

  // ---- merge the four waves' partial results ----
  // statistics: s_stats[wave * 64 + lane] = maximum, the sums 256 floats further on (the maximum is the same
  // in both lanes of a row, the sum is the lane's half)
  s_stats[wave * 64 + lane] = w.row_max[0];
  s_stats[256 + wave * 64 + lane] = w.row_sum[0];
  // unnormalised outputs, register by register, lane-major, into the wave's own slot
  float* mine = reinterpret_cast<float*>(stage);
#pragma unroll
  for (int cc = 0; cc < W::CC; ++cc)
#pragma unroll
    for (int i = 0; i < 16; ++i) mine[(cc * 16 + i) * 64 + lane] = w.o_acc[0][cc][i];
  __syncthreads();
  if (wave != 0) return;
  float scale_of[kWavesPerGroup];
  {
    float top = s_stats[lane];
#pragma unroll
    for (int o = 1; o < kWavesPerGroup; ++o) top = fmaxf(top, s_stats[o * 64 + lane]);
    float total = 0.f;
#pragma unroll
    for (int o = 0; o < kWavesPerGroup; ++o) {
      // (a wave that saw no key of this row still holds the initial maximum: weight 0)
      scale_of[o] = fast_exp2((s_stats[o * 64 + lane] - top) * w.c);
      total += scale_of[o] * s_stats[256 + o * 64 + lane];
    }
    w.row_sum[0] = total;
  }
#pragma unroll
  for (int cc = 0; cc < W::CC; ++cc)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      float acc = w.o_acc[0][cc][i] * scale_of[0];
#pragma unroll
      for (int o = 1; o < kWavesPerGroup; ++o)
        acc += scale_of[o] * reinterpret_cast<const float*>(smem + o * G::kSlotBytes)[(cc * 16 + i) * 64 + lane];
      w.o_acc[0][cc][i] = acc;
    }
  if (whole) {
    w.store_row(0, valid ? a.out + ((q_start + token) * a.n_q_heads + head) * D : nullptr);
    return;
  }
  // this share's partial result: the row's maximum, its sum (both halves of the row added up) and its
  // unnormalised output, for the combine kernel
  const float total = sum_with_other_half(w.row_sum[0]);
  float top = s_stats[lane];
#pragma unroll
  for (int o = 1; o < kWavesPerGroup; ++o) top = fmaxf(top, s_stats[o * 64 + lane]);
  float* rec = a.partials + (((int64_t)request * a.n_kv_heads + kv_head) * a.n_splits + split) * kPartialFloats<D>;
  if (valid) {
    if (w.hf == 0) {
      rec[m] = top;
      rec[kRows + m] = total;
    }
    float* row = rec + 2 * kRows + m * D;
#pragma unroll
    for (int cc = 0; cc < W::CC; ++cc)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = 32 * cc + 8 * g4 + 4 * w.hf;
        if (col < D) {
          f32x4_t v = {w.o_acc[0][cc][4 * g4], w.o_acc[0][cc][4 * g4 + 1], w.o_acc[0][cc][4 * g4 + 2], w.o_acc[0][cc][4 * g4 + 3]};
          *reinterpret_cast<f32x4_t*>(row + col) = v;
        }
      }
  }
}

#endif  // __HIP_DEVICE_COMPILE__

// grid = batch * n_kv_heads * n_splits + n_tile_wgs workgroups, one-dimensional.
//   - The first batch * n_kv_heads * n_splits run the packed-rows form (decode steps, chunks of a few tokens):
//     n_splits workgroups per (request, KV head), each a share of the context; requests of the other form are
//     left at once.
//   - The last n_tile_wgs run the wave-tile form: workgroup w of them serves KV head w % n_kv_heads and group
//     number w / n_kv_heads in the list of all groups of four wave tiles of all requests that take this form
//     (q_len * group > 32), which it finds for itself: the 256 threads add up the groups of a slice of the
//     requests each and a scan over the slices gives every request's place; the requests of this form (few:
//     prefill chunks) are then ranked by context length in LDS and the groups counted off in that order, the
//     longest context first and inside a request from the last token tile down (which sees the most keys).
//     The host sizes n_tile_wgs from the total number of new tokens (it cannot see the lengths); workgroups past
//     the last group leave at once.
// The hardware starts workgroups in index order.  Measured on the hybrid benchmark batch (96 decode steps, 4
// chunks): decode steps first and then the chunks' workgroups from the longest down, 82 us; chunks first in
// batch order, 88 us (the decode steps then wait for the few free slots and the long ones among them end the
// kernel); a grid with one row of workgroups per request (which made every decode request pay for the widest
// chunk's row with workgroups that only looked at its length and left, and started a chunk that stood last in the
// batch last), 95 us.
// Both forms live in one kernel so that the decode requests and the prefill chunks of a batch run side by
// side on the chip; two workgroups per compute unit (a wave keeps within 256 registers, a workgroup within
// half of the LDS).
template <int D>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_paged_kernel(const PagedArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
  using G = StageGeom<D>;
  constexpr int kLds = G::kLdsBytes > TileGeom<D>::kLdsBytes ? G::kLdsBytes : TileGeom<D>::kLdsBytes;
  __shared__ __attribute__((aligned(1024))) unsigned char smem[kLds];
  __shared__ float s_stats[2 * kWavesPerGroup * 64];

  // new tokens and context of request b (context cut to what the table can describe; q_len 0: nothing to do,
  // also for a context shorter than its new tokens, which is invalid)
  auto lengths_of = [&](int b, int& q_len, int& kv_len) {
    q_len = a.cu_seqlens_q[b + 1] - a.cu_seqlens_q[b];
    kv_len = a.kv_lens[b];
    const int64_t table_keys = (int64_t)a.max_blocks_per_seq << a.block_shift;
    if (kv_len > table_keys) kv_len = (int)table_keys;
    if (q_len < 0 || kv_len < q_len) q_len = 0;
  };
  int b, kv_head, f0 = 0;
  const int n_rows_wgs = (int)gridDim.x - a.n_tile_wgs;
  if ((int)blockIdx.x < n_rows_wgs) {
    const int r = (int)blockIdx.x;
    // (share-major: the workgroups of the first shares, which every request has, lie next to each other and are dealt
    // to all dies alike; the further shares, some of them empty when contexts differ in length, come behind them)
    const int pairs = a.batch * a.n_kv_heads;
    const int split = r / pairs, pair = r - split * pairs;
    b = pair / a.n_kv_heads;
    kv_head = pair - b * a.n_kv_heads;
    int q_len, kv_len;
    lengths_of(b, q_len, kv_len);
    if (q_len == 0 || q_len * a.group > kRows) return;
    run_packed_rows<D>(a, smem, s_stats, a.block_tables + (int64_t)b * a.max_blocks_per_seq, a.cu_seqlens_q[b], q_len, kv_len, kv_head, b, split);
    return;
  }
  {
    // which group of which request: see above.  Thread i adds up requests [i * per, (i + 1) * per).
    int* s_scan = reinterpret_cast<int*>(s_stats);  // [0..3] the waves' groups, [4..7] the waves' requests, [256] = request, [257] = group
    const int target = ((int)blockIdx.x - n_rows_wgs) / a.n_kv_heads;
    kv_head = ((int)blockIdx.x - n_rows_wgs) - target * a.n_kv_heads;
    const int per = (a.batch + 255) / 256;
    auto groups_of = [&](int r, int& kv_len) {
      int q_len;
      lengths_of(r, q_len, kv_len);
      if (q_len * a.group <= kRows) return 0;
      return (((q_len + kRows - 1) / kRows) * a.group + kWavesPerGroup - 1) / kWavesPerGroup;
    };
    const int first = (int)threadIdx.x * per, last = first + per < a.batch ? first + per : a.batch;
    int mine = 0, mine_reqs = 0;  // groups, and requests that have groups, in this thread's slice
    for (int r = first; r < last; ++r) {
      int kv;
      const int n = groups_of(r, kv);
      mine += n;
      mine_reqs += n > 0 ? 1 : 0;
    }
    const int lane_ = threadIdx.x & 63, wave_ = threadIdx.x >> 6;
    int incl = mine, incl_reqs = mine_reqs;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int up = __shfl_up(incl, d), up_reqs = __shfl_up(incl_reqs, d);
      if (lane_ >= d) {
        incl += up;
        incl_reqs += up_reqs;
      }
    }
    if (lane_ == 63) {
      s_scan[wave_] = incl;
      s_scan[4 + wave_] = incl_reqs;
    }
    if (threadIdx.x == 0) s_scan[256] = -1;
    __syncthreads();
    int before = incl - mine, before_reqs = incl_reqs - mine_reqs;  // of the slices ahead of this thread's
    for (int i = 0; i < wave_; ++i) {
      before += s_scan[i];
      before_reqs += s_scan[4 + i];
    }
    const int total_reqs = s_scan[4] + s_scan[5] + s_scan[6] + s_scan[7];
    if (target >= s_scan[0] + s_scan[1] + s_scan[2] + s_scan[3]) return;  // past the last group
    // Requests with the longest contexts first: their workgroups run longest, and the kernel is as long as the
    // last of them.  The requests of this form (few: prefill chunks) are gathered in LDS, ranked by context
    // length, and the groups are counted off in that order.  (More than kMaxSorted of them: batch order.)
    constexpr int kMaxSorted = 256;
    if (total_reqs <= kMaxSorted) {
      int* s_req = reinterpret_cast<int*>(smem);  // the tile stages are not in use yet
      int* s_groups = s_req + kMaxSorted, *s_key = s_req + 2 * kMaxSorted;
      int* s_sorted_req = s_req + 3 * kMaxSorted, *s_sorted_groups = s_req + 4 * kMaxSorted;
      int k = before_reqs;
      for (int r = first; r < last; ++r) {
        int kv;
        const int n = groups_of(r, kv);
        if (n > 0) {
          s_req[k] = r;
          s_groups[k] = n;
          s_key[k] = kv;
          ++k;
        }
      }
      __syncthreads();
      if ((int)threadIdx.x < total_reqs) {
        const int key = s_key[threadIdx.x];
        int rank = 0;
        for (int j = 0; j < total_reqs; ++j) rank += (s_key[j] > key || (s_key[j] == key && j < (int)threadIdx.x)) ? 1 : 0;
        s_sorted_req[rank] = s_req[threadIdx.x];
        s_sorted_groups[rank] = s_groups[threadIdx.x];
      }
      __syncthreads();
      if (threadIdx.x == 0) {
        int at = 0;
        for (int e = 0; e < total_reqs; ++e) {
          const int n = s_sorted_groups[e];
          if (target < at + n) {
            s_scan[256] = s_sorted_req[e];
            s_scan[257] = n - 1 - (target - at);  // from the last group down
            break;
          }
          at += n;
        }
      }
    } else if (target >= before && target < before + mine) {
      int at = before;
      for (int r = first; r < last; ++r) {
        int kv;
        const int n = groups_of(r, kv);
        if (target < at + n) {
          s_scan[256] = r;
          s_scan[257] = n - 1 - (target - at);
          break;
        }
        at += n;
      }
    }
    __syncthreads();
    b = s_scan[256];
    if (b < 0) return;  // (cannot happen: the target was below the total)
    f0 = s_scan[257] * kWavesPerGroup;
    __syncthreads();  // (the scan area is the packed-rows form's statistics area, the lists lie in the tile stages)
  }
  const int64_t q_start = a.cu_seqlens_q[b];
  int q_len, kv_len;
  lengths_of(b, q_len, kv_len);
  const int32_t* table = a.block_tables + (int64_t)b * a.max_blocks_per_seq;
  const int n_tok_tiles = (q_len + kRows - 1) / kRows;
  const int n_wave_tiles = n_tok_tiles * a.group;
  if (f0 >= n_wave_tiles) return;  // (cannot happen: the group was counted from these lengths)
  const int shift = kv_len - q_len;  // keys that precede the first new token

  // The group runs on the packed kernel's pipeline when the cache layout allows (see PagedSource); if its row sums
  // leave that path's range, or the layout does not allow, the plain loop below computes (or recomputes) it.
  if constexpr (TileLoader<D>::kUniformStep) {
    if ((1 << a.block_shift) >= PagedSource::Gather<D>::kRowsPerInstr && a.num_blocks <= (0x7fffffff >> a.block_shift)) {
      PagedSource src;
      src.args = &a;
      src.table = table;
      src.q_start = q_start;
      src.q_len = q_len;
      src.kv_len = kv_len;
      src.f0 = f0;
      src.kv_head = kv_head;
      AttnArgs fa;
      fa.q = a.q;
      fa.k = nullptr;
      fa.v = nullptr;
      fa.out = a.out;
      fa.q_stride = a.q_stride;
      fa.k_stride = 0;
      fa.v_stride = 0;
      fa.cu_seqlens = nullptr;
      fa.items = nullptr;
      fa.ctrl = nullptr;
      fa.n_q_heads = a.n_q_heads;
      fa.group = a.group;
      fa.scale_log2 = a.scale_log2;
      int* s_claim = reinterpret_cast<int*>(s_stats);  // (unused by a paged item; the redo flag lives behind it)
      if (!attn_item_loop<D, true>(fa, src, smem, s_claim, s_claim + 8)) return;
    }
  }

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 31;

  // this wave's tile
  int f = f0 + wave;
  const bool active = f < n_wave_tiles;
  if (!active) f = n_wave_tiles - 1;
  const int tok_tile = f / a.group;
  const int head = kv_head * a.group + (f - tok_tile * a.group);
  const int q0 = tok_tile * kRows;
  const int f_last = (f0 + kWavesPerGroup - 1 < n_wave_tiles ? f0 + kWavesPerGroup - 1 : n_wave_tiles - 1);
  // keys visible to the last new token of a tile that starts at q: shift + min(q + 32, q_len)
  auto keys_of_tile = [&](int q) { return shift + (q + kRows < q_len ? q + kRows : q_len); };
  const int tiles_wg = (keys_of_tile((f_last / a.group) * kRows) + kKvTileRows - 1) / kKvTileRows;
  const int tiles_wave = active ? (keys_of_tile(q0) + kKvTileRows - 1) / kKvTileRows : 0;

  // first K/V tile in flight before anything else, and the second tile's block-table lookup behind it
  TileSlots<D, kKvTileRows, kWavesPerGroup> slots, next_slots;
  fetch_tile_slots(slots, a, table, wave, lane, kv_len, 0);
  issue_tile_loads(slots, a, smem, wave, lane, kv_head);
  if (1 < tiles_wg) fetch_tile_slots(slots, a, table, wave, lane, kv_len, kKvTileRows);

  WaveTile<D, 1> w;
  w.init(lane, a.scale_log2);
  int row = q0 + m;
  row = row < q_len ? row : q_len - 1;
  w.load_q(0, a.q + (q_start + row) * a.q_stride + head * D, shift + row);
  const int min_lim = shift + q0;  // smallest limit among the tile's tokens

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  for (int t = 0; t < tiles_wg; ++t) {
    unsigned char* stage = smem + (t & 1) * G::kStageBytes;
    // tile t + 1 is fetched (its slots arrived during the previous iteration) and tile t + 2 is looked up
    // while tile t is used
    if (t + 1 < tiles_wg) issue_tile_loads(slots, a, smem + ((t + 1) & 1) * G::kStageBytes, wave, lane, kv_head);
    if (t + 2 < tiles_wg) fetch_tile_slots(next_slots, a, table, wave, lane, kv_len, (t + 2) * kKvTileRows);
    if (t < tiles_wave) {
      const int kv0 = t * kKvTileRows;
      w.template tile<2>(stage, kv0, kv0 + kKvTileRows - 1 > min_lim);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    slots = next_slots;
  }
  w.store_row(0, active && q0 + m < q_len ? a.out + ((q_start + q0 + m) * a.n_q_heads + head) * D : nullptr);
#else
  (void)a;
#endif
}

// Merges the partial results of the packed-rows form when contexts were split over workgroups
// (n_splits > 1).  grid = (n_kv_heads, batch), 256 threads.  Requests that took the wave-tile form, have
// no new tokens, or whose context fits one share (already finished by one workgroup) are skipped.
// First the shares' row statistics go to LDS and every row's weights (exp2 of its maximum's distance to the
// overall maximum, divided by the overall sum) are formed there; then every thread adds up 4 output
// columns of one row over the shares.
constexpr int kMaxSplits = 16;

template <int D>
__global__ __launch_bounds__(256) void attn_paged_combine_kernel(const PagedArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
  __shared__ float s_max[kMaxSplits][kRows], s_weight[kMaxSplits][kRows];
  const int b = blockIdx.y, kv_head = blockIdx.x;
  const int64_t q_start = a.cu_seqlens_q[b];
  const int q_len = a.cu_seqlens_q[b + 1] - (int)q_start;
  int kv_len = a.kv_lens[b];
  const int64_t table_keys = (int64_t)a.max_blocks_per_seq << a.block_shift;
  if (kv_len > table_keys) kv_len = (int)table_keys;
  if (q_len <= 0 || kv_len < q_len || q_len * a.group > kRows) return;
  const int n_rows = q_len * a.group;
  const int n_halves = (kv_len + kKvTileRows / 2 - 1) / (kKvTileRows / 2);
  if (n_halves <= a.halves_per_split) return;  // done by one workgroup, which wrote the output itself
  int per_share, n_shares;
  share_plan(n_halves, a.halves_per_split, per_share, n_shares);
  const float* recs = a.partials + ((int64_t)b * a.n_kv_heads + kv_head) * a.n_splits * kPartialFloats<D>;
  // share s, row r: maximum -> s_max, sum -> s_weight (for now)
  for (int i = threadIdx.x; i < n_shares * kRows; i += 256) {
    const int s = i / kRows, r = i - s * kRows;
    const bool live = r < n_rows;
    s_max[s][r] = live ? recs[(int64_t)s * kPartialFloats<D> + r] : 0.f;
    s_weight[s][r] = live ? recs[(int64_t)s * kPartialFloats<D> + kRows + r] : 0.f;
  }
  __syncthreads();
  if (threadIdx.x < kRows) {
    const int r = threadIdx.x;
    float top = s_max[0][r];
    for (int s = 1; s < n_shares; ++s) top = fmaxf(top, s_max[s][r]);
    float total = 0.f;
    for (int s = 0; s < n_shares; ++s) {
      const float w = fast_exp2((s_max[s][r] - top) * a.scale_log2);
      total += w * s_weight[s][r];
      s_max[s][r] = w;
    }
    const float inv = r < n_rows ? 1.0f / total : 0.f;
    for (int s = 0; s < n_shares; ++s) s_weight[s][r] = s_max[s][r] * inv;
  }
  __syncthreads();
  constexpr int kColGroups = D / 4;
  for (int i = threadIdx.x; i < n_rows * kColGroups; i += 256) {
    const int row = i / kColGroups, col = (i - row * kColGroups) * 4;
    const float* src = recs + 2 * kRows + row * D + col;
    f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
    for (int s = 0; s < n_shares; ++s) {
      const f32x4_t v = *reinterpret_cast<const f32x4_t*>(src + (int64_t)s * kPartialFloats<D>);
      const float w = s_weight[s][row];
      acc[0] += w * v[0];
      acc[1] += w * v[1];
      acc[2] += w * v[2];
      acc[3] += w * v[3];
    }
    const int token = row / a.group;
    const int head = kv_head * a.group + (row - token * a.group);
    f32x2_t a0 = {acc[0], acc[1]}, a1 = {acc[2], acc[3]};
    u32x2_t pk = {__builtin_bit_cast(uint32_t, __builtin_convertvector(a0, bf16x2_t)),
                  __builtin_bit_cast(uint32_t, __builtin_convertvector(a1, bf16x2_t))};
    *reinterpret_cast<u32x2_t*>(a.out + ((q_start + token) * a.n_q_heads + head) * D + col) = pk;
  }
#else
  (void)a;
#endif
}

}  // namespace paged
}  // namespace hydra
