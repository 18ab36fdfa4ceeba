// Fused packed variable-length attention forward for gfx950 (MI355X).
//
// One workgroup (4 wavefronts of 256 registers each) runs one work-list item: up to four "wave
// tiles" that share a sequence and a KV head.  A wave tile is 32 consecutive query tokens of one
// query head.  K/V tiles of 64 keys stream global -> LDS with direct-to-LDS 128-bit loads into
// rings of two tiles (a tile is loaded while the previous one is consumed) and are shared by the
// four waves.
//
// The kernel is persistent: two workgroups per compute unit (two waves per SIMD, half of the
// LDS each), each pulling items from the queue of the accelerator die (XCD) it runs on.  The
// prepass puts all items of one (sequence, KV head) into the same queue, next to each other, so
// the workgroups that stream the same K/V rows run on the same die at about the same time and
// share them through that die's L2.  The two workgroups of a compute unit work on different
// items: while one loads Q, stores O or waits at a barrier, the other one's matrix instructions
// fill the SIMDs.
//
// Each wave walks its keys in blocks of 32 and software-pipelines three stages, so that the
// matrix pipe and the vector ALU work side by side also within the wave: while the VALU does the
// softmax of block j, the MFMAs issued between its instructions compute S(j+1) = K(j+1) Q^T and
// O += V(j-1)^T P(j-1).
//
// Per wave and key block (scores kept transposed so that no cross-lane movement is needed between
// the two contractions):
//   S^T[key, query] = K_tile * Q^T        v_mfma_f32_32x32x16_bf16, A = K from LDS, B = Q in registers
//   online softmax over keys: each lane owns one query column and 16 keys per 32-key block, the
//   other 16 live in lane ^ 32 (one v_permlane32_swap per row maximum; row sums are merged once,
//   in the epilogue)
//   O^T[c, query] += V_tile^T * P^T       A = V^T via ds_read_b64_tr_b16 from the row-major V tile,
//                                         B = P, which is exactly the register layout S^T came out in
// The operation is scaled-dot-product attention as costed in the paper's Table 2
// (Attention/encode, Attention/prefill); causal tiles above the diagonal are never loaded.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "attn_careful.hpp"
#include "attn_tiles.hpp"

namespace hydra {

template <int D>
struct TileGeom : RowGeom<D> {
  using RowGeom<D>::kTileBytes;
  // K tiles and V tiles each live in a ring of kRing LDS tiles; loads run kRing - 1 tiles ahead of use
  // (a tile's slot is free again after the barrier that ends the iteration consuming it)
  static constexpr int kRing = 2;
  static constexpr int kPrefetch = kRing - 1;
  // D = 80: the third 32-column block of P V has 16 columns to spare.  The lanes that feed them read bf16 ones
  // from a constant area instead of the V tile, so the matrix unit delivers the softmax row sums in output
  // columns 80..95 and the vector unit does not have to add them up (16 additions per key block and wave).
  // The area covers every offset a V fragment read adds to its lane address (ring slot, key block, step).
  static constexpr bool kSumsFromMatrixUnit = D == 80;
  static constexpr int kOnesBytes = kSumsFromMatrixUnit ? (kRing - 1) * kTileBytes + 9 * 1024 : 0;
  static constexpr int kOnesAt = 2 * kRing * kTileBytes + 64;    // (+ slack behind the last V tile)
  static constexpr int kLdsBytes = kOnesAt + kOnesBytes;
};

// Everything below uses gfx950-only types and builtins, so the host pass of hipcc only sees the
// kernel's declaration (it still emits the launch stub).
#if defined(__HIP_DEVICE_COMPILE__)
// Loads of one 64-row K or V tile, global -> LDS, 16 bytes per lane, through a buffer resource
// that covers exactly the rows of this sequence and KV head: rows past the end of the sequence are out
// of range and arrive as zeros (they are masked later; zeros keep V finite).  The descriptor and the
// per-lane offset are fixed for the whole item; the tile advances through the instruction's scalar
// offset, which the hardware's range check takes into account (a scalar offset beyond the end of the
// buffer puts every lane out of range).
//
// The load is issued from inline assembly on purpose: when the compiler knows that vector-memory
// loads write LDS, it makes every later LDS read wait for ALL outstanding loads (vmcnt 0), which
// would serialise the prefetch ring with the compute.  Completion is tracked by hand instead:
// every wave waits for ALL of its outstanding loads (wait_all_loads) at the end of the iteration
// before the one that reads them, followed by the workgroup barrier.  Nothing relies on the order
// in which direct-to-LDS loads complete: a load that misses to HBM was observed to land after a
// younger one that hit in L2.
template <int D>
struct TileLoader {
  using G = TileGeom<D>;
  static constexpr int kPerWave = (G::kLoadInstr + 3) / 4;
  // When four load instructions cover a whole number of rows, the lane offsets of a wave's loads
  // differ by a constant (the swizzle repeats), which also goes into the scalar offset:
  // one offset register instead of kPerWave.
  static constexpr bool kUniformStep = (4 * 64) % G::kChunks == 0 && ((4 * 64) / G::kChunks) % 16 == 0;
  static constexpr int kOffsets = kUniformStep ? 1 : kPerWave;
  u32x4_t rsrc;                 // the sequence's rows of this KV head, from the first row to the end of the last
  uint32_t tile_off;            // bytes from the first row of the sequence to the first row of the next tile
  uint32_t tile_stride;         // bytes between first rows of consecutive tiles
  uint32_t lane_off[kOffsets];  // bytes from the first row of a tile
  uint32_t step_bytes;          // kUniformStep: bytes between the rows of consecutive loads of this wave
  int wave;

  template <bool IS_V>
  __device__ __forceinline__ void init(const uint16_t* base, int64_t stride, int64_t seq_start, int seq_len, int kv_head, int wave_, int lane) {
    wave = wave_;
    __builtin_assume(wave >= 0 && wave < kWavesPerItem);
    const uint32_t row_bytes = (uint32_t)(stride * 2);
    const uint64_t first_row = (uint64_t)(uintptr_t)(base + seq_start * stride + kv_head * D);
    rsrc[0] = __builtin_amdgcn_readfirstlane((uint32_t)first_row);
    rsrc[1] = __builtin_amdgcn_readfirstlane((uint32_t)(first_row >> 32) & 0xffffu);
    rsrc[2] = __builtin_amdgcn_readfirstlane((uint32_t)(((int64_t)(seq_len - 1) * stride + D) * 2));
    rsrc[3] = 0x00020000u;
    tile_off = 0;
    tile_stride = __builtin_amdgcn_readfirstlane((uint32_t)kKvTileRows * row_bytes);
    step_bytes = __builtin_amdgcn_readfirstlane((uint32_t)((4 * 64) / G::kChunks) * row_bytes);
#pragma unroll
    for (int u = 0; u < kOffsets; ++u) {
      const int flat = (wave + 4 * u) * 64 + lane;
      const int row = flat / G::kChunks, phys = flat % G::kChunks;
      const int chunk = IS_V ? v_swizzle<D>(row, phys) : k_swizzle<D>(row, phys);
      lane_off[u] = (uint32_t)row * row_bytes + chunk * 16;
    }
  }
  // Issues load u (0 .. kPerWave - 1) of this wave's share of the next tile; lds_dst: LDS byte address
  // of the tile's ring slot.
  __device__ __forceinline__ void issue_piece(int u, uint32_t lds_dst) const {
    const int instr = wave + 4 * u;
    if (instr < G::kLoadInstr) {
      // (m0 is reserved: the compiler only ever sets it immediately before an instruction of its own that reads it)
      const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_dst + instr * 1024);
      const uint32_t soff = __builtin_amdgcn_readfirstlane(tile_off + (kUniformStep ? (uint32_t)u * step_bytes : 0u));
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                   :
                   : "s"(m0), "v"(lane_off[kUniformStep ? 0 : u]), "s"(rsrc), "s"(soff));
    }
  }
  // Issues all of this wave's loads of the next tile at once and moves on to the tile after it.
  __device__ __forceinline__ void issue_next(uint32_t lds_dst) {
#pragma unroll
    for (int u = 0; u < kPerWave; ++u) issue_piece(u, lds_dst);
    tile_off += tile_stride;
  }
};

// Waits until none of this wave's vector-memory operations is in flight.
__device__ __forceinline__ void wait_all_loads() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }


// ---- matrix instructions -------------------------------------------------------------------
// With 256 registers per wave the kernel uses no accumulation registers at all (the compiler
// splits the budget in two halves as soon as one is needed), so scores and output accumulators
// live in ordinary registers, where the softmax and the epilogue read them directly.
// O += V^T P goes through the compiler's builtin, which inserts the wait states the readers of the
// result need.  S = K Q^T is written as inline assembly: measured faster at head_dim 128 (the
// compiler pads every builtin with its own wait states and is freer to move it).  The compiler does
// not see these as matrix instructions, so
//   - s_results_to_valu() supplies the wait states between the last of them and the first reader of
//     S where no other matrix instruction follows (inside the pipeline steps the trailing PV
//     instructions cover them);
//   - an output that nobody reads must still be kept reserved until the instruction has retired
//     (the compiler takes an assembly statement's outputs as written the moment it issues).
typedef __attribute__((ext_vector_type(4))) uint32_t qreg_t;

// O += A(vf) * B(pf)
__device__ __forceinline__ void mfma_pv(f32x16_t& O, const bf16x8_t& vf, const bf16x8_t& pf) {
  O = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, O, 0, 0, 0);
}
// S = A(kf) * B(q), then S += A(kf) * B(q)
__device__ __forceinline__ void mfma_qk_zero(f32x16_t& S, const bf16x8_t& kf, const qreg_t& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(S) : "v"(kf), "v"(q));
}
__device__ __forceinline__ void mfma_qk_acc(f32x16_t& S, const bf16x8_t& kf, const qreg_t& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(S) : "v"(kf), "v"(q));
}
// Wait states after the last QK matrix instruction, before anything else touches S.
__device__ __forceinline__ void s_results_to_valu(f32x16_t (&S)[1]) { asm volatile("s_nop 15\n\ts_nop 3" : "+v"(S[0])); }
__device__ __forceinline__ void s_results_to_valu(f32x16_t (&S)[2]) { asm volatile("s_nop 15\n\ts_nop 3" : "+v"(S[0]), "+v"(S[1])); }

#endif  // __HIP_DEVICE_COMPILE__

// Scheduling hints: keep the listed instruction classes in this order inside the current region.
#define HYDRA_SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

// Every workgroup of the grid ends up making exactly ONE failing claim on every queue: on its own when that
// runs dry, on each of the others while it looks for work to steal (a queue found empty is not asked again).
// A queue of n items has therefore been asked n + (workgroups) times when the kernel ends, and the workgroup
// whose claim returns position n + (workgroups) - 1 is the last that will ever touch that head in this call: it
// puts the head back to zero, so that the next attention call on the same work list (the next layer of the same
// batch) finds a clean control block.  No counter of finished workgroups is needed, and no launch to tidy up.
// Called by the lane that holds the position.
__device__ __forceinline__ void reset_head_if_last(WorkControl* ctrl, int y, int pos, int n_items) {
  if (pos == n_items + (int)gridDim.x - 1) atomicExch(&ctrl->queue_head[y * kHeadStride], 0);
}

// Claims the next unclaimed entry of queue y.  Called by all lanes of ONE wave; returns the list
// index, or -1 when the queue is empty.
__device__ __forceinline__ int claim_from(WorkControl* ctrl, int y, int lane) {
  const int begin = ctrl->xcd_start[y], end = ctrl->xcd_start[y + 1];
  int pos = 0;
  if (lane == 0) {
    pos = atomicAdd(&ctrl->queue_head[y * kHeadStride], 1);
    reset_head_if_last(ctrl, y, pos, end - begin);
  }
  pos = __builtin_amdgcn_readfirstlane(pos);
  return pos < end - begin ? begin + pos : -1;
}

// A workgroup whose own die's queue is empty helps the other dies: one claim attempt per queue it
// has not yet found empty (`empty_mask`, kept by the caller), starting at a different neighbour for
// different workgroups.  Heads only grow, so a queue found empty stays empty and every workgroup
// makes at most seven failing attempts in its life: no polling, no storm of atomics at the end of
// the kernel.  Returns the list index or -1 when all queues are empty.
__device__ __forceinline__ int steal_item(WorkControl* ctrl, int xcc, int first, int lane, uint32_t& empty_mask) {
  for (int k = 0; k < kXcds - 1; ++k) {
    const int y = (xcc + 1 + (first + k) % (kXcds - 1)) & (kXcds - 1);
    if (empty_mask & (1u << y)) continue;
    const int idx = claim_from(ctrl, y, lane);
    if (idx >= 0) return idx;
    empty_mask |= 1u << y;
  }
  return -1;
}

constexpr int kKeyBlock = 32;         // keys per pipeline step

template <int N>
using NextRB = std::integral_constant<int, N>;  // key block the following step reads in the same tiles (-1: none)

// LDS fragments are requested this many work units (one K or V^T fragment and the matrix instructions it feeds)
// ahead of their use.  Each unit of distance keeps one more K and one more V^T fragment (8 registers) in flight.
// (A distance of three was measured at head_dim 80 and 128, which have the registers: no faster.)
template <int D>
constexpr int kFragsAhead = 2;

#if defined(__HIP_DEVICE_COMPILE__)
// LDS fragments of the first PF QK units and the first PF PV units of a pipeline step.
template <int PF>
struct StepFrags {
  bf16x8_t k[PF], v[PF];
};
#endif
constexpr float kMaxRowSum = 1.0995116e12f;  // 2^40: largest row sum (relative to the reference) the fast kernel accepts


// Where a workgroup's items and their K/V rows come from.  The packed kernel (below) takes items from the work
// list's queues and K/V rows from the packed batch; the paged kernel runs ONE item per call, handed over in its
// source object, with K/V rows gathered from cache pages and queries that are the LAST q_len positions of a
// context of kv_len keys (see attn_paged.hpp for that source).
struct PackedSource {
  static constexpr bool kPaged = false;
  template <int D>
  struct Gather {};  // (the paged source's K/V gatherer; the packed rows use two TileLoaders)
};

#if defined(__HIP_DEVICE_COMPILE__)
// The item loop of a workgroup (4 waves).  smem: TileGeom<D>::kLdsBytes bytes of LDS, 1024-aligned; s_claim: 4
// ints, s_redo: 8 ints of LDS.  Packed source: runs until the queues are empty.  Paged source: runs the source's
// item and returns whether its row sums left the fast path's range (same value in every thread; the caller then
// recomputes the item with its own careful routine).
template <int D, bool CAUSAL, class Src>
__device__ __forceinline__ bool attn_item_loop(const AttnArgs& a, const Src& src, unsigned char* smem, int* s_claim, int* s_redo) {
  using G = TileGeom<D>;
  constexpr int KS = G::kQkSteps;
  constexpr int CC = G::kPvChunks;
  constexpr int ROWB = G::kRowBytes;
  constexpr int NQ = KS;      // QK work units per key block: step s = one K fragment read + 2 MFMAs (qs = 0, 1)
  constexpr int NP = 2 * CC;  // PV work units per key block: (s2, cc) = one V^T fragment + 2 MFMAs
  constexpr int PF = kFragsAhead<D>;
  // LDS: K ring then V ring; tile t of either lives in ring slot t % kRing.
  constexpr int R = G::kRing, PD = G::kPrefetch;
  const uint32_t k_ring = (uint32_t)(uintptr_t)HYDRA_LDS_PTR(smem);  // LDS byte addresses
  const uint32_t v_ring = k_ring + R * G::kTileBytes;

  const int lane_id = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // die this workgroup runs on (hardware id register XCC_ID, bits 3:0)
  const int xcc = (int)__builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20) & (kXcds - 1);
  // s_redo: an item whose exponentials left the fast path's range: {flag, first token, length, first wave tile, KV
  // head}, posted by the waves that noticed, acted upon by the whole workgroup at the top of its next round.
  if (threadIdx.x == 0) s_redo[0] = 0;
  if constexpr (G::kSumsFromMatrixUnit) {
    static_assert((R - 1) * G::kTileBytes + kKvTileRows * ROWB - 8 * ROWB + 8 <= G::kOnesBytes, "a V fragment read stays inside the ones");
    for (int i = threadIdx.x * 16; i < G::kOnesBytes; i += 256 * 16)
      *reinterpret_cast<u32x4_t*>(HYDRA_LDS_BYTE(k_ring + G::kOnesAt + i)) = u32x4_t{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
  }

  // Wave 0 claims the items for the whole workgroup, one round ahead: the claim for the next
  // round is issued at the top of a round, resolved (and the item read) before the hot loop, and
  // posted in LDS after it, so that none of its latency shows.
  auto post_claim = [&](int idx) {  // wave 0: read the item and post it for the next round
    WorkItem it = make_int4(0, 0, 0, 0);
    if (idx >= 0) it = a.items[idx];
    // (used by the whole wave right here, so that the load has completed on every code path that
    // goes on to the hot loop; see the note at pending_claim)
    it.x = __builtin_amdgcn_readfirstlane(it.x);
    it.y = __builtin_amdgcn_readfirstlane(it.y);
    it.z = __builtin_amdgcn_readfirstlane(it.z);
    it.w = __builtin_amdgcn_readfirstlane(it.w);
    if (lane_id == 0) {
      s_claim[0] = it.x;
      s_claim[1] = it.y;
      s_claim[2] = it.z;
      s_claim[3] = it.w;
    }
  };
  int own_begin = 0, own_count = 0;
  if constexpr (!Src::kPaged) {
    own_begin = a.ctrl->xcd_start[xcc];
    own_count = a.ctrl->xcd_start[xcc + 1] - own_begin;
  }
  // Q: a wave's 32 rows come in with direct-to-LDS loads that cover whole rows (loaded straight
  // into the B-operand register layout, one instruction would touch 32 different rows: one address
  // cycle per row in the memory pipeline), into a private staging area in K-tile layout, and are
  // read back with the lane pattern of the K reads.  Staging area: the V ring, which is idle from
  // an item's last iteration until the barrier before the next item's first key block.  The loads
  // of the NEXT item are issued as soon as the current item's last iteration is over, ahead of the
  // epilogue, so that their latency hides behind it.
  static_assert(kWavesPerItem * kWaveTileRows * ROWB <= R * G::kTileBytes, "the Q tiles of the four waves fit the V ring");
  constexpr int kRowInstr = kWaveTileRows * G::kChunks / 64;  // 64-lane instructions that cover a 32-row tile
  static_assert(kWaveTileRows * G::kChunks % 64 == 0, "whole instructions");
  const uint32_t q_stage = v_ring + wave * (kWaveTileRows * ROWB);
  auto issue_q_loads = [&](int64_t seq_start, int seq_len, int q0, int head, int lane) {
    const uint64_t base = (uint64_t)(uintptr_t)(a.q + (seq_start + q0) * a.q_stride + head * D);
    const uint32_t q_row_bytes = (uint32_t)(a.q_stride * 2);
    const int rows = seq_len - q0 < kWaveTileRows ? seq_len - q0 : kWaveTileRows;
    u32x4_t rsrc;
    rsrc[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
    rsrc[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
    rsrc[2] = __builtin_amdgcn_readfirstlane((uint32_t)(rows - 1) * q_row_bytes + D * 2);  // rows past the end arrive as zeros
    rsrc[3] = 0x00020000u;
#pragma unroll
    for (int i = 0; i < kRowInstr; ++i) {
      const int flat = i * 64 + lane;
      const int row = flat / G::kChunks, phys = flat % G::kChunks;
      const uint32_t off = (uint32_t)row * q_row_bytes + k_swizzle<D>(row, phys) * 16;
      const uint32_t m0 = __builtin_amdgcn_readfirstlane(q_stage + i * 1024);
      // (nt: Q is read once; marking its lines for early replacement leaves the L2 to the K/V rows that are re-read)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen nt lds" : : "s"(m0), "v"(off), "s"(rsrc));
    }
  };
  bool q_ahead = false;      // the current item's Q loads were issued at the end of the previous round
  bool own_empty = false;    // this die's queue has run out (same value in all waves)
  uint32_t empty_mask = 0;   // wave 0: other dies' queues found empty
  if constexpr (!Src::kPaged) {
    if (wave == 0) post_claim(claim_from(a.ctrl, xcc, lane_id));
  }

  for (;;) {  // one work item per round
  __syncthreads();
  if constexpr (!Src::kPaged)
  if (__builtin_expect(__builtin_amdgcn_readfirstlane(s_redo[0]) != 0, 0)) {
    // The previous round's item has to be redone carefully.  Its (wrong) output rows are already stored and are
    // overwritten by the same waves; the loads of the next item's Q, in flight into the V ring, are waited for
    // first (the routine takes both rings as its stages) and issued again afterwards.
    const int64_t r_start = __builtin_amdgcn_readfirstlane(s_redo[1]);
    const int r_len = __builtin_amdgcn_readfirstlane(s_redo[2]);
    const int r_f0 = __builtin_amdgcn_readfirstlane(s_redo[3]);
    const int r_kv = __builtin_amdgcn_readfirstlane(s_redo[4]);
    wait_all_loads();
    __syncthreads();
    if (threadIdx.x == 0) s_redo[0] = 0;
    careful::run_item<D, CAUSAL>(a, r_start, r_len, r_f0, r_kv, k_ring);
    q_ahead = false;
  }
  // Everything derived from the lane number is recomputed in every round (the empty statement hides
  // the value from the optimiser): kept across rounds, dozens of such lane constants would sit in
  // registers through the hot loop, which has none to spare.
  int lane = lane_id;
  asm volatile("" : "+v"(lane));
  __builtin_assume(lane >= 0 && lane < 64);  // (divisions of lane-derived indices by constants become shifts)
  const int m = lane & 31, hf = lane >> 5, sl = lane & 15, grp = (lane >> 4) & 1;
  if constexpr (!Src::kPaged)
  if (__builtin_amdgcn_readfirstlane(s_claim[1]) == 0) {
    // Nothing left in this die's queue: take an item from another die's queue.  This is done here, with
    // the workgroup idle, and synchronously (two memory round trips), not ahead of time like the claims
    // from the own queue.  Every wave has seen the empty claim before wave 0 overwrites it.
    own_empty = true;
    __syncthreads();
    if (wave == 0) post_claim(steal_item(a.ctrl, xcc, (int)(blockIdx.x >> 3), lane_id, empty_mask));
    __syncthreads();
  }
  // The item: `seq_len` query rows that start at packed token `seq_start`, and `kv_len` keys; query row i sees
  // keys 0 .. shift + i (causal).  Packed batch: the keys are the sequence's own rows, shift = 0.
  int64_t seq_start;
  int seq_len, f0, kv_head;
  if constexpr (Src::kPaged) {
    seq_start = src.q_start;
    seq_len = src.q_len;
    f0 = src.f0;
    kv_head = src.kv_head;
  } else {
    seq_start = __builtin_amdgcn_readfirstlane(s_claim[0]);
    seq_len = __builtin_amdgcn_readfirstlane(s_claim[1]);
    f0 = __builtin_amdgcn_readfirstlane(s_claim[2]);
    kv_head = __builtin_amdgcn_readfirstlane(s_claim[3]);
    if (seq_len == 0) break;
  }
  int kv_len_, shift_;
  if constexpr (Src::kPaged) {
    kv_len_ = src.kv_len;
    shift_ = src.kv_len - src.q_len;
  } else {
    kv_len_ = seq_len;
    shift_ = 0;
  }
  const int kv_len = kv_len_, shift = shift_;
  // Thread 0: position claimed in this die's queue for the next round.  (Written as a per-thread
  // condition, and read below by every wave, on purpose: the compiler tracks outstanding memory
  // operations per code path, and an atomic that is "maybe still in flight" on some path into
  // the hot loop makes it wait for ALL loads there, which would undo the tile prefetch.)
  int pending_claim = 0x7fffffff;
  if constexpr (!Src::kPaged) {
    if (threadIdx.x == 0 && !own_empty) pending_claim = atomicAdd(&a.ctrl->queue_head[xcc * kHeadStride], 1);
  }
  const int n_tok_tiles = (seq_len + kWaveTileRows - 1) / kWaveTileRows;
  const int n_wave_tiles = n_tok_tiles * a.group;

  // this wave's tile
  int f = f0 + wave;
  const bool active = f < n_wave_tiles;
  if (!active) f = n_wave_tiles - 1;
  const int tok_tile = f / a.group;
  const int head = kv_head * a.group + (f - tok_tile * a.group);
  const int q0 = tok_tile * kWaveTileRows;
  const int f_last = (f0 + kWavesPerItem - 1 < n_wave_tiles ? f0 + kWavesPerItem - 1 : n_wave_tiles - 1);
  // KV tiles (of 64 keys) the workgroup streams
  const int n_kv_tiles = (kv_len + kKvTileRows - 1) / kKvTileRows;
  const int causal_keys = shift + (f_last / a.group + 1) * kWaveTileRows;  // keys visible to the item's last query tile
  const int W = CAUSAL && causal_keys < kv_len ? (causal_keys + kKvTileRows - 1) / kKvTileRows : n_kv_tiles;
  // key blocks this wave consumes: keys [0, kv_end)
  const int kv_end = CAUSAL ? (shift + q0 + kWaveTileRows < kv_len ? shift + q0 + kWaveTileRows : kv_len) : kv_len;
  const int NB = active ? (kv_end + kKeyBlock - 1) / kKeyBlock : 0;

  // Workgroup iterations: iteration 0 is the prologue (needs K(0)); iteration t >= 1 needs K tile t
  // and V tile t - 1 and runs, per wave, key-block steps 2t - 1 and 2t.  There are W + 1 of them.
  // Load order of the whole item: K(0) V(0) K(1) V(1) ..., each tile issued PD = 1 iteration ahead of
  // its use into the ring slot freed by the barrier that ended the previous iteration; everything
  // issued in iteration t is needed in iteration t + 1, so each iteration ends with a wait for all
  // of the wave's loads and a barrier.
  static_assert(PD == 1 && R == 2, "the iteration-end wait is for everything in flight");
  // The loaders of the two sources have different shapes: two independent tile loaders for the packed rows, one
  // gatherer for the pages (a V tile comes from the pages its K tile came from one iteration earlier).
  std::conditional_t<Src::kPaged, int, TileLoader<D>> k_loader, v_loader;
  typename Src::template Gather<D> gather;
  if constexpr (Src::kPaged) {
    gather.init(src, kv_head, wave, lane);
  } else {
    k_loader.template init<false>(a.k, a.k_stride, seq_start, seq_len, kv_head, wave, lane);
    v_loader.template init<true>(a.v, a.v_stride, seq_start, seq_len, kv_head, wave, lane);
  }
  // after the issue of iteration t, tile loads 0 .. 2(t+PD) are out; iteration t needs 0 .. 2t
  auto issue_loads = [&](int t) {
    if constexpr (Src::kPaged) {
      gather.issue(t - 1 + PD < W, v_ring + ((t - 1 + PD) % R) * G::kTileBytes, t + PD < W, k_ring + ((t + PD) % R) * G::kTileBytes);
    } else {
      if (t - 1 + PD < W) v_loader.issue_next(v_ring + ((t - 1 + PD) % R) * G::kTileBytes);
      if (t + PD < W) k_loader.issue_next(k_ring + ((t + PD) % R) * G::kTileBytes);
    }
  };
  if constexpr (Src::kPaged) gather.issue_first(k_ring); else k_loader.issue_next(k_ring);

  if (!q_ahead) issue_q_loads(seq_start, seq_len, q0, head, lane);
  // Q fragments (B operand): lane (m, hf) holds query row q0 + 32*qs + m, columns hf*D/2 + 8*s .. +7, as
  // they come from memory.  The softmax scale is applied to the scores in fp32 (see softmax_half).
  const float c = a.scale_log2;
  qreg_t qf[QS][KS];
  int q_lim[QS];  // largest visible key index for this lane's query of sub-tile qs
  wait_all_loads();  // Q (and this wave's part of K(0)) has landed
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) {
    int row = q0 + 32 * qs + m;
    row = row < seq_len ? row : seq_len - 1;
    q_lim[qs] = CAUSAL ? shift + row : kv_len - 1;
#pragma unroll
    for (int s = 0; s < KS; ++s)
      qf[qs][s] = *reinterpret_cast<const qreg_t*>(HYDRA_LDS_BYTE(q_stage + (32 * qs + m) * ROWB + k_swizzle<D>(32 * qs + m, KS * hf + s) * 16));
  }

  // LDS read addresses: lane part + ring slot of the iteration's K tile / V tile; the key block
  // inside the tile and the step are immediates.  Advanced once per iteration.
  uint32_t k_addr[KS], v_addr[CC];
  const uint32_t lds_base = k_ring;
#pragma unroll
  for (int s = 0; s < KS; ++s) k_addr[s] = lds_base + m * ROWB + k_swizzle<D>(m, KS * hf + s) * 16;  // K tile 0
  {
    const int r = 4 * hf + (sl >> 2);
#pragma unroll
    for (int cc = 0; cc < CC; ++cc) {
      const int chunk = 4 * cc + 2 * grp + ((sl & 3) >> 1);
      v_addr[cc] = lds_base + R * G::kTileBytes + r * ROWB + v_swizzle<D>(r, chunk) * 16 + 8 * (sl & 1);  // V ring, slot 0
    }
    if constexpr (G::kSumsFromMatrixUnit) {
      // columns 80..95 (the upper 16 of the last block): ones (the area is long enough for either ring slot)
      if (grp == 1) v_addr[CC - 1] = lds_base + G::kOnesAt;
    }
  }
  // The address registers point at slot 0 of both rings from here through the hot loop, whose reads name
  // their ring slot in the instruction offset (two iterations per trip: the slots are constants there).  The
  // iterations after the hot loop move the registers instead (position_addresses) and read at offset 0.
  int k_pos = 0, v_pos = 0;  // where the registers point: bytes from slot 0
  auto position_addresses = [&](int t) {  // to K tile t, V tile t - 1 (t >= 1)
    const int k_new = (t % R) * G::kTileBytes, v_new = ((t - 1) % R) * G::kTileBytes;
    const int dk = k_new - k_pos, dv = v_new - v_pos;
#pragma unroll
    for (int s = 0; s < KS; ++s) k_addr[s] += dk;
#pragma unroll
    for (int cc = 0; cc < CC; ++cc) v_addr[cc] += dv;
    k_pos = k_new;
    v_pos = v_new;
  };

  f32x16_t o_acc[QS][CC];
#pragma unroll
  for (int qs = 0; qs < QS; ++qs)
#pragma unroll
    for (int cc = 0; cc < CC; ++cc)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[qs][cc][r] = 0.f;
  // Softmax reference: the row maximum over key block 0, kept for the whole row, so O never has to be
  // rescaled inside the loop.  The matrix unit returns raw scores <q, k>; scale and reference go in with
  // one fused multiply-add per score, p = exp2(score * c - reference * c), c = softmax_scale * log2 e.
  // That is exact as long as the exponentials stay far from the end of the fp32
  // range: a wave whose row sums (which bound every single exponential) exceed kMaxRowSum, or are
  // not finite, posts its work item for the careful routine (attn_careful.hpp), which rescales at every tile
  // and which the workgroup runs at the top of its next round.  (bf16 activations lead the first block's maximum by a few
  // powers of two at most.  Below the limit the unnormalised output is bounded by 2^40 times the sum
  // of |V| over the keys, so it cannot overflow for |V| up to 10^20.)
  float nref[QS];        // -reference * c of this lane's query row
  float row_sum[QS];     // this lane's half of the row sum
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) row_sum[qs] = 0.f;

  // LDS fragment reads; rb = key block inside the tile the address registers point at.
  // (koff / voff: ring slot of the tile, in bytes; constants where it matters, so they end up in the instruction)
  auto load_k_frag = [&](int rb, int s, int koff) -> bf16x8_t {
    return *reinterpret_cast<const bf16x8_t*>(HYDRA_LDS_BYTE(k_addr[s] + koff + rb * kKeyBlock * ROWB));
  };
  // PV unit u = (s2, cc): the V^T fragment of 16 keys x 32 columns
  auto load_v_frag = [&](int rb, int u, int voff) -> bf16x8_t {
    const int cc = u % CC, s2 = u / CC;
    const uint32_t at = v_addr[cc] + voff + rb * kKeyBlock * ROWB + s2 * 16 * ROWB;
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_BYTE(at));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_BYTE(at + 8 * ROWB));
    typedef __attribute__((ext_vector_type(8))) short s16x8_t;
    const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, both);
  };

  // Mask of key block j (only blocks that reach past a query's limit need it).
  auto apply_mask = [&](int j, f32x16_t(&S)[QS]) {
    const int key0 = j * kKeyBlock;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = key0 + 8 * (r >> 2) + 4 * hf + (r & 3);
#pragma unroll
      for (int qs = 0; qs < QS; ++qs)
        if (key > q_lim[qs]) S[qs][r] = -__builtin_inff();
    }
  };
  const int min_lim = CAUSAL ? shift + q0 : kv_len - 1;
  auto needs_mask = [&](int j) { return j * kKeyBlock + kKeyBlock - 1 > min_lim; };

  // Softmax of a key block whose S holds the raw scores, in 16 * QS halves of an element pair (pair = half / 2:
  // sub-tile pair / 8, registers 2 * (pair % 8), +1): scale and reference, exponentials, row sum, rounding to
  // bf16.  A half is one exponential (a quarter-rate instruction) and two or three full-rate ones, about as long
  // as one matrix instruction takes, so that a wave alone on its SIMD can put one behind every matrix
  // instruction and keep the matrix pipe fed; whole pairs behind every other instruction left it idle a third
  // of the time.  The first half leaves its results in the two S registers.
  // (The sum is two plain adds on purpose: the 2-element dot-product instruction would halve them,
  // but it runs in the matrix pipe and stalls behind the matrix instructions it is meant to hide in.)
  auto softmax_half = [&](int half, f32x16_t(&Sc)[QS], bf16x8_t(&Pc)[QS][2], float(&psum)[QS]) __attribute__((always_inline)) {
    const int pair = half / 2, qs = pair / 8, r = 2 * (pair % 8);
    if (half % 2 == 0) {
      float e0 = fast_exp2(__builtin_fmaf(Sc[qs][r], c, nref[qs]));
      float x1 = __builtin_fmaf(Sc[qs][r + 1], c, nref[qs]);
      asm volatile("" : "+v"(e0), "+v"(x1));  // keeps this half's work where it is written
      Sc[qs][r] = e0;
      Sc[qs][r + 1] = x1;
    } else {
      float x1 = Sc[qs][r + 1];
      asm volatile("" : "+v"(x1));  // the second exponential stays behind the matrix instruction it is meant to follow
      f32x2_t pr = {Sc[qs][r], fast_exp2(x1)};
      if constexpr (!G::kSumsFromMatrixUnit) {
        psum[qs] += pr[0];
        psum[qs] += pr[1];
      }
      uint32_t packed = __builtin_bit_cast(uint32_t, __builtin_convertvector(pr, bf16x2_t));
      asm volatile("" : "+v"(packed), "+v"(psum[qs]));
      const bf16x2_t pk = __builtin_bit_cast(bf16x2_t, packed);
      Pc[qs][r / 8][r % 8] = pk[0];
      Pc[qs][r / 8][r % 8 + 1] = pk[1];
    }
  };

  // One pipeline step for key block j >= 1 of this wave.  KRB / VRB: key block of K(j+1) and of
  // V(j-1) inside the tiles the address registers point at.
  //   VALU : softmax of S(j) (in Sc) -> P(j) (into Pc)
  //   MFMA : O += V(j-1)^T P(j-1) (P in Pp) and S(j+1) = K(j+1) Q^T (into Sn)
  // One matrix instruction, then the share of vector work that fits in its shadow, and so on:
  // the wave issues in order, so this is what lets the two pipes run side by side.
  constexpr int NM = QS * (NQ + NP);  // matrix instructions per step
  constexpr int NV = 16 * QS;         // vector work pieces per step: the halves of 8 element pairs per sub-tile
  // qk_tag: false for a wave's last step, which has no S(j+1) to compute.
  // The LDS fragments of a step's first PF QK units and first PF PV units are fetched ahead of the
  // step (the LDS answers after several matrix instructions; fetched at the top of the step that
  // latency would be exposed once per step): `fr` holds them on entry.  next_tag >= 0: the step that
  // follows reads key block next_tag of the SAME tiles, and this step's last units fetch its first
  // fragments into `fr` (next_qk_tag: whether it has QK units).  next_tag < 0: nothing is fetched ahead
  // (the next tiles are only complete after the iteration's barrier; the caller fetches them then).
  auto block_step = [&](auto rb_tag, auto qk_tag, auto next_tag, auto next_qk_tag, int j, f32x16_t(&Sc)[QS], f32x16_t(&Sn)[QS],
                        const bf16x8_t(&Pp)[QS][2], bf16x8_t(&Pc)[QS][2], StepFrags<PF>& fr, int koff, int voff) __attribute__((always_inline)) {
    constexpr int RB = decltype(rb_tag)::value;  // step 2t-1: K(2t), V(2t-2) -> 0; step 2t: K(2t+1), V(2t-1) -> 1
    constexpr bool QK = decltype(qk_tag)::value;
    constexpr int NEXT_RB = decltype(next_tag)::value;
    constexpr bool NEXT_QK = decltype(next_qk_tag)::value;
    constexpr int NMS = QK ? NM : QS * NP;       // matrix instructions of this step
    if (needs_mask(j)) apply_mask(j, Sc);
    // vector work piece i of this step: half a softmax pair
    auto valu_piece = [&](int i) __attribute__((always_inline)) { softmax_half(i, Sc, Pc, row_sum); };
    // kq[i] / vq[i]: fragment of the QK / PV unit i places ahead of the one that runs next
    bf16x8_t kq[PF], vq[PF], k_new, v_new;
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      kq[i] = fr.k[i];
      vq[i] = fr.v[i];
    }
    int ms = 0;  // matrix-instruction index inside the step
    auto shadow = [&](int ms_done) __attribute__((always_inline)) {
      // vector pieces [ms*NV/NMS, (ms+1)*NV/NMS) run behind matrix instruction ms
#pragma unroll
      for (int i = ms_done * NV / NMS; i < (ms_done + 1) * NV / NMS; ++i) valu_piece(i);
      HYDRA_SCHED_FENCE();
    };
    // Order: QK unit 0, then alternately QK unit u and PV unit u - 1; the step ends with (at least)
    // two PV units, whose matrix instructions cover the wait states of the last QK result.
    static_assert(NP >= NQ && NP >= 2, "the step must end with two PV units");
    static_assert(NQ >= PF && NP >= PF, "a step's last units fetch the next step's first fragments");
#pragma unroll
    for (int u = 0; u <= NP; ++u) {
      if (QK && u < NQ) {
        const bool k_more = u + PF < NQ || (NEXT_RB >= 0 && NEXT_QK);
        if (u + PF < NQ) k_new = load_k_frag(RB, u + PF, koff);
        else if (NEXT_RB >= 0 && NEXT_QK) k_new = load_k_frag(NEXT_RB, u + PF - NQ, koff);
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
          if (u == 0) mfma_qk_zero(Sn[qs], kq[0], qf[qs][u]); else mfma_qk_acc(Sn[qs], kq[0], qf[qs][u]);
          shadow(ms++);
        }
#pragma unroll
        for (int i = 0; i + 1 < PF; ++i) kq[i] = kq[i + 1];
        if (k_more) kq[PF - 1] = k_new;
      }
      if (u >= 1) {
        const int pu = u - 1;
        const bool v_more = pu + PF < NP || NEXT_RB >= 0;
        if (pu + PF < NP) v_new = load_v_frag(RB, pu + PF, voff);
        else if (NEXT_RB >= 0) v_new = load_v_frag(NEXT_RB, pu + PF - NP, voff);
        const int cc = pu % CC, s2 = pu / CC;
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
          mfma_pv(o_acc[qs][cc], vq[0], Pp[qs][s2]);
          shadow(ms++);
        }
#pragma unroll
        for (int i = 0; i + 1 < PF; ++i) vq[i] = vq[i + 1];
        if (v_more) vq[PF - 1] = v_new;
      }
    }
    if constexpr (NEXT_RB >= 0) {
#pragma unroll
      for (int i = 0; i < PF; ++i) {
        fr.k[i] = kq[i];
        fr.v[i] = vq[i];
      }
    }
  };
  // first fragments of a step that reads key block rb of the tiles the address registers point at
  auto fetch_step_frags = [&](int rb, bool with_qk, StepFrags<PF>& fr, int koff, int voff) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      fr.v[i] = load_v_frag(rb, i, voff);
      if (with_qk) fr.k[i] = load_k_frag(rb, i, koff);
    }
  };

  // PV only (after this wave's last softmax): O += V^T P for key block rb of the V tile in reach
  auto pv_only = [&](int rb, const bf16x8_t(&Pp)[QS][2]) __attribute__((always_inline)) {
    // (all fragments are requested before the first matrix instruction: left to itself the compiler
    // fetches each one right before its use and the wave sits through the LDS latency NP times)
    bf16x8_t vf[NP];
#pragma unroll
    for (int u = 0; u < NP; ++u) vf[u] = load_v_frag(rb, u, 0);
    HYDRA_SCHED_FENCE();
#pragma unroll
    for (int u = 0; u < NP; ++u) {
#pragma unroll
      for (int qs = 0; qs < QS; ++qs) mfma_pv(o_acc[qs][u % CC], vf[u], Pp[qs][u / CC]);
    }
  };

  f32x16_t s_a[QS], s_b[QS];        // S of even / odd key blocks
  bf16x8_t p_a[QS][2], p_b[QS][2];  // P of even / odd key blocks
  using RB0 = std::integral_constant<int, 0>;
  using RB1 = std::integral_constant<int, 1>;
  using WithQK = std::integral_constant<bool, true>;
  using LastStep = std::integral_constant<bool, false>;

  __syncthreads();  // K(0) is complete; every wave has taken its Q out of the V ring
  // the rest of the prologue loads: V(0) K(1) V(1) ... K(PD)
  if constexpr (Src::kPaged) {
    gather.issue(0 < W, v_ring, 1 < W, k_ring + G::kTileBytes);
  } else {
#pragma unroll
    for (int n = 0; n < PD; ++n) {
      if (n < W) v_loader.issue_next(v_ring + n * G::kTileBytes);
      if (n + 1 < W) k_loader.issue_next(k_ring + (n + 1) * G::kTileBytes);
    }
  }

  // iteration 0: S(0) = K(0) Q^T alone, then S(1) = K(1) Q^T with the vector work of block 0 in its
  // shadow (reference = row maximum of block 0, softmax of block 0)
  if (NB > 0) {
    // (the K fragments of both blocks are requested ahead of the matrix instructions that use them,
    // with scheduling fences in between: see pv_only)
    bf16x8_t kf0[NQ], kf1[NQ];
#pragma unroll
    for (int s = 0; s < NQ; ++s) kf0[s] = load_k_frag(0, s, 0);
    HYDRA_SCHED_FENCE();
#pragma unroll
    for (int s = 0; s < NQ; ++s) {
#pragma unroll
      for (int qs = 0; qs < QS; ++qs) {
        if (s == 0) mfma_qk_zero(s_a[qs], kf0[s], qf[qs][s]); else mfma_qk_acc(s_a[qs], kf0[s], qf[qs][s]);
      }
    }
    HYDRA_SCHED_FENCE();
#pragma unroll
    for (int s = 0; s < NQ; ++s) kf1[s] = load_k_frag(1, s, 0);
    HYDRA_SCHED_FENCE();
    // (S(1) is computed even when NB == 1: harmless, never read.)  Its first two matrix instructions cover
    // the wait states of S(0); the vector work follows behind the others.
    static_assert(NQ * QS >= 4, "two matrix instructions ahead of the first read of S(0), at least two to hide the vector work behind");
    constexpr int kLead = 2;
    int mi = 0;
    auto block0_valu = [&](int piece, int pieces) __attribute__((always_inline)) {
      // piece 0: mask and row maximum; the 16 * QS softmax halves are spread over the others
      if (piece == 0) {
        if (needs_mask(0)) apply_mask(0, s_a);
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
          float t = fmaxf(s_a[qs][0], s_a[qs][1]);
#pragma unroll
          for (int r = 2; r < 16; ++r) t = fmaxf(t, s_a[qs][r]);
          t = max_with_other_half(t);
          nref[qs] = -t * c;
        }
      } else {
        const int n = 16 * QS, per = (n + pieces - 2) / (pieces - 1);
#pragma unroll
        for (int half = (piece - 1) * per; half < piece * per && half < n; ++half) softmax_half(half, s_a, p_a, row_sum);
      }
      HYDRA_SCHED_FENCE();
    };
    constexpr int kPieces = NQ * QS - kLead;
#pragma unroll
    for (int s = 0; s < NQ; ++s) {
#pragma unroll
      for (int qs = 0; qs < QS; ++qs) {
        if (s == 0) mfma_qk_zero(s_b[qs], kf1[s], qf[qs][s]); else mfma_qk_acc(s_b[qs], kf1[s], qf[qs][s]);
        HYDRA_SCHED_FENCE();
        if (mi >= kLead) block0_valu(mi - kLead, kPieces);
        ++mi;
      }
    }
    s_results_to_valu(s_b);
  }
  wait_all_loads();
  __syncthreads();
  const int pos = __builtin_amdgcn_readfirstlane(pending_claim);  // every wave: the claim has returned (see above)
  if constexpr (!Src::kPaged)
  if (wave == 0) {
    // (own queue empty: an empty claim is posted, and the top of the next round goes stealing)
    const int idx = pos < own_count ? own_begin + pos : -1;
    if (lane == 0) reset_head_if_last(a.ctrl, xcc, pos, own_count);
    // The item itself travels memory -> LDS on its own (one more direct-to-LDS load, lane 0 only):
    // it is complete when this wave's last wait of the round (for zero loads in flight) has
    // passed, and the barrier after that wait makes it visible to the other waves.  Every wave
    // has read this round's claim before the two barriers above, so the slot is free.
    if (lane == 0) {
      if (idx >= 0) {
        const uint64_t base = (uint64_t)(uintptr_t)a.items;
        u32x4_t rsrc;
        rsrc[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
        rsrc[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
        rsrc[2] = 0xffffffffu;
        rsrc[3] = 0x00020000u;
        const uint32_t off = (uint32_t)idx * (uint32_t)sizeof(WorkItem);
        const uint32_t m0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)HYDRA_LDS_PTR(&s_claim[0]));
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" : : "s"(m0), "v"(off), "s"(rsrc));
      } else {
        s_claim[0] = 0;
        s_claim[1] = 0;
        s_claim[2] = 0;
        s_claim[3] = 0;
      }
    }
  }

  // Per wave: steps 1 .. NB-1.  Iterations 1 .. F run two steps each (the hot loop), iteration
  // F + 1 runs the odd step left over (if any) and the last P V product, later iterations only
  // keep the workgroup's loads and barriers going.
  const int F = NB > 0 ? (NB - 1) / 2 : 0;
  // The wave's last step (block NB - 1) has no further scores to compute.  With an odd number of
  // steps it is the single step of iteration F + 1; with an even number it is the second step of
  // iteration F, which is therefore run apart from the loop.
  const bool odd_steps = ((NB - 1) & 1) != 0;
  const int F_loop = odd_steps ? F : (F > 0 ? F - 1 : 0);
  int t = 1;
  StepFrags<PF> fr;
  // Inside its pipeline steps a wave goes ahead of the SIMD's other wave when that one is between items
  // (Q scaling, epilogue: long runs of vector instructions that would otherwise take every other issue slot).
  __builtin_amdgcn_s_setprio(1);
  // Iteration t reads K tile t (ring slot t % 2) and V tile t - 1 (slot (t - 1) % 2); t is odd at the top of a trip.
  static_assert(R == 2, "two iterations per trip cover the ring");
  auto hot_iteration = [&](int tt, int koff, int voff) __attribute__((always_inline)) {
    fetch_step_frags(0, true, fr, koff, voff);
    HYDRA_SCHED_FENCE();
    issue_loads(tt);
    block_step(RB0{}, WithQK{}, NextRB<1>{}, WithQK{}, 2 * tt - 1, s_b, s_a, p_a, p_b, fr, koff, voff);
    block_step(RB1{}, WithQK{}, NextRB<-1>{}, WithQK{}, 2 * tt, s_a, s_b, p_b, p_a, fr, koff, voff);
    wait_all_loads();
    __syncthreads();
  };
  for (; t + 1 <= F_loop; t += 2) {
    hot_iteration(t, G::kTileBytes, 0);
    hot_iteration(t + 1, 0, G::kTileBytes);
  }
  if (t <= F_loop) {
    hot_iteration(t, G::kTileBytes, 0);
    ++t;
  }
  if (!odd_steps && F > 0) {
    position_addresses(t);
    fetch_step_frags(0, true, fr, 0, 0);
    HYDRA_SCHED_FENCE();
    issue_loads(t);
    block_step(RB0{}, WithQK{}, NextRB<1>{}, LastStep{}, 2 * t - 1, s_b, s_a, p_a, p_b, fr, 0, 0);
    block_step(RB1{}, LastStep{}, NextRB<-1>{}, LastStep{}, 2 * t, s_a, s_b, p_b, p_a, fr, 0, 0);
    wait_all_loads();
    __syncthreads();
    ++t;
  }
  if (NB > 0 && t <= W) {
    position_addresses(t);
    if (odd_steps) {
      fetch_step_frags(0, false, fr, 0, 0);
      HYDRA_SCHED_FENCE();
    }
    issue_loads(t);
    if (odd_steps) {
      block_step(RB0{}, LastStep{}, NextRB<-1>{}, LastStep{}, NB - 1, s_b, s_a, p_a, p_b, fr, 0, 0);  // NB - 1 = 2t - 1
      pv_only(1, p_b);                                            // V block NB - 1 = 2t - 1: second block of V tile t - 1
    } else {
      pv_only(0, p_a);  // V block NB - 1 = 2t - 2: first block of V tile t - 1
    }
    wait_all_loads();
    __syncthreads();
    ++t;
  }
  for (; t <= W; ++t) {
    issue_loads(t);
    wait_all_loads();
    __syncthreads();
  }
  __builtin_amdgcn_s_setprio(0);
  // a row sum out of the safe range somewhere in this wave's rows: have the item recomputed (top of the next round)
  if (NB > 0) {
    bool too_far = false;
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
      // (with the sums from the matrix unit: output column 80 + 4 hf of this lane's row)
      if constexpr (G::kSumsFromMatrixUnit) row_sum[qs] = o_acc[qs][CC - 1][8];
      too_far = too_far || !(row_sum[qs] <= kMaxRowSum);
    }
    if (__builtin_amdgcn_ballot_w64(too_far) != 0 && lane == 0) {
      s_redo[1] = (int)seq_start;
      s_redo[2] = seq_len;
      s_redo[3] = f0;
      s_redo[4] = kv_head;
      s_redo[0] = 1;
    }
  }
  // The next item (posted during this round; the last iteration's wait and barrier made it visible):
  // start its Q loads now.  (When the die's queue has run out the posted claim is empty, and the
  // item stolen at the top of the next round loads its Q there.)
  q_ahead = false;
  if constexpr (!Src::kPaged) {
    const int next_len = __builtin_amdgcn_readfirstlane(s_claim[1]);
    if (next_len != 0) {
      const int64_t next_start = __builtin_amdgcn_readfirstlane(s_claim[0]);
      const int next_f0 = __builtin_amdgcn_readfirstlane(s_claim[2]);
      const int next_kv = __builtin_amdgcn_readfirstlane(s_claim[3]);
      const int wave_tiles = ((next_len + kWaveTileRows - 1) / kWaveTileRows) * a.group;
      const int nf = next_f0 + wave < wave_tiles ? next_f0 + wave : wave_tiles - 1;
      const int tile = nf / a.group;
      issue_q_loads(next_start, next_len, tile * kWaveTileRows, next_kv * a.group + (nf - tile * a.group), lane);
      q_ahead = true;
    }
  }
  // ---- epilogue: normalise, round to bf16, transpose through LDS, store whole rows ----
  // In the accumulators a lane owns one query row and scattered groups of 4 columns; stored from
  // there, one store instruction would touch 32 different rows.  So each wave writes its 32 x D
  // tile to a private LDS staging area in K-tile layout and reads it back with one row per 16
  // (D = 128) lanes.  Staging area: the K ring, which is idle between an item's last iteration and the
  // next item's first load (issued after the barrier at the top of the next round).  The stores go
  // through a buffer descriptor that ends with the tile's last valid row (rows past it are dropped
  // by the hardware).
  static_assert(kWavesPerItem * kWaveTileRows * ROWB <= R * G::kTileBytes, "the output tiles of the four waves fit the K ring");
  if (active) {
    const uint32_t o_stage = k_ring + wave * (kWaveTileRows * ROWB);
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
      const float total = G::kSumsFromMatrixUnit ? row_sum[qs] : sum_with_other_half(row_sum[qs]);
      const float inv = 1.0f / total;
      const int r_own = 32 * qs + m;
#pragma unroll
      for (int cc = 0; cc < CC; ++cc)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int chunk = 4 * cc + g4;  // columns 32cc + 8*g4 .. +7; this lane has 4*hf .. 4*hf+3 of them
          if (chunk >= G::kChunks) continue;
          f32x2_t x0 = {o_acc[qs][cc][4 * g4] * inv, o_acc[qs][cc][4 * g4 + 1] * inv};
          f32x2_t x1 = {o_acc[qs][cc][4 * g4 + 2] * inv, o_acc[qs][cc][4 * g4 + 3] * inv};
          u32x2_t pk = {__builtin_bit_cast(uint32_t, __builtin_convertvector(x0, bf16x2_t)),
                        __builtin_bit_cast(uint32_t, __builtin_convertvector(x1, bf16x2_t))};
          *reinterpret_cast<u32x2_t*>(HYDRA_LDS_BYTE(o_stage + r_own * ROWB + k_swizzle<D>(r_own, chunk) * 16 + 8 * hf)) = pk;
        }
    }
    const uint64_t base = (uint64_t)(uintptr_t)(a.out + ((seq_start + q0) * a.n_q_heads + head) * D);
    const uint32_t out_row_bytes = (uint32_t)a.n_q_heads * (D * 2);
    const int rows = seq_len - q0 < kWaveTileRows ? seq_len - q0 : kWaveTileRows;
    u32x4_t rsrc;
    rsrc[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
    rsrc[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
    rsrc[2] = __builtin_amdgcn_readfirstlane((uint32_t)(rows - 1) * out_row_bytes + D * 2);
    rsrc[3] = 0x00020000u;
#pragma unroll
    for (int i = 0; i < kRowInstr; ++i) {
      const int flat = i * 64 + lane;
      const int r = flat / G::kChunks, chunk = flat % G::kChunks;
      const u32x4_t piece = *reinterpret_cast<const u32x4_t*>(HYDRA_LDS_BYTE(o_stage + r * ROWB + k_swizzle<D>(r, chunk) * 16));
      const uint32_t off = (uint32_t)r * out_row_bytes + chunk * 16;
      // (a store of more than 8 bytes reads its data registers a little after it issues; the wait
      // states keep the next instruction from overwriting them: the compiler does not see this store)
      // (nt: the output is not read again by this kernel)
      asm volatile("buffer_store_dwordx4 %0, %1, %2, 0 offen nt\n\ts_nop 1" : : "v"(piece), "v"(off), "s"(rsrc) : "memory");
    }
  }
  if constexpr (Src::kPaged) break;
  }  // next work item
  if constexpr (Src::kPaged) {
    __syncthreads();
    return s_redo[0] != 0;
  }
  return false;
}
#endif  // __HIP_DEVICE_COMPILE__

template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(kWorkgroupsPerCu<D>, kWorkgroupsPerCu<D>))) void attn_fwd_kernel(const AttnArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
  __shared__ __attribute__((aligned(1024))) unsigned char smem[TileGeom<D>::kLdsBytes];
  __shared__ __attribute__((aligned(16))) int s_claim[4];
  __shared__ __attribute__((aligned(16))) int s_redo[8];
  attn_item_loop<D, CAUSAL>(a, PackedSource{}, smem, s_claim, s_redo);
#else
  (void)a;
#endif
}

}  // namespace hydra
