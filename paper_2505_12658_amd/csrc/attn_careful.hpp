// The careful attention kernel: recomputes the work items the fast kernel flagged.
//
// The fast kernel (attn_fwd.hpp) takes every exponential of a row relative to the maximum of the
// row's first key block; a wave whose row sums relative to that reference leave the safe range (2^40) flags
// its item instead of overflowing.  This kernel redoes such items with the textbook online
// softmax (running maximum raised, and O rescaled, at every 64-key tile), which is exact for any
// finite input.  It is not software-pipelined; it exists for correctness, not for speed, and on
// ordinary activations it finds no flag set and returns at once.
//
// Same work decomposition, LDS swizzles and register layouts as the fast kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_fwd.hpp"

namespace hydra {
namespace careful {

template <int D>
struct StageGeom {
  static constexpr int kRowBytes = D * 2;
  static constexpr int kChunks = kRowBytes / 16;
  static constexpr int kQkSteps = D / 16;
  static constexpr int kPvChunks = (D + 31) / 32;
  static constexpr int kTileBytes = kKvTileRows * kRowBytes;  // one K or V tile
  static constexpr int kStageBytes = 2 * kTileBytes;          // K then V
  static constexpr int kLoadInstr = kTileBytes / 1024;
  static constexpr int kLdsBytes = 2 * kStageBytes + 64;      // two stages; slack: D=80 reads V columns 80..95
};

#if defined(__HIP_DEVICE_COMPILE__)
// Issue this wave's share of the direct-to-LDS loads of one 64-row K tile and V tile.
// Rows past the end of the sequence re-read the last valid row (always masked later).
template <int D>
__device__ __forceinline__ void issue_kv_tile_loads(const AttnArgs& a, unsigned char* stage, int wave, int lane, int64_t seq_start,
                                                    int seq_len, int kv_head, int kv0) {
  using G = StageGeom<D>;
  constexpr int kPerWave = (G::kLoadInstr + 3) / 4;
#pragma unroll
  for (int u = 0; u < kPerWave; ++u) {
    const int instr = wave + 4 * u;
    if (instr < G::kLoadInstr) {
      const int flat = instr * 64 + lane;
      const int row = flat / G::kChunks;
      const int phys = flat % G::kChunks;
      int tok = kv0 + row;
      tok = tok < seq_len ? tok : seq_len - 1;
      const int64_t t = seq_start + tok;
      const uint16_t* kp = a.k + t * a.k_stride + kv_head * D + k_swizzle<D>(row, phys) * 8;
      const uint16_t* vp = a.v + t * a.v_stride + kv_head * D + v_swizzle<D>(row, phys) * 8;
      __builtin_amdgcn_global_load_lds(HYDRA_GLOBAL_PTR(kp), HYDRA_LDS_PTR(stage + instr * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(HYDRA_GLOBAL_PTR(vp), HYDRA_LDS_PTR(stage + G::kTileBytes + instr * 1024), 16, 0, 0);
    }
  }
}

// One flagged work item, by one workgroup of 4 waves.
template <int D, bool CAUSAL>
__device__ __forceinline__ void run_item(const AttnArgs& a, const WorkItem item, unsigned char* smem) {
  using G = StageGeom<D>;
  constexpr int KS = G::kQkSteps;
  constexpr int CC = G::kPvChunks;
  constexpr int ROWB = G::kRowBytes;
  const int64_t seq_start = item.x;
  const int seq_len = item.y, f0 = item.z, kv_head = item.w;
  // The work item is cut the fast kernel's way: wave tiles of kWaveTileRows query rows, flattened
  // as token_tile * group + head_in_group.  This kernel works on tiles of 64 rows, so each wave
  // redoes the 64-row tile that CONTAINS its wave tile; where two waves (or two flagged items)
  // cover the same rows they store identical values.
  constexpr int kRows = 64;
  const int n_fast_tiles = (seq_len + kWaveTileRows - 1) / kWaveTileRows;
  const int n_wave_tiles = n_fast_tiles * a.group;
  const int n_tok_tiles = (seq_len + kRows - 1) / kRows;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 31, hf = lane >> 5, sl = lane & 15, grp = (lane >> 4) & 1;

  // this wave's tile
  int f = f0 + wave;
  const bool active = f < n_wave_tiles;
  if (!active) f = n_wave_tiles - 1;
  const int fast_tile = f / a.group;
  const int head = kv_head * a.group + (f - fast_tile * a.group);
  const int tok_tile = fast_tile * kWaveTileRows / kRows;
  const int q0 = tok_tile * kRows;
  const int f_last = (f0 + kWavesPerItem - 1 < n_wave_tiles ? f0 + kWavesPerItem - 1 : n_wave_tiles - 1);
  const int tiles_wg = CAUSAL ? (f_last / a.group) * kWaveTileRows / kRows + 1 : n_tok_tiles;
  const int tiles_wave = active ? (CAUSAL ? tok_tile + 1 : n_tok_tiles) : 0;

  // first K/V tile in flight before anything else
  issue_kv_tile_loads<D>(a, smem, wave, lane, seq_start, seq_len, kv_head, 0);

  // Q fragments (B operand): lane (m, hf) holds query row q0 + 32*qs + m, columns hf*D/2 + 8*s .. +7
  bf16x8_t qf[2][KS];
  int q_lim[2];  // largest visible key index for this lane's query of sub-tile qs
#pragma unroll
  for (int qs = 0; qs < 2; ++qs) {
    int row = q0 + 32 * qs + m;
    row = row < seq_len ? row : seq_len - 1;
    q_lim[qs] = CAUSAL ? row : seq_len - 1;
    const uint16_t* qp = a.q + (seq_start + row) * a.q_stride + head * D + hf * (D / 2);
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[qs][s] = *reinterpret_cast<const bf16x8_t*>(qp + 8 * s);
  }

  // LDS read offsets inside a stage
  uint32_t k_off[KS], v_off[CC];
#pragma unroll
  for (int s = 0; s < KS; ++s) k_off[s] = m * ROWB + k_swizzle<D>(m, KS * hf + s) * 16;
  {
    const int r = 4 * hf + (sl >> 2);
#pragma unroll
    for (int cc = 0; cc < CC; ++cc) {
      const int chunk = 4 * cc + 2 * grp + ((sl & 3) >> 1);
      v_off[cc] = G::kTileBytes + r * ROWB + v_swizzle<D>(r, chunk) * 16 + 8 * (sl & 1);
    }
  }

  f32x16_t o_acc[2][CC];
#pragma unroll
  for (int qs = 0; qs < 2; ++qs)
#pragma unroll
    for (int cc = 0; cc < CC; ++cc)
#pragma unroll
      for (int r = 0; r < 16; ++r) o_acc[qs][cc][r] = 0.f;
  float row_max[2] = {-3.0e38f, -3.0e38f};
  float row_sum[2] = {0.f, 0.f};
  const float c = a.scale_log2;

  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  for (int t = 0; t < tiles_wg; ++t) {
    unsigned char* stage = smem + (t & 1) * G::kStageBytes;
    if (t + 1 < tiles_wg)
      issue_kv_tile_loads<D>(a, smem + ((t + 1) & 1) * G::kStageBytes, wave, lane, seq_start, seq_len, kv_head, (t + 1) * kKvTileRows);

    if (t < tiles_wave) {
      const int kv0 = t * kKvTileRows;
      // ---- S^T = K Q^T ----
      f32x16_t s_acc[2][2];  // [rb][qs]
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
        for (int qs = 0; qs < 2; ++qs)
#pragma unroll
          for (int r = 0; r < 16; ++r) s_acc[rb][qs][r] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(stage + rb * 32 * ROWB + k_off[s]);
#pragma unroll
          for (int qs = 0; qs < 2; ++qs) s_acc[rb][qs] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qs][s], s_acc[rb][qs], 0, 0, 0);
        }
      }
      // ---- mask (diagonal and tail tiles only) ----
      const int min_lim = CAUSAL ? q0 : seq_len - 1;
      const bool need_mask = kv0 + kKvTileRows - 1 > min_lim;
      if (need_mask) {
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kv0 + 32 * rb + 8 * (r >> 2) + 4 * hf + (r & 3);
#pragma unroll
            for (int qs = 0; qs < 2; ++qs)
              if (key > q_lim[qs]) s_acc[rb][qs][r] = -__builtin_inff();
          }
      }
      // ---- online softmax, P in bf16 ----
      bf16x8_t p_frag[2][2][2];  // [qs][rb][s2]
#pragma unroll
      for (int qs = 0; qs < 2; ++qs) {
        float tmax = s_acc[0][qs][0];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s_acc[rb][qs][r]);
        tmax = max_with_other_half(tmax);
        const float m_new = fmaxf(row_max[qs], tmax);
        const float alpha = fast_exp2((row_max[qs] - m_new) * c);
        row_max[qs] = m_new;
        const float mc = m_new * c;
        float psum = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
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
      for (int cc = 0; cc < CC; ++cc)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            const unsigned char* vp = stage + v_off[cc] + (32 * rb + 16 * s2) * ROWB;
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_PTR(vp));
            const s16x4_t hi =
                __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_PTR(vp + 8 * ROWB));
            typedef __attribute__((ext_vector_type(8))) short s16x8_t;
            const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, both);
#pragma unroll
            for (int qs = 0; qs < 2; ++qs) o_acc[qs][cc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p_frag[qs][rb][s2], o_acc[qs][cc], 0, 0, 0);
          }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }

  if (!active) return;
  // ---- epilogue: normalise, round to bf16, store ----
#pragma unroll
  for (int qs = 0; qs < 2; ++qs) {
    const float total = sum_with_other_half(row_sum[qs]);
    const float inv = 1.0f / total;
    const int row = q0 + 32 * qs + m;
    if (row < seq_len) {
      uint16_t* op = a.out + ((seq_start + row) * a.n_q_heads + head) * D;
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
            *reinterpret_cast<u32x2_t*>(op + col) = pk;
          }
        }
    }
  }
}

#endif  // __HIP_DEVICE_COMPILE__

// Runs after the fast kernel on the same stream.  It first puts the fast kernel's queue heads back
// to zero for the next call.  When no item was flagged (the normal case) every workgroup reads one
// word and leaves.  Otherwise the workgroups grid-stride over the work list and redo the flagged
// items, clearing each flag they consume; the last workgroup to finish clears the summary word,
// so that everything is zero again for the next call.
template <int D, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_fwd_careful_kernel(const AttnArgs a) {
#if defined(__HIP_DEVICE_COMPILE__)
  __shared__ __attribute__((aligned(1024))) unsigned char smem[StageGeom<D>::kLdsBytes];
  if (blockIdx.x == 0 && threadIdx.x < kXcds) a.ctrl->queue_head[threadIdx.x * kHeadStride] = 0;
  if (__hip_atomic_load(&a.ctrl->redo_any, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) return;
  const int n_items = a.ctrl->n_items;
  for (int i = blockIdx.x; i < n_items; i += gridDim.x) {
    const int flagged = a.redo_flags[i];
    __syncthreads();
    if (flagged == 0) continue;
    if (threadIdx.x == 0) a.redo_flags[i] = 0;
    run_item<D, CAUSAL>(a, a.items[i], smem);
    __syncthreads();
  }
  // every workgroup has read the summary word before it counts itself done
  if (threadIdx.x == 0) {
    __threadfence();
    const int done = atomicAdd(&a.ctrl->careful_done, 1);
    if (done == (int)gridDim.x - 1) {
      a.ctrl->careful_done = 0;
      a.ctrl->redo_any = 0;
    }
  }
#else
  (void)a;
#endif
}

}  // namespace careful
}  // namespace hydra
