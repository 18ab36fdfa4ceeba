// The careful attention routine: one work item recomputed with the textbook online softmax.
//
// The fast path (attn_fwd.hpp) takes every exponential of a row relative to the maximum of the
// row's first key block; a wave whose row sums relative to that reference leave the safe range (2^40)
// does not trust its result.  The workgroup then redoes the whole item here, inside the same kernel:
// running maximum raised, and O rescaled, at every 64-key tile, which is exact for any finite input.
// Not software-pipelined: it exists for correctness, not for speed, and on ordinary activations it
// never runs.
//
// Same work decomposition (a wave tile of 32 query rows per wave, four consecutive flattened wave tiles
// per item), LDS swizzles and register layouts as the fast path; the LDS is used as two stages of one
// K tile and one V tile each.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_tiles.hpp"

namespace hydra {
namespace careful {

template <int D>
struct StageGeom : RowGeom<D> {
  static constexpr int kStageBytes = 2 * RowGeom<D>::kTileBytes;  // K then V
  static constexpr int kLdsBytes = 2 * kStageBytes + 64;          // two stages; slack: D=80 reads V columns 80..95
};

#if defined(__HIP_DEVICE_COMPILE__)
// Issue this wave's share of the direct-to-LDS loads of one 64-row K tile and V tile.
// Rows past the end of the sequence re-read the last valid row (always masked later).
template <int D>
__device__ __forceinline__ void issue_kv_tile_loads(const AttnArgs& a, uint32_t stage, int wave, int lane, int64_t seq_start, int seq_len,
                                                    int kv_head, int kv0) {
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
      __builtin_amdgcn_global_load_lds(HYDRA_GLOBAL_PTR(kp), HYDRA_LDS_BYTE(stage + instr * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(HYDRA_GLOBAL_PTR(vp), HYDRA_LDS_BYTE(stage + G::kTileBytes + instr * 1024), 16, 0, 0);
    }
  }
}

// Waits until none of this wave's vector-memory operations is in flight (vmcnt(0); the other counters at
// their maximum).  Through the builtin, not inline assembly: the routine is inlined into the packed kernel,
// and the compiler, which knows that the loads above write LDS, must also know on every path out of here that
// none of them is still in flight, or it would make the LDS reads of the packed kernel's hot loop wait for them.
__device__ __forceinline__ void wait_for_tile_loads() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// One work item, by one workgroup of 4 waves.  `lds`: LDS byte address of StageGeom<D>::kLdsBytes bytes that
// nothing else uses meanwhile (no load into them in flight).  Called by all threads of the workgroup; ends
// with every wave's loads complete and a barrier.
template <int D, bool CAUSAL>
__device__ __forceinline__ void run_item(const AttnArgs& a, int64_t seq_start, int seq_len, int f0, int kv_head, uint32_t lds) {
  using G = StageGeom<D>;
  constexpr int KS = G::kQkSteps;
  constexpr int CC = G::kPvChunks;
  constexpr int ROWB = G::kRowBytes;
  constexpr int kRows = kWaveTileRows;
  const int n_tok_tiles = (seq_len + kRows - 1) / kRows;
  const int n_wave_tiles = n_tok_tiles * a.group;
  const int n_kv_tiles = (seq_len + kKvTileRows - 1) / kKvTileRows;

  // (The empty statement hides the lane number from the optimiser: the routine is inlined into a cold branch of
  // the packed kernel's item loop, and everything that depends only on the lane would otherwise be computed
  // ahead of that loop and kept, in registers the hot loop does not have, i.e. in scratch memory.)
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 31, hf = lane >> 5, sl = lane & 15, grp = (lane >> 4) & 1;

  // this wave's tile
  int f = f0 + wave;
  const bool active = f < n_wave_tiles;
  if (!active) f = n_wave_tiles - 1;
  const int tok_tile = f / a.group;
  const int head = kv_head * a.group + (f - tok_tile * a.group);
  const int q0 = tok_tile * kRows;
  const int f_last = (f0 + kWavesPerItem - 1 < n_wave_tiles ? f0 + kWavesPerItem - 1 : n_wave_tiles - 1);
  // K/V tiles the workgroup streams, and those this wave uses (keys below q0 + 32 under the causal mask)
  const int tiles_wg = CAUSAL ? ((f_last / a.group + 1) * kRows + kKvTileRows - 1) / kKvTileRows : n_kv_tiles;
  const int tiles_wave = active ? (CAUSAL ? (q0 + kRows + kKvTileRows - 1) / kKvTileRows : n_kv_tiles) : 0;

  // first K/V tile in flight before anything else
  issue_kv_tile_loads<D>(a, lds, wave, lane, seq_start, seq_len, kv_head, 0);

  // Q fragments (B operand): lane (m, hf) holds query row q0 + m, columns hf*D/2 + 8*s .. +7
  bf16x8_t qf[KS];
  int row = q0 + m;
  row = row < seq_len ? row : seq_len - 1;
  const int q_lim = CAUSAL ? row : seq_len - 1;  // largest visible key index for this lane's query
  {
    const uint16_t* qp = a.q + (seq_start + row) * a.q_stride + head * D + hf * (D / 2);
#pragma unroll
    for (int s = 0; s < KS; ++s) qf[s] = *reinterpret_cast<const bf16x8_t*>(qp + 8 * s);
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

  f32x16_t o_acc[CC];
#pragma unroll
  for (int cc = 0; cc < CC; ++cc)
#pragma unroll
    for (int r = 0; r < 16; ++r) o_acc[cc][r] = 0.f;
  float row_max = -3.0e38f, row_sum = 0.f;
  const float c = a.scale_log2;

  wait_for_tile_loads();
  __syncthreads();

  for (int t = 0; t < tiles_wg; ++t) {
    const uint32_t stage = lds + (t & 1) * G::kStageBytes;
    if (t + 1 < tiles_wg)
      issue_kv_tile_loads<D>(a, lds + ((t + 1) & 1) * G::kStageBytes, wave, lane, seq_start, seq_len, kv_head, (t + 1) * kKvTileRows);

    if (t < tiles_wave) {
      const int kv0 = t * kKvTileRows;
      // ---- S^T = K Q^T ----
      f32x16_t s_acc[2];  // [rb]: the two 32-key blocks of the tile
#pragma unroll
      for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) s_acc[rb][r] = 0.f;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
          const bf16x8_t kf = *reinterpret_cast<const bf16x8_t*>(HYDRA_LDS_BYTE(stage + rb * 32 * ROWB + k_off[s]));
          s_acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s_acc[rb], 0, 0, 0);
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
            if (key > q_lim) s_acc[rb][r] = -__builtin_inff();
          }
      }
      // ---- online softmax, P in bf16 ----
      bf16x8_t p_frag[2][2];  // [rb][s2]
      {
        float tmax = s_acc[0][0];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s_acc[rb][r]);
        tmax = max_with_other_half(tmax);
        const float m_new = fmaxf(row_max, tmax);
        const float alpha = fast_exp2((row_max - m_new) * c);
        row_max = m_new;
        const float mc = m_new * c;
        float psum = 0.f;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
          float p[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) p[r] = fast_exp2(__builtin_fmaf(s_acc[rb][r], c, -mc));
          if (need_mask) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int key = kv0 + 32 * rb + 8 * (r >> 2) + 4 * hf + (r & 3);
              if (key > q_lim) p[r] = 0.f;
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
              p_frag[rb][s2][e] = pb[0];
              p_frag[rb][s2][e + 1] = pb[1];
            }
        }
        row_sum = row_sum * alpha + psum;
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
#pragma unroll
          for (int r = 0; r < 16; ++r) o_acc[cc][r] *= alpha;
      }
      // ---- O^T += V^T P^T ----
#pragma unroll
      for (int cc = 0; cc < CC; ++cc)
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int s2 = 0; s2 < 2; ++s2) {
            const uint32_t vp = stage + v_off[cc] + (32 * rb + 16 * s2) * ROWB;
            const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_BYTE(vp));
            const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)HYDRA_LDS_BYTE(vp + 8 * ROWB));
            typedef __attribute__((ext_vector_type(8))) short s16x8_t;
            const s16x8_t both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            const bf16x8_t vf = __builtin_bit_cast(bf16x8_t, both);
            o_acc[cc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p_frag[rb][s2], o_acc[cc], 0, 0, 0);
          }
    }
    wait_for_tile_loads();
    __syncthreads();
  }

  // ---- epilogue: normalise, round to bf16, store ----
  if (active && q0 + m < seq_len) {
    const float total = sum_with_other_half(row_sum);
    const float inv = 1.0f / total;
    uint16_t* op = a.out + ((seq_start + q0 + m) * a.n_q_heads + head) * D;
#pragma unroll
    for (int cc = 0; cc < CC; ++cc)
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        const int col = 32 * cc + 8 * g4 + 4 * hf;
        if (col < D) {
          f32x2_t a0 = {o_acc[cc][4 * g4] * inv, o_acc[cc][4 * g4 + 1] * inv};
          f32x2_t a1 = {o_acc[cc][4 * g4 + 2] * inv, o_acc[cc][4 * g4 + 3] * inv};
          const bf16x2_t b0 = __builtin_convertvector(a0, bf16x2_t);
          const bf16x2_t b1 = __builtin_convertvector(a1, bf16x2_t);
          u32x2_t pk = {__builtin_bit_cast(uint32_t, b0), __builtin_bit_cast(uint32_t, b1)};
          *reinterpret_cast<u32x2_t*>(op + col) = pk;
        }
      }
  }
}

#endif  // __HIP_DEVICE_COMPILE__

}  // namespace careful
}  // namespace hydra
