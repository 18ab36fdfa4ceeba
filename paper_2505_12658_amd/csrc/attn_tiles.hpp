// Types, geometry and LDS layout shared by the attention kernels (packed, careful, paged) for gfx950.
//
// All of them keep K and V tiles in LDS row-major with the same XOR swizzles of the 16-byte chunk index,
// read K fragments as the A operand of S^T = K Q^T with 128-bit reads and V^T fragments with the
// transposing 64-bit read, and hold a 32-query tile per wave; a change of layout lands here once.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hydra {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

#define HYDRA_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define HYDRA_LDS_BYTE(off) ((__attribute__((address_space(3))) unsigned char*)(uintptr_t)(off))
#define HYDRA_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

constexpr int kWaveTileRows = 32;  // query tokens per wave tile
constexpr int QS = kWaveTileRows / 32;  // 32-query sub-tiles per wave tile
constexpr int kKvTileRows = 64;    // keys per LDS tile
constexpr int kWavesPerItem = 4;   // wave tiles per work-list item

// Persistent workgroups of the packed attention kernel per compute unit (= waves per SIMD): as many as the
// register file holds.
template <int D>
constexpr int kWorkgroupsPerCu = D == 64 ? 3 : 2;

// One work-list entry, written by the device prepass from cu_seqlens; it carries everything the
// kernel needs, so a workgroup starts its loads after a single dependent read.
//   x = first packed token of the sequence, y = sequence length (0: empty entry past the end of
//   the list), z = first flattened wave tile of the item (flattened index f = token_tile * group
//   + head_in_group), w = KV head.
typedef int4 WorkItem;

constexpr int kXcds = 8;  // accelerator dies; workgroup ids are dealt to them round-robin, each die has its own L2

// Control block at the start of the workspace.  The work list is one array; the entries
// [xcd_start[x], xcd_start[x + 1]) form the queue of die x and queue_head[x] counts how many of
// them have been claimed in the current attention call.
// Every queue head has a 128-byte line of its own: the heads are the only words of the workspace
// that many workgroups update during the kernel, and claims of different dies must not collide.
constexpr int kHeadStride = 32;  // int32 words between queue heads
struct WorkControl {
  int32_t n_items;
  int32_t xcd_start[kXcds + 1];
  int32_t reserved[22];
  int32_t queue_head[kXcds * kHeadStride];  // head of queue x at [x * kHeadStride]; zero between calls
};
static_assert(sizeof(WorkControl) == 128 + kXcds * 128, "control block layout");

struct AttnArgs {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  uint16_t* out;
  int64_t q_stride, k_stride, v_stride;  // elements per token
  const int32_t* cu_seqlens;
  const WorkItem* items;
  WorkControl* ctrl;
  int32_t n_q_heads;
  int32_t group;     // n_q_heads / n_kv_heads
  float scale_log2;  // softmax_scale * log2(e)
};

// Row and tile sizes that follow from the head dimension alone.
template <int D>
struct RowGeom {
  static constexpr int kRowBytes = D * 2;
  static constexpr int kChunks = kRowBytes / 16;              // 16-byte pieces per row
  static constexpr int kQkSteps = D / 16;                     // 32x32x16 steps of the QK contraction
  static constexpr int kPvChunks = (D + 31) / 32;             // 32-wide output column blocks of PV
  static constexpr int kTileBytes = kKvTileRows * kRowBytes;  // one K or V tile of kKvTileRows keys
  static constexpr int kLoadInstr = kTileBytes / 1024;        // wave-wide 16 B/lane loads per tile
};

// XOR swizzles of the 16-byte chunk index inside an LDS row.  Chosen so that the 16 lanes the
// LDS serves together hit 16 different bank groups: for K, lanes read the same logical chunk of
// 16 consecutive rows; for V, a transposing read touches 4 consecutive rows x 64 bytes.
template <int D>
__device__ __forceinline__ int k_swizzle(int row, int chunk) {
  if constexpr (D == 128) return chunk ^ (row & 15);
  else if constexpr (D == 64) return chunk ^ ((row >> 1) & 7);
  else return chunk ^ ((row >> 3) & 1);
}
template <int D>
__device__ __forceinline__ int v_swizzle(int row, int chunk) {
  if constexpr (D == 128) return chunk ^ ((row & 3) << 2);
  else if constexpr (D == 64) return chunk ^ (((row >> 1) & 1) << 2);
  else return chunk;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Exchange between the two 32-lane halves with v_permlane32_swap, which swaps the upper half
// of its first register with the lower half of its second.  Starting from two copies of x:
//   r0 = x of the low-half lane of the pair (in both lanes), r1 = x of the high-half lane.
// Written as inline assembly so that both registers are explicit read-write operands; the
// s_nop padding covers the wait states between VALU writes/reads and the lane swap, which the
// compiler's hazard pass cannot see inside an asm block.
__device__ __forceinline__ void own_and_other_half(float x, float& r0, float& r1) {
  float a = x, b = x;
  asm volatile("s_nop 3\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 3" : "+v"(a), "+v"(b));
  r0 = a;
  r1 = b;
}
__device__ __forceinline__ float max_with_other_half(float x) {
  float r0, r1;
  own_and_other_half(x, r0, r1);
  return fmaxf(r0, r1);
}
__device__ __forceinline__ float sum_with_other_half(float x) {
  float r0, r1;
  own_and_other_half(x, r0, r1);
  return r0 + r1;
}

}  // namespace hydra
