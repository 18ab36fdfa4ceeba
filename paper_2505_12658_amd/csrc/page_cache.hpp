// Paged image cache: rows of the vision encoder's output -> cache pages, and back.
//
// The paper keeps the encoder's image tokens in an image cache that is paged like the KV cache
// (Section 4.5; image-cache block size
// 576 in Section 5.1), so that a request can migrate between instances and repeated images can be
// reused.  Both directions are pure data movement (HBM-bound): one thread per 16-byte piece of a
// row, 128-bit loads and stores, the lanes of a row consecutive on both sides.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hydra {

struct PageCacheArgs {
  const uint4* src;             // write: packed rows, gather: the cache
  uint4* dst;                   // write: the cache, gather: packed rows
  const int64_t* slot_mapping;  // one cache slot (page * page_rows + row in page) per packed row; < 0: row skipped
  int64_t packed_stride16;      // stride of the packed rows in 16-byte units
  int32_t n_rows;
  int32_t row16;                // 16-byte pieces per row
};

constexpr int kPageCacheThreads = 256;

// GATHER == false: cache[slot[t]] = packed[t];  GATHER == true: packed[t] = cache[slot[t]].
template <bool GATHER>
__global__ __launch_bounds__(kPageCacheThreads) void page_cache_kernel(const PageCacheArgs a) {
  const int64_t total = (int64_t)a.n_rows * a.row16;
  const int64_t step = (int64_t)gridDim.x * kPageCacheThreads;
  for (int64_t i = (int64_t)blockIdx.x * kPageCacheThreads + threadIdx.x; i < total; i += step) {
    const int32_t t = (int32_t)(i / a.row16);
    const int32_t piece = (int32_t)(i - (int64_t)t * a.row16);
    const int64_t slot = a.slot_mapping[t];
    if (slot < 0) continue;
    if (GATHER) a.dst[t * a.packed_stride16 + piece] = a.src[slot * a.row16 + piece];
    else a.dst[slot * a.row16 + piece] = a.src[t * a.packed_stride16 + piece];
  }
}

}  // namespace hydra
