// C ABI of the library: argument validation on the host, then launches.  See include/hydra_attn.h
// for the contract of every entry point.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <atomic>
#include <tuple>

#include "../../include/hydra_attn.h"
#include "attn_fwd.hpp"
#include "attn_paged.hpp"
#include "kv_write.hpp"
#include "page_cache.hpp"
#include "worklist.hpp"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool head_dim_supported(int d) { return d == 64 || d == 80 || d == 128; }

// Enqueues one kernel and returns the status of THIS launch (the runtime's sticky last-error slot
// is shared by every caller of the process and may hold somebody else's failure).
template <typename... Params, typename... Args>
hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, const Args&... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "one argument per kernel parameter");
  std::tuple<Params...> vals(args...);
  return std::apply(
      [&](auto&... v) {
        void* ptrs[] = {static_cast<void*>(&v)...};
        return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, stream);
      },
      vals);
}

// Compute units of the current device (0 if the runtime cannot tell).  Looked up on every call:
// the library keeps no state, and the attribute query does not touch the device.
unsigned compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 0;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 0;
  return (unsigned)n;
}

// One launch: the persistent workgroups drain the work list (an item whose exponentials leave the
// fast path's range is redone on the spot, by the same workgroup, with the careful routine).
template <int D>
hipError_t launch_attn(bool causal, const hydra::AttnArgs& args, unsigned compute_units, int workgroups_per_cu, hipStream_t stream) {
  // two or three persistent workgroups per compute unit (each takes its share of registers and LDS):
  // while one is loading Q, storing O or between key blocks, the others' matrix work fills the SIMDs.
  // A caller that runs another kernel beside this one asks for fewer (workgroups_per_cu > 0); any number
  // of workgroups drains the queues.
  const unsigned per_cu = workgroups_per_cu > 0 && workgroups_per_cu < hydra::kWorkgroupsPerCu<D> ? (unsigned)workgroups_per_cu
                                                                                                  : (unsigned)hydra::kWorkgroupsPerCu<D>;
  const unsigned grid = per_cu * compute_units;
  return causal ? launch(hydra::attn_fwd_kernel<D, true>, dim3(grid), dim3(256), stream, args)
                : launch(hydra::attn_fwd_kernel<D, false>, dim3(grid), dim3(256), stream, args);
}

// Bytes of one partial result of the paged kernel's packed-rows form.
size_t paged_partial_bytes(int head_dim) { return (size_t)(2 * hydra::paged::kRows + hydra::paged::kRows * head_dim) * sizeof(float); }

// Workgroups per (request, KV head) over which the packed-rows form of the paged kernel splits a context.
// A function of the launch sizes alone (both the workspace-size query and the launch use it): as many as
// fit the chip's 512 workgroup slots together (a batch that already brings 256 (request, KV head) pairs or
// more is not split: measured, the extra workgroups and the merge then cost more than the imbalance they
// remove), at least 512 keys per share of the longest context the block table can describe, at most 16, and
// no more than the workspace holds.
int paged_splits(int32_t batch, int32_t n_kv_heads, int32_t head_dim, int32_t max_blocks_per_seq, int32_t block_size, size_t workspace_bytes) {
  const int64_t pairs = (int64_t)batch * n_kv_heads;
  int64_t want = 512 / pairs;
  const int64_t by_length = ((int64_t)max_blocks_per_seq * block_size) / 512;
  if (want > by_length) want = by_length;
  if (want > hydra::paged::kMaxSplits) want = hydra::paged::kMaxSplits;
  const int64_t fits = (int64_t)(workspace_bytes / (paged_partial_bytes(head_dim) * (size_t)pairs));
  if (want > fits) want = fits;
  return want < 2 ? 1 : (int)want;
}

}  // namespace

extern "C" {

size_t hydra_attn_workspace_bytes(int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t n_q_heads, int32_t n_kv_heads,
                                  int32_t head_dim) {
  if (batch < 0 || total_tokens < 0 || max_seqlen < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0 ||
      !head_dim_supported(head_dim))
    return 0;
  return hydra::workspace_layout(batch, total_tokens, n_q_heads, n_kv_heads).total;
}

const char* hydra_status_string(int status) {
  switch (status) {
    case HYDRA_OK: return "ok";
    case HYDRA_ERR_INVALID_ARG: return "invalid argument";
    case HYDRA_ERR_UNSUPPORTED: return "unsupported configuration";
    case HYDRA_ERR_WORKSPACE: return "workspace missing or too small";
    case HYDRA_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
  }
}

namespace {

// Argument checks shared by the three attention entry points.  `need_tensors` is false for the
// work-list builder, which touches only cu_seqlens and the workspace.
int check_attn_sizes(int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim) {
  if (batch < 0 || total_tokens < 0 || n_q_heads <= 0 || n_kv_heads <= 0) return HYDRA_ERR_INVALID_ARG;
  if (n_q_heads % n_kv_heads != 0) return HYDRA_ERR_INVALID_ARG;
  if (!head_dim_supported(head_dim)) return HYDRA_ERR_UNSUPPORTED;
  if (batch > 0 && total_tokens > 0 && max_seqlen < 1) return HYDRA_ERR_INVALID_ARG;
  // 32-bit byte offsets inside one sequence's K/V rows (buffer addressing in the attention kernel)
  // are checked by the callers that know the strides; 32-bit index arithmetic inside the prepass:
  if ((int64_t)n_q_heads * ((int64_t)total_tokens / hydra::kWaveTileRows + batch) > (int64_t)1 << 30) return HYDRA_ERR_UNSUPPORTED;
  return HYDRA_OK;
}

int check_workspace(const void* workspace, size_t workspace_bytes, const hydra::WorkspaceLayout& lay) {
  if (!workspace || workspace_bytes < lay.total || !aligned16(workspace)) return HYDRA_ERR_WORKSPACE;
  return HYDRA_OK;
}

}  // namespace

int hydra_attn_build_worklist(const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen, int32_t n_q_heads,
                              int32_t n_kv_heads, int32_t head_dim, int32_t causal, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (int rc = check_attn_sizes(batch, total_tokens, max_seqlen, n_q_heads, n_kv_heads, head_dim)) return rc;
  if (batch == 0 || total_tokens == 0) return HYDRA_OK;
  if (!cu_seqlens) return HYDRA_ERR_INVALID_ARG;
  const hydra::WorkspaceLayout lay = hydra::workspace_layout(batch, total_tokens, n_q_heads, n_kv_heads);
  if (int rc = check_workspace(workspace, workspace_bytes, lay)) return rc;

  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  hydra::WorkControl* ctrl = reinterpret_cast<hydra::WorkControl*>(ws);
  int32_t* sorted_seq = reinterpret_cast<int32_t*>(ws + lay.sorted_at);
  int32_t* queue_prefix = reinterpret_cast<int32_t*>(ws + lay.prefix_at);
  hydra::WorkItem* items = reinterpret_cast<hydra::WorkItem*>(ws + lay.items_at);
  const int group = n_q_heads / n_kv_heads;
  const int tail_items = hydra::tail_sort_items(group, head_dim);
  const dim3 grid(hydra::prepass_workgroups(lay.capacity)), block(hydra::kPrepassThreads);
  const hipError_t err =
      causal ? launch(hydra::build_worklist_kernel<true>, grid, block, s, cu_seqlens, batch, n_kv_heads, group, ctrl, sorted_seq, queue_prefix,
                      (int)lay.rows, items, (int)lay.capacity, tail_items)
             : launch(hydra::build_worklist_kernel<false>, grid, block, s, cu_seqlens, batch, n_kv_heads, group, ctrl, sorted_seq, queue_prefix,
                      (int)lay.rows, items, (int)lay.capacity, tail_items);
  return err == hipSuccess ? HYDRA_OK : HYDRA_ERR_LAUNCH;
}

namespace {

// Every host-side check of an attention call (sizes, pointers, strides, 32-bit addressing limits, the
// workspace, the device), shared by the entry points so that each of them has finished checking
// before its first launch.  *done is set when the call has nothing to do; *cus receives the number of
// compute units.
int validate_attn_call(const void* q, const void* k, const void* v, const void* out, int64_t q_token_stride, int64_t k_token_stride,
                       int64_t v_token_stride, const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                       int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale, const void* workspace,
                       size_t workspace_bytes, bool* done, unsigned* cus) {
  *done = false;
  if (int rc = check_attn_sizes(batch, total_tokens, max_seqlen, n_q_heads, n_kv_heads, head_dim)) return rc;
  if (!(softmax_scale >= 0.0f) || isinf(softmax_scale)) return HYDRA_ERR_INVALID_ARG;
  if (batch == 0 || total_tokens == 0) {
    *done = true;
    return HYDRA_OK;
  }
  if (!q || !k || !v || !out || !cu_seqlens) return HYDRA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return HYDRA_ERR_INVALID_ARG;
  if (q_token_stride < (int64_t)n_q_heads * head_dim || k_token_stride < (int64_t)n_kv_heads * head_dim ||
      v_token_stride < (int64_t)n_kv_heads * head_dim)
    return HYDRA_ERR_INVALID_ARG;
  if ((q_token_stride | k_token_stride | v_token_stride) & 7) return HYDRA_ERR_INVALID_ARG;
  {
    // the kernel addresses one sequence's K (or V) rows with 32-bit byte offsets
    const int64_t widest = k_token_stride > v_token_stride ? k_token_stride : v_token_stride;
    if (((int64_t)max_seqlen + 2 * hydra::kKvTileRows) * widest * 2 >= ((int64_t)1 << 31)) return HYDRA_ERR_UNSUPPORTED;
  }
  if (int rc = check_workspace(workspace, workspace_bytes, hydra::workspace_layout(batch, total_tokens, n_q_heads, n_kv_heads))) return rc;
  *cus = compute_units();
  if (*cus == 0) return HYDRA_ERR_LAUNCH;
  return HYDRA_OK;
}

// The attention launch against a prebuilt work list; workgroups_per_cu == 0: the kernel's own number.
int attn_prebuilt(const void* q, const void* k, const void* v, void* out, int64_t q_token_stride, int64_t k_token_stride,
                  int64_t v_token_stride, const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                  int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t causal, float softmax_scale, void* workspace,
                  size_t workspace_bytes, int32_t workgroups_per_cu, void* stream) {
  bool done = false;
  unsigned grid = 0;
  if (int rc = validate_attn_call(q, k, v, out, q_token_stride, k_token_stride, v_token_stride, cu_seqlens, batch, total_tokens, max_seqlen,
                                  n_q_heads, n_kv_heads, head_dim, softmax_scale, workspace, workspace_bytes, &done, &grid))
    return rc;
  if (done) return HYDRA_OK;
  const hydra::WorkspaceLayout lay = hydra::workspace_layout(batch, total_tokens, n_q_heads, n_kv_heads);

  unsigned char* ws = static_cast<unsigned char*>(workspace);
  hydra::AttnArgs args;
  args.q = static_cast<const uint16_t*>(q);
  args.k = static_cast<const uint16_t*>(k);
  args.v = static_cast<const uint16_t*>(v);
  args.out = static_cast<uint16_t*>(out);
  args.q_stride = q_token_stride;
  args.k_stride = k_token_stride;
  args.v_stride = v_token_stride;
  args.cu_seqlens = cu_seqlens;
  args.items = reinterpret_cast<const hydra::WorkItem*>(ws + lay.items_at);
  args.ctrl = reinterpret_cast<hydra::WorkControl*>(ws);
  args.n_q_heads = n_q_heads;
  args.group = n_q_heads / n_kv_heads;
  // A scale of exactly 0 is replaced by a vanishing positive one: every visible key still gets
  // weight exp2(~0) = 1, while -inf (masked) times the scale stays -inf instead of becoming NaN.
  const float scale_log2 = softmax_scale * 1.44269504088896340736f;
  args.scale_log2 = scale_log2 > 1e-30f ? scale_log2 : 1e-30f;

  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t err;
  switch (head_dim) {
    case 64: err = launch_attn<64>(causal != 0, args, grid, workgroups_per_cu, s); break;
    case 80: err = launch_attn<80>(causal != 0, args, grid, workgroups_per_cu, s); break;
    default: err = launch_attn<128>(causal != 0, args, grid, workgroups_per_cu, s); break;
  }
  return err == hipSuccess ? HYDRA_OK : HYDRA_ERR_LAUNCH;
}

}  // namespace

int hydra_attn_varlen_fwd_prebuilt(const void* q, const void* k, const void* v, void* out, int64_t q_token_stride,
                                   int64_t k_token_stride, int64_t v_token_stride, const int32_t* cu_seqlens, int32_t batch,
                                   int32_t total_tokens, int32_t max_seqlen, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                   int32_t causal, float softmax_scale, void* workspace, size_t workspace_bytes, void* stream) {
  return attn_prebuilt(q, k, v, out, q_token_stride, k_token_stride, v_token_stride, cu_seqlens, batch, total_tokens, max_seqlen,
                       n_q_heads, n_kv_heads, head_dim, causal, softmax_scale, workspace, workspace_bytes, 0, stream);
}

int hydra_attn_varlen_fwd_shared(const void* q, const void* k, const void* v, void* out, int64_t q_token_stride,
                                 int64_t k_token_stride, int64_t v_token_stride, const int32_t* cu_seqlens, int32_t batch,
                                 int32_t total_tokens, int32_t max_seqlen, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                 int32_t causal, float softmax_scale, void* workspace, size_t workspace_bytes,
                                 int32_t workgroups_per_cu, void* stream) {
  if (workgroups_per_cu < 1) return HYDRA_ERR_INVALID_ARG;
  return attn_prebuilt(q, k, v, out, q_token_stride, k_token_stride, v_token_stride, cu_seqlens, batch, total_tokens, max_seqlen,
                       n_q_heads, n_kv_heads, head_dim, causal, softmax_scale, workspace, workspace_bytes, workgroups_per_cu, stream);
}

int hydra_attn_varlen_fwd(const void* q, const void* k, const void* v, void* out, int64_t q_token_stride, int64_t k_token_stride,
                          int64_t v_token_stride, const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                          int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t causal, float softmax_scale, void* workspace,
                          size_t workspace_bytes, void* stream) {
  // every check of both halves runs before the first launch, so that an error never leaves half the work enqueued
  bool done = false;
  unsigned cus = 0;
  if (int rc = validate_attn_call(q, k, v, out, q_token_stride, k_token_stride, v_token_stride, cu_seqlens, batch, total_tokens, max_seqlen,
                                  n_q_heads, n_kv_heads, head_dim, softmax_scale, workspace, workspace_bytes, &done, &cus))
    return rc;
  if (done) return HYDRA_OK;

  if (int rc = hydra_attn_build_worklist(cu_seqlens, batch, total_tokens, max_seqlen, n_q_heads, n_kv_heads, head_dim, causal, workspace,
                                         workspace_bytes, stream))
    return rc;
  return hydra_attn_varlen_fwd_prebuilt(q, k, v, out, q_token_stride, k_token_stride, v_token_stride, cu_seqlens, batch, total_tokens,
                                        max_seqlen, n_q_heads, n_kv_heads, head_dim, causal, softmax_scale, workspace, workspace_bytes,
                                        stream);
}

}  // extern "C"

namespace {

// Work-list memory of hydra_attn_varlen_fwd_static: one array per device, living in the code
// object's data segment, so that a caller that may not allocate needs no workspace of its own.
constexpr size_t kStaticScratchBytes = HYDRA_ATTN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device.  In host code the array's name is only a
// handle for the runtime, so the address is asked for once per device (with that device current)
// and kept; every use below goes through this pointer.
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int static_scratch(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HYDRA_ERR_LAUNCH;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HYDRA_ERR_LAUNCH;
    g_scratch_ptr[dev].store(p, std::memory_order_release);  // (two first callers get the same address)
  }
  *ptr = p;
  return HYDRA_OK;
}

}  // namespace

extern "C" {

int hydra_attn_varlen_fwd_static(const void* q, const void* k, const void* v, void* out, int64_t q_token_stride, int64_t k_token_stride,
                                 int64_t v_token_stride, const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens,
                                 int32_t max_seqlen, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t causal,
                                 float softmax_scale, void* stream) {
  // sizes first: the work list of this call has to fit the static array
  if (int rc = check_attn_sizes(batch, total_tokens, max_seqlen, n_q_heads, n_kv_heads, head_dim)) return rc;
  if (batch == 0 || total_tokens == 0)  // nothing to launch; the remaining argument checks are the plain call's
    return hydra_attn_varlen_fwd(q, k, v, out, q_token_stride, k_token_stride, v_token_stride, cu_seqlens, batch, total_tokens, max_seqlen,
                                 n_q_heads, n_kv_heads, head_dim, causal, softmax_scale, nullptr, 0, stream);
  if (hydra::workspace_layout(batch, total_tokens, n_q_heads, n_kv_heads).total > kStaticScratchBytes) return HYDRA_ERR_WORKSPACE;
  void* ws = nullptr;
  if (int rc = static_scratch(&ws)) return rc;
  // The prepass rewrites every word of the work list, the counters and the flags that the attention
  // kernels read, so whatever the previous call left in the array does not matter.
  return hydra_attn_varlen_fwd(q, k, v, out, q_token_stride, k_token_stride, v_token_stride, cu_seqlens, batch, total_tokens, max_seqlen,
                               n_q_heads, n_kv_heads, head_dim, causal, softmax_scale, ws, kStaticScratchBytes, stream);
}

int hydra_attn_paged_fwd(const void* q, void* out, int64_t q_token_stride, const void* k_cache, const void* v_cache,
                         const int32_t* block_tables, int32_t max_blocks_per_seq, const int32_t* cu_seqlens_q, const int32_t* kv_lens,
                         int32_t batch, int32_t total_q, int32_t max_q_len, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                         int32_t block_size, int64_t num_blocks, float softmax_scale, void* workspace, size_t workspace_bytes,
                         void* stream) {
  if (batch < 0 || total_q < 0 || n_q_heads <= 0 || n_kv_heads <= 0 || n_q_heads % n_kv_heads != 0) return HYDRA_ERR_INVALID_ARG;
  if (!head_dim_supported(head_dim)) return HYDRA_ERR_UNSUPPORTED;
  if (block_size < 1 || (block_size & (block_size - 1)) != 0) return HYDRA_ERR_UNSUPPORTED;
  if (!(softmax_scale >= 0.0f) || isinf(softmax_scale)) return HYDRA_ERR_INVALID_ARG;
  if (batch == 0 || total_q == 0) return HYDRA_OK;
  if (max_q_len < 1 || max_blocks_per_seq < 1 || num_blocks < 1) return HYDRA_ERR_INVALID_ARG;
  if (!q || !out || !k_cache || !v_cache || !block_tables || !cu_seqlens_q || !kv_lens) return HYDRA_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(out) || !aligned16(k_cache) || !aligned16(v_cache)) return HYDRA_ERR_INVALID_ARG;
  if (q_token_stride < (int64_t)n_q_heads * head_dim || (q_token_stride & 7)) return HYDRA_ERR_INVALID_ARG;
  if (batch > 65535 || n_kv_heads > 65535 || num_blocks * block_size > (int64_t)0x7fffffff) return HYDRA_ERR_UNSUPPORTED;
  if ((int64_t)max_blocks_per_seq * block_size > (int64_t)1 << 30) return HYDRA_ERR_UNSUPPORTED;
  if (workspace_bytes > 0 && (!workspace || !aligned16(workspace))) return HYDRA_ERR_WORKSPACE;

  hydra::paged::PagedArgs args;
  args.q = static_cast<const uint16_t*>(q);
  args.out = static_cast<uint16_t*>(out);
  args.q_stride = q_token_stride;
  args.k_cache = static_cast<const uint16_t*>(k_cache);
  args.v_cache = static_cast<const uint16_t*>(v_cache);
  args.block_tables = block_tables;
  args.cu_seqlens_q = cu_seqlens_q;
  args.kv_lens = kv_lens;
  args.max_blocks_per_seq = max_blocks_per_seq;
  args.num_blocks = (int32_t)num_blocks;
  int shift = 0;
  while ((1 << shift) < block_size) ++shift;
  args.block_shift = shift;
  args.n_q_heads = n_q_heads;
  args.n_kv_heads = n_kv_heads;
  args.group = n_q_heads / n_kv_heads;
  const float scale_log2 = softmax_scale * 1.44269504088896340736f;
  args.scale_log2 = scale_log2 > 1e-30f ? scale_log2 : 1e-30f;  // (see hydra_attn_varlen_fwd_prebuilt)

  const int64_t tok_tiles = ((int64_t)max_q_len + hydra::paged::kRows - 1) / hydra::paged::kRows;
  int64_t groups = (tok_tiles * args.group + hydra::paged::kWavesPerGroup - 1) / hydra::paged::kWavesPerGroup;
  if ((int64_t)max_q_len * args.group <= hydra::paged::kRows) groups = 0;  // every request takes the packed-rows form
  const int splits = paged_splits(batch, n_kv_heads, head_dim, max_blocks_per_seq, block_size, workspace_bytes);
  args.n_splits = splits;
  {
    const int64_t max_halves = ((int64_t)max_blocks_per_seq * block_size + 31) / 32;
    args.halves_per_split = (int32_t)((max_halves + splits - 1) / splits);
  }
  args.partials = static_cast<float*>(workspace);
  args.batch = batch;
  // Workgroups of the wave-tile form: one per group of four wave tiles and KV head.  The request lengths are
  // on the device, so this is an upper bound from the total: a request of q new tokens has at most
  // (q / 32 + 1) * group / 4 + 1 groups.
  int64_t tile_wgs = 0;
  if (groups > 0) tile_wgs = (((int64_t)total_q / hydra::paged::kRows + batch) * args.group / hydra::paged::kWavesPerGroup + batch) * n_kv_heads;
  const int64_t rows_wgs = (int64_t)batch * n_kv_heads * splits;
  if (tile_wgs + rows_wgs > (int64_t)0x7fffffff) return HYDRA_ERR_UNSUPPORTED;
  args.n_tile_wgs = (int32_t)tile_wgs;
  const dim3 grid((unsigned)(tile_wgs + rows_wgs), 1, 1);
  const dim3 combine_grid((unsigned)n_kv_heads, (unsigned)batch);
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t err;
  switch (head_dim) {
    case 64:
      err = launch(hydra::paged::attn_paged_kernel<64>, grid, dim3(256), s, args);
      if (err == hipSuccess && splits > 1) err = launch(hydra::paged::attn_paged_combine_kernel<64>, combine_grid, dim3(256), s, args);
      break;
    case 80:
      err = launch(hydra::paged::attn_paged_kernel<80>, grid, dim3(256), s, args);
      if (err == hipSuccess && splits > 1) err = launch(hydra::paged::attn_paged_combine_kernel<80>, combine_grid, dim3(256), s, args);
      break;
    default:
      err = launch(hydra::paged::attn_paged_kernel<128>, grid, dim3(256), s, args);
      if (err == hipSuccess && splits > 1) err = launch(hydra::paged::attn_paged_combine_kernel<128>, combine_grid, dim3(256), s, args);
      break;
  }
  return err == hipSuccess ? HYDRA_OK : HYDRA_ERR_LAUNCH;
}

size_t hydra_attn_paged_workspace_bytes(int32_t batch, int32_t n_kv_heads, int32_t head_dim, int32_t max_blocks_per_seq, int32_t block_size) {
  if (batch <= 0 || n_kv_heads <= 0 || !head_dim_supported(head_dim) || max_blocks_per_seq < 1 || block_size < 1) return 0;
  const int splits = paged_splits(batch, n_kv_heads, head_dim, max_blocks_per_seq, block_size, ~(size_t)0);
  return splits > 1 ? paged_partial_bytes(head_dim) * (size_t)splits * (size_t)batch * (size_t)n_kv_heads : 0;
}

int hydra_kv_cache_write(const void* k, const void* v, int64_t k_token_stride, int64_t v_token_stride, void* k_cache, void* v_cache,
                         const int64_t* slot_mapping, int32_t total_tokens, int32_t n_kv_heads, int32_t head_dim, int32_t block_size,
                         int64_t num_blocks, void* stream) {
  if (total_tokens < 0 || n_kv_heads <= 0 || head_dim <= 0 || block_size <= 0 || num_blocks < 0) return HYDRA_ERR_INVALID_ARG;
  const int64_t row = (int64_t)n_kv_heads * head_dim;
  if (row % 8 != 0) return HYDRA_ERR_UNSUPPORTED;
  if (row > ((int64_t)1 << 24)) return HYDRA_ERR_UNSUPPORTED;
  if (total_tokens == 0) return HYDRA_OK;
  if (!k || !v || !k_cache || !v_cache || !slot_mapping) return HYDRA_ERR_INVALID_ARG;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_cache) || !aligned16(v_cache)) return HYDRA_ERR_INVALID_ARG;
  if (k_token_stride < row || v_token_stride < row || ((k_token_stride | v_token_stride) & 7)) return HYDRA_ERR_INVALID_ARG;

  hydra::KvWriteArgs args;
  args.k = static_cast<const uint4*>(k);
  args.v = static_cast<const uint4*>(v);
  args.k_cache = static_cast<uint4*>(k_cache);
  args.v_cache = static_cast<uint4*>(v_cache);
  args.slot_mapping = slot_mapping;
  args.k_stride16 = k_token_stride / 8;
  args.v_stride16 = v_token_stride / 8;
  args.total_tokens = total_tokens;
  args.row16 = (int32_t)(row / 8);

  const int64_t pieces = (int64_t)total_tokens * args.row16;
  int64_t blocks = (pieces + hydra::kKvWriteThreads - 1) / hydra::kKvWriteThreads;
  const int64_t max_blocks = 256 * 32;  // grid-stride beyond this
  if (blocks > max_blocks) blocks = max_blocks;
  const hipError_t err = launch(hydra::kv_cache_write_kernel, dim3((unsigned)blocks), dim3(hydra::kKvWriteThreads), static_cast<hipStream_t>(stream), args);
  return err == hipSuccess ? HYDRA_OK : HYDRA_ERR_LAUNCH;
}

namespace {

// Shared by the two image-cache calls: `packed` is the caller's row-major buffer (source of the write,
// destination of the gather).
int launch_page_cache(bool gather, const void* packed, int64_t packed_row_stride, const void* cache, const int64_t* slot_mapping,
                      int32_t n_rows, int32_t row_elems, int64_t num_slots, void* stream) {
  if (n_rows < 0 || row_elems <= 0 || num_slots < 0) return HYDRA_ERR_INVALID_ARG;
  if (row_elems % 8 != 0 || row_elems > (1 << 24)) return HYDRA_ERR_UNSUPPORTED;
  if (n_rows == 0) return HYDRA_OK;
  if (!packed || !cache || !slot_mapping) return HYDRA_ERR_INVALID_ARG;
  if (!aligned16(packed) || !aligned16(cache)) return HYDRA_ERR_INVALID_ARG;
  if (packed_row_stride < row_elems || (packed_row_stride & 7)) return HYDRA_ERR_INVALID_ARG;
  hydra::PageCacheArgs args;
  args.slot_mapping = slot_mapping;
  args.packed_stride16 = packed_row_stride / 8;
  args.n_rows = n_rows;
  args.row16 = row_elems / 8;
  const int64_t pieces = (int64_t)n_rows * args.row16;
  int64_t blocks = (pieces + hydra::kPageCacheThreads - 1) / hydra::kPageCacheThreads;
  const int64_t max_blocks = 256 * 32;  // grid-stride beyond this
  if (blocks > max_blocks) blocks = max_blocks;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t err;
  if (gather) {
    args.src = static_cast<const uint4*>(cache);
    args.dst = static_cast<uint4*>(const_cast<void*>(packed));
    err = launch(hydra::page_cache_kernel<true>, dim3((unsigned)blocks), dim3(hydra::kPageCacheThreads), s, args);
  } else {
    args.src = static_cast<const uint4*>(packed);
    args.dst = static_cast<uint4*>(const_cast<void*>(cache));
    err = launch(hydra::page_cache_kernel<false>, dim3((unsigned)blocks), dim3(hydra::kPageCacheThreads), s, args);
  }
  return err == hipSuccess ? HYDRA_OK : HYDRA_ERR_LAUNCH;
}

}  // namespace

int hydra_page_cache_write(const void* rows, int64_t row_stride, void* cache, const int64_t* slot_mapping, int32_t n_rows, int32_t row_elems,
                           int64_t num_slots, void* stream) {
  return launch_page_cache(false, rows, row_stride, cache, slot_mapping, n_rows, row_elems, num_slots, stream);
}

int hydra_page_cache_gather(const void* cache, const int64_t* slot_mapping, void* rows, int64_t row_stride, int32_t n_rows, int32_t row_elems,
                            int64_t num_slots, void* stream) {
  return launch_page_cache(true, rows, row_stride, cache, slot_mapping, n_rows, row_elems, num_slots, stream);
}

}  // extern "C"
