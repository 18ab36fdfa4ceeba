/*
 * hydra_attn.h - C ABI of the packed variable-length attention library for MI355X (gfx950).
 *
 * The library implements the data-parallel computation that dominates the encode and prefill
 * stages of a multimodal LLM served with stage-level batching (HydraInfer, Section 4.2,
 * Algorithm 1): many images, or many requests, of different lengths are packed into one batch,
 * and every attention layer then runs
 *   - bidirectional attention inside each image (vision encoder, "encode" stage), or
 *   - causal attention inside each request over its image tokens followed by its text tokens
 *     (LLM "prefill" stage, Section 2.1: X = I || T, s = n + m), after which the request's K/V
 *     are kept in a paged KV cache (block size 16 in Section 5.1) for the decode stage.
 * The operation itself is scaled-dot-product attention as costed in the paper's Table 2 (rows
 * Attention/encode, Attention/prefill) and its appendix on computation and memory access:
 * multiply the query with the key, softmax, multiply with the value; 4*B*T^2*H FLOPs.
 *
 * Conventions common to all calls
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library never allocates,
 *     frees or keeps them.  Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and the call returns without synchronising with the device.
 *   - A call only launches kernels on `stream`: no memory is allocated, set or copied, and lengths,
 *     block tables and slot mappings are read on the device when the kernels run.  A call may therefore
 *     be recorded into a HIP graph; a replay acts on whatever the recorded buffers hold at that time.
 *   - bf16 means the upper 16 bits of an IEEE binary32 value.
 *   - Return value: a hydra_status.  Argument errors are detected on the host before anything
 *     is launched; nothing is written in that case.  The library neither prints nor aborts.
 *   - The calls are re-entrant; there is no global mutable state.  Results are bit-identical
 *     from run to run (no floating-point atomics; the order of the work list never affects the
 *     value of any output element).
 *   - Contents of device-side index arrays (cu_seqlens, slot_mapping) cannot be checked without
 *     a device synchronisation; violating their documented preconditions is undefined behaviour.
 */
#ifndef HYDRA_ATTN_H
#define HYDRA_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HYDRA_OK = 0,
  HYDRA_ERR_INVALID_ARG = 1, /* null pointer, negative size, misaligned pointer or stride, bad scale */
  HYDRA_ERR_UNSUPPORTED = 2, /* head_dim not in {64, 80, 128}, or a size beyond the stated limits    */
  HYDRA_ERR_WORKSPACE = 3,   /* workspace missing or smaller than hydra_attn_workspace_bytes()        */
  HYDRA_ERR_LAUNCH = 4       /* the HIP runtime refused a launch                                     */
} hydra_status;

/*
 * Packed variable-length attention, forward.
 *
 * For every sequence b with packed token range [cu_seqlens[b], cu_seqlens[b+1]) of length L, every
 * query head h (KV head h / (n_q_heads / n_kv_heads), i.e. consecutive query heads share a KV head)
 * and every local query index i:
 *     J(i) = {0..L-1} if causal == 0, {0..i} if causal != 0      (indices local to the sequence)
 *     z_j  = softmax_scale * <q[i,h,:], k[j,hk,:]>,  p = softmax over J(i),  out[i,h,:] = sum_j p_j v[j,hk,:]
 * Tokens of different sequences never interact.  Arithmetic: bf16 inputs, both contractions on the
 * bf16 matrix cores with fp32 accumulation, softmax in fp32, probabilities rounded to bf16 before
 * the second contraction, output rounded to bf16 (round to nearest even).
 *
 *   q    bf16 [total_tokens, n_q_heads,  head_dim]   token stride q_token_stride  (elements)
 *   k,v  bf16 [total_tokens, n_kv_heads, head_dim]   token strides k_/v_token_stride (elements)
 *        the head stride is head_dim and head_dim is contiguous, so q/k/v may be views into one
 *        fused QKV buffer.  Base pointers must be 16-byte aligned and strides multiples of 8.
 *   out  bf16 [total_tokens, n_q_heads, head_dim], contiguous, 16-byte aligned; every element of
 *        every token in [0, total_tokens) that belongs to a sequence is written.
 *   cu_seqlens  device int32 [batch + 1]; cu_seqlens[0] == 0, non-decreasing, cu_seqlens[batch] ==
 *        total_tokens, no sequence longer than max_seqlen.  Zero-length sequences are allowed.
 *   max_seqlen  upper bound on the sequence lengths (>= 1); only used to size and order the work.
 *   head_dim    64, 80 or 128.   n_q_heads % n_kv_heads == 0.
 *   softmax_scale  finite and >= 0 (normally 1/sqrt(head_dim)).
 *   workspace   device memory, 16-byte aligned, at least hydra_attn_workspace_bytes(...) bytes.  It
 *        receives the tile work list built on the device from cu_seqlens (entries of
 *        (sequence, KV head, first query tile), grouped into one queue per accelerator die) and
 *        a few counters.  It need not be initialised and may be reused by the next
 *        call on the same stream.
 *
 * batch == 0 or total_tokens == 0 returns HYDRA_OK without launching.
 */
int hydra_attn_varlen_fwd(const void* q, const void* k, const void* v, void* out,
                          int64_t q_token_stride, int64_t k_token_stride, int64_t v_token_stride,
                          const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                          int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                          int32_t causal, float softmax_scale,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two halves of hydra_attn_varlen_fwd, for callers that run many layers over one packed batch:
 * the work list depends only on cu_seqlens, the head counts and the causal flag, so it can be built
 * once per batch (the paper's Request Processor prepares such control parameters ahead of the GPU
 * work, Section 4.1) and reused by the attention call of every layer.
 *
 * hydra_attn_build_worklist writes the work list for (cu_seqlens, n_q_heads, n_kv_heads, causal)
 * into `workspace` (same size rule as above).  hydra_attn_varlen_fwd_prebuilt runs the attention
 * kernel against a workspace filled by an earlier hydra_attn_build_worklist call on the same stream
 * (or one that has completed) with the SAME batch, total_tokens, head counts and causal flag.  It
 * reads the work list and uses queue counters inside the workspace (all
 * left zero again when the call's work completes), so two attention calls that share one workspace
 * must not overlap in time.  Arguments, layouts and errors are those of hydra_attn_varlen_fwd.
 */
int hydra_attn_build_worklist(const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                              int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, int32_t causal,
                              void* workspace, size_t workspace_bytes, void* stream);

int hydra_attn_varlen_fwd_prebuilt(const void* q, const void* k, const void* v, void* out,
                                   int64_t q_token_stride, int64_t k_token_stride, int64_t v_token_stride,
                                   const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                                   int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                   int32_t causal, float softmax_scale,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * hydra_attn_varlen_fwd_prebuilt for an instance that runs its vision encoder and its language model
 * on two streams at once (Section 4.2, dual-stream parallelism; measured in Section 5.5).  The
 * attention kernel is made of persistent workgroups that by default take every compute unit's
 * registers whole, so a kernel launched beside it on another stream only gets the compute units
 * as they drain.  Here the caller says how many persistent
 * workgroups per compute unit the kernel may start:
 *
 *   workgroups_per_cu  >= 1 (otherwise HYDRA_ERR_INVALID_ARG); values above the kernel's own number
 *        (3 at head_dim 64, else 2) mean that number.  With 1, half (two thirds at head_dim 64) of every
 *        compute unit's registers and most of its LDS stay free for the other stream's kernels.
 *
 * Results are bit-identical to hydra_attn_varlen_fwd_prebuilt for every value (work items are
 * independent; only their placement changes).  Everything else as for hydra_attn_varlen_fwd_prebuilt.
 */
int hydra_attn_varlen_fwd_shared(const void* q, const void* k, const void* v, void* out,
                                 int64_t q_token_stride, int64_t k_token_stride, int64_t v_token_stride,
                                 const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                 int32_t causal, float softmax_scale,
                                 void* workspace, size_t workspace_bytes, int32_t workgroups_per_cu, void* stream);

/*
 * hydra_attn_varlen_fwd for callers that cannot allocate device memory or have none to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The work list,
 * counters live in an array of HYDRA_ATTN_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (every GPU the library runs on holds its own copy until the process ends);
 * the call allocates and frees nothing, and neither does anything it calls.
 *
 *   - Arguments, layouts, arithmetic and results (bit for bit) are those of hydra_attn_varlen_fwd
 *     without the workspace pair.
 *   - A batch whose hydra_attn_workspace_bytes(...) exceeds HYDRA_ATTN_STATIC_SCRATCH_BYTES is
 *     refused with HYDRA_ERR_WORKSPACE before anything is launched (4 MiB holds, for example,
 *     4096 sequences with 262 144 tokens at 32 query heads).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on one GPU (two
 *     streams, two threads) race on it.  Calls on one stream are ordered and safe; the array keeps
 *     the previous call's contents and every call rewrites all of what it reads.
 *   - The first call on a device looks the array's address up (a runtime query, not an allocation);
 *     make that first call outside a graph capture.
 */
#define HYDRA_ATTN_STATIC_SCRATCH_BYTES ((size_t)4 << 20)
int hydra_attn_varlen_fwd_static(const void* q, const void* k, const void* v, void* out,
                                 int64_t q_token_stride, int64_t k_token_stride, int64_t v_token_stride,
                                 const int32_t* cu_seqlens, int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                                 int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                                 int32_t causal, float softmax_scale, void* stream);

/*
 * Scatter of the prefill K/V of a packed batch into a paged KV cache (Section 5.1: KV-cache block
 * size 16; the per-request page tables of Section 4.3 are flattened by the caller into one slot per
 * token, slot = block_id * block_size + offset_in_block).
 *
 *   for t in [0, total_tokens): s = slot_mapping[t]; if s >= 0:
 *       k_cache[s / block_size, s % block_size, :, :] = k[t, :, :]     (bit copy), same for v.
 *
 *   k, v       bf16 [total_tokens, n_kv_heads, head_dim], token strides in elements (multiples of 8),
 *              16-byte aligned; may be views into a fused QKV buffer.
 *   k_cache, v_cache  bf16 [num_blocks, block_size, n_kv_heads, head_dim], contiguous, 16-byte aligned.
 *              Slots not named by slot_mapping keep their contents.
 *   slot_mapping  device int64 [total_tokens]; each value is < 0 (token skipped) or in
 *              [0, num_blocks * block_size) and no two tokens share a slot (otherwise undefined).
 *   n_kv_heads * head_dim must be a multiple of 8 (rows are moved in 16-byte pieces).
 *
 * total_tokens == 0 returns HYDRA_OK without launching.
 */
int hydra_kv_cache_write(const void* k, const void* v, int64_t k_token_stride, int64_t v_token_stride,
                         void* k_cache, void* v_cache, const int64_t* slot_mapping,
                         int32_t total_tokens, int32_t n_kv_heads, int32_t head_dim,
                         int32_t block_size, int64_t num_blocks, void* stream);

/*
 * Attention of a hybrid batch over the paged KV cache.
 *
 * The paper's batch scheduler (Algorithm 1) fills one batch, under a token budget, with the decode
 * requests (one new token each) and with chunks of prefill requests (get_chunked_size tokens each);
 * every one of them attends to its request's KV cache, which is paged (Section 4.5, block size 16 in
 * Section 5.1).  Request b brings q_len = cu_seqlens_q[b+1] - cu_seqlens_q[b] new tokens and has
 * kv_lens[b] tokens of context in the cache, the new tokens included (their K/V are written first,
 * with hydra_kv_cache_write).  For new token i, query head h (KV head hk as above):
 *     J(i) = {0 .. kv_len - q_len + i}        (causal mask aligned to the END of the context)
 *     key j lives at cache row  block_tables[b, j / block_size] * block_size + j % block_size
 *     z_j = softmax_scale * <q[i,h,:], K[j,hk,:]>,  p = softmax over J(i),  out[i,h,:] = sum_j p_j V[j,hk,:]
 * q_len == kv_len is an ordinary causal prefill, q_len == 1 a decode step.  Arithmetic as in
 * hydra_attn_varlen_fwd.
 *
 *   q    bf16 [total_q, n_q_heads, head_dim], token stride q_token_stride (elements, multiple of 8),
 *        16-byte aligned.
 *   out  bf16 [total_q, n_q_heads, head_dim], contiguous, 16-byte aligned.
 *   k_cache, v_cache  bf16 [num_blocks, block_size, n_kv_heads, head_dim], contiguous, 16-byte aligned.
 *   block_tables  device int32 [batch, max_blocks_per_seq], row-major; entry [b, n] is the cache block
 *        that holds keys n*block_size .. of request b.  Only the first ceil(kv_len / block_size)
 *        entries of a row are read.  Entries must lie in [0, num_blocks) (values outside are clamped
 *        into the cache, so a bad table gives wrong numbers, not a fault).
 *   cu_seqlens_q  device int32 [batch + 1], as cu_seqlens above, over the new tokens.
 *   kv_lens       device int32 [batch]; q_len <= kv_lens[b] <= max_blocks_per_seq * block_size.  A request
 *        with q_len == 0 (or, invalidly, kv_len < q_len) produces no output.
 *   max_q_len     upper bound on the q_len of the batch (>= 1); sizes the launch.
 *   block_size    a power of two, at least 1 (16 in the paper).   head_dim 64, 80 or 128.
 *   batch and n_kv_heads at most 65535; num_blocks * block_size below 2^31 (HYDRA_ERR_UNSUPPORTED otherwise).
 *   workspace   optional device memory (16-byte aligned; may be NULL with workspace_bytes 0).  With at least
 *        hydra_attn_paged_workspace_bytes(...) bytes, requests with few new tokens (decode steps) have their
 *        context split over several workgroups when the batch alone would not fill the chip or contexts are
 *        long; the partial results pass through the workspace and a second small kernel merges them.  With
 *        less, fewer splits (or none) are used; the result is the same up to rounding.  The workspace need
 *        not be initialised and may be reused by the next call on the same stream.
 *
 * batch == 0 or total_q == 0 returns HYDRA_OK without launching.
 */
int hydra_attn_paged_fwd(const void* q, void* out, int64_t q_token_stride,
                         const void* k_cache, const void* v_cache,
                         const int32_t* block_tables, int32_t max_blocks_per_seq,
                         const int32_t* cu_seqlens_q, const int32_t* kv_lens,
                         int32_t batch, int32_t total_q, int32_t max_q_len,
                         int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                         int32_t block_size, int64_t num_blocks,
                         float softmax_scale, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace with which hydra_attn_paged_fwd splits contexts as far as it would like to for these
 * sizes (0: it would not split, or the sizes are invalid).  Pure host arithmetic. */
size_t hydra_attn_paged_workspace_bytes(int32_t batch, int32_t n_kv_heads, int32_t head_dim,
                                        int32_t max_blocks_per_seq, int32_t block_size);

/*
 * Paged image cache: the vision encoder's output rows into cache pages, and back out of them.
 *
 * The encode stage's output tokens live in an image cache that is organised in fixed-size pages, the
 * same scheme as the KV cache (Section 4.5; image-cache block size 576 in Section 5.1); a request then
 * migrates to another instance by its page table, and an image seen before is served from its pages.  The caller flattens an
 * image's page table into one slot per row, slot = page_id * page_rows + row_in_page.
 *
 *   hydra_page_cache_write :  for t in [0, n_rows): s = slot_mapping[t]; if s >= 0: cache[s, :] = rows[t, :]
 *   hydra_page_cache_gather:  for t in [0, n_rows): s = slot_mapping[t]; if s >= 0: rows[t, :] = cache[s, :]
 *   (bit copies; rows with a negative slot are skipped; everything else keeps its contents)
 *
 *   rows   bf16 [n_rows, row_elems] with row stride row_stride (elements, multiple of 8, >= row_elems),
 *          16-byte aligned: the encoder output (write) or the buffer that receives the image tokens
 *          (gather), e.g. the image positions of the language model's input embeddings.
 *   cache  bf16 [num_slots, row_elems], contiguous, 16-byte aligned (num_slots = pages * page_rows).
 *   slot_mapping  device int64 [n_rows]; each value < 0 or in [0, num_slots); for the write no two rows
 *          share a slot (otherwise undefined).
 *   row_elems  a multiple of 8 (rows are moved in 16-byte pieces), at most 2^24.
 *
 * n_rows == 0 returns HYDRA_OK without launching.
 */
int hydra_page_cache_write(const void* rows, int64_t row_stride, void* cache, const int64_t* slot_mapping,
                           int32_t n_rows, int32_t row_elems, int64_t num_slots, void* stream);
int hydra_page_cache_gather(const void* cache, const int64_t* slot_mapping, void* rows, int64_t row_stride,
                            int32_t n_rows, int32_t row_elems, int64_t num_slots, void* stream);

/* Bytes of workspace hydra_attn_varlen_fwd needs for these sizes (0 if the sizes are invalid).
 * Depends only on batch, total_tokens and the head counts; pure host arithmetic. */
size_t hydra_attn_workspace_bytes(int32_t batch, int32_t total_tokens, int32_t max_seqlen,
                                  int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim);

/* Static, NUL-terminated description of a hydra_status value. */
const char* hydra_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* HYDRA_ATTN_H */
