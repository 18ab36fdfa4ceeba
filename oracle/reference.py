"""Plain NumPy fp64 oracle (test infrastructure only; never on the product path).

Definition followed: scaled-dot-product attention, i.e. the fused operation the paper's cost
model describes as "multiply the query with the key, then multiply the value" with the softmax
in between (Appendix "Computation and Memory Access in MLLMs", attention equations; Table 2,
rows Attention/encode and Attention/prefill).  Encode attends bidirectionally inside each image;
prefill attends causally inside each request (Section 2.1: the prefill input X of a request is
its own image tokens followed by its own text tokens, s = n + m).  Requests packed into one
batch by stage-level batching never attend to each other.

Readings taken where the paper is silent (each also listed in the design notes):
  * softmax scale is an explicit argument; causal means key j visible to query i iff j <= i,
    both indices local to the sequence (prefix cache off in the paper's evaluation, so the
    query length equals the key length);
  * grouped-query attention maps query head h to KV head h // (Hq // Hkv);
  * packed layout is token-major [N, heads, d] with int32 cu_seqlens of length B + 1;
  * a zero-length sequence is legal and contributes nothing;
  * paged KV cache is [num_blocks, block_size, Hkv, d] per K and per V (block size 16 in the
    paper's Section 5.1 setup), slot = block * block_size + offset, slot < 0 skips the token;
  * attention over the paged cache (decode steps and prefill chunks batched by Algorithm 1): the
    new tokens are the last positions of the request's context and the mask is causal.

Nothing here is tiled, fused or reordered: per (sequence, head) one dense score matrix, one
explicit boolean mask, one softmax, one matmul.  np.matmul / np.exp are the library steps.
"""
from __future__ import annotations

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16/int16 array) to float64."""
    u = np.ascontiguousarray(bits).view(np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def visibility_mask(L: int, causal: bool) -> np.ndarray:
    """Explicit L x L boolean matrix: entry [i, j] says whether query i may see key j."""
    if causal:
        i = np.arange(L)[:, None]
        j = np.arange(L)[None, :]
        return j <= i
    return np.ones((L, L), dtype=bool)


def masked_softmax(z: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Row-wise softmax of z with masked entries treated as -inf (probability exactly 0)."""
    zm = np.where(mask, z, -np.inf)
    zmax = zm.max(axis=-1, keepdims=True)
    e = np.where(mask, np.exp(zm - zmax), 0.0)
    return e / e.sum(axis=-1, keepdims=True)


def attention_probs(q: np.ndarray, k: np.ndarray, scale: float, causal: bool) -> np.ndarray:
    """Softmax probabilities for ONE sequence and ONE head.  q, k: [L, d] float64 -> [L, L]."""
    L = q.shape[0]
    z = scale * (q @ k.T)
    return masked_softmax(z, visibility_mask(L, causal))


def attn_varlen(q, k, v, cu_seqlens, causal: bool, scale: float) -> np.ndarray:
    """Packed variable-length attention.

    q: [N, Hq, d], k, v: [N, Hkv, d] float64 (already widened from the bf16 inputs);
    cu_seqlens: int array [B + 1].  Returns float64 [N, Hq, d] (not rounded).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    N, Hq, d = q.shape
    Hkv = k.shape[1]
    if Hq % Hkv != 0:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    if cu[0] != 0 or cu[-1] != N or np.any(np.diff(cu) < 0):
        raise ValueError("cu_seqlens must start at 0, be non-decreasing and end at total_tokens")
    g = Hq // Hkv
    out = np.zeros((N, Hq, d), dtype=np.float64)
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        L = e - s
        if L == 0:
            continue
        mask = visibility_mask(L, causal)
        assert mask.any(axis=1).all(), "every query sees at least one key"
        for h in range(Hq):
            hk = h // g
            z = scale * (q[s:e, h, :] @ k[s:e, hk, :].T)
            p = masked_softmax(z, mask)
            out[s:e, h, :] = p @ v[s:e, hk, :]
    return out


def attn_rows(q, k, v, cu_seqlens, causal: bool, scale: float, rows) -> np.ndarray:
    """Selected output rows only: rows is an iterable of (packed token index, query head).

    Used at full benchmark sizes, where the whole batch is too slow to compute.  Each row is
    evaluated from the same definition (its own mask row, softmax, weighted sum).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    Hq, d = q.shape[1], q.shape[2]
    g = Hq // k.shape[1]
    rows = list(rows)
    out = np.zeros((len(rows), d), dtype=np.float64)
    for r, (t, h) in enumerate(rows):
        b = int(np.searchsorted(cu, t, side="right") - 1)
        s, e = int(cu[b]), int(cu[b + 1])
        i = t - s
        hk = h // g
        mask_row = visibility_mask(e - s, causal)[i] if (e - s) <= 512 else (
            (np.arange(e - s) <= i) if causal else np.ones(e - s, dtype=bool))
        z = scale * (k[s:e, hk, :] @ q[t, h, :])
        p = masked_softmax(z[None, :], mask_row[None, :])[0]
        out[r] = p @ v[s:e, hk, :]
    return out


def end_aligned_mask(q_len: int, kv_len: int) -> np.ndarray:
    """Explicit q_len x kv_len boolean matrix for new tokens that sit at the END of a context of
    kv_len tokens: new token i is context position kv_len - q_len + i and sees every key up to
    and including itself."""
    i = np.arange(q_len)[:, None]
    j = np.arange(kv_len)[None, :]
    return j <= (kv_len - q_len) + i


def attn_paged(q, k_cache, v_cache, block_tables, cu_seqlens_q, kv_lens, scale: float) -> np.ndarray:
    """Attention of a hybrid batch over the paged KV cache.

    What is computed: the batch that the paper's Algorithm 1 assembles holds decode requests (one
    new token) and chunks of prefill requests (get_chunked_size new tokens); each attends to its
    own KV cache, kept in pages (Section 4.5: paged attention; block size 16 in Section 5.1).  Request
    b has q_len = cu_seqlens_q[b+1] - cu_seqlens_q[b] new tokens and kv_lens[b] tokens of context
    in the cache, the new ones included.  Reading taken (the paper does not spell the mask out):
    the new tokens are the LAST q_len positions of the context and attention is causal, so new
    token i sees keys 0 .. kv_len - q_len + i.  Key j of request b is cache row
    (block_tables[b, j // block_size], j % block_size).

    q: [Nq, Hq, d]; caches: [num_blocks, block_size, Hkv, d]; all float64.  Returns [Nq, Hq, d].
    Per request the context is first gathered from its pages into a dense [kv_len, Hkv, d] array;
    then one score matrix, one explicit mask, one softmax, one matmul per head.
    """
    q = np.asarray(q, dtype=np.float64)
    kc = np.asarray(k_cache, dtype=np.float64)
    vc = np.asarray(v_cache, dtype=np.float64)
    tables = np.asarray(block_tables, dtype=np.int64)
    cu = np.asarray(cu_seqlens_q, dtype=np.int64)
    kv_lens = np.asarray(kv_lens, dtype=np.int64)
    Nq, Hq, d = q.shape
    num_blocks, bs, Hkv, _ = kc.shape
    if Hq % Hkv != 0:
        raise ValueError("n_q_heads must be a multiple of n_kv_heads")
    if cu[0] != 0 or cu[-1] != Nq or np.any(np.diff(cu) < 0) or len(kv_lens) != len(cu) - 1:
        raise ValueError("cu_seqlens_q must start at 0, be non-decreasing and end at the number of new tokens")
    g = Hq // Hkv
    out = np.zeros((Nq, Hq, d), dtype=np.float64)
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        Lq, Lk = e - s, int(kv_lens[b])
        if Lq == 0:
            continue
        if Lk < Lq:
            raise ValueError("a context cannot be shorter than its new tokens")
        rows = np.arange(Lk)
        blocks = tables[b, rows // bs]
        if np.any(blocks < 0) or np.any(blocks >= num_blocks):
            raise ValueError("block table entry out of range")
        k_ctx = kc[blocks, rows % bs]  # [Lk, Hkv, d]
        v_ctx = vc[blocks, rows % bs]
        mask = end_aligned_mask(Lq, Lk)
        assert mask.any(axis=1).all(), "every new token sees at least one key"
        for h in range(Hq):
            hk = h // g
            z = scale * (q[s:e, h, :] @ k_ctx[:, hk, :].T)
            p = masked_softmax(z, mask)
            out[s:e, h, :] = p @ v_ctx[:, hk, :]
    return out


def unmasked_pairs(cu_seqlens, causal: bool) -> int:
    """Visible (query, key) pairs per head, counted from the explicit masks.

    Bidirectional this is sum_b L_b^2: the B*T^2 factor of the paper's attention FLOP count
    4*B*T^2*H (H = heads * head_dim).  The FLOP convention used for reporting is
    4 * head_dim * n_q_heads * unmasked_pairs.
    """
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    total = 0
    for b in range(len(cu) - 1):
        L = int(cu[b + 1] - cu[b])
        if L > 0:
            total += int(visibility_mask(L, causal).sum())
    return total


def kv_cache_write(k_bits, v_bits, k_cache_bits, v_cache_bits, slot_mapping, block_size: int):
    """Paged KV scatter on raw bf16 bit patterns (uint16); returns new (k_cache, v_cache).

    k_bits, v_bits: [N, Hkv, d]; caches: [num_blocks, block_size, Hkv, d]; slot_mapping: [N].
    Tokens are taken in order; slot < 0 skips the token; every other byte keeps its old value.
    """
    kc = np.array(k_cache_bits, dtype=np.uint16, copy=True)
    vc = np.array(v_cache_bits, dtype=np.uint16, copy=True)
    kb = np.asarray(k_bits).view(np.uint16)
    vb = np.asarray(v_bits).view(np.uint16)
    num_blocks = kc.shape[0]
    if kc.shape[1] != block_size:
        raise ValueError("cache block dimension does not match block_size")
    for t, slot in enumerate(np.asarray(slot_mapping, dtype=np.int64).tolist()):
        if slot < 0:
            continue
        blk, off = divmod(slot, block_size)
        if blk >= num_blocks:
            raise ValueError("slot out of range")
        kc[blk, off] = kb[t]
        vc[blk, off] = vb[t]
    return kc, vc


def page_cache_write(rows_bits, cache_bits, slot_mapping):
    """Paged image cache, write direction, on raw bf16 bit patterns: returns the new cache.

    The paper pages the image cache like the KV cache (Section 4.5; block size 576 in Section 5.1).
    rows_bits: [n, row_elems]; cache_bits: [num_slots, row_elems] (pages flattened); slot_mapping: [n].
    Rows are taken in order; slot < 0 skips the row; every other cache row keeps its old value."""
    cache = np.array(cache_bits, dtype=np.uint16, copy=True)
    rows = np.asarray(rows_bits).view(np.uint16)
    flat = cache.reshape(-1, rows.shape[1])
    for t, slot in enumerate(np.asarray(slot_mapping, dtype=np.int64).tolist()):
        if slot < 0:
            continue
        if slot >= flat.shape[0]:
            raise ValueError("slot out of range")
        flat[slot] = rows[t]
    return cache


def page_cache_gather(cache_bits, slot_mapping, rows_bits):
    """Paged image cache, read direction: returns the new rows (row t = cache row slot_mapping[t];
    a row whose slot is negative keeps its old value)."""
    rows = np.array(rows_bits, dtype=np.uint16, copy=True)
    flat = np.asarray(cache_bits).view(np.uint16).reshape(-1, rows.shape[1])
    for t, slot in enumerate(np.asarray(slot_mapping, dtype=np.int64).tolist()):
        if slot < 0:
            continue
        if slot >= flat.shape[0]:
            raise ValueError("slot out of range")
        rows[t] = flat[slot]
    return rows
