"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no attention or scatter arithmetic: it only draws sequence lengths, bf16
values and paged-cache slot mappings with the shapes of the paper's workloads (Section 5.1:
LLaVA-1.5 encodes a 336x336 image to 576 tokens, Qwen2-VL's token count follows the image
resolution, KV-cache block size 16).  The paper's datasets are not available; these draws stand
in for the batches its stage-level batching would form.

Lengths, permutations: numpy default_rng(seed).  Values: torch CPU generator, N(0,1)*std in
fp32, rounded to bf16 (round-to-nearest-even); the bf16 tensor is THE input for both the GPU
path and the oracle.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    lengths: List[int]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    causal: bool
    value_std: float = 1.0
    kv_cache: bool = False
    block_size: int = 16
    seed: int = 0
    cu_seqlens: np.ndarray = field(init=False)

    def __post_init__(self):
        self.cu_seqlens = np.concatenate([[0], np.cumsum(self.lengths)]).astype(np.int32)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def batch(self) -> int:
        return len(self.lengths)

    @property
    def max_seqlen(self) -> int:
        return max(self.lengths) if self.lengths else 0

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    def unmasked_pairs(self) -> int:
        """Closed-form count of visible (q, k) pairs per head: sum L^2 or sum L(L+1)/2."""
        if self.causal:
            return sum(L * (L + 1) // 2 for L in self.lengths)
        return sum(L * L for L in self.lengths)

    def attention_flops(self) -> int:
        """4 * head_dim * n_q_heads * visible pairs (two contractions, multiply + add)."""
        return 4 * self.head_dim * self.n_q_heads * self.unmasked_pairs()

    def attention_min_bytes(self) -> int:
        """Q read + O write + K and V read once, bf16."""
        return (2 * self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim * self.total_tokens * 2

    def kv_write_bytes(self) -> int:
        """K and V rows read + written, plus the int64 slot index per token."""
        row = self.n_kv_heads * self.head_dim * 2
        return self.total_tokens * (4 * row + 8)


def _log_uniform_int(rng, lo: int, hi: int) -> int:
    return int(round(math.exp(rng.uniform(math.log(lo), math.log(hi)))))


def tiny(causal: bool, seed: int = 0) -> Workload:
    """4 packed sequences {17, 64, 100, 257}, 2 heads of 64, block-16 paged cache."""
    return Workload("tiny_" + ("causal" if causal else "bidir"), [17, 64, 100, 257], 2, 2, 64, causal, kv_cache=True, seed=seed)


def clip_vit_encode(seed: int = 0) -> Workload:
    """CLIP ViT-L/14-336 encode attention: 32 images x 577 tokens (576 patches + class token)."""
    return Workload("clip_vit_l14_336_encode", [577] * 32, 16, 16, 64, False, value_std=0.5, seed=seed)


def llava15_prefill(seed: int = 0) -> Workload:
    """LLaVA-1.5-7B prefill: 16 requests of 576 image tokens + U{16..256} text tokens, 32 MHA heads of 128."""
    rng = np.random.default_rng(seed)
    lengths = [576 + int(rng.integers(16, 257)) for _ in range(16)]
    return Workload("llava15_7b_prefill", lengths, 32, 32, 128, True, kv_cache=True, seed=seed)


def qwen2vl_vit_encode(seed: int = 0, target_tokens: int = 65536) -> Workload:
    """Qwen2-VL ViT encode, dynamic resolution: per-image tokens log-uniform in [256, 4096]
    (multiples of 4) packed to about 64k tokens; the last image is trimmed to land on the target."""
    rng = np.random.default_rng(seed)
    lengths: List[int] = []
    total = 0
    while total < target_tokens - 256:
        L = 4 * int(round(_log_uniform_int(rng, 256, 4096) / 4))
        L = max(256, min(4096, L))
        if total + L > target_tokens:
            L = max(256, ((target_tokens - total) // 4) * 4)
        lengths.append(L)
        total += L
    return Workload("qwen2vl_vit_encode", lengths, 16, 16, 80, False, seed=seed)


def qwen2vl_prefill(seed: int = 0) -> Workload:
    """Qwen2-VL-7B prefill: 48 requests, image tokens log-uniform in [64, 1024] + text U{32..512},
    GQA 28 query / 4 KV heads of 128, causal, block-16 paged cache."""
    rng = np.random.default_rng(seed)
    lengths = [_log_uniform_int(rng, 64, 1024) + int(rng.integers(32, 513)) for _ in range(48)]
    return Workload("qwen2vl_7b_prefill", lengths, 28, 4, 128, True, kv_cache=True, seed=seed)


def custom(lengths, n_q_heads, n_kv_heads, head_dim, causal, seed=0, value_std=1.0, kv_cache=False, block_size=16) -> Workload:
    return Workload("custom", list(lengths), n_q_heads, n_kv_heads, head_dim, causal, value_std, kv_cache, block_size, seed)


WORKLOADS = {
    "tiny_bidir": lambda seed=0: tiny(False, seed),
    "tiny_causal": lambda seed=0: tiny(True, seed),
    "clip_vit_l14_336_encode": clip_vit_encode,
    "llava15_7b_prefill": llava15_prefill,
    "qwen2vl_vit_encode": qwen2vl_vit_encode,
    "qwen2vl_7b_prefill": qwen2vl_prefill,
}


@dataclass
class HybridBatch:
    """One batch of the paper's Algorithm 1: decode requests (one new token) and chunks of prefill
    requests, each attending to its own paged KV cache.  q_lens[b] new tokens, kv_lens[b] tokens of
    context with the new ones included."""
    name: str
    q_lens: List[int]
    kv_lens: List[int]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block_size: int = 16
    seed: int = 0
    cu_seqlens_q: np.ndarray = field(init=False)

    def __post_init__(self):
        assert len(self.q_lens) == len(self.kv_lens) and all(k >= q >= 0 for q, k in zip(self.q_lens, self.kv_lens))
        self.cu_seqlens_q = np.concatenate([[0], np.cumsum(self.q_lens)]).astype(np.int32)

    @property
    def batch(self) -> int:
        return len(self.q_lens)

    @property
    def total_q(self) -> int:
        return int(self.cu_seqlens_q[-1])

    @property
    def max_q_len(self) -> int:
        return max(self.q_lens) if self.q_lens else 0

    @property
    def softmax_scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    def visible_pairs(self) -> int:
        """New token i of a request sees kv - q + i + 1 keys: q (kv - q) + q (q + 1) / 2 per request."""
        return sum(q * (k - q) + q * (q + 1) // 2 for q, k in zip(self.q_lens, self.kv_lens))

    def attention_flops(self) -> int:
        return 4 * self.head_dim * self.n_q_heads * self.visible_pairs()

    def attention_min_bytes(self) -> int:
        """Q read + O write, and every request's K and V context read once, bf16."""
        ctx = sum(k for q, k in zip(self.q_lens, self.kv_lens) if q > 0)
        return (2 * self.n_q_heads * self.total_q + 2 * self.n_kv_heads * ctx) * self.head_dim * 2


def qwen2vl_hybrid(seed: int = 0, n_decode: int = 96, chunk: int = 512, n_chunked: int = 4) -> HybridBatch:
    """Qwen2-VL-7B-shaped hybrid batch: n_decode decode requests whose context is a prompt drawn like
    the prefill workload's (image log-uniform [64, 1024] + text U{32..512}) plus U{1..256} generated
    tokens, and n_chunked prefill requests contributing one chunk each, with 0, 1, 2, ... chunks of
    the same size already in the cache."""
    rng = np.random.default_rng(seed + 31)
    q_lens, kv_lens = [], []
    for _ in range(n_decode):
        q_lens.append(1)
        kv_lens.append(_log_uniform_int(rng, 64, 1024) + int(rng.integers(32, 513)) + int(rng.integers(1, 257)))
    for c in range(n_chunked):
        q_lens.append(chunk)
        kv_lens.append((c + 1) * chunk)
    order = rng.permutation(len(q_lens))
    return HybridBatch("qwen2vl_7b_hybrid", [q_lens[i] for i in order], [kv_lens[i] for i in order], 28, 4, 128, seed=seed)


def make_paged_inputs(h: HybridBatch, spare_blocks: int = 8, value_std: float = 1.0):
    """bf16 CPU tensors q [Nq, Hq, d], k_cache, v_cache [num_blocks, block_size, Hkv, d] (EVERY slot holds
    a random value, so a read from a wrong page or past the context shows), and int32 block_tables
    [B, max_blocks] taken off a shuffled free list (entries past a request's last block are -1)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(h.seed + 17)
    rng = np.random.default_rng(h.seed + 65537)
    bs = h.block_size
    blocks_of = [(k + bs - 1) // bs for k in h.kv_lens]
    num_blocks = sum(blocks_of) + spare_blocks
    max_blocks = max(blocks_of + [1])
    free = rng.permutation(num_blocks).tolist()
    tables = np.full((h.batch, max_blocks), -1, dtype=np.int32)
    for b, nb in enumerate(blocks_of):
        for n in range(nb):
            tables[b, n] = free.pop()

    def draw(*shape):
        return (torch.randn(shape, generator=g, dtype=torch.float32) * value_std).to(torch.bfloat16)

    q = draw(h.total_q, h.n_q_heads, h.head_dim)
    k_cache = draw(num_blocks, bs, h.n_kv_heads, h.head_dim)
    v_cache = draw(num_blocks, bs, h.n_kv_heads, h.head_dim)
    return q, k_cache, v_cache, tables


@dataclass
class ImageCacheBatch:
    """Image tokens of one encode batch on their way into (or out of) the paged image cache:
    tokens[i] rows of `hidden` bf16 values for image i, pages of `page_rows` rows (576 in the paper's
    Section 5.1; a LLaVA-1.5 image fills exactly one page, a Qwen2-VL image a ragged number)."""
    name: str
    tokens: List[int]
    hidden: int
    page_rows: int = 576
    seed: int = 0

    @property
    def n_rows(self) -> int:
        return sum(self.tokens)

    def bytes_moved(self) -> int:
        """Every row read once and written once, plus the int64 slot per row."""
        return self.n_rows * (2 * self.hidden * 2 + 8)


def llava15_image_cache(seed: int = 0) -> ImageCacheBatch:
    """32 LLaVA-1.5 images x 576 tokens of hidden size 4096: one full page each."""
    return ImageCacheBatch("llava15_image_cache", [576] * 32, 4096, seed=seed)


def qwen2vl_image_cache(seed: int = 0) -> ImageCacheBatch:
    """32 Qwen2-VL images, tokens log-uniform in [64, 1024] (after the 2x2 merge), hidden size 3584:
    ragged pages."""
    rng = np.random.default_rng(seed + 11)
    return ImageCacheBatch("qwen2vl_image_cache", [_log_uniform_int(rng, 64, 1024) for _ in range(32)], 3584, seed=seed)


def make_image_rows(b: ImageCacheBatch):
    """bf16 CPU tensor [n_rows, hidden], N(0,1)."""
    g = torch.Generator(device="cpu")
    g.manual_seed(b.seed + 23)
    return torch.randn((b.n_rows, b.hidden), generator=g, dtype=torch.float32).to(torch.bfloat16)


def make_qkv(w: Workload, seed: Optional[int] = None):
    """bf16 CPU tensors q [N, Hq, d], k, v [N, Hkv, d]."""
    g = torch.Generator(device="cpu")
    g.manual_seed(w.seed if seed is None else seed)
    N = w.total_tokens

    def draw(heads):
        x = torch.randn((N, heads, w.head_dim), generator=g, dtype=torch.float32) * w.value_std
        return x.to(torch.bfloat16)

    return draw(w.n_q_heads), draw(w.n_kv_heads), draw(w.n_kv_heads)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Raw bit patterns of a bf16 tensor as a uint16 numpy array (no value conversion)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def make_slot_mapping(lengths, block_size: int = 16, spare_blocks: int = 8, seed: int = 0, skip_fraction: float = 0.0):
    """Block tables from a randomly permuted free list, flattened to one slot per token.

    Each sequence takes ceil(L / block_size) blocks off a shuffled free list (its last block is
    partly filled); token i of the sequence goes to table[i // block_size] * block_size + i % block_size.
    Returns (slot_mapping int64 [N], num_blocks).  skip_fraction > 0 marks that share of tokens
    with slot -1 (padding convention: such tokens are not written).
    """
    rng = np.random.default_rng(seed + 7919)
    need = sum((L + block_size - 1) // block_size for L in lengths)
    num_blocks = need + spare_blocks
    free = rng.permutation(num_blocks).tolist()
    slots = []
    for L in lengths:
        nb = (L + block_size - 1) // block_size
        table = [free.pop() for _ in range(nb)]
        for i in range(L):
            slots.append(table[i // block_size] * block_size + i % block_size)
    slots = np.asarray(slots, dtype=np.int64)
    if skip_fraction > 0 and len(slots):
        drop = rng.random(len(slots)) < skip_fraction
        slots[drop] = -1
    return slots, num_blocks


def make_cache_sentinel(num_blocks: int, block_size: int, n_kv_heads: int, head_dim: int, seed: int = 0):
    """Initial cache contents: a seeded non-trivial bit pattern, so untouched slots are checkable."""
    rng = np.random.default_rng(seed + 104729)
    return rng.integers(0, 1 << 16, size=(num_blocks, block_size, n_kv_heads, head_dim), dtype=np.uint16)
