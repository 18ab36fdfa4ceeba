"""GPU parity of attention over the paged KV cache: the HIP kernel, called through the C ABI, against
the fp64 oracle on the same seeded bf16 inputs.  Same tolerance as the packed attention: max |diff| <=
2e-2 and mean |diff| <= 2e-3 over all output elements."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import reference

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def _f64(t):
    return reference.bf16_bits_to_f64(si.bf16_bits(t))


def _run_gpu(h, q, k_cache, v_cache, tables, scale=None, out=None, max_q_len=None, **kw):
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    res = hydra.hydra_attn_paged_fwd(q.to(dev), k_cache.to(dev), v_cache.to(dev), torch.from_numpy(tables).to(dev),
                                     torch.from_numpy(h.cu_seqlens_q).to(dev), torch.tensor(h.kv_lens, dtype=torch.int32, device=dev),
                                     max(h.max_q_len, 1) if max_q_len is None else max_q_len, h.softmax_scale if scale is None else scale,
                                     out=out, **kw)
    torch.cuda.synchronize()
    return res


def _want(h, q, k_cache, v_cache, tables, scale=None):
    return reference.attn_paged(_f64(q), _f64(k_cache), _f64(v_cache), tables, h.cu_seqlens_q, h.kv_lens,
                                h.softmax_scale if scale is None else scale)


def _check(out, want):
    got = _f64(out)
    assert np.isfinite(got).all()
    diff = np.abs(got - want)
    print(f"max abs {diff.max():.3e}  mean abs {diff.mean():.3e}")
    assert diff.max() <= MAX_ABS
    assert diff.mean() <= MEAN_ABS


CASES = [
    # q_lens, kv_lens, Hq, Hkv, d, block_size
    ([1], [1], 1, 1, 64, 16),
    ([1, 1, 1], [1, 16, 17], 2, 1, 128, 16),
    ([1, 0, 3, 5], [7, 4, 3, 11], 4, 2, 64, 4),
    ([17, 64, 100, 257], [17, 64, 100, 257], 2, 2, 64, 16),           # full prefills
    ([17, 64, 100, 257], [40, 64, 1000, 300], 2, 2, 128, 16),         # chunks at the end of longer contexts
    ([63, 64, 65, 1, 129], [63, 128, 65, 700, 129 + 64], 7, 1, 128, 16),
    ([1] * 9 + [200], [33, 64, 65, 127, 128, 129, 511, 512, 513, 333], 28, 4, 128, 16),
    ([5, 130], [260, 1027], 2, 2, 80, 16),
    ([1, 70], [2000, 70], 8, 2, 80, 32),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"q{'_'.join(map(str, c[0]))}-h{c[2]}k{c[3]}-d{c[4]}-b{c[5]}")
def test_ragged_hybrid_batches_full(case):
    q_lens, kv_lens, hq, hkv, d, bs = case
    h = si.HybridBatch("case", q_lens, kv_lens, hq, hkv, d, block_size=bs, seed=len(q_lens) * 100 + hq)
    q, kc, vc, tables = si.make_paged_inputs(h)
    _check(_run_gpu(h, q, kc, vc, tables), _want(h, q, kc, vc, tables))


def test_many_requests_with_scattered_chunks():
    """More requests than the threads of a workgroup, with prefill chunks (ragged lengths, some shorter than a
    wave tile, some invalid or empty requests) scattered among decode steps: the workgroups of the wave-tile
    form locate their request by a scan over all requests, several per thread here."""
    rng = np.random.default_rng(8)
    n = 700
    q_lens = [1] * n
    kv_lens = rng.integers(1, 90, size=n).tolist()
    for pos, ql, extra in ((0, 33, 0), (1, 200, 40), (255, 64, 64), (256, 5, 3), (257, 129, 1), (511, 6, 100), (512, 40, 0), (699, 300, 77), (300, 0, 9)):
        q_lens[pos], kv_lens[pos] = ql, ql + extra
    h = si.HybridBatch("many", q_lens, kv_lens, 8, 2, 64, seed=21)
    q, kc, vc, tables = si.make_paged_inputs(h)
    _check(_run_gpu(h, q, kc, vc, tables), _want(h, q, kc, vc, tables))


@pytest.mark.parametrize("seed", range(24))
def test_random_hybrid_batches(seed):
    """Seeded random hybrid batches: decode steps, short and long chunks, whole prefills, empty requests, in
    random order, random head grouping, head_dim and block size; whole output against the oracle."""
    rng = np.random.default_rng(2000 + seed)
    hq, hkv = [(1, 1), (4, 1), (4, 2), (7, 1), (8, 8), (28, 4)][int(rng.integers(6))]
    d = [64, 80, 128][int(rng.integers(3))]
    bs = [1, 4, 16, 32][int(rng.integers(4))]
    q_lens, kv_lens = [], []
    for _ in range(int(rng.integers(1, 60))):
        kind = int(rng.integers(5))
        ql = [1, int(rng.integers(2, 9)), int(rng.integers(9, 200)), int(rng.integers(1, 150)), 0][kind]
        extra = 0 if kind == 3 else int(rng.integers(0, 400))
        q_lens.append(ql)
        kv_lens.append(ql + extra if ql else int(rng.integers(0, 50)))
    if sum(q_lens) == 0:
        q_lens[0], kv_lens[0] = 3, 10
    h = si.HybridBatch("random", q_lens, kv_lens, hq, hkv, d, block_size=bs, seed=seed)
    q, kc, vc, tables = si.make_paged_inputs(h)
    _check(_run_gpu(h, q, kc, vc, tables), _want(h, q, kc, vc, tables))


PIPELINED_CASES = [
    # q_lens, kv_lens, Hq, Hkv, d, block_size: prefill chunks whose groups of wave tiles run on the packed kernel's
    # pipeline (head_dim 64 or 128, a load instruction's rows inside one cache block); contexts of many key tiles,
    # new tokens that start anywhere inside a key block, last tiles partly filled
    ([300], [1500], 4, 2, 128, 4),
    ([300, 1, 77], [1500, 900, 1077], 7, 1, 128, 8),
    ([512, 512], [2048, 513], 28, 4, 128, 16),
    ([129, 64, 33], [129 + 31, 64 + 1, 33 + 1000], 8, 2, 64, 8),
    ([200, 40], [777, 40], 4, 4, 64, 64),
    ([100], [1000], 2, 1, 128, 256),
    ([65, 300], [65, 301], 2, 2, 64, 4),               # head_dim 64 with blocks of 4 rows: the plain loop
    ([5, 33, 9], [7, 40, 9], 7, 1, 128, 16),           # a handful of new tokens whose grouped heads fill more than one tile of rows
    ([2, 6], [2, 70], 28, 4, 64, 16),                  # one key tile, one key block; a context barely longer than a tile
]


@pytest.mark.parametrize("case", PIPELINED_CASES, ids=lambda c: f"q{'_'.join(map(str, c[0]))}-kv{max(c[1])}-h{c[2]}k{c[3]}-d{c[4]}-b{c[5]}")
def test_chunks_over_long_contexts_and_block_sizes(case):
    q_lens, kv_lens, hq, hkv, d, bs = case
    h = si.HybridBatch("case", q_lens, kv_lens, hq, hkv, d, block_size=bs, seed=7 * len(q_lens) + bs)
    q, kc, vc, tables = si.make_paged_inputs(h)
    _check(_run_gpu(h, q, kc, vc, tables), _want(h, q, kc, vc, tables))


@pytest.mark.parametrize("d", [64, 128])
def test_large_scores_in_a_chunk_are_recomputed(d):
    """Keys planted behind the first key block of a chunk's context whose scores lead the block-0 maximum by far more
    than the pipelined path's range: the workgroup notices (row sums beyond 2^40 times the reference term) and
    computes its group of wave tiles again with the plain loop, which rescales at every tile; if it did not, the
    rows would be inf / NaN or wrong."""
    h = si.HybridBatch("planted", [100, 1, 257], [400, 300, 257], 4, 2, d, seed=77)
    q, kc, vc, tables = si.make_paged_inputs(h)
    kc = kc.clone()
    for b, j in ((0, 50), (0, 350), (2, 200)):       # request, key position (>= 32: not in key block 0)
        kc[tables[b, j // 16], j % 16] = 64.0        # score = scale * 64 * sum(q): tens of units either way
    z = h.softmax_scale * 64.0 * _f64(q).sum(axis=-1)
    assert (z * 1.4427 > 100).sum() > 50
    _check(_run_gpu(h, q, kc, vc, tables), _want(h, q, kc, vc, tables))


def test_full_size_hybrid_batch():
    """The benchmark's hybrid batch (96 decode requests + 4 prefill chunks of 512, 28 / 4 heads of 128), whole output."""
    h = si.qwen2vl_hybrid()
    q, kc, vc, tables = si.make_paged_inputs(h)
    _check(_run_gpu(h, q, kc, vc, tables), _want(h, q, kc, vc, tables))


def test_matches_packed_kernel_after_cache_write():
    """A packed causal prefill, its K/V scattered into the cache with hydra_kv_cache_write, then the paged
    kernel over that cache: both HIP paths against the oracle of the packed attention."""
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    w = si.custom([100, 257, 16], 4, 2, 128, True, seed=5, kv_cache=True)
    q, k, v = si.make_qkv(w)
    slots, num_blocks = si.make_slot_mapping(w.lengths, 16, seed=5)
    kc = torch.zeros((num_blocks, 16, 2, 128), dtype=torch.bfloat16, device=dev)
    vc = torch.zeros_like(kc)
    hydra.hydra_kv_cache_write(k.to(dev), v.to(dev), kc, vc, torch.from_numpy(slots).to(dev))
    width = max((L + 15) // 16 for L in w.lengths)
    tables = np.full((w.batch, width), -1, dtype=np.int32)
    for b in range(w.batch):
        s = int(w.cu_seqlens[b])
        for n in range((w.lengths[b] + 15) // 16):
            tables[b, n] = slots[s + 16 * n] // 16
    h = si.HybridBatch("after_write", w.lengths, w.lengths, 4, 2, 128)
    out = _run_gpu(h, q, kc, vc, tables)
    want = reference.attn_varlen(_f64(q), _f64(k), _f64(v), w.cu_seqlens, True, w.softmax_scale)
    _check(out, want)


def test_strided_q_canaries_and_determinism():
    """q as a view into a wider buffer; rows of `out` that belong to no request keep their contents; two runs agree bit for bit."""
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    h = si.HybridBatch("views", [3, 1, 70], [19, 300, 70], 4, 2, 128, seed=9)
    q, kc, vc, tables = si.make_paged_inputs(h)
    wide = torch.zeros((h.total_q + 5, 4 * 128 + 64), dtype=torch.bfloat16, device=dev)
    qv = wide[: h.total_q, 64:].view(h.total_q, 4, 128)
    qv.copy_(q.to(dev))
    out = torch.full((h.total_q, 4, 128), 7.0, dtype=torch.bfloat16, device=dev)
    args = (kc.to(dev), vc.to(dev), torch.from_numpy(tables).to(dev), torch.from_numpy(h.cu_seqlens_q).to(dev),
            torch.tensor(h.kv_lens, dtype=torch.int32, device=dev), h.max_q_len, h.softmax_scale)
    first = hydra.hydra_attn_paged_fwd(qv, *args, out=out).clone()
    second = hydra.hydra_attn_paged_fwd(qv, *args)
    torch.cuda.synchronize()
    assert torch.equal(first.view(torch.int16), second.view(torch.int16))
    _check(first, _want(h, q, kc, vc, tables))
    # a batch whose cu_seqlens_q stops short of the buffer: the rows after it are not written
    short = si.HybridBatch("short", [3, 1], [19, 300], 4, 2, 128, seed=9)
    out.fill_(7.0)
    hydra.hydra_attn_paged_fwd(qv[:4], args[0], args[1], args[2][:2].contiguous(), torch.from_numpy(short.cu_seqlens_q).to(dev),
                               args[4][:2].contiguous(), 3, h.softmax_scale, out=out[:4])
    torch.cuda.synchronize()
    assert bool((out[4:] == 7.0).all())


def test_scale_zero_and_generous_max_q_len():
    """softmax_scale 0 gives plain means of the visible V rows; max_q_len may exceed the batch's longest request."""
    h = si.HybridBatch("zero", [2, 1], [40, 9], 2, 2, 64, seed=3)
    q, kc, vc, tables = si.make_paged_inputs(h)
    _check(_run_gpu(h, q, kc, vc, tables, scale=0.0, max_q_len=500), _want(h, q, kc, vc, tables, scale=0.0))


SPLIT_CASES = [
    # q_lens, kv_lens, Hq, Hkv, d: few requests with long contexts, so that the packed-rows form splits them over workgroups
    ([1, 1, 1], [5000, 40, 1300], 28, 4, 128),          # shares of the short contexts are empty
    ([4, 1], [3000, 2500], 8, 2, 64),                   # 4 tokens x 4 grouped heads = 16 packed rows, end-aligned mask inside a share
    ([1] * 6, [8192, 100, 4097, 33, 2048, 700], 14, 2, 80),
    ([1, 300], [6000, 900], 28, 4, 128),                # a split decode request next to a chunk in the wave-tile form
    ([1, 1, 1], [4100, 1089, 545], 8, 2, 128),          # contexts one key past a multiple of the share size (544 keys here)
]


@pytest.mark.parametrize("seed", range(12))
def test_random_batches_of_long_contexts(seed):
    """Seeded random small batches of ragged, long contexts with one or a few new tokens each (the packed-rows form,
    contexts cut into shares of equal length over several workgroups and merged), random head grouping, head_dim and
    block size; whole output against the oracle."""
    rng = np.random.default_rng(3000 + seed)
    hq, hkv = [(1, 1), (4, 1), (4, 2), (7, 1), (8, 8), (28, 4), (16, 2)][int(rng.integers(7))]
    d = [64, 80, 128][int(rng.integers(3))]
    bs = [4, 16, 32, 64][int(rng.integers(4))]
    g = hq // hkv
    top = [1500, 3000, 6000][int(rng.integers(3))]
    q_lens, kv_lens = [], []
    for _ in range(int(rng.integers(1, 6))):
        ql = int(rng.integers(1, max(2, 32 // g + 1))) if rng.random() < 0.9 else 0
        kv = int(rng.integers(ql, top)) if rng.random() < 0.7 else top - int(rng.integers(0, 40))
        q_lens.append(ql)
        kv_lens.append(max(kv, ql))
    if sum(q_lens) == 0:
        q_lens[0], kv_lens[0] = 1, top
    h = si.HybridBatch("long", q_lens, kv_lens, hq, hkv, d, block_size=bs, seed=seed)
    q, kc, vc, tables = si.make_paged_inputs(h)
    _check(_run_gpu(h, q, kc, vc, tables), _want(h, q, kc, vc, tables))


@pytest.mark.parametrize("case", SPLIT_CASES, ids=lambda c: f"q{'_'.join(map(str, c[0]))}-kv{max(c[1])}-h{c[2]}k{c[3]}-d{c[4]}")
def test_contexts_split_over_workgroups(case):
    """Small batches of long contexts: with the workspace the library asks for, contexts are split over several
    workgroups and merged by the combine kernel; without it one workgroup walks each context.  Both against the oracle."""
    import paper_2505_12658_amd as hydra

    q_lens, kv_lens, hq, hkv, d = case
    h = si.HybridBatch("split", q_lens, kv_lens, hq, hkv, d, seed=hq + len(q_lens))
    q, kc, vc, tables = si.make_paged_inputs(h)
    assert hydra.hydra_attn_paged_workspace_bytes(h.batch, hkv, d, tables.shape[1], 16) > 0
    want = _want(h, q, kc, vc, tables)
    _check(_run_gpu(h, q, kc, vc, tables), want)
    _check(_run_gpu(h, q, kc, vc, tables, use_workspace=False), want)
    # a workspace too small for the preferred number of shares still gives the right answer (fewer shares)
    small = torch.empty(hydra.hydra_attn_paged_workspace_bytes(h.batch, hkv, d, tables.shape[1], 16) // 3, dtype=torch.uint8, device="cuda:0")
    _check(_run_gpu(h, q, kc, vc, tables, workspace=small), want)


def test_requests_pages_move_to_another_cache():
    """What a migration between instances does to a request on the sending and on the receiving GPU (Section 4.3:
    its cache pages are copied, its page table is rewritten), done here between two caches on one GPU with the
    paged-cache copy calls, one row per cache block: the pages of every request are gathered into one contiguous
    buffer (what would travel), written into other blocks of a second cache, and attention over the second cache with
    the rewritten block table gives the same output bit for bit; blocks of the second cache that received nothing
    keep their contents."""
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    h = si.HybridBatch("move", [1, 70, 1, 3], [300, 200, 77, 19], 8, 2, 128, seed=55)
    q, kc, vc, tables = si.make_paged_inputs(h)
    qd, kcd, vcd = q.to(dev), kc.to(dev), vc.to(dev)
    cu = torch.from_numpy(h.cu_seqlens_q).to(dev)
    kv = torch.tensor(h.kv_lens, dtype=torch.int32, device=dev)
    before = hydra.hydra_attn_paged_fwd(qd, kcd, vcd, torch.from_numpy(tables).to(dev), cu, kv, h.max_q_len, h.softmax_scale)
    # the blocks that hold context, request by request, and their new places in a cache of another size
    bs = 16
    used = [tables[b, : (k + bs - 1) // bs] for b, k in enumerate(h.kv_lens)]
    src = np.concatenate(used).astype(np.int64)
    n_dst = len(src) + 13
    rng = np.random.default_rng(5)
    dst = rng.permutation(n_dst)[: len(src)].astype(np.int64)
    tables2 = np.zeros_like(tables)
    at = 0
    for b, u in enumerate(used):
        tables2[b, : len(u)] = dst[at : at + len(u)]
        at += len(u)
    row = bs * 2 * 128
    sentinel = 1.5
    kc2 = torch.full((n_dst, bs, 2, 128), sentinel, dtype=torch.bfloat16, device=dev)
    vc2 = torch.full((n_dst, bs, 2, 128), -sentinel, dtype=torch.bfloat16, device=dev)
    srcd, dstd = torch.from_numpy(src).to(dev), torch.from_numpy(dst).to(dev)
    for cache, cache2 in ((kcd, kc2), (vcd, vc2)):
        packed = torch.empty((len(src), row), dtype=torch.bfloat16, device=dev)
        hydra.hydra_page_cache_gather(cache.view(cache.shape[0], row), srcd, packed)
        hydra.hydra_page_cache_write(packed, cache2.view(n_dst, row), dstd)
    after = hydra.hydra_attn_paged_fwd(qd, kc2, vc2, torch.from_numpy(tables2).to(dev), cu, kv, h.max_q_len, h.softmax_scale)
    torch.cuda.synchronize()
    assert torch.equal(before.view(torch.int16), after.view(torch.int16))
    _check(after, _want(h, q, kc, vc, tables))
    untouched = np.setdiff1d(np.arange(n_dst), dst)
    assert (kc2[torch.from_numpy(untouched).to(dev)] == sentinel).all() and (vc2[torch.from_numpy(untouched).to(dev)] == -sentinel).all()
