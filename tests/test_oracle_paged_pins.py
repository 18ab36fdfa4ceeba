"""Pins for the oracle of attention over the paged KV cache (CPU only).  The paper prints no worked
example, so the oracle is pinned by hand-derived cases, closed forms, invariants, its reduction to
the (separately pinned) packed causal attention, and a brute-force evaluation written here with
Python scalars."""
import json
import math
import os

import numpy as np
import pytest

from oracle import reference

HERE = os.path.dirname(os.path.abspath(__file__))


def _cu(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def _paged(rng, kv_lens, Hkv, d, bs, spare=3):
    """Random caches (every slot random) and block tables off a shuffled free list."""
    blocks_of = [(k + bs - 1) // bs for k in kv_lens]
    num_blocks = sum(blocks_of) + spare
    free = rng.permutation(num_blocks).tolist()
    tables = np.full((len(kv_lens), max(blocks_of + [1])), -1, dtype=np.int32)
    for b, nb in enumerate(blocks_of):
        for n in range(nb):
            tables[b, n] = free.pop()
    kc = rng.standard_normal((num_blocks, bs, Hkv, d))
    vc = rng.standard_normal((num_blocks, bs, Hkv, d))
    return kc, vc, tables


def _context(cache, table, kv_len, bs):
    rows = np.arange(kv_len)
    return cache[table[rows // bs], rows % bs]


def _load_cases():
    with open(os.path.join(HERE, "golden", "hand_cases_paged.json")) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _load_cases(), ids=lambda c: c["name"])
def test_hand_derived_cases(case):
    d, bs, nb = case["d"], case["block_size"], case["num_blocks"]
    kc = np.full((nb, bs, 1, d), 1000.0)
    vc = np.full((nb, bs, 1, d), -1000.0)
    for b, (klog, vals) in enumerate(zip(case["context_k_log_of"], case["context_v"])):
        for j, (kl, vv) in enumerate(zip(klog, vals)):
            blk, off = case["block_table"][b][j // bs], j % bs
            kc[blk, off, 0, :] = np.log(np.asarray(kl, dtype=np.float64))
            if "k_second_coord" in case:
                kc[blk, off, 0, 1] = case["k_second_coord"][b][j]
            vc[blk, off, 0, :] = vv
    q = np.asarray(case["q"], dtype=np.float64)[:, None, :]
    width = max(len(t) for t in case["block_table"])
    tables = np.array([t + [-1] * (width - len(t)) for t in case["block_table"]], dtype=np.int32)
    got = reference.attn_paged(q, kc, vc, tables, _cu(case["q_lens"]), case["kv_lens"], case["scale"])
    np.testing.assert_allclose(got[:, 0, :], np.asarray(case["expect"]), rtol=0, atol=1e-12)


def test_full_prefill_reduces_to_packed_causal_attention():
    """q_len == kv_len for every request: the result is the packed causal attention of the gathered K/V."""
    rng = np.random.default_rng(0)
    lens, Hq, Hkv, d, bs = [5, 16, 1, 37], 4, 2, 8, 4
    kc, vc, tables = _paged(rng, lens, Hkv, d, bs)
    q = rng.standard_normal((sum(lens), Hq, d))
    got = reference.attn_paged(q, kc, vc, tables, _cu(lens), lens, 0.3)
    k = np.concatenate([_context(kc, tables[b], L, bs) for b, L in enumerate(lens)])
    v = np.concatenate([_context(vc, tables[b], L, bs) for b, L in enumerate(lens)])
    want = reference.attn_varlen(q, k, v, _cu(lens), True, 0.3)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_chunks_reproduce_the_whole_prefill():
    """A prompt processed in chunks (each chunk attends to the cache up to its own end) gives, row for
    row, the causal attention of the whole prompt."""
    rng = np.random.default_rng(1)
    L, Hq, Hkv, d, bs = 45, 2, 1, 8, 16
    kc, vc, tables = _paged(rng, [L], Hkv, d, bs)
    q = rng.standard_normal((L, Hq, d))
    whole = reference.attn_paged(q, kc, vc, tables, _cu([L]), [L], 0.25)
    pieces, start = [], 0
    for chunk in (7, 16, 1, 21):
        end = start + chunk
        pieces.append(reference.attn_paged(q[start:end], kc, vc, tables, _cu([chunk]), [end], 0.25))
        start = end
    np.testing.assert_allclose(np.concatenate(pieces), whole, rtol=0, atol=1e-13)


def test_identical_keys_give_prefix_means():
    """All keys equal: new token i returns the plain mean of V over keys 0 .. kv_len - q_len + i."""
    rng = np.random.default_rng(2)
    q_len, kv_len, d, bs = 5, 19, 4, 8
    kc, vc, tables = _paged(rng, [kv_len], 1, d, bs)
    kc[...] = rng.standard_normal(d)
    q = rng.standard_normal((q_len, 1, d))
    got = reference.attn_paged(q, kc, vc, tables, _cu([q_len]), [kv_len], 0.7)
    v = _context(vc, tables[0], kv_len, bs)[:, 0, :]
    for i in range(q_len):
        np.testing.assert_allclose(got[i, 0], v[: kv_len - q_len + i + 1].mean(axis=0), rtol=0, atol=1e-12)


def test_physical_placement_and_unowned_slots_do_not_matter():
    """Moving the pages inside the cache (with the tables following) changes nothing, nor do the values
    of slots past a context's end or in blocks no request owns."""
    rng = np.random.default_rng(3)
    q_lens, kv_lens, Hq, Hkv, d, bs = [1, 6, 3], [21, 6, 40], 4, 2, 8, 16
    kc, vc, tables = _paged(rng, kv_lens, Hkv, d, bs, spare=4)
    q = rng.standard_normal((sum(q_lens), Hq, d))
    base = reference.attn_paged(q, kc, vc, tables, _cu(q_lens), kv_lens, 0.35)
    perm = rng.permutation(kc.shape[0])          # block n moves to perm[n]
    kc2, vc2 = np.empty_like(kc), np.empty_like(vc)
    kc2[perm], vc2[perm] = kc, vc
    tables2 = np.where(tables >= 0, perm[np.maximum(tables, 0)], -1).astype(np.int32)
    moved = reference.attn_paged(q, kc2, vc2, tables2, _cu(q_lens), kv_lens, 0.35)
    np.testing.assert_array_equal(moved, base)
    owned = np.zeros(kc.shape[:2], dtype=bool)
    for b, L in enumerate(kv_lens):
        rows = np.arange(L)
        owned[tables[b, rows // bs], rows % bs] = True
    kc3, vc3 = kc.copy(), vc.copy()
    kc3[~owned] = 1e6
    vc3[~owned] = -1e6
    np.testing.assert_array_equal(reference.attn_paged(q, kc3, vc3, tables, _cu(q_lens), kv_lens, 0.35), base)


def test_requests_are_isolated():
    """Changing one request's context leaves the other requests' outputs bit-identical."""
    rng = np.random.default_rng(4)
    q_lens, kv_lens, bs = [2, 1, 4], [9, 30, 4], 4
    kc, vc, tables = _paged(rng, kv_lens, 1, 8, bs)
    q = rng.standard_normal((sum(q_lens), 2, 8))
    base = reference.attn_paged(q, kc, vc, tables, _cu(q_lens), kv_lens, 0.5)
    kc2 = kc.copy()
    blocks = tables[1, : (30 + bs - 1) // bs]
    kc2[blocks] = rng.standard_normal(kc2[blocks].shape)   # (a common shift of all keys would cancel in the softmax)
    other = reference.attn_paged(q, kc2, vc, tables, _cu(q_lens), kv_lens, 0.5)
    np.testing.assert_array_equal(other[:2], base[:2])
    np.testing.assert_array_equal(other[3:], base[3:])
    assert np.abs(other[2] - base[2]).max() > 1e-6


def test_brute_force_with_python_scalars():
    """Small hybrid batch with grouped query heads, a zero-length request and ragged pages, against a
    loop over (request, head, new token) that walks the block table itself."""
    rng = np.random.default_rng(5)
    q_lens, kv_lens, Hq, Hkv, d, bs, scale = [1, 0, 3, 5], [7, 4, 3, 11], 4, 2, 3, 4, 0.6
    kc, vc, tables = _paged(rng, kv_lens, Hkv, d, bs)
    q = rng.standard_normal((sum(q_lens), Hq, d))
    got = reference.attn_paged(q, kc, vc, tables, _cu(q_lens), kv_lens, scale)
    cu = _cu(q_lens)
    for b in range(len(q_lens)):
        for h in range(Hq):
            hk = h // (Hq // Hkv)
            for i in range(q_lens[b]):
                last = kv_lens[b] - q_lens[b] + i
                zs = []
                for j in range(last + 1):
                    blk, off = int(tables[b, j // bs]), j % bs
                    zs.append(scale * sum(float(q[cu[b] + i, h, c]) * float(kc[blk, off, hk, c]) for c in range(d)))
                top = max(zs)
                ws = [math.exp(z - top) for z in zs]
                tot = math.fsum(ws)
                for c in range(d):
                    want = math.fsum(w * float(vc[int(tables[b, j // bs]), j % bs, hk, c]) for j, w in enumerate(ws)) / tot
                    assert abs(got[cu[b] + i, h, c] - want) < 1e-12


def test_last_new_token_sees_everything_and_mask_counts():
    """The last new token's row is plain softmax attention over the whole context; the explicit masks
    hold q (kv - q) + q (q + 1) / 2 visible pairs."""
    from scipy.special import softmax
    rng = np.random.default_rng(6)
    q_len, kv_len, d, bs = 4, 23, 8, 16
    kc, vc, tables = _paged(rng, [kv_len], 1, d, bs)
    q = rng.standard_normal((q_len, 1, d))
    got = reference.attn_paged(q, kc, vc, tables, _cu([q_len]), [kv_len], 0.4)
    k = _context(kc, tables[0], kv_len, bs)[:, 0, :]
    v = _context(vc, tables[0], kv_len, bs)[:, 0, :]
    np.testing.assert_allclose(got[-1, 0], softmax(0.4 * (k @ q[-1, 0])) @ v, rtol=0, atol=1e-13)
    for ql, kl in [(1, 1), (1, 17), (5, 5), (4, 23), (64, 100)]:
        assert int(reference.end_aligned_mask(ql, kl).sum()) == ql * (kl - ql) + ql * (ql + 1) // 2


def test_invalid_inputs_are_rejected():
    rng = np.random.default_rng(7)
    kc, vc, tables = _paged(rng, [8], 1, 4, 4)
    q = rng.standard_normal((3, 1, 4))
    with pytest.raises(ValueError):
        reference.attn_paged(q, kc, vc, tables, _cu([3]), [2], 1.0)      # context shorter than its new tokens
    bad = tables.copy()
    bad[0, 0] = kc.shape[0]
    with pytest.raises(ValueError):
        reference.attn_paged(q, kc, vc, bad, _cu([3]), [8], 1.0)         # block id outside the cache
