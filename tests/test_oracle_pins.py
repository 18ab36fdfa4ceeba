"""Pins for the fp64 oracle (CPU only).  The paper prints no worked attention example, so the
oracle is pinned by closed forms, invariants, hand-derived cases and a brute-force evaluation
written independently here with Python scalars.  Every pin runs against both oracle
implementations (NumPy and plain C)."""
import json
import math
import os

import numpy as np
import pytest

import synth_inputs as si
from oracle import c_oracle, reference

IMPLS = {"numpy": reference, "c": c_oracle}
HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(params=list(IMPLS))
def impl(request):
    return IMPLS[request.param]


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _cu(lengths):
    return np.concatenate([[0], np.cumsum(lengths)]).astype(np.int32)


def brute_force(q, k, v, cu, causal, scale):
    """Independent evaluation with Python floats, one sequence and one head at a time,
    unpacked: no masks, no arrays of scores, just the visible range per query."""
    N, Hq, d = q.shape
    g = Hq // k.shape[1]
    out = np.zeros_like(q)
    for b in range(len(cu) - 1):
        s, e = int(cu[b]), int(cu[b + 1])
        for h in range(Hq):
            hk = h // g
            for i in range(e - s):
                hi = i + 1 if causal else e - s
                zs = [scale * sum(float(q[s + i, h, c]) * float(k[s + j, hk, c]) for c in range(d)) for j in range(hi)]
                m = max(zs)
                ws = [math.exp(z - m) for z in zs]
                tot = math.fsum(ws)
                for c in range(d):
                    out[s + i, h, c] = math.fsum(w * float(v[s + j, hk, c]) for j, w in enumerate(ws)) / tot
    return out


# --- hand-derived golden cases -------------------------------------------------------------
def _load_cases():
    with open(os.path.join(HERE, "golden", "hand_cases.json")) as f:
        return json.load(f)["cases"]


@pytest.mark.parametrize("case", _load_cases(), ids=lambda c: c["name"])
@pytest.mark.parametrize("causal", [False, True])
def test_hand_cases(impl, case, causal):
    d = case["d"]
    q = np.array(case["q"], dtype=np.float64).reshape(-1, 1, d)
    k = np.log(np.array(case["k_log_of"], dtype=np.float64)).reshape(-1, 1, d)
    if "k_second_coord" in case:
        k[:, 0, 1] = case["k_second_coord"]
    v = np.array(case["v"], dtype=np.float64).reshape(-1, 1, d)
    want = np.array(case["expect_causal" if causal else "expect_bidir"], dtype=np.float64).reshape(-1, 1, d)
    got = impl.attn_varlen(q, k, v, _cu(case["lengths"]), causal, case["scale"])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


# --- P1 rows of the softmax sum to one ------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_softmax_rows_sum_to_one(causal):
    rng = np.random.default_rng(1)
    L, d = 37, 8
    q, k = _rand(rng, L, d), _rand(rng, L, d)
    p = reference.attention_probs(q, k, 0.7, causal)
    assert (p >= 0).all()
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    if causal:
        assert (np.triu(p, 1) == 0).all()
    # the C oracle's probabilities, row by row
    v = _rand(rng, L, 1, d)
    rows = [(i, 0) for i in range(L)]
    _, pc = c_oracle.attn_rows(q[:, None, :], k[:, None, :], v, _cu([L]), causal, 0.7, rows, return_probs=True)
    np.testing.assert_allclose(pc.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    np.testing.assert_allclose(pc, p, rtol=0, atol=1e-14)


# --- P2 / P5 degenerate rows ----------------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_length_one_returns_v(impl, causal):
    rng = np.random.default_rng(2)
    q, k, v = _rand(rng, 3, 2, 4), _rand(rng, 3, 2, 4), _rand(rng, 3, 2, 4)
    out = impl.attn_varlen(q, k, v, _cu([1, 1, 1]), causal, 0.5)
    assert np.array_equal(out, v)


def test_causal_token0_returns_v0(impl):
    rng = np.random.default_rng(3)
    lengths = [5, 9]
    N = sum(lengths)
    q, k, v = _rand(rng, N, 2, 4), _rand(rng, N, 2, 4), _rand(rng, N, 2, 4)
    out = impl.attn_varlen(q, k, v, _cu(lengths), True, 0.5)
    assert np.array_equal(out[0], v[0])
    assert np.array_equal(out[5], v[5])


# --- P3 identical keys -> means --------------------------------------------------------------
def test_identical_keys_give_means(impl):
    rng = np.random.default_rng(4)
    L, H, d = 23, 2, 6
    q, v = _rand(rng, L, H, d), _rand(rng, L, H, d)
    k = np.broadcast_to(_rand(rng, 1, H, d), (L, H, d)).copy()
    out = impl.attn_varlen(q, k, v, _cu([L]), False, 0.3)
    np.testing.assert_allclose(out, np.broadcast_to(v.mean(axis=0), out.shape), rtol=0, atol=1e-13)
    outc = impl.attn_varlen(q, k, v, _cu([L]), True, 0.3)
    prefix_mean = np.cumsum(v, axis=0) / np.arange(1, L + 1)[:, None, None]
    np.testing.assert_allclose(outc, prefix_mean, rtol=0, atol=1e-13)


# --- P4 key permutation invariance (bidirectional) ---------------------------------------------
def test_bidirectional_invariant_to_key_permutation(impl):
    rng = np.random.default_rng(5)
    lengths = [11, 30]
    N = sum(lengths)
    q, k, v = _rand(rng, N, 2, 8), _rand(rng, N, 2, 8), _rand(rng, N, 2, 8)
    cu = _cu(lengths)
    base = impl.attn_varlen(q, k, v, cu, False, 0.4)
    perm = np.concatenate([rng.permutation(11), 11 + rng.permutation(30)])
    out = impl.attn_varlen(q, k[perm], v[perm], cu, False, 0.4)
    np.testing.assert_allclose(out, base, rtol=0, atol=1e-13)
    # and the causal result is NOT invariant (the mask has an orientation)
    c0 = impl.attn_varlen(q, k, v, cu, True, 0.4)
    c1 = impl.attn_varlen(q, k[perm], v[perm], cu, True, 0.4)
    assert np.abs(c0 - c1).max() > 1e-3


# --- P6 brute force, packed + GQA -------------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_matches_brute_force(impl, causal):
    rng = np.random.default_rng(6)
    lengths = [3, 1, 7, 0, 12]
    N = sum(lengths)
    q, k, v = _rand(rng, N, 4, 5), _rand(rng, N, 2, 5), _rand(rng, N, 2, 5)
    cu = _cu(lengths)
    got = impl.attn_varlen(q, k, v, cu, causal, 0.45)
    want = brute_force(q, k, v, cu, causal, 0.45)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_tiny_config_matches_brute_force_sampled(impl):
    """The tiny benchmark configuration itself (bf16 inputs), against brute force on one sequence."""
    w = si.tiny(True)
    qb, kb, vb = si.make_qkv(w)
    q, k, v = (reference.bf16_bits_to_f64(si.bf16_bits(t)) for t in (qb, kb, vb))
    got = impl.attn_varlen(q, k, v, w.cu_seqlens, True, w.softmax_scale)
    s, e = int(w.cu_seqlens[0]), int(w.cu_seqlens[1])
    want = brute_force(q[s:e], k[s:e], v[s:e], _cu([e - s]), True, w.softmax_scale)
    np.testing.assert_allclose(got[s:e], want, rtol=0, atol=1e-13)


# --- P7 isolation between packed sequences ------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_sequences_are_isolated(impl, causal):
    rng = np.random.default_rng(7)
    lengths = [9, 14, 6]
    N = sum(lengths)
    q, k, v = _rand(rng, N, 2, 4), _rand(rng, N, 2, 4), _rand(rng, N, 2, 4)
    cu = _cu(lengths)
    base = impl.attn_varlen(q, k, v, cu, causal, 0.5)
    q2, k2, v2 = q.copy(), k.copy(), v.copy()
    q2[9:23] += 3.0
    k2[9:23] *= -2.0
    v2[9:23] += 100.0
    out = impl.attn_varlen(q2, k2, v2, cu, causal, 0.5)
    assert np.array_equal(out[:9], base[:9])
    assert np.array_equal(out[23:], base[23:])
    assert not np.allclose(out[9:23], base[9:23])


# --- P8 causal prefix property -------------------------------------------------------------------
def test_causal_prefix_property(impl):
    rng = np.random.default_rng(8)
    L, n = 20, 8
    q, k, v = _rand(rng, L, 2, 4), _rand(rng, L, 2, 4), _rand(rng, L, 2, 4)
    full = impl.attn_varlen(q, k, v, _cu([L]), True, 0.5)
    trunc = impl.attn_varlen(q[:n], k[:n], v[:n], _cu([n]), True, 0.5)
    np.testing.assert_allclose(full[:n], trunc, rtol=0, atol=1e-14)
    # the bidirectional result does depend on later tokens
    fb = impl.attn_varlen(q, k, v, _cu([L]), False, 0.5)
    tb = impl.attn_varlen(q[:n], k[:n], v[:n], _cu([n]), False, 0.5)
    assert np.abs(fb[:n] - tb).max() > 1e-3


# --- P9 shift invariance --------------------------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_key_shift_invariance(impl, causal):
    rng = np.random.default_rng(9)
    L = 16
    q, k, v = _rand(rng, L, 1, 4), _rand(rng, L, 1, 4), _rand(rng, L, 1, 4)
    base = impl.attn_varlen(q, k, v, _cu([L]), causal, 0.5)
    shifted = impl.attn_varlen(q, k + np.array([3.0, -50.0, 7.0, 200.0]), v, _cu([L]), causal, 0.5)
    np.testing.assert_allclose(shifted, base, rtol=0, atol=1e-9)


# --- P10 linearity in V and convexity ---------------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_linear_in_v_and_convex(impl, causal):
    rng = np.random.default_rng(10)
    lengths = [13, 5]
    N = sum(lengths)
    q, k = _rand(rng, N, 2, 4), _rand(rng, N, 2, 4)
    v1, v2 = _rand(rng, N, 2, 4), _rand(rng, N, 2, 4)
    cu = _cu(lengths)
    o1 = impl.attn_varlen(q, k, v1, cu, causal, 0.5)
    o2 = impl.attn_varlen(q, k, v2, cu, causal, 0.5)
    o12 = impl.attn_varlen(q, k, v1 + 2.0 * v2, cu, causal, 0.5)
    np.testing.assert_allclose(o12, o1 + 2.0 * o2, rtol=0, atol=1e-12)
    for b in range(2):
        s, e = cu[b], cu[b + 1]
        for i in range(s, e):
            hi = i + 1 if causal else e
            lo_v, hi_v = v1[s:hi].min(axis=0), v1[s:hi].max(axis=0)
            assert (o1[i] >= lo_v - 1e-12).all() and (o1[i] <= hi_v + 1e-12).all()


# --- P11 GQA equals MHA with repeated KV heads ------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_gqa_equals_repeated_kv(impl, causal):
    rng = np.random.default_rng(11)
    L, Hq, Hkv, d = 10, 6, 2, 4
    q, k, v = _rand(rng, L, Hq, d), _rand(rng, L, Hkv, d), _rand(rng, L, Hkv, d)
    gqa = impl.attn_varlen(q, k, v, _cu([L]), causal, 0.5)
    mha = impl.attn_varlen(q, np.repeat(k, 3, axis=1), np.repeat(v, 3, axis=1), _cu([L]), causal, 0.5)
    assert np.array_equal(gqa, mha)
    # an interleaved (wrong) head mapping gives a different answer
    wrong = impl.attn_varlen(q, np.tile(k, (1, 3, 1)), np.tile(v, (1, 3, 1)), _cu([L]), causal, 0.5)
    assert np.abs(wrong - gqa).max() > 1e-3


# --- P12 scale plumbing ---------------------------------------------------------------------------------
def test_scale_zero_and_large(impl):
    rng = np.random.default_rng(12)
    L, d = 9, 4
    q, k, v = _rand(rng, L, 1, d), _rand(rng, L, 1, d), _rand(rng, L, 1, d)
    o0 = impl.attn_varlen(q, k, v, _cu([L]), False, 0.0)
    np.testing.assert_allclose(o0, np.broadcast_to(v.mean(axis=0), o0.shape), rtol=0, atol=1e-14)
    oc = impl.attn_varlen(q, k, v, _cu([L]), True, 0.0)
    np.testing.assert_allclose(oc[4], v[:5].mean(axis=0), rtol=0, atol=1e-14)
    # one dominant key: k_3 = q direction for every query, huge scale
    q[:] = np.array([1.0, 0.0, 0.0, 0.0])
    k[:] = 0.0
    k[3, 0, 0] = 1.0
    ob = impl.attn_varlen(q, k, v, _cu([L]), False, 1000.0)
    np.testing.assert_allclose(ob, np.broadcast_to(v[3], ob.shape), rtol=0, atol=1e-12)


# --- P13 visible-pair counts -----------------------------------------------------------------------------
def test_unmasked_pair_counts(impl):
    w = si.tiny(False)
    assert impl.unmasked_pairs(w.cu_seqlens, False) == 80434 == w.unmasked_pairs()
    assert impl.unmasked_pairs(w.cu_seqlens, True) == 40436 == si.tiny(True).unmasked_pairs()
    # paper's encode formula 4*B*T^2*H with H = heads*head_dim, on the CLIP-shaped batch
    c = si.clip_vit_encode()
    assert c.attention_flops() == 4 * 32 * 577 * 577 * (16 * 64)


# --- the two implementations agree with each other on a ragged GQA batch -----------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_numpy_and_c_agree(causal):
    rng = np.random.default_rng(13)
    lengths = [17, 64, 0, 100, 33]
    N = sum(lengths)
    q, k, v = _rand(rng, N, 4, 16), _rand(rng, N, 2, 16), _rand(rng, N, 2, 16)
    cu = _cu(lengths)
    a = reference.attn_varlen(q, k, v, cu, causal, 0.25)
    b = c_oracle.attn_varlen(q, k, v, cu, causal, 0.25)
    np.testing.assert_allclose(a, b, rtol=0, atol=1e-13)
    rows = [(0, 0), (16, 3), (17, 1), (80, 2), (N - 1, 3), (181, 0)]
    for fn in (reference.attn_rows, c_oracle.attn_rows):
        r = fn(q, k, v, cu, causal, 0.25, rows)
        for n, (t, h) in enumerate(rows):
            np.testing.assert_allclose(r[n], a[t, h], rtol=0, atol=1e-13)


def test_bf16_widening_is_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4049, 0x0001, 0x7F7F, 0x8000], dtype=np.uint16)
    got = reference.bf16_bits_to_f64(bits)
    want = np.array([0.0, 1.0, -1.0, 3.140625, 2.0 ** -133, (2 - 2.0 ** -7) * 2.0 ** 127, -0.0])
    assert np.array_equal(got, want)
    assert np.signbit(got[-1])


# --- P14 paged KV write --------------------------------------------------------------------------------------
def test_kv_write_oracle_gather_back_and_sentinel():
    w = si.tiny(True)
    _, kb, vb = si.make_qkv(w)
    kbits, vbits = si.bf16_bits(kb), si.bf16_bits(vb)
    slots, nb = si.make_slot_mapping(w.lengths, 16, spare_blocks=34, seed=0)
    assert nb == 64 and len(np.unique(slots)) == len(slots)
    kc0 = si.make_cache_sentinel(nb, 16, 2, 64, seed=1)
    vc0 = si.make_cache_sentinel(nb, 16, 2, 64, seed=2)
    kc, vc = reference.kv_cache_write(kbits, vbits, kc0, vc0, slots, 16)
    flat_k, flat_v = kc.reshape(nb * 16, 2, 64), vc.reshape(nb * 16, 2, 64)
    assert np.array_equal(flat_k[slots], kbits) and np.array_equal(flat_v[slots], vbits)
    untouched = np.ones(nb * 16, dtype=bool)
    untouched[slots] = False
    assert np.array_equal(flat_k[untouched], kc0.reshape(nb * 16, 2, 64)[untouched])
    assert np.array_equal(flat_v[untouched], vc0.reshape(nb * 16, 2, 64)[untouched])
    # block table structure: token i of a sequence sits at offset i % 16 of its block, and a
    # sequence's tokens 0..15 share one block
    assert (slots[:16] // 16 == slots[0] // 16).all() and (slots[:17] % 16 == np.arange(17) % 16).all()
    # skip convention
    s2 = slots.copy()
    s2[5] = -1
    kc2, _ = reference.kv_cache_write(kbits, vbits, kc0, vc0, s2, 16)
    assert np.array_equal(kc2.reshape(nb * 16, 2, 64)[slots[5]], kc0.reshape(nb * 16, 2, 64)[slots[5]])
    # a permutation followed by its inverse reproduces K
    perm = np.random.default_rng(0).permutation(len(slots))
    c1, _ = reference.kv_cache_write(kbits, vbits, np.zeros((28, 16, 2, 64), np.uint16), np.zeros((28, 16, 2, 64), np.uint16),
                                     perm[: len(slots)].astype(np.int64), 16)
    assert np.array_equal(c1.reshape(-1, 2, 64)[perm], kbits)


# --- paged image cache -----------------------------------------------------------------------
def test_page_cache_write_then_gather_is_identity_and_leaves_the_rest():
    rng = np.random.default_rng(21)
    b = si.ImageCacheBatch("t", [5, 12, 1], 16, page_rows=8)
    slots, pages = si.make_slot_mapping(b.tokens, b.page_rows, spare_blocks=2, seed=4)
    rows = rng.integers(0, 1 << 16, size=(b.n_rows, b.hidden), dtype=np.uint16)
    cache0 = rng.integers(0, 1 << 16, size=(pages, b.page_rows, b.hidden), dtype=np.uint16)
    cache = reference.page_cache_write(rows, cache0, slots)
    flat, flat0 = cache.reshape(-1, b.hidden), cache0.reshape(-1, b.hidden)
    assert np.array_equal(flat[slots], rows)                       # every row landed in its slot
    untouched = np.setdiff1d(np.arange(flat.shape[0]), slots)
    assert np.array_equal(flat[untouched], flat0[untouched])      # nothing else changed
    back = reference.page_cache_gather(cache, slots, np.zeros_like(rows))
    assert np.array_equal(back, rows)                              # gather o write = identity


def test_page_cache_hand_case_and_skips():
    # two pages of two rows, rows of two values; packed rows 0..2 go to slots 3, 0 and "skip"
    cache0 = np.array([[[1, 2], [3, 4]], [[5, 6], [7, 8]]], dtype=np.uint16)
    rows = np.array([[10, 11], [20, 21], [30, 31]], dtype=np.uint16)
    slots = np.array([3, 0, -1])
    cache = reference.page_cache_write(rows, cache0, slots)
    assert cache.tolist() == [[[20, 21], [3, 4]], [[5, 6], [10, 11]]]
    out = reference.page_cache_gather(cache0, slots, np.array([[0, 0], [0, 0], [9, 9]], dtype=np.uint16))
    assert out.tolist() == [[7, 8], [1, 2], [9, 9]]               # the skipped row keeps its contents
    with pytest.raises(ValueError):
        reference.page_cache_write(rows, cache0, np.array([4, 0, 1]))
