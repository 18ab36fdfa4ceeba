"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

import paper_2505_12658_amd as hydra

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hydra.library_path()):
        from paper_2505_12658_amd import build

        build.build()
    return hydra.load_library()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "hydra_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hydra_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_symbols()
    assert names == ["hydra_attn_build_worklist", "hydra_attn_paged_fwd", "hydra_attn_paged_workspace_bytes", "hydra_attn_varlen_fwd", "hydra_attn_varlen_fwd_prebuilt", "hydra_attn_varlen_fwd_shared", "hydra_attn_varlen_fwd_static", "hydra_attn_workspace_bytes",
                     "hydra_kv_cache_write", "hydra_page_cache_gather", "hydra_page_cache_write", "hydra_status_string"]
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings(lib):
    assert hydra.hydra_status_string(0) == "ok"
    assert len({hydra.hydra_status_string(i) for i in range(5)}) == 5
    assert hydra.hydra_status_string(99) == "unknown status"


def test_workspace_bytes(lib):
    assert hydra.hydra_attn_workspace_bytes(4, 438, 257, 2, 2, 64) > 0
    assert hydra.hydra_attn_workspace_bytes(4, 438, 257, 3, 2, 64) == 0  # heads not divisible
    assert hydra.hydra_attn_workspace_bytes(4, 438, 257, 2, 2, 96) == 0  # unsupported head_dim
    assert hydra.hydra_attn_workspace_bytes(-1, 438, 257, 2, 2, 64) == 0
    # grows with tokens and heads
    a = hydra.hydra_attn_workspace_bytes(48, 30000, 1312, 28, 4, 128)
    b = hydra.hydra_attn_workspace_bytes(48, 60000, 1312, 28, 4, 128)
    assert b > a > 0


def _attn(lib, q=16, k=16, v=16, out=16, qs=128, ks=128, vs=128, cu=16, batch=1, total=8, max_len=8, hq=2, hkv=2, d=64, causal=0,
          scale=0.125, ws=16, ws_bytes=1 << 20, stream=None):
    # fake, never dereferenced device addresses: every case below must be rejected on the host
    return lib.hydra_attn_varlen_fwd(q, k, v, out, qs, ks, vs, cu, batch, total, max_len, hq, hkv, d, causal, scale, ws, ws_bytes, stream)


def test_attn_argument_errors(lib):
    INVALID, UNSUPPORTED, WORKSPACE = 1, 2, 3
    assert _attn(lib, q=None) == INVALID
    assert _attn(lib, out=None) == INVALID
    assert _attn(lib, cu=None) == INVALID
    assert _attn(lib, batch=-1) == INVALID
    assert _attn(lib, total=-5) == INVALID
    assert _attn(lib, hq=3, hkv=2) == INVALID
    assert _attn(lib, hkv=0) == INVALID
    assert _attn(lib, d=96) == UNSUPPORTED
    assert _attn(lib, d=0) == UNSUPPORTED
    assert _attn(lib, q=8) == INVALID  # misaligned
    assert _attn(lib, qs=132) == INVALID  # stride not a multiple of 8 elements
    assert _attn(lib, ks=64) == INVALID  # stride smaller than a token row
    assert _attn(lib, scale=-1.0) == INVALID
    assert _attn(lib, scale=float("nan")) == INVALID
    assert _attn(lib, scale=float("inf")) == INVALID
    assert _attn(lib, max_len=0) == INVALID
    assert _attn(lib, ws=None) == WORKSPACE
    assert _attn(lib, ws_bytes=8) == WORKSPACE
    assert _attn(lib, ws=24) == WORKSPACE  # misaligned workspace
    # K/V byte offsets inside one sequence beyond 31 bits: refused by the combined call before its first
    # launch (a launch attempt would fail differently here: there is no device, and the addresses are fake)
    big = hydra.hydra_attn_workspace_bytes(1, 1 << 20, 1 << 20, 2, 2, 64)
    assert _attn(lib, total=1 << 20, max_len=1 << 20, ks=2048, ws_bytes=big) == UNSUPPORTED
    assert _attn(lib, total=1 << 20, max_len=1 << 20, vs=1 << 20, ws_bytes=big) == UNSUPPORTED
    assert lib.hydra_attn_varlen_fwd_prebuilt(16, 16, 16, 16, 128, 2048, 128, 16, 1, 1 << 20, 1 << 20, 2, 2, 64, 0, 0.125, 16, big, None) == UNSUPPORTED
    # empty batches succeed without touching any pointer
    assert _attn(lib, batch=0, q=None, k=None, v=None, out=None, cu=None, ws=None) == 0
    assert _attn(lib, total=0, q=None, k=None, v=None, out=None, cu=None, ws=None) == 0


def test_shared_attn_argument_errors(lib):
    """The variant for two-stream callers checks its own argument before anything else and otherwise
    validates like the plain call (fake addresses: every case is rejected on the host)."""
    def call(per_cu, q=16, d=64, ws_bytes=1 << 20):
        return lib.hydra_attn_varlen_fwd_shared(q, 16, 16, 16, 128, 128, 128, 16, 1, 8, 8, 2, 2, d, 0, 0.125, 16, ws_bytes, per_cu, None)
    assert call(0) == 1 and call(-3) == 1
    assert call(1, q=None) == 1
    assert call(1, d=96) == 2
    assert call(2, ws_bytes=8) == 3


def test_static_scratch_attn_argument_errors(lib):
    """The allocation-free variant: same host-side checks, and a batch whose work list does not fit its static
    array is refused before anything is launched (fake addresses throughout)."""
    def call(q=16, batch=1, total=8, max_len=8, hq=2, hkv=2, d=64, scale=0.125):
        return lib.hydra_attn_varlen_fwd_static(q, 16, 16, 16, hq * d, hkv * d, hkv * d, 16, batch, total, max_len, hq, hkv, d, 1, scale, None)
    limit = 4 << 20
    assert hydra.hydra_attn_workspace_bytes(4096, 262144, 4096, 32, 8, 128) <= limit < hydra.hydra_attn_workspace_bytes(4096, 1 << 20, 4096, 32, 8, 128)
    assert call(batch=4096, total=1 << 20, max_len=4096, hq=32, hkv=8, d=128) == 3
    assert call(d=96) == 2
    assert call(hq=3) == 1
    assert call(batch=-1) == 1
    assert call(batch=0, q=None) == 0
    assert call(batch=0, q=None, scale=-1.0) == 1


def _kvw(lib, k=16, v=16, ks=128, vs=128, kc=16, vc=16, slots=16, total=4, hkv=2, d=64, bs=16, nb=4, stream=None):
    return lib.hydra_kv_cache_write(k, v, ks, vs, kc, vc, slots, total, hkv, d, bs, nb, stream)


def test_kv_write_argument_errors(lib):
    INVALID, UNSUPPORTED = 1, 2
    assert _kvw(lib, k=None) == INVALID
    assert _kvw(lib, vc=None) == INVALID
    assert _kvw(lib, slots=None) == INVALID
    assert _kvw(lib, total=-1) == INVALID
    assert _kvw(lib, bs=0) == INVALID
    assert _kvw(lib, hkv=0) == INVALID
    assert _kvw(lib, nb=-1) == INVALID
    assert _kvw(lib, hkv=1, d=4) == UNSUPPORTED  # row not a multiple of 16 bytes
    assert _kvw(lib, kc=4) == INVALID
    assert _kvw(lib, ks=64) == INVALID
    assert _kvw(lib, vs=132) == INVALID
    assert _kvw(lib, total=0, k=None, v=None, kc=None, vc=None, slots=None) == 0


def test_paged_attn_argument_errors(lib):
    """Every error is detected on the host before any launch: the pointers here are never dereferenced."""
    import ctypes

    P = ctypes.c_void_p(0x1000)
    f32 = ctypes.c_float

    def call(q=P, out=P, stride=28 * 128, kc=P, vc=P, bt=P, mb=8, cu=P, kl=P, batch=2, total=10, mq=8, hq=28, hkv=4, d=128, bs=16, nb=64,
             scale=0.1, ws=None, wsb=0):
        return lib.hydra_attn_paged_fwd(q, out, stride, kc, vc, bt, mb, cu, kl, batch, total, mq, hq, hkv, d, bs, nb, f32(scale), ws, wsb, None)

    assert call(batch=0) == 0 and call(total=0) == 0            # nothing to do: OK without a launch
    assert call(q=None) == 1 and call(bt=None) == 1 and call(kl=None) == 1
    assert call(q=ctypes.c_void_p(0x1008)) == 1                 # misaligned
    assert call(stride=28 * 128 - 8) == 1 and call(stride=28 * 128 + 4) == 1
    assert call(hq=28, hkv=5) == 1 and call(batch=-1) == 1 and call(mq=0) == 1 and call(mb=0) == 1 and call(nb=0) == 1
    assert call(scale=-1.0) == 1 and call(scale=float("inf")) == 1 and call(scale=float("nan")) == 1
    assert call(d=96) == 2 and call(bs=12) == 2 and call(bs=0) == 2 and call(batch=70000) == 2
    assert call(nb=1 << 27, bs=16) == 2                         # cache rows are counted in 31 bits
    assert call(ws=None, wsb=64) == 3 and call(ws=ctypes.c_void_p(0x1004), wsb=64) == 3
    # workspace size: nothing for a batch that fills the chip or for short contexts, something for a small batch of long contexts
    assert lib.hydra_attn_paged_workspace_bytes(1024, 4, 128, 64, 16) == 0
    assert lib.hydra_attn_paged_workspace_bytes(8, 4, 128, 16, 16) == 0
    assert lib.hydra_attn_paged_workspace_bytes(8, 4, 128, 1024, 16) == 8 * 4 * 16 * (64 + 32 * 128) * 4
    assert lib.hydra_attn_paged_workspace_bytes(0, 4, 128, 1024, 16) == 0 and lib.hydra_attn_paged_workspace_bytes(8, 4, 96, 1024, 16) == 0


def test_page_cache_argument_errors(lib):
    import ctypes

    P = ctypes.c_void_p(0x1000)
    for fn, order in ((lib.hydra_page_cache_write, lambda rows, stride, cache, slots: (rows, stride, cache, slots)),
                      (lib.hydra_page_cache_gather, lambda rows, stride, cache, slots: (cache, slots, rows, stride))):
        def call(rows=P, stride=4096, cache=P, slots=P, n=10, row=4096, num=100):
            return fn(*order(rows, stride, cache, slots), n, row, num, None)

        assert call(n=0) == 0
        assert call(rows=None) == 1 and call(cache=None) == 1 and call(slots=None) == 1
        assert call(rows=ctypes.c_void_p(0x1004)) == 1 and call(stride=4088) == 1 and call(stride=4100) == 1
        assert call(n=-1) == 1 and call(row=0) == 1
        assert call(row=4100, stride=4104) == 2


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2505_12658_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(ImportError):
        binding.load_library()
