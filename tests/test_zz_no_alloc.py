"""The allocation-free attention entry point (work list in the library's static device array) against the
plain entry point with a caller-provided workspace: same kernels, same inputs, so the outputs must agree bit
for bit; two calls in a row on the shared array, the second with a smaller batch, then a larger one again."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import c_oracle, reference

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def _f64(t):
    return reference.bf16_bits_to_f64(si.bf16_bits(t))


def test_static_scratch_entry_point_matches_plain_call():
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    cases = [
        si.custom([300, 17, 0, 640, 129, 64, 1000, 1], 8, 2, 128, True, seed=21),   # first call
        si.custom([45, 200], 4, 4, 64, False, seed=22),                             # smaller: stale list entries behind it
        si.custom([70, 333, 33], 2, 2, 80, True, seed=23),
        si.custom([900, 31, 512, 100, 257, 64], 14, 2, 128, True, seed=24),         # larger again
    ]
    for w in cases:
        q, k, v = si.make_qkv(w)
        qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
        cu = torch.from_numpy(w.cu_seqlens).to(dev)
        plain = hydra.hydra_attn_varlen_fwd(qd, kd, vd, cu, w.max_seqlen, w.causal, w.softmax_scale)
        got = torch.full_like(qd, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(dev)
        hydra.hydra_attn_varlen_fwd_static(qd, kd, vd, cu, w.max_seqlen, w.causal, w.softmax_scale, got)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(dev) == before
        assert torch.equal(got.view(torch.int16), plain.view(torch.int16)), w.lengths
        want = c_oracle.attn_varlen(_f64(q), _f64(k), _f64(v), w.cu_seqlens, w.causal, w.softmax_scale)
        diff = np.abs(_f64(got) - want)
        assert np.isfinite(diff).all() and diff.max() <= MAX_ABS and diff.mean() <= MEAN_ABS


def test_static_scratch_entry_point_refuses_oversized_batches():
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    n = 300_000  # sequences of one token each: their work list is beyond the static array
    assert hydra.hydra_attn_workspace_bytes(n, n, 1, 2, 2, 64) > (4 << 20)
    q = torch.zeros((n, 2, 64), dtype=torch.bfloat16, device=dev)
    kv = torch.zeros((n, 2, 64), dtype=torch.bfloat16, device=dev)
    cu = torch.arange(0, n + 1, dtype=torch.int32, device=dev)
    out = torch.full((n, 2, 64), 3.0, dtype=torch.bfloat16, device=dev)
    with pytest.raises(hydra.HydraError) as e:
        hydra.hydra_attn_varlen_fwd_static(q, kv, kv, cu, 1, True, 0.125, out)
    assert e.value.status == 3
    torch.cuda.synchronize()
    assert (out == 3.0).all()
