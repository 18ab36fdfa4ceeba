"""The entry points recorded into a HIP graph (torch.cuda.CUDAGraph) and replayed: a serving loop records one
layer's attention once and replays it per step.  The library allocates nothing, clears nothing with memset and
reads every length on the device, so a replay must do exactly what the eager call does on the buffers' current
contents.  Every replay is compared bit for bit with an eager call on the same contents (the kernels are
deterministic), with eager work and synchronisations between the replays, and once against the oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import c_oracle, reference

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 2e-2, 2e-3


def _f64(t):
    return reference.bf16_bits_to_f64(si.bf16_bits(t))


def test_packed_attention_and_kv_write_replayed_from_a_graph():
    """Static-scratch attention call + KV scatter in one graph; three replays, new activations before each."""
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    w = si.custom([300, 17, 0, 640, 129, 64, 257, 1], 8, 2, 128, True, seed=31, kv_cache=True)
    slots, num_blocks = si.make_slot_mapping(w.lengths, 16, seed=31)
    cu = torch.from_numpy(w.cu_seqlens).to(dev)
    sm = torch.from_numpy(slots).to(dev)
    q, k, v = (t.to(dev) for t in si.make_qkv(w))
    out = torch.zeros_like(q)
    kc = torch.zeros((num_blocks, 16, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
    vc = torch.zeros_like(kc)

    def step():
        hydra.hydra_attn_varlen_fwd_static(q, k, v, cu, w.max_seqlen, True, w.softmax_scale, out)
        hydra.hydra_kv_cache_write(k, v, kc, vc, sm)

    step()  # (first use outside the capture: the library looks up its static array's address once per device)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    for rep in range(3):
        fresh = si.make_qkv(w, seed=100 + rep)
        for dst, src in zip((q, k, v), fresh):
            dst.copy_(src.to(dev))
        out.fill_(float("nan"))
        kc.zero_()
        vc.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got, got_kc, got_vc = out.clone(), kc.clone(), vc.clone()
        out.fill_(float("nan"))
        kc.zero_()
        vc.zero_()
        step()
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), out.view(torch.int16)), rep
        assert torch.equal(got_kc.view(torch.int16), kc.view(torch.int16)) and torch.equal(got_vc.view(torch.int16), vc.view(torch.int16)), rep
        if rep == 2:
            want = c_oracle.attn_varlen(_f64(fresh[0]), _f64(fresh[1]), _f64(fresh[2]), w.cu_seqlens, True, w.softmax_scale)
            diff = np.abs(_f64(got) - want)
            assert np.isfinite(diff).all() and diff.max() <= MAX_ABS and diff.mean() <= MEAN_ABS


@pytest.mark.parametrize("split", [False, True], ids=["one_workgroup_per_context", "contexts_split"])
def test_decode_steps_replayed_from_a_graph(split):
    """One recorded decode step over the paged cache, replayed while the contexts grow: the kernel reads the
    lengths and the block table from device memory at replay time.  With a workspace the long contexts are split
    over workgroups and merged by a second kernel inside the graph."""
    import paper_2505_12658_amd as hydra

    dev = torch.device("cuda:0")
    base = [2500, 40, 1300, 700] if split else [300, 40, 130, 257, 64, 1]
    steps = 3
    h_last = si.HybridBatch("decode", [1] * len(base), [b + steps for b in base], 8, 2, 128, seed=41)
    # the cache and the tables are those of the LAST step; earlier steps see a prefix of every context
    _, kc, vc, tables = si.make_paged_inputs(h_last)
    kcd, vcd, td = kc.to(dev), vc.to(dev), torch.from_numpy(tables).to(dev)
    cu = torch.from_numpy(h_last.cu_seqlens_q).to(dev)
    kv = torch.zeros(len(base), dtype=torch.int32, device=dev)
    q = torch.zeros((len(base), 8, 128), dtype=torch.bfloat16, device=dev)
    out = torch.zeros_like(q)
    need = hydra.hydra_attn_paged_workspace_bytes(len(base), 2, 128, tables.shape[1], 16)
    assert (need > 0) == split
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

    def step():
        hydra.hydra_attn_paged_fwd(q, kcd, vcd, td, cu, kv, 1, h_last.softmax_scale, out=out, workspace=ws)

    kv.copy_(torch.tensor(base, dtype=torch.int32))
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    for s in range(1, steps + 1):
        lens = [b + s for b in base]
        h = si.HybridBatch("decode", [1] * len(base), lens, 8, 2, 128, seed=41)
        q_new = si.make_paged_inputs(h)[0]  # (only the new tokens' queries are taken from this draw)
        q.copy_(q_new.to(dev))
        kv.copy_(torch.tensor(lens, dtype=torch.int32))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = out.clone()
        out.fill_(float("nan"))
        step()
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), out.view(torch.int16)), s
        want = reference.attn_paged(_f64(q_new), _f64(kc), _f64(vc), tables, h.cu_seqlens_q, h.kv_lens, h.softmax_scale)
        diff = np.abs(_f64(got) - want)
        assert np.isfinite(diff).all() and diff.max() <= MAX_ABS and diff.mean() <= MEAN_ABS
