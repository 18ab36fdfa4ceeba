#!/usr/bin/env python3
"""Benchmark of the packed varlen attention + paged KV write path on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: the device work-list build,
the fused attention kernel and (for prefill workloads) the paged KV scatter.  Inputs are resident
in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

PEAK_BF16_TFLOPS = 2516.6  # MI355X dense bf16 MFMA, 256 CUs x 4096 FLOP/clk x 2.4 GHz
PEAK_HBM_GBS = 8000.0
CALIBRATION_COPY_BYTES = 1 << 30
HEADLINE = "qwen2vl_7b_prefill"
OTHERS = ["clip_vit_l14_336_encode", "llava15_7b_prefill", "qwen2vl_vit_encode"]


def profile_figures(workload: str):
    """Counter figures of the attention kernel on one workload, from the tracked rocprofv3 summary
    profiles/attn_fwd_<workload>.md: its `figures:` line is a JSON object written together with the tables
    (HBM bytes per launch from the FETCH_SIZE / WRITE_SIZE passes scaled by the calibration copy, share of
    cycles with the matrix pipe busy, kernel duration under the trace, the commit the profile was taken at).
    Counters cannot be read inside a timed run, so the bench line carries them from there, with their source."""
    path = os.path.join(ROOT, "profiles", f"attn_fwd_{workload}.md")
    try:
        for line in open(path):
            if line.startswith("figures: "):
                fig = json.loads(line[len("figures: "):])
                fig["source"] = os.path.relpath(path, ROOT)
                return fig
    except (OSError, ValueError):
        pass
    return None


class DeviceBatch:
    """One workload resident on the GPU, with `n_sets` rotating copies of every buffer so that
    consecutive steps do not find their Q/K/V/O in the 256 MB last-level cache."""

    def __init__(self, w: si.Workload, n_sets: int, dev):
        import paper_2505_12658_amd as hydra

        self.hydra = hydra
        self.w = w
        self.dev = dev
        q, k, v = si.make_qkv(w)
        self.host_qkv = (q, k, v)
        self.cu = torch.from_numpy(w.cu_seqlens).to(dev)
        self.sets = []
        for i in range(n_sets):
            s = {"q": q.to(dev), "k": k.to(dev), "v": v.to(dev), "out": torch.empty(q.shape, dtype=torch.bfloat16, device=dev)}
            if w.kv_cache:
                slots, nb = si.make_slot_mapping(w.lengths, w.block_size, spare_blocks=8, seed=w.seed + i)
                s["slots"] = torch.from_numpy(slots).to(dev)
                s["k_cache"] = torch.zeros((nb, w.block_size, w.n_kv_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
                s["v_cache"] = torch.zeros_like(s["k_cache"])
            self.sets.append(s)
        need = hydra.hydra_attn_workspace_bytes(w.batch, w.total_tokens, w.max_seqlen, w.n_q_heads, w.n_kv_heads, w.head_dim)
        self.ws = torch.empty(need, dtype=torch.uint8, device=dev)
        # The KV scatter does not depend on the attention of the same batch (both only read K/V), so it can go
        # to a second stream (measured: the step is as long as on one stream).
        self.side = torch.cuda.Stream(device=dev) if w.kv_cache else None

    def step(self, i: int, events=None, two_streams=False, workgroups_per_cu=None):
        """One pass of the whole path over one batch.  two_streams: the KV scatter goes to the side
        stream, behind the attention launch (call drain() before reading the clock).  workgroups_per_cu:
        the attention kernel leaves room on every compute unit for another stream's kernels."""
        h, w, s = self.hydra, self.w, self.sets[i % len(self.sets)]
        h.hydra_attn_build_worklist(self.cu, w.total_tokens, w.max_seqlen, w.n_q_heads, w.n_kv_heads, w.head_dim, w.causal, self.ws)
        if events is not None:
            events[0].record()
        if workgroups_per_cu is None:
            h.hydra_attn_varlen_fwd_prebuilt(s["q"], s["k"], s["v"], self.cu, w.max_seqlen, w.causal, w.softmax_scale, s["out"], self.ws)
        else:
            h.hydra_attn_varlen_fwd_shared(s["q"], s["k"], s["v"], self.cu, w.max_seqlen, w.causal, w.softmax_scale, s["out"], self.ws,
                                           workgroups_per_cu)
        if events is not None:
            events[1].record()
        if w.kv_cache:
            if two_streams:
                h.hydra_kv_cache_write(s["k"], s["v"], s["k_cache"], s["v_cache"], s["slots"], stream=self.side)
            else:
                h.hydra_kv_cache_write(s["k"], s["v"], s["k_cache"], s["v_cache"], s["slots"])
            if events is not None:
                events[2].record()


SETTLE_SECONDS = 0.15


def settle(launch, seconds: float = SETTLE_SECONDS):
    """Keeps the device under the load about to be measured until its clocks have settled: after any idle
    stretch (input generation on the host, uploads) the first ~50 ms of kernels run up to 20 % slower than
    the steady state.  Untimed; the stated warm-up steps and the timed steps follow without a gap."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    i = 0
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            launch(i)
            i += 1
        torch.cuda.synchronize()


def time_steps(batch: DeviceBatch, steps: int, warmup: int, two_streams: bool = False):
    """Wall-clock over exactly `steps` steps, bracketed by device synchronisation (all streams)."""
    settle(lambda i: batch.step(i, two_streams=two_streams))
    for i in range(warmup):
        batch.step(i, two_streams=two_streams)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        batch.step(i, two_streams=two_streams)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps


def time_kernels(batch: DeviceBatch, steps: int, hot_cache: bool = False):
    """Same steps again with HIP events (on the launch stream) around the attention kernel and the
    KV scatter.  Returns per-step attention-kernel and KV-write durations in seconds.  hot_cache: every step
    uses the same buffer set, so whatever of Q/K/V/O fits the 256 MB last-level cache is found there."""
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    pick = (lambda i: 0) if hot_cache else (lambda i: i)
    settle(lambda i: batch.step(pick(i)))
    for i in range(steps):
        batch.step(pick(i), evs[i])
    torch.cuda.synchronize()
    attn = np.array([e[0].elapsed_time(e[1]) for e in evs]) * 1e-3
    kvw = np.array([e[1].elapsed_time(e[2]) for e in evs]) * 1e-3 if batch.w.kv_cache else None
    return attn, kvw


def cpu_baseline(w: si.Workload, host_qkv, budget_s: float = 15.0):
    """The fp64 oracle as it stands, on the host cores, on a bounded sample of the same workload:
    whole sequences (all heads) taken in a seeded shuffled order until the estimated time reaches
    the budget."""
    from oracle import c_oracle, reference

    q, k, v = (reference.bf16_bits_to_f64(si.bf16_bits(t)) for t in host_qkv)
    cu = w.cu_seqlens
    order = np.random.default_rng(1).permutation(w.batch)

    def sub_batch(seqs):
        idx = np.concatenate([np.arange(cu[b], cu[b + 1]) for b in seqs])
        lens = [int(cu[b + 1] - cu[b]) for b in seqs]
        return q[idx], k[idx], v[idx], np.concatenate([[0], np.cumsum(lens)]).astype(np.int32), lens

    def flops(lens):
        pairs = sum(L * (L + 1) // 2 for L in lens) if w.causal else sum(L * L for L in lens)
        return 4 * w.head_dim * w.n_q_heads * pairs

    # calibration on the shortest sequence
    shortest = [int(np.argmin(np.diff(cu)))]
    qs, ks, vs, cus, lens = sub_batch(shortest)
    t0 = time.perf_counter()
    _, threads = c_oracle.attn_varlen(qs, ks, vs, cus, w.causal, w.softmax_scale, return_threads=True)
    rate = flops(lens) / max(time.perf_counter() - t0, 1e-6)
    chosen, total = [], 0.0
    for b in order:
        f = flops([int(cu[b + 1] - cu[b])])
        if chosen and (total + f) / rate > budget_s:
            break
        chosen.append(int(b))
        total += f
    qs, ks, vs, cus, lens = sub_batch(chosen)
    t0 = time.perf_counter()
    _, threads = c_oracle.attn_varlen(qs, ks, vs, cus, w.causal, w.softmax_scale, return_threads=True)
    dt = time.perf_counter() - t0
    return {
        "value": flops(lens) / dt * 1e-12,
        "unit": "TFLOP/s",
        "cores": int(threads),
        "kind": "oracle",
        "sample": f"{len(chosen)} of {w.batch} sequences ({sum(lens)} of {w.total_tokens} tokens), all {w.n_q_heads} heads, "
                  f"{flops(lens):.3e} FLOP in {dt:.2f} s, fp64 plain C + OpenMP",
        "seconds": dt,
    }


def dual_stream(dev, n_sets: int, steps: int, encode: str = "qwen2vl_vit_encode", prefill: str = HEADLINE):
    """The paper runs the vision encoder and the language model of one instance on two streams
    (Section 4.2, the paragraph on dual-stream parallelism; measured in Section 5.5).  Here: encode attention steps on one stream and prefill steps (attention + KV scatter)
    on another, launched together, against the same steps launched one after the other."""
    we, wp = si.WORKLOADS[encode](), si.WORKLOADS[prefill]()
    be, bp = DeviceBatch(we, n_sets, dev), DeviceBatch(wp, n_sets, dev)
    se, sp = torch.cuda.Stream(device=dev), torch.cuda.Stream(device=dev)

    def run(concurrent: bool):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            with torch.cuda.stream(se):
                be.step(i)
            if not concurrent:
                sp.wait_stream(se)
            with torch.cuda.stream(sp):
                bp.step(i)
            if not concurrent:
                se.wait_stream(sp)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    for c in (False, True):
        run(c)  # warm-up
    seq, con = run(False), run(True)
    flops = we.attention_flops() + wp.attention_flops()
    report = {"encode": encode, "prefill": prefill, "steps": steps, "ms_sequential": seq * 1e3, "ms_two_streams": con * 1e3,
              "tflops_sequential": flops / seq * 1e-12, "tflops_two_streams": flops / con * 1e-12, "speedup": seq / con}
    del bp
    report["encode_decode"] = encode_beside_decode(dev, be, se, sp, n_sets, steps)
    return report


def encode_beside_decode(dev, be: DeviceBatch, se, sd, n_sets: int, steps: int, n_requests: int = 256, kv_len: int = 1024):
    """The pairing the paper's two-stream experiment uses (Section 5.5: encode beside decode, context length 1024):
    encode attention (matrix-bound) on one stream, decode attention over the paged cache (memory-bound) on the
    other, as many decode launches per encode launch as take about the same time.  Three ways: one after the
    other; launched together with the encode kernel at its own size (its persistent workgroups hold every
    compute unit's registers, so the decode kernel only gets what drains); launched together with the encode
    kernel at one workgroup per compute unit (hydra_attn_varlen_fwd_shared), so that both run on every compute unit."""
    import paper_2505_12658_amd as hydra

    we = be.w
    h = si.HybridBatch("qwen2vl_7b_decode", [1] * n_requests, [kv_len] * n_requests, 28, 4, 128, seed=3)
    sets = []
    for i in range(n_sets):
        q, kc, vc, tables = si.make_paged_inputs(h)
        sets.append((q.to(dev), kc.to(dev), vc.to(dev), torch.from_numpy(tables).to(dev), torch.empty(q.shape, dtype=torch.bfloat16, device=dev)))
    cu = torch.from_numpy(h.cu_seqlens_q).to(dev)
    kv_lens = torch.tensor(h.kv_lens, dtype=torch.int32, device=dev)

    def decode(i):
        q, kc, vc, tables, out = sets[i % n_sets]
        hydra.hydra_attn_paged_fwd(q, kc, vc, tables, cu, kv_lens, 1, h.softmax_scale, out=out, use_workspace=False)

    def run(mode: str, n_dec: int, per_cu=None):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            if mode != "decode":
                with torch.cuda.stream(se):
                    be.step(i, workgroups_per_cu=per_cu)
            if mode == "sequential":
                sd.wait_stream(se)
            if mode != "encode":
                with torch.cuda.stream(sd):
                    for j in range(n_dec):
                        decode(i * n_dec + j)
            if mode == "sequential":
                se.wait_stream(sd)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    run("encode", 1), run("decode", 1)  # warm-up
    t_enc, t_dec = run("encode", 1), run("decode", 1)
    n_dec = max(1, round(t_enc / t_dec))
    for args in (("sequential", n_dec), ("together", n_dec), ("together", n_dec, 1)):
        run(*args)
    t_dec_n, seq, con, shared = run("decode", n_dec), run("sequential", n_dec), run("together", n_dec), run("together", n_dec, 1)
    return {"encode": we.name, "decode": f"{n_requests} requests x {kv_len} tokens of context, Qwen2-VL-7B heads", "decode_launches_per_encode_launch": n_dec,
            "steps": steps, "ms_encode_alone": t_enc * 1e3, "ms_decode_alone": t_dec_n * 1e3, "ms_encode_alone_one_workgroup_per_cu": run("encode", 1, 1) * 1e3,
            "ms_sequential": seq * 1e3, "ms_two_streams": con * 1e3, "ms_two_streams_shared_cus": shared * 1e3,
            "speedup_two_streams": seq / con, "speedup_two_streams_shared_cus": seq / shared}


def paged_attention(dev, n_sets: int, steps: int):
    """Attention over the paged KV cache (hydra_attn_paged_fwd) on the hybrid batch of decode requests and
    prefill chunks, on its decode requests alone, and on 8 decode requests with 16 384 tokens of context each
    (few requests, long contexts: the library splits every context over several workgroups).  HIP events on the launch stream around every launch;
    rotating buffer sets.  Bound: HBM (the batch's arithmetic intensity is below the ridge point)."""
    import paper_2505_12658_amd as hydra

    full = si.qwen2vl_hybrid()
    decode_only = si.HybridBatch("qwen2vl_7b_decode_only", [q for q in full.q_lens if q == 1], [k for q, k in zip(full.q_lens, full.kv_lens) if q == 1],
                                 full.n_q_heads, full.n_kv_heads, full.head_dim, seed=full.seed)
    long_decode = si.HybridBatch("qwen2vl_7b_long_context_decode", [1] * 8, [16384] * 8, full.n_q_heads, full.n_kv_heads, full.head_dim, seed=full.seed)
    report = []
    for h in (full, decode_only, long_decode):
        sets = []
        for i in range(n_sets):
            q, kc, vc, tables = si.make_paged_inputs(h)
            sets.append((q.to(dev), kc.to(dev), vc.to(dev), torch.from_numpy(tables).to(dev), torch.empty(q.shape, dtype=torch.bfloat16, device=dev)))
        cu = torch.from_numpy(h.cu_seqlens_q).to(dev)
        kv_lens = torch.tensor(h.kv_lens, dtype=torch.int32, device=dev)

        need = hydra.hydra_attn_paged_workspace_bytes(h.batch, h.n_kv_heads, h.head_dim, sets[0][3].shape[1], h.block_size)
        ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

        def launch(i):
            q, kc, vc, tables, out = sets[i % n_sets]
            hydra.hydra_attn_paged_fwd(q, kc, vc, tables, cu, kv_lens, h.max_q_len, h.softmax_scale, out=out, workspace=ws)

        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        settle(launch)
        for i, (e0, e1) in enumerate(evs):
            e0.record()
            launch(i)
            e1.record()
        torch.cuda.synchronize()
        t = np.array([e0.elapsed_time(e1) for e0, e1 in evs]) * 1e-3
        avg = float(t.mean())
        gbs = h.attention_min_bytes() / avg * 1e-9
        report.append({"workload": h.name, "requests": h.batch, "new_tokens": h.total_q, "context_tokens": int(sum(h.kv_lens)),
                       "kernel": "attn_paged_kernel", "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": gbs / PEAK_HBM_GBS, "avg_kernel_us": avg * 1e6, "min_kernel_us": float(t.min()) * 1e6,
                       "algorithmic_bytes": h.attention_min_bytes(), "attention_flops": h.attention_flops(),
                       "tflops": h.attention_flops() / avg * 1e-12})
        del sets
        torch.cuda.empty_cache()
    return report


def image_cache(dev, steps: int, n_sets: int = 3):
    """Paged image cache (hydra_page_cache_write / hydra_page_cache_gather): encoder output rows into cache pages
    and back.  HIP events around every launch; bytes = each row read once and written once + its slot.  `frac` is
    the cold figure: the launches rotate over `n_sets` separate sets of buffers (rows, cache, output), together
    larger than the 256 MB last-level cache; `warm` repeats every launch on one set, which it partly or wholly
    finds in that cache."""
    import paper_2505_12658_amd as hydra

    report = []
    for b in (si.llava15_image_cache(), si.qwen2vl_image_cache()):
        host_rows = si.make_image_rows(b)
        slots, pages = si.make_slot_mapping(b.tokens, b.page_rows, spare_blocks=2, seed=b.seed)
        slots = torch.from_numpy(slots).to(dev)
        sets = [(host_rows.to(dev), torch.zeros((pages, b.page_rows, b.hidden), dtype=torch.bfloat16, device=dev)) for _ in range(n_sets)]
        sets = [(rows, cache, torch.empty_like(rows)) for rows, cache in sets]
        entry = {"workload": b.name, "rows": b.n_rows, "row_elems": b.hidden, "page_rows": b.page_rows, "bytes": b.bytes_moved(), "bound": "hbm",
                 "peak": PEAK_HBM_GBS, "unit": "GB/s", "buffer_sets": n_sets}

        def write(i):
            rows, cache, _ = sets[i % n_sets]
            hydra.hydra_page_cache_write(rows, cache, slots)

        def gather(i):
            _, cache, out = sets[i % n_sets]
            hydra.hydra_page_cache_gather(cache, slots, out)

        for name, fn in (("write", write), ("gather", gather)):
            figures = {}
            for label, pick in (("cold", lambda i: i), ("warm", lambda i: 0)):
                evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
                settle(lambda i: fn(pick(i)))
                for i, (e0, e1) in enumerate(evs):
                    e0.record()
                    fn(pick(i))
                    e1.record()
                torch.cuda.synchronize()
                avg = float(np.mean([e0.elapsed_time(e1) for e0, e1 in evs])) * 1e-3
                figures[label] = {"avg_kernel_us": avg * 1e6, "achieved": b.bytes_moved() / avg * 1e-9, "frac": b.bytes_moved() / avg * 1e-9 / PEAK_HBM_GBS}
            entry[name] = dict(figures["cold"], warm=figures["warm"])
        report.append(entry)
        del sets
        torch.cuda.empty_cache()
    return report


def describe(w: si.Workload):
    return {
        "workload": w.name,
        "sequences": w.batch,
        "total_tokens": w.total_tokens,
        "max_seqlen": w.max_seqlen,
        "n_q_heads": w.n_q_heads,
        "n_kv_heads": w.n_kv_heads,
        "head_dim": w.head_dim,
        "causal": w.causal,
        "kv_block_size": w.block_size if w.kv_cache else None,
        "seed": w.seed,
        "attention_flops": w.attention_flops(),
        "flop_convention": "4*head_dim*n_q_heads*visible (q,k) pairs",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=HEADLINE, choices=sorted(si.WORKLOADS))
    ap.add_argument("--sets", type=int, default=3, help="rotating buffer sets (cold last-level cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the secondary workloads")
    ap.add_argument("--kv-write-side-stream", action="store_true",
                    help="`value` from the step with the KV scatter on a second stream behind the attention launch (measured equal to one stream)")
    ap.add_argument("--dual-stream", action="store_true",
                    help="the two-stream measurements (an encode workload beside the prefill workload, and beside decode steps, "
                         "launched together on two streams against the same launches one after the other: the paper's vision || "
                         "language streams) at full length; the default run includes a short form of them")
    ap.add_argument("--paged-only", action="store_true", help="only the paged-attention measurements (for profiling that kernel)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain elementwise copy of 1 GiB (fp32 x + 0 -> y): the known-size kernel that "
                         "hardware-counter readings of FETCH_SIZE / WRITE_SIZE are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this path runs on ONE GPU (sequences are independent, so more GPUs would each take a "
              "share of the batch with no exchange); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.paged_only:
        print(json.dumps({"paged_attention": paged_attention(dev, args.sets, args.steps), "image_cache": image_cache(dev, args.steps)}))
        return
    w = si.WORKLOADS[args.workload]()
    batch = DeviceBatch(w, args.sets, dev)
    sec_one_stream = time_steps(batch, args.steps, args.warmup)
    sec_two_streams = time_steps(batch, args.steps, args.warmup, two_streams=True) if w.kv_cache else sec_one_stream
    sec_per_step = sec_two_streams if args.kv_write_side_stream else sec_one_stream
    attn_t, kvw_t = time_kernels(batch, args.steps)
    hot_t, _ = time_kernels(batch, max(20, args.steps // 2), hot_cache=True)
    flops = w.attention_flops()
    fig = profile_figures(w.name)
    attn_avg = float(attn_t.mean())
    achieved = flops / attn_avg * 1e-12

    result = {
        "metric": "attention TFLOP/s and % of bf16 MFMA peak, packed varlen encode+prefill",
        "value": flops / sec_per_step * 1e-12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": sec_per_step * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": describe(w),
        "step": "work-list build + fused attention" + (" + paged KV write" + (" (on a second stream)" if args.kv_write_side_stream else "") if w.kv_cache else ""),
        "ms_per_step_kv_write_on_side_stream": sec_two_streams * 1e3,
        "pct_of_bf16_mfma_peak": 100.0 * flops / sec_per_step * 1e-12 / PEAK_BF16_TFLOPS,
        "buffer_sets": args.sets,
        "roofline": {
            "kernel": "attn_fwd_kernel",
            "bound": "mfma",
            "achieved": achieved,
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": achieved / PEAK_BF16_TFLOPS,
            "traffic": fig["traffic_bytes"] if fig else None,
            "traffic_over_algorithmic": fig["traffic_bytes"] / w.attention_min_bytes() if fig else None,
            "mfma_busy": fig["mfma_busy"] if fig else None,
            "counters_from": {k: fig[k] for k in ("source", "commit", "kernel_avg_us_under_trace")} if fig else None,
            "avg_kernel_us": attn_avg * 1e6,
            "median_kernel_us": float(np.median(attn_t)) * 1e6,
            "min_kernel_us": float(attn_t.min()) * 1e6,
            "hbm_floor_us": w.attention_min_bytes() / (PEAK_HBM_GBS * 1e9) * 1e6,
            "algorithmic_bytes": w.attention_min_bytes(),
            "frac_hbm_peak": w.attention_min_bytes() / attn_avg * 1e-9 / PEAK_HBM_GBS,
            # the same launches on ONE buffer set (hot last-level cache; the figures above rotate over `buffer_sets`)
            "hot_cache": {"avg_kernel_us": float(hot_t.mean()) * 1e6, "median_kernel_us": float(np.median(hot_t)) * 1e6,
                          "achieved": flops / float(hot_t.mean()) * 1e-12, "frac": flops / float(hot_t.mean()) * 1e-12 / PEAK_BF16_TFLOPS},
        },
    }
    if kvw_t is not None:
        gbs = w.kv_write_bytes() / float(kvw_t.mean()) * 1e-9
        result["kv_write"] = {"kernel": "kv_cache_write_kernel", "bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                              "frac": gbs / PEAK_HBM_GBS, "avg_kernel_us": float(kvw_t.mean()) * 1e6, "bytes": w.kv_write_bytes()}
    host_qkv = batch.host_qkv
    del batch
    if args.calibration_copy:
        src = torch.ones(CALIBRATION_COPY_BYTES // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        result["calibration_copy"] = {"kernel": "torch elementwise add(x, 0) -> y, fp32", "bytes_read": CALIBRATION_COPY_BYTES,
                                      "bytes_written": CALIBRATION_COPY_BYTES, "launches": 3}
        del src, dst
    torch.cuda.empty_cache()

    if not args.no_others:
        others = []
        for name in OTHERS:
            ow = si.WORKLOADS[name]()
            ob = DeviceBatch(ow, args.sets, dev)
            sps = time_steps(ob, max(20, args.steps // 4), 5)
            at, kt = time_kernels(ob, max(20, args.steps // 4))
            f = ow.attention_flops()
            entry = {"workload": name, "ms_per_step": sps * 1e3, "attn_kernel_us": float(at.mean()) * 1e6,
                     "attn_tflops": f / float(at.mean()) * 1e-12, "frac_mfma_peak": f / float(at.mean()) * 1e-12 / PEAK_BF16_TFLOPS,
                     "frac_hbm_peak": ow.attention_min_bytes() / float(at.mean()) * 1e-9 / PEAK_HBM_GBS}
            if kt is not None:
                entry["kv_write_gbs"] = ow.kv_write_bytes() / float(kt.mean()) * 1e-9
            ofig = profile_figures(name)
            entry["algorithmic_bytes"] = ow.attention_min_bytes()
            entry["traffic"] = ofig["traffic_bytes"] if ofig else None
            entry["traffic_over_algorithmic"] = ofig["traffic_bytes"] / ow.attention_min_bytes() if ofig else None
            entry["mfma_busy"] = ofig["mfma_busy"] if ofig else None
            entry["counters_from"] = {k: ofig[k] for k in ("source", "commit", "kernel_avg_us_under_trace")} if ofig else None
            others.append(entry)
            del ob
            torch.cuda.empty_cache()
        result["other_workloads"] = others

    if not args.no_others:
        result["paged_attention"] = paged_attention(dev, args.sets, max(20, args.steps // 4))
        result["image_cache"] = image_cache(dev, max(20, args.steps // 4))
    if args.dual_stream or not args.no_others:
        # (short form in the default run; --dual-stream takes as many steps as the other secondary measurements)
        result["dual_stream"] = dual_stream(dev, args.sets, max(20, args.steps // 4) if args.dual_stream else max(10, args.steps // 20))
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, host_qkv)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
