#!/usr/bin/env python3
"""Benchmark of the multi-query-attention decode step on one MI355X.

Workload ("long_context_probe", the configuration the headline metric is quoted
on): one MQA decode step with b=64 sequences, m=8192 cached positions, h=32
query heads, k=v=128, bf16 K/V cache ~N(0,1), q fp32 ~N(0,1)/sqrt(k), all
sequences full length.  One step = one mqa_decode_step call (logits, softmax,
weighted sum over the whole cache, including the merge of the position ranges).
Inputs are seeded synthetic tensors resident in HBM before the timed region.
Several distinct K/V sets (>= 1 GiB in total, four times the 256 MB Infinity
Cache) are rotated so that every step streams its cache from HBM.

Prints ONE JSON line: the whole-step K/V throughput (`value`, GB/s on the K/V
bytes a step must read), the step latency, a roofline object for the dominant
kernel timed alone, the multi-head twin (32x the bytes) and the float64 CPU
oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# The paper's own decoder timings (Table 2 and the inference-speed paragraph of section 4):
# another machine, a trained model, an unstated precision and a whole six-layer decoder step.
# Printed beside this run's numbers as context; never a target and never in vs_baseline.
PAPER_CONTEXT = {
    "hardware": "one TPUv2, 8 cores",
    "workload": "WMT14 EN-DE decoder, 6 layers, d=1024, h=8, k=v=128, batch 1024, source and target length 128",
    "decoder_us_per_token_greedy": {"multi_head": 46, "multi_query": 3.8,
                                    "multi_head_local": 23, "multi_query_local": 3.3},
    "decoder_us_per_token_beam4": {"multi_head": 203, "multi_query": 32,
                                   "multi_head_local": 47, "multi_query_local": 16},
    "comparable_here": "other_workloads.3_decoder_stack_*: us_per_token of this build's six-layer self-attention stack",
    "use": "context only",
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--skip-mha", action="store_true", help="do not time the 8 GiB multi-head twin")
    ap.add_argument("--skip-cpu-baseline", action="store_true", help="do not time the CPU oracle")
    ap.add_argument("--skip-other-workloads", action="store_true", help="do not time workloads 1, 2, 3 and 5")
    ap.add_argument("--only-ragged", action="store_true",
                    help="time only the ragged large-batch workload (b=512, h=64) and print its record: for profiling it alone")
    ap.add_argument("--splits", type=int, default=0, help="override the number of position ranges")
    ap.add_argument("--flags", type=int, default=0, help="override kernel variant flags")
    return ap.parse_args()


def time_region(fn, steps, warmup, settle_s=0.25):
    """W untimed warm-up calls, then exactly `steps` timed calls between two events on the
    current stream.  Before the warm-up the same call is repeated for `settle_s` seconds so
    that clocks and power state have settled (a cold first region reads several us slow)."""
    import torch
    t_end = time.perf_counter() + settle_s
    while time.perf_counter() < t_end:
        for i in range(20):
            fn(i)
        torch.cuda.synchronize()
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps          # ms per call


def step_distribution(fn, steps, warmup):
    """Per-step intervals (event before every step, one after the last): median / min / p90 in us.
    The events add a little to each interval; the headline rate comes from time_region."""
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    for i in range(steps):
        ev[i].record()
        fn(i)
    ev[steps].record()
    torch.cuda.synchronize()
    us = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(steps))
    return {"median": us[len(us) // 2], "min": us[0], "p90": us[min(len(us) - 1, (9 * len(us)) // 10)], "n": steps}


def traffic_from_profile():
    """HBM bytes per launch of the dominant kernel, from the committed counter summary (or None)."""
    path = os.path.join(ROOT, "profiles", "mqa_decode_mfma_long_context_probe_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def graph_time_us(fn, replays=20, repeat=10):
    """GPU time of the launches `fn(stream)` enqueues.  `repeat` copies of them are captured in one HIP
    graph (so that neither the host's launch rate nor the ~10 us cost of launching a graph is measured)
    and the graph is replayed `replays` times; returns microseconds per copy."""
    import torch
    fn(None)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            for _ in range(repeat):
                fn(side)
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(5):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (replays * repeat) * 1e3


def other_workloads(m, mi, dev):
    """Latency of the other workloads' steps (synthetic tensors of their shapes; values do not matter
    for timing, parity is in the tests).  Appends past capacity are no-ops, so replays are identical."""
    import numpy as np
    import torch
    out = {}

    def layer_step_fn(b, h, d, k, v, cap, length, mh, dtype):
        x = torch.randn(b, d, device=dev)
        Pq = torch.randn(h, d, k, device=dev) / d ** 0.5
        Po = torch.randn(h, d, v, device=dev) / d ** 0.5
        Pk = torch.randn((h, d, k) if mh else (d, k), device=dev) / d ** 0.5
        Pv = torch.randn((h, d, v) if mh else (d, v), device=dev) / d ** 0.5
        shp = (b, h, cap, k) if mh else (b, cap, k)
        K = torch.randn(shp, device=dev).to(dtype)
        V = torch.randn(shp, device=dev).to(dtype)
        lens = torch.full((b,), length, dtype=torch.int32, device=dev)       # full: the append is a no-op
        q = torch.empty(b, h, k, device=dev)
        kn = torch.empty((b, h, k) if mh else (b, k), device=dev)
        vn = torch.empty_like(kn)
        o = torch.empty(b, h, v, device=dev)
        y = torch.empty(b, d, device=dev)
        ws = torch.empty(m.mqa_decode_workspace_bytes(b, h, cap, v), dtype=torch.uint8, device=dev)
        kvm = m.MQA_PROJ_KV_MH if mh else m.MQA_PROJ_KV
        dec = m.mha_decode_step if mh else m.mqa_decode_step

        lens2 = torch.empty_like(lens)

        def fn(st):          # three launches: q/k/v projections + append, attention, output projection
            m.mqa_project_append_qkv(x, Pq, Pk, Pv, K, V, lens, lens2, q=q, stream=st)
            dec(q, K, V, lens2, o=o, workspace=ws, stream=st)
            m.mqa_project_qkvo(m.MQA_PROJ_O, o, Po, out=y, stream=st)

        def fn_separate(st):  # the same step through the four separate calls
            m.mqa_project_qkvo(m.MQA_PROJ_Q, x, Pq, out=q, stream=st)
            m.mqa_project_qkvo(kvm, x, Pk, out=kn, stream=st)
            m.mqa_project_qkvo(kvm, x, Pv, out=vn, stream=st)
            m.mqa_append_kv(K, V, kn, vn, lens, stream=st)
            dec(q, K, V, lens, o=o, workspace=ws, stream=st)
            m.mqa_project_qkvo(m.MQA_PROJ_O, o, Po, out=y, stream=st)

        def attn(st):
            dec(q, K, V, lens, o=o, workspace=ws, stream=st)
        return fn, attn, fn_separate

    # workload 1: one fp32 step, b=1, m=128 (projection of the 128-row memory excluded)
    fn, attn, sep = layer_step_fn(1, 8, 1024, 128, 128, 128, 128, False, torch.float32)
    out["1_single_step_fp32"] = {"layer_step_us": graph_time_us(fn), "attention_us": graph_time_us(attn),
                                 "layer_step_separate_calls_us": graph_time_us(sep)}
    # workload 2: b=128, cache of 128 positions, one layer: q/k/v projections, append, attention, output projection
    for mh in (False, True):
        fn, attn, sep = layer_step_fn(128, 8, 1024, 128, 128, 128, 128, mh, torch.bfloat16)
        t, ta = graph_time_us(fn), graph_time_us(attn)
        # the latency curve over the decode loop: attention alone at t cached positions (capacity 128)
        curve = {}
        for t_pos in (1, 8, 32, 64, 96):
            curve[str(t_pos)] = graph_time_us(layer_step_fn(128, 8, 1024, 128, 128, 128, t_pos, mh, torch.bfloat16)[1])
        curve["128"] = ta
        out["2_incremental_b128_" + ("mha" if mh else "mqa")] = {
            "layer_step_us": t, "attention_us": ta, "layer_step_separate_calls_us": graph_time_us(sep),
            "tokens_per_s": 128 / (t * 1e-6), "cached_positions": 128, "attention_us_by_cached_positions": curve}
    # the paper's local-attention variants (Section 4.1: current position and the 31 before it), attention only,
    # at 256 cached positions
    bq, hq, capq = 128, 8, 256
    q = torch.randn(bq, hq, 128, device=dev) / 128 ** 0.5
    o = torch.empty(bq, hq, 128, device=dev)
    lens = torch.full((bq,), capq, dtype=torch.int32, device=dev)
    Kq, Vq = (torch.randn(bq, capq, 128, device=dev).to(torch.bfloat16) for _ in range(2))
    Kh, Vh = (torch.randn(bq, hq, capq, 128, device=dev).to(torch.bfloat16) for _ in range(2))
    ws = torch.empty(m.mha_decode_workspace_bytes(bq, hq, capq, 128), dtype=torch.uint8, device=dev)
    out["local_window32_b128_len256"] = {
        "mqa_attention_us": graph_time_us(lambda st: m.mqa_decode_step_window(q, Kq, Vq, lens, 32, o=o, workspace=ws, stream=st)),
        "mha_attention_us": graph_time_us(lambda st: m.mha_decode_step_window(q, Kh, Vh, lens, 32, o=o, workspace=ws, stream=st)),
        "mqa_full_attention_us": graph_time_us(lambda st: m.mqa_decode_step(q, Kq, Vq, lens, o=o, workspace=ws, stream=st)),
        "mha_full_attention_us": graph_time_us(lambda st: m.mha_decode_step(q, Kh, Vh, lens, o=o, workspace=ws, stream=st))}
    del Kq, Vq, Kh, Vh
    # workload 3: six such layers at 256 cached positions plus feed-forward, final layernorm, logits, argmax
    # (b = 1024 is the paper's whole batch, which it spread over 8 TPU cores, on the one GPU)
    for mh, bsz in ((False, None), (True, None), (False, 1024), (True, 1024)):
        from paper_1911_02150_amd.decoder_stack import DecoderStack
        cfg = mi.CONFIGS[3]
        bsz = bsz or cfg["b"]
        w = mi.config3_weights(cfg["layers"], cfg["d"], cfg["h"], cfg["k"], cfg["v"], cfg["d_ff"], cfg["vocab"],
                               cfg["cap"], mh)
        st_ = DecoderStack(w, bsz, cfg["cap"], mh, dev)
        for l in range(cfg["layers"]):
            st_.lens[l].fill_(cfg["cap"])
            st_._lens_next[l].fill_(cfg["cap"])
        tok = torch.zeros(bsz, dtype=torch.int32, device=dev)

        def full(stream):
            with torch.cuda.stream(stream) if stream is not None else torch.cuda.stream(torch.cuda.current_stream()):
                st_.greedy(st_.step(tok, cfg["cap"] - 1))
        t = graph_time_us(full, replays=10, repeat=3)
        name = "3_decoder_stack_" + ("mha" if mh else "mqa") + ("" if bsz == cfg["b"] else f"_b{bsz}")
        out[name] = {"step_us": t, "us_per_token": t / bsz, "tokens_per_s": bsz / (t * 1e-6), "b": bsz,
                     "cached_positions": cfg["cap"], "layers": cfg["layers"]}
        if not mh and bsz == cfg["b"]:
            # the 128-token prompts of the same workload in one prefill pass (bulk append + causal attention per layer)
            prompts = torch.randint(0, cfg["vocab"], (bsz, cfg["prompt"]), dtype=torch.int32, device=dev)

            def prefill(i):
                for l in range(cfg["layers"]):
                    st_.lens[l].zero_()
                st_.prefill(prompts)
            ms = time_region(prefill, 3, 1, settle_s=0.0)
            ntok = bsz * cfg["prompt"]
            out["3_decoder_stack_mqa_prefill"] = {"prompt_ms": ms, "us_per_token": ms * 1e3 / ntok,
                                                  "tokens_per_s": ntok / (ms * 1e-3), "b": bsz, "prompt": cfg["prompt"]}
        del st_, w
    # beam-4 decoding: (a) workload 2's shape, 128 sources, 128 shared + 128 own positions per hypothesis;
    # (b) long prompts, 16 sources, 8192 shared + 128 own.  Against the same step over per-hypothesis copies of
    # the memory (multi-query and multi-head), and the per-step cache reorder for the two cache layouts.
    def beam_case(b, beam, h, cs, co, with_mha):
        n = b * beam
        bf = torch.bfloat16
        q = torch.randn(b, beam, h, 128, device=dev) / 128 ** 0.5
        o = torch.empty(b, beam, h, 128, device=dev)
        Ksrc, Vsrc = torch.randn(b, cs, 128, device=dev).to(bf), torch.randn(b, cs, 128, device=dev).to(bf)
        Kown, Vown = torch.randn(b, beam, co, 128, device=dev).to(bf), torch.randn(b, beam, co, 128, device=dev).to(bf)
        lsrc = torch.full((b,), cs, dtype=torch.int32, device=dev)
        lown = torch.full((n,), co, dtype=torch.int32, device=dev)
        ws = torch.empty(m.mqa_decode_beams_workspace_bytes(b, beam, h, cs, co, 128, 128, m.MQA_BF16), dtype=torch.uint8, device=dev)
        r = {"mqa_shared_source_attention_us": graph_time_us(
            lambda st: m.mqa_decode_step_beams(q, Ksrc, Vsrc, lsrc, Kown, Vown, lown, o=o, workspace=ws, stream=st))}
        Kf, Vf = torch.randn(n, cs + co, 128, device=dev).to(bf), torch.randn(n, cs + co, 128, device=dev).to(bf)
        lf = torch.full((n,), cs + co, dtype=torch.int32, device=dev)
        wsf = torch.empty(m.mqa_decode_workspace_bytes(n, h, cs + co, 128), dtype=torch.uint8, device=dev)
        qf, of = q.view(n, h, 128), o.view(n, h, 128)
        r["mqa_per_hypothesis_copies_attention_us"] = graph_time_us(
            lambda st: m.mqa_decode_step(qf, Kf, Vf, lf, o=of, workspace=wsf, stream=st))
        parent = ((torch.arange(n, device=dev) // beam) * beam + torch.randint(0, beam, (n,), device=dev)).to(torch.int32)
        K2, V2, l2 = torch.empty_like(Kown), torch.empty_like(Vown), torch.empty_like(lown)
        r["mqa_reorder_own_rows_us"] = graph_time_us(
            lambda st: m.mqa_beam_reorder_kv(Kown.view(n, co, 128), Vown.view(n, co, 128), lown, parent,
                                             K2.view(n, co, 128), V2.view(n, co, 128), l2, stream=st))
        if with_mha:
            Kh, Vh = torch.randn(n, h, cs + co, 128, device=dev).to(bf), torch.randn(n, h, cs + co, 128, device=dev).to(bf)
            r["mha_attention_us"] = graph_time_us(lambda st: m.mha_decode_step(qf, Kh, Vh, lf, o=of, workspace=wsf, stream=st))
            Kh2, Vh2 = torch.empty_like(Kh), torch.empty_like(Vh)
            r["mha_reorder_whole_cache_us"] = graph_time_us(lambda st: m.mqa_beam_reorder_kv(Kh, Vh, lf, parent, Kh2, Vh2, l2, stream=st))
        return r
    out["beam4_b128_src128_own128"] = beam_case(128, 4, 8, 128, 128, True)
    out["beam4_b16_src8192_own128"] = beam_case(16, 4, 8, 8192, 128, False)
    out["5_ragged_large_batch"] = ragged_workload(m, mi, dev)
    return out


def ragged_workload(m, mi, dev, steps=30, warmup=5):
    """Workload 5: ragged batch (b=512, h=64, capacity 4096, lengths ~ U{1..4096}), attention only, on the seeded
    inputs the parity test checks: its lengths, its +30 logits, NaN beyond the lengths; two copies at different
    addresses alternate (1.1 GB of valid rows against the 256 MB Infinity Cache)."""
    import torch
    cfg = mi.CONFIGS[5]
    b, h, cap = cfg["b"], cfg["h"], cfg["cap"]
    q_np, K_np, V_np, lens_np = mi.config5(b, h, cfg["k"], cfg["v"], cap, cfg["outlier_fraction"], cfg["outlier_boost"])
    lens = torch.from_numpy(lens_np).to(dev)
    q = torch.from_numpy(q_np).to(dev)
    o = torch.empty(b, h, 128, device=dev)
    Ks = [mi.bits_to_torch_bf16(K_np).to(dev)]
    Vs = [mi.bits_to_torch_bf16(V_np).to(dev)]
    Ks.append(Ks[0].clone())
    Vs.append(Vs[0].clone())
    ws = torch.empty(m.mqa_decode_workspace_bytes(b, h, cap, 128), dtype=torch.uint8, device=dev)
    ms = time_region(lambda i: m.mqa_decode_step(q, Ks[i % 2], Vs[i % 2], lens, o=o, workspace=ws), steps, warmup)
    kvb = int(lens_np.sum()) * 512
    qob = 2 * b * h * 128 * 4
    return {"step_us": ms * 1e3, "kv_bytes": kvb, "kv_GBps": kvb / (ms * 1e-3) / 1e9,
            "frac_of_peak": kvb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "q_and_o_bytes": qob, "frac_of_peak_with_q_and_o": (kvb + qob) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "b": b, "h": h, "cap": cap, "sum_of_lengths": int(lens_np.sum()),
            "data": "mqa_inputs.config5 (the seeded lengths, outliers and NaN tails of the parity test)"}


def cpu_baseline(q, K_bits, V_bits, budget_s=12.0):
    """The float64 oracle on the host cores over whole passes of the same workload."""
    import numpy as np
    import mqa_inputs as mi
    from oracle import mqa_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])      # threads the BLAS under numpy uses
    except Exception:
        cores = os.cpu_count() or 1
    b, m, k = K_bits.shape
    lens = np.full((b,), m, dtype=np.int64)
    done, t0 = 0, time.perf_counter()
    while True:
        i = done % b
        orc.mqa_decode(q[i:i + 1], mi.bf16_bits_to_f64(K_bits[i:i + 1]), mi.bf16_bits_to_f64(V_bits[i:i + 1]), lens[i:i + 1])
        done += 1
        el = time.perf_counter() - t0
        if (el >= budget_s and done >= 8) or done >= 200 * b:
            break
    bytes_done = done * m * 2 * k * 2
    # the oracle's time for one attention step of the other workloads (float64, same host cores; one run each;
    # the ragged workload on 64 of its 512 sequences, scaled)
    others = {}
    g = np.random.default_rng(0)
    for name, (bb, hh, mm, scale_up) in {"1_single_step_fp32": (1, 8, 128, 1), "2_incremental_b128": (128, 8, 128, 1),
                                         "3_decoder_stack_one_layer": (128, 8, 256, 1),
                                         "5_ragged_large_batch": (64, 64, 4096, 8)}.items():
        ln = g.integers(1, mm + 1, size=bb) if name.startswith("5") else np.full(bb, mm)
        qq = g.standard_normal((bb, hh, k), dtype=np.float32)
        KK, VV = g.standard_normal((bb, mm, k), dtype=np.float32), g.standard_normal((bb, mm, k), dtype=np.float32)
        t1 = time.perf_counter()
        orc.mqa_decode(qq, KK, VV, ln)
        others[name] = {"oracle_attention_ms": (time.perf_counter() - t1) * 1e3 * scale_up}
    return {
        "other_workloads": others,
        "value": bytes_done / el / 1e9, "unit": "GB/s", "cores": int(cores), "host_cpu_count": os.cpu_count(),
        "kind": "oracle",
        "sample": f"{done} single-sequence calls of oracle.mqa_decode in float64 ({done / b:.1f} passes over the "
                  f"workload's {b} sequences, m={m}, h={q.shape[1]}) in {el:.1f} s; bytes counted as the bf16 K/V "
                  f"bytes of the sequences processed",
        "step_seconds_extrapolated": el / done * b,
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import mqa_inputs as mi
    import paper_1911_02150_amd as m

    m.load_library()                      # raises if the HIP library has not been built
    dev = torch.device("cuda:0")
    if args.only_ragged:
        print(json.dumps({"workload": "5_ragged_large_batch", **ragged_workload(m, mi, dev, args.steps, args.warmup)}))
        return
    cfg = mi.CONFIGS[4]
    b, h, cap, k, v = cfg["b"], cfg["h"], cfg["cap"], cfg["k"], cfg["v"]
    kv_bytes = b * cap * (k + v) * 2
    nbuf = 5                              # 5 x 256 MiB of distinct K/V

    # ---- seeded inputs, resident in HBM before timing
    q_np = mi.config4_q(b, h, k)
    K_np, V_np = mi.config4_kv(b=b * nbuf, m=cap, k=k, v=v, threads=min(16, os.cpu_count() or 8))
    q = torch.from_numpy(q_np).to(dev)
    Ks = [mi.bits_to_torch_bf16(K_np[i * b:(i + 1) * b]).to(dev) for i in range(nbuf)]
    Vs = [mi.bits_to_torch_bf16(V_np[i * b:(i + 1) * b]).to(dev) for i in range(nbuf)]
    lens = torch.full((b,), cap, dtype=torch.int32, device=dev)
    o = torch.empty((b, h, v), dtype=torch.float32, device=dev)
    ws = torch.empty(m.mqa_decode_workspace_bytes(b, h, cap, v), dtype=torch.uint8, device=dev)
    tuning = dict(splits=args.splits, flags=args.flags) if (args.splits or args.flags) else None
    splits = m.mqa_decode_num_splits(b, h, cap, k, v, m.MQA_BF16, False, tuning)

    # ---- the timed region: K whole steps
    def step(i):
        m.mqa_decode_step(q, Ks[i % nbuf], Vs[i % nbuf], lens, o=o, workspace=ws, tuning=tuning)

    ms_step = time_region(step, args.steps, args.warmup)
    step_us = ms_step * 1e3
    value = kv_bytes / (ms_step * 1e-3) / 1e9

    latency = step_distribution(step, args.steps, args.warmup)
    # the same step with a single K/V set: the 256 MB Infinity Cache serves part of the reads (NOT an HBM figure)
    ms_warm = time_region(lambda i: m.mqa_decode_step(q, Ks[0], Vs[0], lens, o=o, workspace=ws, tuning=tuning),
                          args.steps, args.warmup, settle_s=0.05)

    # ---- dominant kernel alone (the streaming pass), same launch configuration
    def main_only(i):
        m.mqa_decode_partials(q, Ks[i % nbuf], Vs[i % nbuf], lens, o, ws, tuning=tuning)

    ms_main = time_region(main_only, args.steps, args.warmup)
    alg_bytes = kv_bytes + b * h * k * 4 + b * h * v * 4 + b * 4
    achieved = alg_bytes / (ms_main * 1e-3) / 1e9
    roofline = {
        "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic_from_profile(),
        "kernel": "decode_mfma_kernel", "avg_launch_us": ms_main * 1e3, "algorithmic_bytes": alg_bytes,
    }

    # ---- the box's achievable streaming-read rate, same run
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    sink = torch.zeros(4096, dtype=torch.float32, device=dev)
    ms_read = time_region(lambda i: m.mqa_stream_read(big, sink), 20, 3)
    stream_read_gbps = big.numel() / (ms_read * 1e-3) / 1e9
    # the same streaming read over exactly the decode step's K/V bytes: what a kernel that only reads them takes
    nsame = kv_bytes
    ms_same = time_region(lambda i: m.mqa_stream_read(big[(i % 3) * nsame:(i % 3 + 1) * nsame], sink), args.steps, args.warmup,
                          settle_s=0.05)
    big2 = torch.empty_like(big)          # plain copy of known size: the reference for the byte counters
    ms_copy = time_region(lambda i: m.mqa_stream_copy(big, big2), 10, 2)
    stream_copy_gbps = 2 * big.numel() / (ms_copy * 1e-3) / 1e9
    del big, big2

    # ---- multi-head twin: per-head K/V, 32x the bytes
    mha = None
    if not args.skip_mha:
        gen = torch.Generator(device=dev)
        gen.manual_seed(mi.SEED_BASE + 4)
        Kh = torch.empty((b, h, cap, k), dtype=torch.bfloat16, device=dev)
        Vh = torch.empty((b, h, cap, v), dtype=torch.bfloat16, device=dev)
        for i in range(b):
            Kh[i].copy_(torch.randn((h, cap, k), device=dev, generator=gen))
            Vh[i].copy_(torch.randn((h, cap, v), device=dev, generator=gen))
        wsh = torch.empty(m.mha_decode_workspace_bytes(b, h, cap, v), dtype=torch.uint8, device=dev)
        ms_mha = time_region(lambda i: m.mha_decode_step(q, Kh, Vh, lens, o=o, workspace=wsh), 10, 2)
        mha_bytes = kv_bytes * h
        mha = {"step_us": ms_mha * 1e3, "kv_bytes": mha_bytes, "kv_GBps": mha_bytes / (ms_mha * 1e-3) / 1e9,
               "frac_of_peak": mha_bytes / (ms_mha * 1e-3) / 1e9 / HBM_PEAK_GBPS,
               "mha_over_mqa_time": ms_mha / ms_step, "kv_bytes_ratio": h, "ratio_predicted_by_the_paper": h,
               "data": "torch.randn on the device, seeded (timing only; parity uses the host-seeded blocks)"}
        del Kh, Vh

    # the secondary legs must not cost the headline line: a failure is reported in place
    others = None
    if not args.skip_other_workloads:
        del Ks, Vs
        try:
            others = other_workloads(m, mi, dev)
        except Exception as e:          # noqa: BLE001
            others = {"error": f"{type(e).__name__}: {e}"}

    cpu = None
    if not args.skip_cpu_baseline:
        try:
            cpu = cpu_baseline(q_np, K_np[:b], V_np[:b])
        except Exception as e:          # noqa: BLE001
            cpu = {"error": f"{type(e).__name__}: {e}", "kind": "oracle"}

    out = {
        "metric": "MQA decode-step µs + achieved HBM GB/s on K/V bytes (fraction of peak) vs MHA",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "long_context_probe: MQA decode step b=64 m=8192 h=32 k=v=128, bf16 K/V, all lengths full",
                   "b": b, "h": h, "m": cap, "k": k, "v": v, "kv_bytes_per_step": kv_bytes,
                   "kv_sets_rotated": nbuf, "position_ranges": splits},
        "step_us": step_us, "step_us_distribution": latency, "tokens_per_s": b / (ms_step * 1e-3),
        "frac_of_peak": value / HBM_PEAK_GBPS, "frac_of_stream_read": value / stream_read_gbps,
        "single_kv_set_step_us_cache_warm": ms_warm * 1e3,
        "stream_read_GBps": stream_read_gbps, "stream_copy_GBps": stream_copy_gbps,
        "stream_read_of_the_same_kv_bytes_us": ms_same * 1e3,
        "roofline": roofline, "mha": mha, "other_workloads": others, "cpu_baseline": cpu,
        "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
