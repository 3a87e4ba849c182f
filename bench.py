#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: fused RoPE + append
of the new chunk's K/V into the paged cache, then chunk attention of the new chunk's queries
over cache + chunk (attention kernel + split-KV combine).  Workload at one GPU: a single
layer of a 7B-class GQA decoder (28 query / 4 KV heads, d = 128, bf16, RoPE base 1e6) at step
32 of a stream (256-token prefix + 31 cached steps of 204 tokens = 6580 cached tokens), new
chunk of 204 tokens, 16-token pages in random order.  Inputs are resident in HBM before the
timed region starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
# what a register-resident loop of nothing but v_mfma_f32_32x32x16_bf16 reached on this chip
# (constant operands, a few milliseconds)
ACHIEVABLE_BF16_MFMA_TFLOPS = 2470.0
ACHIEVABLE_COPY_GBS = 5100.0     # a 1 GiB device-to-device copy, read + write
PEAK_HBM_GBS = 8000.0
# HBM bytes one attention launch of the workload below moves, from two rocprofv3 --pmc passes
# (FETCH_SIZE, WRITE_SIZE) over this very command, each scaled by what the same counter reads
# for a 256 MiB device copy (fetch x2.000, write x1.000); summary and commands in
# profiles/attn_layer7b_step32_6580cached_204new.txt.  The figure belongs to one state of the
# kernel source: it is stamped with that file's SHA-1, and the bench line says "traffic_stale"
# when the source has changed since.  Beside it the line carries the bytes the launch must move
# by construction ("traffic_modelled": K and V once, the queries once per piece of the key
# range, the partial rows of every piece), which cannot go stale.
ATTN_TRAFFIC_BYTES_PER_LAUNCH = 41.36e6
ATTN_TRAFFIC_MEASURED_ON_SHA1 = "ce17f7f87807851d973de5469805419217037104"
KERNEL_SOURCE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2512_10310_amd", "csrc",
                             "evl_kernels.hip")


def kernel_source_sha1():
    import hashlib
    with open(KERNEL_SOURCE, "rb") as f:
        return hashlib.sha1(f.read()).hexdigest()


def attention_flops(Hq, d, C, n):
    """Algorithmic flops of chunk attention: two contractions over the visible (query, key) pairs."""
    return 4.0 * d * Hq * (n * C + n * (n + 1) / 2.0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--lead-in", type=float, default=0.25,
                    help="seconds of untimed steps before the warm-up steps (lets the clocks settle)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-latency", action="store_true", help="skip the 28-layer 20k-cache latency leg")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the ragged-batch, redundancy and sampled-history legs (extra context, not "
                         "the metric)")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device copy (a kernel of known traffic, used to scale the "
                         "FETCH_SIZE / WRITE_SIZE counters when this command runs under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2512_10310_amd as evl
    from synth import LAYER7B, page_permutation

    evl.load()   # fails loudly if the HIP library is missing: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    shape = LAYER7B
    Hq, Hkv, d, n = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.step_tokens
    PAGE = evl.PAGE_SIZE
    gen = torch.Generator(device=dev)
    gen.manual_seed(20251210)

    def randn_bf16(*s):
        return torch.randn(*s, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)

    # everything runs on one dedicated (non-default) stream: torch's allocations and fills and the
    # library's kernels alike
    stream = torch.cuda.Stream()
    torch.cuda.set_stream(stream)

    def make_layers(n_layers, total_tokens, ws_bytes):
        """Device memory for n_layers caches of one sequence each, pages in seeded random order."""
        pages_per_layer = -(-total_tokens // PAGE)
        n_pages = n_layers * pages_per_layer
        k_pool = torch.empty((n_pages, Hkv, PAGE, d), dtype=torch.bfloat16, device=dev)
        v_pool = torch.empty((n_pages, Hkv, d, PAGE), dtype=torch.bfloat16, device=dev)
        order = page_permutation(n_pages, 1)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        layers = []
        for l in range(n_layers):
            tbl = torch.from_numpy(order[l * pages_per_layer:(l + 1) * pages_per_layer].copy()).to(dev)
            c = evl.Cache(Hq, Hkv, d, shape.rope_base, k_pool, v_pool, tbl, n_pages, pages_per_layer,
                          max_seqs=1, workspace=ws, workspace_bytes=ws_bytes,
                          stream=stream.cuda_stream)
            layers.append((c, tbl))
        return layers, (k_pool, v_pool, ws)

    def fill(cache, lengths):
        for m in lengths:
            cache.rope_append(randn_bf16(m, Hkv, d), randn_bf16(m, Hkv, d), cache.len(), m)

    if args.copy_calibration:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        a.fill_(1)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    # ---------------- main leg: single layer, step 32 ----------------
    C = shape.prefix + 31 * n
    ws_bytes = evl.workspace_bytes(Hq, d, n, 1)
    layers, keep = make_layers(1, C + n, ws_bytes)
    cache = layers[0][0]
    fill(cache, [shape.prefix] + [n] * 31)
    assert cache.len() == C
    q_new, k_new, v_new = randn_bf16(n, Hq, d), randn_bf16(n, Hkv, d), randn_bf16(n, Hkv, d)
    out = torch.empty((n, Hq, d), dtype=torch.bfloat16, device=dev)

    def step():
        cache.truncate(C)
        cache.rope_append(k_new, v_new, C, n)
        cache.chunk_attention(q_new, C, n, out)

    # Lead-in, untimed and outside the warm-up count: the chip raises its clocks only after some tens of
    # milliseconds of continuous work, and W + K steps of 40 us each can be over before that.
    lead_in_s, t_lead = args.lead_in, time.perf_counter()
    while time.perf_counter() - t_lead < lead_in_s:
        for _ in range(50):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the timed region: exactly `steps` steps, inputs resident, bracketed by synchronisations
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # The same region once more with a HIP-event pair attached to every attention kernel dispatch
    # (on the launch stream; the pair takes the kernel's own begin and end time) for the roofline
    # figure.  The throughput above is taken without them.
    cache.timing_enable(args.steps)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    kernel_ms = cache.timing_read(args.steps)
    cache.timing_enable(0)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = n / (ms_per_step * 1e-3)
    assert torch.isfinite(out.float()).all()
    plan = cache.last_plan()

    # What the chip reaches with nothing in the way, measured here and now (skipped with --no-extra, which
    # the profiling commands use; then the figures recorded earlier stand in): an MFMA-only loop
    # (csrc/peak_probe.hip) and a 1 GiB device-to-device copy.
    achievable_mfma, achievable_copy, achievable_src = ACHIEVABLE_BF16_MFMA_TFLOPS, ACHIEVABLE_COPY_GBS, "recorded earlier"
    probe_path = os.path.join(ROOT, "paper_2512_10310_amd", "libevl_peakprobe.so")
    if not args.no_extra and os.path.exists(probe_path):
        import ctypes
        probe = ctypes.CDLL(probe_path)
        probe.evl_peakprobe_mfma_bf16_tflops.restype = ctypes.c_double
        probe.evl_peakprobe_mfma_bf16_tflops.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
        scratch = torch.empty(256 * 512, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        tf = probe.evl_peakprobe_mfma_bf16_tflops(scratch.data_ptr(), 256, 20000, stream.cuda_stream)
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        a.fill_(1)
        b.copy_(a)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            b.copy_(a)
        e1.record(stream)
        torch.cuda.synchronize()
        copy_gbs = 5 * 2 * a.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9
        del a, b, scratch
        if tf > 0:
            achievable_mfma, achievable_copy, achievable_src = round(tf, 1), round(copy_gbs, 1), "measured in this run"

    flops = attention_flops(Hq, d, C, n)
    k_avg_ms = float(np.mean(kernel_ms))
    achieved_tflops = flops / (k_avg_ms * 1e-3) / 1e12
    alg_bytes = 2 * (C + n) * Hkv * d * 2 + 2 * n * Hq * d * 2
    roofline = {"bound": "mfma", "kernel": "attn_kernel<128>", "achieved": round(achieved_tflops, 2),
                "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved_tflops / PEAK_BF16_MFMA_TFLOPS, 4),
                "achievable_peak": achievable_mfma,
                "frac_of_achievable": round(achieved_tflops / achievable_mfma, 4),
                "achievable_peak_source": achievable_src,
                "traffic": ATTN_TRAFFIC_BYTES_PER_LAUNCH,
                "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size, on kernel "
                                  "source " + ATTN_TRAFFIC_MEASURED_ON_SHA1[:12],
                "traffic_stale": ATTN_TRAFFIC_MEASURED_ON_SHA1 != kernel_source_sha1(),
                # by construction: K and V once per KV head, the queries once per piece of the key range, and
                # the partial rows (d outputs + 2 floats) of every piece written; the merge kernel's reads
                # and the final output are the next launch's
                "traffic_modelled": float(2 * (C + n) * Hkv * d * 2 + plan[1] * n * Hq * d * 2 +
                                          (plan[1] * n * Hq * (d * 2 + 8) if plan[1] > 1 else n * Hq * d * 2)),
                "flops_per_launch": flops, "avg_launch_us": round(k_avg_ms * 1e3, 2),
                "p50_launch_us": round(float(np.median(kernel_ms)) * 1e3, 2),
                "algorithmic_bytes_per_launch": alg_bytes,
                "achieved_hbm_GBps": round(alg_bytes / (k_avg_ms * 1e-3) / 1e9, 1),
                "workgroups": plan[0], "key_splits": plan[1],
                "ms_per_step_with_kernel_events": round((t3 - t2) * 1e3 / args.steps, 5)}

    # ---------------- RoPE + append alone (HBM bound): the step's chunk and a whole-window prefill ----------------
    def append_leg(cache_, k_, v_, C_, m_, calls=10, reps=30):
        """p50 time of one evl_rope_append of m_ tokens behind C_ cached ones (several calls per event pair)."""
        def many():
            for _ in range(calls):
                cache_.truncate(C_)
                cache_.rope_append(k_, v_, C_, m_)
        for _ in range(3):
            many()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a_, b_ in evs:
            a_.record(stream)
            many()
            b_.record(stream)
        torch.cuda.synchronize()
        us = float(np.median([a_.elapsed_time(b_) for a_, b_ in evs])) / calls * 1e3
        nbytes = 2 * (2 * m_ * Hkv * d * 2)        # K and V read, K and V written
        return {"n_new": m_, "cached_tokens": C_, "us_per_call": round(us, 2), "algorithmic_bytes": nbytes,
                "GBps": round(nbytes / us / 1e3, 1), "frac_of_hbm_peak": round(nbytes / us / 1e3 / PEAK_HBM_GBS, 4),
                "frac_of_measured_copy": round(nbytes / us / 1e3 / achievable_copy, 4)}

    rope_legs = [append_leg(cache, k_new, v_new, C, n)]
    Wp = shape.prefix + 16 * n
    layers_p, keep_p = make_layers(1, Wp, 16)
    kp_, vp_ = randn_bf16(Wp, Hkv, d), randn_bf16(Wp, Hkv, d)
    rope_legs.append(append_leg(layers_p[0][0], kp_, vp_, 0, Wp))
    del layers_p, keep_p, kp_, vp_

    result = {
        "metric": "new-frame tokens/sec in chunk attention; p50 per-step latency at 20k cache",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: one layer, 28q/4kv heads, d=128, bf16, RoPE base 1e6, "
                               "6580 cached tokens (256 prefix + 31 steps x 204), new chunk 204, "
                               "16-token pages in random order; step = rope_append + chunk_attention",
                   "cache_len": C, "n_new": n, "page_size": PAGE,
                   "untimed_lead_in_s": lead_in_s},
        "roofline": roofline,
        "rope_append": {"bound": "hbm", "kernel": "rope_append_kernel<128>", "peak_GBps": PEAK_HBM_GBS,
                        "what": "evl_rope_append alone, back-to-back calls on one stream (time per call, launch "
                                "included); bytes = K and V of the chunk read + written; the 204-token chunk of "
                                "the step and the 3520-token window of the re-prefill",
                        "legs": rope_legs},
        "achievable": {"mfma_bf16_TFLOPs": achievable_mfma, "hbm_copy_GBps": achievable_copy,
                       "source": achievable_src,
                       "what": "register-resident v_mfma_f32_32x32x16_bf16 loop, constant operands, about 9 ms; "
                               "1 GiB device-to-device copy, read + write bytes"},
    }

    # ---------------- 20k-cache latency leg: 28 layers, last step of a 100-step episode ----------------
    if not args.no_latency:
        del layers, keep, cache
        n_layers, C2 = 28, shape.prefix + 99 * n
        layers, keep = make_layers(n_layers, C2 + n, ws_bytes)
        for c, _ in layers:
            fill(c, [shape.prefix + 49 * n, 50 * n])
        qs = [randn_bf16(n, Hq, d) for _ in range(n_layers)]
        ks = [randn_bf16(n, Hkv, d) for _ in range(n_layers)]
        vs = [randn_bf16(n, Hkv, d) for _ in range(n_layers)]

        def episode_step():
            # layers run back to back on one stream, as they would in a decoder
            for l, (c, _) in enumerate(layers):
                c.truncate(C2)
                c.rope_append(ks[l], vs[l], C2, n)
                c.chunk_attention(qs[l], C2, n, out)

        reps = 50
        for _ in range(5):
            episode_step()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for a, b in evs:
            a.record(stream)
            episode_step()
            b.record(stream)
        torch.cuda.synchronize()
        lat = np.array([a.elapsed_time(b) for a, b in evs])
        # the episode's curve: the same 28-layer step at earlier points of the episode (truncated caches)
        curve = []
        for st_ in (100, 75, 50, 25, 1):
            Cc = shape.prefix + (st_ - 1) * n

            def curve_step():
                for l, (c, _) in enumerate(layers):
                    c.truncate(Cc)
                    c.rope_append(ks[l], vs[l], Cc, n)
                    c.chunk_attention(qs[l], Cc, n, out)
            for _ in range(2):
                curve_step()
            torch.cuda.synchronize()
            evc = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(15)]
            for a, b in evc:
                a.record(stream)
                curve_step()
                b.record(stream)
            torch.cuda.synchronize()
            lc = np.array([a.elapsed_time(b) for a, b in evc])
            curve.append({"step": st_, "cached_tokens": Cc, "p50_ms": round(float(np.median(lc)), 4),
                          "p99_ms": round(float(np.percentile(lc, 99)), 4)})
        fl2 = attention_flops(Hq, d, C2, n) * n_layers
        result["latency_20k_cache"] = {
            "workload": "configs[2] last step: 28 layers, 20452 cached + 204 new tokens per layer",
            "p50_ms": round(float(np.median(lat)), 4), "min_ms": round(float(lat.min()), 4),
            "p99_ms": round(float(np.percentile(lat, 99)), 4), "repeats": reps,
            "tokens_per_s": round(n / (float(np.median(lat)) * 1e-3), 1),
            "attention_TFLOPs_at_p50": round(fl2 / (float(np.median(lat)) * 1e-3) / 1e12, 1),
            "episode_curve": curve[::-1],
            "paper_context": "paper reports 159 ms per step for the whole model (vision encoder + "
                             "8B LLM + decode) on 1x H200, FP16: context, not comparable",
        }
        del layers, keep

    # ---------------- extra legs (context): ragged batch, redundancy of re-prefill ----------------
    if not args.no_extra:
        from synth import ragged_cache_lengths

        def timed_ms(fn, reps, warm=3, calls=1):
            """p50 over `reps` event pairs of the time of one fn(); short steps are timed `calls` at a time,
            back to back as a serving loop issues them (an event pair around a single 15 us step measures the
            pair and an idling chip as much as the step)."""
            for _ in range(warm * calls):
                fn()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
            for a, b in evs:
                a.record(stream)
                for _ in range(calls):
                    fn()
                b.record(stream)
            torch.cuda.synchronize()
            return float(np.median([a.elapsed_time(b) for a, b in evs])) / calls

        # 16 episodes, cached lengths uniform in [2048, 65536], one 204-token chunk each, one launch
        lens = ragged_cache_lengths(16, 2048, 65536).tolist()
        need = [-(-(c_ + n) // PAGE) for c_ in lens]
        n_pages, maxp = sum(need), max(need)
        k_pool = torch.empty((n_pages, Hkv, PAGE, d), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        v_pool = torch.empty((n_pages, Hkv, d, PAGE), dtype=torch.bfloat16, device=dev).normal_(generator=gen)
        order = page_permutation(n_pages, 3)
        tbl = np.zeros((16, maxp), np.int32)
        cur = 0
        for s_, m in enumerate(need):
            tbl[s_, :m] = order[cur:cur + m]
            cur += m
        tbl = torch.from_numpy(tbl).to(dev)
        ws3 = torch.empty(512 << 20, dtype=torch.uint8, device=dev)
        c3 = evl.Cache(Hq, Hkv, d, shape.rope_base, k_pool, v_pool, tbl, n_pages, maxp, max_seqs=16,
                       workspace=ws3, workspace_bytes=512 << 20, stream=stream.cuda_stream)
        zk = torch.zeros((8192, Hkv, d), dtype=torch.bfloat16, device=dev)
        for s_ in range(16):           # bookkeeping only: the pools already hold random values
            done = 0
            while done < lens[s_]:
                m = min(8192, lens[s_] - done)
                c3.rope_append_batched(zk, zk, [s_], [done], [m])
                done += m
        k_pool.normal_(generator=gen)
        v_pool.normal_(generator=gen)
        q3, k3, v3 = randn_bf16(16 * n, Hq, d), randn_bf16(16 * n, Hkv, d), randn_bf16(16 * n, Hkv, d)
        out3 = torch.empty((16 * n, Hq, d), dtype=torch.bfloat16, device=dev)
        ids = list(range(16))

        def ragged_step():
            for s_ in ids:
                c3.truncate(lens[s_], s_)
            c3.rope_append_batched(k3, v3, ids, lens, [n] * 16)
            c3.chunk_attention_batched(q3, ids, lens, [n] * 16, out3)

        ms3 = timed_ms(ragged_step, 10)
        fl3 = sum(attention_flops(Hq, d, c_, n) for c_ in lens)
        result["ragged_batch"] = {
            "workload": "configs[3]: 16 episodes, cached lengths uniform in [2048, 65536] (sum %d), 204 new "
                        "tokens each, one launch through a randomly ordered 16-token-page pool" % sum(lens),
            "ms_per_step": round(ms3, 4), "tokens_per_s": round(16 * n / (ms3 * 1e-3), 1),
            "attention_TFLOPs": round(fl3 / (ms3 * 1e-3) / 1e12, 1),
            "frac_of_mfma_peak": round(fl3 / (ms3 * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
            # K and V of every sequence once per KV head + queries in + outputs out
            "algorithmic_GBps": round((sum(2 * (c_ + n) * Hkv * d * 2 for c_ in lens) + 16 * 2 * n * Hq * d * 2)
                                      / (ms3 * 1e-3) / 1e9, 1),
            "plan": c3.last_plan()}
        # small batches of the same cache: the first 2, 4 and 8 episodes in one launch (attention + merge only)
        small = []
        for S in (2, 4, 8):
            sub, sub_lens = ids[:S], lens[:S]
            ms_s = timed_ms(lambda: c3.chunk_attention_batched(q3[:S * n], sub, sub_lens, [n] * S, out3[:S * n]), 20, calls=3)
            fl_s = sum(attention_flops(Hq, d, c_, n) for c_ in sub_lens)
            small.append({"episodes": S, "cached_tokens": sub_lens, "ms": round(ms_s, 4),
                          "attention_TFLOPs": round(fl_s / (ms_s * 1e-3) / 1e12, 1), "plan": c3.last_plan()[:2]})
        result["ragged_batch"]["small_batches"] = small
        del c3, k_pool, v_pool, ws3, q3, k3, v3, out3

        # redundancy: re-prefill of a 16-frame window every step vs cache reuse of one chunk
        W = shape.prefix + 16 * n
        layersW, keepW = make_layers(1, W, ws_bytes)
        cW = layersW[0][0]
        qW, kW, vW = randn_bf16(W, Hq, d), randn_bf16(W, Hkv, d), randn_bf16(W, Hkv, d)
        outW = torch.empty((W, Hq, d), dtype=torch.bfloat16, device=dev)

        def reprefill_step():
            cW.truncate(0)
            cW.rope_append(kW, vW, 0, W)
            cW.chunk_attention(qW, 0, W, outW)

        def reuse_step():
            cW.truncate(W - n)
            cW.rope_append(kW[W - n:], vW[W - n:], W - n, n)
            cW.chunk_attention(qW[W - n:], W - n, n, outW[:n])

        msA = timed_ms(reprefill_step, 50, calls=5)
        msB = timed_ms(reuse_step, 50, calls=10)
        result["redundancy"] = {
            "workload": "configs[4]: (A) full causal re-prefill of the 16-frame window (%d tokens) each step vs "
                        "(B) cache reuse: %d cached + %d new" % (W, W - n, n),
            "reprefill_ms": round(msA, 4), "reuse_ms": round(msB, 4), "speedup": round(msA / msB, 2),
            "algorithmic_flop_ratio": round(attention_flops(Hq, d, 0, W) / attention_flops(Hq, d, W - n, n), 2),
            "reprefill_attention_TFLOPs": round(attention_flops(Hq, d, 0, W) / (msA * 1e-3) / 1e12, 1),
            "paper_context": "paper: 898 ms without cache vs 159 ms with cache (5.6x), whole model, 1x H200, FP16"}
        del layersW, keepW, cW

        # sampled history (paper Sec. 3.2 sampler): per-step time with 16 of the frames seen so far
        # retained (uniform sampler) vs attending to the whole history, one layer
        Cmax = shape.prefix + 100 * n
        layersS, keepS = make_layers(1, Cmax + n, evl.workspace_bytes_sampled(Hq, d, n, 17))
        cS = layersS[0][0]
        fill(cS, [shape.prefix + 50 * n, 50 * n])
        series = []
        for seen in (100, 50, 20):   # descending: truncation only ever shortens the sequence
            Cs = shape.prefix + seen * n
            runs = [(0, shape.prefix)] + [(shape.prefix + f * n, n) for f in evl.sample_uniform(seen, 16)]
            kept = sum(l for _, l in runs)
            runs = evl.make_runs(runs)

            def sampled_step():
                cS.truncate(Cs)
                cS.rope_append(k_new, v_new, Cs, n)
                cS.chunk_attention_sampled(q_new, runs, Cs, n, out)

            def whole_step():
                cS.truncate(Cs)
                cS.rope_append(k_new, v_new, Cs, n)
                cS.chunk_attention(q_new, Cs, n, out)

            ms_s = timed_ms(sampled_step, 50, calls=10)
            ms_w = timed_ms(whole_step, 50, calls=10)
            series.append({"frames_seen": seen, "cached_tokens": Cs, "retained_tokens": kept,
                           "sampled_ms": round(ms_s, 4), "whole_history_ms": round(ms_w, 4),
                           "sampled_attention_TFLOPs": round(attention_flops(Hq, d, kept, n) / (ms_s * 1e-3) / 1e12, 1)})
        # action-token decode shape (one new token, then four, over the same cache): bandwidth bound
        dec = []
        zeros_kv = torch.zeros((8192, Hkv, d), dtype=torch.bfloat16, device=dev)
        for Cs, label in ((shape.prefix + 16 * n, "16 retained frames"), (shape.prefix + 100 * n, "100 frames")):
            grown = cS.len() < Cs
            while cS.len() < Cs:      # bookkeeping back up to this length ...
                m_ = min(8192, Cs - cS.len())
                cS.rope_append(zeros_kv, zeros_kv, cS.len(), m_)
            if grown:                 # ... then random values again: timing depends on the data
                keepS[0].normal_()
                keepS[1].normal_()
            for nd in (1, 4):
                def decode_step():
                    cS.truncate(Cs)
                    cS.rope_append(k_new[:nd], v_new[:nd], Cs, nd)
                    cS.chunk_attention(q_new[:nd], Cs, nd, out[:nd])
                ms_d = timed_ms(decode_step, 50, calls=10)
                kv_bytes = 2 * (Cs + nd) * Hkv * d * 2
                dec.append({"cached_tokens": Cs, "history": label, "n_new": nd, "ms": round(ms_d, 4),
                            "kv_read_GBps": round(kv_bytes / (ms_d * 1e-3) / 1e9, 1),
                            "frac_of_hbm_peak": round(kv_bytes / (ms_d * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)})
        # the paper's decode step: one new token over the sampler's choice (prefix + 16 frames of the 100
        # seen + the frame just processed), as 18 runs of the append-only cache
        Cd = shape.prefix + 100 * n
        grown = cS.len() < Cd
        while cS.len() < Cd:
            m_ = min(8192, Cd - cS.len())
            cS.rope_append(zeros_kv, zeros_kv, cS.len(), m_)
        if grown:
            keepS[0].normal_()
            keepS[1].normal_()
        runs_d = [(0, shape.prefix)] + [(shape.prefix + f * n, n) for f in evl.sample_uniform(99, 16)] + \
                 [(shape.prefix + 99 * n, n)]
        kept_d = sum(l for _, l in runs_d)
        runs_d = evl.make_runs(runs_d)    # marshalled once: the step is short enough for that to matter

        def sampled_decode_step():
            cS.truncate(Cd)
            cS.rope_append(k_new[:1], v_new[:1], Cd, 1)
            cS.chunk_attention_sampled(q_new[:1], runs_d, Cd, 1, out[:1])
        ms_sd = timed_ms(sampled_decode_step, 50, calls=10)
        dec.append({"cached_tokens": Cd, "history": "prefix + 17 of 100 frames retained (%d tokens)" % kept_d,
                    "n_new": 1, "ms": round(ms_sd, 4),
                    "kv_read_GBps": round(2 * (kept_d + 1) * Hkv * d * 2 / (ms_sd * 1e-3) / 1e9, 1),
                    "frac_of_hbm_peak": round(2 * (kept_d + 1) * Hkv * d * 2 / (ms_sd * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)})
        def fused_sampled_decode_step():
            cS.truncate(Cd)
            cS.step_sampled(q_new[:1], k_new[:1], v_new[:1], runs_d, Cd, 1, out[:1])
        ms_fsd = timed_ms(fused_sampled_decode_step, 50, calls=10)
        dec.append({"cached_tokens": Cd, "history": "prefix + 17 of 100 frames retained (%d tokens), evl_step_sampled "
                                                    "(one launch)" % kept_d,
                    "n_new": 1, "ms": round(ms_fsd, 4),
                    "kv_read_GBps": round(2 * (kept_d + 1) * Hkv * d * 2 / (ms_fsd * 1e-3) / 1e9, 1),
                    "frac_of_hbm_peak": round(2 * (kept_d + 1) * Hkv * d * 2 / (ms_fsd * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)})
        # the same one-token steps through the one-call entry point (append + attention in one launch)
        # (longest first: truncation only goes down)
        for Cs, label in ((shape.prefix + 100 * n, "100 frames"), (shape.prefix + 16 * n, "16 retained frames")):
            def fused_decode_step():
                cS.truncate(Cs)
                cS.step(q_new[:1], k_new[:1], v_new[:1], Cs, 1, out[:1])
            ms_f = timed_ms(fused_decode_step, 50, calls=10)
            kv_bytes = 2 * (Cs + 1) * Hkv * d * 2
            dec.append({"cached_tokens": Cs, "history": label + ", evl_step (one launch)", "n_new": 1,
                        "ms": round(ms_f, 4), "kv_read_GBps": round(kv_bytes / (ms_f * 1e-3) / 1e9, 1),
                        "frac_of_hbm_peak": round(kv_bytes / (ms_f * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)})
        result["decode_shape"] = {
            "workload": "one layer, step = rope_append + chunk_attention[_sampled] of 1 or 4 new tokens; bytes = K "
                        "and V of the attended tokens once; p50 over 50 groups of 10 steps issued back to back",
            "steps": dec}
        result["sampled_history"] = {
            "workload": "one layer; prefix 256 + 16 uniformly sampled frames of 204 tokens retained out of "
                        "the frames seen so far, 204 new tokens; step = rope_append + chunk_attention_sampled; p50 over 50 "
                        "groups of 10 steps issued back to back",
            "steps": series[::-1]}
        del layersS, keepS, cS

        # packed sequence under the action-isolating mask (paper Sec. 3.3), forward attention of one layer:
        # prefix 256 + 16 x (196 + 8) tokens, against plain causal attention over the same 3520 tokens
        Fv, Av, Nf = shape.frame_tokens, shape.action_tokens, 16
        Lp = shape.prefix + Nf * (Fv + Av)
        layersP, keepP = make_layers(1, Lp, 64 << 20)
        cP = layersP[0][0]
        qP, kP, vP = randn_bf16(Lp, Hq, d), randn_bf16(Lp, Hkv, d), randn_bf16(Lp, Hkv, d)
        outP = torch.empty((Lp, Hq, d), dtype=torch.bfloat16, device=dev)
        cP.rope_append(kP, vP, 0, Lp)
        ms_pack = timed_ms(lambda: cP.isolated_pack_attention(qP, shape.prefix, Fv, Av, Nf, outP), 30)
        plan_pack = cP.last_plan()
        ms_causal = timed_ms(lambda: cP.chunk_attention(qP, 0, Lp, outP), 30)
        # the same pack appended with the ids the mask implies (evl_isolated_pack_append): one causal launch
        # in which the earlier steps' action tokens are holes of the key range
        layersQ, keepQ = make_layers(1, Lp, 64 << 20)
        cQ = layersQ[0][0]
        cQ.isolated_pack_append(kP, vP, 0, shape.prefix, Fv, Av, Nf)
        ms_pack_ids = timed_ms(lambda: cQ.isolated_pack_attention(qP, shape.prefix, Fv, Av, Nf, outP), 30)
        plan_pack_ids = cQ.last_plan()
        del layersQ, keepQ, cQ
        pairs = 0   # visible (query, key) pairs under the mask
        nv = shape.prefix
        pairs += shape.prefix * (shape.prefix + 1) // 2
        for t_ in range(Nf):
            pairs += Fv * nv + Fv * (Fv + 1) // 2
            nv += Fv
            pairs += Av * nv + Av * (Av + 1) // 2
        fl_pack = 4.0 * d * Hq * pairs
        result["isolated_pack"] = {
            "workload": "one layer; pack of 256 instruction tokens + 16 x (196 visual + 8 action) tokens = %d tokens; "
                        "attention of every token under the action-isolating mask (17 groups of the batched "
                        "sampled call)" % Lp,
            "ms": round(ms_pack, 4), "attention_TFLOPs": round(fl_pack / (ms_pack * 1e-3) / 1e12, 1),
            "visible_pairs": pairs, "plan": plan_pack,
            "appended_with_pack_ids_ms": round(ms_pack_ids, 4),
            "appended_with_pack_ids_TFLOPs": round(fl_pack / (ms_pack_ids * 1e-3) / 1e12, 1),
            "appended_with_pack_ids_plan": plan_pack_ids,
            "plain_causal_same_tokens_ms": round(ms_causal, 4)}
        del layersP, keepP, cP

        # one long sequence: 65 536 cached tokens (random values: the clock under load depends on the
        # data), the 204-token chunk through attention + merge, and one token through the decode kernel
        CL = 65536
        layersL, keepL = make_layers(1, CL + n, evl.workspace_bytes(Hq, d, n, 1))
        cL = layersL[0][0]
        zeros_l = torch.zeros((8192, Hkv, d), dtype=torch.bfloat16, device=dev)
        while cL.len() < CL + n:      # bookkeeping only; the pools are filled below
            m_ = min(8192, CL + n - cL.len())
            cL.rope_append(zeros_l, zeros_l, cL.len(), m_)
        torch.cuda.synchronize()
        keepL[0].normal_()
        keepL[1].normal_()

        # (several calls per event pair, so that the GPU never waits for the host in between)
        def long_attention():
            for _ in range(5):
                cL.chunk_attention(q_new, CL, n, out)

        def long_decode():
            for _ in range(10):
                cL.chunk_attention(q_new[:1], CL + n - 1, 1, out[:1])
        ms_la = timed_ms(long_attention, 30) / 5
        ms_ld = timed_ms(long_decode, 30) / 10
        fl_l = attention_flops(Hq, d, CL, n)
        kv_l = 2 * (CL + n) * Hkv * d * 2
        result["long_context"] = {
            "workload": "one layer, one sequence of 65 536 cached tokens in randomly ordered pages: (a) a 204-token "
                        "chunk, chunk_attention (attention + merge kernels); (b) one token, chunk_attention (decode "
                        "kernel, no append)",
            "chunk_ms": round(ms_la, 4), "chunk_attention_TFLOPs": round(fl_l / (ms_la * 1e-3) / 1e12, 1),
            "chunk_frac_of_mfma_peak": round(fl_l / (ms_la * 1e-3) / 1e12 / PEAK_BF16_MFMA_TFLOPS, 4),
            "decode_ms": round(ms_ld, 4), "decode_kv_read_GBps": round(kv_l / (ms_ld * 1e-3) / 1e9, 1),
            "decode_frac_of_hbm_peak": round(kv_l / (ms_ld * 1e-3) / 1e9 / PEAK_HBM_GBS, 3)}
        del layersL, keepL, cL, zeros_l

        # cache offload (paper Sec. 3.2, memory management): one layer's cache of 100 frames mirrored in
        # pinned host memory; per step the new frame's pages go out and the sampler's missing frames come
        # back into scattered device pages.  Bound: the host link (PCIe 5.0 x16, 64 GB/s each way).
        Co = shape.prefix + 100 * n
        n_seq_pages = -(-Co // PAGE)
        layersO, keepO = make_layers(1, Co, 16)
        cO, tblO = layersO[0]
        kO, vO = keepO[0], keepO[1]
        host_k = torch.empty((n_seq_pages, Hkv, PAGE, d), dtype=torch.bfloat16).pin_memory()
        host_v = torch.empty((n_seq_pages, Hkv, d, PAGE), dtype=torch.bfloat16).pin_memory()
        dev_of = tblO.cpu().tolist()
        page_bytes = 2 * Hkv * PAGE * d * 2        # the K block and the V block of a page
        def pages_of(a, b):
            return list(range(a // PAGE, (b - 1) // PAGE + 1))
        def out_fn(pages):
            dp = [dev_of[p_] for p_ in pages]
            return lambda: cO.pages_copy(host_k, host_v, pages, n_seq_pages, kO, vO, dp, n_seq_pages)
        def in_fn(pages):
            dp = [dev_of[p_] for p_ in pages]
            return lambda: cO.pages_copy(kO, vO, dp, n_seq_pages, host_k, host_v, pages, n_seq_pages)
        one_frame = pages_of(shape.prefix + 50 * n, shape.prefix + 51 * n)
        eight = sorted(set(sum([pages_of(shape.prefix + f * n, shape.prefix + (f + 1) * n)
                                for f in evl.sample_uniform(99, 16)[::2]], [])))
        everything = list(range(n_seq_pages))
        legs = []
        for label, pages in (("one frame (sliding window: one new segment per step)", one_frame),
                             ("8 of 16 sampled frames (uniform sampling: half of the set changes)", eight),
                             ("the whole 100-frame cache", everything)):
            for direction, fn in (("device_to_host", out_fn(pages)), ("host_to_device", in_fn(pages))):
                ms_c = timed_ms(fn, 30)
                legs.append({"what": label, "direction": direction, "pages": len(pages),
                             "MB": round(len(pages) * page_bytes / 1e6, 3), "ms": round(ms_c, 4),
                             "GBps": round(len(pages) * page_bytes / (ms_c * 1e-3) / 1e9, 2),
                             "frac_of_link_peak": round(len(pages) * page_bytes / (ms_c * 1e-3) / 1e9 / 64.0, 3)})
        # the link's rate for one contiguous block of the same size, by the runtime's own copy
        flat_d = kO.view(torch.uint8).view(-1)[:n_seq_pages * page_bytes // 2]
        flat_h = host_k.view(torch.uint8).view(-1)
        ms_h2d = timed_ms(lambda: flat_d.copy_(flat_h, non_blocking=True), 20)
        ms_d2h = timed_ms(lambda: flat_h.copy_(flat_d, non_blocking=True), 20)
        result["offload_reload"] = {
            "workload": "one layer, cache of 256 + 100 x 204 tokens in %d pages of %d KB (K and V), device pages "
                        "in random order, host pool pinned; evl_pages_copy" % (n_seq_pages, page_bytes // 1024),
            "link_peak_GBps": 64.0, "copies": legs,
            "runtime_contiguous_copy_GBps": {
                "host_to_device": round(flat_h.numel() / (ms_h2d * 1e-3) / 1e9, 2),
                "device_to_host": round(flat_h.numel() / (ms_d2h * 1e-3) / 1e9, 2)}}
        del layersO, keepO, cO, host_k, host_v

    # ---------------- CPU baseline: the oracle as it stands, on the host cores ----------------
    if not args.no_cpu_baseline:
        import oracle
        from synth import qkv_chunk, episode_chunk_lengths
        ost = oracle.Stream(Hq, Hkv, d, shape.rope_base)
        for s, m in enumerate(episode_chunk_lengths(shape, 31)):
            _, k, v = qkv_chunk(shape, m, 1, 0, s)
            ost.append(k, v, len(ost))
        q, k, v = qkv_chunk(shape, n, 1, 0, 32)
        done, t_cpu = 0, 0.0
        while t_cpu < args.cpu_seconds and done < 24:
            ost.truncate(C)
            a = time.perf_counter()
            ost.step(q, k, v, C)
            t_cpu += time.perf_counter() - a
            done += 1
        result["cpu_baseline"] = {
            "value": round(n * done / t_cpu, 2), "unit": "tokens/s", "cores": oracle.threads(),
            "kind": "oracle",
            "sample": "%d full steps of the same workload (append 204 + attend 204 rows over 6784 keys, "
                      "double precision), %.1f s" % (done, t_cpu)}

    print(json.dumps(result))


if __name__ == "__main__":
    main()
