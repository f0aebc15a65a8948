#!/usr/bin/env python3
"""Benchmark of the quantized-pruned KV cache hot path on one MI355X.

Workload (the headline configuration, configs[1]): Llama-3-8B-shaped KV cache -- 32 layers,
32 query / 8 KV heads, head_dim 128, half precision, batch 1, prompt L = 32768,
synthetic N(0,1) data with four x10 outlier key channels per head -- swept over
the equal-memory settings (tokens, bits) in {(2048,16), (4096,8), (8192,4),
(16384,2)}, group 32, window 32, pool 7, 128 decode steps per setting.

One "step" = one pass of the whole hot path over that workload: for every
setting, compress all 32 layers (score, pool, top-k, gather, quantize, pack)
and then run 128 decode-attention steps over all 32 layers.  Inputs are
resident in HBM before timing starts.

`value` is decode-attention throughput in algorithmic GB/s (bytes of packed
cache + tail + q + out that one decode step must move, summed over the sweep,
divided by the HIP-event time of the decode calls).  The 32 layers' caches are
passed to the library as one batch per call -- valid here because the synthetic
decode queries do not depend on the previous layer's output; the same bytes
issued as 32 per-layer calls are reported next to it (`per_layer_calls`).
Compress throughput (prompt tokens/s through all 32 layers) is reported in the
same line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)

PEAK_HBM_GBS = 8000.0
PEAK_FP32_VECTOR_TFLOPS = 157.3
LAYERS, HQ, HKV, D, L, W, POOL, G = 32, 32, 8, 128, 32768, 32, 7, 32
SWEEP = [(2048, 16), (4096, 8), (8192, 4), (16384, 2)]
DECODE_STEPS = 128
CONFIG_ID = 2


def bytes_per_token(bits, group):
    return 4 * D if bits == 16 else 2 * (D * bits // 8 + 4 * D // group)


def decode_bytes(n_caches, n_kept, bits, group, tail):
    """Algorithmic bytes of one decode step over n_caches caches (all KV heads)."""
    return n_caches * HKV * (n_kept * bytes_per_token(bits, group) + tail * 4 * D) + 2 * n_caches * HQ * D * 2


def compress_bytes(n_caches, n_kept, bits, group):
    """Algorithmic bytes of compressing n_caches layers: K once, q_obs, selected V rows, outputs."""
    per = HKV * L * 2 * D + HQ * W * D * 2 + HKV * n_kept * 2 * D + HKV * (n_kept * bytes_per_token(bits, group) + W * 4 * D + 4 * n_kept)
    return n_caches * per


def read_traffic_note(kernel_tag):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE/WRITE_SIZE),
    recorded by hand in profiles/; None when no such note exists."""
    path = os.path.join(HERE, "profiles", f"traffic_{kernel_tag}.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(q_obs1, k1, v1, sm_scale):
    """The CPU checker, untuned, timed on the host cores on a bounded sample:
    one layer of the (8192 tokens, 4 bit) setting -- compress once, then as
    many decode steps as the GPU's timed loop runs per setting (about 10 s of
    CPU work in all)."""
    import numpy as np
    from oracle import kvqp_oracle as orc
    from paper_2412_12706_amd import synth
    t0 = time.perf_counter()
    cache, idx, _ = orc.compress(q_obs1, k1, v1, window=W, pool=POOL, budget=8192, bits=4, G=G, sm_scale=sm_scale,
                                 want_pooled=False)
    t1 = time.perf_counter()
    n_dec = DECODE_STEPS
    for s in range(n_dec):
        q = synth.decode_query_host(1, HQ, D, config=CONFIG_ID, layer=0, step=s)
        orc.decode_attn(q, cache, sm_scale)
    t2 = time.perf_counter()
    dec_gbs = decode_bytes(1, 8192, 4, G, W) * n_dec / (t2 - t1) / 1e9
    return {
        "value": round(dec_gbs, 4), "unit": "GB/s", "cores": orc.threads(), "kind": "oracle",
        "sample": f"1 of 32 layers at (8192 tok, 4 bit): 1 compress ({t1 - t0:.2f} s) + {n_dec} decode steps ({t2 - t1:.2f} s)",
        "compress_mtok_s_one_layer": round(L / (t1 - t0) / 1e6, 4),
        "compress_mtok_s_32_layers_extrapolated": round(L / (t1 - t0) / 1e6 / LAYERS, 5),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sweep-only", action="store_true",
                    help="only the timed sweep (used by the profiling commands so that their per-kernel averages "
                         "cover exactly the timed launches)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="kept for the profiling commands: the plain 1 GiB device copy (known size) that scales profiler "
                         "byte counters is always run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives or sharding are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2412_12706_amd import kvqp, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    kvqp.lib()  # fail loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    sm_scale = float(np.float32(D ** -0.5))

    # ---- inputs, resident in HBM: the 32 layers are the batch axis ----
    q_obs, k, v = synth.prompt_device(LAYERS, HQ, HKV, L, W, D, outlier=10.0, config=CONFIG_ID, device=dev)
    queries = [synth.decode_query_device(LAYERS, HQ, D, config=CONFIG_ID, step=s, device=dev) for s in range(DECODE_STEPS)]
    out = torch.empty_like(queries[0])

    settings = []
    for n_kept, bits in SWEEP:
        cfg = kvqp.Cfg(batch=LAYERS, n_q_heads=HQ, n_kv_heads=HKV, head_dim=D, seq_len=L, window=W, pool_kernel=POOL,
                       budget=n_kept, bits=bits, group_size=G, sm_scale=sm_scale)
        wc, wd = kvqp.workspace_bytes(cfg)
        settings.append({
            "cfg": cfg, "cache": kvqp.alloc_cache(cfg, device=dev), "ws_c": kvqp.alloc_workspace(wc, dev),
            "ws_d": kvqp.alloc_decode_workspace(cfg, dev), "n_kept": n_kept, "bits": bits,
            "t_compress_ms": 0.0, "t_decode_ms": 0.0,
        })

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def one_step(record):
        for s in settings:
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
            kvqp.compress(s["cfg"], q_obs, k, v, s["cache"], workspace=s["ws_c"])
            e1.record()
            for t in range(DECODE_STEPS):
                kvqp.decode_attn(s["cfg"], queries[t], s["cache"], out, s["ws_d"])
            e2.record()
            if record:
                s["_ev"] = s.get("_ev", []) + [(e0, e1, e2)]

    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(True)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    for s in settings:
        for e0, e1, e2 in s["_ev"]:
            s["t_compress_ms"] += e0.elapsed_time(e1)
            s["t_decode_ms"] += e1.elapsed_time(e2)

    # ---- per-setting figures ----
    sweep = []
    tot_bytes = tot_ms = 0.0
    for s in settings:
        n_calls = args.steps * DECODE_STEPS
        b = decode_bytes(LAYERS, s["n_kept"], s["bits"], G, W)
        us_call = s["t_decode_ms"] * 1e3 / n_calls
        gbs = b / (us_call * 1e-6) / 1e9
        c_ms = s["t_compress_ms"] / args.steps
        # two lower bounds of one decode launch: its bytes at the HBM peak, and its multiply-adds
        # (Gq per stored code, keys and values) at the plain fp32 vector peak -- what a kernel
        # that dequantizes with ordinary ALU instructions would be held to
        t_hbm_us = b / (PEAK_HBM_GBS * 1e9) * 1e6
        macs = LAYERS * HKV * s["n_kept"] * 2 * (HQ // HKV) * D
        t_alu_us = 2 * macs / (PEAK_FP32_VECTOR_TFLOPS * 1e12) * 1e6
        sweep.append({
            "tokens": s["n_kept"], "bits": s["bits"], "decode_us_per_step": round(us_call, 2),
            "decode_gbs": round(gbs, 1), "pct_of_8TBs": round(100 * gbs / PEAK_HBM_GBS, 1),
            "t_hbm_us": round(t_hbm_us, 1), "t_plain_alu_us": round(t_alu_us, 1),
            "bytes_per_step": b, "compress_ms_32_layers": round(c_ms, 3),
            "compress_mtok_s": round(L / (c_ms * 1e-3) / 1e6, 2),
            "compress_gbs": round(compress_bytes(LAYERS, s["n_kept"], s["bits"], G) / (c_ms * 1e-3) / 1e9, 1),
        })
        tot_bytes += b * n_calls
        tot_ms += s["t_decode_ms"]
    value = tot_bytes / (tot_ms * 1e-3) / 1e9

    def extra_legs():
        """Measurements outside the timed steps: per-layer calls, cache update, layer-wise counts, outlier filtering."""
        # ---- the same decode bytes issued as 32 per-layer calls (outside the timed steps) ----
        per_layer = []
        for s in settings:
            cfg1 = kvqp.Cfg(**{**s["cfg"].__dict__, "batch": 1})
            caches = []
            for l in range(LAYERS):
                bufs = {}
                for name, t in s["cache"].buffers.items():
                    per = t.numel() // LAYERS
                    bufs[name] = t[l * per:(l + 1) * per]
                caches.append(kvqp.Cache(bufs, s["cache"].n_kept, s["cache"].tail_len, s["cache"].tail_cap))
            ws1 = kvqp.alloc_decode_workspace(cfg1, dev)
            reps = 8
            for rep in range(reps + 1):
                if rep == 1:
                    torch.cuda.synchronize()
                    a, bq = ev(), ev()
                    a.record()
                for l in range(LAYERS):
                    kvqp.decode_attn(cfg1, queries[rep][l:l + 1], caches[l], out[l:l + 1], ws1)
            bq.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(bq) * 1e3 / reps
            b = decode_bytes(LAYERS, s["n_kept"], s["bits"], G, W)
            # the same with the caller's knowledge of its working set put into the cache hint: the layers
            # whose caches fit the memory-side cache together (240 MB) keep, the rest stream
            keep_layers = int(240e6 // (b / LAYERS))
            cfg_h = [kvqp.Cfg(**{**cfg1.__dict__, "decode_cache_hint": kvqp.CACHE_KEEP if l < keep_layers else kvqp.CACHE_STREAM})
                     for l in range(LAYERS)]
            for rep in range(reps + 1):
                if rep == 1:
                    torch.cuda.synchronize()
                    h0, h1 = ev(), ev()
                    h0.record()
                for l in range(LAYERS):
                    kvqp.decode_attn(cfg_h[l], queries[rep][l:l + 1], caches[l], out[l:l + 1], ws1)
            h1.record()
            torch.cuda.synchronize()
            us_h = h0.elapsed_time(h1) * 1e3 / reps
            # the same 32 launches recorded once in a HIP graph and replayed (no host work per launch)
            us_g = None
            try:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for l in range(LAYERS):
                        kvqp.decode_attn(cfg1, queries[0][l:l + 1], caches[l], out[l:l + 1], ws1)
                graph.replay()
                torch.cuda.synchronize()
                g0, g1 = ev(), ev()
                g0.record()
                for rep in range(reps):
                    graph.replay()
                g1.record()
                torch.cuda.synchronize()
                us_g = g0.elapsed_time(g1) * 1e3 / reps
                del graph
            except RuntimeError as e:       # (a leg outside the timed steps must not take the benchmark down)
                print(f"bench.py: graph replay of the per-layer calls skipped: {e}", file=sys.stderr)
            per_layer.append({"tokens": s["n_kept"], "bits": s["bits"], "decode_us_per_step": round(us, 1),
                              "decode_gbs": round(b / (us * 1e-6) / 1e9, 1), "hinted_us_per_step": round(us_h, 1),
                              "hinted_keep_layers": min(keep_layers, LAYERS), "graph_us_per_step": None if us_g is None else round(us_g, 1),
                              "graph_gbs": None if us_g is None else round(b / (us_g * 1e-6) / 1e9, 1)})

        # ---- decode-time cache update (outside the timed steps): 32 decoded tokens per layer move from the
        # full-precision tail into the 4-bit part of a cache laid out with room to grow ----
        s4 = next(s for s in settings if s["bits"] == 4)
        grow = kvqp.alloc_cache(s4["cfg"], tail_cap=W + G, device=dev, n_cap=s4["n_kept"] + 64)
        kvqp.compress(s4["cfg"], q_obs, k, v, grow, workspace=s4["ws_c"])
        grow.buffers["tail_k"].view(torch.float16).normal_()
        grow.buffers["tail_v"].view(torch.float16).normal_()
        reps = 20
        for rep in range(reps + 2):
            if rep == 2:
                torch.cuda.synchronize()
                a0, a1 = ev(), ev()
                a0.record()
            grow.n_kept, grow.tail_len = s4["n_kept"], W + G      # (the counts live on the host; the rows are re-quantized)
            kvqp.append_tail(s4["cfg"], grow, G)
        a1.record()
        torch.cuda.synchronize()
        append_us = a0.elapsed_time(a1) * 1e3 / reps
        del grow

        # ---- layer-wise token counts (outside the timed steps): the 4-bit setting's memory spread over the
        # layers as a falling schedule, 1.5x the mean in the first layer down to 0.5x in the last, one batch ----
        mean = s4["n_kept"]
        counts = [int(round(mean * (1.5 - l / (LAYERS - 1)) / 64)) * 64 for l in range(LAYERS)]
        cfg_r = kvqp.Cfg(**{**s4["cfg"].__dict__, "budget": max(counts)})
        rag = kvqp.alloc_cache(cfg_r, device=dev, ragged=True)
        ws_rc, ws_rd = kvqp.alloc_workspace(kvqp.workspace_bytes(cfg_r)[0], dev), kvqp.alloc_decode_workspace(cfg_r, dev)
        head_counts = [counts[h // HKV] for h in range(LAYERS * HKV)]
        reps = 3
        for rep in range(reps + 1):
            if rep == 1:
                torch.cuda.synchronize()
                r0, r1 = ev(), ev()
                r0.record()
            kvqp.compress_ragged(cfg_r, q_obs, k, v, head_counts, rag, workspace=ws_rc)
        r1.record()
        for t in range(DECODE_STEPS):        # a full untimed round first: the first calls after a compress run slow
            kvqp.decode_attn(cfg_r, queries[t], rag, out, ws_rd)
        torch.cuda.synchronize()
        r2, r3 = ev(), ev()
        r2.record()
        for t in range(DECODE_STEPS):
            kvqp.decode_attn(cfg_r, queries[t], rag, out, ws_rd)
        r3.record()
        torch.cuda.synchronize()
        rag_bytes = sum(decode_bytes(1, n, 4, G, W) for n in counts)
        rag_us = r2.elapsed_time(r3) * 1e3 / DECODE_STEPS
        layer_wise = {
            "counts": f"{counts[0]} .. {counts[-1]} tokens per layer (mean {sum(counts) // LAYERS}), 4 bit",
            "compress_ms_32_layers": round(r0.elapsed_time(r1) / reps, 3), "decode_us_per_step": round(rag_us, 2),
            "decode_gbs": round(rag_bytes / (rag_us * 1e-6) / 1e9, 1), "bytes_per_step": rag_bytes,
        }
        del rag

        # ---- outlier filtering at the paper's threshold (outside the timed steps): the 4-bit setting with
        # |x| > 6 kept beside the codes, four slot words per token row and tensor ----
        cfg_o = kvqp.Cfg(**{**s4["cfg"].__dict__, "outlier_threshold": 6.0})
        oc_cache = kvqp.alloc_cache(cfg_o, device=dev)
        ws_oc, ws_od = kvqp.alloc_workspace(kvqp.workspace_bytes(cfg_o)[0], dev), kvqp.alloc_decode_workspace(cfg_o, dev)
        reps = 3
        for rep in range(reps + 1):
            if rep == 1:
                torch.cuda.synchronize()
                o0, o1 = ev(), ev()
                o0.record()
            kvqp.compress(cfg_o, q_obs, k, v, oc_cache, workspace=ws_oc)
        o1.record()
        for t in range(DECODE_STEPS):
            kvqp.decode_attn(cfg_o, queries[t], oc_cache, out, ws_od)
        torch.cuda.synchronize()
        o2, o3 = ev(), ev()
        o2.record()
        for t in range(DECODE_STEPS):
            kvqp.decode_attn(cfg_o, queries[t], oc_cache, out, ws_od)
        o3.record()
        torch.cuda.synchronize()
        slot_bytes = LAYERS * HKV * s4["n_kept"] * 2 * 16
        o_bytes = decode_bytes(LAYERS, s4["n_kept"], 4, G, W) + slot_bytes
        o_us = o2.elapsed_time(o3) * 1e3 / DECODE_STEPS
        n_slots = int((oc_cache.buffers["k_out"].view(torch.int32) != 0).sum().item())
        outlier_leg = {
            "threshold": 6.0, "bits": 4, "tokens": s4["n_kept"],
            "key_outliers_per_row": round(n_slots / (LAYERS * HKV * s4["n_kept"]), 2),
            "compress_ms_32_layers": round(o0.elapsed_time(o1) / reps, 3), "decode_us_per_step": round(o_us, 2),
            "decode_gbs": round(o_bytes / (o_us * 1e-6) / 1e9, 1), "bytes_per_step": o_bytes,
            "note": "the decode kernel's outlier variant runs two waves per SIMD (eight per workgroup) instead of three",
        }
        del oc_cache

        # ---- per-token key groups (the FlexGen axis of the paper's ablation and of its head-level methods) ----
        cfg_t = kvqp.Cfg(**{**s4["cfg"].__dict__, "key_axis": kvqp.KEY_PER_TOKEN})
        tc = kvqp.alloc_cache(cfg_t, device=dev)
        ws_tc, ws_td = kvqp.alloc_workspace(kvqp.workspace_bytes(cfg_t)[0], dev), kvqp.alloc_decode_workspace(cfg_t, dev)
        for rep in range(reps + 1):
            if rep == 1:
                torch.cuda.synchronize()
                t0_, t1_ = ev(), ev()
                t0_.record()
            kvqp.compress(cfg_t, q_obs, k, v, tc, workspace=ws_tc)
        t1_.record()
        for t in range(DECODE_STEPS):
            kvqp.decode_attn(cfg_t, queries[t], tc, out, ws_td)
        torch.cuda.synchronize()
        t2_, t3_ = ev(), ev()
        t2_.record()
        for t in range(DECODE_STEPS):
            kvqp.decode_attn(cfg_t, queries[t], tc, out, ws_td)
        t3_.record()
        torch.cuda.synchronize()
        t_bytes = decode_bytes(LAYERS, s4["n_kept"], 4, G, W)      # same count: a scale and a zero per 32 elements either way
        t_us = t2_.elapsed_time(t3_) * 1e3 / DECODE_STEPS
        token_keys = {
            "bits": 4, "tokens": s4["n_kept"], "compress_ms_32_layers": round(t0_.elapsed_time(t1_) / reps, 3),
            "decode_us_per_step": round(t_us, 2), "decode_gbs": round(t_bytes / (t_us * 1e-6) / 1e9, 1),
            "bytes_per_step": t_bytes,
        }
        del tc

        # ---- the sweep's launches with the memory-side cache flushed before each one (outside the timed
        # steps): consecutive decode steps re-read the same cache, and the library leaves the first 240 MB
        # of a large launch's working set resident in the 256 MB memory-side cache while the rest streams
        # past it; this leg shows the launches with nothing resident (2 GiB are read before each; a reading
        # flush, so that no write-back of dirty lines lands inside the timed interval) ----
        f_src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        f_dst = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        cold = []
        for s in settings:
            rec = {"tokens": s["n_kept"], "bits": s["bits"]}
            b = decode_bytes(LAYERS, s["n_kept"], s["bits"], G, W)
            # (library's choice of loads, then the hint of a caller who knows the cache will not survive)
            for key, hint in (("", kvqp.CACHE_AUTO), ("stream_hint_", kvqp.CACHE_STREAM)):
                cfg_h = kvqp.Cfg(**{**s["cfg"].__dict__, "decode_cache_hint": hint})
                pairs = []
                for t in range(17):
                    sink += f_src.sum()
                    sink += f_dst.sum()
                    a, bq = ev(), ev()
                    a.record()
                    kvqp.decode_attn(cfg_h, queries[t], s["cache"], out, s["ws_d"])
                    bq.record()
                    pairs.append((a, bq))
                torch.cuda.synchronize()
                us = sorted(x.elapsed_time(y) * 1e3 for x, y in pairs[1:])[len(pairs) // 2 - 1]
                rec[key + "decode_us_per_step"] = round(us, 2)
                rec[key + "decode_gbs"] = round(b / (us * 1e-6) / 1e9, 1)
                rec[key + "pct_of_8TBs"] = round(100 * b / (us * 1e-6) / 1e9 / PEAK_HBM_GBS, 1)
            cold.append(rec)
        del f_src, f_dst
        return per_layer, append_us, layer_wise, outlier_leg, token_keys, cold

    per_layer, append_us, layer_wise, outlier_leg, token_keys, cold = (None,) * 6 if args.sweep_only else extra_legs()

    # ---- roofline of the dominant kernel: the decode launch that takes most of the step ----
    dom = max(range(len(settings)), key=lambda i: settings[i]["t_decode_ms"])
    dom_s, dom_r = settings[dom], sweep[dom]
    tag = f"decode_attn_pipe_{dom_s['bits']}bit_cfg2"
    roofline = {
        "bound": "hbm", "kernel": f"decode_attn_pipe<{dom_s['bits']} bit> (one launch per decode call; HIP events around the {DECODE_STEPS} calls)",
        "achieved": dom_r["decode_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
        "frac": round(dom_r["decode_gbs"] / PEAK_HBM_GBS, 4), "traffic": read_traffic_note(tag),
        "algorithmic_bytes_per_launch": dom_r["bytes_per_step"], "launch_us": dom_r["decode_us_per_step"],
        "roofline_time_us": max(dom_r["t_hbm_us"], dom_r["t_plain_alu_us"]),
        "note": "the products run on the matrix cores with the codes as operands, so the plain-ALU bound does not "
                "apply; at 2 bits the measured limit is vector-instruction issue for operand preparation; in the timed loop "
                "consecutive steps re-read the same cache and part of the bytes comes from the 256 MB memory-side cache "
                "(the traffic counter sits before it): cold_memory_side_cache has the launches with nothing resident",
    }

    # ---- what a plain device copy reaches on this machine (1 GiB read + 1 GiB written per copy) ----
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)
    dst.copy_(src)                           # also the known-size dispatch that calibrates profiler byte counters
    torch.cuda.synchronize()
    c0, c1 = ev(), ev()
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(q_obs[:1].cpu().numpy(), k[:1].cpu().numpy(), v[:1].cpu().numpy(), sm_scale)

    c4 = next(r for r in sweep if r["bits"] == 4)
    line = {
        "metric": "packed-KV decode attn HBM GB/s (% of peak) + compress Mtok/s at 32k ctx",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(wall_ms / args.steps, 3), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {
            "workload": "configs[1]: Llama-3-8B-shaped KV, 32 layers x (32 Q / 8 KV heads, d=128), batch 1, L=32768, "
                        "sweep (tokens,bits) in {(2048,16),(4096,8),(8192,4),(16384,2)}, group 32, window 32, pool 7, "
                        "128 decode steps per setting",
            "launch": "all 32 layers' caches as one batch per library call",
            "value_is": "sum of algorithmic decode bytes over the sweep / sum of decode HIP-event time",
        },
        "pct_of_peak_hbm": round(100 * value / PEAK_HBM_GBS, 1),
        "device_copy_gbs": round(copy_gbs, 1), "pct_of_device_copy": round(100 * value / copy_gbs, 1),
        "compress_mtok_s": c4["compress_mtok_s"],
        "compress_note": "prompt tokens/s through all 32 layers at the (8192 tok, 4 bit) setting",
        "append_tail_us": None if append_us is None else round(append_us, 2),
        "append_note": f"kvqp_append_tail of {G} tokens per cache, 32 layers as one batch, 4-bit setting",
        "layer_wise_counts": layer_wise, "outlier_filtering": outlier_leg, "per_token_keys": token_keys,
        "sweep": sweep, "per_layer_calls": per_layer,
        "cold_memory_side_cache": cold,
        "cold_value_gbs": None if cold is None else round(
            sum(decode_bytes(LAYERS, c["tokens"], c["bits"], G, W) for c in cold)
            / sum(min(c["decode_us_per_step"], c["stream_hint_decode_us_per_step"]) for c in cold) / 1e3, 1),
        "cold_note": "each launch timed alone (median of 16, HIP events around the one launch) right after 2 GiB of "
                     "other data were read, so nothing of the cache is resident in the 256 MB memory-side cache; in "
                     "the timed sweep consecutive steps re-read the same cache and up to 240 MB of it stay resident; "
                     "stream_hint_*: the same with cfg.decode_cache_hint = KVQP_CACHE_STREAM (every load non-temporal); "
                     "cold_value_gbs: the sweep figure from the better of the two cold times of each setting",
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
