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
divided by the HIP-event time of the decode calls) WITH NOTHING RESIDENT IN THE
CHIP'S 256 MB MEMORY-SIDE CACHE: every setting keeps several identical copies of
its compressed cache (together well over 1 GB) and consecutive decode steps read
different copies, as a real decode step finds its cache after the model's weights
have passed through the chip.  The loop that re-reads one copy, where part of the
bytes never comes from HBM, is reported separately (`warm_same_cache_loop`).
The 32 layers' caches are passed to the library as one batch per call -- valid
here because the synthetic decode queries do not depend on the previous layer's
output; the same bytes issued as 32 per-layer calls are reported next to it
(`per_layer_calls`).  Compress throughput (prompt tokens/s through all 32 layers)
is in the same line, as are the other configurations' shapes (`other_configs`).

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import math
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
ROTATE_BYTES = 1.2e9          # copies of a cache the decode steps rotate over add up to at least this
# which resource the issue counters (profiles/issue_counters_*) show as binding, per bit width
BOUND = {16: "hbm", 8: "hbm", 4: "hbm", 2: "alu"}


def bytes_per_token(bits, group):
    return 4 * D if bits == 16 else 2 * (D * bits // 8 + 4 * D // group)


def decode_bytes(n_caches, n_kept, bits, group, tail, hkv=HKV, hq=HQ):
    """Algorithmic bytes of one decode step over n_caches caches (all KV heads)."""
    return n_caches * hkv * (n_kept * bytes_per_token(bits, group) + tail * 4 * D) + 2 * n_caches * hq * D * 2


def compress_bytes(n_caches, n_kept, bits, group, seq=L, win=W, hkv=HKV, hq=HQ):
    """Algorithmic bytes of compressing n_caches layers: K once, q_obs, selected V rows, outputs."""
    per = hkv * seq * 2 * D + hq * win * D * 2 + hkv * n_kept * 2 * D + hkv * (n_kept * bytes_per_token(bits, group) + win * 4 * D + 4 * n_kept)
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
    """The CPU checker, untuned, timed on the host cores on a bounded sample of the headline workload:
    one layer of the (8192 tokens, 4 bit) setting -- compress once, then as many decode steps as the
    GPU's timed loop runs per setting -- on all cores (about 10 s), and a smaller sample on one thread
    (one KV head's compress, 16 decode steps; about 10 s)."""
    from oracle import kvqp_oracle as orc
    from paper_2412_12706_amd import synth
    n_threads = orc.threads()
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
    # one thread: the first KV head's share of the compress, 16 decode steps of the layer
    orc.set_threads(1)
    gq = HQ // HKV
    s0 = time.perf_counter()
    orc.compress(q_obs1[:, :gq], k1[:, :1], v1[:, :1], window=W, pool=POOL, budget=8192, bits=4, G=G, sm_scale=sm_scale,
                 want_pooled=False)
    s1 = time.perf_counter()
    n1 = 16
    for s in range(n1):
        q = synth.decode_query_host(1, HQ, D, config=CONFIG_ID, layer=0, step=s)
        orc.decode_attn(q, cache, sm_scale)
    s2 = time.perf_counter()
    orc.set_threads(n_threads)
    return {
        "value": round(dec_gbs, 4), "unit": "GB/s", "cores": n_threads, "kind": "oracle",
        "sample": f"1 of 32 layers at (8192 tok, 4 bit): 1 compress ({t1 - t0:.2f} s) + {n_dec} decode steps ({t2 - t1:.2f} s)",
        "compress_mtok_s_one_layer": round(L / (t1 - t0) / 1e6, 4),
        "compress_mtok_s_32_layers_extrapolated": round(L / (t1 - t0) / 1e6 / LAYERS, 5),
        "single_thread": {
            "decode_gbs": round(decode_bytes(1, 8192, 4, G, W) * n1 / (s2 - s1) / 1e9, 4),
            "compress_mtok_s_one_layer_extrapolated": round(L / ((s1 - s0) * HKV) / 1e6, 5),
            "sample": f"1 of 8 KV heads of that layer compressed ({s1 - s0:.2f} s, x8 for the layer) + {n1} decode steps of the layer ({s2 - s1:.2f} s)",
        },
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

    def ev():
        return torch.cuda.Event(enable_timing=True)

    def clone_cache(c):
        return kvqp.Cache({n: t.clone() for n, t in c.buffers.items()}, c.n_kept, c.tail_len, c.tail_cap, c.n_cap)

    # ---- inputs, resident in HBM: the 32 layers are the batch axis ----
    q_obs, k, v = synth.prompt_device(LAYERS, HQ, HKV, L, W, D, outlier=10.0, config=CONFIG_ID, device=dev)
    queries = [synth.decode_query_device(LAYERS, HQ, D, config=CONFIG_ID, step=s, device=dev) for s in range(DECODE_STEPS)]
    out = torch.empty_like(queries[0])

    settings = []
    for n_kept, bits in SWEEP:
        cfg = kvqp.Cfg(batch=LAYERS, n_q_heads=HQ, n_kv_heads=HKV, head_dim=D, seq_len=L, window=W, pool_kernel=POOL,
                       budget=n_kept, bits=bits, group_size=G, sm_scale=sm_scale)
        n_copies = max(3, math.ceil(ROTATE_BYTES / decode_bytes(LAYERS, n_kept, bits, G, W)))
        settings.append({
            "cfg": cfg, "caches": [kvqp.alloc_cache(cfg, device=dev) for _ in range(n_copies)],
            "ws_c": kvqp.alloc_workspace(kvqp.workspace_bytes(cfg)[0], dev),
            "ws_d": kvqp.alloc_decode_workspace(cfg, dev), "n_kept": n_kept, "bits": bits,
            "t_compress_ms": 0.0, "t_decode_ms": 0.0, "_ev": [],
        })
    # every copy holds the compressed prompt before anything is timed
    for s in settings:
        for c in s["caches"]:
            kvqp.compress(s["cfg"], q_obs, k, v, c, workspace=s["ws_c"])
    torch.cuda.synchronize()

    def one_step(record, i_step):
        for s in settings:
            n = len(s["caches"])
            e0, e1, e2 = ev(), ev(), ev()
            e0.record()
            kvqp.compress(s["cfg"], q_obs, k, v, s["caches"][i_step % n], workspace=s["ws_c"])
            e1.record()
            for t in range(DECODE_STEPS):       # consecutive decode steps read different copies: nothing is resident
                kvqp.decode_attn(s["cfg"], queries[t], s["caches"][(i_step + 1 + t) % n], out, s["ws_d"])
            e2.record()
            if record:
                s["_ev"].append((e0, e1, e2))

    for i in range(args.warmup):
        one_step(False, i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        one_step(True, args.warmup + i)
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
            "tokens": s["n_kept"], "bits": s["bits"], "cache_copies_rotated": len(s["caches"]),
            "decode_us_per_step": round(us_call, 2),
            "decode_gbs": round(gbs, 1), "pct_of_8TBs": round(100 * gbs / PEAK_HBM_GBS, 1),
            "bound": BOUND[s["bits"]],
            "t_hbm_us": round(t_hbm_us, 1), "t_plain_alu_us": round(t_alu_us, 1),
            "algorithmic_tflops": round(2 * macs / (us_call * 1e-6) / 1e12, 1),
            "bytes_per_step": b, "compress_ms_32_layers": round(c_ms, 3),
            "compress_mtok_s": round(L / (c_ms * 1e-3) / 1e6, 2),
            "compress_gbs": round(compress_bytes(LAYERS, s["n_kept"], s["bits"], G) / (c_ms * 1e-3) / 1e9, 1),
        })
        tot_bytes += b * n_calls
        tot_ms += s["t_decode_ms"]
    value = tot_bytes / (tot_ms * 1e-3) / 1e9

    def timed_loop(fn, n, rounds_before=1):
        """n calls of fn(t) between two events, after rounds_before untimed rounds; microseconds per call."""
        for _ in range(rounds_before):
            for t in range(n):
                fn(t)
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for t in range(n):
            fn(t)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / n

    def extra_legs():
        """Measurements outside the timed steps."""
        # ---- the loop that re-reads ONE copy (what the 128 steps of a setting would do without the rotation):
        # part of every step's bytes then comes from the memory-side cache, not from HBM ----
        warm = []
        for s in settings:
            rec = {"tokens": s["n_kept"], "bits": s["bits"]}
            b = decode_bytes(LAYERS, s["n_kept"], s["bits"], G, W)
            for key, hint in (("", kvqp.CACHE_AUTO), ("keep_hint_", kvqp.CACHE_KEEP)):
                cfg_h = kvqp.Cfg(**{**s["cfg"].__dict__, "decode_cache_hint": hint})
                us = timed_loop(lambda t: kvqp.decode_attn(cfg_h, queries[t], s["caches"][0], out, s["ws_d"]), DECODE_STEPS)
                rec[key + "decode_us_per_step"] = round(us, 2)
                rec[key + "decode_gbs_algorithmic"] = round(b / (us * 1e-6) / 1e9, 1)
            warm.append(rec)

        # ---- the same decode bytes issued as 32 per-layer calls ----
        per_layer = []
        for s in settings:
            cfg1 = kvqp.Cfg(**{**s["cfg"].__dict__, "batch": 1})
            layer_caches = []
            for c in s["caches"][:2]:                   # two copies alternate, so a layer's cache is not re-read at once
                for l in range(LAYERS):
                    bufs = {}
                    for name, t in c.buffers.items():
                        per = t.numel() // LAYERS
                        bufs[name] = t[l * per:(l + 1) * per]
                    layer_caches.append(kvqp.Cache(bufs, c.n_kept, c.tail_len, c.tail_cap))
            ws1 = kvqp.alloc_decode_workspace(cfg1, dev)
            n_calls = 2 * LAYERS

            def fn(t):
                l = t % LAYERS
                kvqp.decode_attn(cfg1, queries[t // LAYERS][l:l + 1], layer_caches[t], out[l:l + 1], ws1)
            us = timed_loop(fn, n_calls, rounds_before=2) * LAYERS
            b = decode_bytes(LAYERS, s["n_kept"], s["bits"], G, W)
            # the same launches recorded once in a HIP graph and replayed (no host work per launch)
            us_g = None
            try:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    for t in range(n_calls):
                        fn(t)
                graph.replay()
                torch.cuda.synchronize()
                g0, g1 = ev(), ev()
                g0.record()
                for rep in range(4):
                    graph.replay()
                g1.record()
                torch.cuda.synchronize()
                us_g = g0.elapsed_time(g1) * 1e3 / 4 / 2
                del graph
            except RuntimeError as e:       # (a leg outside the timed steps must not take the benchmark down)
                print(f"bench.py: graph replay of the per-layer calls skipped: {e}", file=sys.stderr)
            per_layer.append({"tokens": s["n_kept"], "bits": s["bits"], "decode_us_per_step": round(us, 1),
                              "us_per_layer_call": round(us / LAYERS, 2),
                              "decode_gbs": round(b / (us * 1e-6) / 1e9, 1),
                              "graph_us_per_step": None if us_g is None else round(us_g, 1),
                              "graph_gbs": None if us_g is None else round(b / (us_g * 1e-6) / 1e9, 1)})

        # ---- decode-time cache update: 32 decoded tokens per layer move from the
        # full-precision tail into the 4-bit part of a cache laid out with room to grow ----
        s4 = next(s for s in settings if s["bits"] == 4)
        grow = kvqp.alloc_cache(s4["cfg"], tail_cap=W + G, device=dev, n_cap=s4["n_kept"] + 64)
        kvqp.compress(s4["cfg"], q_obs, k, v, grow, workspace=s4["ws_c"])
        grow.buffers["tail_k"].view(torch.float16).normal_()
        grow.buffers["tail_v"].view(torch.float16).normal_()

        def append_once(t):
            grow.n_kept, grow.tail_len = s4["n_kept"], W + G      # (the counts live on the host; the rows are re-quantized)
            kvqp.append_tail(s4["cfg"], grow, G)
        append_us = timed_loop(append_once, 20, rounds_before=1)
        del grow

        def leg(cfg_x, make_caches, compress_into, nbytes, reps=3):
            """Compress time and decode time (three rotating copies) of a variant of the 4-bit setting."""
            caches = make_caches()
            ws_c = kvqp.alloc_workspace(kvqp.workspace_bytes(cfg_x)[0], dev)
            ws_d = kvqp.alloc_decode_workspace(cfg_x, dev)
            for c in caches:
                compress_into(c, ws_c)
            c_us = timed_loop(lambda t: compress_into(caches[t % len(caches)], ws_c), reps, rounds_before=0)
            d_us = timed_loop(lambda t: kvqp.decode_attn(cfg_x, queries[t], caches[t % len(caches)], out, ws_d), DECODE_STEPS)
            return caches, {"compress_ms_32_layers": round(c_us / 1e3, 3), "decode_us_per_step": round(d_us, 2),
                            "decode_gbs": round(nbytes / (d_us * 1e-6) / 1e9, 1), "bytes_per_step": nbytes}

        # ---- layer-wise token counts: the 4-bit setting's memory spread over the layers as a falling
        # schedule, 1.5x the mean in the first layer down to 0.5x in the last, one batch ----
        mean = s4["n_kept"]
        counts = [int(round(mean * (1.5 - l / (LAYERS - 1)) / 64)) * 64 for l in range(LAYERS)]
        cfg_r = kvqp.Cfg(**{**s4["cfg"].__dict__, "budget": max(counts)})
        head_counts = [counts[h // HKV] for h in range(LAYERS * HKV)]
        rag, layer_wise = leg(cfg_r, lambda: [kvqp.alloc_cache(cfg_r, device=dev, ragged=True) for _ in range(3)],
                              lambda c, ws: kvqp.compress_ragged(cfg_r, q_obs, k, v, head_counts, c, workspace=ws),
                              sum(decode_bytes(1, n, 4, G, W) for n in counts))
        layer_wise["counts"] = f"{counts[0]} .. {counts[-1]} tokens per layer (mean {sum(counts) // LAYERS}), 4 bit"
        del rag

        # ---- outlier filtering at the paper's threshold: the 4-bit setting with |x| > 6 kept beside the
        # codes, four slot words per token row and tensor ----
        cfg_o = kvqp.Cfg(**{**s4["cfg"].__dict__, "outlier_threshold": 6.0, "outlier_overflow_cap": 4096})
        slot_bytes = LAYERS * HKV * s4["n_kept"] * 2 * (16 + 4 / 32)      # slot words and the overflow lists' prefix counts
        slot_bytes = int(slot_bytes)
        oc, outlier_leg = leg(cfg_o, lambda: [kvqp.alloc_cache(cfg_o, device=dev) for _ in range(3)],
                              lambda c, ws: kvqp.compress(cfg_o, q_obs, k, v, c, workspace=ws),
                              decode_bytes(LAYERS, s4["n_kept"], 4, G, W) + slot_bytes)
        n_slots = int((oc[0].buffers["k_out"].view(torch.int32) != 0).sum().item())
        outlier_leg.update({"threshold": 6.0, "bits": 4, "tokens": s4["n_kept"],
                            "key_outliers_per_row": round(n_slots / (LAYERS * HKV * s4["n_kept"]), 2),
                            "note": "the decode kernel's outlier variant runs two waves per SIMD (eight per workgroup) instead of three"})
        del oc

        # ---- per-token key groups (the FlexGen axis of the paper's ablation and of its head-level methods) ----
        cfg_t = kvqp.Cfg(**{**s4["cfg"].__dict__, "key_axis": kvqp.KEY_PER_TOKEN})
        tc, token_keys = leg(cfg_t, lambda: [kvqp.alloc_cache(cfg_t, device=dev) for _ in range(3)],
                             lambda c, ws: kvqp.compress(cfg_t, q_obs, k, v, c, workspace=ws),
                             decode_bytes(LAYERS, s4["n_kept"], 4, G, W))   # same count: a scale and a zero per 32 elements either way
        token_keys.update({"bits": 4, "tokens": s4["n_kept"]})
        del tc
        return warm, per_layer, append_us, layer_wise, outlier_leg, token_keys

    def other_configs():
        """The other configurations of the benchmark spec at their real shapes (outside the timed steps): one call's
        prompt resident, decode calls rotating over identical copies of that call's cache."""
        res = []
        # name, sequences x layers in one call, Hq, Hkv, L, W, tokens, bits, group, key axis, outlier factor, layers of the model, layers per call, config id
        for name, B_, hq_, hkv_, L_, W_, n_kept_, bits_, g_, axis_, outl_, n_layers_, lpc_, cid in (
                ("configs[2]: batch 16, L=16384, 4096 tokens at 4 bits; one call per layer", 16, 32, 8, 16384, 32, 4096, 4, 32, 0, 10.0, 32, 1, 3),
                ("configs[4]: 70B-shaped (64 Q / 8 KV heads, 80 layers), batch 8, L=32768, 8192 tokens at 4 bits; one call per layer", 8, 64, 8, 32768, 32, 8192, 4, 32, 0, 10.0, 80, 1, 5),
                ("configs[4] ablation: the same with per-token key groups", 8, 64, 8, 32768, 32, 8192, 4, 32, 1, 10.0, 80, 1, 5),
                ("configs[3]: batch 1, L=131072, 16384 tokens at 2 bits in groups of 64, window 64, x20 outlier channels; 8 of the 32 layers as one batch per call", 8, 32, 8, 131072, 64, 16384, 2, 64, 0, 20.0, 32, 8, 4)):
            qo, kk, vv = synth.prompt_device(B_, hq_, hkv_, L_, W_, D, outlier=outl_, config=cid, device=dev)
            cfg_x = kvqp.Cfg(batch=B_, n_q_heads=hq_, n_kv_heads=hkv_, head_dim=D, seq_len=L_, window=W_, pool_kernel=POOL,
                             budget=n_kept_, bits=bits_, group_size=g_, key_axis=axis_, sm_scale=sm_scale)
            b = B_ * hkv_ * (n_kept_ * bytes_per_token(bits_, g_) + W_ * 4 * D) + 2 * B_ * hq_ * D * 2
            n_copies = max(3, math.ceil(ROTATE_BYTES / b))
            ws_c = kvqp.alloc_workspace(kvqp.workspace_bytes(cfg_x)[0], dev)
            ws_d = kvqp.alloc_decode_workspace(cfg_x, dev)
            first = kvqp.alloc_cache(cfg_x, device=dev)
            kvqp.compress(cfg_x, qo, kk, vv, first, workspace=ws_c)
            c_us = timed_loop(lambda t: kvqp.compress(cfg_x, qo, kk, vv, first, workspace=ws_c), 3, rounds_before=0)
            caches = [first] + [clone_cache(first) for _ in range(n_copies - 1)]
            qs = [synth.decode_query_device(B_, hq_, D, config=cid, step=s, device=dev) for s in range(8)]
            o = torch.empty_like(qs[0])
            d_us = timed_loop(lambda t: kvqp.decode_attn(cfg_x, qs[t % 8], caches[t % n_copies], o, ws_d), 4 * n_copies)
            cb = (B_ * hkv_ * L_ * 2 * D + B_ * hq_ * W_ * D * 2 + B_ * hkv_ * n_kept_ * 2 * D
                  + B_ * hkv_ * (n_kept_ * bytes_per_token(bits_, g_) + W_ * 4 * D + 4 * n_kept_))
            res.append({"workload": name, "decode_us_per_call": round(d_us, 2), "bytes_per_call": b,
                        "decode_gbs": round(b / (d_us * 1e-6) / 1e9, 1),
                        "pct_of_8TBs": round(100 * b / (d_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 1),
                        "cache_copies_rotated": n_copies, "compress_ms_per_call": round(c_us / 1e3, 3),
                        # prompt tokens of the whole batch per second through all layers of the model
                        "compress_mtok_s_all_layers": round((B_ // lpc_) * L_ / (c_us * 1e-6 * n_layers_ / lpc_) / 1e6, 2),
                        "compress_gbs": round(cb / (c_us * 1e-6) / 1e9, 1)})
            del qo, kk, vv, caches, first, qs, o
            torch.cuda.empty_cache()
        return res

    warm = per_layer = append_us = layer_wise = outlier_leg = token_keys = others = None
    if not args.sweep_only:
        warm, per_layer, append_us, layer_wise, outlier_leg, token_keys = extra_legs()

    # ---- roofline of the dominant kernel: the decode launch that takes most of the step ----
    dom = max(range(len(settings)), key=lambda i: settings[i]["t_decode_ms"])
    dom_s, dom_r = settings[dom], sweep[dom]
    tag = f"decode_attn_pipe_{dom_s['bits']}bit_cfg2"
    hbm = {"achieved": dom_r["decode_gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(dom_r["decode_gbs"] / PEAK_HBM_GBS, 4)}
    alu = {"achieved": dom_r["algorithmic_tflops"], "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
           "frac": round(dom_r["algorithmic_tflops"] / PEAK_FP32_VECTOR_TFLOPS, 4)}
    main_r = alu if dom_r["bound"] == "alu" else hbm
    roofline = {
        "bound": dom_r["bound"],
        "kernel": f"decode_attn_pipe<{dom_s['bits']} bit> (one launch per decode call; HIP events around the {DECODE_STEPS} calls "
                  "of a step, rotating cache copies)",
        "achieved": main_r["achieved"], "peak": main_r["peak"], "unit": main_r["unit"], "frac": main_r["frac"],
        "traffic": read_traffic_note(tag), "hbm": hbm, "alu": alu,
        "algorithmic_bytes_per_launch": dom_r["bytes_per_step"], "launch_us": dom_r["decode_us_per_step"],
        "algorithmic_flops_per_launch": 2 * LAYERS * HKV * dom_s["n_kept"] * 2 * (HQ // HKV) * D,
        "roofline_time_us": max(dom_r["t_hbm_us"], dom_r["t_plain_alu_us"]),
        "note": "bound per setting from the issue counters (profiles/issue_counters_bench_config2.txt): HBM at 16, 8 and 4 bits; at "
                "2 bits vector-instruction issue (unpacking the codes and preparing the scaled operands of the matrix products), so "
                "that launch is held against the plain fp32 vector peak with 2 flops x Gq x (K and V) x D per stored token-head as the "
                "algorithmic work, and the HBM fraction is given beside it",
    }

    cpu = None
    if not args.no_cpu_baseline and not args.sweep_only:
        cpu = cpu_baseline(q_obs[:1].cpu().numpy(), k[:1].cpu().numpy(), v[:1].cpu().numpy(), sm_scale)

    if not args.sweep_only:
        del settings, q_obs, k, v
        torch.cuda.empty_cache()
        others = other_configs()

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
            "value_is": "sum of algorithmic decode bytes over the sweep / sum of decode HIP-event time, consecutive decode "
                        "steps reading different copies of the cache so that nothing is resident in the 256 MB memory-side cache",
        },
        "pct_of_peak_hbm": round(100 * value / PEAK_HBM_GBS, 1),
        "device_copy_gbs": round(copy_gbs, 1), "pct_of_device_copy": round(100 * value / copy_gbs, 1),
        "compress_mtok_s": c4["compress_mtok_s"],
        "compress_note": "prompt tokens/s through all 32 layers at the (8192 tok, 4 bit) setting",
        "append_tail_us": None if append_us is None else round(append_us, 2),
        "append_note": f"kvqp_append_tail of {G} tokens per cache, 32 layers as one batch, 4-bit setting",
        "layer_wise_counts": layer_wise, "outlier_filtering": outlier_leg, "per_token_keys": token_keys,
        "sweep": sweep, "per_layer_calls": per_layer,
        "warm_same_cache_loop": warm,
        "warm_note": "the 128 decode calls of a setting on ONE copy of the cache (what the timed steps avoid): the copy is "
                     "re-read at every step and a part of it is served by the memory-side cache, so these are algorithmic "
                     "bytes per second, not HBM bandwidth; keep_hint_*: with cfg.decode_cache_hint = KVQP_CACHE_KEEP",
        "other_configs": others,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
