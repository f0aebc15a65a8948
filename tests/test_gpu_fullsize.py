"""Parity at the benchmark's full size and launch configuration: the
Llama-3-8B-shaped workload (32 layers as the batch axis, 32 Q / 8 KV heads,
L = 32768) compressed and decoded exactly as bench.py does, checked against
the CPU checker on sampled (layer, KV head) slices of the very bytes the GPU
used.  Sampling keeps the checker's share to a few seconds per slice."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth

pytestmark = pytest.mark.gpu

LAYERS, HQ, HKV, D, L, W, POOL, G = 32, 32, 8, 128, 32768, 32, 7, 32
GQ = HQ // HKV
SAMPLES = [(0, 0), (13, 5), (31, 7)]


@pytest.fixture(scope="module")
def workload():
    q_obs, k, v = synth.prompt_device(LAYERS, HQ, HKV, L, W, D, outlier=10.0, config=2, device="cuda:0")
    return q_obs, k, v


def head_bytes(cache, name, layer, g):
    t = cache.buffers[name]
    per = t.numel() // (LAYERS * HKV)
    i = layer * HKV + g
    return t[i * per:(i + 1) * per].cpu().numpy()


@pytest.mark.parametrize("n_kept,bits", [(8192, 4), (16384, 2), (4096, 8), (2048, 16)])
def test_full_size_compress_and_decode(orc, workload, n_kept, bits):
    print(f"case tokens={n_kept} bits={bits}", flush=True)
    q_obs, k, v = workload
    sm = float(np.float32(D ** -0.5))
    cfg = kvqp.Cfg(batch=LAYERS, n_q_heads=HQ, n_kv_heads=HKV, seq_len=L, window=W, pool_kernel=POOL, budget=n_kept,
                   bits=bits, group_size=G, sm_scale=sm)
    cache = kvqp.alloc_cache(cfg, device="cuda:0")
    idx_dev = torch.empty((LAYERS, HKV, n_kept), dtype=torch.int32, device="cuda:0")
    unrefined = torch.full((LAYERS * HKV,), -1, dtype=torch.int32, device="cuda:0")
    kvqp.compress(cfg, q_obs, k, v, cache, idx_out=idx_dev, unrefined_out=unrefined)
    q = synth.decode_query_device(LAYERS, HQ, D, config=2, step=0, device="cuda:0")
    out = kvqp.decode_attn(cfg, q, cache)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    # every one of the 256 heads re-scored its candidates near the cut in binary64: none fell back to binary32
    assert int(unrefined.abs().sum().item()) == 0, unrefined.nonzero().flatten().tolist()
    idx_all = idx_dev.cpu().numpy()
    assert np.all(np.diff(idx_all, axis=-1) > 0) and idx_all.min() >= 0 and idx_all.max() < L - W

    for layer, g in SAMPLES:
        print(f"  slice layer={layer} kv_head={g}", flush=True)
        qs = q_obs[layer:layer + 1, g * GQ:(g + 1) * GQ].cpu().numpy()
        ks = k[layer:layer + 1, g:g + 1].cpu().numpy()
        vs = v[layer:layer + 1, g:g + 1].cpu().numpy()
        oc, idx_ref, pooled = orc.compress(qs, ks, vs, window=W, pool=POOL, budget=n_kept, bits=bits, G=G, sm_scale=sm)
        got = idx_all[layer, g]
        if not np.array_equal(got, idx_ref[0, 0]):
            kth = np.sort(pooled[0, 0])[-n_kept]
            diff = np.setxor1d(got, idx_ref[0, 0])
            rel = np.abs(pooled[0, 0][diff] - kth) / kth
            assert np.all(rel <= 1e-6), f"{diff.size} indices differ, worst relative gap {rel.max():.3e}"
            print(f"    {diff.size} index differences inside the 1e-6 tie band", flush=True)
            oc = orc.quantize_selected(ks, vs, got.reshape(1, 1, -1), W=W, bits=bits, G=G)
        for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v"):
            ref = np.ascontiguousarray(getattr(oc, name)).view(np.uint8).reshape(-1)
            assert np.array_equal(head_bytes(cache, name, layer, g), ref), f"{name} differs at layer {layer}, head {g}"
        qd = q[layer:layer + 1, g * GQ:(g + 1) * GQ].cpu().numpy()
        ref = orc.decode_attn(qd, oc, sm)
        err = np.abs(out[layer, g * GQ:(g + 1) * GQ].cpu().numpy().astype(np.float64) - ref[0]).max()
        print(f"    decode max-abs error {err:.2e}", flush=True)
        assert err <= 2e-3


def test_per_layer_calls_agree_with_the_batched_call(workload):
    """bench.py also issues the same work as 32 per-layer calls; both launch
    shapes must give the same bytes."""
    q_obs, k, v = workload
    sm = float(np.float32(D ** -0.5))
    cfg = kvqp.Cfg(batch=LAYERS, n_q_heads=HQ, n_kv_heads=HKV, seq_len=L, window=W, budget=8192, bits=4, group_size=G, sm_scale=sm)
    cache = kvqp.alloc_cache(cfg, device="cuda:0")
    kvqp.compress(cfg, q_obs, k, v, cache)
    q = synth.decode_query_device(LAYERS, HQ, D, config=2, step=1, device="cuda:0")
    out = kvqp.decode_attn(cfg, q, cache)
    cfg1 = kvqp.Cfg(**{**cfg.__dict__, "batch": 1})
    for layer in (0, 17, 31):
        c1 = kvqp.alloc_cache(cfg1, device="cuda:0")
        kvqp.compress(cfg1, q_obs[layer:layer + 1], k[layer:layer + 1], v[layer:layer + 1], c1)
        for name, t in c1.buffers.items():
            per = cache.buffers[name].numel() // LAYERS
            assert torch.equal(t, cache.buffers[name][layer * per:(layer + 1) * per]), name
        o1 = kvqp.decode_attn(cfg1, q[layer:layer + 1], c1)
        # split counts differ between the two launch shapes, so sums are reassociated
        assert (o1.float() - out[layer:layer + 1].float()).abs().max().item() <= 2e-3
    torch.cuda.synchronize()


def test_longest_context_shape(orc):
    """The long-context configuration of the benchmark spec at its real size, one
    layer: L = 131072 (the library's longest prefix), window 64 (256 query rows
    per KV head: the 64-rows-per-wave scoring variant), 16384 tokens kept at
    2 bits in groups of 64, key outlier channels x20.  Two KV heads are checked
    against the CPU checker."""
    Lc, Wc, Gc, n_kept, bits = 131072, 64, 64, 16384, 2
    print(f"case L={Lc} W={Wc} G={Gc} tokens={n_kept} bits={bits}", flush=True)
    q_obs, k, v = synth.prompt_device(1, HQ, HKV, Lc, Wc, D, outlier=20.0, config=4, device="cuda:0")
    sm = float(np.float32(D ** -0.5))
    cfg = kvqp.Cfg(batch=1, n_q_heads=HQ, n_kv_heads=HKV, seq_len=Lc, window=Wc, pool_kernel=POOL, budget=n_kept,
                   bits=bits, group_size=Gc, sm_scale=sm)
    cache = kvqp.alloc_cache(cfg, device="cuda:0")
    idx_dev = torch.empty((1, HKV, n_kept), dtype=torch.int32, device="cuda:0")
    unrefined = torch.full((HKV,), -1, dtype=torch.int32, device="cuda:0")
    kvqp.compress(cfg, q_obs, k, v, cache, idx_out=idx_dev, unrefined_out=unrefined)
    q = synth.decode_query_device(1, HQ, D, config=4, step=0, device="cuda:0")
    out = kvqp.decode_attn(cfg, q, cache)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    assert int(unrefined.abs().sum().item()) == 0, unrefined.tolist()      # no head fell back to binary32 at the cut
    idx_all = idx_dev.cpu().numpy()
    assert np.all(np.diff(idx_all, axis=-1) > 0) and idx_all.min() >= 0 and idx_all.max() < Lc - Wc
    heads = [1, 6]
    qs = np.concatenate([q_obs[:, g * GQ:(g + 1) * GQ].cpu().numpy() for g in heads], axis=1)
    ks = np.concatenate([k[:, g:g + 1].cpu().numpy() for g in heads], axis=1)
    vs = np.concatenate([v[:, g:g + 1].cpu().numpy() for g in heads], axis=1)
    print("  checker: 2 KV heads", flush=True)
    oc, idx_ref, pooled = orc.compress(qs, ks, vs, window=Wc, pool=POOL, budget=n_kept, bits=bits, G=Gc, sm_scale=sm)
    got = idx_all[0, heads]
    if not np.array_equal(got, idx_ref[0]):
        for i in range(len(heads)):
            kth = np.sort(pooled[0, i])[-n_kept]
            diff = np.setxor1d(got[i], idx_ref[0, i])
            if diff.size:
                rel = np.abs(pooled[0, i][diff] - kth) / kth
                assert np.all(rel <= 1e-6), f"head {heads[i]}: {diff.size} indices differ, worst relative gap {rel.max():.3e}"
                print(f"    head {heads[i]}: {diff.size} index differences inside the 1e-6 tie band", flush=True)
        oc = orc.quantize_selected(ks, vs, got.reshape(1, len(heads), -1), W=Wc, bits=bits, G=Gc)
    for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v"):
        t = cache.buffers[name]
        per = t.numel() // HKV
        ref = np.ascontiguousarray(getattr(oc, name)).view(np.uint8).reshape(len(heads), -1)
        for i, g in enumerate(heads):
            assert np.array_equal(t[g * per:(g + 1) * per].cpu().numpy(), ref[i]), f"{name} differs at head {g}"
    qd = np.concatenate([q[:, g * GQ:(g + 1) * GQ].cpu().numpy() for g in heads], axis=1)
    ref = orc.decode_attn(qd, oc, sm)
    gpu = np.concatenate([out[:, g * GQ:(g + 1) * GQ].cpu().numpy() for g in heads], axis=1).astype(np.float64)
    err = np.abs(gpu - ref).max()
    print(f"    decode max-abs error {err:.2e}", flush=True)
    assert err <= 2e-3


def check_one_layer(orc, *, B, Hq, Hkv, Lc, Wc, n_kept, bits, Gc, axis, config, samples, outlier=10.0):
    """One layer of a configuration at its real shape: compress and one decode step on the device,
    the sampled (sequence, KV head) slices against the CPU checker on the same bytes."""
    gq = Hq // Hkv
    q_obs, k, v = synth.prompt_device(B, Hq, Hkv, Lc, Wc, D, outlier=outlier, config=config, device="cuda:0")
    sm = float(np.float32(D ** -0.5))
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=Lc, window=Wc, pool_kernel=POOL, budget=n_kept,
                   bits=bits, group_size=Gc, key_axis=axis, sm_scale=sm)
    cache = kvqp.alloc_cache(cfg, device="cuda:0")
    idx_dev = torch.empty((B, Hkv, n_kept), dtype=torch.int32, device="cuda:0")
    unrefined = torch.full((B * Hkv,), -1, dtype=torch.int32, device="cuda:0")
    kvqp.compress(cfg, q_obs, k, v, cache, idx_out=idx_dev, unrefined_out=unrefined)
    q = synth.decode_query_device(B, Hq, D, config=config, step=0, device="cuda:0")
    out = kvqp.decode_attn(cfg, q, cache)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    assert int(unrefined.abs().sum().item()) == 0, unrefined.nonzero().flatten().tolist()   # no head fell back to binary32 at the cut
    idx_all = idx_dev.cpu().numpy()
    assert np.all(np.diff(idx_all, axis=-1) > 0) and idx_all.min() >= 0 and idx_all.max() < Lc - Wc
    for b, g in samples:
        print(f"  slice sequence={b} kv_head={g}", flush=True)
        qs = q_obs[b:b + 1, g * gq:(g + 1) * gq].cpu().numpy()
        ks, vs = k[b:b + 1, g:g + 1].cpu().numpy(), v[b:b + 1, g:g + 1].cpu().numpy()
        oc, idx_ref, pooled = orc.compress(qs, ks, vs, window=Wc, pool=POOL, budget=n_kept, bits=bits, G=Gc, sm_scale=sm,
                                           key_axis=axis)
        got = idx_all[b, g]
        if not np.array_equal(got, idx_ref[0, 0]):
            kth = np.sort(pooled[0, 0])[-n_kept]
            diff = np.setxor1d(got, idx_ref[0, 0])
            rel = np.abs(pooled[0, 0][diff] - kth) / kth
            assert np.all(rel <= 1e-6), f"{diff.size} indices differ, worst relative gap {rel.max():.3e}"
            print(f"    {diff.size} index differences inside the 1e-6 tie band", flush=True)
            oc = orc.quantize_selected(ks, vs, got.reshape(1, 1, -1), W=Wc, bits=bits, G=Gc, key_axis=axis)
        for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v"):
            t = cache.buffers[name]
            per = t.numel() // (B * Hkv)
            i = b * Hkv + g
            ref = np.ascontiguousarray(getattr(oc, name)).view(np.uint8).reshape(-1)
            assert np.array_equal(t[i * per:(i + 1) * per].cpu().numpy(), ref), f"{name} differs at sequence {b}, head {g}"
        qd = q[b:b + 1, g * gq:(g + 1) * gq].cpu().numpy()
        ref = orc.decode_attn(qd, oc, sm)
        err = np.abs(out[b, g * gq:(g + 1) * gq].cpu().numpy().astype(np.float64) - ref[0]).max()
        print(f"    decode max-abs error {err:.2e}", flush=True)
        assert err <= 2e-3


def test_batched_sequences_shape(orc):
    """The batched-decode configuration, one layer at its real shape: 16 sequences of L = 16384,
    4096 tokens kept at 4 bits."""
    print("case batch 16, L=16384, 4096 tokens at 4 bits", flush=True)
    check_one_layer(orc, B=16, Hq=HQ, Hkv=HKV, Lc=16384, Wc=32, n_kept=4096, bits=4, Gc=32, axis=kvqp.KEY_PER_CHANNEL,
                    config=3, samples=[(0, 2), (15, 7)])


@pytest.mark.parametrize("axis", [kvqp.KEY_PER_CHANNEL, kvqp.KEY_PER_TOKEN])
def test_seventy_b_shape(orc, axis):
    """The 70B-shaped configuration, one layer at its real shape: 64 query / 8 KV heads (eight query
    heads per KV head: 256 window rows per head), 8 sequences of L = 32768, 8192 tokens kept at
    4 bits; per-channel keys and the per-token-key ablation."""
    print(f"case 64/8 heads, batch 8, L=32768, 8192 tokens at 4 bits, key axis {axis}", flush=True)
    check_one_layer(orc, B=8, Hq=64, Hkv=8, Lc=32768, Wc=32, n_kept=8192, bits=4, Gc=32, axis=axis, config=5,
                    samples=[(0, 0), (7, 5)])
