"""GPU parity of compression and decode attention with a token count of its own
per KV head (Section 5, Q1 / Table 1: head-level allocation keeps different
numbers of tokens per head and is paired with per-token key groups; a
layer-wise schedule varies the count by layer; Appendix B: window 8).

The definition is per head: head h is the uniform method run on that head
alone with its own count.  So the CPU checker is called once per head on the
head's slice and compared with the head's share of the device buffers: indices
bit-exact up to the checker's own near-ties, packed words, scales, zeros and
tail rows bit-exact, attention outputs within 2e-3."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import assert_overflow_equal, attn_excess, attn_maxabs, dev, download
from tests.test_gpu_compress import check_indices

pytestmark = pytest.mark.gpu


def head_reference(orc, q_obs, k, v, b, g, gq, nb, *, W, pool, bits, G, key_axis, sm_scale):
    """The checker on one head alone: (cache, idx [nb], pooled [P]) with count nb."""
    qs, ks, vs = q_obs[b:b + 1, g * gq:(g + 1) * gq], k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1]
    if nb == 0:
        return orc.quantize_selected(ks, vs, np.zeros((1, 1, 0), np.int32), W=W, bits=bits, G=G, key_axis=key_axis), None, None
    c, idx, pooled = orc.compress(qs, ks, vs, window=W, pool=pool, budget=nb, bits=bits, G=G, sm_scale=sm_scale,
                                  key_axis=key_axis)
    return c, idx, pooled


def head_share(gc, name, dtype, heads, h, count):
    """First `count` elements of head h's share of a device buffer."""
    arr = download(gc, name, dtype)
    per = arr.size // heads
    return arr.reshape(heads, per)[h, :count]


def run_case(orc, B, Hq, Hkv, L, W, pool, bound, bits, G, key_axis, budgets, config, decode_splits=0, outlier=10.0):
    gq = Hq // Hkv
    heads = B * Hkv
    assert len(budgets) == heads
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, outlier=outlier, config=config)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, pool_kernel=pool, budget=bound,
                   bits=bits, group_size=G, key_axis=key_axis, decode_splits=decode_splits)
    sm = float(np.float32(cfg.sm_scale))
    n_bound = cfg.n_kept
    gc = kvqp.alloc_cache(cfg, ragged=True)
    for t in gc.buffers.values():
        t.fill_(0xA5)                      # whatever lies beyond a head's count must not matter
    idx_dev = torch.full((B, Hkv, n_bound), -7, dtype=torch.int32, device="cuda")
    kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), budgets, gc, idx_out=idx_dev)
    torch.cuda.synchronize()
    assert gc.n_kept == n_bound and gc.tail_len == W
    assert gc.head_n_kept.cpu().tolist() == list(budgets)
    idx_gpu = idx_dev.cpu().numpy()
    refs = []
    exempt_total = 0
    E = 32 // bits
    for h in range(heads):
        b, g, nb = h // Hkv, h % Hkv, budgets[h]
        print(f"  head {h}: count {nb}", flush=True)
        oc, idx_orc, pooled = head_reference(orc, q_obs, k, v, b, g, gq, nb, W=W, pool=pool, bits=bits, G=G,
                                             key_axis=key_axis, sm_scale=sm)
        if nb:
            got = idx_gpu[b:b + 1, g:g + 1, :nb]
            exempt = check_indices(got, idx_orc, pooled)
            exempt_total += exempt
            if exempt:
                oc = orc.quantize_selected(k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1], got, W=W, bits=bits, G=G,
                                           key_axis=key_axis)
        # the head's share of every buffer, up to its own count
        kw = nb * 128 // E
        assert np.array_equal(head_share(gc, "k_codes", np.uint32, heads, h, kw), oc.k_codes.reshape(-1)[:kw])
        vw = oc.v_codes.size
        assert np.array_equal(head_share(gc, "v_codes", np.uint32, heads, h, vw), oc.v_codes.reshape(-1))
        if bits != 16:
            for nm in ("k_scale", "k_zero", "v_scale", "v_zero"):
                ref = getattr(oc, nm).reshape(-1)
                assert np.array_equal(head_share(gc, nm, np.uint16, heads, h, ref.size), ref), nm
        for nm in ("tail_k", "tail_v"):
            ref = getattr(oc, nm).reshape(-1)[: W * 128]
            assert np.array_equal(head_share(gc, nm, np.uint16, heads, h, W * 128), ref), nm
        refs.append(oc)
    print(f"  exempt index differences: {exempt_total}", flush=True)
    worst = 0.0
    for step in range(2):
        q = synth.decode_query_host(B, Hq, 128, config=config, step=step)
        out = kvqp.decode_attn(cfg, dev(q), gc)
        torch.cuda.synchronize()
        out = out.cpu().numpy().astype(np.float64)
        for h in range(heads):
            b, g = h // Hkv, h % Hkv
            ref = orc.decode_attn(q[b:b + 1, g * gq:(g + 1) * gq], refs[h], sm)
            worst = max(worst, np.abs(out[b, g * gq:(g + 1) * gq] - ref[0]).max())
    print(f"  worst attention error {worst:.2e}", flush=True)
    assert worst <= 2e-3
    return gc


def test_head_level_counts_per_token_keys(orc):
    """The pairing the paper uses for head-level allocation: per-token key groups of 64, window 8."""
    print("case head-level, per-token keys", flush=True)
    run_case(orc, 1, 8, 4, 1500, 8, 7, 512, 4, 64, kvqp.KEY_PER_TOKEN, [32, 256, 96, 512], config=60)


def test_head_level_counts_per_channel_keys(orc):
    """Per-channel key groups work too as long as every head keeps whole groups; one head keeps
    nothing and one keeps the whole prefix (L - W = 1024)."""
    print("case head-level, per-channel keys", flush=True)
    run_case(orc, 1, 8, 4, 1056, 32, 7, 1024, 2, 64, kvqp.KEY_PER_CHANNEL, [0, 1024, 64, 448], config=61)


def test_layer_wise_schedule(orc):
    """Counts falling from the first to the last layer of a batch of layers (window 8)."""
    print("case layer-wise schedule", flush=True)
    layers, Hkv = 4, 2
    per_layer = [640, 480, 320, 160]
    budgets = [per_layer[h // Hkv] for h in range(layers * Hkv)]
    run_case(orc, layers, 8, Hkv, 1300, 8, 5, 640, 8, 32, kvqp.KEY_PER_CHANNEL, budgets, config=62)


def test_sixteen_bit_and_token_axis_splits(orc):
    """Few heads and a long prefix: the decode launch splits every head along the token axis, each
    head by its own count; 16-bit cache and a caller-chosen split of a 4-bit per-token cache."""
    print("case splits, 16-bit", flush=True)
    run_case(orc, 1, 4, 2, 6000, 32, 7, 4096, 16, 32, kvqp.KEY_PER_CHANNEL, [4096, 640], config=63)
    print("case splits, per-token 4-bit, 5 splits", flush=True)
    run_case(orc, 1, 4, 2, 3000, 32, 7, 2048, 4, 32, kvqp.KEY_PER_TOKEN, [2048, 96], config=64, decode_splits=5)
    print("case splits, per-channel 4-bit", flush=True)
    run_case(orc, 1, 8, 2, 6000, 32, 7, 4096, 4, 32, kvqp.KEY_PER_CHANNEL, [1024, 4096], config=65)


def test_uniform_counts_equal_the_uniform_call(orc):
    """Every head given the bound: the buffers are those of kvqp_compress, bit for bit."""
    B, Hq, Hkv, L, W = 2, 8, 2, 1111, 32
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=66)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=256, bits=4, group_size=32)
    a, b_ = kvqp.alloc_cache(cfg), kvqp.alloc_cache(cfg, ragged=True)
    kvqp.compress(cfg, dev(q_obs), dev(k), dev(v), a)
    kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), [256] * (B * Hkv), b_)
    torch.cuda.synchronize()
    for n in a.buffers:
        assert torch.equal(a.buffers[n], b_.buffers[n]), n
    q = synth.decode_query_host(B, Hq, 128, config=66, step=0)
    oa, ob = kvqp.decode_attn(cfg, dev(q), a), kvqp.decode_attn(cfg, dev(q), b_)
    torch.cuda.synchronize()
    assert (oa.float() - ob.float()).abs().max().item() <= 2e-3


def test_calls_that_do_not_take_head_level_counts(orc):
    B, Hq, Hkv, L, W = 1, 8, 2, 800, 32
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=67)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=256, bits=4, group_size=32)
    gc = kvqp.alloc_cache(cfg, ragged=True)
    with pytest.raises(kvqp.KvqpError):
        kvqp.compress(cfg, dev(q_obs), dev(k), dev(v), gc)            # uniform call, ragged cache
    kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), [256, 100], gc)       # any count under the bound is fine
    with pytest.raises(kvqp.KvqpError):
        kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), [256, 288], gc)   # above the bound
    with pytest.raises(kvqp.KvqpError):
        kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), [256, 64], kvqp.alloc_cache(cfg))   # no count array
    kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), [256, 64], gc)
    with pytest.raises(kvqp.KvqpError) as e:
        kvqp.append_tail(cfg, gc, 32)
    assert e.value.code == -2
    torch.cuda.synchronize()


@pytest.mark.parametrize("bits,G,key_axis", [(4, 64, kvqp.KEY_PER_TOKEN), (2, 32, kvqp.KEY_PER_CHANNEL),
                                             (8, 128, kvqp.KEY_PER_CHANNEL), (16, 32, kvqp.KEY_PER_CHANNEL)])
def test_quantize_given_survivors_with_head_level_counts(orc, bits, G, key_axis):
    """Survivors from a head-level method of the caller's (here: seeded random positions): every
    head's share equals the checker's quantization of that head's own list."""
    print(f"case given survivors bits={bits} G={G} axis={key_axis}", flush=True)
    B, Hq, Hkv, L, W, bound = 2, 8, 2, 900, 8, 512
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=68)
    counts = [512, 128, 0, 384]
    rng = np.random.default_rng(68)
    idx = np.zeros((B, Hkv, bound), np.int32)
    for h, n in enumerate(counts):
        idx[h // Hkv, h % Hkv, :n] = np.sort(rng.choice(L - W, n, replace=False))
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=bound, bits=bits, group_size=G,
                   key_axis=key_axis)
    gc = kvqp.alloc_cache(cfg, ragged=True)
    for t in gc.buffers.values():
        t.fill_(0x5A)
    kvqp.quantize_selected_ragged(cfg, dev(k), dev(v), dev(idx), counts, gc)
    torch.cuda.synchronize()
    assert gc.head_n_kept.cpu().tolist() == counts and gc.n_kept == bound and gc.tail_len == W
    heads, E, sm = B * Hkv, 32 // bits, float(np.float32(cfg.sm_scale))
    q = synth.decode_query_host(B, Hq, 128, config=68, step=0)
    out = kvqp.decode_attn(cfg, dev(q), gc)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    gq = Hq // Hkv
    for h, n in enumerate(counts):
        b, g = h // Hkv, h % Hkv
        oc = orc.quantize_selected(k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1], idx[b:b + 1, g:g + 1, :n], W=W, bits=bits,
                                   G=G, key_axis=key_axis)
        assert np.array_equal(head_share(gc, "k_codes", np.uint32, heads, h, n * 128 // E), oc.k_codes.reshape(-1))
        assert np.array_equal(head_share(gc, "v_codes", np.uint32, heads, h, oc.v_codes.size), oc.v_codes.reshape(-1))
        if bits != 16:
            for nm in ("k_scale", "k_zero", "v_scale", "v_zero"):
                ref = getattr(oc, nm).reshape(-1)
                assert np.array_equal(head_share(gc, nm, np.uint16, heads, h, ref.size), ref), nm
        ref = orc.decode_attn(q[b:b + 1, g * gq:(g + 1) * gq], oc, sm)
        assert np.abs(out[b, g * gq:(g + 1) * gq] - ref[0]).max() <= 2e-3


@pytest.mark.parametrize("bits,G,key_axis,n_app,tau", [(4, 64, kvqp.KEY_PER_TOKEN, 32, 0.0), (2, 32, kvqp.KEY_PER_CHANNEL, 64, 0.0),
                                                        (4, 128, kvqp.KEY_PER_CHANNEL, 128, 0.0), (8, 32, kvqp.KEY_PER_TOKEN, 96, 0.0),
                                                        (16, 32, kvqp.KEY_PER_CHANNEL, 32, 0.0), (4, 32, kvqp.KEY_PER_CHANNEL, 64, 6.0)])
def test_append_with_head_level_counts(orc, bits, G, key_axis, n_app, tau):
    """Decode-time update (Eq. (2)) of a cache with head-level counts: every head takes the oldest
    tail rows onto the end of its own packed part.  Per head, the result is the checker's
    quantization of that head's survivors plus the moved rows in one go; twice in a row."""
    print(f"case ragged append bits={bits} G={G} axis={key_axis} n={n_app} tau={tau}", flush=True)
    B, Hq, Hkv, W, bound, P = 2, 8, 2, 8, 512, 900
    q_app = 64 if bits == 2 else 32
    if bits != 16 and key_axis == kvqp.KEY_PER_CHANNEL:
        q_app = max(q_app, G)
    counts = [c - c % q_app for c in (512, 128, 0, 384)]
    grown = W + 2 * n_app + 5                          # tail rows after some decoding
    _, k, v = synth.prompt_host(B, Hq, Hkv, P + grown, grown, 128, config=69)
    if tau:
        v[..., [3, 64]] *= 12                          # value outliers too
    rng = np.random.default_rng(69 + bits)
    idx = np.zeros((B, Hkv, bound), np.int32)
    for h, n in enumerate(counts):
        idx[h // Hkv, h % Hkv, :n] = np.sort(rng.choice(P, n, replace=False))
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=P + grown, window=W, budget=bound, bits=bits,
                   group_size=G, key_axis=key_axis, outlier_threshold=tau, outlier_overflow_cap=500 if tau else 0)
    cap = grown + 3
    gc = kvqp.alloc_cache(cfg, tail_cap=cap, n_cap=bound + 2 * n_app + (-(bound + 2 * n_app)) % 128, ragged=True)
    for t in gc.buffers.values():
        t.fill_(0x3C)
    kvqp.quantize_selected_ragged(cfg, dev(k), dev(v), dev(idx), counts, gc)
    heads, E, sm, gq = B * Hkv, 32 // bits, float(np.float32(cfg.sm_scale)), Hq // Hkv
    for name, src in (("tail_k", k), ("tail_v", v)):   # the caller's appended rows
        rows = torch.from_numpy(np.ascontiguousarray(src[:, :, P:P + grown]).view(np.uint16).copy()).cuda()
        gc.buffers[name].view(torch.uint16).view(heads, cap, 128)[:, :grown] = rows.view(heads, grown, 128)
    gc.tail_len = grown
    ws = kvqp.alloc_decode_workspace(cfg)
    kw = dict(tau=tau, ovf_cap=500) if tau else {}
    for rnd in (1, 2):
        kvqp.append_tail_ragged(cfg, gc, n_app, counts)
        counts = [c + n_app for c in counts]
        moved = rnd * n_app
        torch.cuda.synchronize()
        assert gc.head_n_kept.cpu().tolist() == counts and gc.n_kept == bound + moved and gc.tail_len == grown - moved
        q = synth.decode_query_host(B, Hq, 128, config=69, step=rnd)
        out = kvqp.decode_attn(cfg, dev(q), gc, workspace=ws)
        torch.cuda.synchronize()
        out = out.cpu().numpy().astype(np.float64)
        for h, n in enumerate(counts):
            b, g = h // Hkv, h % Hkv
            own = np.concatenate([idx[b, g, :n - moved], np.arange(P, P + moved, dtype=np.int32)]).reshape(1, 1, n)
            oc = orc.quantize_selected(k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1], own, W=grown - moved, bits=bits, G=G,
                                       key_axis=key_axis, **kw)
            assert np.array_equal(head_share(gc, "k_codes", np.uint32, heads, h, n * 128 // E), oc.k_codes.reshape(-1)), h
            assert np.array_equal(head_share(gc, "v_codes", np.uint32, heads, h, oc.v_codes.size), oc.v_codes.reshape(-1)), h
            names = ["k_scale", "k_zero", "v_scale", "v_zero"] if bits != 16 else []
            dts = {nm: np.uint16 for nm in names}
            if tau:
                names += ["k_out", "v_out"]
                dts.update(k_out=np.uint32, v_out=np.uint32)
            for nm in names:
                ref = getattr(oc, nm).reshape(-1)
                assert np.array_equal(head_share(gc, nm, dts[nm], heads, h, ref.size), ref), (nm, h)
            if tau:
                for nm in ("k_ovf", "v_ovf"):
                    assert_overflow_equal(download(gc, nm, np.uint32).reshape(heads, -1)[h], gc.n_cap, getattr(oc, nm).reshape(-1), n, 500, (nm, h))
            for nm in ("tail_k", "tail_v"):
                ref = getattr(oc, nm).reshape(-1)[: (grown - moved) * 128]
                assert np.array_equal(head_share(gc, nm, np.uint16, heads, h, ref.size), ref), (nm, h)
            ref = orc.decode_attn(q[b:b + 1, g * gq:(g + 1) * gq], oc, sm)
            # plain max-abs 2e-3 (with outlier slots: the checker rounded to binary16 where |ref| >= 4)
            excess = attn_excess(out[b, g * gq:(g + 1) * gq], ref[0]) if tau else attn_maxabs(out[b, g * gq:(g + 1) * gq], ref[0]) - 2e-3
            assert excess <= 0.0, (h, excess)
    with pytest.raises(kvqp.KvqpError):
        kvqp.append_tail_ragged(cfg, gc, n_app, counts)          # the tail no longer holds that many rows
