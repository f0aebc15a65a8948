"""Token counts that fill neither a block of 32 nor a key group (Section 3 asks only for s < n
kept tokens; Appendix B's quantizer keeps a residual): the head's last per-channel key group is
short, its last value block partly filled, and decode masks the rows past the count.  Everything
is compared with the CPU checker: indices, every packed byte (the rows past the count are zeros
on both sides), attention within 2e-3."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import assert_cache_equal, assert_overflow_equal, attn_excess, dev, download
from tests.test_gpu_compress import check_indices

pytestmark = pytest.mark.gpu
TOL = 2e-3


def survivors(B, Hkv, P, n, seed):
    rng = np.random.default_rng(seed)
    return np.stack([[np.sort(rng.choice(P, n, replace=False)) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32).reshape(B, Hkv, n)


@pytest.mark.parametrize("n", [1, 31, 33, 100, 1000, 1037])
@pytest.mark.parametrize("bits,G,axis,Gq", [(4, 32, 0, 4), (2, 64, 0, 4), (8, 128, 0, 2), (2, 32, 1, 4), (4, 64, 1, 8), (16, 32, 0, 4), (2, 128, 0, 8)])
def test_any_count_quantizes_and_decodes_like_the_checker(orc, n, bits, G, axis, Gq):
    print(f"case n={n} bits={bits} G={G} axis={axis} Gq={Gq}", flush=True)
    B, Hkv, W = 1, 2, 8
    Hq, L = Hkv * Gq, n + W + 90
    _, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=700 + bits)
    idx = survivors(B, Hkv, L - W, n, 700 + n)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G, key_axis=axis)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n, bits=bits, group_size=G, key_axis=axis)
    gc = kvqp.alloc_cache(cfg)
    for t in gc.buffers.values():
        t.fill_(0x7E)                                   # as binary16: NaN patterns, so nothing unwritten can hide
    kvqp.quantize_selected(cfg, dev(k), dev(v), dev(idx), gc)
    torch.cuda.synchronize()
    assert_cache_equal(gc, oc)
    for step in range(2):
        q = synth.decode_query_host(B, Hq, 128, config=700, step=step)
        out = kvqp.decode_attn(cfg, dev(q), gc)
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        assert np.all(np.isfinite(got))
        assert np.abs(got - orc.decode_attn(q, oc, cfg.sm_scale)).max() <= TOL


def test_budget_of_one_thousand_end_to_end(orc):
    """A caller's budget of 1000 at 4 bits, per-channel key groups of 32: compress, then decode with the
    token axis split over several workgroups (two heads on the whole chip)."""
    print("case budget 1000 end to end", flush=True)
    B, Hq, Hkv, L, W, n = 1, 8, 2, 3000, 32, 1000
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=710)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n, bits=4, group_size=32)
    sm = float(np.float32(cfg.sm_scale))
    oc, idx_orc, pooled = orc.compress(q_obs, k, v, window=W, pool=7, budget=n, bits=4, G=32, sm_scale=sm)
    gc = kvqp.alloc_cache(cfg)
    idx_dev = torch.empty((B, Hkv, n), dtype=torch.int32, device="cuda")
    kvqp.compress(cfg, dev(q_obs), dev(k), dev(v), gc, idx_out=idx_dev)
    torch.cuda.synchronize()
    if check_indices(idx_dev.cpu().numpy(), idx_orc, pooled):
        oc = orc.quantize_selected(k, v, idx_dev.cpu().numpy(), W=W, bits=4, G=32)
    assert_cache_equal(gc, oc)
    for splits in (0, 1, 3):
        c2 = kvqp.Cfg(**{**cfg.__dict__, "decode_splits": splits})
        q = synth.decode_query_host(B, Hq, 128, config=710, step=splits)
        out = kvqp.decode_attn(c2, dev(q), gc)
        torch.cuda.synchronize()
        assert np.abs(out.cpu().numpy().astype(np.float64) - orc.decode_attn(q, oc, sm)).max() <= TOL


@pytest.mark.parametrize("bits,G,axis,tau", [(4, 32, 0, 0.0), (2, 64, 1, 0.0), (4, 64, 0, 6.0), (8, 32, 1, 6.0)])
def test_head_level_counts_of_any_size(orc, bits, G, axis, tau):
    """Every head keeps its own, arbitrary number of tokens (head-level allocation hands out whatever
    its rule gives): per head the result equals the checker run on that head alone."""
    print(f"case ragged any count bits={bits} G={G} axis={axis} tau={tau}", flush=True)
    B, Hq, Hkv, L, W, bound, cap = 2, 8, 2, 1500, 16, 700, 400
    counts = [700, 37, 0, 513]
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=720 + bits, outlier=20.0 if tau else 10.0)
    if tau:
        v[..., [9, 70]] = (v[..., [9, 70]].astype(np.float32) * 10).astype(np.float16)
        k[..., [50, 51, 90]] = (k[..., [50, 51, 90]].astype(np.float32) * 15).astype(np.float16)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=bound, bits=bits, group_size=G,
                   key_axis=axis, outlier_threshold=tau, outlier_overflow_cap=cap if tau else 0)
    sm = float(np.float32(cfg.sm_scale))
    gc = kvqp.alloc_cache(cfg, ragged=True)
    for t in gc.buffers.values():
        t.fill_(0x7E)
    idx_dev = torch.full((B, Hkv, bound), -5, dtype=torch.int32, device="cuda")
    kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), counts, gc, idx_out=idx_dev)
    q = synth.decode_query_host(B, Hq, 128, config=720, step=0)
    out = kvqp.decode_attn(cfg, dev(q), gc)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(out))
    idx_gpu = idx_dev.cpu().numpy()
    heads, gq = B * Hkv, Hq // Hkv
    kw = dict(tau=tau, ovf_cap=cap) if tau else {}
    for h, n in enumerate(counts):
        b, g = h // Hkv, h % Hkv
        ks, vs = k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1]
        got = idx_gpu[b:b + 1, g:g + 1, :n]
        if n:
            _, idx_orc, pooled = orc.compress(q_obs[b:b + 1, g * gq:(g + 1) * gq], ks, vs, window=W, pool=7, budget=n, bits=bits,
                                              G=G, sm_scale=sm, key_axis=axis, **kw)
            check_indices(got, idx_orc, pooled)
        oc = orc.quantize_selected(ks, vs, got, W=W, bits=bits, G=G, key_axis=axis, **kw)
        names = ["k_codes", "v_codes"] + (["k_scale", "k_zero", "v_scale", "v_zero"] if bits != 16 else []) + (["k_out", "v_out"] if tau else [])
        for nm in names:
            ref = np.ascontiguousarray(getattr(oc, nm)).reshape(-1)
            share = download(gc, nm, ref.dtype).reshape(heads, -1)[h]
            assert np.array_equal(share[: ref.size], ref), (nm, h)
        if tau:
            for nm in ("k_ovf", "v_ovf"):
                assert_overflow_equal(download(gc, nm, np.uint32).reshape(heads, -1)[h], bound, getattr(oc, nm).reshape(-1), n, cap, (nm, h))
        ref = orc.decode_attn(q[b:b + 1, g * gq:(g + 1) * gq], oc, sm)[0]
        assert attn_excess(out[b, g * gq:(g + 1) * gq], ref) <= 0.0, h
