"""GPU parity of outlier filtering (Section 6.3 item (1), Appendix B: numbers with |x| > 6 are
excluded from quantization) against the CPU checker: packed codes, scales, zeros and the outlier
slot words bit-exact; decode attention over such a cache within 2e-3."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import ATTN_TOL, assert_cache_equal, assert_overflow_equal, attn_excess, dev, upload_cache
from tests.test_gpu_compress import check_indices

pytestmark = pytest.mark.gpu
TAU = 6.0
CAP = 3000      # overflow list entries per head in these cases (enough unless a case says otherwise)


def attn_close(out, ref):
    """Error against the 2e-3 bar, shifted so that <= 2e-3 means "met" (tests/gpu_util.attn_excess):
    plain max-abs below magnitude 4; the value channels that carry outliers here reach |out| of 10
    to 40, where the checker's result rounded to binary16 is the reference."""
    return attn_excess(out, ref) + ATTN_TOL


def prompt(B, Hq, Hkv, L, W, config, k_outlier=20.0, v_channels=(3, 64), extra_k_channels=()):
    """The usual synthetic prompt with outlier channels in the values too (x12), and optionally more
    key channels than the four slots a row has."""
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, outlier=k_outlier, config=config)
    v[..., list(v_channels)] = (v[..., list(v_channels)].astype(np.float32) * 12).astype(np.float16)
    if extra_k_channels:
        k[..., list(extra_k_channels)] = (k[..., list(extra_k_channels)].astype(np.float32) * 15).astype(np.float16)
    return q_obs, k, v


def random_survivors(B, Hkv, P, n, seed):
    rng = np.random.default_rng(seed)
    return np.stack([[np.sort(rng.choice(P, n, replace=False)) for _ in range(Hkv)] for _ in range(B)]).astype(np.int32)


@pytest.mark.parametrize("bits", [2, 4, 8])
@pytest.mark.parametrize("G,axis", [(32, 0), (64, 0), (128, 0), (32, 1), (64, 1), (128, 1)])
def test_quantize_with_outliers_matches_checker(orc, bits, G, axis):
    print(f"case bits={bits} G={G} axis={axis}", flush=True)
    B, Hq, Hkv, L, W, n = 2, 4, 2, 700, 8, 384
    q_obs, k, v = prompt(B, Hq, Hkv, L, W, config=80, extra_k_channels=(50, 51, 90))   # up to 7 candidates per key row
    idx = random_survivors(B, Hkv, L - W, n, 80)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G, key_axis=axis, tau=TAU, ovf_cap=CAP)
    assert (oc.k_out != 0).sum() > 0.9 * 4 * B * Hkv * n * 0.5 and (oc.v_out != 0).sum() > 0      # the case is not empty
    k_over = [int(oc.k_ovf[b, g][n // 32]) for b in range(B) for g in range(Hkv)]
    assert min(k_over) > n // 4 and max(k_over) <= CAP                                              # rows beyond their four slots, all stored
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n, bits=bits, group_size=G,
                   key_axis=axis, outlier_threshold=TAU, outlier_overflow_cap=CAP)
    gc = kvqp.alloc_cache(cfg)
    for t in gc.buffers.values():
        t.fill_(0x3C)
    kvqp.quantize_selected(cfg, dev(k), dev(v), dev(idx), gc)
    torch.cuda.synchronize()
    assert_cache_equal(gc, oc)
    sm = float(np.float32(cfg.sm_scale))
    for step in range(2):
        q = synth.decode_query_host(B, Hq, 128, config=80, step=step)
        ref = orc.decode_attn(q, oc, sm)
        out = kvqp.decode_attn(cfg, dev(q), gc)
        torch.cuda.synchronize()
        err = attn_close(out, ref)
        print(f"  decode error {err:.2e}", flush=True)
        assert err <= 2e-3


@pytest.mark.parametrize("Hq,Hkv", [(8, 1), (2, 2), (4, 4)])
def test_decode_over_checker_cache_other_group_sizes(orc, Hq, Hkv):
    """Gq = 8 (one token slot per tile), 1 and ... : the cache is the checker's, uploaded."""
    print(f"case Hq={Hq} Hkv={Hkv}", flush=True)
    B, L, W, n = 1, 900, 32, 512
    q_obs, k, v = prompt(B, Hq, Hkv, L, W, config=81)
    idx = random_survivors(B, Hkv, L - W, n, 81)
    for bits, G, axis in ((4, 32, 0), (2, 64, 1)):
        oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G, key_axis=axis, tau=TAU, ovf_cap=CAP)
        cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n, bits=bits, group_size=G,
                       key_axis=axis, outlier_threshold=TAU, outlier_overflow_cap=CAP)
        gc = upload_cache(oc)
        q = synth.decode_query_host(B, Hq, 128, config=81, step=0)
        ref = orc.decode_attn(q, oc, float(np.float32(cfg.sm_scale)))
        out = kvqp.decode_attn(cfg, dev(q), gc)
        torch.cuda.synchronize()
        assert attn_close(out, ref) <= 2e-3


def test_compress_with_outliers_end_to_end_and_long_context_splits(orc):
    """Whole compression at tau = 6 (same survivors as without filtering), then decode with the
    token axis split over several workgroups (few heads, 4096 tokens)."""
    B, Hq, Hkv, L, W, n = 1, 8, 2, 6000, 32, 4096
    q_obs, k, v = prompt(B, Hq, Hkv, L, W, config=82)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n, bits=4, group_size=32,
                   outlier_threshold=TAU, outlier_overflow_cap=CAP)
    sm = float(np.float32(cfg.sm_scale))
    oc, idx_orc, pooled = orc.compress(q_obs, k, v, window=W, pool=7, budget=n, bits=4, G=32, sm_scale=sm, tau=TAU, ovf_cap=CAP)
    gc = kvqp.alloc_cache(cfg)
    idx_dev = torch.empty((B, Hkv, n), dtype=torch.int32, device="cuda")
    kvqp.compress(cfg, dev(q_obs), dev(k), dev(v), gc, idx_out=idx_dev)
    torch.cuda.synchronize()
    if check_indices(idx_dev.cpu().numpy(), idx_orc, pooled):
        oc = orc.quantize_selected(k, v, idx_dev.cpu().numpy(), W=W, bits=4, G=32, tau=TAU, ovf_cap=CAP)
    assert_cache_equal(gc, oc)
    q = synth.decode_query_host(B, Hq, 128, config=82, step=0)
    ref = orc.decode_attn(q, oc, sm)
    out = kvqp.decode_attn(cfg, dev(q), gc)
    torch.cuda.synchronize()
    assert attn_close(out, ref) <= 2e-3


def test_threshold_out_of_reach_equals_no_filtering(orc):
    B, Hq, Hkv, L, W, n = 1, 8, 2, 800, 32, 256
    q_obs, k, v = prompt(B, Hq, Hkv, L, W, config=83)
    idx = random_survivors(B, Hkv, L - W, n, 83)
    base = dict(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n, bits=4, group_size=32)
    a = kvqp.alloc_cache(kvqp.Cfg(**base))
    cfg_b = kvqp.Cfg(**base, outlier_threshold=7.0e4, outlier_overflow_cap=16)
    b = kvqp.alloc_cache(cfg_b)
    kvqp.quantize_selected(kvqp.Cfg(**base), dev(k), dev(v), dev(idx), a)
    kvqp.quantize_selected(cfg_b, dev(k), dev(v), dev(idx), b)
    torch.cuda.synchronize()
    for nm in a.buffers:
        assert torch.equal(a.buffers[nm], b.buffers[nm]), nm
    assert not b.buffers["k_out"].any() and not b.buffers["v_out"].any()
    assert not b.buffers["k_ovf"].view(torch.int32).view(Hkv, -1)[:, : n // 32 + 1].any()         # no list entries either
    q = synth.decode_query_host(B, Hq, 128, config=83, step=0)
    oa, ob = kvqp.decode_attn(kvqp.Cfg(**base), dev(q), a), kvqp.decode_attn(cfg_b, dev(q), b)
    torch.cuda.synchronize()
    assert (oa.float() - ob.float()).abs().max().item() <= 2e-3


def test_head_level_counts_and_append_with_outliers(orc):
    """The slots follow their tokens through the ragged form and through the decode-time append."""
    B, Hq, Hkv, L, W = 1, 8, 2, 1000, 32
    q_obs, k, v = prompt(B, Hq, Hkv, L, W, config=84)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=512, bits=4, group_size=32,
                   outlier_threshold=TAU, outlier_overflow_cap=CAP)
    sm = float(np.float32(cfg.sm_scale))
    counts = [512, 160]
    gc = kvqp.alloc_cache(cfg, ragged=True)
    idx_dev = torch.empty((B, Hkv, 512), dtype=torch.int32, device="cuda")
    kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), counts, gc, idx_out=idx_dev)
    torch.cuda.synchronize()
    idx_gpu = idx_dev.cpu().numpy()
    q = synth.decode_query_host(B, Hq, 128, config=84, step=0)
    out = kvqp.decode_attn(cfg, dev(q), gc).cpu().numpy().astype(np.float64)
    for g, nb in enumerate(counts):
        oc = orc.quantize_selected(k[:, g:g + 1], v[:, g:g + 1], idx_gpu[:, g:g + 1, :nb], W=W, bits=4, G=32, tau=TAU, ovf_cap=CAP)
        got = gc.buffers["k_out"].cpu().numpy().view(np.uint32).reshape(Hkv, 512, 4)[g, :nb]
        assert np.array_equal(got, oc.k_out[0, 0])
        for nm in ("k_ovf", "v_ovf"):
            assert_overflow_equal(gc.buffers[nm].cpu().numpy().view(np.uint32).reshape(Hkv, -1)[g], 512, getattr(oc, nm)[0, 0], nb, CAP, nm)
        ref = orc.decode_attn(q[:, 4 * g:4 * g + 4], oc, sm)
        assert attn_close(out[0, 4 * g:4 * g + 4], ref[0]) <= 2e-3
    # append: 32 more rows through the tail of a cache with room to grow == one-shot quantization
    n0, G = 256, 32
    idx = random_survivors(B, Hkv, L - W - G, n0, 84)
    cfg2 = kvqp.Cfg(**{**cfg.__dict__, "budget": n0})
    grow = kvqp.alloc_cache(cfg2, tail_cap=W + G, n_cap=n0 + 64)
    kvqp.quantize_selected(cfg2, dev(k), dev(v), dev(idx), grow)
    rows_k, rows_v = k[:, :, L - W - G:L - W], v[:, :, L - W - G:L - W]          # G rows that sit right before the window
    tk = grow.buffers["tail_k"].view(torch.float16).view(B, Hkv, W + G, 128)
    tv = grow.buffers["tail_v"].view(torch.float16).view(B, Hkv, W + G, 128)
    tk[:, :, G:] = tk[:, :, :W].clone(); tv[:, :, G:] = tv[:, :, :W].clone()
    tk[:, :, :G] = dev(rows_k); tv[:, :, :G] = dev(rows_v)
    grow.tail_len = W + G
    kvqp.append_tail(cfg2, grow, G)
    torch.cuda.synchronize()
    idx_all = np.concatenate([idx, np.broadcast_to(np.arange(L - W - G, L - W, dtype=np.int32), (B, Hkv, G))], axis=-1)
    oc = orc.quantize_selected(k, v, idx_all, W=W, bits=4, G=32, tau=TAU, ovf_cap=CAP)
    got = grow.buffers["k_out"].cpu().numpy().view(np.uint32).reshape(B, Hkv, n0 + 64, 4)[:, :, :n0 + G]
    assert np.array_equal(got, oc.k_out)
    got = grow.buffers["v_out"].cpu().numpy().view(np.uint32).reshape(B, Hkv, n0 + 64, 4)[:, :, :n0 + G]
    assert np.array_equal(got, oc.v_out)
    for nm in ("k_ovf", "v_ovf"):
        for g in range(Hkv):
            assert_overflow_equal(grow.buffers[nm].cpu().numpy().view(np.uint32).reshape(Hkv, -1)[g], n0 + 64, getattr(oc, nm)[0, g], n0 + G, CAP, nm)
    grow_ref = upload_cache(oc)
    o1 = kvqp.decode_attn(cfg2, dev(q), grow)
    ref = orc.decode_attn(q, oc, sm)
    torch.cuda.synchronize()
    assert attn_close(o1, ref) <= 2e-3
    del grow_ref


def test_list_that_is_too_short_shows_its_shortfall(orc):
    """A caller that sizes the overflow list too small loses the entries beyond it -- those elements
    read as their group's zero -- and sees it: the last prefix count is the number needed.  Library
    and checker drop the same entries, so packed bytes and attention still agree."""
    B, Hq, Hkv, L, W, n, cap = 1, 4, 2, 700, 8, 256, 40
    q_obs, k, v = prompt(B, Hq, Hkv, L, W, config=86, extra_k_channels=(50, 51, 90))
    idx = random_survivors(B, Hkv, L - W, n, 86)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=4, G=32, key_axis=0, tau=TAU, ovf_cap=cap)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n, bits=4, group_size=32,
                   outlier_threshold=TAU, outlier_overflow_cap=cap)
    gc = kvqp.alloc_cache(cfg)
    for t in gc.buffers.values():
        t.fill_(0x5A)
    kvqp.quantize_selected(cfg, dev(k), dev(v), dev(idx), gc)
    torch.cuda.synchronize()
    assert_cache_equal(gc, oc)
    needed = gc.buffers["k_ovf"].cpu().numpy().view(np.int32).reshape(Hkv, -1)[:, n // 32]
    assert needed.min() > cap                                       # the shortfall is there to be seen
    q = synth.decode_query_host(B, Hq, 128, config=86, step=0)
    out = kvqp.decode_attn(cfg, dev(q), gc)
    torch.cuda.synchronize()
    assert attn_close(out, orc.decode_attn(q, oc, float(np.float32(cfg.sm_scale)))) <= 2e-3


def test_argument_checks():
    cfg16 = kvqp.Cfg(batch=1, n_q_heads=8, n_kv_heads=2, seq_len=800, window=32, budget=256, bits=16, outlier_threshold=TAU, outlier_overflow_cap=CAP)
    with pytest.raises(kvqp.KvqpError):
        kvqp.cache_sizes(cfg16, 32)
    cfg = kvqp.Cfg(batch=1, n_q_heads=8, n_kv_heads=2, seq_len=800, window=32, budget=256, bits=4, outlier_threshold=TAU, outlier_overflow_cap=CAP)
    assert kvqp.outlier_sizes(cfg) == [2 * 256 * 4 * 4] * 2 + [2 * (12 + 2 * CAP) * 4] * 2     # slots; 9 prefix counts padded to 12, CAP entries
    assert kvqp.outlier_sizes(kvqp.Cfg(**{**cfg.__dict__, "outlier_threshold": 0.0})) == [0, 0, 0, 0]
    plain = kvqp.alloc_cache(kvqp.Cfg(**{**cfg.__dict__, "outlier_threshold": 0.0}))
    q_obs, k, v = synth.prompt_host(1, 8, 2, 800, 32, 128, config=85)
    with pytest.raises(kvqp.KvqpError):
        kvqp.compress(cfg, dev(q_obs), dev(k), dev(v), plain)       # no slot buffers
