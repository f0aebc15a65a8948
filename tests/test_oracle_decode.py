"""Pins for the decode half of the CPU checker.

Paper, Section 3: decode attends with Softmax(h_Q X_K^T) X_V over the cache;
with quantized pruning the cache is the dequantized survivors G' = Q(G) s + z.
"""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import synth


def sdpa_f64(q, K, V, scale):
    """Independent library route: torch's scaled_dot_product_attention on CPU, float64."""
    qt = torch.from_numpy(q.astype(np.float64))[None, None, None, :]
    Kt = torch.from_numpy(K.astype(np.float64))[None, None]
    Vt = torch.from_numpy(V.astype(np.float64))[None, None]
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=scale)[0, 0, 0].numpy()


def test_16bit_full_budget_is_exact_attention_over_the_prompt(orc):
    B, Hq, Hkv, L, W, D = 2, 4, 2, 96, 32, 64
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=70)
    q = synth.decode_query_host(B, Hq, D, config=70)
    cache, idx, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=10**6, bits=16, G=32, sm_scale=0.125)
    out = orc.decode_attn(q, cache, 0.125)
    for b in range(B):
        for h in range(Hq):
            ref = sdpa_f64(q[b, h], k[b, h // 2], v[b, h // 2], 0.125)
            np.testing.assert_allclose(out[b, h], ref, rtol=1e-12, atol=1e-14)


def test_16bit_partial_budget_is_exact_attention_over_survivors_and_window(orc):
    B, Hq, Hkv, L, W, D = 1, 8, 2, 200, 8, 128
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=71)
    q = synth.decode_query_host(B, Hq, D, config=71)
    cache, idx, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=64, bits=16, G=32, sm_scale=0.088)
    out = orc.decode_attn(q, cache, 0.088)
    for h in range(Hq):
        g = h // 4
        rows = np.concatenate([idx[0, g], np.arange(L - W, L)])
        ref = sdpa_f64(q[0, h], k[0, g, rows], v[0, g, rows], 0.088)
        np.testing.assert_allclose(out[0, h], ref, rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("bits,G,axis", [(4, 32, 0), (2, 64, 0), (8, 32, 0), (4, 32, 1), (2, 32, 0)])
def test_quantized_decode_is_attention_over_dequantized_rows(orc, bits, G, axis):
    # decode must equal library attention run on the dense dequantized cache
    # (whose elements are pinned to the inputs by the half-scale bound elsewhere)
    B, Hq, Hkv, L, W, D = 1, 4, 2, 300, 8, 128
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=72)
    q = synth.decode_query_host(B, Hq, D, config=72)
    cache, idx, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=128, bits=bits, G=G, key_axis=axis, sm_scale=0.088)
    out = orc.decode_attn(q, cache, 0.088)
    for h in range(Hq):
        g = h // 2
        Kd, Vd = orc.dequantize_head(cache, 0, g)
        Kall = np.concatenate([Kd, k[0, g, L - W:].astype(np.float64)])
        Vall = np.concatenate([Vd, v[0, g, L - W:].astype(np.float64)])
        ref = sdpa_f64(q[0, h], Kall, Vall, 0.088)
        np.testing.assert_allclose(out[0, h], ref, rtol=1e-12, atol=1e-14)
        # and stays close to exact attention over the same rows at 8 bits
        if bits == 8:
            rows = np.concatenate([idx[0, g], np.arange(L - W, L)])
            exact = sdpa_f64(q[0, h], k[0, g, rows], v[0, g, rows], 0.088)
            assert np.abs(out[0, h] - exact).max() < 0.02


def test_all_keys_equal_gives_mean_of_values(orc):
    B, H, L, W, D = 1, 2, 72, 8, 64
    q_obs, k, v = synth.prompt_host(B, H, H, L, W, D, config=73)
    k[:] = k[:, :, :1, :]
    q = synth.decode_query_host(B, H, D, config=73)
    cache, idx, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=32, bits=4, G=32, sm_scale=0.1)
    out = orc.decode_attn(q, cache, 0.1)
    for h in range(H):
        _, Vd = orc.dequantize_head(cache, 0, h)
        Kd, _ = orc.dequantize_head(cache, 0, h)
        # constant key columns are degenerate groups: dequantization is exact
        assert np.array_equal(Kd, np.broadcast_to(k[0, h, 0].astype(np.float64), Kd.shape))
        mean = np.concatenate([Vd, v[0, h, L - W:].astype(np.float64)]).mean(axis=0)
        np.testing.assert_allclose(out[0, h], mean, rtol=1e-12, atol=1e-14)


def test_single_token_returns_its_value_row(orc):
    D = 64
    rng = np.random.default_rng(2)
    k = rng.standard_normal((1, 1, 2, D)).astype(np.float16)
    v = rng.standard_normal((1, 1, 2, D)).astype(np.float16)
    q = rng.standard_normal((1, 1, D)).astype(np.float16)
    idx = np.zeros((1, 1, 0), np.int32)
    cache = orc.quantize_selected(k, v, idx, W=1, bits=4, G=32)          # nothing kept, one tail row
    out = orc.decode_attn(q, cache, 0.3)
    assert np.array_equal(out[0, 0], v[0, 0, 1].astype(np.float64))


def test_rows_may_move_between_packed_16bit_part_and_tail(orc):
    B, H, L, D = 1, 2, 96, 64
    q_obs, k, v = synth.prompt_host(B, H, H, L, 32, D, config=74)
    q = synth.decode_query_host(B, H, D, config=74)
    outs = []
    for W in (32, 64):                      # same 96 rows, split 64+32 or 32+64
        idx = np.broadcast_to(np.arange(L - W, dtype=np.int32), (B, H, L - W)).copy()
        cache = orc.quantize_selected(k, v, idx, W=W, bits=16, G=32)
        outs.append(orc.decode_attn(q, cache, 0.1))
    np.testing.assert_allclose(outs[0], outs[1], rtol=1e-12, atol=1e-14)


def test_error_against_16bit_grows_as_bits_shrink(orc):
    B, Hq, Hkv, L, W, D = 1, 4, 1, 600, 8, 128
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=75)
    idx = np.arange(512, dtype=np.int32).reshape(1, 1, 512)
    errs = []
    ref = None
    for bits in (16, 8, 4, 2):
        cache = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=32)
        acc = 0.0
        for step in range(8):
            q = synth.decode_query_host(B, Hq, D, config=75, step=step)
            o = orc.decode_attn(q, cache, 1 / np.sqrt(D))
            if bits == 16:
                ref = ref or {}
                ref[step] = o
            else:
                acc += np.abs(o - ref[step]).mean()
        if bits != 16:
            errs.append(acc)
    assert errs[0] < errs[1] < errs[2]


def test_decode_over_a_count_that_is_no_multiple_of_the_block_or_group(orc):
    """1000 kept tokens (Section 3: any s < n) at 4 bits, per-channel key groups of 32 (the last one
    holds 8 tokens): decode equals plain float64 attention on the dequantized rows plus the tail."""
    B, Hq, Hkv, L, W, n = 1, 4, 2, 1300, 8, 1000
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=93)
    c, idx, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=n, bits=4, G=32, sm_scale=0.0883883)
    assert idx.shape == (B, Hkv, n) and c.k_scale.shape == (B, Hkv, 32, 128) and c.v_scale.shape == (B, Hkv, 1024, 4)
    q = synth.decode_query_host(B, Hq, 128, config=93, step=0)
    out = orc.decode_attn(q, c, 0.0883883)
    for g in range(Hkv):
        Kd, Vd = orc.dequantize_head(c, 0, g)
        assert Kd.shape == (n, 128)
        Kall = np.concatenate([Kd, k[0, g, L - W:].astype(np.float64)])
        Vall = np.concatenate([Vd, v[0, g, L - W:].astype(np.float64)])
        for hh in range(2 * g, 2 * g + 2):
            s = 0.0883883 * (Kall @ q[0, hh].astype(np.float64))
            p = np.exp(s - s.max())
            assert np.abs(out[0, hh] - (p / p.sum()) @ Vall).max() <= 1e-12
        # half-step error bound on every element, the short group included
        x = k[0, g][idx[0, g]].astype(np.float64)
        sc = c.k_scale[0, g].view(np.float16).astype(np.float64)                        # [32 groups, 128]
        step = np.repeat(sc, 32, axis=0)[:n]
        assert np.all(np.abs(Kd - x) <= step / 2 * (1 + 2.0**-9) + 15 * step * 2.0**-11 + 1e-12)
