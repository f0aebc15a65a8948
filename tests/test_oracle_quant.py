"""Pins for the quantizer and the bit layout of the CPU checker.

Formula under test (paper, Section 3 "KV Quantization"): z = min G, m = max G,
s = (m - z)/(2^B - 1), Q(G) = round((G - z)/s), G' = Q(G) s + z.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

from paper_2412_12706_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
BITS = [2, 4, 8]


def h2f(bits16):
    return float(np.array([bits16], np.uint16).view(np.float16)[0])


@pytest.mark.parametrize("bits", BITS)
def test_end_codes_present_and_error_within_half_scale(orc, bits):
    rng = np.random.default_rng(bits)
    for trial in range(200):
        n = int(rng.choice([32, 64, 128]))
        x = (rng.standard_normal(n) * rng.choice([0.01, 1.0, 10.0, 300.0])).astype(np.float16)
        s, z, codes = orc.quantize_group(x, bits)
        sf, zf = h2f(s), h2f(z)
        assert zf == float(x.min())
        if sf == 0.0:
            assert np.all(codes == 0)
            continue
        assert codes.min() == 0 and codes.max() == 2**bits - 1
        assert codes[np.argmin(x)] == 0 and codes[np.argmax(x)] == 2**bits - 1
        deq = codes.astype(np.float64) * sf + zf
        err = np.abs(deq - x.astype(np.float64))
        # interior codes: half a step; the top code also absorbs the rounding of
        # the stored scale, (2^B - 1) * |s_h - s| <= (2^B - 1) * s * 2^-11
        assert np.all(err <= sf / 2 * (1 + 2.0**-9) + (2**bits - 1) * sf * 2.0**-11)
        inner = (codes > 0) & (codes < 2**bits - 1)
        assert np.all(err[inner] <= sf / 2 * (1 + 2.0**-9))


@pytest.mark.parametrize("bits", BITS)
def test_ramp_is_lossless(orc, bits):
    # 2^B equally spaced binary16 values with an exact step: codes 0..2^B-1 in order
    n = 2**bits
    for start, step in [(-1.0, 0.25), (3.0, 0.5), (-8.0, 0.0625 if bits < 8 else 0.125)]:
        ramp = start + step * np.arange(n)
        x = np.tile(ramp, max(1, 32 // n) if n < 32 else 1).astype(np.float16)
        assert np.array_equal(x.astype(np.float64), np.tile(ramp, max(1, 32 // n) if n < 32 else 1))
        s, z, codes = orc.quantize_group(x, bits)
        assert h2f(s) == step and h2f(z) == start
        assert np.array_equal(codes, np.tile(np.arange(n), max(1, 32 // n) if n < 32 else 1))
        assert np.array_equal(codes * h2f(s) + h2f(z), x.astype(np.float64))


@pytest.mark.parametrize("bits", BITS)
def test_constant_group_is_degenerate(orc, bits):
    for val in (0.0, -2.5, 1e-5):
        x = np.full(32, val, np.float16)
        s, z, codes = orc.quantize_group(x, bits)
        assert s == 0 and h2f(z) == float(np.float16(val)) and np.all(codes == 0)


@pytest.mark.parametrize("bits", BITS)
def test_two_valued_group_uses_only_end_codes(orc, bits):
    rng = np.random.default_rng(7)
    x = np.where(rng.random(64) < 0.5, np.float16(-1.5), np.float16(2.25)).astype(np.float16)
    x[0], x[1] = np.float16(-1.5), np.float16(2.25)
    s, z, codes = orc.quantize_group(x, bits)
    assert set(codes.tolist()) == {0, 2**bits - 1}
    assert np.array_equal(codes == 0, x == np.float16(-1.5))


def test_eight_bit_grid_is_lossless(orc):
    grid = (-4.0 + np.arange(256) / 32.0)
    rng = np.random.default_rng(8)
    x = np.concatenate([[grid[0], grid[-1]], rng.choice(grid, 126)]).astype(np.float16)
    s, z, codes = orc.quantize_group(x, 8)
    assert np.array_equal(codes * h2f(s) + h2f(z), x.astype(np.float64))


@pytest.mark.parametrize("bits", BITS)
def test_codes_agree_with_exact_rational_rounding(orc, bits):
    # the binary32 sequence may differ from exact arithmetic only next to a tie
    rng = np.random.default_rng(100 + bits)
    near_tie = 0
    for trial in range(60):
        x = (rng.standard_normal(32) * rng.choice([0.1, 1.0, 20.0])).astype(np.float16)
        s, z, codes = orc.quantize_group(x, bits)
        sF, zF = Fraction(h2f(s)), Fraction(h2f(z))
        if sF == 0:
            continue
        for xi, ci in zip(x, codes):
            t = (Fraction(float(xi)) - zF) / sF
            exact = min(max(round(t), 0), 2**bits - 1)          # Fraction.round = half to even
            if exact != ci:
                frac = t - int(t)
                assert abs(frac - Fraction(1, 2)) < Fraction(1, 2**16), (float(t), ci)
                near_tie += 1
    assert near_tie < 30


def test_scale_is_half_rounding_of_binary32_quotient(orc):
    # independent route: numpy float32 arithmetic and numpy's float16 cast
    rng = np.random.default_rng(11)
    for bits in BITS:
        for trial in range(100):
            x = (rng.standard_normal(32) * 3).astype(np.float16)
            s, z, _ = orc.quantize_group(x, bits)
            r = np.float32(x.max()) - np.float32(x.min())
            ref = (r / np.float32(2**bits - 1)).astype(np.float16)
            assert s == int(ref.view(np.uint16))


def test_signed_zero_minimum(orc):
    x = np.zeros(32, np.float16)
    x[5] = np.float16(-0.0)
    x[9] = np.float16(1.0)
    s, z, codes = orc.quantize_group(x, 4)
    assert z == 0x8000 and codes[9] == 15 and codes[0] == 0


def test_value_layout_matches_worked_examples(orc):
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLD, "v_layout_examples.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) > 25
    for bits, t, d, word, shift in rows:
        n_tok = 128
        buf = np.zeros(orc.v_words(n_tok, 128, bits), np.uint32)
        buf[word] = np.uint32((1 << shift) & 0xFFFFFFFF)
        got = orc.v_code_at(buf, 128, bits, t, d)
        assert got == 1, (bits, t, d, word, shift)


def test_key_layout_matches_worked_examples(orc):
    # hand-derived from the format statement (adjacent channels share a field index, low / high half-word)
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLD, "k_layout_examples.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) >= 24 and {r[0] for r in rows} == {2, 4, 8, 16}
    for bits, t, d, word, shift in rows:
        n_tok = 64
        buf = np.zeros(orc.k_words(n_tok, 128, bits), np.uint32)
        buf[word] = np.uint32((1 << shift) & 0xFFFFFFFF)
        assert orc.k_code_at(buf, 128, bits, t, d) == 1, (bits, t, d, word, shift)
        # and nobody else reads that bit
        hits = sum(orc.k_code_at(buf, 128, bits, tt, dd) != 0 for tt in sorted({0, t}) for dd in range(128))
        assert hits == 1, (bits, t, d)


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
@pytest.mark.parametrize("D", [64, 128])
def test_layouts_are_bijections(orc, bits, D):
    # every (token, channel) owns its own bit field; together they tile the buffer
    n_tok = 64
    for words, fn in ((orc.k_words(n_tok, D, bits), orc.k_code_at), (orc.v_words(n_tok, D, bits), orc.v_code_at)):
        assert words * 32 == n_tok * D * bits
        seen = np.zeros(words * 32 // bits, bool)
        # set one field at a time and find who reads it
        owner = {}
        buf = np.zeros(words, np.uint32)
        for w in sorted({0, 1, words // 3 + 1, words // 2 + 5, words - 1}):   # sampled words, all fields in them
            for f in range(32 // bits):
                buf[:] = 0
                buf[w] = np.uint32(((1 << bits) - 1) << (f * bits) if bits < 32 else 0)
                hits = [(t, d) for t in range(n_tok) for d in range(D) if fn(buf, D, bits, t, d)]
                assert len(hits) == 1, (w, f, hits)
                assert hits[0] not in owner
                owner[hits[0]] = (w, f)


def test_key_layout_16bit_is_plain_little_endian_half(orc):
    rng = np.random.default_rng(5)
    k = rng.standard_normal((1, 1, 40, 128)).astype(np.float16)
    idx = np.arange(32, dtype=np.int32).reshape(1, 1, 32)
    c = orc.quantize_selected(k, k, idx, W=8, bits=16, G=32)
    assert np.array_equal(c.k_codes[0, 0].view(np.uint16).reshape(32, 128), k[0, 0, :32].view(np.uint16))
    assert np.array_equal(c.tail_k[0, 0], k[0, 0, 32:].view(np.uint16))


@pytest.mark.parametrize("bits,G,axis", [(4, 32, 0), (2, 64, 0), (8, 32, 0), (4, 32, 1), (4, 64, 1), (2, 128, 0)])
def test_cache_groups_follow_the_stated_axes(orc, bits, G, axis):
    """Keys per channel over G consecutive *kept* tokens (axis 0) or per token
    over G consecutive channels (axis 1); values always per token (paper,
    Section 2 "KV Quantization" and Section 6.3)."""
    B, Hkv, L, W, D = 1, 2, 300, 8, 128
    _, k, v = synth.prompt_host(B, 4, Hkv, L, W, D, config=80)
    rng = np.random.default_rng(bits * G)
    n_kept = 128
    idx = np.stack([np.sort(rng.choice(L - W, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    c = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G, key_axis=axis)
    for g in range(Hkv):
        ks, vs = k[0, g, idx[0, g]], v[0, g, idx[0, g]]            # gathered survivors, ascending
        Kd, Vd = orc.dequantize_head(c, 0, g)
        # group extrema are reproduced exactly: z is stored exactly and code 0 sits on it
        if axis == 0:
            mins = ks.reshape(n_kept // G, G, D).min(axis=1)
            assert np.array_equal(c.k_zero[0, g].view(np.float16), mins)
            sc = c.k_scale[0, g].view(np.float16).astype(np.float64)
            err = np.abs(Kd - ks.astype(np.float64)).reshape(n_kept // G, G, D)
            assert np.all(err <= sc[:, None, :] * (0.5 + 2.0**-10 + (2**bits - 1) * 2.0**-11))
        else:
            mins = ks.reshape(n_kept, D // G, G).min(axis=2)
            assert np.array_equal(c.k_zero[0, g].view(np.float16), mins)
            sc = c.k_scale[0, g].view(np.float16).astype(np.float64)
            err = np.abs(Kd - ks.astype(np.float64)).reshape(n_kept, D // G, G)
            assert np.all(err <= sc[:, :, None] * (0.5 + 2.0**-10 + (2**bits - 1) * 2.0**-11))
        vmins = vs.reshape(n_kept, D // G, G).min(axis=2)
        assert np.array_equal(c.v_zero[0, g].view(np.float16), vmins)
        vsc = c.v_scale[0, g].view(np.float16).astype(np.float64)
        verr = np.abs(Vd - vs.astype(np.float64)).reshape(n_kept, D // G, G)
        assert np.all(verr <= vsc[:, :, None] * (0.5 + 2.0**-10 + (2**bits - 1) * 2.0**-11))
        # codes in the cache are exactly the single-group quantizer's codes
        t0, d0 = 37, 77
        if axis == 0:
            u = t0 // G
            _, _, codes = orc.quantize_group(ks[u * G:(u + 1) * G, d0].copy(), bits)
            assert c.k_code(0, g, t0, d0) == codes[t0 % G]
        _, _, codes = orc.quantize_group(vs[t0, (d0 // G) * G:(d0 // G + 1) * G].copy(), bits)
        assert c.v_code(0, g, t0, d0) == codes[d0 % G]
    assert np.array_equal(c.tail_v[0, :, :W].view(np.float16), v[0, :, L - W:])


def test_per_channel_keys_beat_per_token_keys_with_outlier_channels(orc):
    # qualitative agreement with the paper's ablation (Section 6.3): with a few
    # large key channels, grouping keys along the channel axis loses less
    B, Hkv, L, W, D = 1, 2, 600, 8, 128
    _, k, v = synth.prompt_host(B, 4, Hkv, L, W, D, config=81)
    idx = np.broadcast_to(np.arange(512, dtype=np.int32), (B, Hkv, 512)).copy()
    errs = []
    for axis in (0, 1):
        c = orc.quantize_selected(k, v, idx, W=W, bits=4, G=32, key_axis=axis)
        Kd, _ = orc.dequantize_head(c, 0, 0)
        errs.append(np.abs(Kd - k[0, 0, :512].astype(np.float64)).mean())
    assert errs[0] < errs[1]


def test_fewer_bits_lose_more(orc):
    B, Hkv, L, W, D = 1, 1, 300, 8, 128
    _, k, v = synth.prompt_host(B, 4, Hkv, L, W, D, config=82)
    idx = np.arange(256, dtype=np.int32).reshape(1, 1, 256)
    e = []
    for bits in (8, 4, 2):
        c = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=32)
        Kd, Vd = orc.dequantize_head(c, 0, 0)
        e.append(np.abs(Vd - v[0, 0, :256].astype(np.float64)).mean() + np.abs(Kd - k[0, 0, :256].astype(np.float64)).mean())
    assert e[0] < e[1] < e[2]


def test_token_count_that_fills_neither_a_block_nor_a_key_group(orc):
    """Section 3 only asks for s < n kept tokens.  40 tokens with per-channel key groups of 32: group 0
    has 32 members, group 1 the remaining 8 -- the same quantizer on fewer members, so closed forms
    hold inside it: a ramp of the four 2-bit levels is lossless with scale = step, a constant channel
    has scale 0, and the scale is the numpy float32 route of that group's own range.  Rows past the
    count (the arrays are laid out for whole blocks of 32) stay zero."""
    rng = np.random.default_rng(11)
    n, G, D = 40, 32, 128
    rows = rng.standard_normal((n, D)).astype(np.float16)
    rows[32:, 5] = np.array([0.5, 1.0, 1.5, 2.0, 0.5, 2.0, 1.0, 1.5], np.float16)     # ramp 0.5 .. 2.0 in steps of 0.5
    rows[32:, 6] = np.float16(-3.25)                                                    # constant in the short group only
    k = np.concatenate([rows, np.zeros((1, D), np.float16)])[None, None]
    idx = np.arange(n, dtype=np.int32)[None, None]
    c = orc.quantize_selected(k, k.copy(), idx, W=1, bits=2, G=G, key_axis=0)
    assert c.k_scale.shape == (1, 1, 2, D) and c.v_scale.shape == (1, 1, 64, D // G) and c.k_codes.shape[-1] == 64 * D * 2 // 32
    h = lambda bits16: float(np.array([bits16], np.uint16).view(np.float16)[0])
    assert h(c.k_scale[0, 0, 1, 5]) == 0.5 and h(c.k_zero[0, 0, 1, 5]) == 0.5
    assert [c.k_code(0, 0, 32 + e, 5) for e in range(8)] == [0, 1, 2, 3, 0, 3, 1, 2]
    assert c.k_scale[0, 0, 1, 6] == 0 and h(c.k_zero[0, 0, 1, 6]) == -3.25 and all(c.k_code(0, 0, 32 + e, 6) == 0 for e in range(8))
    for d in range(D):
        for u, (a, b) in enumerate(((0, 32), (32, 40))):
            x = rows[a:b, d]
            r = np.float32(x.max()) - np.float32(x.min())
            assert c.k_scale[0, 0, u, d] == int((r / np.float32(3)).astype(np.float16).view(np.uint16)), (u, d)
            assert h(c.k_zero[0, 0, u, d]) == float(x.min())
    # nothing leaks into the rows past the count
    assert not c.v_scale[0, 0, n:].any() and not c.v_zero[0, 0, n:].any()
    assert all(c.k_code(0, 0, t, d) == 0 and c.v_code(0, 0, t, d) == 0 for t in range(n, 64) for d in (0, 5, 127))
    Kd, Vd = orc.dequantize_head(c, 0, 0)
    assert Kd.shape == (n, D) and np.array_equal(Kd[32:, 5], rows[32:, 5].astype(np.float64))
    # the first group does not depend on what follows it: the same 32 tokens alone give the same codes
    c32 = orc.quantize_selected(k, k.copy(), idx[..., :32], W=1, bits=2, G=G, key_axis=0)
    assert np.array_equal(c32.k_scale[0, 0, 0], c.k_scale[0, 0, 0])
    assert all(c32.k_code(0, 0, t, d) == c.k_code(0, 0, t, d) for t in range(32) for d in range(0, D, 7))
