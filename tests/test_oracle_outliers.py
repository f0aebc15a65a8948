"""Pins for the CPU checker's outlier filtering (paper, Section 6.3 item (1) and
Appendix B "KV quantization": numbers with |x| > 6, about 1 %, are excluded from
quantization -- every such number, with no limit per row).  Where the excluded
numbers are kept (four slots per token row, an overflow list per head for rows with
more) and the word format are this build's; the pins below fix them with hand-worked
values, closed forms and properties that do not go through the checker's own
arithmetic."""
import numpy as np
import pytest

from paper_2412_12706_amd import synth


def h2f(bits16):
    return float(np.array([bits16], np.uint16).view(np.float16)[0])


def f32_bits(x):
    return int(np.array([x], np.float32).view(np.uint32)[0])


def one_head(k_rows, v_rows, W=1):
    """[n, 128] float16 rows -> k, v [1,1,n+W,128] with W zero rows appended as the window."""
    pad = np.zeros((W, 128), np.float16)
    return (np.concatenate([k_rows, pad])[None, None].copy(), np.concatenate([v_rows, pad])[None, None].copy())


def test_hand_worked_row_2_bits(orc):
    """Values 0,1,2,3 repeating (range 3 -> 2-bit scale exactly 1, codes = values) with 100 in
    channel 5 and -50 in channel 77.  Unfiltered, the range is 150 and the scale 50; filtered at
    6 the two are slots (difference to the zero-point 0, top 24 bits of its binary32 pattern,
    valid bit, channel) and everything else is lossless."""
    base = (np.arange(128) % 4).astype(np.float16)
    row = base.copy()
    row[5], row[77] = 100.0, -50.0
    rows = np.tile(row, (32, 1))
    k, v = one_head(rows, rows)
    idx = np.arange(32, dtype=np.int32)[None, None]
    plain = orc.quantize_selected(k, v, idx, W=1, bits=2, G=128, key_axis=1)
    assert h2f(plain.v_scale[0, 0, 0, 0]) == 50.0 and h2f(plain.v_zero[0, 0, 0, 0]) == -50.0
    c = orc.quantize_selected(k, v, idx, W=1, bits=2, G=128, key_axis=1, tau=6.0)
    # 100.0f = 0x42C80000, -50.0f = 0xC2480000
    want = np.array([0x42C80000 | 0x80 | 5, 0xC2480000 | 0x80 | 77, 0, 0], np.uint32)
    assert f32_bits(100.0) == 0x42C80000 and f32_bits(-50.0) == 0xC2480000
    for t in range(32):
        assert np.array_equal(c.v_out[0, 0, t], want) and np.array_equal(c.k_out[0, 0, t], want)
        assert h2f(c.v_scale[0, 0, t, 0]) == 1.0 and h2f(c.v_zero[0, 0, t, 0]) == 0.0
        for d in range(128):
            expect = 0 if d in (5, 77) else int(base[d])
            assert c.v_code(0, 0, t, d) == expect and c.k_code(0, 0, t, d) == expect
    Kd, Vd = orc.dequantize_head(c, 0, 0)
    assert np.array_equal(Kd, rows.astype(np.float64)) and np.array_equal(Vd, rows.astype(np.float64))


def test_hand_worked_row_with_more_outliers_than_slots(orc):
    """Six outliers in a row: the four in the lowest channels fill the slots, the other two go to
    the head's overflow list as (word, token) in (token, channel) order, with the prefix count of
    every block of 32 tokens in front.  Token 40 alone has them; 64 tokens, so the prefix array is
    (0, 0, 2) padded to four ints.  All six come back exactly; the rest is lossless."""
    base = (np.arange(128) % 4).astype(np.float16)
    rows = np.tile(base, (64, 1))
    big = {3: 100.0, 10: -50.0, 64: 7.0, 65: -6.5, 100: 24.0, 127: 9.0}      # channel -> value, all |x| > 6
    for d, x in big.items():
        rows[40, d] = x
    k, v = one_head(rows, rows)
    idx = np.arange(64, dtype=np.int32)[None, None]
    c = orc.quantize_selected(k, v, idx, W=1, bits=2, G=128, key_axis=1, tau=6.0, ovf_cap=5)
    word = lambda x, d: (f32_bits(x) & 0xFFFFFF00) | 0x80 | d            # the group's zero-point is 0
    want_slots = np.array([word(100.0, 3), word(-50.0, 10), word(7.0, 64), word(-6.5, 65)], np.uint32)
    assert f32_bits(7.0) == 0x40E00000 and f32_bits(-6.5) == 0xC0D00000 and f32_bits(24.0) == 0x41C00000 and f32_bits(9.0) == 0x41100000
    for out, ovf in ((c.k_out, c.k_ovf), (c.v_out, c.v_ovf)):
        assert np.array_equal(out[0, 0, 40], want_slots)
        assert not out[0, 0, :40].any() and not out[0, 0, 41:].any()
        buf = ovf[0, 0]
        assert buf.size == 4 + 2 * 5                                      # three prefix counts padded to four, five entries of two words
        assert buf[:4].tolist() == [0, 0, 2, 0]
        assert buf[4:8].tolist() == [0x41C00000 | 0x80 | 100, 40, 0x41100000 | 0x80 | 127, 40]
        assert not buf[8:].any()
    for t in range(64):
        for d in range(128):
            expect = 0 if (t == 40 and d in big) else int(base[d])
            assert c.v_code(0, 0, t, d) == expect and c.k_code(0, 0, t, d) == expect
    Kd, Vd = orc.dequantize_head(c, 0, 0)
    assert np.array_equal(Kd, rows.astype(np.float64)) and np.array_equal(Vd, rows.astype(np.float64))
    # an overflow list that is too short loses the entries beyond it (those elements read as their
    # group's zero-point) and shows the shortfall in the prefix counts
    short = orc.quantize_selected(k, v, idx, W=1, bits=2, G=128, key_axis=1, tau=6.0, ovf_cap=1)
    assert short.k_ovf[0, 0][:3].tolist() == [0, 0, 2] and short.k_ovf[0, 0][4:6].tolist() == [0x41C00000 | 0x80 | 100, 40]
    Ks, _ = orc.dequantize_head(short, 0, 0)
    lost = rows.astype(np.float64).copy()
    lost[40, 127] = 0.0
    assert np.array_equal(Ks, lost)


def test_threshold_out_of_reach_changes_nothing(orc):
    B, Hq, Hkv, L, W = 1, 4, 2, 300, 8
    _, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, outlier=10.0, config=70)
    idx = np.stack([[np.sort(np.random.default_rng(g).choice(L - W, 128, replace=False)) for g in range(Hkv)]]).astype(np.int32)
    for axis in (0, 1):
        a = orc.quantize_selected(k, v, idx, W=W, bits=4, G=32, key_axis=axis)
        b = orc.quantize_selected(k, v, idx, W=W, bits=4, G=32, key_axis=axis, tau=7.0e4)   # above the binary16 range
        for n in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero"):
            assert np.array_equal(getattr(a, n), getattr(b, n)), n
        assert not b.k_out.any() and not b.v_out.any() and not b.k_ovf.any() and not b.v_ovf.any()


def test_which_elements_are_outliers(orc):
    """Brute force: every element with |x| > tau, numbered in ascending channel order.  Includes rows
    with none, with more than four and with magnitudes exactly at the threshold."""
    rng = np.random.default_rng(71)
    for trial in range(300):
        row = rng.standard_normal(128).astype(np.float16)
        n_big = int(rng.integers(0, 9))
        pos = rng.choice(128, n_big, replace=False)
        mags = rng.choice([6.0, 6.5, 8.0, 8.0, 20.0, 33.0], n_big)     # 6.0 is not above the threshold; ties on 8.0
        row[pos] = (mags * rng.choice([-1.0, 1.0], n_big)).astype(np.float16)
        mask = orc.mark_outliers(row, 6.0)
        a = np.abs(row.astype(np.float64))
        cand = [d for d in range(128) if a[d] > 6.0]
        want = np.zeros(128, np.uint8)
        want[cand] = np.arange(1, len(cand) + 1)                  # 1 + outliers in lower channels
        assert np.array_equal(mask, want)


def test_slot_word_and_value(orc):
    """The slot keeps the top 24 bits of float(x) - float(z): reconstructed value within 2^-15
    of the difference; channel and valid bit in the low byte."""
    rng = np.random.default_rng(72)
    for trial in range(2000):
        x = np.float16(rng.choice([-1, 1]) * rng.uniform(6, 60000))
        z = np.float16(rng.uniform(-6, 6))
        d = int(rng.integers(0, 128))
        slot = orc.outlier_slot(x.view(np.uint16), z.view(np.uint16), d)
        assert slot & 0x7F == d and slot & 0x80
        diff = float(x) - float(z)                      # exact in binary64
        got = orc.outlier_value(slot, z.view(np.uint16))
        assert abs(got - float(x)) <= abs(diff) * 2.0**-15
        # truncation, never away from zero: |stored difference| <= |binary32 difference|
        assert abs(got - float(z)) <= abs(float(np.float32(x) - np.float32(z)))


@pytest.mark.parametrize("bits,G,axis", [(2, 32, 0), (4, 64, 1), (8, 128, 0), (4, 32, 1)])
def test_group_ranges_exclude_outliers_and_errors_stay_bounded(orc, bits, G, axis):
    """With a few channels scaled by 20 (the structure behind the paper's 1 % figure) every
    group's stored range is that of its non-outlier elements, their error is within half a step,
    and outliers come back to 2^-15 of their distance from the zero-point."""
    B, Hq, Hkv, L, W, n = 1, 4, 1, 400, 8, 256
    _, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, outlier=20.0, config=73)
    v[..., [3, 64]] = (v[..., [3, 64]].astype(np.float32) * 12).astype(np.float16)   # values get outlier channels too
    k[..., [50, 51, 90]] = (k[..., [50, 51, 90]].astype(np.float32) * 15).astype(np.float16)   # key rows with up to seven
    idx = np.sort(np.random.default_rng(73).choice(L - W, n, replace=False)).astype(np.int32)[None, None]
    c = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G, key_axis=axis, tau=6.0)
    Kd, Vd = orc.dequantize_head(c, 0, 0)
    levels = 2**bits - 1
    for name, src, deq, scale, zero, out, ovf, ax in (("k", k, Kd, c.k_scale, c.k_zero, c.k_out, c.k_ovf, axis),
                                                      ("v", v, Vd, c.v_scale, c.v_zero, c.v_out, c.v_ovf, 1)):
        rows = src[0, 0][idx[0, 0]]                                  # [n, 128] float16
        x = rows.astype(np.float64)
        mask = np.abs(x) > 6.0                                       # the paper's rule, nothing else
        assert mask.sum() > 0.003 * mask.size                        # the case does contain outliers
        if name == "k":
            assert (mask.sum(axis=1) > 4).sum() > n // 4             # and key rows that overflow their slots
        # slots list the first four marked channels in ascending order, zeros after; the overflow
        # list holds the rest in (token, channel) order and its prefix counts match
        start, entries = orc.ovf_entries(ovf[0, 0], n, c.ovf_cap)
        want_entries, want_start = [], [0]
        for t in range(n):
            marked = np.flatnonzero(mask[t]).tolist()
            chans = [int(s & 0x7F) for s in out[0, 0, t] if s & 0x80]
            assert chans == marked[:4]
            assert all(s == 0 for s in out[0, 0, t][len(chans):])
            want_entries += [(d, t) for d in marked[4:]]
            if t % 32 == 31:
                want_start.append(len(want_entries))
        assert start.tolist() == want_start
        assert [(int(w & 0x7F), int(t)) for w, t in entries] == want_entries and all(w & 0x80 for w, _ in entries)
        if ax == 0:    # groups of G tokens per channel
            xs = x.reshape(n // G, G, 128).transpose(0, 2, 1)        # [group, channel, member]
            ms = mask.reshape(n // G, G, 128).transpose(0, 2, 1)
            ds = deq.reshape(n // G, G, 128).transpose(0, 2, 1)
            sc, ze = scale[0, 0].astype(np.uint16), zero[0, 0].astype(np.uint16)   # [n/G, 128]
        else:          # groups of G channels per token
            xs, ms, ds = x.reshape(n, 128 // G, G), mask.reshape(n, 128 // G, G), deq.reshape(n, 128 // G, G)
            sc, ze = scale[0, 0], zero[0, 0]                                        # [n, 128/G]
        sf = sc.view(np.float16).astype(np.float64)
        zf = ze.view(np.float16).astype(np.float64)
        for gi in np.ndindex(xs.shape[:2]):
            keep = ~ms[gi]
            if not keep.any():
                assert sf[gi] == 0.0 and zf[gi] == 0.0
                continue
            lo, hi = xs[gi][keep].min(), xs[gi][keep].max()
            assert zf[gi] == lo
            assert abs(sf[gi] - (hi - lo) / levels) <= (hi - lo) / levels * 2.0**-10 + 1e-12
            err = np.abs(ds[gi] - xs[gi])
            assert np.all(err[keep] <= sf[gi] / 2 * (1 + 2.0**-9) + levels * sf[gi] * 2.0**-11 + 1e-12), name
            assert np.all(err[ms[gi]] <= np.abs(xs[gi][ms[gi]] - zf[gi]) * 2.0**-15), name


def test_channel_that_is_an_outlier_in_every_token(orc):
    """Per-channel key groups: a channel at 50 in all tokens leaves its groups empty (scale 0,
    zero +0, codes 0) and still dequantizes to 50."""
    rng = np.random.default_rng(74)
    rows = rng.standard_normal((64, 128)).astype(np.float16)
    rows[:, 9] = 50.0
    k, v = one_head(rows, rows)
    idx = np.arange(64, dtype=np.int32)[None, None]
    c = orc.quantize_selected(k, v, idx, W=1, bits=4, G=32, key_axis=0, tau=6.0)
    assert np.all(c.k_scale[0, 0, :, 9] == 0) and np.all(c.k_zero[0, 0, :, 9] == 0)
    assert all(c.k_code(0, 0, t, 9) == 0 for t in range(64))
    Kd, _ = orc.dequantize_head(c, 0, 0)
    assert np.all(Kd[:, 9] == 50.0)


def test_decode_over_outlier_cache_is_plain_attention_on_its_dequantized_rows(orc):
    B, Hq, Hkv, L, W, n = 1, 4, 2, 300, 8, 128
    q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, outlier=20.0, config=75)
    c, idx, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=n, bits=4, G=32, sm_scale=0.0883883, tau=6.0)
    plain, idx2, _ = orc.compress(q_obs, k, v, window=W, pool=7, budget=n, bits=4, G=32, sm_scale=0.0883883)
    assert np.array_equal(idx, idx2)                 # selection does not look at the quantizer
    q = synth.decode_query_host(B, Hq, 128, config=75, step=0)
    out = orc.decode_attn(q, c, 0.0883883)
    for g in range(Hkv):
        Kd, Vd = orc.dequantize_head(c, 0, g)
        Kall = np.concatenate([Kd, k[0, g, L - W:].astype(np.float64)])
        Vall = np.concatenate([Vd, v[0, g, L - W:].astype(np.float64)])
        for h in range(2 * g, 2 * g + 2):
            s = 0.0883883 * (Kall @ q[0, h].astype(np.float64))
            p = np.exp(s - s.max())
            ref = (p / p.sum()) @ Vall
            assert np.abs(out[0, h] - ref).max() <= 1e-12
    # and filtering does what it is for: the dequantized keys are closer to the originals
    Kp, _ = orc.dequantize_head(plain, 0, 0)
    Ko, _ = orc.dequantize_head(c, 0, 0)
    x = k[0, 0][idx[0, 0]].astype(np.float64)
    assert np.abs(Ko - x).mean() < np.abs(Kp - x).mean()
