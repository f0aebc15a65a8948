"""Decode-time cache update (paper Section 3, Eq. (2): new keys and values
are concatenated to the cache; the quantizer of Section 2 keeps the most
recent tokens at full precision and quantizes them group by group).

The reference needs no new arithmetic: moving the oldest tail rows into the
low-precision part must give, bit for bit, the cache that quantizing the
survivors plus those rows in one go gives -- which the CPU checker's
quantize_selected already defines."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import NAMES, dev

pytestmark = pytest.mark.gpu
TOL = 2e-3
D = 128


def head_prefix(cache, name, head, n_heads, nbytes):
    """First nbytes of one (batch, kv head)'s share of a capacity-strided buffer."""
    t = cache.buffers[name]
    per = t.numel() // n_heads
    return t[head * per: head * per + nbytes].cpu().numpy()


def assert_packed_equal(gc, oc, n_heads):
    for name in NAMES[:6]:
        ref = np.ascontiguousarray(getattr(oc, name)).view(np.uint8).reshape(n_heads, -1)
        for h in range(n_heads):
            got = head_prefix(gc, name, h, n_heads, ref.shape[1])
            assert np.array_equal(got, ref[h]), f"{name} differs at head {h}"


def assert_tail_equal(gc, oc, n_heads):
    for name in ("tail_k", "tail_v"):
        ref = np.ascontiguousarray(getattr(oc, name)).reshape(n_heads, oc.tail_cap, D)[:, : oc.tail_len]
        got = gc.buffers[name].cpu().numpy().view(np.uint16).reshape(n_heads, gc.tail_cap, D)[:, : gc.tail_len]
        assert gc.tail_len == oc.tail_len and np.array_equal(got, ref), name


@pytest.mark.parametrize("bits,G,axis", [(4, 32, 0), (2, 64, 0), (8, 32, 1), (16, 32, 0)])
def test_capacity_layout_holds_the_same_bytes(orc, bits, G, axis):
    """Buffers laid out for more tokens than are kept: every head's share
    starts with exactly the compact bytes, and decode reads them there."""
    B, Hkv, Gq, n_kept, W, L = 2, 2, 4, 192, 32, 400
    Hq = Hkv * Gq
    _, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=80 + bits)
    rng = np.random.default_rng(bits + G)
    idx = np.stack([np.sort(rng.choice(L - W, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G, key_axis=axis)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n_kept, bits=bits, group_size=G, key_axis=axis)
    gc = kvqp.alloc_cache(cfg, n_cap=n_kept + 256)
    for t in gc.buffers.values():
        t.fill_(0x5A)
    kvqp.quantize_selected(cfg, dev(k), dev(v), dev(idx), gc)
    torch.cuda.synchronize()
    assert_packed_equal(gc, oc, B * Hkv)
    assert_tail_equal(gc, oc, B * Hkv)
    q = synth.decode_query_host(B, Hq, D, config=80)
    ref = orc.decode_attn(q, oc, cfg.sm_scale)
    out = kvqp.decode_attn(cfg, dev(q), gc)
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy().astype(np.float64) - ref).max() <= TOL


@pytest.mark.parametrize("bits,G,axis,n_app", [(4, 32, 0, 64), (4, 32, 0, 32), (2, 32, 0, 128), (2, 64, 0, 64),
                                               (8, 64, 0, 64), (4, 128, 0, 128), (4, 64, 1, 32), (16, 32, 0, 96)])
def test_append_equals_quantizing_everything_at_once(orc, bits, G, axis, n_app):
    B, Hkv, Gq, n_kept, W = 1, 2, 4, 256, 32
    Hq = Hkv * Gq
    grown = W + n_app + 41                        # tail rows after some decoding: window + appended tokens
    P = 700
    _, k, v = synth.prompt_host(B, Hq, Hkv, P + grown, grown, D, config=90 + bits)
    rng = np.random.default_rng(bits * 7 + G + n_app)
    idx = np.stack([np.sort(rng.choice(P, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    print(f"case bits={bits} G={G} axis={axis} append={n_app}", flush=True)

    # reference: survivors plus the first n_app tail rows quantized in one go, the rest is the tail
    moved = np.broadcast_to(np.arange(P, P + n_app, dtype=np.int32), (B, Hkv, n_app))
    idx_all = np.concatenate([idx, moved], axis=-1)
    oc = orc.quantize_selected(k, v, idx_all, W=grown - n_app, bits=bits, G=G, key_axis=axis)

    # library: quantize the survivors; the caller then holds all `grown` recent rows in the tail
    # (as after some decoding), and asks for the oldest n_app of them to be moved
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=P + grown, window=W, budget=n_kept, bits=bits,
                   group_size=G, key_axis=axis)
    cap = grown + 7
    gc = kvqp.alloc_cache(cfg, tail_cap=cap, n_cap=n_kept + 256)
    for t in gc.buffers.values():
        t.fill_(0xC3)
    kvqp.quantize_selected(cfg, dev(k), dev(v), dev(idx), gc)
    assert gc.n_kept == n_kept and gc.tail_len == W
    for name, src in (("tail_k", k), ("tail_v", v)):
        rows = torch.from_numpy(np.ascontiguousarray(src[:, :, P:P + grown]).view(np.uint16).copy()).cuda()
        gc.buffers[name].view(torch.uint16).view(B * Hkv, cap, D)[:, :grown] = rows.view(B * Hkv, grown, D)
    gc.tail_len = grown
    kvqp.append_tail(cfg, gc, n_app)
    torch.cuda.synchronize()
    assert gc.n_kept == n_kept + n_app and gc.tail_len == grown - n_app
    assert_packed_equal(gc, oc, B * Hkv)
    assert_tail_equal(gc, oc, B * Hkv)

    q = synth.decode_query_host(B, Hq, D, config=90)
    ref = orc.decode_attn(q, oc, cfg.sm_scale)
    out = kvqp.decode_attn(cfg, dev(q), gc)
    torch.cuda.synchronize()
    err = np.abs(out.cpu().numpy().astype(np.float64) - ref).max()
    print(f"  decode max-abs error after append {err:.3e}", flush=True)
    assert err <= TOL


def test_append_rejects_counts_that_break_groups():
    cfg = kvqp.Cfg(batch=1, n_q_heads=4, n_kv_heads=1, seq_len=400, window=96, budget=128, bits=2, group_size=32)
    gc = kvqp.alloc_cache(cfg, tail_cap=96, n_cap=256)
    gc.n_kept, gc.tail_len = 128, 96
    for n in (0, 32, 48, 128):                    # 2-bit value superblocks hold 64 tokens; only 96 rows exist
        with pytest.raises(kvqp.KvqpError):
            kvqp.append_tail(cfg, gc, n)
    gc.n_kept = 224                               # 224 + 64 > capacity
    with pytest.raises(kvqp.KvqpError):
        kvqp.append_tail(cfg, gc, 64)


def test_decode_loop_with_periodic_appends(orc):
    """A caller's decode loop: every step adds the new token's K/V row to the
    tail; whenever a whole group has accumulated beyond the window, the oldest
    group moves into the low-precision part.  The final cache must equal the
    one built in one go, and attention over it must match the checker."""
    B, Hkv, Gq, n_kept, W, G, bits, steps = 1, 2, 4, 128, 32, 32, 4, 75
    Hq = Hkv * Gq
    P = 500
    _, k, v = synth.prompt_host(B, Hq, Hkv, P + W + steps, W, D, config=99)   # rows past P + W play the decoded tokens
    rng = np.random.default_rng(99)
    idx = np.stack([np.sort(rng.choice(P, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=P + W, window=W, budget=n_kept, bits=bits, group_size=G)
    cap = W + G + 8
    gc = kvqp.alloc_cache(cfg, tail_cap=cap, n_cap=n_kept + 128)
    kd, vd = dev(k), dev(v)
    kvqp.quantize_selected(cfg, kd[:, :, :P + W].contiguous(), vd[:, :, :P + W].contiguous(), dev(idx), gc)
    tk = gc.buffers["tail_k"].view(torch.float16).view(B * Hkv, cap, D)
    tv = gc.buffers["tail_v"].view(torch.float16).view(B * Hkv, cap, D)
    moved = 0
    for s in range(steps):
        q = synth.decode_query_host(B, Hq, D, config=99, step=s)
        kvqp.decode_attn(cfg, dev(q), gc)                      # the step's attention (result unused here)
        tk[:, gc.tail_len] = kd[:, :, P + W + s].reshape(B * Hkv, D)
        tv[:, gc.tail_len] = vd[:, :, P + W + s].reshape(B * Hkv, D)
        gc.tail_len += 1
        if gc.tail_len - W >= G:
            kvqp.append_tail(cfg, gc, G)
            moved += G
    torch.cuda.synchronize()
    assert moved == 64 and gc.n_kept == n_kept + 64 and gc.tail_len == W + steps - 64
    idx_all = np.concatenate([idx, np.broadcast_to(np.arange(P, P + moved, dtype=np.int32), (B, Hkv, moved))], axis=-1)
    oc = orc.quantize_selected(k, v, idx_all, W=W + steps - moved, bits=bits, G=G)
    assert_packed_equal(gc, oc, B * Hkv)
    assert_tail_equal(gc, oc, B * Hkv)
    q = synth.decode_query_host(B, Hq, D, config=99, step=steps)
    ref = orc.decode_attn(q, oc, cfg.sm_scale)
    out = kvqp.decode_attn(cfg, dev(q), gc)
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy().astype(np.float64) - ref).max() <= TOL
