"""Seeded random walks through the whole path on the GPU: compress (uniform or
with head-level counts), optionally the decode-time append (Section 3, Eq. (2)),
then decode attention -- every configuration switch drawn at random from the
supported space (bits, group size, key axis, heads per KV head, window, pool
width, budget, outlier filtering, capacity layout, cache hint of the loads).

The definition is per head (each KV head is the uniform method run on that head
alone), so the CPU checker is called per head on the head's slice: indices
bit-exact up to the checker's own near-ties, every packed word, scale, zero,
outlier slot and tail row bit-exact, attention outputs within 2e-3 of
max(1, |reference|)."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import ATTN_TOL, assert_overflow_equal, attn_excess, attn_maxabs, dev, download
from tests.test_gpu_compress import check_indices
from tests.test_gpu_ragged import head_share

pytestmark = pytest.mark.gpu
D = 128


def draw_case(rng):
    bits = int(rng.choice([2, 4, 8, 16]))
    G = int(rng.choice([32, 64, 128]))
    axis = int(rng.choice([0, 1])) if bits != 16 else 0
    Gq = int(rng.choice([1, 2, 4, 8]))
    Hkv = int(rng.choice([1, 2, 3]))
    B = int(rng.choice([1, 2]))
    W = int(rng.choice([1, 8, 16, 32, 64]))
    W = min(W, 256 // Gq, 64)
    pool = int(rng.choice([1, 3, 7, 9, 13]))
    tau = float(rng.choice([0.0, 0.0, 5.0])) if bits != 16 else 0.0
    ragged = bool(rng.integers(0, 2))
    append = bool(rng.integers(0, 2))
    quantum = G if (bits != 16 and axis == 0) else 32
    q_app = max(quantum, 64 if bits == 2 else 32)          # what appended counts must be multiples of
    unit = q_app if append else quantum
    P = int(rng.integers(2 * unit + 5, 2600))
    bound = unit * int(rng.integers(1, 1 + min(P, 1536) // unit))
    heads = B * Hkv
    counts = [unit * int(rng.integers(0, 1 + bound // unit)) for _ in range(heads)] if ragged else [bound] * heads
    n_app = q_app * int(rng.integers(1, 3)) if append else 0
    hint = int(rng.choice([kvqp.CACHE_AUTO, kvqp.CACHE_STREAM, kvqp.CACHE_KEEP]))
    return dict(hint=hint, bits=bits, G=G, axis=axis, Gq=Gq, Hkv=Hkv, B=B, W=W, pool=pool, tau=tau, ragged=ragged, P=P, bound=bound,
                counts=counts, n_app=n_app)


OVF_CAP = 600     # overflow list entries per head in the walks with outlier filtering


def compare_head(orc, gc, oc, h, heads, n, bits, tau, tail_rows, n_layout):
    E = 32 // bits
    assert np.array_equal(head_share(gc, "k_codes", np.uint32, heads, h, n * D // E), oc.k_codes.reshape(-1)), ("k_codes", h)
    assert np.array_equal(head_share(gc, "v_codes", np.uint32, heads, h, oc.v_codes.size), oc.v_codes.reshape(-1)), ("v_codes", h)
    names = {nm: np.uint16 for nm in ("k_scale", "k_zero", "v_scale", "v_zero")} if bits != 16 else {}
    if tau:
        names.update(k_out=np.uint32, v_out=np.uint32)
    for nm, dt in names.items():
        ref = getattr(oc, nm).reshape(-1)
        assert np.array_equal(head_share(gc, nm, dt, heads, h, ref.size), ref), (nm, h)
    if tau:    # the rows' outliers beyond their four slots: prefix counts and list entries
        for nm in ("k_ovf", "v_ovf"):
            got = download(gc, nm, np.uint32)
            assert_overflow_equal(got.reshape(heads, -1)[h], n_layout, getattr(oc, nm).reshape(-1), n, OVF_CAP, (nm, h))
    for nm in ("tail_k", "tail_v"):
        ref = getattr(oc, nm).reshape(-1)[: tail_rows * D]
        assert np.array_equal(head_share(gc, nm, np.uint16, heads, h, ref.size), ref), (nm, h)


def decode_and_compare(orc, cfg, gc, refs, q, ws, Hkv, gq, sm):
    out = kvqp.decode_attn(cfg, dev(q), gc, workspace=ws)
    torch.cuda.synchronize()
    out = out.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(out))
    worst = 0.0
    for h, oc in enumerate(refs):
        b, g = h // Hkv, h % Hkv
        ref = orc.decode_attn(q[b:b + 1, g * gq:(g + 1) * gq], oc, sm)[0]
        got = out[b, g * gq:(g + 1) * gq]
        # plain max-abs; only the walks with planted value outliers (tau > 0) use the large-output allowance
        worst = max(worst, attn_excess(got, ref) + ATTN_TOL if cfg.outlier_threshold > 0 else attn_maxabs(got, ref))
    return worst


@pytest.mark.parametrize("block", range(8))
def test_random_walks_through_the_path(orc, block):
    rng = np.random.default_rng(41212706 + block)
    for case in range(6):
        c = draw_case(rng)
        print(f"walk {block}.{case}: {c}", flush=True)
        bits, G, axis, Gq, Hkv, B, W, pool, tau = (c[k] for k in ("bits", "G", "axis", "Gq", "Hkv", "B", "W", "pool", "tau"))
        P, bound, counts, n_app, ragged = c["P"], c["bound"], list(c["counts"]), c["n_app"], c["ragged"]
        Hq, heads = Hkv * Gq, B * Hkv
        extra = 2 * n_app + 3 if n_app else 0              # rows "decoded" after the prompt
        L = P + W
        # rows of a second seeded tensor play the tokens decoded after the prompt
        _, k_all, v_all = synth.prompt_host(B, Hq, Hkv, L + extra, W, D, config=500 + 10 * block + case)
        if tau:
            v_all[..., [5, 77]] *= 10                      # value outliers too
        q_obs, k, v = synth.prompt_host(B, Hq, Hkv, L, W, D, config=500 + 10 * block + case)
        if tau:
            v[..., [5, 77]] *= 10
        cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, pool_kernel=pool, budget=bound, bits=bits,
                       group_size=G, key_axis=axis, outlier_threshold=tau, decode_cache_hint=c["hint"],
                       outlier_overflow_cap=OVF_CAP if tau else 0)
        sm = float(np.float32(cfg.sm_scale))
        assert cfg.n_kept == bound
        n_cap = 0
        if n_app:
            n_cap = bound + 2 * n_app
            n_cap += (-n_cap) % 128
        tail_cap = W + extra + 1
        gc = kvqp.alloc_cache(cfg, tail_cap=tail_cap, n_cap=n_cap, ragged=ragged)
        for t in gc.buffers.values():
            t.fill_(0x69)
        idx_dev = torch.full((B, Hkv, bound), -3, dtype=torch.int32, device="cuda")
        if ragged:
            kvqp.compress_ragged(cfg, dev(q_obs), dev(k), dev(v), counts, gc, idx_out=idx_dev)
        else:
            kvqp.compress(cfg, dev(q_obs), dev(k), dev(v), gc, idx_out=idx_dev)
        torch.cuda.synchronize()
        assert gc.n_kept == bound and gc.tail_len == W
        idx_gpu = idx_dev.cpu().numpy()
        kw = dict(tau=tau, ovf_cap=OVF_CAP) if tau else {}
        refs, kept = [], []
        for h in range(heads):
            b, g, n = h // Hkv, h % Hkv, counts[h]
            ks, vs = k[b:b + 1, g:g + 1], v[b:b + 1, g:g + 1]
            got = idx_gpu[b:b + 1, g:g + 1, :n]
            if n:
                _, idx_orc, pooled = orc.compress(q_obs[b:b + 1, g * Gq:(g + 1) * Gq], ks, vs, window=W, pool=pool, budget=n,
                                                  bits=bits, G=G, sm_scale=sm, key_axis=axis, **kw)
                check_indices(got, idx_orc, pooled)
            oc = orc.quantize_selected(ks, vs, got, W=W, bits=bits, G=G, key_axis=axis, **kw)
            compare_head(orc, gc, oc, h, heads, n, bits, tau, W, n_cap or bound)
            refs.append(oc)
            kept.append(got.reshape(-1))
        ws = kvqp.alloc_decode_workspace(cfg)
        q = synth.decode_query_host(B, Hq, D, config=500 + 10 * block + case, step=0)
        worst = decode_and_compare(orc, cfg, gc, refs, q, ws, Hkv, Gq, sm)
        print(f"    after compress: worst attention error {worst:.2e}", flush=True)
        assert worst <= 2e-3
        if not n_app:
            continue
        # decoded tokens arrive in the tail, then the oldest n_app rows move over
        new_k, new_v = k_all[:, :, L:L + extra], v_all[:, :, L:L + extra]
        for name, rows in (("tail_k", new_k), ("tail_v", new_v)):
            t = torch.from_numpy(np.ascontiguousarray(rows).view(np.uint16).copy()).cuda().view(heads, extra, D)
            gc.buffers[name].view(torch.uint16).view(heads, tail_cap, D)[:, W:W + extra] = t
        gc.tail_len = W + extra
        if ragged:
            kvqp.append_tail_ragged(cfg, gc, n_app, counts)
        else:
            kvqp.append_tail(cfg, gc, n_app)
        torch.cuda.synchronize()
        assert gc.n_kept == bound + n_app and gc.tail_len == W + extra - n_app
        refs = []
        for h in range(heads):
            b, g, n = h // Hkv, h % Hkv, counts[h] + n_app
            # the head's whole history as one tensor: prompt rows, then the decoded rows
            ks = np.concatenate([k[b:b + 1, g:g + 1], new_k[b:b + 1, g:g + 1]], axis=2)
            vs = np.concatenate([v[b:b + 1, g:g + 1], new_v[b:b + 1, g:g + 1]], axis=2)
            own = np.concatenate([kept[h], np.arange(P, P + n_app, dtype=np.int32)]).reshape(1, 1, n)
            oc = orc.quantize_selected(ks, vs, own, W=W + extra - n_app, bits=bits, G=G, key_axis=axis, **kw)
            compare_head(orc, gc, oc, h, heads, n, bits, tau, W + extra - n_app, n_cap or bound)
            refs.append(oc)
        q = synth.decode_query_host(B, Hq, D, config=500 + 10 * block + case, step=1)
        worst = decode_and_compare(orc, cfg, gc, refs, q, ws, Hkv, Gq, sm)
        print(f"    after append of {n_app}: worst attention error {worst:.2e}", flush=True)
        assert worst <= 2e-3
