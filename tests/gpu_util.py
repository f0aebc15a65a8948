"""Helpers for the GPU parity tests: move caches between the CPU checker's
numpy layout and the library's device buffers (byte-for-byte, no arithmetic)."""
import numpy as np
import torch

from paper_2412_12706_amd import kvqp

NAMES = ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v")


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def upload_cache(oc, device="cuda"):
    """oracle Cache (numpy) -> kvqp.Cache (device byte tensors)."""
    bufs = {}
    for n in NAMES:
        arr = np.ascontiguousarray(getattr(oc, n))
        bufs[n] = torch.from_numpy(arr.view(np.uint8).reshape(-1).copy()).to(device)
    if getattr(oc, "k_out", None) is not None:        # outlier slots and overflow lists (compact layout: the same bytes)
        for n in ("k_out", "v_out", "k_ovf", "v_ovf"):
            bufs[n] = torch.from_numpy(np.ascontiguousarray(getattr(oc, n)).view(np.uint8).reshape(-1).copy()).to(device)
    return kvqp.Cache(bufs, oc.n_kept, oc.tail_len, oc.tail_cap)


def ovf_split(words, n_layout, cap):
    """One head's overflow buffer (uint32 words, laid out for n_layout tokens and cap entries, the
    format statement of kvqp.h) -> (prefix counts [n_layout/32 + 1], entry words [cap, 2])."""
    blocks = (n_layout + 31) // 32
    n_start = (blocks + 1 + 3) // 4 * 4
    words = np.asarray(words).reshape(-1)
    assert words.size == n_start + 2 * cap, (words.size, n_start, cap)
    return words[: blocks + 1], words[n_start:].reshape(cap, 2)


def assert_overflow_equal(got_words, n_layout, ref_words, n_tok, cap, what=""):
    """The library's overflow buffer of one head (laid out for n_layout >= n_tok tokens) against the
    checker's (laid out for n_tok): the prefix counts of the n_tok tokens and the stored entries;
    what lies beyond them is unspecified."""
    gs, ge = ovf_split(got_words, n_layout, cap)
    rs, re_ = ovf_split(ref_words, n_tok, cap)
    nb = (n_tok + 31) // 32 + 1
    assert np.array_equal(gs[:nb], rs), (what, gs[:nb][-4:], rs[-4:])
    n = min(int(rs[-1]), cap)
    assert np.array_equal(ge[:n], re_[:n]), (what, n)
    return int(rs[-1])


def download(cache, name, dtype):
    return cache.buffers[name].cpu().numpy().view(dtype)


def assert_cache_equal(gc, oc):
    """Every buffer of the device cache equals the checker's, bit for bit."""
    assert gc.n_kept == oc.n_kept and gc.tail_len == oc.tail_len
    names = NAMES + (("k_out", "v_out") if getattr(oc, "k_out", None) is not None else ())
    if getattr(oc, "k_out", None) is not None:
        heads = oc.B * oc.Hkv
        for n in ("k_ovf", "v_ovf"):
            got = download(gc, n, np.uint32).reshape(heads, -1)
            ref = np.ascontiguousarray(getattr(oc, n)).reshape(heads, -1)
            for h in range(heads):
                assert_overflow_equal(got[h], gc.n_cap or gc.n_kept, ref[h], oc.n_kept, oc.ovf_cap, f"{n} head {h}")
    for n in names:
        ref = np.ascontiguousarray(getattr(oc, n))
        got = download(gc, n, ref.dtype)
        if n.startswith("tail"):
            got = got.reshape(ref.shape)[:, :, : oc.tail_len]
            ref = ref[:, :, : oc.tail_len]
        bad = np.flatnonzero(got.reshape(-1) != ref.reshape(-1))
        assert bad.size == 0, f"{n}: {bad.size} of {ref.size} words differ, first at {bad[:5]}"


ATTN_TOL = 2e-3


def attn_excess(out, ref):
    """Largest amount by which |out - ref| exceeds its allowance (<= 0 means the bar is met).

    The bar is plain max-abs 2e-3 between the library's binary16 output and the checker's binary64
    result.  Only where |ref| >= 4 -- outputs that the cases with planted value outliers produce,
    and whose binary16 neighbours are 2^-8 |ref| or more apart, so that no binary16 number need
    lie within 2e-3 of the exact result -- is the exact result's own distance to the nearest
    binary16 number added to the allowance: the comparison is then against the checker's output
    rounded to binary16, plus 2e-3.  Nothing is relaxed below magnitude 4."""
    out = out.cpu().numpy() if hasattr(out, "cpu") else np.asarray(out)
    out = out.astype(np.float64)
    ref = np.asarray(ref, np.float64)
    own_rounding = np.abs(ref.astype(np.float16).astype(np.float64) - ref)
    allow = ATTN_TOL + np.where(np.abs(ref) >= 4.0, own_rounding, 0.0)
    return float((np.abs(out - ref) - allow).max())


def attn_maxabs(out, ref):
    """Plain max-abs error of a decode output against the checker's binary64 result."""
    out = out.cpu().numpy() if hasattr(out, "cpu") else np.asarray(out)
    return float(np.abs(out.astype(np.float64) - np.asarray(ref, np.float64)).max())
