"""ctypes/numpy front end of the CPU oracle (oracle/kvqp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and
by bench.py's cpu_baseline leg.  Nothing in the product package may import
this module, and this module imports nothing from the product package.

All arrays are numpy, host memory.  binary16 data travels as uint16 bit
patterns or np.float16 (viewed, never converted).  Argument marshalling only:
every number is produced by the C file.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvqp_oracle.c")
_LIB = os.path.join(_HERE, "libkvqp_oracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  No fast-math, no FMA contraction: the
    quantizer is a fixed binary32 operation sequence."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.orc_half_to_double.restype = C.c_double
        L.orc_half_to_double.argtypes = [C.c_uint16]
        L.orc_float_to_half.restype = C.c_uint16
        L.orc_float_to_half.argtypes = [C.c_float]
        L.orc_k_words.restype = C.c_size_t
        L.orc_v_words.restype = C.c_size_t
        L.orc_k_code_get.restype = C.c_uint32
        L.orc_v_code_get.restype = C.c_uint32
        L.orc_k_code_get.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_v_code_get.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_threads.restype = C.c_int
        L.orc_rows.restype = C.c_int
        L.orc_rows.argtypes = [C.c_int]
        L.orc_key_groups.restype = C.c_int
        L.orc_key_groups.argtypes = [C.c_int, C.c_int]
        L.orc_mark_outliers.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_void_p]
        L.orc_ovf_words.restype = C.c_size_t
        L.orc_ovf_words.argtypes = [C.c_int, C.c_int]
        L.orc_outlier_slot.restype = C.c_uint32
        L.orc_outlier_slot.argtypes = [C.c_uint16, C.c_uint16, C.c_int]
        L.orc_outlier_value.restype = C.c_double
        L.orc_outlier_value.argtypes = [C.c_uint32, C.c_uint16]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    assert a.dtype == np.uint16, a.dtype
    return a


def threads() -> int:
    return int(lib().orc_threads())


def set_threads(n: int) -> None:
    """OpenMP threads used from now on (the benchmark times the oracle on one thread and on all)."""
    lib().orc_set_threads(int(n))


def half_to_double(bits16):
    a = _u16(bits16)
    out = np.empty(a.shape, np.float64)
    lib().orc_half_to_double_array(_p(a), _p(out), C.c_size_t(a.size))
    return out


def float_to_half_bits(x):
    a = np.ascontiguousarray(x, np.float32)
    out = np.empty(a.shape, np.uint16)
    lib().orc_float_to_half_array(_p(a), _p(out), C.c_size_t(a.size))
    return out


def window_votes(q_obs, k, sm_scale):
    """q_obs [B,Hq,W,D], k [B,Hkv,L,D] (float16) -> vote [B,Hkv,L-W] float64."""
    q_obs, k = _u16(q_obs), _u16(k)
    B, Hq, W, D = q_obs.shape
    _, Hkv, L, _ = k.shape
    vote = np.empty((B, Hkv, L - W), np.float64)
    rc = lib().orc_window_votes(B, Hq, Hkv, D, L, W, C.c_double(sm_scale), _p(q_obs), _p(k), _p(vote))
    if rc:
        raise ValueError(f"orc_window_votes rc={rc}")
    return vote


def max_pool(vote, pool):
    vote = np.ascontiguousarray(vote, np.float64)
    P = vote.shape[-1]
    out = np.empty_like(vote)
    rc = lib().orc_max_pool(int(vote.size // max(P, 1)), P, pool, _p(vote), _p(out))
    if rc:
        raise ValueError(f"orc_max_pool rc={rc}")
    return out


def topk(pooled_row, k):
    pooled_row = np.ascontiguousarray(pooled_row, np.float64)
    idx = np.empty(k, np.int32)
    rc = lib().orc_topk(pooled_row.size, k, _p(pooled_row), _p(idx))
    if rc:
        raise ValueError(f"orc_topk rc={rc}")
    return idx


def quantize_group(x, bits):
    """x: 1-D float16 group -> (scale_bits, zero_bits, codes uint8)."""
    x = _u16(x)
    s = C.c_uint16()
    z = C.c_uint16()
    codes = np.empty(x.size, np.uint8)
    rc = lib().orc_quantize_group(_p(x), x.size, 1, bits, C.byref(s), C.byref(z), _p(codes))
    if rc:
        raise ValueError(f"orc_quantize_group rc={rc}")
    return s.value, z.value, codes


OUT_SLOTS = 4


def ovf_words(n_tok, cap):
    """32-bit words of one head's overflow buffer laid out for n_tok tokens and cap entries."""
    return int(lib().orc_ovf_words(int(n_tok), int(cap)))


def ovf_entries(buf, n_tok, cap):
    """One head's overflow buffer -> (start int32 [n_tok/32 + 1], entries uint32 [min(total, cap), 2])."""
    buf = np.ascontiguousarray(buf).view(np.uint32).reshape(-1)
    n_start = ovf_words(n_tok, cap) - 2 * cap
    start = buf[: rows(n_tok) // 32 + 1].astype(np.int64)
    n = min(int(start[-1]), cap)
    return start, buf[n_start:n_start + 2 * n].reshape(n, 2)


def mark_outliers(row, tau):
    """row: 1-D float16 token row -> uint8 array: 1 + (outliers of the row in lower channels) at its
    outliers (|x| > tau), 0 elsewhere."""
    row = _u16(row)
    mask = np.zeros(row.size, np.uint8)
    lib().orc_mark_outliers(_p(row), row.size, C.c_double(tau), _p(mask))
    return mask


def outlier_slot(x_bits, zero_bits, d):
    return int(lib().orc_outlier_slot(int(x_bits), int(zero_bits), int(d)))


def outlier_value(slot, zero_bits):
    return float(lib().orc_outlier_value(int(slot), int(zero_bits)))


def k_code_at(words, D, bits, t, d):
    """Field (t, d) of a key-code buffer of one head (uint32 array)."""
    return int(lib().orc_k_code_get(_p(words), D, bits, t, d))


def v_code_at(words, D, bits, t, d):
    """Field (t, d) of a value-code buffer of one head (uint32 array)."""
    return int(lib().orc_v_code_get(_p(words), D, bits, t, d))


def rows(n_tok):
    """Rows the per-token arrays of a head are laid out for (whole blocks of 32; the rest zeros)."""
    return int(lib().orc_rows(int(n_tok)))


def key_groups(n_tok, G):
    """Per-channel key groups of n_tok tokens (the last one short when G does not divide n_tok)."""
    return int(lib().orc_key_groups(int(n_tok), int(G)))


def k_words(n_tok, D, bits):
    return int(lib().orc_k_words(n_tok, D, bits))


def v_words(n_tok, D, bits):
    return int(lib().orc_v_words(n_tok, D, bits))


@dataclass
class Cache:
    """One layer's packed cache in host memory (layouts in kvqp_oracle.c)."""
    B: int
    Hkv: int
    D: int
    n_kept: int
    bits: int
    G: int
    key_axis: int
    tail_len: int
    tail_cap: int
    k_codes: np.ndarray  # uint32 [B,Hkv,k_words]
    v_codes: np.ndarray  # uint32 [B,Hkv,v_words]
    k_scale: np.ndarray  # uint16 [B,Hkv,key_groups,D] per channel, [B,Hkv,rows,D/G] per token
    k_zero: np.ndarray
    v_scale: np.ndarray
    v_zero: np.ndarray
    tail_k: np.ndarray  # uint16 [B,Hkv,tail_cap,D]
    tail_v: np.ndarray
    k_out: np.ndarray = None  # uint32 [B,Hkv,n_kept,OUT_SLOTS] outlier slots, or None (no filtering)
    v_out: np.ndarray = None
    ovf_cap: int = 0          # entries per head of the overflow lists
    k_ovf: np.ndarray = None  # uint32 [B,Hkv,ovf_words(n_kept, ovf_cap)] overflow buffers (with k_out)
    v_ovf: np.ndarray = None

    def k_code(self, b, g, t, d):
        return k_code_at(self.k_codes[b, g], self.D, self.bits, t, d)

    def v_code(self, b, g, t, d):
        return v_code_at(self.v_codes[b, g], self.D, self.bits, t, d)


def _alloc_cache(B, Hkv, D, n_kept, bits, G, key_axis, W, tail_cap):
    kw, vw = k_words(n_kept, D, bits), v_words(n_kept, D, bits)
    if bits == 16:
        ks = (B, Hkv, 0)
        vs = (B, Hkv, 0)
    else:
        ks = (B, Hkv, key_groups(n_kept, G), D) if key_axis == 0 else (B, Hkv, rows(n_kept), D // G)
        vs = (B, Hkv, rows(n_kept), D // G)
    return Cache(B, Hkv, D, n_kept, bits, G, key_axis, W, tail_cap,
                 np.zeros((B, Hkv, kw), np.uint32), np.zeros((B, Hkv, vw), np.uint32),
                 np.zeros(ks, np.uint16), np.zeros(ks, np.uint16),
                 np.zeros(vs, np.uint16), np.zeros(vs, np.uint16),
                 np.zeros((B, Hkv, tail_cap, D), np.uint16), np.zeros((B, Hkv, tail_cap, D), np.uint16))


def quantize_selected(k, v, idx, W, bits, G, key_axis=0, tail_cap=None, tau=None, ovf_cap=None):
    """Quantize the survivors listed in idx [B,Hkv,n_kept] (ascending); tau: outlier threshold or None;
    ovf_cap: entries per head of the overflow lists (default: room for every element)."""
    k, v = _u16(k), _u16(v)
    B, Hkv, L, D = k.shape
    idx = np.ascontiguousarray(idx, np.int32)
    n_kept = idx.shape[-1]
    tail_cap = W if tail_cap is None else tail_cap
    c = _alloc_cache(B, Hkv, D, n_kept, bits, G, key_axis, W, tail_cap)
    if tau is None:
        rc = lib().orc_quantize_selected(B, Hkv, D, L, W, n_kept, bits, G, key_axis, tail_cap, _p(k), _p(v),
                                         _p(idx), _p(c.k_codes), _p(c.v_codes), _p(c.k_scale), _p(c.k_zero),
                                         _p(c.v_scale), _p(c.v_zero), _p(c.tail_k), _p(c.tail_v))
    else:
        c.k_out = np.zeros((B, Hkv, rows(n_kept), OUT_SLOTS), np.uint32)
        c.v_out = np.zeros((B, Hkv, rows(n_kept), OUT_SLOTS), np.uint32)
        c.ovf_cap = n_kept * (D - OUT_SLOTS) if ovf_cap is None else int(ovf_cap)
        c.k_ovf = np.zeros((B, Hkv, ovf_words(n_kept, c.ovf_cap)), np.uint32)
        c.v_ovf = np.zeros((B, Hkv, ovf_words(n_kept, c.ovf_cap)), np.uint32)
        rc = lib().orc_quantize_selected_outliers(B, Hkv, D, L, W, n_kept, bits, G, key_axis, tail_cap,
                                                  C.c_double(tau), _p(k), _p(v), _p(idx), _p(c.k_codes),
                                                  _p(c.v_codes), _p(c.k_scale), _p(c.k_zero), _p(c.v_scale),
                                                  _p(c.v_zero), _p(c.tail_k), _p(c.tail_v), _p(c.k_out), _p(c.v_out),
                                                  c.ovf_cap, _p(c.k_ovf), _p(c.v_ovf))
    if rc:
        raise ValueError(f"orc_quantize_selected rc={rc}")
    return c


def compress(q_obs, k, v, *, window, pool, budget, bits, G, sm_scale, key_axis=0, tail_cap=None,
             want_pooled=True, tau=None, ovf_cap=None):
    """Whole prefill-time compression.  Returns (cache, idx, pooled).  With an outlier threshold
    the survivors are the same (selection looks at the unquantized keys) and only their
    quantization differs."""
    if tau is not None:
        _, idx, pooled = compress(q_obs, k, v, window=window, pool=pool, budget=budget, bits=bits, G=G,
                                  sm_scale=sm_scale, key_axis=key_axis, tail_cap=tail_cap, want_pooled=want_pooled)
        return quantize_selected(k, v, idx, window, bits, G, key_axis, tail_cap, tau, ovf_cap), idx, pooled
    q_obs, k, v = _u16(q_obs), _u16(k), _u16(v)
    B, Hq, W, D = q_obs.shape
    assert W == window
    _, Hkv, L, _ = k.shape
    P = L - W
    n_kept = min(budget, P)
    tail_cap = W if tail_cap is None else tail_cap
    c = _alloc_cache(B, Hkv, D, n_kept, bits, G, key_axis, W, tail_cap)
    idx = np.empty((B, Hkv, n_kept), np.int32)
    pooled = np.empty((B, Hkv, P), np.float64) if want_pooled else None
    rc = lib().orc_compress(B, Hq, Hkv, D, L, W, pool, budget, bits, G, key_axis, C.c_double(sm_scale),
                            tail_cap, _p(q_obs), _p(k), _p(v), _p(idx), _p(pooled), _p(c.k_codes),
                            _p(c.v_codes), _p(c.k_scale), _p(c.k_zero), _p(c.v_scale), _p(c.v_zero),
                            _p(c.tail_k), _p(c.tail_v))
    if rc:
        raise ValueError(f"orc_compress rc={rc}")
    return c, idx, pooled


def decode_attn(q, cache: Cache, sm_scale, n_q_heads=None):
    """q [B,Hq,D] float16 -> out [B,Hq,D] float64."""
    q = _u16(q)
    B, Hq, D = q.shape
    out = np.empty((B, Hq, D), np.float64)
    c = cache
    if c.k_out is None:
        rc = lib().orc_decode_attn(B, Hq, c.Hkv, D, c.n_kept, c.bits, c.G, c.key_axis, C.c_double(sm_scale),
                                   c.tail_len, c.tail_cap, _p(q), _p(c.k_codes), _p(c.v_codes), _p(c.k_scale),
                                   _p(c.k_zero), _p(c.v_scale), _p(c.v_zero), _p(c.tail_k), _p(c.tail_v), _p(out))
    else:
        rc = lib().orc_decode_attn_outliers(B, Hq, c.Hkv, D, c.n_kept, c.bits, c.G, c.key_axis,
                                            C.c_double(sm_scale), c.tail_len, c.tail_cap, _p(q), _p(c.k_codes),
                                            _p(c.v_codes), _p(c.k_scale), _p(c.k_zero), _p(c.v_scale),
                                            _p(c.v_zero), _p(c.tail_k), _p(c.tail_v), _p(c.k_out), _p(c.v_out),
                                            c.ovf_cap, _p(c.k_ovf), _p(c.v_ovf), _p(out))
    if rc:
        raise ValueError(f"orc_decode_attn rc={rc}")
    return out


def dequantize_head(cache: Cache, b, g):
    """Dense K', V' [n_kept, D] float64 of one head (kept tokens only)."""
    c = cache
    Kd = np.empty((c.n_kept, c.D), np.float64)
    Vd = np.empty((c.n_kept, c.D), np.float64)
    if c.k_out is None:
        lib().orc_dequantize_head(c.D, c.n_kept, c.bits, c.G, c.key_axis, _p(c.k_codes[b, g]), _p(c.v_codes[b, g]),
                                  _p(c.k_scale[b, g]), _p(c.k_zero[b, g]), _p(c.v_scale[b, g]), _p(c.v_zero[b, g]),
                                  _p(Kd), _p(Vd))
    else:
        lib().orc_dequantize_head_outliers(c.D, c.n_kept, c.bits, c.G, c.key_axis, _p(c.k_codes[b, g]),
                                           _p(c.v_codes[b, g]), _p(c.k_scale[b, g]), _p(c.k_zero[b, g]),
                                           _p(c.v_scale[b, g]), _p(c.v_zero[b, g]),
                                           _p(np.ascontiguousarray(c.k_out[b, g])),
                                           _p(np.ascontiguousarray(c.v_out[b, g])), c.ovf_cap,
                                           _p(np.ascontiguousarray(c.k_ovf[b, g])),
                                           _p(np.ascontiguousarray(c.v_ovf[b, g])), _p(Kd), _p(Vd))
    return Kd, Vd
