"""Thin ctypes binding of libkvqp.so (declarations: include/kvqp.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch supplies device memory and streams.  There is no fallback:
if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvqp.so")

KVQP_OK = 0
KEY_PER_CHANNEL = 0
KEY_PER_TOKEN = 1
CACHE_AUTO, CACHE_STREAM, CACHE_KEEP = 0, 1, 2     # kvqp_cfg.decode_cache_hint
EXPORTS = ["kvqp_cache_sizes", "kvqp_cache_sizes_cap", "kvqp_outlier_sizes", "kvqp_workspace_bytes", "kvqp_compress",
           "kvqp_compress_ragged", "kvqp_quantize_selected", "kvqp_quantize_selected_ragged", "kvqp_append_tail", "kvqp_append_tail_ragged", "kvqp_decode_attn", "kvqp_decode_attn_static", "kvqp_decode_workspace_init", "kvqp_strerror", "kvqp_version"]


class KvqpError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class CfgStruct(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "n_q_heads", "n_kv_heads", "head_dim", "seq_len", "window",
                                         "pool_kernel", "budget", "bits", "group_size", "key_axis",
                                         "decode_splits")] + [("sm_scale", C.c_float), ("outlier_threshold", C.c_float),
                                                            ("decode_cache_hint", C.c_int32),
                                                            ("outlier_overflow_cap", C.c_int32)]


class CacheStruct(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero",
                                          "tail_k", "tail_v")] + [(n, C.c_int32) for n in
                                                                  ("n_kept", "tail_len", "tail_cap", "n_cap")] + [
        ("head_n_kept", C.c_void_p), ("k_out", C.c_void_p), ("v_out", C.c_void_p), ("k_ovf", C.c_void_p),
        ("v_ovf", C.c_void_p)]


_lib = None


def lib():
    """Load the library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built; run `python -m paper_2412_12706_amd.build`")
        L = C.CDLL(LIB_PATH)
        L.kvqp_strerror.restype = C.c_char_p
        L.kvqp_strerror.argtypes = [C.c_int]
        L.kvqp_cache_sizes.argtypes = [C.POINTER(CfgStruct), C.c_int32, C.POINTER(C.c_size_t)]
        L.kvqp_cache_sizes_cap.argtypes = [C.POINTER(CfgStruct), C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        L.kvqp_outlier_sizes.argtypes = [C.POINTER(CfgStruct), C.c_int32, C.POINTER(C.c_size_t)]
        L.kvqp_append_tail.argtypes = [C.POINTER(CfgStruct), C.POINTER(CacheStruct), C.c_int32, C.c_void_p]
        L.kvqp_append_tail_ragged.argtypes = [C.POINTER(CfgStruct), C.POINTER(CacheStruct), C.c_int32, C.POINTER(C.c_int32), C.c_void_p]
        L.kvqp_workspace_bytes.argtypes = [C.POINTER(CfgStruct), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.kvqp_compress.argtypes = [C.POINTER(CfgStruct), C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(CacheStruct),
                                    C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvqp_compress_ragged.argtypes = [C.POINTER(CfgStruct), C.c_void_p, C.c_void_p, C.c_void_p,
                                           C.POINTER(C.c_int32), C.POINTER(CacheStruct), C.c_void_p, C.c_void_p,
                                           C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvqp_quantize_selected.argtypes = [C.POINTER(CfgStruct), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                             C.POINTER(CacheStruct), C.c_void_p]
        L.kvqp_quantize_selected_ragged.argtypes = [C.POINTER(CfgStruct), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                                    C.POINTER(C.c_int32), C.POINTER(CacheStruct), C.c_void_p]
        L.kvqp_decode_attn.argtypes = [C.POINTER(CfgStruct), C.c_void_p, C.POINTER(CacheStruct), C.c_void_p,
                                       C.c_void_p, C.c_size_t, C.c_void_p]
        L.kvqp_decode_attn_static.argtypes = [C.POINTER(CfgStruct), C.c_void_p, C.POINTER(CacheStruct), C.c_void_p, C.c_void_p]
        L.kvqp_decode_workspace_init.argtypes = [C.POINTER(CfgStruct), C.c_void_p, C.c_size_t, C.c_void_p]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().kvqp_strerror(code).decode()


def version() -> int:
    return int(lib().kvqp_version())


@dataclass
class Cfg:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int = 128
    seq_len: int = 0
    window: int = 32
    pool_kernel: int = 7
    budget: int = 0
    bits: int = 4
    group_size: int = 32
    key_axis: int = KEY_PER_CHANNEL
    decode_splits: int = 0
    sm_scale: float = 128 ** -0.5
    outlier_threshold: float = 0.0
    decode_cache_hint: int = 0      # CACHE_AUTO / CACHE_STREAM / CACHE_KEEP
    outlier_overflow_cap: int = 0   # entries of one head's overflow list (outlier filtering)

    def struct(self) -> CfgStruct:
        return CfgStruct(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.seq_len, self.window,
                         self.pool_kernel, self.budget, self.bits, self.group_size, self.key_axis,
                         self.decode_splits, self.sm_scale, self.outlier_threshold, self.decode_cache_hint,
                         self.outlier_overflow_cap)

    @property
    def n_kept(self) -> int:
        return min(self.budget, self.seq_len - self.window)


def cache_sizes(cfg: Cfg, tail_cap: int):
    out = (C.c_size_t * 8)()
    rc = lib().kvqp_cache_sizes(C.byref(cfg.struct()), tail_cap, out)
    if rc:
        raise KvqpError(rc, "kvqp_cache_sizes")
    return list(out)


def cache_sizes_cap(cfg: Cfg, n_cap: int, tail_cap: int):
    out = (C.c_size_t * 8)()
    rc = lib().kvqp_cache_sizes_cap(C.byref(cfg.struct()), n_cap, tail_cap, out)
    if rc:
        raise KvqpError(rc, "kvqp_cache_sizes_cap")
    return list(out)


def outlier_sizes(cfg: Cfg, n_cap: int = 0):
    out = (C.c_size_t * 4)()
    rc = lib().kvqp_outlier_sizes(C.byref(cfg.struct()), n_cap, out)
    if rc:
        raise KvqpError(rc, "kvqp_outlier_sizes")
    return list(out)


def workspace_bytes(cfg: Cfg):
    a, b = C.c_size_t(), C.c_size_t()
    rc = lib().kvqp_workspace_bytes(C.byref(cfg.struct()), C.byref(a), C.byref(b))
    if rc:
        raise KvqpError(rc, "kvqp_workspace_bytes")
    return a.value, b.value


_NAMES = ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v")


@dataclass
class Cache:
    """Device buffers of one layer's compressed cache (byte tensors) plus the ABI struct."""
    buffers: dict
    n_kept: int = 0
    tail_len: int = 0
    tail_cap: int = 0
    n_cap: int = 0      # tokens the packed buffers are laid out for; 0 = n_kept (compact)
    head_n_kept: object = None   # int32 device tensor [batch * Hkv] of a cache with head-level counts
    _keep: list = field(default_factory=list)

    def struct(self) -> CacheStruct:
        ptrs = [self.buffers[n].data_ptr() if self.buffers[n].numel() else None for n in _NAMES]
        outs = [self.buffers[n].data_ptr() if n in self.buffers and self.buffers[n].numel() else None
                for n in ("k_out", "v_out", "k_ovf", "v_ovf")]
        return CacheStruct(*ptrs, self.n_kept, self.tail_len, self.tail_cap, self.n_cap,
                           None if self.head_n_kept is None else self.head_n_kept.data_ptr(), *outs)

    def nbytes(self) -> int:
        return sum(t.numel() for t in self.buffers.values())


def alloc_cache(cfg: Cfg, tail_cap: int | None = None, device="cuda", n_cap: int = 0, ragged: bool = False) -> Cache:
    """Buffers for cfg's budget (compact) or, with n_cap, laid out for n_cap tokens per head;
    ragged adds the device array of head-level token counts."""
    import torch
    tail_cap = cfg.window if tail_cap is None else tail_cap
    sizes = cache_sizes_cap(cfg, n_cap, tail_cap) if n_cap else cache_sizes(cfg, tail_cap)
    bufs = {n: torch.empty(max(s, 0), dtype=torch.uint8, device=device) for n, s in zip(_NAMES, sizes)}
    if cfg.outlier_threshold > 0:
        for n, s in zip(("k_out", "v_out", "k_ovf", "v_ovf"), outlier_sizes(cfg, n_cap)):
            bufs[n] = torch.empty(s, dtype=torch.uint8, device=device)
    counts = torch.zeros(cfg.batch * cfg.n_kv_heads, dtype=torch.int32, device=device) if ragged else None
    return Cache(bufs, 0, 0, tail_cap, n_cap, counts)


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def alloc_workspace(nbytes: int, device="cuda"):
    import torch
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)


def decode_workspace_init(cfg: Cfg, workspace, stream=None):
    """kvqp_decode_workspace_init: zero the arrival counters at the head of a decode workspace."""
    rc = lib().kvqp_decode_workspace_init(C.byref(cfg.struct()), _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_decode_workspace_init")
    return workspace


def alloc_decode_workspace(cfg: Cfg, device="cuda", stream=None):
    """A decode workspace of kvqp_workspace_bytes' size, prepared for its first use."""
    return decode_workspace_init(cfg, alloc_workspace(workspace_bytes(cfg)[1], device), stream)


def compress(cfg: Cfg, q_obs, k, v, cache: Cache, idx_out=None, workspace=None, stream=None, unrefined_out=None):
    """kvqp_compress: q_obs [B,Hq,W,D], k/v [B,Hkv,L,D] half tensors on the device;
    unrefined_out: int32 device tensor [B*Hkv] or None."""
    if workspace is None:
        workspace = alloc_workspace(workspace_bytes(cfg)[0], k.device)
    cs = cache.struct()
    rc = lib().kvqp_compress(C.byref(cfg.struct()), _ptr(q_obs), _ptr(k), _ptr(v), C.byref(cs), _ptr(idx_out),
                             _ptr(unrefined_out), _ptr(workspace), workspace.numel(), _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_compress")
    cache.n_kept, cache.tail_len = cs.n_kept, cs.tail_len
    return cache


def compress_ragged(cfg: Cfg, q_obs, k, v, head_budget, cache: Cache, idx_out=None, workspace=None, stream=None,
                    unrefined_out=None):
    """kvqp_compress_ragged: head_budget is a host sequence of batch * Hkv token counts."""
    if workspace is None:
        workspace = alloc_workspace(workspace_bytes(cfg)[0], k.device)
    n = cfg.batch * cfg.n_kv_heads
    if len(head_budget) != n:
        raise ValueError(f"head_budget needs {n} entries")
    hb = (C.c_int32 * n)(*[int(x) for x in head_budget])
    cs = cache.struct()
    rc = lib().kvqp_compress_ragged(C.byref(cfg.struct()), _ptr(q_obs), _ptr(k), _ptr(v), hb, C.byref(cs),
                                    _ptr(idx_out), _ptr(unrefined_out), _ptr(workspace), workspace.numel(),
                                    _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_compress_ragged")
    cache.n_kept, cache.tail_len = cs.n_kept, cs.tail_len
    return cache


def quantize_selected(cfg: Cfg, k, v, idx, cache: Cache, stream=None):
    """kvqp_quantize_selected: idx int32 [B,Hkv,n_kept] ascending."""
    n_kept = int(idx.shape[-1])
    cs = cache.struct()
    rc = lib().kvqp_quantize_selected(C.byref(cfg.struct()), _ptr(k), _ptr(v), _ptr(idx) if n_kept else None, n_kept,
                                      C.byref(cs), _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_quantize_selected")
    cache.n_kept, cache.tail_len = cs.n_kept, cs.tail_len
    return cache


def quantize_selected_ragged(cfg: Cfg, k, v, idx, head_count, cache: Cache, stream=None):
    """kvqp_quantize_selected_ragged: idx int32 [B,Hkv,n_kept]; head h uses its first head_count[h] entries."""
    n_kept = int(idx.shape[-1])
    n = cfg.batch * cfg.n_kv_heads
    if len(head_count) != n:
        raise ValueError(f"head_count needs {n} entries")
    hc = (C.c_int32 * n)(*[int(x) for x in head_count])
    cs = cache.struct()
    rc = lib().kvqp_quantize_selected_ragged(C.byref(cfg.struct()), _ptr(k), _ptr(v), _ptr(idx) if n_kept else None,
                                             n_kept, hc, C.byref(cs), _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_quantize_selected_ragged")
    cache.n_kept, cache.tail_len = cs.n_kept, cs.tail_len
    return cache


def append_tail(cfg: Cfg, cache: Cache, n_tokens: int, stream=None):
    """kvqp_append_tail: the n_tokens oldest tail rows join the low-precision part."""
    cs = cache.struct()
    rc = lib().kvqp_append_tail(C.byref(cfg.struct()), C.byref(cs), n_tokens, _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_append_tail")
    cache.n_kept, cache.tail_len = cs.n_kept, cs.tail_len
    return cache


def append_tail_ragged(cfg: Cfg, cache: Cache, n_tokens: int, head_count, stream=None):
    """kvqp_append_tail_ragged: every head takes the n_tokens oldest tail rows at its own count
    (head_count: the heads' current counts, a host sequence)."""
    n = cfg.batch * cfg.n_kv_heads
    if len(head_count) != n:
        raise ValueError(f"head_count needs {n} entries")
    hc = (C.c_int32 * n)(*[int(x) for x in head_count])
    cs = cache.struct()
    rc = lib().kvqp_append_tail_ragged(C.byref(cfg.struct()), C.byref(cs), n_tokens, hc, _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_append_tail_ragged")
    cache.n_kept, cache.tail_len = cs.n_kept, cs.tail_len
    return cache


def decode_attn(cfg: Cfg, q, cache: Cache, out=None, workspace=None, stream=None):
    """kvqp_decode_attn: q [B,Hq,D] half -> out [B,Hq,D] half."""
    import torch
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = alloc_decode_workspace(cfg, q.device, stream)
    cs = cache.struct()
    rc = lib().kvqp_decode_attn(C.byref(cfg.struct()), _ptr(q), C.byref(cs), _ptr(out), _ptr(workspace),
                                workspace.numel(), _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_decode_attn")
    return out


def decode_attn_static(cfg: Cfg, q, cache: Cache, out, stream=None):
    """kvqp_decode_attn_static: the decode step on the library's own scratch array; out is the caller's."""
    cs = cache.struct()
    rc = lib().kvqp_decode_attn_static(C.byref(cfg.struct()), _ptr(q), C.byref(cs), _ptr(out), _stream_ptr(stream))
    if rc:
        raise KvqpError(rc, "kvqp_decode_attn_static")
    return out
