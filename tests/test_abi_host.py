"""Host-side checks of the C ABI that need no GPU: the library loads, exports
every symbol include/kvqp.h declares, answers its size queries, and rejects bad
arguments before anything could be launched."""
import ctypes as C
import os
import re

import pytest

from paper_2412_12706_amd import kvqp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kvqp.LIB_PATH):
        from paper_2412_12706_amd import build
        build.build()
    return kvqp.lib()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "kvqp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvqp_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) == set(kvqp.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 on its own, with no C++ or HIP types."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = tmp_path / "t.c"
    src.write_text('#include "kvqp.h"\nint main(void) { kvqp_cfg c; kvqp_cache k; (void)c; (void)k; return KVQP_OK; }\n')
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr


def test_version_and_strerror(lib):
    assert kvqp.version() >= 100
    assert kvqp.strerror(0) == "ok"
    for code in (-1, -2, -3, -4):
        assert kvqp.strerror(code) and kvqp.strerror(code) != kvqp.strerror(0)
    assert "unknown" in kvqp.strerror(-99)


def bpt(bits, G):
    return 512 if bits == 16 else 2 * (128 * bits // 8 + 4 * 128 // G)


@pytest.mark.parametrize("bits,G", [(2, 32), (2, 64), (4, 32), (4, 128), (8, 32), (16, 32)])
def test_cache_sizes_match_bytes_per_token(lib, bits, G):
    cfg = kvqp.Cfg(batch=3, n_q_heads=32, n_kv_heads=8, seq_len=4096 + 32, window=32, budget=1024, bits=bits, group_size=G)
    sizes = kvqp.cache_sizes(cfg, tail_cap=40)
    heads = 3 * 8
    assert sum(sizes[:6]) == heads * 1024 * bpt(bits, G)
    assert sizes[6] == sizes[7] == heads * 40 * 128 * 2
    # 2-bit value codes are padded to 64-token superblocks
    cfg2 = kvqp.Cfg(batch=1, n_q_heads=8, n_kv_heads=2, seq_len=1000, window=32, budget=96, bits=2, group_size=32)
    s2 = kvqp.cache_sizes(cfg2, 32)
    assert s2[0] == 2 * 96 * 128 * 2 // 8 and s2[1] == 2 * 128 * 128 * 2 // 8


def test_workspace_sizes_are_positive_and_compress_grows_with_the_problem(lib):
    small = kvqp.Cfg(batch=1, n_q_heads=32, n_kv_heads=8, seq_len=4096, window=32, budget=1024)
    big = kvqp.Cfg(batch=32, n_q_heads=32, n_kv_heads=8, seq_len=32768, window=32, budget=8192)
    (c0, d0), (c1, d1) = kvqp.workspace_bytes(small), kvqp.workspace_bytes(big)
    assert 0 < c0 < c1 and d0 > 0 and d1 > 0     # (decode: partials of the token-axis splits, few heads -> more splits)


BAD = [
    (dict(bits=3), -1), (dict(bits=0), -1), (dict(group_size=48), -1), (dict(group_size=16), -2),
    (dict(head_dim=64), -2), (dict(n_q_heads=30), -1), (dict(n_q_heads=8 * 16), -2), (dict(pool_kernel=4), -1),
    (dict(pool_kernel=0), -1), (dict(window=0), -1), (dict(window=5000), -1), (dict(budget=-1), -1),
    (dict(outlier_overflow_cap=-1), -1),
    (dict(key_axis=2), -1), (dict(batch=0), -1), (dict(window=128), -2), (dict(decode_splits=-1), -1),
    (dict(sm_scale=float("nan")), -1), (dict(decode_cache_hint=3), -1), (dict(decode_cache_hint=-1), -1),
]


@pytest.mark.parametrize("patch,code", BAD)
def test_invalid_configurations_are_rejected_on_the_host(lib, patch, code):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=4096, window=32, pool_kernel=7, budget=1024,
                bits=4, group_size=32, key_axis=0, decode_splits=0, sm_scale=0.088)
    base.update(patch)
    cfg = kvqp.Cfg(**base)
    sizes = (C.c_size_t * 8)()
    assert lib.kvqp_cache_sizes(C.byref(cfg.struct()), max(cfg.window, 1), sizes) == code


def test_entry_points_reject_null_pointers_without_touching_the_device(lib):
    cfg = kvqp.Cfg(batch=1, n_q_heads=32, n_kv_heads=8, seq_len=4096, window=32, budget=1024)
    cs = kvqp.CacheStruct()
    st = cfg.struct()
    assert lib.kvqp_compress(C.byref(st), None, None, None, C.byref(cs), None, None, None, 0, None) == -1
    assert lib.kvqp_compress(None, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.kvqp_quantize_selected(C.byref(st), None, None, None, 1024, C.byref(cs), None) == -1
    assert lib.kvqp_decode_attn(C.byref(st), None, C.byref(cs), None, None, 0, None) == -1
    # plausible non-null data pointers but cache buffers missing
    fake = C.c_void_p(0x1000)
    cs.tail_cap = 32
    assert lib.kvqp_compress(C.byref(st), fake, fake, fake, C.byref(cs), None, None, None, 0, None) == -1
    # complete pointers, workspace missing -> workspace error, still nothing launched
    for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v"):
        setattr(cs, name, 0x1000)
    assert lib.kvqp_compress(C.byref(st), fake, fake, fake, C.byref(cs), None, None, None, 0, None) == -3
    cs.n_kept, cs.tail_len = 1024, 32
    assert lib.kvqp_decode_attn(C.byref(st), fake, C.byref(cs), fake, None, 0, None) == -3
    assert lib.kvqp_decode_attn(C.byref(st), fake, C.byref(cs), fake, fake, 16, None) == -3
    cs.tail_len = 64                      # beyond tail_cap
    assert lib.kvqp_decode_attn(C.byref(st), fake, C.byref(cs), fake, fake, 1 << 30, None) == -1
    cs.n_kept, cs.tail_len = 0, 0         # empty cache
    assert lib.kvqp_decode_attn(C.byref(st), fake, C.byref(cs), fake, fake, 1 << 30, None) == -1


def test_capacity_sizes_and_append_argument_checks(lib):
    """Buffers laid out for n_cap tokens are sized like a compact cache of n_cap
    tokens; kvqp_append_tail validates counts on the host before any launch."""
    cfg = kvqp.Cfg(batch=2, n_q_heads=32, n_kv_heads=8, seq_len=4096, window=32, budget=1024, bits=4, group_size=32)
    compact = kvqp.cache_sizes(cfg, 40)
    same = kvqp.cache_sizes_cap(cfg, 1024, 40)
    assert compact == same
    big = kvqp.cache_sizes_cap(cfg, 2048, 40)
    assert all(b == 2 * a for a, b in zip(compact[:6], big[:6])) and big[6:] == compact[6:]
    for bad in (1000, 1040, -64):         # not a multiple of 64 / negative
        with pytest.raises(kvqp.KvqpError):
            kvqp.cache_sizes_cap(cfg, bad, 40)
    st = cfg.struct()
    cs = kvqp.CacheStruct()
    for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v"):
        setattr(cs, name, 0x1000)
    cs.n_kept, cs.tail_len, cs.tail_cap, cs.n_cap = 1024, 64, 96, 1088
    assert lib.kvqp_append_tail(None, C.byref(cs), 32, None) == -1
    assert lib.kvqp_append_tail(C.byref(st), None, 32, None) == -1
    assert lib.kvqp_append_tail(C.byref(st), C.byref(cs), 0, None) == -1       # nothing to move
    assert lib.kvqp_append_tail(C.byref(st), C.byref(cs), 48, None) == -1      # not whole groups
    assert lib.kvqp_append_tail(C.byref(st), C.byref(cs), 96, None) == -1      # more than the tail holds
    cs.tail_len = 96
    assert lib.kvqp_append_tail(C.byref(st), C.byref(cs), 96, None) == -1      # beyond the capacity
    cs.n_cap = 1000
    assert lib.kvqp_append_tail(C.byref(st), C.byref(cs), 32, None) == -1      # capacity below n_kept / misaligned
    assert (cs.n_kept, cs.tail_len) == (1024, 96)                               # untouched by rejected calls


def test_head_level_count_argument_checks(lib):
    """kvqp_compress_ragged validates every head's count on the host before anything is enqueued;
    the calls that do not take head-level counts say so."""
    cfg = kvqp.Cfg(batch=1, n_q_heads=8, n_kv_heads=2, seq_len=800, window=32, budget=256, bits=4, group_size=64)
    st = cfg.struct()
    cs = kvqp.CacheStruct()
    for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v", "head_n_kept"):
        setattr(cs, name, 0x1000)
    cs.tail_cap = 32
    fake = C.c_void_p(0x1000)
    call = lambda counts, cache=cs: lib.kvqp_compress_ragged(C.byref(st), fake, fake, fake, (C.c_int32 * 2)(*counts),
                                                             C.byref(cache), None, None, fake, 1 << 30, None)
    assert lib.kvqp_compress_ragged(C.byref(st), fake, fake, fake, (C.c_int32 * 2)(256, 97), C.byref(cs), None, None, fake,
                                    16, None) == -3      # any count under the bound is fine: the call gets as far as the workspace check
    assert call([256, 320]) == -1         # above the bound is not
    assert call([-64, 64]) == -1
    assert lib.kvqp_compress_ragged(C.byref(st), fake, fake, fake, None, C.byref(cs), None, None, fake, 1 << 30, None) == -1
    no_counts = kvqp.CacheStruct.from_buffer_copy(cs)
    no_counts.head_n_kept = None
    assert call([256, 64], no_counts) == -1
    assert lib.kvqp_compress_ragged(C.byref(st), fake, fake, fake, (C.c_int32 * 2)(256, 64), C.byref(cs), None, None, fake,
                                    16, None) == -3      # counts fine, workspace too small: still nothing launched
    assert lib.kvqp_quantize_selected_ragged(C.byref(st), fake, fake, fake, 256, (C.c_int32 * 2)(256, 257), C.byref(cs),
                                             None) == -1      # above the bound
    assert lib.kvqp_quantize_selected_ragged(C.byref(st), fake, fake, fake, 256, None, C.byref(cs), None) == -1
    assert lib.kvqp_quantize_selected(C.byref(st), fake, fake, fake, 256, C.byref(cs), None) == -1
    # uniform calls refuse a cache that carries head-level counts
    assert lib.kvqp_compress(C.byref(st), fake, fake, fake, C.byref(cs), None, None, fake, 1 << 30, None) == -1
    cs.n_kept, cs.tail_len, cs.n_cap = 256, 32, 320
    assert lib.kvqp_append_tail(C.byref(st), C.byref(cs), 64, None) == -2
    # the head-level form checks the heads' current counts before anything is enqueued
    app = lambda counts, n=64, cache=cs: lib.kvqp_append_tail_ragged(C.byref(st), C.byref(cache), n,
                                                                      (C.c_int32 * 2)(*counts) if counts else None, None)
    cs.tail_len = 64
    assert app(None) == -1
    assert app([256, 96]) == -1           # appending wants whole key groups under the new rows
    assert app([256, 320]) == -1          # above the bound n_kept
    assert app([-64, 64]) == -1
    assert app([256, 64], 32) == -1       # n_tokens not whole groups
    assert app([256, 64], 128) == -1      # more than the tail holds (and than the capacity)
    no_counts = kvqp.CacheStruct.from_buffer_copy(cs)
    no_counts.head_n_kept = None
    assert app([256, 64], 64, no_counts) == -1
    assert (cs.n_kept, cs.tail_len) == (256, 64)
    cs.tail_len = 0
    assert lib.kvqp_decode_attn(C.byref(st), fake, C.byref(cs), fake, fake, 1 << 30, None) == -1   # a head may be empty


def test_outlier_filtering_argument_checks(lib):
    """Slot buffer sizes and the host-side rejects of the outlier-filtering mode."""
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, seq_len=800, window=32, budget=256, bits=4, group_size=32)
    on = kvqp.Cfg(**base, outlier_threshold=6.0)
    assert kvqp.outlier_sizes(on)[:2] == [2 * 2 * 256 * 4 * 4] * 2          # heads x tokens x 4 slots x 4 bytes
    assert kvqp.outlier_sizes(on, 320)[:2] == [2 * 2 * 320 * 4 * 4] * 2
    assert kvqp.outlier_sizes(on)[2:] == [2 * 2 * 12 * 4] * 2               # no list entries asked for: the prefix counts (9, padded to 12) alone
    assert kvqp.outlier_sizes(kvqp.Cfg(**{**on.__dict__, 'outlier_overflow_cap': 100}), 320)[2:] == [2 * 2 * (12 + 200) * 4] * 2
    assert kvqp.outlier_sizes(kvqp.Cfg(**base)) == [0, 0, 0, 0]
    for bad in (-1.0, float("nan"), float("inf")):
        with pytest.raises(kvqp.KvqpError):
            kvqp.outlier_sizes(kvqp.Cfg(**base, outlier_threshold=bad))
    with pytest.raises(kvqp.KvqpError):                                      # nothing is quantized at 16 bits
        kvqp.cache_sizes(kvqp.Cfg(**{**base, "bits": 16}, outlier_threshold=6.0), 32)
    st = on.struct()
    cs = kvqp.CacheStruct()
    for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v"):
        setattr(cs, name, 0x1000)
    cs.tail_cap = 32
    fake = C.c_void_p(0x1000)
    assert lib.kvqp_compress(C.byref(st), fake, fake, fake, C.byref(cs), None, None, fake, 1 << 30, None) == -1   # no slot buffers
    cs.n_kept, cs.tail_len = 256, 32
    assert lib.kvqp_decode_attn(C.byref(st), fake, C.byref(cs), fake, fake, 1 << 30, None) == -1


def test_decode_workspace_covers_every_token_count(lib):
    """The decode workspace size does not depend on the token count, so a cache grown by appended
    tokens never outgrows it."""
    for heads, bits in ((8, 4), (8, 2), (256, 4), (2, 16)):
        sizes = set()
        for budget in (64, 1024, 8192, 32768):
            cfg = kvqp.Cfg(batch=heads // 2, n_q_heads=8, n_kv_heads=2, seq_len=40000, window=32, budget=budget, bits=bits,
                           group_size=32)
            sizes.add(kvqp.workspace_bytes(cfg)[1])
        assert len(sizes) == 1 and min(sizes) > 0, (heads, bits, sizes)
    a = kvqp.workspace_bytes(kvqp.Cfg(batch=1, n_q_heads=8, n_kv_heads=2, seq_len=4096, window=32, budget=1024, bits=4))[1]
    b = kvqp.workspace_bytes(kvqp.Cfg(batch=1, n_q_heads=8, n_kv_heads=2, seq_len=4096, window=32, budget=1024, bits=4,
                                      decode_splits=500))[1]
    assert b >= 2 * 500 * 4 * 256 * 4 and b > a      # the caller's split count is covered


def test_binding_raises_with_the_library_message(lib):
    cfg = kvqp.Cfg(batch=1, n_q_heads=32, n_kv_heads=8, seq_len=4096, window=32, budget=1024, bits=5)
    with pytest.raises(kvqp.KvqpError) as e:
        kvqp.cache_sizes(cfg, 32)
    assert "invalid argument" in str(e.value)


def test_product_package_does_not_import_the_checker():
    for root, _, files in os.walk(os.path.join(ROOT, "paper_2412_12706_amd")):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(root, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the checker"


def test_decode_workspace_init_and_static_entry_validate_on_the_host(lib):
    """The two decode-side additions reject bad calls before anything is enqueued (no GPU needed):
    the workspace preparation wants a workspace that holds the arrival counters, and the entry
    point on the library's own scratch array refuses launches whose partials do not fit it."""
    cfg = kvqp.Cfg(batch=4, n_q_heads=32, n_kv_heads=8, seq_len=4096, window=32, budget=1024, bits=4)
    st = cfg.struct()
    fake = C.c_void_p(0x1000)
    assert lib.kvqp_decode_workspace_init(None, fake, 1 << 20, None) == -1
    assert lib.kvqp_decode_workspace_init(C.byref(st), None, 1 << 20, None) == -3
    assert lib.kvqp_decode_workspace_init(C.byref(st), fake, 64, None) == -3            # 32 counters need 128 bytes
    assert lib.kvqp_decode_workspace_init(C.byref(st), C.c_void_p(0x1004), 1 << 20, None) == -1
    assert kvqp.workspace_bytes(cfg)[1] >= 256 + 32 * 4 * 256 * 4                         # counters, then partials
    cs = kvqp.CacheStruct()
    for name in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v"):
        setattr(cs, name, 0x1000)
    cs.n_kept, cs.tail_len, cs.tail_cap = 1024, 32, 32
    assert lib.kvqp_decode_attn_static(C.byref(st), None, C.byref(cs), fake, None) == -1
    assert lib.kvqp_decode_attn_static(C.byref(st), fake, None, fake, None) == -1
    # 128 heads cut into 16 splits by the caller: 16 MB of partials, beyond the library's array
    big = kvqp.Cfg(batch=16, n_q_heads=64, n_kv_heads=8, seq_len=4096, window=32, budget=1024, bits=4, decode_splits=16)
    assert kvqp.workspace_bytes(big)[1] > (8 << 20)
    assert lib.kvqp_decode_attn_static(C.byref(big.struct()), fake, C.byref(cs), fake, None) == -3
