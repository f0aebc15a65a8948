"""GPU parity of the quantize-and-pack step against the CPU checker: every
code word, scale, zero and tail row must match bit for bit (paper Section 3,
"KV Quantization"; grouping axes of Section 6.3)."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import assert_cache_equal, dev

pytestmark = pytest.mark.gpu

CASES = [
    # bits, G, axis, n_kept, L, W, B, Hkv
    (4, 32, 0, 1024, 1200, 32, 1, 2),
    (4, 32, 0, 96, 300, 32, 2, 2),       # ragged: 96 = one and a half 64-token chunks
    (2, 32, 0, 160, 400, 32, 1, 2),      # 2-bit: last 64-token value superblock half empty
    (2, 64, 0, 256, 400, 64, 1, 2),
    (2, 128, 0, 256, 400, 8, 1, 1),
    (8, 32, 0, 224, 400, 32, 1, 2),
    (8, 64, 1, 192, 400, 32, 1, 2),
    (4, 32, 1, 160, 400, 32, 1, 2),
    (4, 64, 0, 320, 500, 32, 1, 1),
    (4, 128, 0, 384, 500, 32, 1, 2),
    (4, 128, 1, 96, 500, 32, 1, 2),
    (16, 32, 0, 160, 300, 32, 1, 2),
    (4, 32, 0, 0, 100, 32, 1, 2),        # nothing kept: tail only
]


@pytest.mark.parametrize("bits,G,axis,n_kept,L,W,B,Hkv", CASES)
def test_quantize_selected_bit_exact(orc, bits, G, axis, n_kept, L, W, B, Hkv):
    print(f"case bits={bits} G={G} axis={axis} n_kept={n_kept} L={L} W={W} B={B} Hkv={Hkv}", flush=True)
    _, k, v = synth.prompt_host(B, Hkv * 4, Hkv, L, W, 128, config=60 + bits)
    rng = np.random.default_rng(bits * 1000 + G + n_kept)
    idx = np.stack([np.sort(rng.choice(L - W, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G, key_axis=axis, tail_cap=W + 8)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hkv * 4, n_kv_heads=Hkv, seq_len=L, window=W, budget=n_kept, bits=bits,
                   group_size=G, key_axis=axis)
    gc = kvqp.alloc_cache(cfg, tail_cap=W + 8)
    for t in gc.buffers.values():
        t.fill_(0xA5)                    # stale bytes must all be overwritten
    kvqp.quantize_selected(cfg, dev(k), dev(v), dev(idx), gc)
    torch.cuda.synchronize()
    assert_cache_equal(gc, oc)


def test_quantizer_edge_values_bit_exact(orc):
    """Constant groups, tiny ranges (scale rounds to a subnormal or to zero),
    signed zeros and large magnitudes go through the same binary32 sequence."""
    B, Hkv, L, W, n_kept = 1, 1, 160, 32, 128
    rng = np.random.default_rng(5)
    k = rng.standard_normal((B, Hkv, L, 128)).astype(np.float16)
    v = rng.standard_normal((B, Hkv, L, 128)).astype(np.float16)
    k[..., 0] = np.float16(1.25)                                   # constant column
    k[..., 1] = (1.0 + rng.integers(0, 2, (B, Hkv, L)) * 2.0**-10).astype(np.float16)   # one-ulp range
    k[..., 2] = (rng.integers(-3, 4, (B, Hkv, L)) * 2.0**-24).astype(np.float16)        # subnormals
    k[..., 3] = np.where(rng.random((B, Hkv, L)) < 0.5, np.float16(0.0), np.float16(-0.0))
    k[..., 4] = (rng.standard_normal((B, Hkv, L)) * 20000).astype(np.float16)
    v[:, :, :, :32] = np.float16(-7.0)
    v[:, :, :, 32:64] = (rng.integers(0, 3, (B, Hkv, L, 32)) * 2.0**-20).astype(np.float16)
    idx = np.arange(n_kept, dtype=np.int32).reshape(1, 1, n_kept)
    for bits in (2, 4, 8):
        oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=32, key_axis=0)
        cfg = kvqp.Cfg(batch=B, n_q_heads=4, n_kv_heads=Hkv, seq_len=L, window=W, budget=n_kept, bits=bits, group_size=32)
        gc = kvqp.alloc_cache(cfg)
        kvqp.quantize_selected(cfg, dev(k), dev(v), dev(idx), gc)
        torch.cuda.synchronize()
        assert_cache_equal(gc, oc)
