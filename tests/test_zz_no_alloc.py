"""kvqp_decode_attn_static -- the decode step for callers that cannot allocate device memory --
against kvqp_decode_attn on the same inputs (max-abs 2e-3, the decode bar; the two run the same
kernels on different scratch memory) and against the CPU checker: two calls in a row on the
library's one scratch array, the second with a smaller input, both split launches so that the
scratch (partials and arrival counters) is really used."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import dev, upload_cache

pytestmark = pytest.mark.gpu
TOL = 2e-3


def make(orc, bits, Gq, Hkv, n_kept, seed, B=1):
    W, G = 32, 32
    Hq, L = Hkv * Gq, n_kept + W + 40
    _, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=seed)
    rng = np.random.default_rng(seed)
    idx = np.stack([np.sort(rng.choice(L - W, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n_kept, bits=bits, group_size=G)
    return cfg, oc, upload_cache(oc)


def test_static_scratch_entry_matches_the_workspace_entry(orc):
    print("case static scratch: 4 bit 4 heads x 4096 tokens, then 2 bit 2 heads x 1024 tokens", flush=True)
    first = make(orc, 4, 4, 4, 4096, 951)
    second = make(orc, 2, 8, 2, 1024, 952)          # smaller: fewer heads, fewer splits, fewer partial rows
    for round_ in range(2):                          # the pair twice: the array keeps the last call's contents
        for cfg, oc, gc in (first, second):
            q = synth.decode_query_host(1, cfg.n_q_heads, 128, config=953, step=round_)
            qd = dev(q)
            ref_out = kvqp.decode_attn(cfg, qd, gc)              # the existing entry point, caller's workspace
            out = torch.full_like(qd, float("nan"))
            kvqp.decode_attn_static(cfg, qd, gc, out)            # same inputs, library's array
            torch.cuda.synchronize()
            got = out.cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(got))
            assert np.abs(got - ref_out.cpu().numpy().astype(np.float64)).max() <= TOL
            assert np.abs(got - orc.decode_attn(q, oc, cfg.sm_scale)).max() <= TOL


def test_static_scratch_entry_rejects_what_does_not_fit():
    # 128 heads of eight query heads each, cut into 64 splits by the caller: 64 MB of partials (1 KB per split and query head)
    cfg = kvqp.Cfg(batch=16, n_q_heads=64, n_kv_heads=8, seq_len=4224, window=32, budget=4096, bits=4, group_size=32, decode_splits=64)
    assert kvqp.workspace_bytes(cfg)[1] > (8 << 20)
    dummy = torch.zeros(64, dtype=torch.uint8, device="cuda")
    cache = kvqp.Cache({n: dummy for n in ("k_codes", "v_codes", "k_scale", "k_zero", "v_scale", "v_zero", "tail_k", "tail_v")},
                       n_kept=4096, tail_len=32, tail_cap=32)
    with pytest.raises(kvqp.KvqpError) as e:
        kvqp.decode_attn_static(cfg, dummy, cache, dummy)        # rejected on the host: nothing is launched
    assert e.value.code == -3
