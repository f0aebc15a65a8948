"""Two decode calls in flight at once (Section 3, Eq. (3), evaluated in token ranges whose partial
results meet in the call's workspace): calls with workspaces of their own share nothing, so they
may run on different streams at the same time.  Both are split launches (few heads, many tokens),
issued alternately on two streams many times over, and every output is checked against the CPU
checker."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import dev, upload_cache

pytestmark = pytest.mark.gpu
TOL = 2e-3


def make(orc, bits, Gq, Hkv, n_kept, seed):
    B, W, G = 1, 32, 32
    Hq, L = Hkv * Gq, n_kept + W + 40
    _, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=seed)
    rng = np.random.default_rng(seed)
    idx = np.stack([np.sort(rng.choice(L - W, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n_kept, bits=bits, group_size=G)
    return cfg, oc, upload_cache(oc)


def test_calls_with_their_own_workspaces_overlap_on_two_streams(orc):
    print("case two streams, two workspaces", flush=True)
    jobs = [make(orc, 4, 4, 2, 4096, 901), make(orc, 2, 4, 2, 3072, 902)]     # same head indices in both: one shared counter array would collide
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ws = [kvqp.alloc_decode_workspace(cfg) for cfg, _, _ in jobs]
    torch.cuda.synchronize()
    steps = 24
    qs = [[synth.decode_query_host(1, cfg.n_q_heads, 128, config=900 + j, step=s) for s in range(steps)] for j, (cfg, _, _) in enumerate(jobs)]
    qd = [[dev(q) for q in row] for row in qs]
    outs = [[torch.empty_like(qd[j][s]) for s in range(steps)] for j in range(2)]
    torch.cuda.synchronize()
    for s in range(steps):
        for j, (cfg, _, gc) in enumerate(jobs):
            kvqp.decode_attn(cfg, qd[j][s], gc, outs[j][s], ws[j], stream=streams[j])
    torch.cuda.synchronize()
    worst = 0.0
    for j, (cfg, oc, _) in enumerate(jobs):
        for s in range(steps):
            ref = orc.decode_attn(qs[j][s], oc, cfg.sm_scale)
            got = outs[j][s].cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(got))
            worst = max(worst, np.abs(got - ref).max())
    print(f"  max-abs error over {2 * steps} overlapping calls {worst:.3e}", flush=True)
    assert worst <= TOL
    # the counters at the head of both workspaces are back at zero
    for j, (cfg, _, _) in enumerate(jobs):
        assert int(ws[j][: 4 * cfg.batch * cfg.n_kv_heads].view(torch.int32).abs().sum().item()) == 0


def test_workspace_of_a_larger_batch_serves_a_smaller_one(orc):
    print("case workspace reuse across head counts", flush=True)
    big = make(orc, 4, 4, 4, 2048, 903)
    small = make(orc, 8, 2, 1, 1024, 904)
    ws = kvqp.alloc_decode_workspace(big[0])
    for cfg, oc, gc in (big, small, big):
        assert kvqp.workspace_bytes(cfg)[1] <= ws.numel()
        q = synth.decode_query_host(1, cfg.n_q_heads, 128, config=905, step=0)
        out = kvqp.decode_attn(cfg, dev(q), gc, workspace=ws)
        torch.cuda.synchronize()
        assert np.abs(out.cpu().numpy().astype(np.float64) - orc.decode_attn(q, oc, cfg.sm_scale)).max() <= TOL
