"""The decode call under HIP graph capture: it allocates nothing, never
synchronises and enqueues only on the caller's stream, so a serving loop can
record it once and replay it every step.  Each replay is checked against the
CPU checker and against an eager call, with eager work between the replays;
the split case also shows that the library's arrival counters are back at zero
after every replay (they are reset by the last workgroup of each head)."""
import numpy as np
import pytest
import torch

from paper_2412_12706_amd import kvqp, synth
from tests.gpu_util import dev, upload_cache

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.mark.parametrize("bits,Gq,Hkv,n_kept,splits,hint", [(4, 4, 2, 2048, 0, 0), (2, 8, 1, 1024, 3, 1), (16, 2, 4, 512, 0, 0),
                                                             (8, 4, 8, 384, 1, 2)])
def test_decode_replays_from_a_captured_graph(orc, bits, Gq, Hkv, n_kept, splits, hint):
    B, W, G = 1, 32, 32
    Hq, L = Hkv * Gq, n_kept + W + 50
    _, k, v = synth.prompt_host(B, Hq, Hkv, L, W, 128, config=800 + bits)
    rng = np.random.default_rng(800 + bits)
    idx = np.stack([np.sort(rng.choice(L - W, n_kept, replace=False)) for _ in range(B * Hkv)]).astype(np.int32).reshape(B, Hkv, n_kept)
    oc = orc.quantize_selected(k, v, idx, W=W, bits=bits, G=G)
    gc = upload_cache(oc)
    cfg = kvqp.Cfg(batch=B, n_q_heads=Hq, n_kv_heads=Hkv, seq_len=L, window=W, budget=n_kept, bits=bits, group_size=G,
                   decode_splits=splits, decode_cache_hint=hint)
    ws = kvqp.alloc_decode_workspace(cfg)
    q_in = torch.zeros(B, Hq, 128, dtype=torch.float16, device="cuda")
    out = torch.empty_like(q_in)
    kvqp.decode_attn(cfg, q_in, gc, out, ws)                  # one eager call first (the library's one-time set-up)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        kvqp.decode_attn(cfg, q_in, gc, out, ws)
    torch.cuda.synchronize()
    for step in range(4):
        q = synth.decode_query_host(B, Hq, 128, config=800 + bits, step=step)
        ref = orc.decode_attn(q, oc, cfg.sm_scale)
        q_in.copy_(dev(q))
        eager = kvqp.decode_attn(cfg, q_in, gc, workspace=ws)  # eager work between the replays
        torch.cuda.synchronize()
        out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = out.cpu().numpy().astype(np.float64)
        err = np.abs(got - ref).max()
        print(f"  bits={bits} replay {step}: max-abs error {err:.3e}", flush=True)
        assert err <= TOL
        assert np.abs(got - eager.cpu().numpy().astype(np.float64)).max() <= TOL
