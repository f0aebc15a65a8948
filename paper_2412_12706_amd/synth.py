"""Seeded synthetic inputs shaped like the paper's workloads.

The paper evaluates on long prompts run through Llama/Mistral checkpoints
(Section 4, Appendix A); neither the prompts nor the weights exist here, so
the tests and the benchmark use tensors with the same shapes and the one
structural property the paper's quantization study leans on: a few key
channels carry outliers, which is why keys are quantized per channel
(Section 2 "KV Quantization", Section 6.3).

This module contains no arithmetic of the method itself.  Both the HIP path
and the CPU checker receive the bytes produced here.

Recipe: every element i.i.d. N(0,1) drawn in float32 and rounded to float16;
keys are then multiplied by `outlier` (10, or 20 for the 128k configuration)
on four fixed channels per KV head, ch_i = (7 + 29*g + 37*i) mod D.
Streams are keyed by (config, layer, tensor, step) under one base seed.
"""
from __future__ import annotations

import numpy as np

BASE_SEED = 241212706
TENSOR_IDS = {"q_obs": 0, "k": 1, "v": 2, "q_dec": 3}


def outlier_channels(g: int, D: int = 128):
    return [(7 + 29 * g + 37 * i) % D for i in range(4)]


def stream_seed(config: int, layer: int, tensor: str, step: int = 0) -> int:
    return (BASE_SEED * 1000003 + config * 7919 + layer * 104729 + TENSOR_IDS[tensor] * 15485863 + step) % (2**63 - 1)


def _normal_f16(shape, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    return rng.standard_normal(shape, dtype=np.float32).astype(np.float16)


def prompt_host(B, Hq, Hkv, L, W, D=128, outlier=10.0, config=0, layer=0):
    """(q_obs [B,Hq,W,D], k [B,Hkv,L,D], v [B,Hkv,L,D]) as numpy float16."""
    q_obs = _normal_f16((B, Hq, W, D), stream_seed(config, layer, "q_obs"))
    k = _normal_f16((B, Hkv, L, D), stream_seed(config, layer, "k"))
    v = _normal_f16((B, Hkv, L, D), stream_seed(config, layer, "v"))
    for g in range(Hkv):
        ch = outlier_channels(g, D)
        k[:, g, :, ch] = (k[:, g, :, ch].astype(np.float32) * np.float32(outlier)).astype(np.float16)
    return q_obs, k, v


def decode_query_host(B, Hq, D=128, config=0, layer=0, step=0):
    return _normal_f16((B, Hq, D), stream_seed(config, layer, "q_dec", step))


def prompt_device(B, Hq, Hkv, L, W, D=128, outlier=10.0, config=0, layer=0, device="cuda"):
    """Same recipe drawn on the device with torch's generator (large shapes).
    The CPU checker is given copies of these exact bytes, never a re-draw."""
    import torch

    def draw(shape, name):
        gen = torch.Generator(device=device)
        gen.manual_seed(stream_seed(config, layer, name))
        return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(torch.float16)

    q_obs = draw((B, Hq, W, D), "q_obs")
    k = draw((B, Hkv, L, D), "k")
    v = draw((B, Hkv, L, D), "v")
    for g in range(Hkv):
        ch = outlier_channels(g, D)
        k[:, g, :, ch] = (k[:, g, :, ch].float() * outlier).to(torch.float16)
    return q_obs, k, v


def decode_query_device(B, Hq, D=128, config=0, layer=0, step=0, device="cuda"):
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(stream_seed(config, layer, "q_dec", step))
    return torch.randn((B, Hq, D), generator=gen, device=device, dtype=torch.float32).to(torch.float16)
