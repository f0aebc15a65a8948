"""MI355X-native quantized-pruned KV cache (arXiv 2412.12706, Section 3).

`paper_2412_12706_amd.kvqp` is the thin ctypes binding of the C-ABI library
(kvqp_compress, kvqp_decode_attn); `paper_2412_12706_amd.synth` holds the
seeded synthetic input generators.  Importing the package loads nothing.
"""
__all__ = ["kvqp", "synth"]
