"""LagKV KV-cache compression pass for MI355X (gfx950).

`paper_2504_04704_amd.lagkv` is the thin ctypes binding over the C-ABI library
built from `csrc/`; `paper_2504_04704_amd.synth` draws the seeded synthetic
caches used by tests and benchmarks.  Nothing is loaded at import time.
"""
__all__ = ["lagkv", "synth"]
