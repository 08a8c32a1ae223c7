"""Seeded synthetic KV caches shaped like the paper's long-context workloads.

This module only draws random numbers and scales them; it contains none of
the LagKV arithmetic (no min/max normalisation, spread, softmax, selection or
compaction) so that both the CPU oracle tests and the HIP path can be fed the
same bytes without sharing any of the method's code.

Recipe (stands in for the RULER / LongBench / passkey caches of Llama-3.1-8B
used in the paper's Comparisons and Ablations sections, whose prompts and
weights are not available): keys are Gaussian with a per-channel scale (keys
are known to have channel-wise structure, Introduction, paragraph on KV
statistics) plus a few strong outlier channels; values are Gaussian with a
per-token scale (values vary along the sequence).

    K[l,b,h,t,c] = N(0,1) * sK[l,h,c] * (10 if c in outliers[l,h] else 1)
    V[l,b,h,t,c] = N(0,1) * sV[l,b,h,t]
    sK ~ LogNormal(0, 0.5)      sV ~ LogNormal(0, 0.3)

Layers are folded into the leading (batch) axis: the returned tensors are
[layers*B, H, T, D] with D contiguous.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

import torch

MASTER_SEED = 20250404


@dataclass(frozen=True)
class KVConfig:
    name: str
    layers: int
    B: int
    H: int
    D: int
    T: int
    S: int
    L: int
    r: float
    dtype: str              # "f32" | "bf16"
    n_outlier: int = 0      # outlier key channels per head (scaled x10)
    outlier_per_layer: bool = False  # redraw outlier positions for every layer
    k_sigma: float = 0.5    # sigma of the log-normal per-channel key scale
    v_sigma: float = 0.3    # sigma of the log-normal per-token value scale

    @property
    def streams(self) -> int:
        return self.layers * self.B * self.H

    @property
    def torch_dtype(self) -> torch.dtype:
        return {"f32": torch.float32, "bf16": torch.bfloat16}[self.dtype]

    def scaled(self, **kw) -> "KVConfig":
        return replace(self, **kw)


# The five workload configurations (tiny fp32, Llama-3-8B-shaped bf16 at 16K,
# 64K and 128K context, and the decode-time starting cache).
CONFIGS = {
    "cfg1_tiny_f32": KVConfig("cfg1_tiny_f32", layers=1, B=1, H=2, D=64, T=1024,
                              S=16, L=128, r=0.5, dtype="f32"),
    "cfg2_llama8b_16k": KVConfig("cfg2_llama8b_16k", layers=32, B=1, H=8, D=128, T=16384,
                                 S=16, L=128, r=0.25, dtype="bf16", n_outlier=4),
    "cfg3_llama8b_64k": KVConfig("cfg3_llama8b_64k", layers=32, B=1, H=8, D=128, T=65536,
                                 S=16, L=256, r=0.125, dtype="bf16", n_outlier=4,
                                 outlier_per_layer=True),
    "cfg4_llama8b_128k_b4": KVConfig("cfg4_llama8b_128k_b4", layers=32, B=4, H=8, D=128,
                                     T=131072, S=16, L=512, r=0.25, dtype="bf16",
                                     n_outlier=4),
    "cfg5_decode_b32": KVConfig("cfg5_decode_b32", layers=32, B=32, H=8, D=128, T=32768,
                                S=16, L=128, r=0.25, dtype="bf16", n_outlier=4),
}


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def _sub_seed(seed: int, *tags: int) -> int:
    """Deterministic sub-seed from a master seed and integer tags (splitmix-style)."""
    x = (int(seed) + 0x9E3779B97F4A7C15) & 0xFFFFFFFFFFFFFFFF
    for t in tags:
        x ^= (int(t) + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2)) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def outlier_channels(cfg: KVConfig, seed: int, layer: int) -> torch.Tensor:
    """[H, n_outlier] int64 channel positions (CPU); shared by all layers unless
    cfg.outlier_per_layer."""
    tag = layer if cfg.outlier_per_layer else 0
    g = _gen("cpu", _sub_seed(seed, 101, tag))
    rows = [torch.randperm(cfg.D, generator=g)[: cfg.n_outlier] for _ in range(cfg.H)]
    return torch.stack(rows) if cfg.n_outlier > 0 else torch.zeros(cfg.H, 0, dtype=torch.int64)


def key_channel_scale(cfg: KVConfig, seed: int, layer: int, device) -> torch.Tensor:
    """[H, D] fp32 per-channel key scale, outlier channels included."""
    g = _gen("cpu", _sub_seed(seed, 202, layer))
    s = torch.exp(cfg.k_sigma * torch.randn(cfg.H, cfg.D, generator=g, dtype=torch.float32))
    if cfg.n_outlier > 0:
        oc = outlier_channels(cfg, seed, layer)
        s.scatter_(1, oc, s.gather(1, oc) * 10.0)
    return s.to(device)


def fill_layer(cfg: KVConfig, seed: int, layer: int, K_out: torch.Tensor, V_out: torch.Tensor,
               t0: int = 0, T: Optional[int] = None) -> None:
    """Write tokens [t0, t0+T) of one layer into K_out, V_out ([B, H, T, D] views).

    Tokens are drawn in blocks so that a slice [t0, t0+T) is reproducible only
    for identical (t0, T) calls; callers that need the same cache twice call
    with the same arguments.
    """
    device = K_out.device
    T = cfg.T if T is None else T
    sK = key_channel_scale(cfg, seed, layer, device)            # [H, D]
    gk = _gen(device, _sub_seed(seed, 303, layer, t0))
    gv = _gen(device, _sub_seed(seed, 404, layer, t0))
    gs = _gen(device, _sub_seed(seed, 505, layer, t0))
    # generate per batch entry to bound the fp32 temporaries at large T
    for b in range(cfg.B):
        k = torch.randn(cfg.H, T, cfg.D, generator=gk, device=device, dtype=torch.float32)
        k.mul_(sK[:, None, :])
        K_out[b].copy_(k)
        del k
        v = torch.randn(cfg.H, T, cfg.D, generator=gv, device=device, dtype=torch.float32)
        sV = torch.exp(cfg.v_sigma * torch.randn(cfg.H, T, 1, generator=gs, device=device,
                                                 dtype=torch.float32))
        v.mul_(sV)
        V_out[b].copy_(v)
        del v, sV


def make_kv(cfg: KVConfig, device="cpu", seed: int = MASTER_SEED,
            layers: Optional[int] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Full cache for `cfg`: K, V of shape [layers*B, H, T, D] in cfg's dtype."""
    nl = cfg.layers if layers is None else layers
    shape = (nl * cfg.B, cfg.H, cfg.T, cfg.D)
    K = torch.empty(shape, dtype=cfg.torch_dtype, device=device)
    V = torch.empty(shape, dtype=cfg.torch_dtype, device=device)
    for l in range(nl):
        fill_layer(cfg, seed, l, K[l * cfg.B:(l + 1) * cfg.B], V[l * cfg.B:(l + 1) * cfg.B])
    return K, V


def make_new_tokens(cfg: KVConfig, n_new: int, round_idx: int, device="cpu",
                    seed: int = MASTER_SEED, layers: Optional[int] = None
                    ) -> Tuple[torch.Tensor, torch.Tensor]:
    """[layers*B, H, n_new, D] tokens to append at decode round `round_idx`, same
    distributions as the cache itself."""
    nl = cfg.layers if layers is None else layers
    shape = (nl * cfg.B, cfg.H, n_new, cfg.D)
    K = torch.empty(shape, dtype=cfg.torch_dtype, device=device)
    V = torch.empty(shape, dtype=cfg.torch_dtype, device=device)
    for l in range(nl):
        fill_layer(cfg, seed, l, K[l * cfg.B:(l + 1) * cfg.B], V[l * cfg.B:(l + 1) * cfg.B],
                   t0=cfg.T + round_idx * n_new, T=n_new)
    return K, V


def stream_sample(n_streams: int, n_sample: int, seed: int = MASTER_SEED) -> list:
    """Seeded sample of stream ids that always contains the first and the last stream."""
    if n_sample >= n_streams:
        return list(range(n_streams))
    g = _gen("cpu", _sub_seed(seed, 606, n_streams))
    perm = torch.randperm(n_streams, generator=g).tolist()
    picked = [0, n_streams - 1]
    for s in perm:
        if len(picked) >= n_sample:
            break
        if s not in picked:
            picked.append(s)
    return sorted(picked)
