"""Comparison of the HIP path with the CPU oracle, stream by stream.

Bar (stated here, used by every GPU test):
  * fp32 scores within 1e-5 relative of the fp64 oracle;
  * kept positions and kept K/V rows bit-exact, except in chunks where the two
    selections differ only by tokens whose oracle score lies within 1e-5
    relative of the oracle's k-th score (near-ties; counted and reported);
  * the selection is also checked in the kernel's own precision: the oracle's
    top-k applied to the GPU's fp32 scores must reproduce the GPU's kept
    positions exactly;
  * every output row must be a bit copy of the input row its index names.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch

from oracle import lagkv_oracle as O

SCORE_RTOL = 1e-5
TIE_RTOL = 1e-5


@dataclass
class StreamReport:
    chunks: int = 0
    flipped_chunks: int = 0
    max_score_rel: float = 0.0

    def merge(self, o: "StreamReport") -> None:
        self.chunks += o.chunks
        self.flipped_chunks += o.flipped_chunks
        self.max_score_rel = max(self.max_score_rel, o.max_score_rel)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def raw_view(t: torch.Tensor) -> np.ndarray:
    """Bit pattern of a CPU tensor as a NumPy array (bf16 -> uint16)."""
    t = t.detach().to("cpu").contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def check_scores(g_scores: np.ndarray, o_scores: np.ndarray) -> float:
    assert g_scores.shape == o_scores.shape
    if o_scores.size == 0:
        return 0.0
    rel = np.abs(g_scores.astype(np.float64) - o_scores) / np.abs(o_scores)
    worst = float(rel.max())
    assert worst <= SCORE_RTOL, f"score relative error {worst:.3e} > {SCORE_RTOL}"
    return worst


def check_selection(g_kept: np.ndarray, o_scores: np.ndarray, g_scores, L: int, k: int,
                    first_row: int) -> int:
    """g_kept [n_s, k] absolute rows.  Returns the number of chunks that differ from the
    fp64 selection (all of them must be near-ties)."""
    n_s = g_kept.shape[0]
    flipped = 0
    for p in range(n_s):
        lo = first_row + p * L
        got = g_kept[p].astype(np.int64) - lo
        assert np.all(np.diff(got) > 0) and got[0] >= 0 and got[-1] < L, f"chunk {p}: not ascending in range"
        s = o_scores[p * L:(p + 1) * L]
        want = O.top_k(s, k)
        if not np.array_equal(got, want):
            kth = np.sort(s)[::-1][k - 1]
            diff = np.setxor1d(got, want)
            gap = np.abs(s[diff] - kth) / abs(kth)
            assert gap.max() <= TIE_RTOL, \
                f"chunk {p}: selections differ at tokens {diff.tolist()} with relative gap {gap.max():.3e}"
            flipped += 1
        if g_scores is not None:   # decision in the kernel's own precision: exact
            mine = O.top_k(g_scores[p * L:(p + 1) * L].astype(np.float64), k)
            assert np.array_equal(got, mine), f"chunk {p}: kept set is not the top-k of the GPU's own scores"
    return flipped


def check_stream(K: torch.Tensor, V: torch.Tensor, S: int, L: int, r: float, g_idx: torch.Tensor,
                 g_K: torch.Tensor, g_V: torch.Tensor, g_scores=None, ddof: int = 1,
                 variant: str = "lag") -> StreamReport:
    """K, V: [T, D] input stream (CPU or GPU); g_*: the HIP path's outputs for it."""
    K = K.detach().to("cpu"); V = V.detach().to("cpu")
    T = K.shape[0]
    pl = O.plan(T, S, L, r)
    n_s, k = pl["n_scored"], pl["k"]
    g_idx = g_idx.detach().to("cpu").numpy().astype(np.int64)
    assert g_idx.shape[0] == pl["T_out"], "output length differs from Eq. 12"
    rep = StreamReport(chunks=n_s)
    Kr, Vr = raw_view(K), raw_view(V)
    gKr, gVr = raw_view(g_K), raw_view(g_V)
    # rows are bit copies of the rows the indices name
    assert np.array_equal(gKr, Kr[g_idx]) and np.array_equal(gVr, Vr[g_idx]), "output rows are not bit copies"
    if n_s == 0:
        assert np.array_equal(g_idx, np.arange(T))
        return rep
    _, _, o_idx, o_sc = O.compress(to_f64(K), to_f64(V), S, L, r, ddof, variant)
    gs = None
    if g_scores is not None:
        gs = g_scores.detach().to("cpu").numpy()
        if variant == "l2":
            assert np.allclose(gs, o_sc, rtol=SCORE_RTOL, atol=0)
        else:
            rep.max_score_rel = check_scores(gs, o_sc)
    # sink and window
    assert np.array_equal(g_idx[:S], np.arange(S))
    assert np.array_equal(g_idx[S + n_s * k:], np.arange(S + n_s * L, T))
    body = g_idx[S:S + n_s * k].reshape(n_s, k)
    rep.flipped_chunks = check_selection(body, o_sc, gs, L, k, S)
    if rep.flipped_chunks == 0:
        assert np.array_equal(g_idx, o_idx)
    return rep


def check_index_invariants(idx: torch.Tensor, T: int, S: int, L: int, k: int, n_s: int) -> None:
    """Properties that hold at any size, on all streams at once (runs where idx lives):
    sink and window present, exactly k ascending positions inside each scored chunk."""
    B, H, T_out = idx.shape
    assert T_out == S + n_s * k + (T - S - n_s * L)
    dev = idx.device
    i64 = idx.to(torch.int64)
    assert torch.equal(i64[..., :S], torch.arange(S, device=dev).expand(B, H, S))
    win = torch.arange(S + n_s * L, T, device=dev)
    assert torch.equal(i64[..., S + n_s * k:], win.expand(B, H, win.numel()))
    body = i64[..., S:S + n_s * k].reshape(B, H, n_s, k)
    lo = (S + torch.arange(n_s, device=dev) * L).view(1, 1, n_s, 1)
    assert bool(((body >= lo) & (body < lo + L)).all()), "kept position outside its chunk"
    if k > 1:
        assert bool((body[..., 1:] > body[..., :-1]).all()), "kept positions not strictly ascending"
