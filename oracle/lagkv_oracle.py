"""CPU oracle for the LagKV KV-cache compression pass (arXiv 2504.04704).

TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 NumPy restatement of
the method of the paper's Methodology section (subsection "LagKV"), written
so that it can be checked against the paper by eye.  It shares no code with
the HIP library and must never be imported by the product path; only the
tests, the smoke check and the benchmark's CPU-baseline leg may call it.

What each function follows:

  plan()                 the partition rules of subsection LagKV (sink kept, nothing
                         done below S + 2L, chunks of L, the remainder belongs to
                         the sliding window) and Eq. 12-13
  reference_min_max()    Eq. 7-8   (per-channel min/max over the sequence axis
                         of the NEXT chunk)
  normalise()            Eq. 9
  token_spread()         Eq. 10, "Std." part (std over a token's channels)
  chunk_softmax()        Eq. 10, "Softmax" part (over the chunk's L tokens)
  chunk_score()          Eq. 11    (score(K) + score(V))
  top_k()                selection step after Eq. 11: per chunk and per head, k = floor(r*L)
  compress()             the whole pass for one stream, compaction included
  IncrementalCache       the recursive / decode-time use of the same pass
  variants "local","l2"  Eq. 14-15 and Eq. 16 of the Scoring Methods ablation

Readings taken where the paper is silent (each is a choice of this build):
  * std uses divisor D - ddof with ddof = 1 by default;
  * a reference channel with max == min contributes 0 for every token;
  * k = floor(r * L) evaluated in double precision;
  * top-k ties go to the lower position; kept tokens are emitted in
    ascending position; the reference chunk is always the raw next chunk.

Pins (see tests/test_oracle_*.py): Eq. 12 lengths, sink/window retention,
exact per-chunk counts, brute-force rank-count top-k, per-channel affine
invariance, numpy.std / scipy softmax special case, locality, recursion
(one-shot == shorter one-shot + appends), identity at r = 1, a hand-derived
closed-form micro example.  Fidelity to the authors' released code and to the
paper's accuracy tables is "parity unpinned": neither is available here.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Tuple

import numpy as np

VARIANTS = ("lag", "local", "l2")


# --------------------------------------------------------------------------
# partitioning and the closed-form output length (Eq. 12-13)
# --------------------------------------------------------------------------
def keep_count(L: int, r: float) -> int:
    """Tokens kept per chunk, k = floor(r*L) (the text around Eq. 12)."""
    k = int(math.floor(float(r) * int(L)))
    if not (1 <= k <= L):
        raise ValueError(f"k = floor(r*L) = {k} must lie in [1, L]")
    return k


def plan(T: int, S: int, L: int, r: float, n_static: Optional[int] = None) -> Dict[str, int]:
    """Partition of a cache of T rows whose first n_static rows are static
    (sink + already compressed part; n_static = S for a fresh cache).

    Returns n_chunks (full L-chunks after the static part), rem (the modulo,
    which joins the sliding window), n_scored (chunks that have a reference,
    i.e. all but the last), k and T_out (Eq. 12 when n_static == S)."""
    if n_static is None:
        n_static = S
    k = keep_count(L, r)
    rest = T - n_static
    if rest < 2 * L:                         # below S + 2L nothing is compressed
        return dict(n_chunks=max(rest, 0) // L, n_scored=0, rem=max(rest, 0) % L, k=k, T_out=T)
    n = rest // L
    m = rest % L
    n_s = n - 1                              # the last chunk has no reference
    return dict(n_chunks=n, n_scored=n_s, rem=m, k=k, T_out=n_static + k * n_s + L + m)


def eq12_length(Ls: int, S: int, L: int, rL: int) -> int:
    """L_R of Eq. 12, literally; valid for Ls >= S + 2L."""
    return S + rL * ((Ls - S) // L - 1) + L + (Ls - S) % L


def compression_ratio(Ls: int, S: int, L: int, rL: int) -> float:
    """C of Eq. 13; zero when Ls < S + 2L."""
    if Ls < S + 2 * L:
        return 0.0
    return 1.0 - eq12_length(Ls, S, L, rL) / Ls


def keep_for_compression(Ls: int, S: int, L: int, C: float) -> int:
    """Inverse of Eq. 13 by exhaustion: the largest rL in [1, L] whose compression
    ratio is at least C (the Experiments section adapts r to a target ratio at fixed
    L this way).  Raises when Ls < S + 2L or when even rL = 1 compresses less than C."""
    if Ls < S + 2 * L or not (0.0 <= C < 1.0):
        raise ValueError("no compression ratio to reach")
    for rL in range(L, 0, -1):
        if compression_ratio(Ls, S, L, rL) >= C:
            return rL
    raise ValueError("C is not reachable with rL >= 1")


# --------------------------------------------------------------------------
# scoring one chunk (Eq. 7-11)
# --------------------------------------------------------------------------
def reference_min_max(Zref: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Eq. 7-8: per-channel min and max over the sequence axis of the
    reference chunk.  Zref is [L_ref, D]; returns two [D] vectors."""
    return Zref.min(axis=0), Zref.max(axis=0)


def normalise(Zc: np.ndarray, mn: np.ndarray, mx: np.ndarray) -> np.ndarray:
    """Eq. 9: (Z - min) / (max - min) channel by channel.  A channel whose
    reference has max == min gives 0 for every token (no epsilon)."""
    span = mx - mn
    ok = span > 0
    safe = np.where(ok, span, 1.0)
    return np.where(ok[None, :], (Zc - mn[None, :]) / safe[None, :], 0.0)


def token_spread(Zbar: np.ndarray, ddof: int = 1) -> np.ndarray:
    """"Std." of Eq. 10: standard deviation over the D channels of each
    normalised token.  Zbar is [L, D]; returns [L]."""
    D = Zbar.shape[1]
    mu = Zbar.sum(axis=1) / D
    dev = Zbar - mu[:, None]
    return np.sqrt((dev * dev).sum(axis=1) / (D - ddof))


def chunk_softmax(sigma: np.ndarray) -> np.ndarray:
    """"Softmax" of Eq. 10 over the L tokens of one chunk."""
    e = np.exp(sigma - sigma.max())
    return e / e.sum()


def tensor_score(Zc: np.ndarray, Zref: np.ndarray, ddof: int = 1) -> np.ndarray:
    """score(Z) of Eq. 10 for one chunk Zc [L, D] with reference Zref."""
    mn, mx = reference_min_max(Zref)
    return chunk_softmax(token_spread(normalise(Zc, mn, mx), ddof))


def chunk_score(Kc, Kref, Vc, Vref, ddof: int = 1, variant: str = "lag") -> np.ndarray:
    """Final per-token score of one chunk (Eq. 11), fp64 [L].

    variant "lag":   reference = the next chunk (Eq. 7-8)
            "local": reference = the chunk itself (Eq. 14-15)
            "l2":    score = -||K_t||_2 (Eq. 16); V and the reference unused
    """
    Kc = np.asarray(Kc, dtype=np.float64)
    if variant == "l2":
        return -np.sqrt((Kc * Kc).sum(axis=1))
    Vc = np.asarray(Vc, dtype=np.float64)
    if variant == "local":
        Kref, Vref = Kc, Vc
    elif variant != "lag":
        raise ValueError(variant)
    Kref = np.asarray(Kref, dtype=np.float64)
    Vref = np.asarray(Vref, dtype=np.float64)
    return tensor_score(Kc, Kref, ddof) + tensor_score(Vc, Vref, ddof)


# --------------------------------------------------------------------------
# selection
# --------------------------------------------------------------------------
def top_k(score: np.ndarray, k: int) -> np.ndarray:
    """Positions (within the chunk) of the k highest scores, ascending.
    Order: score descending, then position ascending (ties to the earlier
    token)."""
    L = score.shape[0]
    order = np.lexsort((np.arange(L), -score))     # last key is the primary one
    return np.sort(order[:k])


# --------------------------------------------------------------------------
# whole pass over one stream
# --------------------------------------------------------------------------
def score(K: np.ndarray, V: np.ndarray, S: int, L: int, ddof: int = 1,
          variant: str = "lag", n_static: Optional[int] = None) -> np.ndarray:
    """Scores of every scored chunk of one stream.  K, V are [T, D].
    Returns fp64 [n_scored * L]; entry j belongs to row n_static + j."""
    if n_static is None:
        n_static = S
    T = K.shape[0]
    rest = T - n_static
    if rest < 2 * L:
        return np.zeros(0, dtype=np.float64)
    n = rest // L
    out = np.empty((n - 1) * L, dtype=np.float64)
    for p in range(n - 1):
        a = n_static + p * L
        cur = slice(a, a + L)
        ref = slice(a + L, a + 2 * L)
        out[p * L:(p + 1) * L] = chunk_score(K[cur], K[ref], V[cur], V[ref], ddof, variant)
    return out


def select(scores: np.ndarray, L: int, k: int, n_static: int) -> np.ndarray:
    """Kept absolute row positions, [n_scored, k], ascending in each chunk."""
    n_s = scores.shape[0] // L
    kept = np.empty((n_s, k), dtype=np.int64)
    for p in range(n_s):
        kept[p] = n_static + p * L + top_k(scores[p * L:(p + 1) * L], k)
    return kept


def compress(K: np.ndarray, V: np.ndarray, S: int, L: int, r: float, ddof: int = 1,
             variant: str = "lag", n_static: Optional[int] = None,
             raw: Optional[Tuple[np.ndarray, np.ndarray]] = None):
    """One compression pass over one stream.

    K, V: [T, D] values used for scoring (any real dtype; computed in fp64).
    raw:  optional pair of [T, ...] arrays to gather the output rows from (for
          instance the bf16 bit patterns); defaults to K, V themselves.
    Returns (K_out, V_out, idx, scores): rows [0, n_static) unchanged, then the
    kept rows of each scored chunk in order, then the sliding window (last
    full chunk + remainder); idx holds the source row of every output row."""
    if n_static is None:
        n_static = S
    T = K.shape[0]
    pl = plan(T, S, L, r, n_static)
    Kr, Vr = raw if raw is not None else (K, V)
    if pl["n_scored"] == 0:
        idx = np.arange(T, dtype=np.int64)
        return Kr[idx], Vr[idx], idx, np.zeros(0, dtype=np.float64)
    sc = score(K, V, S, L, ddof, variant, n_static)
    kept = select(sc, L, pl["k"], n_static)
    window_start = n_static + pl["n_scored"] * L
    idx = np.concatenate([np.arange(n_static, dtype=np.int64), kept.reshape(-1),
                          np.arange(window_start, T, dtype=np.int64)])
    assert idx.shape[0] == pl["T_out"]
    return Kr[idx], Vr[idx], idx, sc


# --------------------------------------------------------------------------
# recursive (prefill-then-decode) use
# --------------------------------------------------------------------------
class IncrementalCache:
    """One stream's cache under recursive compression.

    State: `pos` (original position of every row held), `n_static` rows that
    are final (sink + kept), the rest being the uncompressed tail.  Each
    append adds rows to the tail; whenever the tail holds at least 2L rows its
    oldest L rows are scored against the next L and reduced to k rows."""

    def __init__(self, D: int, S: int, L: int, r: float, ddof: int = 1,
                 variant: str = "lag", dtype=np.float64):
        self.S, self.L, self.r, self.ddof, self.variant = S, L, r, ddof, variant
        self.k = keep_count(L, r)
        self.K = np.zeros((0, D), dtype=dtype)
        self.V = np.zeros((0, D), dtype=dtype)
        self.pos = np.zeros(0, dtype=np.int64)
        self.n_seen = 0
        self.n_compressed_chunks = 0

    @classmethod
    def from_state(cls, K, V, pos, n_seen: int, n_compressed_chunks: int, S: int, L: int,
                   r: float, ddof: int = 1, variant: str = "lag") -> "IncrementalCache":
        """Resume from rows already held (for instance the output of compress())."""
        c = cls(K.shape[1], S, L, r, ddof, variant, dtype=K.dtype)
        c.K, c.V, c.pos = K.copy(), V.copy(), np.asarray(pos, dtype=np.int64).copy()
        c.n_seen, c.n_compressed_chunks = int(n_seen), int(n_compressed_chunks)
        return c

    @property
    def n_static(self) -> int:
        return min(self.n_seen, self.S) + self.k * self.n_compressed_chunks

    @property
    def n_tail(self) -> int:
        return self.K.shape[0] - self.n_static

    def append(self, K_new: np.ndarray, V_new: np.ndarray) -> int:
        """Append rows, then compress while the tail is at least 2L long.
        Returns the number of chunks compressed by this call."""
        n_new = K_new.shape[0]
        self.K = np.concatenate([self.K, K_new.astype(self.K.dtype)])
        self.V = np.concatenate([self.V, V_new.astype(self.V.dtype)])
        self.pos = np.concatenate([self.pos, self.n_seen + np.arange(n_new, dtype=np.int64)])
        self.n_seen += n_new
        rounds = 0
        L, k = self.L, self.k
        while self.n_tail >= 2 * L:
            a = self.n_static
            sc = chunk_score(self.K[a:a + L], self.K[a + L:a + 2 * L],
                             self.V[a:a + L], self.V[a + L:a + 2 * L], self.ddof, self.variant)
            keep = a + top_k(sc, k)
            rows = np.concatenate([np.arange(a), keep, np.arange(a + L, self.K.shape[0])])
            self.K, self.V, self.pos = self.K[rows], self.V[rows], self.pos[rows]
            self.n_compressed_chunks += 1
            rounds += 1
        return rounds
