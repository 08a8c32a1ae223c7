"""Pins for the CPU oracle: each test ties one part of oracle/lagkv_oracle.py to
something other than itself (a closed form, an invariant of the method, a
library routine on a special case, brute force on tiny inputs)."""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import lagkv_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.default_rng(seed)


def rand_stream(seed, T, D, k_sigma=0.5, v_sigma=0.3):
    g = rng(seed)
    K = g.standard_normal((T, D)) * np.exp(k_sigma * g.standard_normal(D))[None, :]
    V = g.standard_normal((T, D)) * np.exp(v_sigma * g.standard_normal(T))[:, None]
    return K, V


# ------------------------------------------------------------------ Eq. 12-13
def _golden_rows():
    rows = []
    for line in open(os.path.join(GOLDEN, "eq12_lengths.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            rows.append(tuple(int(x) for x in f[:6]) + (float(f[6]),))
    return rows


@pytest.mark.parametrize("row", _golden_rows())
def test_eq12_golden_lengths(row):
    T, S, L, rL, n_s, LR, C = row
    pl = O.plan(T, S, L, rL / L)
    assert pl["k"] == rL and pl["n_scored"] == n_s and pl["T_out"] == LR
    assert O.eq12_length(T, S, L, rL) == LR
    assert abs(O.compression_ratio(T, S, L, rL) - C) < 5e-4


def test_plan_matches_eq12_everywhere():
    g = rng(1)
    for _ in range(2000):
        S = int(g.integers(0, 40)); L = int(g.integers(1, 70)); k = int(g.integers(1, L + 1))
        T = int(g.integers(0, 600))
        pl = O.plan(T, S, L, (k + 0.5) / L if k < L else 1.0)
        assert pl["k"] == k
        if T >= S + 2 * L:
            assert pl["T_out"] == O.eq12_length(T, S, L, k)
            assert pl["n_chunks"] * L + pl["rem"] == T - S
        else:                                   # "the compression ratio is zero"
            assert pl["T_out"] == T and pl["n_scored"] == 0
            assert O.compression_ratio(T, S, L, k) == 0.0


def test_compress_output_length_and_structure():
    for seed, (T, S, L, r, D) in enumerate([(1024, 16, 128, 0.5, 8), (700, 5, 37, 0.3, 6),
                                            (300, 0, 50, 0.125, 4), (257, 1, 128, 0.25, 4)]):
        K, V = rand_stream(seed, T, D)
        Ko, Vo, idx, sc = O.compress(K, V, S, L, r)
        pl = O.plan(T, S, L, r)
        k, n_s = pl["k"], pl["n_scored"]
        assert idx.shape[0] == pl["T_out"] == O.eq12_length(T, S, L, k)
        # sinks first, window (last full chunk + remainder) last, bit-identical rows
        assert np.array_equal(idx[:S], np.arange(S))
        w0 = S + n_s * L
        assert np.array_equal(idx[S + n_s * k:], np.arange(w0, T))
        assert T - w0 >= L
        assert np.array_equal(Ko, K[idx]) and np.array_equal(Vo, V[idx])
        # exactly k per scored chunk, strictly ascending
        body = idx[S:S + n_s * k].reshape(n_s, k)
        for p in range(n_s):
            assert np.all((body[p] >= S + p * L) & (body[p] < S + (p + 1) * L))
            assert np.all(np.diff(body[p]) > 0)
        assert sc.shape[0] == n_s * L


def test_below_two_lags_is_identity():
    K, V = rand_stream(3, 16 + 2 * 32 - 1, 4)
    Ko, Vo, idx, sc = O.compress(K, V, 16, 32, 0.25)
    assert np.array_equal(idx, np.arange(K.shape[0])) and np.array_equal(Ko, K)
    assert sc.size == 0


def test_identity_when_r_is_one():
    K, V = rand_stream(4, 333, 5)
    Ko, Vo, idx, _ = O.compress(K, V, 7, 20, 1.0)
    assert np.array_equal(idx, np.arange(333)) and np.array_equal(Vo, V)


# ---------------------------------------------------------------- top-k
def brute_rank_topk(score, k):
    L = len(score)
    keep = []
    for t in range(L):
        rank = sum(1 for u in range(L) if score[u] > score[t] or (score[u] == score[t] and u < t))
        if rank < k:
            keep.append(t)
    return np.array(keep)


def test_topk_against_rank_counting():
    g = rng(5)
    for _ in range(300):
        L = int(g.integers(1, 40)); k = int(g.integers(1, L + 1))
        s = g.standard_normal(L)
        if g.random() < 0.5:                    # force exact ties
            s = np.round(s * 2) / 2
        assert np.array_equal(O.top_k(s, k), brute_rank_topk(s, k))


def test_topk_tie_goes_to_lower_position():
    s = np.array([0.1, 0.7, 0.7, 0.7, 0.2])
    assert O.top_k(s, 2).tolist() == [1, 2]
    assert O.top_k(s, 1).tolist() == [1]
    # duplicated tokens give exactly equal scores through the whole pipeline
    K, V = rand_stream(6, 3 * 8, 4)
    K[2] = K[5]; V[2] = V[5]
    sc = O.score(K, V, 0, 8, 1)
    assert sc[2] == sc[5]


# ------------------------------------------------- normalisation and spread
def test_micro_example_closed_form():
    vals = {}
    for line in open(os.path.join(GOLDEN, "micro_example.txt")):
        if line.strip() and not line.startswith("#"):
            f = line.split()
            vals[f[0]] = [float(x) for x in f[1:]]
    K = np.array([[1., 2.], [2., 0.], [0., 0.], [2., 4.]])
    V = np.array([[0., 1.], [1., 1.], [0., -1.], [2., 1.]])
    # the fixture's numbers are themselves closed forms: recompute them here
    a, b = 1 / math.sqrt(2), 1 / (2 * math.sqrt(2))
    closed = [1 / (1 + math.exp(a)) + 1 / (1 + math.exp(-b)),
              1 / (1 + math.exp(-a)) + 1 / (1 + math.exp(b))]
    assert np.allclose(closed, vals["score_ddof1"], atol=1e-11)
    s1 = O.score(K, V, 0, 2, ddof=1)
    s0 = O.score(K, V, 0, 2, ddof=0)
    assert np.allclose(s1, vals["score_ddof1"], atol=1e-11)
    assert np.allclose(s0, vals["score_ddof0"], atol=1e-11)
    _, _, idx, _ = O.compress(K, V, 0, 2, 0.5)
    assert idx.tolist() == [int(vals["kept"][0]), 2, 3]
    # intermediate quantities of the derivation
    mn, mx = O.reference_min_max(K[2:])
    assert mn.tolist() == [0, 0] and mx.tolist() == [2, 4]
    assert O.normalise(K[:2], mn, mx).tolist() == [[.5, .5], [1., 0.]]
    assert np.allclose(O.token_spread(np.array([[.5, .5], [1., 0.]]), 1), [0, a])


def test_single_pair_equals_library_std_and_softmax():
    g = rng(7)
    for ddof in (0, 1):
        L, D = 24, 10
        Kc, Kr, Vc, Vr = (g.standard_normal((L, D)) for _ in range(4))
        def lib(Zc, Zr):
            zb = (Zc - Zr.min(0)) / (Zr.max(0) - Zr.min(0))
            return scipy.special.softmax(np.std(zb, axis=-1, ddof=ddof))
        want = lib(Kc, Kr) + lib(Vc, Vr)
        got = O.chunk_score(Kc, Kr, Vc, Vr, ddof)
        assert np.allclose(got, want, rtol=1e-13, atol=0)


def test_scores_sum_to_two_and_are_bounded():
    K, V = rand_stream(8, 16 + 5 * 32 + 7, 12)
    sc = O.score(K, V, 16, 32).reshape(-1, 32)
    assert np.allclose(sc.sum(axis=1), 2.0, atol=1e-12)
    assert np.all((sc > 0) & (sc < 2))


def test_reference_is_the_next_chunk_not_another():
    """A dropped '+1' (own chunk, previous chunk) changes the result."""
    L, D = 8, 4
    K, V = rand_stream(9, 4 * L, D)
    sc = O.score(K, V, 0, L).reshape(3, L)
    for p in range(3):
        cur = slice(p * L, (p + 1) * L); nxt = slice((p + 1) * L, (p + 2) * L)
        want = scipy.special.softmax(np.std((K[cur] - K[nxt].min(0)) / np.ptp(K[nxt], axis=0), axis=1, ddof=1)) \
            + scipy.special.softmax(np.std((V[cur] - V[nxt].min(0)) / np.ptp(V[nxt], axis=0), axis=1, ddof=1))
        assert np.allclose(sc[p], want, rtol=1e-12)
        own = O.chunk_score(K[cur], K[cur], V[cur], V[cur])
        assert not np.allclose(sc[p], own, rtol=1e-3)
    # axis check: min/max are per channel (over the sequence), std per token (over channels)
    mn, mx = O.reference_min_max(K[:L])
    assert mn.shape == (D,) and O.token_spread(K[:L]).shape == (L,)


def test_affine_invariance_per_channel():
    L, D = 16, 12
    K, V = rand_stream(10, 16 + 4 * L, D)
    base = O.score(K, V, 16, L)
    g = rng(11)
    # power-of-two scales: bit-identical
    a = 2.0 ** g.integers(-6, 7, D)
    assert np.array_equal(O.score(K * a, V * a[::-1], 16, L), base)
    # general positive scale and shift: equal to rounding
    a = np.exp(g.standard_normal(D)); b = 3 * g.standard_normal(D)
    got = O.score(K * a + b, V * a[::-1] - b, 16, L)
    assert np.allclose(got, base, rtol=1e-10, atol=0)
    # flipping the sign of SOME channels maps zbar -> 1 - zbar there, which changes a
    # token's spread: not an invariance (sanity: the test has teeth)
    sgn = np.where(np.arange(D) < D // 2, -1.0, 1.0)
    assert not np.allclose(O.score(K * sgn, V, 16, L), base, rtol=1e-6)
    # ... while flipping ALL channels of a tensor maps every zbar -> 1 - zbar: same spread
    assert np.allclose(O.score(-K, -V, 16, L), base, rtol=1e-10)


def test_degenerate_reference_channel_contributes_zero():
    L, D = 8, 5
    K, V = rand_stream(12, 3 * L, D)
    K[L:2 * L, 2] = 1.25                          # constant channel in the reference of chunk 0
    zb = O.normalise(K[:L], *O.reference_min_max(K[L:2 * L]))
    assert np.all(zb[:, 2] == 0) and np.all(np.isfinite(zb))
    sc = O.score(K, V, 0, L)
    assert np.all(np.isfinite(sc))
    # it stays degenerate, hence invariant, under a positive affine map
    K2 = K.copy(); K2[:, 2] = K2[:, 2] * 4 + 3
    assert np.array_equal(O.score(K2, V, 0, L)[:L], sc[:L])


def test_local_variant_normalises_into_unit_interval():
    K, _ = rand_stream(13, 32, 6)
    zb = O.normalise(K, *O.reference_min_max(K))
    assert zb.min() == 0.0 and zb.max() == 1.0
    assert np.all(zb.min(axis=0) == 0) and np.all(zb.max(axis=0) == 1)
    s_local = O.chunk_score(K, None, K[::-1].copy(), None, variant="local")
    want = O.tensor_score(K, K) + O.tensor_score(K[::-1], K[::-1])
    assert np.array_equal(s_local, want)


def test_l2_variant_is_negative_key_norm():
    K, V = rand_stream(14, 20, 7)
    assert np.allclose(O.chunk_score(K, None, V, None, variant="l2"), -np.linalg.norm(K, axis=1))


# ---------------------------------------------------------------- locality
def test_locality_and_permutations():
    S, L, D = 4, 16, 6
    K, V = rand_stream(15, S + 5 * L + 3, D)
    base = O.score(K, V, S, L).reshape(4, L)
    g = rng(16)
    # tokens outside chunks p and p+1 do not matter for chunk p (p = 1)
    K2, V2 = K.copy(), V.copy()
    K2[:S + L] = g.standard_normal((S + L, D)); V2[S + 3 * L:] = 7.0
    assert np.array_equal(O.score(K2, V2, S, L).reshape(4, L)[1], base[1])
    # permuting the reference chunk's tokens: bit-identical
    K3, V3 = K.copy(), V.copy()
    perm = g.permutation(L)
    K3[S + 2 * L:S + 3 * L] = K[S + 2 * L:S + 3 * L][perm]
    V3[S + 2 * L:S + 3 * L] = V[S + 2 * L:S + 3 * L][perm]
    assert np.array_equal(O.score(K3, V3, S, L).reshape(4, L)[1], base[1])
    # permuting the chunk's own tokens permutes its scores
    K4, V4 = K.copy(), V.copy()
    K4[S + L:S + 2 * L] = K[S + L:S + 2 * L][perm]; V4[S + L:S + 2 * L] = V[S + L:S + 2 * L][perm]
    assert np.allclose(O.score(K4, V4, S, L).reshape(4, L)[1], base[1][perm], rtol=1e-13)
    # permuting channels jointly: equal up to summation order
    cp = g.permutation(D)
    assert np.allclose(O.score(K[:, cp], V[:, cp], S, L).reshape(4, L), base, rtol=1e-12)


# --------------------------------------------------------------- recursion
@pytest.mark.parametrize("T,S,L,r,j", [(16 + 6 * 16 + 5, 16, 16, 0.25, 3), (8 * 10, 0, 10, 0.5, 5),
                                       (3 + 4 * 7 + 6, 3, 7, 0.3, 2)])
def test_one_shot_equals_shorter_one_shot_plus_appends(T, S, L, r, j):
    D = 5
    K, V = rand_stream(17, T, D)
    Ko, Vo, idx, _ = O.compress(K, V, S, L, r)
    T0 = T - j * L
    K0, V0, idx0, _ = O.compress(K[:T0], V[:T0], S, L, r)
    n_s0 = O.plan(T0, S, L, r)["n_scored"]
    c = O.IncrementalCache.from_state(K0, V0, idx0, T0, n_s0, S, L, r)
    for i in range(j):
        rounds = c.append(K[T0 + i * L:T0 + (i + 1) * L], V[T0 + i * L:T0 + (i + 1) * L])
        assert rounds == (1 if T0 >= S + 2 * L or (T0 + (i + 1) * L - S) >= 2 * L else 0)
    assert np.array_equal(c.pos, idx) and np.array_equal(c.K, Ko) and np.array_equal(c.V, Vo)
    assert c.n_static + c.n_tail == O.plan(T, S, L, r)["T_out"]


def test_incremental_from_empty_token_by_token_and_in_bulk():
    S, L, r, D, T = 3, 6, 0.5, 4, 3 + 6 * 7 + 4
    K, V = rand_stream(18, T, D)
    _, _, idx, _ = O.compress(K, V, S, L, r)
    one = O.IncrementalCache(D, S, L, r)
    for t in range(T):
        one.append(K[t:t + 1], V[t:t + 1])
    bulk = O.IncrementalCache(D, S, L, r)
    bulk.append(K[:20], V[:20]); bulk.append(K[20:], V[20:])    # several chunks in one call
    for c in (one, bulk):
        assert np.array_equal(c.pos, idx) and np.array_equal(c.K, K[idx])
        assert c.n_tail == L + (T - S) % L


def test_second_pass_on_compressed_output_is_noop():
    S, L, r, D = 4, 8, 0.25, 4
    K, V = rand_stream(19, S + 5 * L + 3, D)
    Ko, Vo, idx, _ = O.compress(K, V, S, L, r)
    n_static = S + 4 * 2
    K2, V2, idx2, sc2 = O.compress(Ko, Vo, S, L, r, n_static=n_static)
    assert np.array_equal(idx2, np.arange(Ko.shape[0])) and sc2.size == 0


def test_gather_from_raw_arrays():
    K, V = rand_stream(20, 100, 4)
    rawK = np.arange(100, dtype=np.uint16); rawV = rawK + 1000
    Ko, Vo, idx, _ = O.compress(K, V, 2, 10, 0.5, raw=(rawK, rawV))
    assert np.array_equal(Ko, idx.astype(np.uint16)) and np.array_equal(Vo, Ko + 1000)


# ---------------------------------------------------------------- inverse of Eq. 13
def test_keep_for_compression_inverts_eq13():
    """Round trip through the printed formula: the ratio of Eq. 13 at rL = k0 is reached
    with exactly k0; anything above it needs fewer rows; the answer is the boundary of
    the definition (C(k) >= C > C(k+1)); a long sequence approaches 1 - r."""
    rng = np.random.default_rng(5)
    for _ in range(300):
        L = int(rng.integers(1, 200)); S = int(rng.integers(0, 40))
        T = S + 2 * L + int(rng.integers(0, 50 * L))
        k0 = int(rng.integers(1, L + 1))
        c0 = O.compression_ratio(T, S, L, k0)
        if c0 < 0:
            continue
        assert O.keep_for_compression(T, S, L, c0) == k0 or (T - S) // L - 1 == 0
        k = O.keep_for_compression(T, S, L, max(c0 - 1e-9, 0.0))
        assert O.compression_ratio(T, S, L, k) >= max(c0 - 1e-9, 0.0)
        assert k == L or O.compression_ratio(T, S, L, k + 1) < max(c0 - 1e-9, 0.0)
        if k0 > 1:
            c_up = 0.5 * (c0 + O.compression_ratio(T, S, L, k0 - 1))
            assert O.keep_for_compression(T, S, L, c_up) == k0 - 1
    # the Experiments grid: 2x, 4x, 8x of a long cache at L = 128 keep ~ r*L rows per chunk
    T = 16 + 128 * 100000
    for times, rL in ((2, 64), (4, 32), (8, 16)):
        assert O.keep_for_compression(T, 16, 128, 1.0 - 1.0 / times - 1e-4) == rL
    assert O.keep_for_compression(T, 16, 128, 0.0) == 128
    with pytest.raises(ValueError):
        O.keep_for_compression(16 + 255, 16, 128, 0.1)            # shorter than S + 2L: C is 0
    with pytest.raises(ValueError):
        O.keep_for_compression(T, 16, 128, 0.9999)                # below one row per chunk
