"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs (element by element at small sizes; sampled streams plus size-free
invariants at the full workload sizes)."""
import ctypes
import sys

import numpy as np
import pytest
from concurrent.futures import ThreadPoolExecutor
import torch

from oracle import lagkv_oracle as O
from paper_2504_04704_amd import lagkv, synth
from tests import parity_util as PU

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
VARIANT_NAME = {lagkv.SCORE_LAG: "lag", lagkv.SCORE_LOCAL: "local", lagkv.SCORE_L2: "l2"}


def say(*a):
    print("[gpu-test]", *a, flush=True)
    sys.stdout.flush()


@pytest.fixture(autouse=True)
def _library():
    lagkv.load()
    yield


def hint(path=lagkv.PATH_AUTO, waves=0, segments=0, order=0, select=0):
    """Launch override of one call (a pure function of its arguments; the library keeps no state)."""
    return lagkv.launch_hint(path, waves, segments, order, select)


def gen(B, H, T, D, dtype, seed, device=DEV):
    cfg = synth.KVConfig("t", layers=1, B=B, H=H, D=D, T=T, S=0, L=1, r=1.0,
                         dtype="bf16" if dtype == torch.bfloat16 else "f32", n_outlier=min(2, D // 8))
    K, V = synth.make_kv(cfg, device=device, seed=seed)
    if dtype == torch.float16:   # generated in fp32, rounded to binary16 (values are O(10): in range)
        K, V = K.to(torch.float16), V.to(torch.float16)
    return K, V


def run_and_check(K, V, S, L, r, variant=lagkv.SCORE_LAG, ddof=1, streams=None, launch=0):
    out = lagkv.compress(K, V, S, L, r, variant=variant, std_ddof=ddof, want_scores=True, launch=launch)
    torch.cuda.synchronize()
    B, H, T, D = K.shape
    rep = PU.StreamReport()
    todo = streams if streams is not None else [(b, h) for b in range(B) for h in range(H)]
    for b, h in todo:
        sc = out.scores[b, h] if out.scores is not None and out.scores.numel() else None
        rep.merge(PU.check_stream(K[b, h], V[b, h], S, L, r, out.idx[b, h], out.K[b, h], out.V[b, h],
                                  sc, ddof, VARIANT_NAME[variant]))
    return out, rep


# ---------------------------------------------------------------- one-shot pass
@pytest.mark.parametrize("path", [lagkv.PATH_FUSED, lagkv.PATH_STAGED])
def test_config1_tiny_fp32(path):
    cfg = synth.CONFIGS["cfg1_tiny_f32"]
    say("config 1", cfg, "path", path)
    K, V = synth.make_kv(cfg, device=DEV)
    out, rep = run_and_check(K, V, cfg.S, cfg.L, cfg.r, launch=hint(path))
    assert out.plan.T_out == 640 and rep.chunks == 12
    say("config 1 ok: flipped", rep.flipped_chunks, "max score rel", rep.max_score_rel)


SHAPES = [
    # B, H, T, D, dtype, S, L, r
    (2, 2, 16 + 5 * 128 + 37, 128, torch.bfloat16, 16, 128, 0.25),
    (1, 3, 4 + 6 * 100 + 99, 128, torch.bfloat16, 4, 100, 0.33),     # ragged L, odd k
    (1, 2, 7 * 24, 64, torch.float32, 0, 24, 0.5),                   # S = 0, no remainder
    (2, 1, 16 + 3 * 512 + 11, 128, torch.bfloat16, 16, 512, 0.25),
    (1, 2, 9 + 4 * 257, 64, torch.bfloat16, 9, 257, 0.125),          # LPR = 8
    (1, 2, 5 + 5 * 64 + 3, 256, torch.bfloat16, 5, 64, 0.5),         # LPR = 32
    (1, 2, 5 + 5 * 70 + 3, 32, torch.bfloat16, 5, 70, 0.1),          # LPR = 4
    (1, 2, 3 + 4 * 130, 128, torch.float32, 3, 130, 0.3),            # fp32, LPR = 32
    (1, 1, 16 + 2 * 1024 + 5, 128, torch.bfloat16, 16, 1024, 0.125),
    (1, 1, 2 + 2 * 1500 + 1, 64, torch.float32, 2, 1500, 0.01),      # L > 1024: LDS-resident keys
    (3, 2, 1 + 9 * 3, 16, torch.float32, 1, 3, 0.67),                # tiny L
    (1, 2, 3 + 5 * 64 + 9, 128, torch.bfloat16, 3, 64, 0.02),        # k = 1
    (1, 2, 3 + 5 * 64 + 9, 128, torch.bfloat16, 3, 64, 0.99),        # k = L - 1
    (1, 1, 16 + 3 * 4096 + 5, 128, torch.bfloat16, 16, 4096, 0.25),  # long lag: keys and scores through LDS
    (1, 1, 4 + 2 * 6000, 64, torch.bfloat16, 4, 6000, 0.001),        # near the largest lag the LDS budget serves
    (2, 2, 16 + 4 * 128 + 50, 128, torch.float16, 16, 128, 0.25),    # fp16, ring path
    (1, 2, 7 + 5 * 100 + 3, 64, torch.float16, 7, 100, 0.167),       # fp16, register path, r*L = 16.7
]


@pytest.mark.parametrize("shape", SHAPES, ids=lambda s: f"B{s[0]}H{s[1]}T{s[2]}D{s[3]}{str(s[4]).split('.')[-1]}S{s[5]}L{s[6]}r{s[7]}")
@pytest.mark.parametrize("path", [lagkv.PATH_FUSED, lagkv.PATH_STAGED])
def test_shapes_against_oracle(shape, path):
    B, H, T, D, dtype, S, L, r = shape
    say("shape", shape, "path", path)
    K, V = gen(B, H, T, D, dtype, seed=hash(shape[:4]) & 0xffff)
    out, rep = run_and_check(K, V, S, L, r, launch=hint(path))
    assert out.plan.T_out == O.plan(T, S, L, r)["T_out"]
    say("ok: chunks", rep.chunks, "flipped", rep.flipped_chunks, "max rel", rep.max_score_rel)


@pytest.mark.parametrize("D,dtype", [(42, torch.float32), (100, torch.bfloat16), (5, torch.float32), (300, torch.bfloat16),
                                     (13, torch.float16)])
def test_unaligned_head_dims_use_the_staged_path(D, dtype):
    say("unaligned D", D, dtype)
    K, V = gen(1, 2, 8 + 4 * 50 + 7, D, dtype, seed=D)
    assert lagkv.workspace_bytes(lagkv.params_for(K, 8, 50, 0.3), K.shape[2]) > 0
    run_and_check(K, V, 8, 50, 0.3)


# rows of 3, 5, 7, 9, 10, 12, 17, 25 and 31 16-byte slices: fewer than the 4, 8, 16 or 32 lanes that hold a row
RAGGED_ROWS = [(24, torch.bfloat16), (12, torch.float32), (40, torch.bfloat16), (56, torch.float16), (72, torch.float16),
               (40, torch.float32), (96, torch.bfloat16), (48, torch.float32), (80, torch.bfloat16),
               (136, torch.bfloat16), (100, torch.float32), (248, torch.bfloat16)]


@pytest.mark.parametrize("variant", [lagkv.SCORE_LAG, lagkv.SCORE_LOCAL, lagkv.SCORE_L2])
@pytest.mark.parametrize("D,dtype", RAGGED_ROWS)
def test_rows_that_do_not_fill_their_lanes_use_the_fused_kernels(D, dtype, variant):
    """Head sizes whose rows are whole 16-byte slices but not 64, 128, 256 or 512 bytes (D = 96 or
    80 in bf16, 48 in fp32, ...): the streaming kernel takes them, with asynchronous loads (a lag
    that divides evenly) and without (L = 50), several launch shapes, strided views included."""
    say("ragged rows D", D, dtype, "variant", variant)
    for (S, L, r, nw, nseg) in ((16, 64, 0.25, 8, 1), (8, 50, 0.3, 4, 2), (3, 128, 0.125, 2, 3)):
        T = S + 5 * L + 7
        K, V = gen(2, 3, T + 5, D, dtype, seed=D + L)
        K, V = K[:, :, 2:T + 2], V[:, :, 2:T + 2]        # a view: the row stride stays, the base moves by two rows
        p = lagkv.params_for(K, S, L, r, variant=variant)
        assert lagkv.workspace_bytes(p, T) == 0 and lagkv.path_for(p, T) == lagkv.PATH_FUSED
        run_and_check(K, V, S, L, r, variant=variant, launch=hint(lagkv.PATH_FUSED, nw, nseg))


@pytest.mark.parametrize("nw", [1, 2, 4, 8])
@pytest.mark.parametrize("nseg", [1, 3, 1000])
def test_launch_shapes_agree(nw, nseg):
    say("launch shape nw", nw, "nseg", nseg)
    K, V = gen(2, 2, 16 + 9 * 96 + 50, 128, torch.bfloat16, seed=5)
    run_and_check(K, V, 16, 96, 0.25, launch=hint(lagkv.PATH_FUSED, nw, nseg))


@pytest.mark.parametrize("order", [lagkv.ORDER_EVEN_ODD, lagkv.ORDER_XCD, lagkv.ORDER_BITREV])
@pytest.mark.parametrize("B,H", [(2, 4), (3, 1), (1, 5)])
def test_stream_orders_agree(order, B, H):
    """Every workgroup-to-stream order is a permutation: same result as the linear one (8, 3 and 5
    streams: multiple of 8 and power of two, odd, neither)."""
    say("stream order", order, B, H)
    K, V = gen(B, H, 16 + 6 * 64 + 9, 128, torch.bfloat16, seed=17)
    for path in (lagkv.PATH_FUSED, lagkv.PATH_RESIDENT):
        L = 128 if path == lagkv.PATH_RESIDENT else 64
        ref = lagkv.compress(K, V, 16, L, 0.25, launch=hint(path))
        out = lagkv.compress(K, V, 16, L, 0.25, launch=hint(path, segments=2, order=order))
        torch.cuda.synchronize()
        assert torch.equal(out.idx, ref.idx) and torch.equal(out.K, ref.K) and torch.equal(out.V, ref.V)


@pytest.mark.parametrize("select", [lagkv.SELECT_WAVE, lagkv.SELECT_GROUP])
@pytest.mark.parametrize("variant", [lagkv.SCORE_LAG, lagkv.SCORE_LOCAL, lagkv.SCORE_L2])
@pytest.mark.parametrize("L,r,nw", [(512, 0.25, 8), (128, 0.25, 2), (256, 0.125, 4), (100, 0.33, 2), (24, 0.5, 8),
                                    (96, 0.99, 4), (64, 0.02, 1), (300, 0.1, 4)])
def test_selection_modes_against_oracle(select, variant, L, r, nw):
    """Selection by one (rotating) wavefront and by all wavefronts (digit histograms), incl. a lag
    with more tokens than threads (falls back to one wavefront), k = 1 and k = L - 1."""
    say("selection mode", select, "variant", variant, "L", L, "r", r, "waves", nw)
    K, V = gen(1, 3, 16 + 5 * L + 7, 128, torch.bfloat16, seed=L + select)
    K[0, 1, 16 + 5] = K[0, 1, 16 + 2]; V[0, 1, 16 + 5] = V[0, 1, 16 + 2]     # an exact tie
    run_and_check(K, V, 16, L, r, variant=variant, launch=hint(lagkv.PATH_FUSED, nw, 2, select=select))


@pytest.mark.parametrize("variant", [lagkv.SCORE_LAG, lagkv.SCORE_LOCAL, lagkv.SCORE_L2])
@pytest.mark.parametrize("L,r,nw", [(1024, 0.25, 8), (640, 0.3, 8), (1500, 0.1, 8), (2048, 0.125, 8), (1024, 0.125, 4),
                                    (600, 0.5, 2), (1024, 0.999, 8), (1024, 0.125, 0), (600, 0.5, 8)])
def test_long_chunks_are_selected_by_the_whole_workgroup(variant, L, r, nw):
    """Chunks with more tokens than the workgroup has threads (the paper's L = 1024 among them):
    several tokens per thread in the digit-histogram selection (the streaming kernel's default
    above 512 tokens; 2, 3 or 4 tokens per thread here, 5 where a workgroup of 128 threads falls
    back to one wavefront), with exact ties across the slabs of a thread.  (The case of L = 1024
    with 4 wavefronts once ended in a memory fault: a score store went out with a stale base
    address, see the note at the scalar-base stores in lds_dma.hpp.)"""
    say("long chunks", variant, L, r, nw)
    S = 16
    K, V = gen(1, 2, S + 4 * L + 3, 128, torch.bfloat16, seed=L + nw)
    # exact ties: rows duplicated across the first and the last slab of a chunk, and a run of equal rows
    for T_ in (K, V):
        T_[0, 0, S + L - 7] = T_[0, 0, S + 3]
        T_[0, 0, S + L + 600 % L] = T_[0, 0, S + L + 5]
        T_[0, 1, S + 2 * L + 100:S + 2 * L + 140] = T_[0, 1, S + 2 * L + 100]
    for select in (lagkv.SELECT_AUTO, lagkv.SELECT_WAVE):
        out, rep = run_and_check(K, V, S, L, r, variant=variant, launch=hint(lagkv.PATH_FUSED, nw, 2, select=select))
        assert rep.chunks == 2 * 3


def test_group_selection_with_many_ties():
    """Whole chunks of identical rows (every score tied) and rows duplicated in blocks: the
    histogram selection must admit ties from the lowest position up, exactly as the oracle."""
    say("group selection, ties")
    L, S = 256, 8
    K, V = gen(1, 2, S + 4 * L, 128, torch.bfloat16, seed=33)
    K[0, 0, S:S + L] = K[0, 0, S]; V[0, 0, S:S + L] = V[0, 0, S]              # chunk 0 of head 0: all tied
    K[0, 1, S + L:S + 2 * L:2] = K[0, 1, S + L + 1:S + 2 * L:2]               # pairs of equal rows
    V[0, 1, S + L:S + 2 * L:2] = V[0, 1, S + L + 1:S + 2 * L:2]
    for variant in (lagkv.SCORE_LAG, lagkv.SCORE_L2):
        out, _ = run_and_check(K, V, S, L, 0.3, variant=variant,
                               launch=hint(lagkv.PATH_FUSED, 4, select=lagkv.SELECT_GROUP))
        k = out.plan.k
        assert torch.equal(out.idx[0, 0, S:S + k].cpu(), torch.arange(S, S + k, dtype=torch.int32))


RESIDENT_SHAPES = [
    # B, H, n_chunks, rem, D, dtype, L, r, segments
    (2, 2, 6, 37, 128, torch.bfloat16, 512, 0.25, 1),
    (1, 3, 9, 0, 128, torch.bfloat16, 512, 0.125, 2),
    (2, 1, 11, 5, 128, torch.bfloat16, 256, 0.125, 1),      # 2 chunks per batch, odd chunk count
    (1, 2, 14, 100, 128, torch.bfloat16, 128, 0.25, 3),     # 4 chunks per batch, ragged segments
    (1, 2, 3, 1, 128, torch.bfloat16, 128, 0.5, 1),         # fewer chunks than one batch
    (1, 2, 7, 9, 64, torch.float32, 256, 0.167, 2),
    (1, 2, 6, 9, 128, torch.float16, 128, 0.33, 1),
    (1, 1, 2, 0, 128, torch.bfloat16, 512, 0.5, 1),         # one scored chunk
]


@pytest.mark.parametrize("shape", RESIDENT_SHAPES, ids=lambda s: f"B{s[0]}H{s[1]}n{s[2]}m{s[3]}D{s[4]}{str(s[5]).split('.')[-1]}L{s[6]}r{s[7]}seg{s[8]}")
@pytest.mark.parametrize("variant", [lagkv.SCORE_LAG, lagkv.SCORE_LOCAL])
def test_register_resident_kernel_against_oracle(shape, variant):
    """The one-shot kernel that keeps a batch of rows in registers (every row read once)."""
    B, H, n, m, D, dtype, L, r, nseg = shape
    S = 16
    say("resident kernel", shape, "variant", variant)
    K, V = gen(B, H, S + n * L + m, D, dtype, seed=n * 31 + L)
    K[0, 0, S + 3] = K[0, 0, S + 1]; V[0, 0, S + 3] = V[0, 0, S + 1]          # an exact tie
    out, rep = run_and_check(K, V, S, L, r, variant=variant, launch=hint(lagkv.PATH_RESIDENT, segments=nseg))
    assert rep.chunks == B * H * (n - 1)
    sc = lagkv.score(K, V, S, L, r, variant=variant, launch=hint(lagkv.PATH_RESIDENT, segments=nseg))
    torch.cuda.synchronize()
    assert torch.equal(sc, out.scores)


@pytest.mark.parametrize("variant", [lagkv.SCORE_LAG, lagkv.SCORE_LOCAL])
@pytest.mark.parametrize("L", [128, 256, 512])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_resident_kernel_where_the_one_sweep_variance_is_not_enough(L, dtype, variant):
    """The register-resident kernel computes a token's variance in one sweep over its channels
    and must fall back on the two-pass form for statistics with a huge offset against
    their range and for tokens whose normalised values are nearly all equal."""
    S, D = 8, (128 if dtype == torch.bfloat16 else 64)      # rows of 256 bytes
    say("resident kernel, fallback cases", L, dtype, variant)
    K, V = gen(1, 3, S + 5 * L + 3, D, dtype, seed=77 + L)
    # head 0: half of the channels sit far from zero compared with their spread
    K[0, 0, :, ::2] = K[0, 0, :, ::2] * 0.25 + 300.0
    V[0, 0, :, 1::2] = V[0, 0, :, 1::2] * 0.25 - 200.0
    ref_of = (lambda c: c) if variant == lagkv.SCORE_LOCAL else (lambda c: c + 1)
    # head 1: in chunks 2 and 1 every other token equals its reference's channel minima plus
    # a ramp that is tiny against the range (normalised values all within 1e-3 of each other)
    for c in (2, 1):
        lo, rlo = S + c * L, S + ref_of(c) * L
        for T_ in (K, V):
            mn = T_[0, 1, rlo:rlo + L].float().amin(dim=0)
            rg = T_[0, 1, rlo:rlo + L].float().amax(dim=0) - mn
            ramp = torch.linspace(0.5, 0.501, D, device=DEV)
            T_[0, 1, lo + 1:lo + L:2] = (mn + rg * ramp).to(dtype)
    # head 2: one token of chunk 0 is its reference's channel minimum everywhere (variance zero)
    rlo = S + ref_of(0) * L
    K[0, 2, S + 5] = K[0, 2, rlo:rlo + L].float().amin(dim=0).to(dtype)
    V[0, 2, S + 5] = V[0, 2, rlo:rlo + L].float().amin(dim=0).to(dtype)
    out, rep = run_and_check(K, V, S, L, 0.25, variant=variant, launch=hint(lagkv.PATH_RESIDENT))
    assert rep.chunks == 3 * 4
    assert torch.isfinite(out.scores).all()


def test_register_resident_kernel_refuses_other_shapes():
    K, V = gen(1, 1, 16 + 3 * 100, 128, torch.bfloat16, seed=1)
    for kw in (dict(L=100), dict(L=128, variant=lagkv.SCORE_L2)):
        with pytest.raises(lagkv.LagKVError) as e:
            lagkv.compress(K, V, 16, kw.get("L"), 0.25, variant=kw.get("variant", lagkv.SCORE_LAG),
                           launch=hint(lagkv.PATH_RESIDENT))
        assert e.value.status == lagkv.ESHAPE


def test_strided_input_views():
    say("strided views")
    B, H, T, D = 2, 3, 16 + 4 * 64 + 9, 128
    base_k = torch.empty(B, T, H, 2 * D, dtype=torch.bfloat16, device=DEV)      # [B,T,H,2D] storage
    base_v = torch.empty_like(base_k)
    K0, V0 = gen(B, H, T, D, torch.bfloat16, seed=11)
    K = base_k[..., :D].permute(0, 2, 1, 3); V = base_v[..., :D].permute(0, 2, 1, 3)
    K.copy_(K0); V.copy_(V0)
    assert not K.is_contiguous() and K.stride(3) == 1
    out, _ = run_and_check(K, V, 16, 64, 0.25)
    ref = lagkv.compress(K0, V0, 16, 64, 0.25)
    torch.cuda.synchronize()
    assert torch.equal(out.idx, ref.idx) and torch.equal(out.K, ref.K) and torch.equal(out.V, ref.V)


def test_noop_below_two_lags_and_identity_at_r1():
    say("no-op / identity")
    K, V = gen(1, 2, 16 + 2 * 128 - 1, 128, torch.bfloat16, seed=3)
    out = lagkv.compress(K, V, 16, 128, 0.25, want_scores=True)
    torch.cuda.synchronize()
    assert out.plan.n_scored == 0 and torch.equal(out.K, K) and torch.equal(out.V, V)
    assert torch.equal(out.idx[0, 0].cpu(), torch.arange(K.shape[2], dtype=torch.int32))
    assert lagkv.score(K, V, 16, 128, 0.25).numel() == 0
    K, V = gen(1, 2, 16 + 4 * 32 + 5, 128, torch.bfloat16, seed=4)
    for path in (lagkv.PATH_FUSED, lagkv.PATH_STAGED):
        out = lagkv.compress(K, V, 16, 32, 1.0, launch=hint(path))
        torch.cuda.synchronize()
        assert torch.equal(out.K, K) and torch.equal(out.V, V)


@pytest.mark.parametrize("path", [lagkv.PATH_FUSED, lagkv.PATH_STAGED])
def test_degenerate_channel_and_duplicate_tokens(path):
    say("degenerate channel / duplicates, path", path)
    K, V = gen(1, 2, 8 + 4 * 64, 128, torch.bfloat16, seed=21)
    K[:, :, 8 + 64:8 + 128, 5] = 1.25          # constant channel in the reference of chunk 0
    V[:, :, :, 17] = -3.0                      # constant in every reference
    K[0, 0, 8 + 10] = K[0, 0, 8 + 3]; V[0, 0, 8 + 10] = V[0, 0, 8 + 3]   # exact duplicates -> exact tie
    out, rep = run_and_check(K, V, 8, 64, 0.5, launch=hint(path))
    sc = out.scores[0, 0].cpu()
    assert torch.isfinite(out.scores).all()
    assert sc[3] == sc[10]


@pytest.mark.parametrize("path", [lagkv.PATH_FUSED, lagkv.PATH_STAGED])
@pytest.mark.parametrize("variant", [lagkv.SCORE_LOCAL, lagkv.SCORE_L2])
@pytest.mark.parametrize("dtype,D,L,r", [(torch.bfloat16, 128, 64, 0.25), (torch.float32, 48, 64, 0.25), (torch.float32, 42, 64, 0.25),
                                         (torch.bfloat16, 128, 512, 0.125), (torch.float16, 64, 100, 0.33),
                                         (torch.float32, 128, 24, 0.5)])
def test_scoring_variants(variant, dtype, D, L, r, path):
    say("variant", variant, dtype, D, L, "path", path)
    K, V = gen(2, 2, 16 + 5 * L + 3, D, dtype, seed=31 + variant)
    if path == lagkv.PATH_FUSED and D == 42:
        # 168-byte rows are served by the three-kernel path only; asking for the fused one is an error
        with pytest.raises(lagkv.LagKVError) as e:
            lagkv.compress(K, V, 16, L, r, variant=variant, launch=hint(path))
        assert e.value.status == lagkv.ESHAPE
        return
    run_and_check(K, V, 16, L, r, variant=variant, launch=hint(path))


@pytest.mark.parametrize("path", [lagkv.PATH_FUSED, lagkv.PATH_STAGED])
def test_l2_scores_need_no_values(path):
    """Eq. 16 reads K only: lagkv_score accepts V = NULL for it."""
    K, _ = gen(1, 2, 8 + 4 * 128, 128, torch.bfloat16, seed=77)
    sc = lagkv.score(K, None, 8, 128, 0.25, variant=lagkv.SCORE_L2, launch=hint(path))
    torch.cuda.synchronize()
    want = -torch.linalg.vector_norm(K[:, :, 8:8 + 3 * 128].double(), dim=-1)
    assert torch.allclose(sc.double(), want, rtol=1e-5, atol=0)


def test_ddof_zero():
    K, V = gen(1, 2, 16 + 3 * 64, 128, torch.bfloat16, seed=41)
    for path in (lagkv.PATH_FUSED, lagkv.PATH_STAGED):
        run_and_check(K, V, 16, 64, 0.25, ddof=0, launch=hint(path))


# ------------------------------------------------------- stage-by-stage entry points
def test_score_entry_point_matches_oracle():
    say("lagkv_score")
    K, V = gen(2, 2, 16 + 4 * 128 + 9, 128, torch.bfloat16, seed=51)
    for path in (lagkv.PATH_FUSED, lagkv.PATH_STAGED):
        sc = lagkv.score(K, V, 16, 128, 0.25, launch=hint(path))
        torch.cuda.synchronize()
        for b in range(2):
            for h in range(2):
                want = O.score(PU.to_f64(K[b, h]), PU.to_f64(V[b, h]), 16, 128)
                PU.check_scores(sc[b, h].cpu().numpy(), want)
        assert torch.allclose(sc.view(2, 2, 3, 128).sum(-1), torch.full((2, 2, 3), 2.0, device=DEV), atol=1e-5)


@pytest.mark.parametrize("L,k", [(128, 32), (100, 33), (512, 128), (64, 64), (1500, 7), (3, 1), (70, 69)])
def test_select_entry_point_is_exact_with_ties(L, k):
    say("lagkv_select", L, k)
    g = torch.Generator(device="cpu"); g.manual_seed(L * 1000 + k)
    B, H, n_s, S = 2, 2, 5, 4
    T = S + (n_s + 1) * L + 1
    sc = torch.randn(B, H, n_s * L, generator=g)
    sc[0] = torch.round(sc[0] * 4) / 4                      # many exact ties, negative values, zeros
    sc[1, 0, :L] = 0.5                                      # a whole chunk tied
    sc[1, 1, 0] = -0.0; sc[1, 1, 1] = 0.0
    kept = lagkv.select(sc.to(DEV), T, S, L, (k + 0.5) / L if k < L else 1.0)
    torch.cuda.synchronize()
    assert kept.shape == (B, H, n_s, k)
    kept = kept.cpu().numpy()
    s64 = sc.numpy().astype(np.float64)
    for b in range(B):
        for h in range(H):
            want = O.select(s64[b, h], L, k, S)
            assert np.array_equal(kept[b, h], want)


# -------------------------------------------------------------- decode-time variant
def oracle_history_check(cache, Kh, Vh, S, L, r, variant="lag"):
    gK, gV, gpos = cache.view()
    B, H = gK.shape[:2]
    flipped = 0
    for b in range(B):
        for h in range(H):
            rep = PU.check_stream(Kh[b, h], Vh[b, h], S, L, r, gpos[b, h], gK[b, h], gV[b, h], None, 1, variant)
            flipped += rep.flipped_chunks
    pl = O.plan(Kh.shape[2], S, L, r)
    assert cache.length == pl["T_out"] and cache.n_seen == Kh.shape[2]
    if pl["n_scored"]:
        assert cache.n_static == S + pl["k"] * pl["n_scored"] and cache.n_tail == L + pl["rem"]
    return flipped


@pytest.mark.parametrize("path", [lagkv.PATH_FUSED, lagkv.PATH_STAGED])
@pytest.mark.parametrize("steps", [[1] * 150, [7, 64, 1, 200, 3, 3, 130], [400], [16, 127, 1, 128, 128]])
def test_append_from_empty_equals_one_shot(path, steps):
    say("append from empty", steps[:6], "path", path)
    S, L, r, D = 6, 32, 0.25, 128
    T = sum(steps)
    Kh, Vh = gen(1, 2, T, D, torch.bfloat16, seed=61)
    cache = lagkv.Cache(1, 2, D, T + 8, S, L, r, launch=hint(path))
    t = 0
    for n in steps:
        cache.append_and_compress(Kh[:, :, t:t + n], Vh[:, :, t:t + n])
        t += n
        assert cache.n_tail < 2 * L or cache.n_seen < S + 2 * L
    torch.cuda.synchronize()
    oracle_history_check(cache, Kh, Vh, S, L, r)


@pytest.mark.parametrize("path", [lagkv.PATH_FUSED, lagkv.PATH_STAGED])
@pytest.mark.parametrize("dtype,D,variant", [(torch.bfloat16, 128, lagkv.SCORE_LAG), (torch.float32, 64, lagkv.SCORE_LAG),
                                             (torch.bfloat16, 128, lagkv.SCORE_LOCAL), (torch.float32, 42, lagkv.SCORE_L2),
                                             (torch.float32, 40, lagkv.SCORE_L2), (torch.bfloat16, 96, lagkv.SCORE_LAG),
                                             (torch.float16, 72, lagkv.SCORE_LOCAL), (torch.bfloat16, 24, lagkv.SCORE_LAG),
                                             (torch.bfloat16, 128, lagkv.SCORE_L2), (torch.float16, 64, lagkv.SCORE_L2)])
def test_append_after_one_shot_equals_one_shot_on_history(path, dtype, D, variant):
    say("append after compress", dtype, D, variant, "path", path)
    S, L, r = 16, 64, 0.25
    T0, rounds = 16 + 6 * 64 + 20, 5
    Kh, Vh = gen(2, 2, T0 + rounds * L, D, dtype, seed=71)
    if path == lagkv.PATH_FUSED and D == 42:
        # 168-byte rows are served by the three-kernel path only; asking for the fused one is an error
        cache = lagkv.Cache(2, 2, D, T0, S, L, r, dtype=dtype, variant=variant, launch=hint(path))
        with pytest.raises(lagkv.LagKVError) as e:
            cache.append_and_compress(Kh[:, :, :T0], Vh[:, :, :T0])
        assert e.value.status == lagkv.ESHAPE and cache.length == 0
        return
    comp = lagkv.compress(Kh[:, :, :T0].contiguous(), Vh[:, :, :T0].contiguous(), S, L, r, variant=variant,
                          launch=hint(path))
    cache = lagkv.Cache.from_compressed(comp, T0, comp.plan.T_out + 3 * L, S, L, r, variant=variant,
                                        launch=hint(path))
    for i in range(rounds):
        a = T0 + i * L
        cache.append_and_compress(Kh[:, :, a:a + L], Vh[:, :, a:a + L])     # strided views of the history
    cache.append_and_compress(None, None)                                   # n_new = 0 is allowed
    torch.cuda.synchronize()
    oracle_history_check(cache, Kh, Vh, S, L, r, VARIANT_NAME[variant])


@pytest.mark.parametrize("variant,select", [(lagkv.SCORE_LAG, lagkv.SELECT_AUTO), (lagkv.SCORE_L2, lagkv.SELECT_AUTO),
                                            (lagkv.SCORE_LAG, lagkv.SELECT_GROUP), (lagkv.SCORE_L2, lagkv.SELECT_GROUP)])
@pytest.mark.parametrize("L,D,dtype,r", [(32, 128, torch.bfloat16, 0.25), (24, 64, torch.float32, 0.5),
                                         (128, 128, torch.bfloat16, 0.25), (70, 32, torch.bfloat16, 0.1),
                                         (16, 256, torch.bfloat16, 0.9), (50, 128, torch.float32, 0.33),
                                         (32, 96, torch.bfloat16, 0.25), (50, 40, torch.float32, 0.33),
                                         (64, 24, torch.float16, 0.25), (24, 200, torch.bfloat16, 0.5)])
def test_single_round_decode_step_with_the_boundary_anywhere(L, D, dtype, r, variant, select):
    """The steady decode step (exactly one chunk completes) with the border between cached
    and new rows inside the chunk, inside the reference, at their ends, and in the rest; Eq. 7-11
    and Eq. 16 scoring, selection by one wavefront and by the whole workgroup."""
    S = 5
    cases = [(0, 2 * L), (1, 3 * L - 2), (L - 1, L + 1), (L, L), (L + 1, L - 1), (L + L // 2, L // 2 + 3),
             (2 * L - 1, 1), (2 * L - 1, L), (L + 3, 2 * L - 4)]
    for n_tail, n_new in cases:
        say("decode step", L, D, dtype, "tail", n_tail, "new", n_new)
        T = S + n_tail + n_new
        Kh, Vh = gen(2, 3, T, D, dtype, seed=L * 7 + n_tail)
        cache = lagkv.Cache(2, 3, D, T + 4, S, L, r, dtype=dtype, variant=variant,
                            launch=hint(lagkv.PATH_FUSED, select=select))
        cache.append_and_compress(Kh[:, :, :S + n_tail], Vh[:, :, :S + n_tail])
        assert cache.n_static == S and cache.n_tail == n_tail
        cache.append_and_compress(Kh[:, :, S + n_tail:], Vh[:, :, S + n_tail:])
        torch.cuda.synchronize()
        assert cache.n_tail == n_tail + n_new - L
        oracle_history_check(cache, Kh, Vh, S, L, r, VARIANT_NAME[variant])


def test_single_round_decode_step_repeats_and_without_positions():
    S, L, r, D = 16, 128, 0.25, 128
    T = S + 2 * L + 112 + 5 * L
    Kh, Vh = gen(1, 4, T, D, torch.bfloat16, seed=99)
    with_pos = lagkv.Cache(1, 4, D, T, S, L, r, track_positions=True, launch=hint(lagkv.PATH_FUSED))
    without = lagkv.Cache(1, 4, D, T, S, L, r, track_positions=False, launch=hint(lagkv.PATH_FUSED))
    t = 0
    for n in [S + L + 112] + [L] * 6:
        say("decode steps", t, n)
        with_pos.append_and_compress(Kh[:, :, t:t + n], Vh[:, :, t:t + n])
        without.append_and_compress(Kh[:, :, t:t + n], Vh[:, :, t:t + n])
        t += n
    torch.cuda.synchronize()
    oracle_history_check(with_pos, Kh, Vh, S, L, r)
    n = with_pos.length
    assert without.length == n
    assert torch.equal(without.K[:, :, :n], with_pos.K[:, :, :n]) and torch.equal(without.V[:, :, :n], with_pos.V[:, :, :n])


@pytest.mark.parametrize("dtype", [torch.float16, torch.bfloat16])
def test_prefill_chunk_by_chunk_equals_one_shot(dtype):
    """S + 2L rows first, then L rows per call (the chunked prefill of the ablation)."""
    S, L, r, D = 16, 64, 0.25, 128
    T = S + 2 * L + 7 * L + 13
    Kh, Vh = gen(2, 2, T, D, dtype, seed=123)
    cache = lagkv.Cache(2, 2, D, T, S, L, r, dtype=dtype)
    calls = cache.prefill_chunked(Kh, Vh)
    torch.cuda.synchronize()
    assert calls == 1 + 8
    oracle_history_check(cache, Kh, Vh, S, L, r)


def _prefill_at_scale(cfg, layers, n_sample):
    """Chunk-by-chunk prefill (S + 2L rows, then one lag per lagkv_append_and_compress call) of
    `layers` layers of a workload configuration: the final cache against the one-shot oracle on
    sampled streams, against the one-shot pass on all of them, and both timings."""
    import time
    sub = cfg.scaled(layers=layers)
    K, V = synth.make_kv(sub, device=DEV)
    pl = lagkv.plan(lagkv.params_for(K, cfg.S, cfg.L, cfg.r), cfg.T)
    cache = lagkv.Cache(K.shape[0], cfg.H, cfg.D, pl.T_out + 2 * cfg.L, cfg.S, cfg.L, cfg.r)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    calls = cache.prefill_chunked(K, V)
    torch.cuda.synchronize()
    t_chunked = time.perf_counter() - t0
    assert calls == 1 + -(-(cfg.T - cfg.S - 2 * cfg.L) // cfg.L)
    assert cache.length == pl.T_out and cache.n_seen == cfg.T
    one = lagkv.compress(K, V, cfg.S, cfg.L, cfg.r)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    one = lagkv.compress(K, V, cfg.S, cfg.L, cfg.r)
    torch.cuda.synchronize()
    t_one = time.perf_counter() - t0
    gK, gV, gpos = cache.view()
    PU.check_index_invariants(gpos, cfg.T, cfg.S, cfg.L, pl.k, pl.n_scored)
    same = (gpos == one.idx).all(dim=-1)
    say(f"prefill chunk by chunk, {sub.streams} streams of {cfg.name}: {calls} calls in {t_chunked * 1e3:.1f} ms "
        f"({cfg.B * cfg.T / t_chunked:.3g} tokens/s per {layers} layers); one-shot pass {t_one * 1e3:.2f} ms; "
        f"{int(same.sum())} of {same.numel()} streams identical to the one-shot pass")

    def check(s):
        b, h = divmod(s, cfg.H)
        return PU.check_stream(K[b, h], V[b, h], cfg.S, cfg.L, cfg.r, gpos[b, h], gK[b, h], gV[b, h])

    rep = PU.StreamReport()
    with ThreadPoolExecutor(8) as ex:
        for r in ex.map(check, synth.stream_sample(sub.streams, n_sample)):
            rep.merge(r)
    # the recursion and the one-shot pass may differ only where the oracle sees a near-tie
    assert int((~same).sum()) <= max(2, same.numel() // 16)
    return rep


def test_prefill_chunk_by_chunk_at_config2_scale():
    """All 32 layers of the 16K configuration (256 streams, L = 128): 1 + 126 calls, each the
    single-round decode kernel."""
    rep = _prefill_at_scale(synth.CONFIGS["cfg2_llama8b_16k"], 32, 32)
    assert rep.chunks == 32 * 126


def test_prefill_chunk_by_chunk_on_one_layer_of_config4():
    """One layer of the 128K configuration (B=4 x 8 heads = 32 streams, L = 512): 1 + 254 calls
    through the general append kernel (a 512-row reference chunk does not fit the LDS of the
    single-round kernel)."""
    rep = _prefill_at_scale(synth.CONFIGS["cfg4_llama8b_128k_b4"], 1, 8)
    assert rep.chunks == 8 * 254


GRID_K = {(128, 0.5): 64, (128, 0.25): 32, (128, 0.167): 21, (128, 0.125): 16,
          (512, 0.5): 256, (512, 0.25): 128, (512, 0.167): 85, (512, 0.125): 64,
          (1024, 0.5): 512, (1024, 0.25): 256, (1024, 0.167): 171, (1024, 0.125): 128}


@pytest.mark.parametrize("variant", [lagkv.SCORE_LAG, lagkv.SCORE_LOCAL, lagkv.SCORE_L2])
@pytest.mark.parametrize("L,r", sorted(GRID_K))
def test_paper_parameter_grid_on_qwen_shaped_streams(L, r, variant):
    """The settings of the Experiments and Ablation sections: S = 16, L in {128, 512, 1024},
    r in {1/2, 1/4, 0.167, 1/8} (floor(r L) kept per chunk), on a stream set shaped like
    Qwen2.5-7B's cache (28 layers x 4 KV heads, D = 128, bf16), every scoring variant.  Index
    invariants on all 112 streams, 10 sampled streams against the oracle."""
    S, n_chunks = 16, 5
    T = S + n_chunks * L + 77
    say("grid", L, r, "variant", variant)
    K, V = gen(28, 4, T, 128, torch.bfloat16, seed=L + int(r * 1000))
    out = lagkv.compress(K, V, S, L, r, variant=variant, want_scores=True)
    torch.cuda.synchronize()
    assert out.plan.k == GRID_K[(L, r)] and out.plan.n_scored == n_chunks - 1
    PU.check_index_invariants(out.idx, T, S, L, out.plan.k, out.plan.n_scored)

    def check(s):
        b, h = divmod(s, 4)
        return PU.check_stream(K[b, h], V[b, h], S, L, r, out.idx[b, h], out.K[b, h], out.V[b, h],
                               out.scores[b, h], 1, VARIANT_NAME[variant])

    rep = PU.StreamReport()
    with ThreadPoolExecutor(8) as ex:
        for x in ex.map(check, synth.stream_sample(112, 10)):
            rep.merge(x)
    assert rep.chunks == 10 * (n_chunks - 1)


def test_append_capacity_error_leaves_cache_untouched():
    cache = lagkv.Cache(1, 1, 128, 64, 4, 16, 0.5)
    Kn, Vn = gen(1, 1, 65, 128, torch.bfloat16, seed=81)
    with pytest.raises(lagkv.LagKVError) as e:
        cache.append_and_compress(Kn, Vn)
    assert e.value.status == lagkv.ECAPACITY and cache.length == 0 and cache.n_seen == 0


# ------------------------------------------------------------ full workload sizes
def _full_config(name, n_sample, want_scores=True):
    cfg = synth.CONFIGS[name]
    say("full config", name, "streams", cfg.streams, "T", cfg.T)
    K, V = synth.make_kv(cfg, device=DEV)
    out = lagkv.compress(K, V, cfg.S, cfg.L, cfg.r, want_scores=want_scores)
    torch.cuda.synchronize()
    pl = out.plan
    PU.check_index_invariants(out.idx, cfg.T, cfg.S, cfg.L, pl.k, pl.n_scored)
    rep = PU.StreamReport()

    def one(s):
        b, h = divmod(s, cfg.H)
        sc = out.scores[b, h] if want_scores else None
        return PU.check_stream(K[b, h], V[b, h], cfg.S, cfg.L, cfg.r, out.idx[b, h], out.K[b, h],
                               out.V[b, h], sc)

    # the oracle is NumPy: a few host threads check different streams at the same time
    with ThreadPoolExecutor(8) as ex:
        for r in ex.map(one, synth.stream_sample(cfg.streams, n_sample)):
            rep.merge(r)
    say(name, "ok: sampled chunks", rep.chunks, "near-tie flips", rep.flipped_chunks,
        "max score rel err", f"{rep.max_score_rel:.2e}")
    return out, rep


@pytest.mark.parametrize("L,r,path", [(512, 0.25, lagkv.PATH_AUTO), (1024, 0.125, lagkv.PATH_AUTO), (128, 0.25, lagkv.PATH_FUSED)])
def test_a_stream_of_a_million_tokens(L, r, path):
    """One long context instead of many streams: 2^20 tokens and a ragged end per stream (two streams,
    so the register-resident kernel cuts each into 128 segments; the streaming kernel likewise), every
    chunk against the oracle, scores included."""
    T = 16 + (1 << 20) + 37
    say("a million tokens", L, r, path)
    K, V = gen(1, 2, T, 128, torch.bfloat16, seed=2020 + L)
    out, rep = run_and_check(K, V, 16, L, r, launch=hint(path))
    pl = O.plan(T, 16, L, r)
    assert out.plan.T_out == pl["T_out"] and rep.chunks == 2 * pl["n_scored"]
    say("ok: chunks", rep.chunks, "flipped", rep.flipped_chunks, "max rel", rep.max_score_rel)


def test_config2_llama8b_16k():
    out, _ = _full_config("cfg2_llama8b_16k", 256)  # every stream
    assert out.plan.T_out == 4288


def test_config3_llama8b_64k():
    out, _ = _full_config("cfg3_llama8b_64k", 256)  # every stream
    assert out.plan.T_out == 8640


def test_config4_llama8b_128k_b4_bench_configuration():
    """The headline workload in the launch configuration bench.py times (defaults,
    no score dump): 64 GiB scanned, 128 sampled streams against the oracle.  A second launch
    of the same configuration with the score dump on must reproduce the first one's output, and
    its scores are compared with the oracle on the same sample; so are the streaming kernel's
    (the other one-shot kernel that serves this shape)."""
    cfg = synth.CONFIGS["cfg4_llama8b_128k_b4"]
    say("full config", cfg.name, "streams", cfg.streams, "T", cfg.T)
    K, V = synth.make_kv(cfg, device=DEV)
    out = lagkv.compress(K, V, cfg.S, cfg.L, cfg.r)
    torch.cuda.synchronize()
    pl = out.plan
    assert pl.T_out == 33536
    PU.check_index_invariants(out.idx, cfg.T, cfg.S, cfg.L, pl.k, pl.n_scored)
    scores = torch.empty((K.shape[0], cfg.H, pl.n_scored * cfg.L), dtype=torch.float32, device=DEV)
    again = lagkv.compress(K, V, cfg.S, cfg.L, cfg.r, scores_out=scores)
    torch.cuda.synchronize()
    assert torch.equal(again.idx, out.idx) and torch.equal(again.K, out.K) and torch.equal(again.V, out.V)
    del again
    sample = synth.stream_sample(cfg.streams, 128)
    rep = PU.StreamReport()

    def one(s):
        b, h = divmod(s, cfg.H)
        return PU.check_stream(K[b, h], V[b, h], cfg.S, cfg.L, cfg.r, out.idx[b, h], out.K[b, h], out.V[b, h],
                               scores[b, h])

    with ThreadPoolExecutor(8) as ex:
        for r in ex.map(one, sample):
            rep.merge(r)
    say(cfg.name, "ok: sampled chunks", rep.chunks, "near-tie flips", rep.flipped_chunks,
        "max score rel err", f"{rep.max_score_rel:.2e}")
    assert rep.chunks == 128 * 254
    # the streaming kernel on the same workload: index invariants everywhere, scores on a few streams
    del out
    fused = lagkv.compress(K, V, cfg.S, cfg.L, cfg.r, scores_out=scores, launch=hint(lagkv.PATH_FUSED))
    torch.cuda.synchronize()
    PU.check_index_invariants(fused.idx, cfg.T, cfg.S, cfg.L, pl.k, pl.n_scored)
    for s in sample[:16]:
        b, h = divmod(s, cfg.H)
        PU.check_stream(K[b, h], V[b, h], cfg.S, cfg.L, cfg.r, fused.idx[b, h], fused.K[b, h], fused.V[b, h],
                        scores[b, h])


def test_config5_decode_rounds_reduced_batch():
    """Config 5 at reduced batch (B=1 instead of 32: 256 streams), all 64 rounds;
    bench.py times the full batch.  Final caches of sampled streams against the one-shot
    oracle on the concatenated history."""
    cfg = synth.CONFIGS["cfg5_decode_b32"].scaled(B=1)
    say("config 5 (B=1)", cfg)
    K, V = synth.make_kv(cfg, device=DEV)
    comp = lagkv.compress(K, V, cfg.S, cfg.L, cfg.r)
    assert comp.plan.T_out == 8384
    rounds = 64
    cache = lagkv.Cache.from_compressed(comp, cfg.T, comp.plan.T_out + rounds * 32 + cfg.L, cfg.S, cfg.L, cfg.r)
    hist_k, hist_v = [K], [V]
    for i in range(rounds):
        Kn, Vn = synth.make_new_tokens(cfg, cfg.L, i, device=DEV)
        cache.append_and_compress(Kn, Vn)
        hist_k.append(Kn); hist_v.append(Vn)
        assert cache.n_tail == 240 and cache.length == 8384 + 32 * (i + 1)
    torch.cuda.synchronize()
    Kh, Vh = torch.cat(hist_k, dim=2), torch.cat(hist_v, dim=2)
    gK, gV, gpos = cache.view()
    PU.check_index_invariants(gpos, Kh.shape[2], cfg.S, cfg.L, 32, 254 + rounds)

    def one(s):
        b, h = divmod(s, cfg.H)
        return PU.check_stream(Kh[b, h], Vh[b, h], cfg.S, cfg.L, cfg.r, gpos[b, h], gK[b, h], gV[b, h])

    rep = PU.StreamReport()
    with ThreadPoolExecutor(8) as ex:               # every one of the 256 streams
        for r in ex.map(one, range(cfg.streams)):
            rep.merge(r)
    assert rep.chunks == cfg.streams * (254 + rounds)
    say("config 5 (B=1) ok: chunks", rep.chunks, "near-tie flips", rep.flipped_chunks)


# ------------------------------------------------------------------ HIP graph capture
@pytest.mark.parametrize("L", [128, 512])     # 512: the launch that opts in to more than 64 KiB of LDS
def test_compress_can_be_captured_in_a_graph_and_replayed(L):
    """The pass enqueues kernels only (no allocation, no memset, no synchronisation), so a
    caller may capture it in a HIP graph.  Replays, with eager work between them, must all
    reproduce the eager result."""
    S, r = 16, 0.25
    K, V = gen(2, 4, S + 9 * L + 17, 128, torch.bfloat16, seed=404)
    eager = lagkv.compress(K, V, S, L, r)
    torch.cuda.synchronize()
    Ko, Vo = torch.zeros_like(eager.K), torch.zeros_like(eager.V)
    idx = torch.zeros_like(eager.idx)
    ws = torch.empty(max(lagkv.workspace_bytes(lagkv.params_for(K, S, L, r), K.shape[2]), 16), dtype=torch.uint8, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                       # warm-up on the capture stream
        lagkv.compress(K, V, S, L, r, out=(Ko, Vo), idx_out=idx, ws=ws)
    torch.cuda.current_stream().wait_stream(side)
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        lagkv.compress(K, V, S, L, r, out=(Ko, Vo), idx_out=idx, ws=ws)
    for rep in range(3):
        Ko.zero_(); Vo.zero_(); idx.zero_()             # eager work between the replays
        _ = (K.float().sum() + rep).item()
        g.replay()
        torch.cuda.synchronize()
        say("graph replay", rep)
        assert torch.equal(Ko, eager.K) and torch.equal(Vo, eager.V) and torch.equal(idx, eager.idx)
    # new input bytes in the same buffers: the replay follows them
    K2, V2 = gen(2, 4, S + 9 * L + 17, 128, torch.bfloat16, seed=405)
    K.copy_(K2); V.copy_(V2)
    g.replay()
    torch.cuda.synchronize()
    fresh = lagkv.compress(K, V, S, L, r)
    torch.cuda.synchronize()
    assert torch.equal(Ko, fresh.K) and torch.equal(idx, fresh.idx)


def test_config5_decode_full_batch_sampled_streams():
    """Config 5 at its real size (B = 32: 8192 streams, the launch bench.py times), all 64
    rounds: the compressed starting cache is built layer by layer (the uncompressed one would be
    128 GiB), the history of 64 sampled streams is kept on the host, and their final caches are
    compared with the one-shot oracle on that history."""
    cfg = synth.CONFIGS["cfg5_decode_b32"]
    rounds = 64
    say("config 5 full batch", cfg.streams, "streams")
    pl = lagkv.plan(lagkv.make_params(cfg.layers * cfg.B, cfg.H, cfg.D, cfg.S, cfg.L, cfg.r), cfg.T)
    assert pl.T_out == 8384
    cap = pl.T_out + rounds * pl.k + cfg.L
    cache = lagkv.Cache(cfg.layers * cfg.B, cfg.H, cfg.D, cap, cfg.S, cfg.L, cfg.r, track_positions=True)
    sample = synth.stream_sample(cfg.streams, 64)
    hist = {s: ([], []) for s in sample}
    Kl = torch.empty((cfg.B, cfg.H, cfg.T, cfg.D), dtype=torch.bfloat16, device=DEV)
    Vl = torch.empty_like(Kl)
    for l in range(cfg.layers):
        synth.fill_layer(cfg, synth.MASTER_SEED, l, Kl, Vl)
        comp = lagkv.compress(Kl, Vl, cfg.S, cfg.L, cfg.r)
        sl = slice(l * cfg.B, (l + 1) * cfg.B)
        cache.K[sl, :, :pl.T_out].copy_(comp.K)
        cache.V[sl, :, :pl.T_out].copy_(comp.V)
        cache.pos[sl, :, :pl.T_out].copy_(comp.idx)
        for s in sample:
            bb, h = divmod(s, cfg.H)
            if l * cfg.B <= bb < (l + 1) * cfg.B:
                hist[s][0].append(Kl[bb - l * cfg.B, h].cpu())
                hist[s][1].append(Vl[bb - l * cfg.B, h].cpu())
    del Kl, Vl, comp
    cache.mark_compressed(cfg.T)
    for i in range(rounds):
        Kn, Vn = synth.make_new_tokens(cfg, cfg.L, i, device=DEV)
        cache.append_and_compress(Kn, Vn)
        for s in sample:
            bb, h = divmod(s, cfg.H)
            hist[s][0].append(Kn[bb, h].cpu())
            hist[s][1].append(Vn[bb, h].cpu())
        assert cache.n_tail == 240 and cache.length == 8384 + 32 * (i + 1)
    torch.cuda.synchronize()
    gK, gV, gpos = cache.view()
    T_hist = cfg.T + rounds * cfg.L
    PU.check_index_invariants(gpos, T_hist, cfg.S, cfg.L, 32, 254 + rounds)

    def one(s):
        bb, h = divmod(s, cfg.H)
        Kh, Vh = torch.cat(hist[s][0], dim=0), torch.cat(hist[s][1], dim=0)
        assert Kh.shape[0] == T_hist
        return PU.check_stream(Kh, Vh, cfg.S, cfg.L, cfg.r, gpos[bb, h], gK[bb, h], gV[bb, h])

    rep = PU.StreamReport()
    with ThreadPoolExecutor(8) as ex:
        for r in ex.map(one, sample):
            rep.merge(r)
    assert rep.chunks == 64 * (254 + rounds)
    say("config 5 full batch ok: chunks", rep.chunks, "near-tie flips", rep.flipped_chunks)
