"""lagkv_compress_static (the entry point for callers that cannot allocate) against
lagkv_compress, through the C ABI: two calls in a row on one GPU, the second with a smaller
input, on shapes that take the three-kernel path (whose scratch is the static device array)
and on one the fused kernels serve; plus its size limit."""
import ctypes as C

import pytest
import torch

from paper_2504_04704_amd import lagkv, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _gen(B, H, T, D, dtype, seed):
    cfg = synth.KVConfig("t", layers=1, B=B, H=H, D=D, T=T, S=0, L=1, r=1.0,
                         dtype="bf16" if dtype == torch.bfloat16 else "f32", n_outlier=min(2, D // 8))
    return synth.make_kv(cfg, device=DEV, seed=seed)


def _both(K, V, S, L, r, variant, launch=0):
    print("[gpu-test] compress_static", tuple(K.shape), K.dtype, "L", L, "variant", variant, flush=True)
    want = lagkv.compress(K, V, S, L, r, variant=variant, want_scores=True, launch=launch)
    torch.cuda.synchronize()
    Ko, Vo = torch.zeros_like(want.K), torch.zeros_like(want.V)
    idx = torch.full_like(want.idx, -1)
    sc = torch.zeros_like(want.scores)
    pl = lagkv.compress_static(K, V, S, L, r, (Ko, Vo), idx, sc, variant=variant, launch=launch)
    torch.cuda.synchronize()
    assert pl.T_out == want.plan.T_out
    # bit-exact rows and positions, identical scores: the same kernels ran on the same inputs
    assert torch.equal(idx, want.idx) and torch.equal(Ko, want.K) and torch.equal(Vo, want.V)
    assert torch.equal(sc, want.scores)
    # without the optional outputs as well.  By now the library's array exists on this GPU (the
    # runtime places it when the first call resolves its address), so the free device memory must
    # not shrink any more: the call itself allocates nothing.
    Ko.zero_(); Vo.zero_()
    free_before = torch.cuda.mem_get_info()[0]
    lagkv.compress_static(K, V, S, L, r, (Ko, Vo), None, None, variant=variant, launch=launch)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before
    assert torch.equal(Ko, want.K) and torch.equal(Vo, want.V)


@pytest.mark.parametrize("variant", [lagkv.SCORE_LAG, lagkv.SCORE_LOCAL, lagkv.SCORE_L2])
def test_static_scratch_two_calls_in_a_row_second_one_smaller(variant):
    lagkv.load()
    # 200-byte rows (D = 100 bf16): only the three-kernel path serves them, so the scratch is used
    K, V = _gen(3, 4, 16 + 9 * 64 + 21, 100, torch.bfloat16, seed=7)
    assert lagkv.workspace_bytes(lagkv.params_for(K, 16, 64, 0.25), K.shape[2]) > 0
    _both(K, V, 16, 64, 0.25, variant)
    # second call: fewer streams, shorter, another lag; the array still holds the first call's data
    K2, V2 = _gen(1, 2, 8 + 4 * 50 + 3, 100, torch.bfloat16, seed=8)
    _both(K2, V2, 8, 50, 0.3, variant)
    # and a larger one again
    _both(K, V, 16, 64, 0.25, variant)


def test_static_scratch_staged_by_hint_and_fused_shapes():
    lagkv.load()
    K, V = _gen(2, 2, 16 + 5 * 128 + 9, 128, torch.bfloat16, seed=9)
    _both(K, V, 16, 128, 0.25, lagkv.SCORE_LAG, lagkv.launch_hint(lagkv.PATH_STAGED))
    _both(K[:1], V[:1], 16, 128, 0.5, lagkv.SCORE_LAG, lagkv.launch_hint(lagkv.PATH_STAGED))
    _both(K, V, 16, 128, 0.25, lagkv.SCORE_LAG)                 # fused kernels: no scratch at all
    Kn, Vn = _gen(1, 2, 100, 40, torch.float32, seed=10)        # below 2L: the no-op copy
    _both(Kn, Vn, 16, 64, 0.25, lagkv.SCORE_LAG)


def test_static_scratch_rejects_sizes_beyond_its_limit():
    lib = lagkv.load()
    # 64 streams x 4 chunks x (L + k) x 4 B would fit; this one needs about 40 MiB
    p = lagkv.make_params(64, 8, 100, 16, 128, 0.25, lagkv.BF16)
    T = 16 + 128 * 160
    assert lagkv.workspace_bytes(p, T) > lagkv.STATIC_SCRATCH_BYTES
    fake = 0x1000                                               # never dereferenced: the size check comes first
    rc = lib.lagkv_compress_static(C.byref(p), fake, fake, T, fake, fake, None, None, None)
    assert rc == lagkv.EWORKSPACE
    assert "workspace" in lagkv.strerror(rc)
