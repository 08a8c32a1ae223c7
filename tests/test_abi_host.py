"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, its partition arithmetic equals Eq. 12 / the oracle, and
every validation error is returned before any device work."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import lagkv_oracle as O
from paper_2504_04704_amd import lagkv

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lagkv.lib_path()):
        from paper_2504_04704_amd import build
        build.build_library(verbose=False)
    return lagkv.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "lagkv.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(lagkv_[a-z_]+)\s*\(", header))
    assert declared == set(lagkv.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_layouts_match_header(tmp_path):
    """The header compiles as plain C and ctypes mirrors its struct layouts."""
    src = tmp_path / "layout.c"
    src.write_text(r"""
#include <stdio.h>
#include <stddef.h>
#include "lagkv.h"
int main(void) {
  printf("%zu %zu %zu %zu %zu %zu %zu %zu %zu %zu\n", sizeof(lagkv_params), offsetof(lagkv_params, r),
         offsetof(lagkv_params, dtype), offsetof(lagkv_params, stride_b), offsetof(lagkv_params, stride_t),
         sizeof(lagkv_plan_t), offsetof(lagkv_plan_t, T_out), sizeof(lagkv_cache),
         offsetof(lagkv_cache, capacity), offsetof(lagkv_cache, n_seen));
  return 0;
}
""")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    got = [int(x) for x in subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.split()]
    P, T, K = lagkv.Params, lagkv.PlanT, lagkv.CacheT
    assert got == [C.sizeof(P), P.r.offset, P.dtype.offset, P.stride_b.offset, P.stride_t.offset,
                   C.sizeof(T), T.T_out.offset, C.sizeof(K), K.capacity.offset, K.n_seen.offset]


def test_plan_equals_eq12_and_oracle(lib):
    rng = np.random.default_rng(0)
    for _ in range(500):
        S = int(rng.integers(0, 40)); L = int(rng.integers(1, 300)); k = int(rng.integers(1, L + 1))
        T = int(rng.integers(1, 5000)); r = (k + 0.5) / L if k < L else 1.0
        p = lagkv.make_params(1, 1, 8, S, L, r)
        pl = lagkv.plan(p, T)
        want = O.plan(T, S, L, r)
        assert (pl.n_chunks, pl.n_scored, pl.rem, pl.k, pl.T_out) == \
            (want["n_chunks"], want["n_scored"], want["rem"], want["k"], want["T_out"])
        if T >= S + 2 * L:
            assert pl.T_out == O.eq12_length(T, S, L, k)
    for T, S, L, rL, n_s, LR in [(1024, 16, 128, 64, 6, 640), (16384, 16, 128, 32, 126, 4288),
                                 (65536, 16, 256, 32, 254, 8640), (131072, 16, 512, 128, 254, 33536),
                                 (32768, 16, 128, 32, 254, 8384), (40960, 16, 128, 32, 318, 10432)]:
        pl = lagkv.plan(lagkv.make_params(4, 8, 128, S, L, rL / L), T)
        assert (pl.k, pl.n_scored, pl.T_out) == (rL, n_s, LR)
    # explicit static part (second pass over a compressed cache is a no-op)
    pl = lagkv.plan(lagkv.make_params(1, 1, 8, 16, 128, 0.25), 4288, 16 + 126 * 32)
    assert pl.n_scored == 0 and pl.T_out == 4288


def _status(fn, *a):
    try:
        fn(*a)
    except lagkv.LagKVError as e:
        return e.status
    return lagkv.OK


def test_keep_for_compression_matches_the_exhaustive_oracle(lib):
    """lagkv_keep_for_compression (closed form + boundary fix-up) against the oracle's
    exhaustive search over rL, on a random grid and at its error cases."""
    import random
    from paper_2504_04704_amd import lagkv
    rnd = random.Random(11)
    for _ in range(2000):
        L = rnd.randint(1, 300); S = rnd.randint(0, 64)
        T = S + 2 * L + rnd.randint(0, 80 * L)
        target = rnd.choice([0.0, rnd.random() * 0.999, O.compression_ratio(T, S, L, rnd.randint(1, L))])
        target = min(max(target, 0.0), 0.999)
        try:
            want = O.keep_for_compression(T, S, L, target)
        except ValueError:
            with pytest.raises(lagkv.LagKVError):
                lagkv.keep_for_compression(T, S, L, target)
            continue
        k, r = lagkv.keep_for_compression(T, S, L, target)
        assert k == want, (T, S, L, target)
        assert O.keep_count(L, r) == k and 0 < r <= 1
    for bad in [(100, 16, 128, 0.5), (10**6, 16, 128, 1.0), (10**6, 16, 128, -0.1), (10**6, -1, 128, 0.5),
                (10**6, 16, 0, 0.5), (10**6, 16, 128, float("nan"))]:
        with pytest.raises(lagkv.LagKVError):
            lagkv.keep_for_compression(*bad)


def test_parameter_validation(lib):
    ok = dict(B=1, H=2, D=64, S=16, L=128, r=0.5)
    def P(**kw):
        d = dict(ok); d.update(kw)
        extra = {k: d.pop(k) for k in ("dtype", "variant", "std_ddof", "strides") if k in d}
        return lagkv.make_params(d["B"], d["H"], d["D"], d["S"], d["L"], d["r"], **extra)
    assert _status(lagkv.plan, P(), 1024) == lagkv.OK
    assert _status(lagkv.plan, P(r=0.0), 1024) == lagkv.EINVAL
    assert _status(lagkv.plan, P(r=1.5), 1024) == lagkv.EINVAL
    assert _status(lagkv.plan, P(r=float("nan")), 1024) == lagkv.EINVAL
    assert _status(lagkv.plan, P(r=0.001), 1024) == lagkv.EINVAL          # floor(r*L) < 1
    assert _status(lagkv.plan, P(L=0), 1024) == lagkv.EINVAL
    assert _status(lagkv.plan, P(S=-1), 1024) == lagkv.EINVAL
    assert _status(lagkv.plan, P(D=1), 1024) == lagkv.ESHAPE              # ddof=1 needs D>=2
    assert _status(lagkv.plan, P(D=1, std_ddof=0), 1024) == lagkv.OK
    assert _status(lagkv.plan, P(std_ddof=2), 1024) == lagkv.EINVAL
    assert _status(lagkv.plan, P(B=0), 1024) == lagkv.ESHAPE
    assert _status(lagkv.plan, P(dtype=7), 1024) == lagkv.EDTYPE
    assert _status(lagkv.plan, P(variant=3), 1024) == lagkv.EDTYPE
    assert _status(lagkv.plan, P(strides=(-1, 0, 0)), 1024) == lagkv.ESHAPE
    assert _status(lagkv.plan, P(), -5) == lagkv.ESHAPE
    assert lib.lagkv_plan(None, 10, -1, C.byref(lagkv.PlanT())) == lagkv.EINVAL
    assert lib.lagkv_plan(C.byref(P()), 10, -1, None) == lagkv.EINVAL
    p = P(); p.launch = -1
    assert _status(lagkv.plan, p, 1024) == lagkv.EINVAL
    p = P(); p.launch = 3 << 2            # 3 wavefronts: not a value lagkv_launch_hint returns
    assert _status(lagkv.plan, p, 1024) == lagkv.EINVAL


def test_calls_reject_bad_arguments_before_touching_the_device(lib):
    p = lagkv.make_params(1, 2, 64, 16, 128, 0.5, lagkv.F32)
    fake = 0x1000                      # never dereferenced: validation fails first
    assert lib.lagkv_score(C.byref(p), None, fake, 1024, fake, None, 0, None) == lagkv.EINVAL
    assert lib.lagkv_score(C.byref(p), fake, fake, 1024, None, None, 0, None) == lagkv.EINVAL
    assert lib.lagkv_score(C.byref(p), fake + 2, fake, 1024, fake, None, 0, None) == lagkv.EINVAL
    assert lib.lagkv_score(C.byref(p), fake, fake, 0, fake, None, 0, None) == lagkv.ESHAPE
    assert lib.lagkv_score(C.byref(p), fake, fake, 100, None, None, 0, None) == lagkv.OK  # below 2L: no-op
    assert lib.lagkv_select(C.byref(p), None, 1024, fake, None) == lagkv.EINVAL
    assert lib.lagkv_select(C.byref(p), fake, 100, None, None) == lagkv.OK
    assert lib.lagkv_compress(C.byref(p), fake, fake, 1024, None, fake, None, None, None, 0, None) == lagkv.EINVAL
    bad_stride = lagkv.make_params(1, 2, 64, 16, 128, 0.5, lagkv.F32, strides=(0, 0, 32))
    assert lib.lagkv_compress(C.byref(bad_stride), fake, fake, 1024, fake, fake, None, None, None, 0,
                              None) == lagkv.ESHAPE
    # positions are int32: a cache of 2^31 rows or more is refused before anything is enqueued
    for T_big in (2 ** 31, 2 ** 40):
        assert lib.lagkv_compress(C.byref(p), fake, fake, T_big, fake, fake, None, None, None, 0, None) == lagkv.ESHAPE
        assert lib.lagkv_score(C.byref(p), fake, fake, T_big, fake, None, 0, None) == lagkv.ESHAPE
        assert lagkv.workspace_bytes(p, T_big) == 0
    # a shape only the three-kernel path serves needs a workspace
    odd = lagkv.make_params(1, 2, 42, 16, 128, 0.5, lagkv.F32)
    need = lagkv.workspace_bytes(odd, 1024)
    assert need > 0 and lagkv.workspace_bytes(p, 1024) == 0
    assert lib.lagkv_compress(C.byref(odd), fake, fake, 1024, fake, fake, None, None, None, 0,
                              None) == lagkv.EWORKSPACE
    assert lib.lagkv_compress(C.byref(odd), fake, fake, 1024, fake, fake, None, None, fake, 64,
                              None) == lagkv.EWORKSPACE
    # forcing the fused kernels on a shape they do not cover is an error, not a fallback
    forced = lagkv.make_params(1, 2, 42, 16, 128, 0.5, lagkv.F32, launch=lagkv.launch_hint(lagkv.PATH_FUSED))
    assert lib.lagkv_compress(C.byref(forced), fake, fake, 1024, fake, fake, None, None, fake, need,
                              None) == lagkv.ESHAPE
    # the staged path asked for by hint needs its workspace even on a fused shape, and says so
    staged = lagkv.make_params(1, 2, 64, 16, 128, 0.5, lagkv.F32, launch=lagkv.launch_hint(lagkv.PATH_STAGED))
    assert lagkv.workspace_bytes(staged, 1024) > 0
    assert lib.lagkv_compress(C.byref(staged), fake, fake, 1024, fake, fake, None, None, None, 0,
                              None) == lagkv.EWORKSPACE
    # L beyond what fits the per-workgroup LDS budget
    huge = lagkv.make_params(1, 1, 64, 0, 1 << 20, 0.5, lagkv.F32)
    assert lib.lagkv_score(C.byref(huge), fake, fake, 1 << 22, fake, None, 0, None) == lagkv.ESHAPE


def test_append_validation(lib):
    p = lagkv.make_params(1, 2, 64, 16, 128, 0.5, lagkv.F32)
    fake = 0x1000
    c = lagkv.CacheT(fake, fake, None, 512, 16, 200, 216)
    assert lib.lagkv_append_and_compress(C.byref(p), C.byref(c), fake, fake, 400, None, 0, None) \
        == lagkv.ECAPACITY
    assert (c.n_static, c.n_tail, c.n_seen) == (16, 200, 216)          # untouched on error
    assert lib.lagkv_append_and_compress(C.byref(p), C.byref(c), None, fake, 4, None, 0, None) == lagkv.EINVAL
    assert lib.lagkv_append_and_compress(C.byref(p), None, fake, fake, 4, None, 0, None) == lagkv.EINVAL
    assert lib.lagkv_append_and_compress(C.byref(p), C.byref(c), fake, fake, -1, None, 0, None) == lagkv.EINVAL
    c2 = lagkv.CacheT(None, fake, None, 512, 0, 0, 0)
    assert lib.lagkv_append_and_compress(C.byref(p), C.byref(c2), fake, fake, 4, None, 0, None) == lagkv.EINVAL


def test_launch_hint_is_a_pure_function(lib):
    """lagkv_launch_hint(_ex) packs its arguments, rejects unknown values, and a call with the
    hint behaves the same however often and in whatever order hints were made (no state)."""
    assert lib.lagkv_launch_hint(0, 0, 0) == 0 and lib.lagkv_launch_hint_ex(0, 0, 0, 0, 0) == 0
    seen = set()
    for path in range(4):
        for waves in (0, 1, 2, 4, 8):
            for seg in (0, 1, 7, 1 << 20):
                v = lib.lagkv_launch_hint(path, waves, seg)
                assert v >= 0 and v == lib.lagkv_launch_hint(path, waves, seg) and v not in seen
                seen.add(v)
                for order in range(4):
                    for sel in range(3):
                        w = lib.lagkv_launch_hint_ex(path, waves, seg, order, sel)
                        assert w >= 0 and (w == v) == (order == 0 and sel == 0)
                        assert _status(lagkv.plan, lagkv.make_params(1, 2, 64, 16, 128, 0.5, launch=w), 1024) == lagkv.OK
    for bad in [(4, 0, 0), (-1, 0, 0), (0, 3, 0), (0, 16, 0), (0, 0, -1), (0, 0, (1 << 20) + 1)]:
        assert lib.lagkv_launch_hint(*bad) == -1
    assert lib.lagkv_launch_hint_ex(0, 0, 0, 4, 0) == -1 and lib.lagkv_launch_hint_ex(0, 0, 0, 0, 3) == -1
    # making other hints in between changes nothing for a call that carries its own
    staged = lagkv.make_params(1, 2, 64, 16, 128, 0.5, lagkv.F32, launch=lagkv.launch_hint(lagkv.PATH_STAGED))
    before = lagkv.workspace_bytes(staged, 4096)
    lagkv.launch_hint(lagkv.PATH_FUSED, 8, 5)
    assert lagkv.workspace_bytes(staged, 4096) == before > 0
    assert lagkv.workspace_bytes(lagkv.make_params(1, 2, 64, 16, 128, 0.5, lagkv.F32), 4096) == 0


def test_path_for_names_the_kernels_of_a_call(lib):
    """lagkv_path_for: rows of 256 bytes with a lag of 128, 256 or 512 go to the register-resident
    kernel (not Eq. 16), other fused shapes to the streaming kernel, the rest to the
    three-kernel path; hints are honoured or refused as lagkv_compress does."""
    mk = lagkv.make_params
    T = 16 + 8 * 512
    for L in (128, 256, 512):
        assert lagkv.path_for(mk(2, 8, 128, 16, L, 0.25, lagkv.BF16), T) == lagkv.PATH_RESIDENT
        assert lagkv.path_for(mk(2, 8, 64, 16, L, 0.25, lagkv.F32), T) == lagkv.PATH_RESIDENT
        assert lagkv.path_for(mk(2, 8, 128, 16, L, 0.25, lagkv.BF16, variant=lagkv.SCORE_LOCAL), T) == lagkv.PATH_RESIDENT
        assert lagkv.path_for(mk(2, 8, 128, 16, L, 0.25, lagkv.BF16, variant=lagkv.SCORE_L2), T) == lagkv.PATH_FUSED
        assert lagkv.path_for(mk(2, 8, 128, 16, L, 0.25, lagkv.BF16, launch=lagkv.launch_hint(lagkv.PATH_FUSED)), T) \
            == lagkv.PATH_FUSED
        assert lagkv.path_for(mk(2, 8, 128, 16, L, 0.25, lagkv.BF16, launch=lagkv.launch_hint(lagkv.PATH_STAGED)), T) \
            == lagkv.PATH_STAGED
    assert lagkv.path_for(mk(2, 8, 128, 16, 100, 0.25, lagkv.BF16), T) == lagkv.PATH_FUSED
    assert lagkv.path_for(mk(2, 8, 128, 16, 512, 0.25, lagkv.F32), T) == lagkv.PATH_FUSED      # rows of 512 bytes
    assert lagkv.path_for(mk(2, 8, 40, 16, 128, 0.25, lagkv.F32), T) == lagkv.PATH_FUSED       # rows of 160 bytes
    assert lagkv.path_for(mk(2, 8, 96, 16, 128, 0.25, lagkv.BF16), T) == lagkv.PATH_FUSED      # rows of 192 bytes
    assert lagkv.path_for(mk(2, 8, 24, 16, 128, 0.25, lagkv.BF16), T) == lagkv.PATH_FUSED      # rows of 48 bytes
    assert lagkv.path_for(mk(2, 8, 16, 16, 128, 0.25, lagkv.BF16), T) == lagkv.PATH_STAGED     # rows of 32 bytes
    assert lagkv.path_for(mk(2, 8, 42, 16, 128, 0.25, lagkv.F32), T) == lagkv.PATH_STAGED      # rows of 168 bytes
    assert lagkv.path_for(mk(2, 8, 264, 16, 128, 0.25, lagkv.BF16), T) == lagkv.PATH_STAGED    # rows of 528 bytes
    for bad in (mk(2, 8, 128, 16, 100, 0.25, lagkv.BF16, launch=lagkv.launch_hint(lagkv.PATH_RESIDENT)),
                mk(2, 8, 42, 16, 128, 0.25, lagkv.F32, launch=lagkv.launch_hint(lagkv.PATH_FUSED))):
        assert lib.lagkv_path_for(C.byref(bad), T) == -lagkv.ESHAPE
    for L, nw in ((1024, 4), (600, 2), (1024, 8), (1024, 0), (512, 4)):          # any workgroup size the hint allows
        hinted = mk(2, 8, 128, 16, L, 0.25, lagkv.BF16, launch=lagkv.launch_hint(lagkv.PATH_FUSED, nw))
        assert lib.lagkv_path_for(C.byref(hinted), 16 + 8 * 1024) == lagkv.PATH_FUSED
    assert lib.lagkv_path_for(C.byref(mk(2, 8, 128, 16, 128, 0.001, lagkv.BF16)), T) == -lagkv.EINVAL
    assert lib.lagkv_path_for(C.byref(mk(2, 8, 128, 16, 128, 0.25, lagkv.BF16)), 0) == -lagkv.ESHAPE


def test_cache_after_compress_and_prefill_rows_follow_eq12(lib):
    """The host calls that keep the partition integers behind the ABI, against the oracle's plan."""
    rng = np.random.default_rng(5)
    for _ in range(300):
        S = int(rng.integers(0, 40)); L = int(rng.integers(1, 200)); k = int(rng.integers(1, L + 1))
        T = int(rng.integers(0, 4000)); r = (k + 0.5) / L if k < L else 1.0
        p = lagkv.make_params(2, 3, 8, S, L, r)
        want = O.plan(T, S, L, r)
        c = lagkv.CacheT(0x1000, 0x1000, None, want["T_out"] + int(rng.integers(0, 3)), 7, 7, 7)
        assert lib.lagkv_cache_after_compress(C.byref(p), T, C.byref(c)) == lagkv.OK
        if want["n_scored"]:
            assert (c.n_static, c.n_tail, c.n_seen) == (S + k * want["n_scored"], L + want["rem"], T)
        else:
            assert (c.n_static, c.n_tail, c.n_seen) == (min(T, S), T - min(T, S), T)
        assert c.n_static + c.n_tail == want["T_out"]
        # chunk-by-chunk prefill: S + 2L rows first, then one lag per call
        empty = lagkv.CacheT(0x1000, 0x1000, None, 10, 0, 0, 0)
        assert lib.lagkv_prefill_rows(C.byref(p), C.byref(empty), 10**9) == S + 2 * L
        assert lib.lagkv_prefill_rows(C.byref(p), C.byref(empty), 5) == min(5, S + 2 * L)
        assert lib.lagkv_prefill_rows(C.byref(p), C.byref(c), 10**9) == (L if T > 0 else S + 2 * L)
        assert lib.lagkv_prefill_rows(C.byref(p), C.byref(c), 0) == 0
    p = lagkv.make_params(1, 1, 8, 16, 128, 0.25)
    small = lagkv.CacheT(0x1000, 0x1000, None, 100, 0, 0, 0)
    assert lib.lagkv_cache_after_compress(C.byref(p), 4096, C.byref(small)) == lagkv.ECAPACITY
    assert (small.n_static, small.n_tail, small.n_seen) == (0, 0, 0)
    assert lib.lagkv_cache_after_compress(C.byref(p), 4096, None) == lagkv.EINVAL
    assert lib.lagkv_cache_after_compress(None, 4096, C.byref(small)) == lagkv.EINVAL
    assert lib.lagkv_prefill_rows(None, C.byref(small), 5) == 0


def test_strerror_and_version(lib):
    for s in range(7):
        assert len(lagkv.strerror(s)) > 1
    assert lagkv.strerror(1234) == "unknown status"
    assert lagkv.version() >= 200


def test_binding_refuses_cpu_tensors():
    import torch
    K = torch.zeros(1, 1, 512, 64)
    with pytest.raises(RuntimeError):
        lagkv.compress(K, K.clone(), 16, 128, 0.5)
    with pytest.raises(RuntimeError):
        lagkv.score(K, K.clone(), 16, 128, 0.5)
