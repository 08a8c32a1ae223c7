"""Thin ctypes binding over liblagkv.so (the C ABI declared in include/lagkv.h).

Argument marshalling only: every step of the pass runs in the HIP kernels.
Functions carry the C names (`plan`, `workspace_bytes`, `score`, `select`,
`compress`, `append_and_compress`, `launch_hint`, ...).  torch is used for device memory
and the current HIP stream; there is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Tuple

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblagkv.so")
_lib = None

OK, EINVAL, ESHAPE, EDTYPE, ECAPACITY, EWORKSPACE, EHIP = range(7)
F32, BF16, F16 = 0, 1, 2
SCORE_LAG, SCORE_LOCAL, SCORE_L2 = 0, 1, 2
PATH_AUTO, PATH_FUSED, PATH_STAGED, PATH_RESIDENT = 0, 1, 2, 3
ORDER_LINEAR, ORDER_EVEN_ODD, ORDER_XCD, ORDER_BITREV = 0, 1, 2, 3
SELECT_AUTO, SELECT_WAVE, SELECT_GROUP = 0, 1, 2

EXPORTS = ("lagkv_plan", "lagkv_keep_for_compression", "lagkv_workspace_bytes", "lagkv_score",
           "lagkv_select", "lagkv_compress", "lagkv_compress_static", "lagkv_cache_after_compress",
           "lagkv_prefill_rows",
           "lagkv_append_and_compress", "lagkv_launch_hint", "lagkv_launch_hint_ex", "lagkv_path_for",
           "lagkv_strerror",
           "lagkv_version")


class LagKVError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class Params(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("D", C.c_int32),
                ("S", C.c_int32), ("L", C.c_int32),
                ("r", C.c_double),
                ("dtype", C.c_int32), ("variant", C.c_int32), ("std_ddof", C.c_int32),
                ("launch", C.c_int32),
                ("stride_b", C.c_int64), ("stride_h", C.c_int64), ("stride_t", C.c_int64)]


class PlanT(C.Structure):
    _fields_ = [("n_chunks", C.c_int64), ("n_scored", C.c_int64), ("rem", C.c_int64),
                ("k", C.c_int64), ("T_out", C.c_int64)]


class CacheT(C.Structure):
    _fields_ = [("K", C.c_void_p), ("V", C.c_void_p), ("pos", C.c_void_p),
                ("capacity", C.c_int64), ("n_static", C.c_int64), ("n_tail", C.c_int64),
                ("n_seen", C.c_int64)]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load liblagkv.so (built by paper_2504_04704_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                          f"g.build()'` (hipcc, gfx950) first; there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    vp, i64, sz = C.c_void_p, C.c_int64, C.c_size_t
    lib.lagkv_plan.argtypes = [C.POINTER(Params), i64, i64, C.POINTER(PlanT)]
    lib.lagkv_plan.restype = C.c_int
    lib.lagkv_keep_for_compression.argtypes = [i64, C.c_int32, C.c_int32, C.c_double,
                                               C.POINTER(C.c_int64), C.POINTER(C.c_double)]
    lib.lagkv_keep_for_compression.restype = C.c_int
    lib.lagkv_workspace_bytes.argtypes = [C.POINTER(Params), i64]
    lib.lagkv_workspace_bytes.restype = sz
    lib.lagkv_score.argtypes = [C.POINTER(Params), vp, vp, i64, vp, vp, sz, vp]
    lib.lagkv_score.restype = C.c_int
    lib.lagkv_select.argtypes = [C.POINTER(Params), vp, i64, vp, vp]
    lib.lagkv_select.restype = C.c_int
    lib.lagkv_compress.argtypes = [C.POINTER(Params), vp, vp, i64, vp, vp, vp, vp, vp, sz, vp]
    lib.lagkv_compress.restype = C.c_int
    lib.lagkv_append_and_compress.argtypes = [C.POINTER(Params), C.POINTER(CacheT), vp, vp, i64, vp,
                                              sz, vp]
    lib.lagkv_append_and_compress.restype = C.c_int
    lib.lagkv_compress_static.argtypes = [C.POINTER(Params), vp, vp, i64, vp, vp, vp, vp, vp]
    lib.lagkv_compress_static.restype = C.c_int
    lib.lagkv_cache_after_compress.argtypes = [C.POINTER(Params), i64, C.POINTER(CacheT)]
    lib.lagkv_cache_after_compress.restype = C.c_int
    lib.lagkv_prefill_rows.argtypes = [C.POINTER(Params), C.POINTER(CacheT), i64]
    lib.lagkv_prefill_rows.restype = C.c_int64
    lib.lagkv_launch_hint.argtypes = [C.c_int, C.c_int, C.c_int]
    lib.lagkv_launch_hint.restype = C.c_int32
    lib.lagkv_launch_hint_ex.argtypes = [C.c_int] * 5
    lib.lagkv_launch_hint_ex.restype = C.c_int32
    lib.lagkv_path_for.argtypes = [C.POINTER(Params), C.c_int64]
    lib.lagkv_path_for.restype = C.c_int
    lib.lagkv_strerror.argtypes = [C.c_int]
    lib.lagkv_strerror.restype = C.c_char_p
    lib.lagkv_version.argtypes = []
    lib.lagkv_version.restype = C.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().lagkv_strerror(int(status)).decode()


def version() -> int:
    return load().lagkv_version()


def _check(status: int, where: str):
    if status != OK:
        raise LagKVError(status, where)


_DTYPES = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16}


def path_for(p: "Params", T: int) -> int:
    """lagkv_path_for: the PATH_* lagkv_compress takes for these parameters."""
    v = load().lagkv_path_for(C.byref(p), T)
    if v < 0:
        raise LagKVError(-v, "lagkv_path_for")
    return v


def launch_hint(path: int = PATH_AUTO, waves: int = 0, segments: int = 0, order: int = 0,
                select: int = 0) -> int:
    """lagkv_launch_hint(_ex): the value of Params.launch that overrides the launch choice of one call."""
    v = load().lagkv_launch_hint_ex(path, waves, segments, order, select) if (order or select) \
        else load().lagkv_launch_hint(path, waves, segments)
    if v < 0:
        raise LagKVError(EINVAL, "lagkv_launch_hint")
    return v


def make_params(B: int, H: int, D: int, S: int, L: int, r: float, dtype=BF16, variant=SCORE_LAG,
                std_ddof: int = 1, strides: Tuple[int, int, int] = (0, 0, 0), launch: int = 0) -> Params:
    if isinstance(dtype, torch.dtype):
        dtype = _DTYPES[dtype]
    return Params(B, H, D, S, L, float(r), dtype, variant, std_ddof, launch, *strides)


def params_for(K: torch.Tensor, S: int, L: int, r: float, variant=SCORE_LAG, std_ddof: int = 1,
               launch: int = 0) -> Params:
    """Parameters for a [B,H,T,D] tensor (any strides with a contiguous channel axis)."""
    if K.dim() != 4 or K.stride(3) != 1:
        raise ValueError("expected a [B,H,T,D] tensor with contiguous channels")
    if K.dtype not in _DTYPES:
        raise TypeError(f"unsupported dtype {K.dtype}")
    B, H, _, D = K.shape
    return make_params(B, H, D, S, L, r, _DTYPES[K.dtype], variant, std_ddof,
                       (K.stride(0), K.stride(1), K.stride(2)), launch)


def plan(p: Params, T: int, n_static: int = -1) -> PlanT:
    out = PlanT()
    _check(load().lagkv_plan(C.byref(p), T, n_static, C.byref(out)), "lagkv_plan")
    return out


def keep_for_compression(T: int, S: int, L: int, ratio: float) -> Tuple[int, float]:
    """lagkv_keep_for_compression: (k, r) reaching compression ratio >= `ratio` at fixed S, L."""
    k, r = C.c_int64(), C.c_double()
    _check(load().lagkv_keep_for_compression(T, S, L, ratio, C.byref(k), C.byref(r)),
           "lagkv_keep_for_compression")
    return int(k.value), float(r.value)


def workspace_bytes(p: Params, T: int) -> int:
    return int(load().lagkv_workspace_bytes(C.byref(p), T))


def _stream_ptr(device) -> int:
    return torch.cuda.current_stream(device).cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _workspace(p: Params, T: int, device) -> Optional[torch.Tensor]:
    n = workspace_bytes(p, T)
    return torch.empty(n, dtype=torch.uint8, device=device) if n else None


def _same_layout(K: torch.Tensor, V: torch.Tensor):
    if V.shape != K.shape or V.stride() != K.stride() or V.dtype != K.dtype or V.device != K.device:
        raise ValueError("K and V must share shape, strides, dtype and device")


def score(K: torch.Tensor, V: Optional[torch.Tensor], S: int, L: int, r: float, variant=SCORE_LAG,
          std_ddof: int = 1, ws: Optional[torch.Tensor] = None, launch: int = 0) -> torch.Tensor:
    """lagkv_score: fp32 scores [B,H,n_scored*L] of every scored chunk."""
    if not K.is_cuda:
        raise RuntimeError("lagkv.score needs device tensors; there is no CPU path")
    if V is not None:
        _same_layout(K, V)
    p = params_for(K, S, L, r, variant, std_ddof, launch)
    T = K.shape[2]
    pl = plan(p, T)
    out = torch.empty((p.B, p.H, pl.n_scored * L), dtype=torch.float32, device=K.device)
    _check(load().lagkv_score(C.byref(p), K.data_ptr(), _ptr(V), T, out.data_ptr(), _ptr(ws),
                              0 if ws is None else ws.numel(), _stream_ptr(K.device)), "lagkv_score")
    return out


def select(scores: torch.Tensor, T: int, S: int, L: int, r: float) -> torch.Tensor:
    """lagkv_select: int32 kept positions [B,H,n_scored,k], ascending per chunk."""
    if not scores.is_cuda:
        raise RuntimeError("lagkv.select needs device tensors; there is no CPU path")
    if scores.dim() != 3 or not scores.is_contiguous() or scores.dtype != torch.float32:
        raise ValueError("scores must be a dense fp32 [B,H,n_scored*L] tensor")
    B, H, _ = scores.shape
    p = make_params(B, H, 2, S, L, r, F32)
    pl = plan(p, T)
    if scores.shape[2] != pl.n_scored * L:
        raise ValueError("scores do not match the partition of T")
    kept = torch.empty((B, H, pl.n_scored, pl.k), dtype=torch.int32, device=scores.device)
    _check(load().lagkv_select(C.byref(p), scores.data_ptr(), T, kept.data_ptr(),
                               _stream_ptr(scores.device)), "lagkv_select")
    return kept


@dataclass
class Compressed:
    K: torch.Tensor                 # [B,H,T_out,D]
    V: torch.Tensor
    idx: Optional[torch.Tensor]     # [B,H,T_out] int32 source rows
    scores: Optional[torch.Tensor]  # [B,H,n_scored*L] fp32
    plan: PlanT


def compress(K: torch.Tensor, V: torch.Tensor, S: int, L: int, r: float, variant=SCORE_LAG,
             std_ddof: int = 1, want_idx: bool = True, want_scores: bool = False,
             out: Optional[Tuple[torch.Tensor, torch.Tensor]] = None,
             idx_out: Optional[torch.Tensor] = None, scores_out: Optional[torch.Tensor] = None,
             ws: Optional[torch.Tensor] = None, launch: int = 0) -> Compressed:
    """lagkv_compress: one whole pass.  Output buffers may be passed in (benchmarks)."""
    if not K.is_cuda:
        raise RuntimeError("lagkv.compress needs device tensors; there is no CPU path")
    _same_layout(K, V)
    p = params_for(K, S, L, r, variant, std_ddof, launch)
    B, H, T, D = K.shape
    pl = plan(p, T)
    if out is None:
        Ko = torch.empty((B, H, pl.T_out, D), dtype=K.dtype, device=K.device)
        Vo = torch.empty_like(Ko)
    else:
        Ko, Vo = out
        if tuple(Ko.shape) != (B, H, pl.T_out, D) or not Ko.is_contiguous() or not Vo.is_contiguous() \
                or Vo.shape != Ko.shape or Ko.dtype != K.dtype or Vo.dtype != K.dtype:
            raise ValueError("output buffers must be dense [B,H,T_out,D] of the input dtype")
    if idx_out is None and want_idx:
        idx_out = torch.empty((B, H, pl.T_out), dtype=torch.int32, device=K.device)
    if scores_out is None and want_scores:
        scores_out = torch.empty((B, H, pl.n_scored * L), dtype=torch.float32, device=K.device)
    if ws is None:
        ws = _workspace(p, T, K.device)
    _check(load().lagkv_compress(C.byref(p), K.data_ptr(), V.data_ptr(), T, Ko.data_ptr(),
                                 Vo.data_ptr(), _ptr(idx_out), _ptr(scores_out), _ptr(ws),
                                 0 if ws is None else ws.numel(), _stream_ptr(K.device)),
           "lagkv_compress")
    return Compressed(Ko, Vo, idx_out, scores_out, pl)


STATIC_SCRATCH_BYTES = 16 << 20


def compress_static(K: torch.Tensor, V: torch.Tensor, S: int, L: int, r: float, out: Tuple[torch.Tensor, torch.Tensor],
                    idx_out: Optional[torch.Tensor] = None, scores_out: Optional[torch.Tensor] = None,
                    variant=SCORE_LAG, std_ddof: int = 1, launch: int = 0) -> PlanT:
    """lagkv_compress_static: the whole pass into caller-provided buffers with no workspace and no
    allocation anywhere (the three-kernel path stages in the library's static device array)."""
    if not K.is_cuda:
        raise RuntimeError("lagkv.compress_static needs device tensors; there is no CPU path")
    _same_layout(K, V)
    p = params_for(K, S, L, r, variant, std_ddof, launch)
    B, H, T, D = K.shape
    pl = plan(p, T)
    Ko, Vo = out
    if tuple(Ko.shape) != (B, H, pl.T_out, D) or not Ko.is_contiguous() or not Vo.is_contiguous() \
            or Vo.shape != Ko.shape or Ko.dtype != K.dtype or Vo.dtype != K.dtype:
        raise ValueError("output buffers must be dense [B,H,T_out,D] of the input dtype")
    _check(load().lagkv_compress_static(C.byref(p), K.data_ptr(), V.data_ptr(), T, Ko.data_ptr(),
                                        Vo.data_ptr(), _ptr(idx_out), _ptr(scores_out),
                                        _stream_ptr(K.device)), "lagkv_compress_static")
    return pl


class Cache:
    """Caller-owned decode-time cache: dense [B,H,capacity,D] buffers + the host
    counters of lagkv_cache.  `append_and_compress` forwards to the C call."""

    def __init__(self, B: int, H: int, D: int, capacity: int, S: int, L: int, r: float,
                 dtype=torch.bfloat16, device="cuda", variant=SCORE_LAG, std_ddof: int = 1,
                 track_positions: bool = True, launch: int = 0):
        self.S, self.L, self.r, self.variant, self.std_ddof = S, L, r, variant, std_ddof
        self.launch = launch
        self.K = torch.empty((B, H, capacity, D), dtype=dtype, device=device)
        self.V = torch.empty_like(self.K)
        self.pos = torch.empty((B, H, capacity), dtype=torch.int32, device=device) \
            if track_positions else None
        self.c = CacheT(self.K.data_ptr(), self.V.data_ptr(), _ptr(self.pos), capacity, 0, 0, 0)
        self._ws = None

    @classmethod
    def from_compressed(cls, comp: Compressed, T: int, capacity: int, S: int, L: int, r: float,
                        variant=SCORE_LAG, std_ddof: int = 1, launch: int = 0) -> "Cache":
        """Cache holding the output of compress() on T rows, with room to grow."""
        B, H, T_out, D = comp.K.shape
        c = cls(B, H, D, capacity, S, L, r, comp.K.dtype, comp.K.device, variant, std_ddof,
                comp.idx is not None, launch)
        c.K[:, :, :T_out].copy_(comp.K)
        c.V[:, :, :T_out].copy_(comp.V)
        if comp.idx is not None:
            c.pos[:, :, :T_out].copy_(comp.idx)
        c.mark_compressed(T)
        return c

    def _params(self, strides=(0, 0, 0)) -> Params:
        B, H, _, D = self.K.shape
        return make_params(B, H, D, self.S, self.L, self.r, _DTYPES[self.K.dtype], self.variant,
                           self.std_ddof, strides, self.launch)

    def mark_compressed(self, T: int) -> None:
        """lagkv_cache_after_compress: the buffers now hold the output of compress() on T rows."""
        _check(load().lagkv_cache_after_compress(C.byref(self._params()), T, C.byref(self.c)),
               "lagkv_cache_after_compress")

    @property
    def n_static(self) -> int:
        return self.c.n_static

    @property
    def n_tail(self) -> int:
        return self.c.n_tail

    @property
    def n_seen(self) -> int:
        return self.c.n_seen

    @property
    def length(self) -> int:
        return self.c.n_static + self.c.n_tail

    def append_and_compress(self, K_new: Optional[torch.Tensor], V_new: Optional[torch.Tensor]) -> None:
        B, H, cap, D = self.K.shape
        if K_new is None:
            n_new, strides, dev = 0, (0, 0, 0), self.K.device
        else:
            _same_layout(K_new, V_new)
            if K_new.dim() != 4 or K_new.stride(3) != 1 or K_new.shape[:2] != (B, H) \
                    or K_new.shape[3] != D or K_new.dtype != self.K.dtype:
                raise ValueError("K_new must be [B,H,n_new,D] of the cache dtype")
            n_new = K_new.shape[2]
            strides = (K_new.stride(0), K_new.stride(1), K_new.stride(2))
        p = self._params(strides)
        need = workspace_bytes(p, cap)
        if need and (self._ws is None or self._ws.numel() < need):
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.K.device)
        _check(load().lagkv_append_and_compress(
            C.byref(p), C.byref(self.c), _ptr(K_new), _ptr(V_new), n_new, _ptr(self._ws),
            0 if self._ws is None else self._ws.numel(), _stream_ptr(self.K.device)),
            "lagkv_append_and_compress")


    def prefill_chunked(self, K: torch.Tensor, V: torch.Tensor) -> int:
        """Chunk-by-chunk compression during prefill (Ablation, subsection on the prefill
        stage): the first S + 2L rows in one call, then L rows per call until all rows
        are in; every call is lagkv_append_and_compress.  The model forward that would produce
        each slice between the calls is the caller's; here the rows are given.  Returns the
        number of calls made."""
        T = K.shape[2]
        p = self._params()
        calls, t = 0, 0
        while t < T:
            n = load().lagkv_prefill_rows(C.byref(p), C.byref(self.c), T - t)
            if n <= 0:
                raise LagKVError(EINVAL, "lagkv_prefill_rows")
            self.append_and_compress(K[:, :, t:t + n], V[:, :, t:t + n])
            t += n
            calls += 1
        return calls

    def view(self) -> Tuple[torch.Tensor, torch.Tensor, Optional[torch.Tensor]]:
        n = self.length
        return self.K[:, :, :n], self.V[:, :, :n], None if self.pos is None else self.pos[:, :, :n]
