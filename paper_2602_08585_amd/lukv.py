"""Thin ctypes binding of liblukv's C ABI (include/lukv.h).

Argument marshalling only: every step of the eviction path runs in the HIP kernels of
liblukv.so.  Tensors are torch CUDA(ROCm) tensors used as device memory; the binding passes
their `data_ptr()` and the current torch stream.  There is no CPU fallback: importing works
without the library (so that host-only tools can import the package), but every call raises
if liblukv.so is missing.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
from typing import Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblukv.so")

LUKV_OK = 0
LUKV_EINVAL = -1
LUKV_EDTYPE = -2
LUKV_EINFEASIBLE = -3
LUKV_EWORKSPACE = -4
LUKV_ELAUNCH = -5
LUKV_BF16 = 0
LUKV_F32 = 1
LUKV_MAX_SEQS = 64
LUKV_ST_INFEASIBLE = 1
LUKV_ST_CLAMPED = 2

EXPORTS = ("lukv_workspace_bytes", "lukv_allocate_workspace_bytes", "lukv_score", "lukv_allocate",
           "lukv_select_compact", "lukv_evict", "lukv_score_lse", "lukv_evict_lse",
           "lukv_profile_workspace_bytes", "lukv_profile_curves", "lukv_profile_build", "lukv_budgets_from_profile",
           "lukv_evict_budgets", "lukv_decode_workspace_bytes", "lukv_decode_attention",
           "lukv_evict_static", "lukv_allocate_topk", "lukv_strerror")
# include/lukv_bench.h: instrumentation for programs that time the path
BENCH_EXPORTS = ("lukv_set_stage_events", "lukv_stage_name", "lukv_bench_stream_read", "lukv_bench_copy")
LUKV_STATIC_SCRATCH_BYTES = 16 << 20
LUKV_NUM_STAGES = 9
LUKV_NUM_STAGE_EVENTS = 2 * LUKV_NUM_STAGES


class _CConfig(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("window", ctypes.c_int32), ("pool_kernel", ctypes.c_int32),
                ("n_sink", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("n_seqs", ctypes.c_int32), ("cu_seqlens", ctypes.POINTER(ctypes.c_int32)),
                ("stride_layer", ctypes.c_int64), ("stride_head", ctypes.c_int64),
                ("stride_tok", ctypes.c_int64), ("qstride_layer", ctypes.c_int64),
                ("qstride_head", ctypes.c_int64), ("qstride_tok", ctypes.c_int64),
                ("softmax_scale", ctypes.c_float)]


class LukvError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (%d)" % (where, strerror(code), code))


_lib = None


def load_library() -> ctypes.CDLL:
    """dlopen liblukv.so built in-tree; raises if it is not there (no fallback)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("liblukv.so is not built: run `python -m paper_2602_08585_amd.build` "
                           "(or __graft_entry__.build()) first; there is no CPU fallback")
    lib = ctypes.CDLL(LIB_PATH)
    P, I32, I64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    CP = ctypes.POINTER(_CConfig)
    lib.lukv_workspace_bytes.argtypes = [CP, I32, ctypes.POINTER(I64)]
    lib.lukv_allocate_workspace_bytes.argtypes = [I32, I32, I32, ctypes.POINTER(I64)]
    lib.lukv_score.argtypes = [CP, P, P, P, P, I64, P]
    lib.lukv_allocate.argtypes = [I32, I32, I32, P, P, P, P, ctypes.POINTER(I64), P, P, P, P, I64, P]
    lib.lukv_allocate_topk.argtypes = [CP, P, ctypes.POINTER(I64), I32, P, P, P, P, I64, P]
    lib.lukv_select_compact.argtypes = [CP, P, P, P, P, P, I64, P, P, P, P, P, I64, P]
    lib.lukv_evict.argtypes = [CP, P, P, P, I32, P, P, P, P, ctypes.POINTER(I64),
                               P, P, P, P, P, P, P, P, I64, P]
    lib.lukv_score_lse.argtypes = [CP, P, P, P, P, P, I64, P]
    lib.lukv_evict_lse.argtypes = [CP, P, P, P, P, I32, P, P, P, P, ctypes.POINTER(I64),
                                   P, P, P, P, P, P, P, P, I64, P]
    F64P = ctypes.POINTER(ctypes.c_double)
    lib.lukv_profile_workspace_bytes.argtypes = [I32, I32, I32, ctypes.POINTER(I64)]
    lib.lukv_profile_curves.argtypes = [I32, I32, I32, P, P, P, P, P]
    lib.lukv_profile_build.argtypes = [I32, I32, I32, P, P, P, P, I32, I32, F64P, P, P, I64, P]
    lib.lukv_budgets_from_profile.argtypes = [I32, I32, F64P, P, ctypes.c_double, I32, P, P, P, P, P]
    lib.lukv_evict_budgets.argtypes = [CP, P, P, P, P, P, P, I64, P, P, P, P, P, P, I64, P]
    lib.lukv_decode_workspace_bytes.argtypes = [CP, ctypes.POINTER(I64)]
    lib.lukv_decode_attention.argtypes = [CP, P, P, P, P, P, P, I64, P]
    lib.lukv_evict_static.argtypes = [CP, P, P, P, I32, P, P, P, P, ctypes.POINTER(I64),
                                      P, P, P, P, P, P, P, P]
    lib.lukv_bench_stream_read.argtypes = [P, I64, P, I32, P]
    lib.lukv_bench_copy.argtypes = [P, P, I64, I32, P]
    lib.lukv_set_stage_events.argtypes = [ctypes.POINTER(ctypes.c_void_p), I32]
    lib.lukv_stage_name.argtypes = [I32]
    lib.lukv_stage_name.restype = ctypes.c_char_p
    for name in EXPORTS + BENCH_EXPORTS:
        if name not in ("lukv_strerror", "lukv_stage_name"):
            getattr(lib, name).restype = ctypes.c_int
    lib.lukv_strerror.argtypes = [ctypes.c_int]
    lib.lukv_strerror.restype = ctypes.c_char_p
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return load_library().lukv_strerror(int(code)).decode()


@dataclasses.dataclass
class Config:
    """Mirror of `lukv_config`; strides are in elements, cu_seqlens is a host sequence."""
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    pool_kernel: int
    n_sink: int
    dtype: int
    cu_seqlens: Sequence[int]
    stride_layer: int
    stride_head: int
    stride_tok: int
    qstride_layer: int
    qstride_head: int
    qstride_tok: int
    softmax_scale: float = 0.0

    def to_c(self):
        """The C struct for this configuration (built once and reused: a Config is not meant to be
        mutated after its first use)."""
        cached = self.__dict__.get("_c")
        if cached is not None:
            return cached
        cu = (ctypes.c_int32 * len(self.cu_seqlens))(*[int(x) for x in self.cu_seqlens])
        c = _CConfig(self.n_layers, self.n_q_heads, self.n_kv_heads, self.head_dim, self.window,
                     self.pool_kernel, self.n_sink, self.dtype, len(self.cu_seqlens) - 1,
                     ctypes.cast(cu, ctypes.POINTER(ctypes.c_int32)), self.stride_layer,
                     self.stride_head, self.stride_tok, self.qstride_layer, self.qstride_head,
                     self.qstride_tok, self.softmax_scale)
        c._keepalive = cu
        self.__dict__["_c"] = c
        return c

    @property
    def n_seqs(self) -> int:
        return len(self.cu_seqlens) - 1

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def n_heads_total(self) -> int:
        return self.n_seqs * self.n_layers * self.n_kv_heads

    @staticmethod
    def for_tensors(q_win: torch.Tensor, k: torch.Tensor, window: int, cu_seqlens: Sequence[int],
                    pool_kernel: int = 7, n_sink: int = 4, softmax_scale: float = 0.0) -> "Config":
        """Config for q_win [NL, H_q, n_seqs*w, d] and k [NL, H_kv, T, d] (last dim contiguous)."""
        assert q_win.dim() == 4 and k.dim() == 4 and q_win.stride(3) == 1 and k.stride(3) == 1
        dt = {torch.bfloat16: LUKV_BF16, torch.float32: LUKV_F32}[k.dtype]
        return Config(k.shape[0], q_win.shape[1], k.shape[1], k.shape[3], window, pool_kernel, n_sink,
                      dt, list(cu_seqlens), k.stride(0), k.stride(1), k.stride(2),
                      q_win.stride(0), q_win.stride(1), q_win.stride(2), softmax_scale)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("lukv: expected a device tensor")
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) or None


def _check(rc: int, where: str) -> None:
    if rc != LUKV_OK:
        raise LukvError(rc, where)


def _host_i64(x: Sequence[int]):
    arr = np.ascontiguousarray(np.asarray(x, dtype=np.int64))
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def lukv_workspace_bytes(cfg: Config, n_grid: int = 0) -> int:
    out = ctypes.c_int64(0)
    _check(load_library().lukv_workspace_bytes(ctypes.byref(cfg.to_c()), n_grid, ctypes.byref(out)),
           "lukv_workspace_bytes")
    return out.value


def lukv_allocate_workspace_bytes(n_problems: int, n_heads: int, n_grid: int) -> int:
    out = ctypes.c_int64(0)
    _check(load_library().lukv_allocate_workspace_bytes(n_problems, n_heads, n_grid, ctypes.byref(out)),
           "lukv_allocate_workspace_bytes")
    return out.value


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Device scratch of at least nbytes (torch's allocator returns >=256-byte aligned blocks)."""
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def lukv_score(cfg: Config, q_win, k, pooled, ws, stream=None) -> None:
    _check(load_library().lukv_score(ctypes.byref(cfg.to_c()), _ptr(q_win), _ptr(k), _ptr(pooled),
                                     _ptr(ws), ws.numel(), _stream(stream)), "lukv_score")


def lukv_score_lse(cfg: Config, q_win, k, lse, pooled, ws, stream=None) -> None:
    _check(load_library().lukv_score_lse(ctypes.byref(cfg.to_c()), _ptr(q_win), _ptr(k), _ptr(lse),
                                         _ptr(pooled), _ptr(ws), ws.numel(), _stream(stream)),
           "lukv_score_lse")


def lukv_allocate(n_problems: int, n_heads: int, n_grid: int, curves, knots, b_min, b_max,
                  B_total: Sequence[int], budgets, offsets, status, ws, stream=None) -> None:
    keep, Bp = _host_i64(B_total)
    _check(load_library().lukv_allocate(n_problems, n_heads, n_grid, _ptr(curves), _ptr(knots),
                                        _ptr(b_min), _ptr(b_max), Bp, _ptr(budgets), _ptr(offsets),
                                        _ptr(status), _ptr(ws), ws.numel(), _stream(stream)),
           "lukv_allocate")


def lukv_allocate_topk(cfg: Config, pooled, B_total: Sequence[int], b_floor: int, budgets, offsets, status,
                       ws, stream=None) -> None:
    keep, Bp = _host_i64(B_total)
    _check(load_library().lukv_allocate_topk(ctypes.byref(cfg.to_c()), _ptr(pooled), Bp, int(b_floor),
                                             _ptr(budgets), _ptr(offsets), _ptr(status), _ptr(ws),
                                             ws.numel(), _stream(stream)), "lukv_allocate_topk")


def lukv_select_compact(cfg: Config, pooled, budgets, offsets, k, v, out_rows: int, kept_idx, k_out,
                        v_out, status, ws, stream=None) -> None:
    _check(load_library().lukv_select_compact(ctypes.byref(cfg.to_c()), _ptr(pooled), _ptr(budgets),
                                              _ptr(offsets), _ptr(k), _ptr(v), int(out_rows),
                                              _ptr(kept_idx),
                                              _ptr(k_out), _ptr(v_out), _ptr(status), _ptr(ws),
                                              ws.numel(), _stream(stream)), "lukv_select_compact")


def lukv_evict(cfg: Config, q_win, k, v, n_grid: int, curves, knots, b_min, b_max,
               B_total: Sequence[int], budgets, offsets, kept_idx, k_out, v_out, pooled, status,
               ws, stream=None) -> None:
    keep, Bp = _host_i64(B_total)
    _check(load_library().lukv_evict(ctypes.byref(cfg.to_c()), _ptr(q_win), _ptr(k), _ptr(v), n_grid,
                                     _ptr(curves), _ptr(knots), _ptr(b_min), _ptr(b_max), Bp,
                                     _ptr(budgets), _ptr(offsets), _ptr(kept_idx), _ptr(k_out),
                                     _ptr(v_out), _ptr(pooled), _ptr(status), _ptr(ws), ws.numel(),
                                     _stream(stream)), "lukv_evict")


def lukv_evict_static(cfg: Config, q_win, k, v, n_grid: int, curves, knots, b_min, b_max,
                      B_total: Sequence[int], budgets, offsets, kept_idx, k_out, v_out, pooled, status,
                      stream=None) -> None:
    keep, Bp = _host_i64(B_total)
    _check(load_library().lukv_evict_static(ctypes.byref(cfg.to_c()), _ptr(q_win), _ptr(k), _ptr(v), n_grid,
                                            _ptr(curves), _ptr(knots), _ptr(b_min), _ptr(b_max), Bp,
                                            _ptr(budgets), _ptr(offsets), _ptr(kept_idx), _ptr(k_out),
                                            _ptr(v_out), _ptr(pooled), _ptr(status), _stream(stream)),
           "lukv_evict_static")


def lukv_evict_lse(cfg: Config, q_win, k, v, lse, n_grid: int, curves, knots, b_min, b_max,
                   B_total: Sequence[int], budgets, offsets, kept_idx, k_out, v_out, pooled, status,
                   ws, stream=None) -> None:
    keep, Bp = _host_i64(B_total)
    _check(load_library().lukv_evict_lse(ctypes.byref(cfg.to_c()), _ptr(q_win), _ptr(k), _ptr(v),
                                         _ptr(lse), n_grid, _ptr(curves), _ptr(knots), _ptr(b_min),
                                         _ptr(b_max), Bp, _ptr(budgets), _ptr(offsets),
                                         _ptr(kept_idx), _ptr(k_out), _ptr(v_out), _ptr(pooled),
                                         _ptr(status), _ptr(ws), ws.numel(), _stream(stream)),
           "lukv_evict_lse")


def _host_f64(x: Sequence[float]):
    arr = np.ascontiguousarray(np.asarray(x, dtype=np.float64))
    return arr, arr.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def lukv_profile_workspace_bytes(n_queries: int, n_heads: int, n_grid: int) -> int:
    out = ctypes.c_int64(0)
    _check(load_library().lukv_profile_workspace_bytes(n_queries, n_heads, n_grid, ctypes.byref(out)),
           "lukv_profile_workspace_bytes")
    return out.value


def lukv_profile_curves(n_curves: int, T: int, n_grid: int, importance, scores, knots, curves,
                        stream=None) -> None:
    _check(load_library().lukv_profile_curves(n_curves, T, n_grid, _ptr(importance), _ptr(scores), _ptr(knots),
                                              _ptr(curves), _stream(stream)), "lukv_profile_curves")


def lukv_profile_build(n_queries: int, n_heads: int, n_grid: int, curves, knots, b_min, b_max, L: int,
                       rho: Sequence[float], phi, ws, stream=None) -> None:
    keep, rp = _host_f64(rho)
    _check(load_library().lukv_profile_build(n_queries, n_heads, n_grid, _ptr(curves), _ptr(knots),
                                             _ptr(b_min), _ptr(b_max), int(L), len(keep), rp, _ptr(phi),
                                             _ptr(ws), ws.numel(), _stream(stream)), "lukv_profile_build")


def lukv_budgets_from_profile(n_heads: int, rho: Sequence[float], phi, sigma_target: float, L: int,
                              b_min, b_max, budgets, offsets, stream=None) -> None:
    keep, rp = _host_f64(rho)
    _check(load_library().lukv_budgets_from_profile(n_heads, len(keep), rp, _ptr(phi), float(sigma_target),
                                                    int(L), _ptr(b_min), _ptr(b_max), _ptr(budgets),
                                                    _ptr(offsets), _stream(stream)),
           "lukv_budgets_from_profile")


def lukv_evict_budgets(cfg: Config, q_win, k, v, lse, budgets, offsets, out_rows: int, kept_idx, k_out,
                       v_out, pooled, status, ws, stream=None) -> None:
    _check(load_library().lukv_evict_budgets(ctypes.byref(cfg.to_c()), _ptr(q_win), _ptr(k), _ptr(v),
                                             _ptr(lse), _ptr(budgets), _ptr(offsets), int(out_rows),
                                             _ptr(kept_idx), _ptr(k_out), _ptr(v_out), _ptr(pooled),
                                             _ptr(status), _ptr(ws), ws.numel(), _stream(stream)),
           "lukv_evict_budgets")


def lukv_decode_workspace_bytes(cfg: Config) -> int:
    out = ctypes.c_int64(0)
    _check(load_library().lukv_decode_workspace_bytes(ctypes.byref(cfg.to_c()), ctypes.byref(out)),
           "lukv_decode_workspace_bytes")
    return out.value


def lukv_decode_attention(cfg: Config, q_dec, k_packed, v_packed, offsets, out, ws, stream=None) -> None:
    _check(load_library().lukv_decode_attention(ctypes.byref(cfg.to_c()), _ptr(q_dec), _ptr(k_packed),
                                                _ptr(v_packed), _ptr(offsets), _ptr(out), _ptr(ws),
                                                ws.numel(), _stream(stream)), "lukv_decode_attention")


def lukv_set_stage_events(events) -> None:
    """events: a ctypes array of hipEvent_t handles (kept alive by the caller), or None to stop."""
    if events is None:
        _check(load_library().lukv_set_stage_events(None, 0), "lukv_set_stage_events")
    else:
        _check(load_library().lukv_set_stage_events(events, len(events)), "lukv_set_stage_events")


def lukv_stage_name(stage: int) -> str:
    return load_library().lukv_stage_name(int(stage)).decode()


def lukv_bench_stream_read(src, nbytes: int, sink, blocks: int, stream=None) -> None:
    _check(load_library().lukv_bench_stream_read(_ptr(src), int(nbytes), _ptr(sink), int(blocks), _stream(stream)),
           "lukv_bench_stream_read")


def lukv_bench_copy(src, dst, nbytes: int, blocks: int, stream=None) -> None:
    _check(load_library().lukv_bench_copy(_ptr(src), _ptr(dst), int(nbytes), int(blocks), _stream(stream)),
           "lukv_bench_copy")
