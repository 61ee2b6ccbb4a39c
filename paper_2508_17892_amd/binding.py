"""Thin ctypes binding of libilre's C ABI (include/ilre.h).

Argument marshalling only: every step of the recall path runs in the library's HIP kernels.
PyTorch is used for device memory and the current stream, nothing else.  There is no fallback:
if the shared library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libilre.so")

ILRE_OK, ILRE_EINVAL, ILRE_EUNSUPPORTED, ILRE_ENOMEM, ILRE_EHIP = range(5)
ILRE_F32, ILRE_BF16 = 0, 1
ILRE_SCORE_SUM, ILRE_SCORE_MAX = 0, 1
ILRE_FLAG_EXACT_ROW_MAX = 1
ILRE_ROPE_HALF, ILRE_ROPE_INTERLEAVED = 0, 1
ILRE_MAX_BUDGET = 8192
ILRE_MAX_POOL_KERNEL = 2047
ILRE_MAX_POOL_KERNELS = 64
ILRE_MAX_MAX_KERNEL = 1024
ILRE_MAX_AVG_KERNEL = 1024

ILRE_STATIC_SCRATCH_BYTES = 4 << 20

EXPORTS = ("ilre_workspace_bytes", "ilre_recall", "ilre_row_stats", "ilre_row_stats_static", "ilre_col_scores", "ilre_select",
           "ilre_select_max_avg", "ilre_recall_max_avg", "ilre_workspace_bytes_max_avg", "ilre_rerope_keys",
           "ilre_gather_ids", "ilre_probe_mfma_ceiling", "ilre_probe_describe", "ilre_last_error")


class IlreOpts(ctypes.Structure):
    _fields_ = [
        ("struct_size", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("n_pool_kernels", ctypes.c_int32),
        ("score_mode", ctypes.c_int32),
        ("scale", ctypes.c_float),
        ("flags", ctypes.c_int32),
        ("k_stride_head", ctypes.c_int64),
        ("k_stride_token", ctypes.c_int64),
        ("q_stride_head", ctypes.c_int64),
        ("q_stride_token", ctypes.c_int64),
        ("workspace", ctypes.c_void_p),
        ("workspace_bytes", ctypes.c_size_t),
        ("stream", ctypes.c_void_p),
        ("sink", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
    ]


class IlreError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ilre status {status}: {message}")
        self.status = status


_lib = None


def load() -> ctypes.CDLL:
    """Load libilre.so (built in-tree by paper_2508_17892_amd.build); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2508_17892_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
        po = ctypes.POINTER(IlreOpts)
        lib.ilre_workspace_bytes.restype = ctypes.c_int
        lib.ilre_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i32, i32, ctypes.POINTER(ctypes.c_size_t)]
        lib.ilre_recall.restype = ctypes.c_int
        lib.ilre_recall.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, ctypes.POINTER(i32), vp, vp, po]
        lib.ilre_row_stats.restype = ctypes.c_int
        lib.ilre_row_stats.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, po]
        lib.ilre_row_stats_static.restype = ctypes.c_int
        lib.ilre_row_stats_static.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, po]
        lib.ilre_col_scores.restype = ctypes.c_int
        lib.ilre_col_scores.argtypes = [vp, vp, i64, i32, i32, i32, i32, vp, vp, vp, po]
        lib.ilre_select.restype = ctypes.c_int
        lib.ilre_select.argtypes = [vp, i64, i32, ctypes.POINTER(i32), vp, po]
        pi = ctypes.POINTER(i32)
        lib.ilre_select_max_avg.restype = ctypes.c_int
        lib.ilre_select_max_avg.argtypes = [vp, i64, i32, i32, pi, i32, pi, i32, vp, vp, po]
        lib.ilre_recall_max_avg.restype = ctypes.c_int
        lib.ilre_recall_max_avg.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, i32, pi, i32, pi, i32, vp, vp, vp, po]
        lib.ilre_workspace_bytes_max_avg.restype = ctypes.c_int
        lib.ilre_workspace_bytes_max_avg.argtypes = [i64, i32, i32, i32, i32, i32, pi, i32, i32, i32,
                                                     ctypes.POINTER(ctypes.c_size_t)]
        lib.ilre_rerope_keys.restype = ctypes.c_int
        lib.ilre_rerope_keys.argtypes = [vp, vp, i64, i32, i32, i32, i32, ctypes.c_double, ctypes.POINTER(ctypes.c_double),
                                         i32, po]
        lib.ilre_gather_ids.restype = ctypes.c_int
        lib.ilre_gather_ids.argtypes = [vp, i64, vp, i32, vp, po]
        lib.ilre_probe_mfma_ceiling.restype = ctypes.c_int
        lib.ilre_probe_mfma_ceiling.argtypes = [i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double), po]
        lib.ilre_probe_describe.restype = ctypes.c_char_p
        lib.ilre_probe_describe.argtypes = [i32]
        lib.ilre_last_error.restype = ctypes.c_char_p
        lib.ilre_last_error.argtypes = []
        _lib = lib
    return _lib


def to_device(arr, device="cuda") -> torch.Tensor:
    """Host array (float32, or uint16 holding bf16 bit patterns) -> device tensor of the same bits."""
    import numpy as np
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def ilre_last_error() -> str:
    return load().ilre_last_error().decode()


def _check(rc: int) -> None:
    if rc != ILRE_OK:
        raise IlreError(rc, ilre_last_error())


def ilre_workspace_bytes(L: int, Lq: int, Hq: int, Hkv: int, d: int, n_pool_kernels: int, dtype: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().ilre_workspace_bytes(L, Lq, Hq, Hkv, d, n_pool_kernels, dtype, ctypes.byref(out)))
    return int(out.value)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return ILRE_BF16
    if t.dtype == torch.float32:
        return ILRE_F32
    raise TypeError(f"unsupported element type {t.dtype}")


def _qk_meta(q: torch.Tensor, k: torch.Tensor):
    if q.dim() != 3 or k.dim() != 3:
        raise ValueError("q is [Hq, Lq, d], k_cache is [Hkv, L, d] (any strides with the last dim contiguous)")
    if q.dtype != k.dtype:
        raise TypeError("q and k_cache must share an element type")
    if not (q.is_cuda and k.is_cuda):
        raise ValueError("q and k_cache must be device tensors")
    if q.stride(2) != 1 or k.stride(2) != 1:
        raise ValueError("the head dimension must be contiguous")
    Hq, Lq, d = q.shape
    Hkv, L, d2 = k.shape
    if d != d2:
        raise ValueError("head dims differ")
    return L, Lq, Hq, Hkv, d


def _opts(dtype: int, n_pool_kernels: int, scale: float, score_mode: int, workspace: Optional[torch.Tensor],
          q: Optional[torch.Tensor] = None, k: Optional[torch.Tensor] = None, flags: int = 0, sink: int = 0) -> IlreOpts:
    o = IlreOpts()
    o.struct_size = ctypes.sizeof(IlreOpts)
    o.dtype = dtype
    o.n_pool_kernels = n_pool_kernels
    o.score_mode = score_mode
    o.scale = float(scale)
    o.flags = int(flags)
    o.sink = int(sink)
    if q is not None:
        o.q_stride_head, o.q_stride_token = q.stride(0), q.stride(1)
    if k is not None:
        o.k_stride_head, o.k_stride_token = k.stride(0), k.stride(1)
    if workspace is not None:
        o.workspace = workspace.data_ptr()
        o.workspace_bytes = workspace.numel() * workspace.element_size()
    o.stream = torch.cuda.current_stream().cuda_stream
    return o


def alloc_workspace(L: int, Lq: int, Hq: int, Hkv: int, d: int, n_pool_kernels: int, dtype: int,
                    device="cuda") -> torch.Tensor:
    return torch.empty(ilre_workspace_bytes(L, Lq, Hq, Hkv, d, n_pool_kernels, dtype), dtype=torch.uint8, device=device)


def _kernel_array(pool_kernels: Sequence[int]):
    arr = (ctypes.c_int32 * len(pool_kernels))(*[int(w) for w in pool_kernels])
    return arr


def ilre_recall(q: torch.Tensor, k_cache: torch.Tensor, budget: int, pool_kernels: Sequence[int], *,
                scale: float = 0.0, score_mode: int = ILRE_SCORE_SUM, flags: int = 0, sink: int = 0,
                workspace: Optional[torch.Tensor] = None,
                out_idx: Optional[torch.Tensor] = None, out_scores: Optional[torch.Tensor] = None
                ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Whole path; returns (out_idx int32[sink + min(budget, L - sink)] ascending, out_scores float32[L])."""
    L, Lq, Hq, Hkv, d = _qk_meta(q, k_cache)
    dt = _dtype_code(q)
    n = len(pool_kernels)
    if workspace is None:
        workspace = alloc_workspace(L, Lq, Hq, Hkv, d, n, dt, q.device)
    if out_idx is None:
        out_idx = torch.empty(int(sink) + min(int(budget), L - int(sink)), dtype=torch.int32, device=q.device)
    if out_scores is None:
        out_scores = torch.empty(L, dtype=torch.float32, device=q.device)
    o = _opts(dt, n, scale, score_mode, workspace, q, k_cache, flags, sink)
    _check(load().ilre_recall(q.data_ptr(), k_cache.data_ptr(), L, Lq, Hq, Hkv, d, int(budget), _kernel_array(pool_kernels),
                              out_idx.data_ptr(), out_scores.data_ptr(), ctypes.byref(o)))
    return out_idx, out_scores


def ilre_row_stats(q: torch.Tensor, k_cache: torch.Tensor, *, scale: float = 0.0, flags: int = 0,
                   workspace: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Softmax row reference (the row maximum with ILRE_FLAG_EXACT_ROW_MAX) and sum of exponentials
    against it for every row r = h*Lq + i (float32[Hq*Lq] each)."""
    L, Lq, Hq, Hkv, d = _qk_meta(q, k_cache)
    dt = _dtype_code(q)
    if workspace is None:
        workspace = alloc_workspace(L, Lq, Hq, Hkv, d, 0, dt, q.device)
    row_max = torch.empty(Hq * Lq, dtype=torch.float32, device=q.device)
    row_sumexp = torch.empty(Hq * Lq, dtype=torch.float32, device=q.device)
    o = _opts(dt, 0, scale, ILRE_SCORE_SUM, workspace, q, k_cache, flags)
    _check(load().ilre_row_stats(q.data_ptr(), k_cache.data_ptr(), L, Lq, Hq, Hkv, d, row_max.data_ptr(),
                                 row_sumexp.data_ptr(), ctypes.byref(o)))
    return row_max, row_sumexp


def ilre_row_stats_static(q: torch.Tensor, k_cache: torch.Tensor, row_ref: torch.Tensor, row_sumexp: torch.Tensor, *,
                          scale: float = 0.0, flags: int = 0) -> None:
    """ilre_row_stats into the caller's float32[Hq*Lq] outputs, with the library's built-in scratch buffer:
    this wrapper and the call beneath it allocate nothing."""
    L, Lq, Hq, Hkv, d = _qk_meta(q, k_cache)
    for t in (row_ref, row_sumexp):
        if t.dtype != torch.float32 or t.numel() != Hq * Lq or not t.is_contiguous() or not t.is_cuda:
            raise ValueError("row_ref and row_sumexp must be contiguous float32 device vectors of Hq*Lq entries")
    o = _opts(_dtype_code(q), 0, scale, ILRE_SCORE_SUM, None, q, k_cache, flags)
    _check(load().ilre_row_stats_static(q.data_ptr(), k_cache.data_ptr(), L, Lq, Hq, Hkv, d, row_ref.data_ptr(),
                                        row_sumexp.data_ptr(), ctypes.byref(o)))


def ilre_col_scores(q: torch.Tensor, k_cache: torch.Tensor, row_max: torch.Tensor, row_sumexp: torch.Tensor, *,
                    scale: float = 0.0, score_mode: int = ILRE_SCORE_SUM,
                    workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Per-token score (float32[L]) from the row statistics of ilre_row_stats."""
    L, Lq, Hq, Hkv, d = _qk_meta(q, k_cache)
    dt = _dtype_code(q)
    if row_max.numel() != Hq * Lq or row_sumexp.numel() != Hq * Lq:
        raise ValueError("row statistics must have Hq*Lq entries")
    if row_max.dtype != torch.float32 or row_sumexp.dtype != torch.float32:
        raise TypeError("row statistics must be float32")
    if workspace is None:
        workspace = alloc_workspace(L, Lq, Hq, Hkv, d, 0, dt, q.device)
    out = torch.empty(L, dtype=torch.float32, device=q.device)
    o = _opts(dt, 0, scale, score_mode, workspace, q, k_cache)
    _check(load().ilre_col_scores(q.data_ptr(), k_cache.data_ptr(), L, Lq, Hq, Hkv, d, row_max.contiguous().data_ptr(),
                                  row_sumexp.contiguous().data_ptr(), out.data_ptr(), ctypes.byref(o)))
    return out


def ilre_select(scores: torch.Tensor, budget: int, pool_kernels: Sequence[int], *, sink: int = 0,
                workspace: Optional[torch.Tensor] = None, out_idx: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Algorithm 1 on a float32 score vector; returns int32[sink + min(budget, L - sink)] ascending."""
    if scores.dtype != torch.float32 or scores.dim() != 1 or not scores.is_contiguous() or not scores.is_cuda:
        raise ValueError("scores must be a contiguous float32 device vector")
    L = scores.numel()
    n = len(pool_kernels)
    if workspace is None:
        # the selection region is the tail of the full workspace; sized on its own here
        workspace = alloc_workspace(L, 1, 1, 1, 128, n, ILRE_F32, scores.device)
    if out_idx is None:
        out_idx = torch.empty(int(sink) + min(int(budget), L - int(sink)), dtype=torch.int32, device=scores.device)
    o = _opts(ILRE_F32, n, 0.0, ILRE_SCORE_SUM, workspace, sink=sink)
    _check(load().ilre_select(scores.data_ptr(), L, int(budget), _kernel_array(pool_kernels), out_idx.data_ptr(),
                              ctypes.byref(o)))
    return out_idx


def ilre_workspace_bytes_max_avg(L: int, Lq: int, Hq: int, Hkv: int, d: int, sink: int, max_kernels: Sequence[int],
                                 n_avg: int, dtype: int) -> int:
    out = ctypes.c_size_t(0)
    _check(load().ilre_workspace_bytes_max_avg(L, Lq, Hq, Hkv, d, int(sink), _kernel_array(max_kernels), len(max_kernels),
                                               int(n_avg), dtype, ctypes.byref(out)))
    return int(out.value)


def alloc_workspace_max_avg(L: int, Lq: int, Hq: int, Hkv: int, d: int, sink: int, max_kernels: Sequence[int], n_avg: int,
                            dtype: int, device="cuda") -> torch.Tensor:
    return torch.empty(ilre_workspace_bytes_max_avg(L, Lq, Hq, Hkv, d, sink, max_kernels, n_avg, dtype), dtype=torch.uint8,
                       device=device)


def ilre_select_max_avg(scores: torch.Tensor, budget: int, max_kernels: Sequence[int], avg_kernels: Sequence[int],
                        sink: int = 0, *, workspace: Optional[torch.Tensor] = None, out_idx: Optional[torch.Tensor] = None,
                        out_count: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Algorithm 1 as printed on a float32 score vector; returns (out_idx int32[sink + min(budget, L - sink)] with
    -1 in unused slots, out_count int32[1])."""
    if scores.dtype != torch.float32 or scores.dim() != 1 or not scores.is_contiguous() or not scores.is_cuda:
        raise ValueError("scores must be a contiguous float32 device vector")
    L = scores.numel()
    if workspace is None:
        workspace = alloc_workspace_max_avg(L, 1, 1, 1, 128, sink, max_kernels, len(avg_kernels), ILRE_F32, scores.device)
    if out_idx is None:
        out_idx = torch.empty(int(sink) + min(int(budget), L - int(sink)), dtype=torch.int32, device=scores.device)
    if out_count is None:
        out_count = torch.empty(1, dtype=torch.int32, device=scores.device)
    o = _opts(ILRE_F32, 0, 0.0, ILRE_SCORE_SUM, workspace)
    _check(load().ilre_select_max_avg(scores.data_ptr(), L, int(sink), int(budget), _kernel_array(max_kernels),
                                      len(max_kernels), _kernel_array(avg_kernels), len(avg_kernels), out_idx.data_ptr(),
                                      out_count.data_ptr(), ctypes.byref(o)))
    return out_idx, out_count


def ilre_recall_max_avg(q: torch.Tensor, k_cache: torch.Tensor, budget: int, max_kernels: Sequence[int],
                        avg_kernels: Sequence[int], sink: int = 0, *, scale: float = 0.0,
                        score_mode: int = ILRE_SCORE_SUM, flags: int = 0, workspace: Optional[torch.Tensor] = None,
                        out_idx: Optional[torch.Tensor] = None, out_count: Optional[torch.Tensor] = None,
                        out_scores: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor]:
    """Whole path with Algorithm 1 as printed; returns (out_idx, out_count, out_scores float32[L])."""
    L, Lq, Hq, Hkv, d = _qk_meta(q, k_cache)
    dt = _dtype_code(q)
    if workspace is None:
        workspace = alloc_workspace_max_avg(L, Lq, Hq, Hkv, d, sink, max_kernels, len(avg_kernels), dt, q.device)
    if out_idx is None:
        out_idx = torch.empty(int(sink) + min(int(budget), L - int(sink)), dtype=torch.int32, device=q.device)
    if out_count is None:
        out_count = torch.empty(1, dtype=torch.int32, device=q.device)
    if out_scores is None:
        out_scores = torch.empty(L, dtype=torch.float32, device=q.device)
    o = _opts(dt, 0, scale, score_mode, workspace, q, k_cache, flags)
    _check(load().ilre_recall_max_avg(q.data_ptr(), k_cache.data_ptr(), L, Lq, Hq, Hkv, d, int(sink), int(budget),
                                      _kernel_array(max_kernels), len(max_kernels), _kernel_array(avg_kernels),
                                      len(avg_kernels), out_idx.data_ptr(), out_count.data_ptr(), out_scores.data_ptr(),
                                      ctypes.byref(o)))
    return out_idx, out_count, out_scores


def ilre_rerope_keys(k_cache: torch.Tensor, chunk_tokens: int, first_extra: int = 0, *, rope_base: float = 10000.0,
                     inv_freq: Optional[Sequence[float]] = None, pairing: int = ILRE_ROPE_HALF,
                     out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """DCA re-RoPE of a key cache [Hkv, L, d]; `out` may be k_cache itself (in place) and must share its strides."""
    if k_cache.dim() != 3 or not k_cache.is_cuda or k_cache.stride(2) != 1:
        raise ValueError("k_cache is a device tensor [Hkv, L, d] with the head dimension contiguous")
    Hkv, L, d = k_cache.shape
    if out is None:
        out = torch.empty_strided(k_cache.shape, k_cache.stride(), dtype=k_cache.dtype, device=k_cache.device)
    if out.shape != k_cache.shape or out.stride() != k_cache.stride() or out.dtype != k_cache.dtype:
        raise ValueError("out must have the shape, strides and element type of k_cache")
    o = _opts(_dtype_code(k_cache), 0, 0.0, ILRE_SCORE_SUM, None, None, k_cache)
    freq = None
    if inv_freq is not None:
        if len(inv_freq) != d // 2:
            raise ValueError("inv_freq must have d/2 entries")
        freq = (ctypes.c_double * (d // 2))(*[float(x) for x in inv_freq])
    _check(load().ilre_rerope_keys(k_cache.data_ptr(), out.data_ptr(), L, Hkv, d, int(chunk_tokens), int(first_extra),
                                   float(rope_base), freq, int(pairing), ctypes.byref(o)))
    return out


def ilre_gather_ids(input_ids: torch.Tensor, idx: torch.Tensor, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """C[I]: the input IDs (int32 device vector) of an index list; -1 where the list holds -1."""
    if input_ids.dtype != torch.int32 or idx.dtype != torch.int32 or not input_ids.is_contiguous() or not idx.is_contiguous():
        raise ValueError("input_ids and idx must be contiguous int32 device vectors")
    if out is None:
        out = torch.empty_like(idx)
    o = _opts(ILRE_F32, 0, 0.0, ILRE_SCORE_SUM, None)
    _check(load().ilre_gather_ids(input_ids.data_ptr(), input_ids.numel(), idx.data_ptr(), idx.numel(), out.data_ptr(),
                                  ctypes.byref(o)))
    return out


ILRE_PROBE_OPERAND_BYTES = 65536
ILRE_PROBE_OUT_BYTES = (1 << 20) + 4096


def ilre_probe_describe(variant: int) -> Optional[str]:
    text = load().ilre_probe_describe(int(variant))
    return text.decode() if text else None


def ilre_probe_mfma_ceiling(variant: int, iters: int, operands: torch.Tensor, out: torch.Tensor) -> float:
    """Enqueue one launch of a register-only MFMA loop (measurement aid); returns the MFMA flops of the launch.
    `out` (uint8, ILRE_PROBE_OUT_BYTES) receives, from byte 1 MiB on, per workgroup (shader cycles, 100 MHz ticks)."""
    if operands.numel() * operands.element_size() < ILRE_PROBE_OPERAND_BYTES or not operands.is_cuda:
        raise ValueError("operands must hold ILRE_PROBE_OPERAND_BYTES on the device")
    if out.numel() * out.element_size() < ILRE_PROBE_OUT_BYTES or not out.is_cuda:
        raise ValueError("out must hold ILRE_PROBE_OUT_BYTES on the device")
    o = _opts(ILRE_BF16, 0, 0.0, ILRE_SCORE_SUM, None)
    flops = ctypes.c_double(0.0)
    _check(load().ilre_probe_mfma_ceiling(int(variant), int(iters), operands.data_ptr(), out.data_ptr(), ctypes.byref(flops),
                                          ctypes.byref(o)))
    return float(flops.value)
