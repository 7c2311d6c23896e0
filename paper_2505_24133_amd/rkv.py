"""ctypes binding of librkv.so: the same entry points as ``include/rkv.h``, taking torch
tensors that live on the GPU.  This layer only marshals arguments (pointers, sizes, the
current HIP stream) and allocates outputs / scratch with torch; every step of the
compression runs in the library's HIP kernels.  There is no CPU fallback: if the
library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librkv.so")

RKV_OK = 0
RKV_NOT_TRIGGERED = 1
RKV_ERR_NULL = -1
RKV_ERR_SHAPE = -2
RKV_ERR_UNSUPPORTED = -3
RKV_ERR_WORKSPACE = -4
RKV_ERR_PARAM = -5
RKV_ERR_HIP = -6
RKV_FLAG_SKIP_SATURATED = 1
RKV_FLAG_POOL_AFTER_MEAN = 2
RKV_FLAG_SHARED_SELECTION = 4
RKV_FLAG_GQA_SOFTMAX_THEN_MAX = 8
RKV_FLAG_GQA_SOFTMAX_THEN_MEAN = 16
RKV_FLAG_RECENCY_TRANSPOSED = 32
RKV_FLAG_TRIANGULAR_SCAN = 64
RKV_STATIC_SCRATCH_BYTES = 32 << 20
RKV_PROBE_OPERAND_BYTES = 64 << 10
RKV_PROBE_SINK_BYTES = 1 << 20


class RkvParams(ctypes.Structure):
    """Mirror of ``rkv_params``."""
    _fields_ = [
        ("num_problems", ctypes.c_int32), ("kv_heads", ctypes.c_int32), ("q_heads", ctypes.c_int32),
        ("n_tokens", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("alpha", ctypes.c_int32),
        ("budget", ctypes.c_int32), ("pool_w", ctypes.c_int32), ("beta", ctypes.c_int32),
        ("sim_threshold", ctypes.c_float), ("lam", ctypes.c_float), ("eps", ctypes.c_float),
        ("flags", ctypes.c_uint32),
        ("k_stride_problem", ctypes.c_int64), ("k_stride_head", ctypes.c_int64), ("k_stride_token", ctypes.c_int64),
        ("v_stride_problem", ctypes.c_int64), ("v_stride_head", ctypes.c_int64), ("v_stride_token", ctypes.c_int64),
        ("o_stride_problem", ctypes.c_int64), ("o_stride_head", ctypes.c_int64), ("o_stride_token", ctypes.c_int64),
        ("q_stride_problem", ctypes.c_int64), ("q_stride_head", ctypes.c_int64), ("q_stride_token", ctypes.c_int64),
        ("page_size", ctypes.c_int32), ("table_stride", ctypes.c_int32), ("block_table", ctypes.c_void_p),
        ("k_stride_page", ctypes.c_int64), ("v_stride_page", ctypes.c_int64),
    ]


class RkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def load_library() -> ctypes.CDLL:
    """Load librkv.so (built in-tree by ``paper_2505_24133_amd.build``); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2505_24133_amd.build`")
    lib = ctypes.CDLL(LIB_PATH)
    P, V, S = ctypes.POINTER(RkvParams), ctypes.c_void_p, ctypes.c_size_t
    lib.rkv_workspace_size.argtypes = [P, ctypes.POINTER(S)]
    lib.rkv_score_importance.argtypes = [P, V, V, V, V, S, V]
    lib.rkv_score_redundancy.argtypes = [P, V, V, V, V, S, V]
    lib.rkv_select_topk.argtypes = [P, V, V, V, V, V, S, V]
    lib.rkv_compact.argtypes = [P, V, V, V, V, V, V]
    lib.rkv_compress.argtypes = [P, V, V, V, V, V, V, V, V, S, V]
    lib.rkv_compress_static.argtypes = [P, V, V, V, V, V, V, V, V]
    lib.rkv_compress_events.argtypes = [P, V, V, V, V, V, V, V, V, S, V, ctypes.POINTER(ctypes.c_void_p)]
    lib.rkv_compact_inplace.argtypes = [P, V, V, V, V]
    lib.rkv_compress_inplace.argtypes = [P, V, V, V, V, V, V, S, V]
    lib.rkv_should_compress.argtypes = [P, ctypes.c_int32]
    lib.rkv_cache_append.argtypes = [P, V, V, V, V, V, V, ctypes.c_int32, ctypes.c_int32, V]
    lib.rkv_probe_mfma.argtypes = [V, V, ctypes.c_int, V, ctypes.POINTER(ctypes.c_int64)]
    for name in ("rkv_workspace_size", "rkv_score_importance", "rkv_score_redundancy", "rkv_select_topk",
                 "rkv_compact", "rkv_compress", "rkv_compress_events", "rkv_compress_static", "rkv_should_compress", "rkv_cache_append",
                 "rkv_compact_inplace", "rkv_compress_inplace", "rkv_probe_mfma"):
        getattr(lib, name).restype = ctypes.c_int
    lib.rkv_status_string.argtypes = [ctypes.c_int]
    lib.rkv_status_string.restype = ctypes.c_char_p
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().rkv_status_string(int(status)).decode()


@dataclass
class Shape:
    num_problems: int
    kv_heads: int
    q_heads: int
    n_tokens: int
    budget: int
    alpha: int = 8
    head_dim: int = 128
    pool_w: int = 4
    beta: int = 1
    sim_threshold: float = 0.5
    lam: float = 0.1
    eps: float = 1e-8
    flags: int = 0
    # paged caches: k and v are page pools [num_pages, kv_heads, page_size, d] and block_table is a
    # contiguous int32 GPU tensor [num_problems, table_stride] of page indices
    page_size: int = 0
    block_table: Optional[torch.Tensor] = field(default=None, compare=False, repr=False)

    def params(self, k: Optional[torch.Tensor] = None, v: Optional[torch.Tensor] = None,
               out: Optional[torch.Tensor] = None, q: Optional[torch.Tensor] = None) -> RkvParams:
        p = RkvParams(self.num_problems, self.kv_heads, self.q_heads, self.n_tokens, self.head_dim, self.alpha,
                      self.budget, self.pool_w, self.beta, self.sim_threshold, self.lam, self.eps, self.flags,
                      0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, None, 0, 0)
        if q is not None and not q.is_contiguous():
            p.q_stride_problem, p.q_stride_head, p.q_stride_token = q.stride(0), q.stride(1), q.stride(2)
        if self.page_size:
            bt = self.block_table
            if bt is None or bt.dtype != torch.int32 or not bt.is_cuda or not bt.is_contiguous() or bt.dim() != 2 \
                    or bt.shape[0] != self.num_problems:
                raise ValueError("paged caches need block_table: contiguous int32 GPU tensor [num_problems, entries]")
            p.page_size, p.table_stride, p.block_table = self.page_size, bt.shape[1], bt.data_ptr()
            d = self.head_dim
            natural = (self.kv_heads * self.page_size * d, self.page_size * d, d)
            for name, t in (("k", k), ("v", v)):
                sp, sh, st = natural if t is None else (t.stride(0), t.stride(1), t.stride(2))
                setattr(p, f"{name}_stride_page", sp)
                setattr(p, f"{name}_stride_head", sh)
                setattr(p, f"{name}_stride_token", st)
            if out is not None and not out.is_contiguous():
                p.o_stride_problem, p.o_stride_head, p.o_stride_token = out.stride(0), out.stride(1), out.stride(2)
            return p
        if k is not None:
            p.k_stride_problem, p.k_stride_head, p.k_stride_token = k.stride(0), k.stride(1), k.stride(2)
        if v is not None:
            p.v_stride_problem, p.v_stride_head, p.v_stride_token = v.stride(0), v.stride(1), v.stride(2)
        if out is not None and not out.is_contiguous():
            p.o_stride_problem, p.o_stride_head, p.o_stride_token = out.stride(0), out.stride(1), out.stride(2)
        return p

    @property
    def n_cand(self) -> int:
        return self.n_tokens - self.alpha


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _need_gpu(*tensors: torch.Tensor) -> None:
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise RuntimeError("librkv works on GPU tensors only; there is no CPU path")


def _check_kv(shape: Shape, t: torch.Tensor, what: str) -> None:
    if shape.page_size:
        if t.dim() != 4 or tuple(t.shape[1:]) != (shape.kv_heads, shape.page_size, shape.head_dim) \
                or t.dtype != torch.bfloat16 or t.stride(3) != 1:
            raise ValueError(f"{what} must be a bf16 page pool [pages, {shape.kv_heads}, {shape.page_size}, {shape.head_dim}]")
        return
    want = (shape.num_problems, shape.kv_heads, shape.n_tokens, shape.head_dim)
    if tuple(t.shape) != want or t.dtype != torch.bfloat16 or t.stride(3) != 1:
        raise ValueError(f"{what} must be bf16 {want} with a contiguous last dimension, got {tuple(t.shape)} {t.dtype}")


def _check_q(shape: Shape, q: torch.Tensor) -> None:
    want = (shape.num_problems, shape.q_heads, shape.alpha, shape.head_dim)
    if tuple(q.shape) != want or q.dtype != torch.bfloat16 or q.stride(3) != 1:
        raise ValueError(f"q_obs must be bf16 {want} with a contiguous last dimension")


def _check_out(shape: Shape, k_out: torch.Tensor, v_out: torch.Tensor) -> None:
    want = (shape.num_problems, shape.kv_heads, shape.budget, shape.head_dim)
    for t in (k_out, v_out):
        if tuple(t.shape) != want or t.dtype != torch.bfloat16 or t.stride(3) != 1:
            raise ValueError(f"k_out / v_out must be bf16 {want} with a contiguous last dimension")
    if k_out.stride() != v_out.stride():
        raise ValueError("k_out and v_out must share their strides")


def rkv_should_compress(shape: Shape, cached_tokens: int) -> bool:
    """Trigger test of the decode loop: True once the buffer behind the budget is full."""
    prm = shape.params()
    s = load_library().rkv_should_compress(ctypes.byref(prm), int(cached_tokens))
    if s < 0:
        raise RkvError(s, "rkv_should_compress")
    return s == RKV_OK


def rkv_cache_append(shape: Shape, k_cache: torch.Tensor, v_cache: torch.Tensor, q_cache: torch.Tensor,
                     k_new: torch.Tensor, v_new: torch.Tensor, q_new: torch.Tensor, position: int, q_slot: int) -> None:
    """Write one decoded token's key/value rows at `position` and its query state into slot `q_slot`."""
    _need_gpu(k_cache, v_cache, q_cache, k_new, v_new, q_new)
    _check_kv(shape, k_cache, "k_cache")
    _check_kv(shape, v_cache, "v_cache")
    _check_q(shape, q_cache)
    kv = (shape.num_problems, shape.kv_heads, shape.head_dim)
    qs = (shape.num_problems, shape.q_heads, shape.head_dim)
    for t, want in ((k_new, kv), (v_new, kv), (q_new, qs)):
        if tuple(t.shape) != want or t.dtype != torch.bfloat16 or not t.is_contiguous():
            raise ValueError(f"new rows must be contiguous bf16 {want}")
    prm = shape.params(k_cache, v_cache, q=q_cache)
    s = load_library().rkv_cache_append(ctypes.byref(prm), _ptr(k_cache), _ptr(v_cache), _ptr(q_cache), _ptr(k_new),
                                        _ptr(v_new), _ptr(q_new), int(position), int(q_slot), _stream())
    if s != RKV_OK:
        raise RkvError(s, "rkv_cache_append")


def rkv_workspace_size(shape: Shape) -> int:
    n = ctypes.c_size_t(0)
    prm = shape.params()
    s = load_library().rkv_workspace_size(ctypes.byref(prm), ctypes.byref(n))
    if s != RKV_OK:
        raise RkvError(s, "rkv_workspace_size")
    return int(n.value)


def make_workspace(shape: Shape, device="cuda") -> torch.Tensor:
    return torch.empty(rkv_workspace_size(shape) + 256, dtype=torch.uint8, device=device)


def _ws_args(shape: Shape, ws: Optional[torch.Tensor], device) -> Tuple[torch.Tensor, int, int]:
    if ws is None:
        ws = make_workspace(shape, device)
    base = ws.data_ptr()
    aligned = (base + 255) & ~255
    return ws, aligned, ws.numel() - (aligned - base)


def rkv_score_importance(shape: Shape, q_obs: torch.Tensor, k: torch.Tensor, ws: Optional[torch.Tensor] = None,
                         out: Optional[torch.Tensor] = None) -> torch.Tensor:
    _need_gpu(q_obs, k)
    _check_q(shape, q_obs)
    _check_kv(shape, k, "k")
    if out is None:
        out = torch.empty((shape.num_problems, shape.kv_heads, shape.n_cand), dtype=torch.float32, device=k.device)
    ws, wp, wb = _ws_args(shape, ws, k.device)
    prm = shape.params(k, q=q_obs)
    s = load_library().rkv_score_importance(ctypes.byref(prm), _ptr(q_obs), _ptr(k), _ptr(out), wp, wb, _stream())
    if s != RKV_OK:
        raise RkvError(s, "rkv_score_importance")
    return out


def rkv_score_redundancy(shape: Shape, k: torch.Tensor, ws: Optional[torch.Tensor] = None,
                         want_mean_sim: bool = False):
    _need_gpu(k)
    _check_kv(shape, k, "k")
    red = torch.empty((shape.num_problems, shape.kv_heads, shape.n_cand), dtype=torch.float32, device=k.device)
    ms = torch.empty_like(red) if want_mean_sim else None
    ws, wp, wb = _ws_args(shape, ws, k.device)
    prm = shape.params(k)
    s = load_library().rkv_score_redundancy(ctypes.byref(prm), _ptr(k), _ptr(red), _ptr(ms), wp, wb, _stream())
    if s != RKV_OK:
        raise RkvError(s, "rkv_score_redundancy")
    return (red, ms) if want_mean_sim else red


def rkv_select_topk(shape: Shape, importance: torch.Tensor, redundancy: torch.Tensor,
                    ws: Optional[torch.Tensor] = None, want_score: bool = False):
    _need_gpu(importance, redundancy)
    want = (shape.num_problems, shape.kv_heads, shape.n_cand)
    for t in (importance, redundancy):
        if tuple(t.shape) != want or t.dtype != torch.float32 or not t.is_contiguous():
            raise ValueError(f"scores must be contiguous fp32 {want}")
    dev = importance.device
    kept = torch.empty((shape.num_problems, shape.kv_heads, shape.budget), dtype=torch.int32, device=dev)
    score = torch.empty(want, dtype=torch.float32, device=dev) if want_score else None
    ws, wp, wb = _ws_args(shape, ws, dev)
    prm = shape.params()
    s = load_library().rkv_select_topk(ctypes.byref(prm), _ptr(importance), _ptr(redundancy), _ptr(score),
                                       _ptr(kept), wp, wb, _stream())
    if s != RKV_OK:
        raise RkvError(s, "rkv_select_topk")
    return (kept, score) if want_score else kept


def rkv_compact(shape: Shape, k: torch.Tensor, v: torch.Tensor, kept_idx: torch.Tensor,
                k_out: Optional[torch.Tensor] = None, v_out: Optional[torch.Tensor] = None):
    _need_gpu(k, v, kept_idx)
    _check_kv(shape, k, "k")
    _check_kv(shape, v, "v")
    want = (shape.num_problems, shape.kv_heads, shape.budget)
    if tuple(kept_idx.shape) != want or kept_idx.dtype != torch.int32 or not kept_idx.is_contiguous():
        raise ValueError(f"kept_idx must be contiguous int32 {want}")
    oshape = (shape.num_problems, shape.kv_heads, shape.budget, shape.head_dim)
    if k_out is None:
        k_out = torch.empty(oshape, dtype=torch.bfloat16, device=k.device)
    if v_out is None:
        v_out = torch.empty(oshape, dtype=torch.bfloat16, device=k.device)
    _check_out(shape, k_out, v_out)
    prm = shape.params(k, v, k_out)
    s = load_library().rkv_compact(ctypes.byref(prm), _ptr(k), _ptr(v), _ptr(kept_idx), _ptr(k_out), _ptr(v_out),
                                   _stream())
    if s != RKV_OK:
        raise RkvError(s, "rkv_compact")
    return k_out, v_out


def _check_idx(shape: Shape, kept_idx: torch.Tensor) -> None:
    want = (shape.num_problems, shape.kv_heads, shape.budget)
    if tuple(kept_idx.shape) != want or kept_idx.dtype != torch.int32 or not kept_idx.is_contiguous():
        raise ValueError(f"kept_idx must be contiguous int32 {want}")


def rkv_compact_inplace(shape: Shape, k: torch.Tensor, v: torch.Tensor, kept_idx: torch.Tensor) -> None:
    """Move the kept rows (strictly ascending per head) to rows 0 .. budget-1 of k and v themselves."""
    _need_gpu(k, v, kept_idx)
    _check_kv(shape, k, "k")
    _check_kv(shape, v, "v")
    _check_idx(shape, kept_idx)
    prm = shape.params(k, v)
    s = load_library().rkv_compact_inplace(ctypes.byref(prm), _ptr(k), _ptr(v), _ptr(kept_idx), _stream())
    if s != RKV_OK:
        raise RkvError(s, "rkv_compact_inplace")


def rkv_compress_inplace(shape: Shape, q_obs: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                         ws: Optional[torch.Tensor] = None, kept_idx: Optional[torch.Tensor] = None,
                         score: Optional[torch.Tensor] = None, want_idx: bool = True, want_score: bool = False):
    """The whole step with the compaction done inside k and v.  Returns (status, kept_idx, score)."""
    _need_gpu(q_obs, k, v)
    _check_q(shape, q_obs)
    _check_kv(shape, k, "k")
    _check_kv(shape, v, "v")
    dev = k.device
    if kept_idx is None and want_idx:
        kept_idx = torch.empty((shape.num_problems, shape.kv_heads, shape.budget), dtype=torch.int32, device=dev)
    if kept_idx is not None:
        _check_idx(shape, kept_idx)
    if score is None and want_score:
        score = torch.empty((shape.num_problems, shape.kv_heads, shape.n_cand), dtype=torch.float32, device=dev)
    ws, wp, wb = _ws_args(shape, ws, dev)
    prm = shape.params(k, v, q=q_obs)
    s = load_library().rkv_compress_inplace(ctypes.byref(prm), _ptr(q_obs), _ptr(k), _ptr(v), _ptr(kept_idx),
                                            _ptr(score), wp, wb, _stream())
    if s < 0:
        raise RkvError(s, "rkv_compress_inplace")
    return s, kept_idx, score


def rkv_compress(shape: Shape, q_obs: torch.Tensor, k: torch.Tensor, v: torch.Tensor,
                 ws: Optional[torch.Tensor] = None, k_out: Optional[torch.Tensor] = None,
                 v_out: Optional[torch.Tensor] = None, kept_idx: Optional[torch.Tensor] = None,
                 score: Optional[torch.Tensor] = None, want_idx: bool = True, want_score: bool = False,
                 events=None):
    """The whole step.  Returns (status, k_out, v_out, kept_idx, score); status is RKV_OK or
    RKV_NOT_TRIGGERED (then nothing was computed).  `events`, if given, is a ctypes array of five
    hipEvent_t handles recorded around the four stages (rkv_compress_events)."""
    _need_gpu(q_obs, k, v)
    _check_q(shape, q_obs)
    _check_kv(shape, k, "k")
    _check_kv(shape, v, "v")
    dev = k.device
    oshape = (shape.num_problems, shape.kv_heads, shape.budget, shape.head_dim)
    if k_out is None:
        k_out = torch.empty(oshape, dtype=torch.bfloat16, device=dev)
    if v_out is None:
        v_out = torch.empty(oshape, dtype=torch.bfloat16, device=dev)
    if kept_idx is None and want_idx:
        kept_idx = torch.empty(oshape[:3], dtype=torch.int32, device=dev)
    if score is None and want_score:
        score = torch.empty((shape.num_problems, shape.kv_heads, shape.n_cand), dtype=torch.float32, device=dev)
    ws, wp, wb = _ws_args(shape, ws, dev)
    _check_out(shape, k_out, v_out)
    prm = shape.params(k, v, k_out, q=q_obs)
    lib = load_library()
    if events is None:
        s = lib.rkv_compress(ctypes.byref(prm), _ptr(q_obs), _ptr(k), _ptr(v), _ptr(k_out), _ptr(v_out),
                             _ptr(kept_idx), _ptr(score), wp, wb, _stream())
    else:
        s = lib.rkv_compress_events(ctypes.byref(prm), _ptr(q_obs), _ptr(k), _ptr(v), _ptr(k_out), _ptr(v_out),
                                    _ptr(kept_idx), _ptr(score), wp, wb, _stream(), events)
    if s < 0:
        raise RkvError(s, "rkv_compress")
    return s, k_out, v_out, kept_idx, score


def rkv_probe_mfma(operands: torch.Tensor, sink: torch.Tensor, chains: int) -> int:
    """Measurement aid: one launch of nothing but the similarity pass's MFMA instruction on fragments of
    `operands` (bf16, at least RKV_PROBE_OPERAND_BYTES), on the current stream; returns its flop count."""
    _need_gpu(operands, sink)
    if operands.dtype != torch.bfloat16 or not operands.is_contiguous() or operands.numel() * 2 < RKV_PROBE_OPERAND_BYTES:
        raise ValueError("operands: contiguous bf16 tensor of at least RKV_PROBE_OPERAND_BYTES")
    if not sink.is_contiguous() or sink.numel() * sink.element_size() < RKV_PROBE_SINK_BYTES:
        raise ValueError("sink: contiguous tensor of at least RKV_PROBE_SINK_BYTES")
    flops = ctypes.c_int64(0)
    s = load_library().rkv_probe_mfma(_ptr(operands), _ptr(sink), int(chains), _stream(), ctypes.byref(flops))
    if s < 0:
        raise RkvError(s, "rkv_probe_mfma")
    return flops.value


def rkv_compress_static(shape: Shape, q_obs: torch.Tensor, k: torch.Tensor, v: torch.Tensor, k_out: torch.Tensor,
                        v_out: torch.Tensor, kept_idx: Optional[torch.Tensor] = None,
                        score: Optional[torch.Tensor] = None) -> int:
    """The whole step with the library's fixed scratch array instead of a workspace.  Every buffer is the
    caller's; nothing is allocated here or in the library.  Returns RKV_OK or RKV_NOT_TRIGGERED; shapes whose
    scratch exceeds RKV_STATIC_SCRATCH_BYTES raise (RKV_ERR_WORKSPACE)."""
    _need_gpu(q_obs, k, v, k_out, v_out, kept_idx, score)
    _check_q(shape, q_obs)
    _check_kv(shape, k, "k")
    _check_kv(shape, v, "v")
    _check_out(shape, k_out, v_out)
    if kept_idx is not None:
        _check_idx(shape, kept_idx)
    prm = shape.params(k, v, k_out, q=q_obs)
    s = load_library().rkv_compress_static(ctypes.byref(prm), _ptr(q_obs), _ptr(k), _ptr(v), _ptr(k_out), _ptr(v_out),
                                           _ptr(kept_idx), _ptr(score), _stream())
    if s < 0:
        raise RkvError(s, "rkv_compress_static")
    return s
