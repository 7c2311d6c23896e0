"""Decode-loop view of the compression step (Sec. 3.1, Alg. 1, App. C.1).

``DecodeCache`` keeps, per (sequence, layer) problem and KV head, a cache of
N = B_budget + B_buffer rows and the query states of the last alpha decode steps.  Every decode
step appends one token; when the buffer behind the budget is full the cache is compressed to
``budget`` rows (the selected candidates in their original order, then the alpha observation
tokens) and decoding continues.  By default two cache allocations are used alternately so that
the compaction is a plain gather from one into the other; with ``inplace=True`` there is one
allocation and the kept rows are moved to its front.  All work runs in the HIP library; this
class only owns the buffers and the counters.
"""
from __future__ import annotations

import torch

from . import rkv


class DecodeCache:
    def __init__(self, shape: rkv.Shape, device="cuda", inplace: bool = False):
        self.shape = shape
        self.inplace = inplace
        P, H, Hq, N, d = shape.num_problems, shape.kv_heads, shape.q_heads, shape.n_tokens, shape.head_dim
        copies = 1 if inplace else 2
        self._k = [torch.zeros((P, H, N, d), dtype=torch.bfloat16, device=device) for _ in range(copies)]
        self._v = [torch.zeros((P, H, N, d), dtype=torch.bfloat16, device=device) for _ in range(copies)]
        self.q_cache = torch.zeros((P, Hq, shape.alpha, d), dtype=torch.bfloat16, device=device)
        self.kept_idx = torch.zeros((P, H, shape.budget), dtype=torch.int32, device=device)
        self._ws = rkv.make_workspace(shape, device)
        self._cur = 0
        self.length = 0            # rows currently held per head
        self.tokens_seen = 0       # decode steps so far
        self.compressions = 0

    @property
    def k(self) -> torch.Tensor:
        """Current key cache [P, H, N, d]; rows [0, length) are valid."""
        return self._k[self._cur]

    @property
    def v(self) -> torch.Tensor:
        return self._v[self._cur]

    def append(self, k_new: torch.Tensor, v_new: torch.Tensor, q_new: torch.Tensor) -> bool:
        """One decode step: k_new, v_new [P, H, d], q_new [P, Hq, d].  Returns True if the step
        ended with a compression."""
        s = self.shape
        rkv.rkv_cache_append(s, self.k, self.v, self.q_cache, k_new, v_new, q_new,
                             self.length, self.tokens_seen % s.alpha)
        self.length += 1
        self.tokens_seen += 1
        if rkv.rkv_should_compress(s, self.length):
            self.compress()
            return True
        return False

    def compress(self) -> None:
        s = self.shape
        if self.length != s.n_tokens:
            raise RuntimeError("compress() runs when the cache holds budget + buffer rows")
        if self.inplace:
            st, *_ = rkv.rkv_compress_inplace(s, self.q_cache, self.k, self.v, ws=self._ws, kept_idx=self.kept_idx)
            if st != rkv.RKV_OK:
                raise RuntimeError("compression was not triggered")
            self.length = s.budget
            self.compressions += 1
            return
        nxt = 1 - self._cur
        st, *_ = rkv.rkv_compress(s, self.q_cache, self.k, self.v, ws=self._ws,
                                  k_out=self._k[nxt][:, :, :s.budget], v_out=self._v[nxt][:, :, :s.budget],
                                  kept_idx=self.kept_idx)
        if st != rkv.RKV_OK:
            raise RuntimeError("compression was not triggered")
        self._cur = nxt
        self.length = s.budget
        self.compressions += 1
