"""Convenience holder for a cache handle plus the torch tensors (pool, workspace) it needs.

PyTorch is used for device memory and streams only; every step of the path runs in the HIP
library.  Inputs arrive as numpy arrays (float32, or uint16 bfloat16 bit patterns) and are
uploaded unchanged.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import binding as M


def to_device(x: np.ndarray, dtype: int) -> torch.Tensor:
    """Uploads float32 data (MS_F32) or uint16 bit patterns (MS_BF16) without changing a bit."""
    if dtype == M.MS_BF16:
        assert x.dtype == np.uint16
        return torch.from_numpy(x.view(np.int16).copy()).cuda().view(torch.bfloat16)
    assert x.dtype == np.float32
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


def ints_dev(xs) -> torch.Tensor:
    return torch.tensor(np.asarray(xs, dtype=np.int32).reshape(-1), dtype=torch.int32, device="cuda")


class Session:
    def __init__(self, n_layers: int, n_q_heads: int, n_kv_heads: int, head_dim: int, n_pages: int,
                 dtype: int, rope_base: float, max_seqs: int = 64, max_pages_per_seq: int = 1100,
                 pool: Optional[np.ndarray] = None):
        if not torch.cuda.is_available():
            raise RuntimeError("a GPU is required: the HIP path has no CPU fallback")
        self.dtype = dtype
        self.tdtype = torch.bfloat16 if dtype == M.MS_BF16 else torch.float32
        self.shape = (n_layers, n_pages, n_kv_heads, 2, M.MS_PAGE_SIZE, head_dim)
        self.n_layers, self.n_q_heads, self.n_kv_heads, self.head_dim = n_layers, n_q_heads, n_kv_heads, head_dim
        if pool is not None:
            assert tuple(pool.shape) == self.shape
            self.pool = to_device(pool, dtype)
        else:
            self.pool = torch.zeros(self.shape, dtype=self.tdtype, device="cuda")
        desc = M.make_desc(n_layers, n_q_heads, n_kv_heads, head_dim, n_pages, max_seqs,
                           max_pages_per_seq, dtype, rope_base, self.pool)
        assert M.ms_pool_bytes(desc) == self.pool.numel() * self.pool.element_size()
        self.cache = M.ms_cache_create(desc)
        self.workspace: Optional[torch.Tensor] = None
        self._ws_need = {}

    def close(self) -> None:
        if self.cache:
            M.ms_cache_destroy(self.cache)
            self.cache = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def ensure_workspace(self, B: int, n_q: int) -> torch.Tensor:
        need = self._ws_need.get((B, n_q))
        if need is None:
            need = self._ws_need[(B, n_q)] = M.ms_attention_workspace_bytes(self.cache, B, n_q)
        if self.workspace is None or self.workspace.numel() < need:
            self.workspace = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self.workspace

    def attention(self, layer: int, seq_ids: Sequence[int], n_verify: int, n_foresight: int, q: torch.Tensor,
                  k_new: torch.Tensor, v_new: torch.Tensor, pos_ids: torch.Tensor,
                  ctx_new: Optional[torch.Tensor] = None, scale: float = 0.0,
                  out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        ws = self.ensure_workspace(len(seq_ids), n_verify + n_foresight)
        if out is None:
            out = torch.empty_like(q)
        M.ms_predict_verify_attention(self.cache, layer, seq_ids, n_verify, n_foresight, q, k_new, v_new,
                                      pos_ids, ctx_new, scale, out, ws, stream)
        return out

    def page_tables(self, seq_ids: Sequence[int]) -> List[List[int]]:
        return [M.ms_seq_page_table(self.cache, s) for s in seq_ids]

    def lengths(self, seq_ids: Sequence[int]) -> List[int]:
        return [M.ms_seq_len(self.cache, s) for s in seq_ids]

    def pool_host_f32(self) -> np.ndarray:
        return to_host_f32(self.pool)
