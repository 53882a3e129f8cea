"""Token-major KVCache slots -> the in-slot element order the kernels read.

In an engine the KV-append step writes slots in this order directly; here the synthetic
pools are generated token-major and permuted once.  The order itself is defined by the
library (fs_kv_elem_offset); this module only applies it as a gather.
"""
from __future__ import annotations

import numpy as np

from .binding import fs_kv_elem_offset

_CACHE: dict = {}


def slot_permutation(kv_dtype: int, is_v: bool, page_tokens: int = 16, head_dim: int = 128) -> np.ndarray:
    """src[i] = token-major index (tok*head_dim + d) of the element stored at offset i."""
    key = (kv_dtype, bool(is_v), page_tokens, head_dim)
    if key not in _CACHE:
        n = page_tokens * head_dim
        src = np.full(n, -1, dtype=np.int64)
        for tok in range(page_tokens):
            for d in range(head_dim):
                off = fs_kv_elem_offset(kv_dtype, int(is_v), tok, d)
                if off < 0 or off >= n or src[off] != -1:
                    raise RuntimeError("fs_kv_elem_offset is not a permutation")
                src[off] = tok * head_dim + d
        _CACHE[key] = src
    return _CACHE[key]


def pack_slots(pool, kv_dtype: int, is_v: bool):
    """pool [n_slots][page_tokens][head_dim] (numpy array or torch tensor, any 1/2-byte dtype)
    -> same shape and dtype with every slot's elements in kernel order."""
    n, T, D = pool.shape
    src = slot_permutation(kv_dtype, is_v, T, D)
    if isinstance(pool, np.ndarray):
        return np.ascontiguousarray(pool.reshape(n, T * D)[:, src]).reshape(n, T, D)
    import torch
    idx = torch.from_numpy(src).to(pool.device)
    return pool.reshape(n, T * D).index_select(1, idx).reshape(n, T, D).contiguous()
