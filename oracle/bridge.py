"""Helpers that hand device-resident test data to the CPU oracle.  TEST INFRASTRUCTURE ONLY.

The oracle works on host numpy arrays.  For pools too large to mirror on the host (tens of GB),
`compact_pool` copies only the blocks that the sampled requests reference into one small host
range and renumbers their block tables; by the oracle's own invariance to physical placement this
does not change any result.  No attention arithmetic lives here.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np
import torch

from . import paged_attention as O


def host_bits(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def full_pool(ranges: Sequence[torch.Tensor], Hkv: int, d: int, B: int, dtype: str) -> O.OraclePool:
    return O.OraclePool([host_bits(r).reshape(-1) for r in ranges], Hkv, d, B, dtype)


def compact_pool(ranges: Sequence[torch.Tensor], range_blocks: Sequence[int], tables: List[np.ndarray],
                 lens: Sequence[int], Hkv: int, d: int, B: int, dtype: str):
    """tables[i]: physical block ids of request i (logical order), lens[i] its context length.
    Returns (OraclePool with one range, int32 table array [n, max_blocks] of renumbered ids)."""
    firsts = np.concatenate([[0], np.cumsum(range_blocks)]).astype(np.int64)
    need = [int((int(L) + B - 1) // B) for L in lens]
    ids = np.concatenate([np.asarray(t[:n], dtype=np.int64) for t, n in zip(tables, need)]) if tables else np.zeros(0, np.int64)
    r = np.searchsorted(firsts, ids, side="right") - 1
    local = ids - firsts[r]
    block_elems = 2 * Hkv * B * d
    parts = []
    out = torch.empty((len(ids), block_elems), dtype=ranges[0].dtype)
    for ri in np.unique(r):
        sel = np.nonzero(r == ri)[0]
        src = ranges[int(ri)].view(-1, block_elems)
        idx = torch.from_numpy(local[sel]).to(src.device)
        out[torch.from_numpy(sel)] = src[idx].cpu()
    mb = max(1, max(need, default=1))
    tab = np.full((len(tables), mb), -1, dtype=np.int32)
    o = 0
    for i, n in enumerate(need):
        tab[i, :n] = np.arange(o, o + n, dtype=np.int32)
        o += n
    pool = O.OraclePool([host_bits(out).reshape(-1)], Hkv, d, B, dtype)
    return pool, tab
