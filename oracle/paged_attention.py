"""CPU oracle for paged attention over an extensible KV block pool.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this module: only tests, the smoke check and the
benchmark's cpu_baseline leg use it.  It shares no code with the HIP library.

What it computes is the plain definition of softmax attention, in fp64, over the keys and values
of a request gathered in logical order from its KV blocks:

* the KVCache holds K and V of all previous tokens of a request (Section 2.1), kept as
  fixed-size blocks behind a base address (Section 4.1, "Local instance memory management");
  here the pool is a list of byte ranges, the first pool plus every extension appended at the
  tail, and a block id counts through them in order;
* a decode step attends to every cached token including its own;
* a prefill chunk of c new tokens after p prior tokens attends to the p prior tokens
  ("prefix-attn") and causally to itself, diagonal included ("self-attn"), which is
  p*c + (c^2 + c)/2 (query, key) pairs (Section 4.3, Eq. 1).

KV quantisation is what Section 7 names as the lossy alternative for a KVCache under memory pressure:
pages may hold K and V as 8-bit floats (OCP FP8 "E4M3": 1 sign, 4 exponent bits with bias 7, 3 mantissa
bits, no infinities, the one NaN pattern S.1111.111) while queries and outputs stay bf16; the oracle
widens the page bytes exactly and computes as before, so the same tolerance applies.

Readings where the paper is silent: consecutive query heads share a KV head (GQA); the context
length counts the token being decoded; one page (block, kv head) is a row of tiles of min(B, 16)
tokens, a tile storing K as [token][dim] then V as [dim][token] (the paper fixes no layout inside
a block); table entries past ceil(L/B) and slots past L are never read.

Every function has a pin in tests/test_oracle_pins.py (dense brute force, permutation invariance,
rows summing to 1, length-1 context, closed forms, Eq. 1 pair count, chunking equivalence).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np


# ---------------------------------------------------------------------------------------------
# pool and indexing (integer side)
# ---------------------------------------------------------------------------------------------

@dataclass
class OraclePool:
    """ranges[r]: flat numpy array of raw elements of range r (float32, uint16 holding bf16, or uint8
    holding FP8 E4M3 codes)."""
    ranges: List[np.ndarray]
    Hkv: int
    d: int
    B: int
    dtype: str  # 'f32' | 'bf16' | 'fp8' (what the pages hold)

    @property
    def elt(self) -> int:
        return {"f32": 4, "bf16": 2, "fp8": 1}[self.dtype]

    @property
    def q_dtype(self) -> str:
        """Element type of queries (and outputs): the pages' type, except that FP8 pages go with bf16."""
        return "bf16" if self.dtype == "fp8" else self.dtype

    @property
    def block_elems(self) -> int:
        return 2 * self.Hkv * self.B * self.d

    @property
    def block_bytes(self) -> int:
        return self.block_elems * self.elt

    @property
    def range_blocks(self) -> List[int]:
        return [int(r.size) // self.block_elems for r in self.ranges]

    @property
    def num_blocks(self) -> int:
        return sum(self.range_blocks)


def usable_blocks(range_bytes: int, block_bytes: int) -> int:
    """A byte range holds floor(bytes / block_bytes) blocks; the remainder is unused."""
    return range_bytes // block_bytes


def resolve_block(range_blocks: Sequence[int], block: int) -> Tuple[int, int]:
    """Physical block id -> (range index, block index inside that range).

    Ids are cumulative over the ranges in the order they were added and never renumbered.
    """
    if block < 0:
        raise IndexError("negative block id")
    first = 0
    for r, n in enumerate(range_blocks):
        if block < first + n:
            return r, block - first
        first += n
    raise IndexError("block id beyond the pool")


def block_byte_offset(range_blocks: Sequence[int], block: int, block_bytes: int) -> Tuple[int, int]:
    """Physical block id -> (range index, byte offset from that range's base)."""
    r, local = resolve_block(range_blocks, block)
    return r, local * block_bytes


def token_slot(table_row: Sequence[int], t: int, B: int) -> Tuple[int, int]:
    """Logical token t of a request -> (physical block id, slot inside the block)."""
    return int(table_row[t // B]), t % B


TILE_TOKENS = 16


def tile_tokens(B: int) -> int:
    """Tokens per tile: a page is a row of tiles of min(B, 16) tokens, each holding its K rows and
    then its V columns (a page of 64 tokens is four pages of 16 tokens in a row)."""
    return min(B, TILE_TOKENS)


def k_elem_offset(pool: OraclePool, local_block: int, kvh: int, slot: int) -> int:
    """Element offset (inside a range) of K[slot][0] of page (local_block, kvh)."""
    T = tile_tokens(pool.B)
    page = (local_block * pool.Hkv + kvh) * 2 * pool.B * pool.d
    return page + (slot // T) * 2 * T * pool.d + (slot % T) * pool.d


def v_elem_offset(pool: OraclePool, local_block: int, kvh: int, slot: int, j: int) -> int:
    """Element offset (inside a range) of V[slot][j]: V is stored as [dim][token] inside a tile."""
    T = tile_tokens(pool.B)
    page = (local_block * pool.Hkv + kvh) * 2 * pool.B * pool.d
    return page + (slot // T) * 2 * T * pool.d + T * pool.d + j * T + slot % T


def widen(raw: np.ndarray, dtype: str) -> np.ndarray:
    """Raw elements -> fp64, exactly (bf16 is the upper half of an fp32; an FP8 E4M3 code S.EEEE.MMM is
    (-1)^S (1 + M/8) 2^(E - 7) for E > 0, (-1)^S (M/8) 2^-6 for E = 0, and NaN for S.1111.111)."""
    if dtype == "bf16":
        return (raw.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if dtype == "fp8":
        c = raw.astype(np.int64)
        sign = np.where((c >> 7) & 1, -1.0, 1.0)
        e, m = (c >> 3) & 15, c & 7
        val = np.where(e == 0, np.ldexp(m / 8.0, -6), np.ldexp(1.0 + m / 8.0, (e - 7).astype(np.int64)))
        return np.where((e == 15) & (m == 7), np.nan, sign * val)
    return raw.astype(np.float64)


def gather_kv(pool: OraclePool, table_row: Sequence[int], L: int, kvh: int):
    """K and V of tokens 0..L-1 of one request and KV head, in logical order: two [L, d] fp64."""
    B, d = pool.B, pool.d
    T = tile_tokens(B)
    rb = pool.range_blocks
    K = np.empty((L, d), dtype=np.float64)
    V = np.empty((L, d), dtype=np.float64)
    for b0 in range(0, L, T):                                         # one tile at a time
        n = min(T, L - b0)
        blk, slot = token_slot(table_row, b0, B)
        r, local = resolve_block(rb, blk)
        mem = pool.ranges[r]
        ko = k_elem_offset(pool, local, kvh, slot)
        K[b0:b0 + n] = widen(mem[ko:ko + n * d], pool.dtype).reshape(n, d)
        vo = v_elem_offset(pool, local, kvh, slot, 0)
        vt = widen(mem[vo:vo + T * d], pool.dtype).reshape(d, T)      # [dim][slot of the tile]
        V[b0:b0 + n] = vt[:, :n].T
    return K, V


# ---------------------------------------------------------------------------------------------
# attention (floating-point side)
# ---------------------------------------------------------------------------------------------

def attention_rows(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float,
                   n_visible: Sequence[int]):
    """Softmax attention of query rows q [R, d] over keys K, values V [L, d], all fp64.

    Row i sees keys 0..n_visible[i]-1.  z = scale * q.k; w = exp(z - max z); o = sum(w v) / sum w.
    Returns (o [R, d], normalised weights [R, max n_visible], zero on hidden keys).
    """
    nv = np.asarray(n_visible, dtype=np.int64)
    L = int(nv.max())
    z = scale * (q @ K[:L].T)                                   # [R, L]
    hidden = np.arange(L)[None, :] >= nv[:, None]
    z[hidden] = -np.inf
    m = z.max(axis=1, keepdims=True)
    w = np.exp(z - m)                                           # hidden keys get exactly 0
    l = w.sum(axis=1, keepdims=True)
    o = (w @ V[:L]) / l
    return o, w / l


def paged_decode(pool: OraclePool, q: np.ndarray, tables: np.ndarray, ctx_len: Sequence[int],
                 Hq: int, scale: float) -> np.ndarray:
    """Decode step: q [S, Hq, d] raw elements; the query of request s sits at position L_s - 1 and
    sees L_s keys.  Returns fp64 [S, Hq, d].  Requests with L_s == 0 give NaN rows (skipped)."""
    S = q.shape[0]
    G = Hq // pool.Hkv
    scale = float(np.float32(scale))
    q64 = widen(q.reshape(-1), pool.q_dtype).reshape(S, Hq, pool.d)
    out = np.full((S, Hq, pool.d), np.nan, dtype=np.float64)
    for s in range(S):
        L = int(ctx_len[s])
        if L == 0:
            continue
        for kvh in range(pool.Hkv):
            K, V = gather_kv(pool, tables[s], L, kvh)
            o, _ = attention_rows(q64[s, kvh * G:(kvh + 1) * G], K, V, scale, [L] * G)
            out[s, kvh * G:(kvh + 1) * G] = o
    return out


def paged_prefill_chunk(pool: OraclePool, q: np.ndarray, table_row: Sequence[int], p: int, c: int,
                        Hq: int, scale: float, rows: Sequence[int] = None):
    """One prefill chunk: q [c, Hq, d] raw elements for the tokens at positions p..p+c-1, whose K/V
    are already in the pages.  Row r sees keys 0..p+r.  Returns (fp64 [len(rows), Hq, d], number of
    (query, key) pairs visited per head).  `rows` restricts the computation to some chunk rows."""
    G = Hq // pool.Hkv
    scale = float(np.float32(scale))
    if rows is None:
        rows = range(c)
    rows = list(rows)
    q64 = widen(q.reshape(-1), pool.q_dtype).reshape(c, Hq, pool.d)
    out = np.empty((len(rows), Hq, pool.d), dtype=np.float64)
    pairs = 0
    if not rows:
        return out, 0
    Lmax = p + max(rows) + 1
    for kvh in range(pool.Hkv):
        K, V = gather_kv(pool, table_row, Lmax, kvh)
        for g in range(G):
            h = kvh * G + g
            vis = [p + r + 1 for r in rows]
            o, _ = attention_rows(q64[rows, h], K, V, scale, vis)
            out[:, h] = o
            if h == 0:
                pairs = sum(vis)
    return out, pairs


def merge_partials(m: np.ndarray, l: np.ndarray, acc: np.ndarray) -> np.ndarray:
    """Combine split-K partial results of one query row: partition i holds m_i = max z,
    l_i = sum exp(z - m_i), acc_i = sum exp(z - m_i) v.  o = sum acc_i e^(m_i - M) / sum l_i
    e^(m_i - M), M = max m_i.  m, l: [P]; acc: [P, d]."""
    M = m.max()
    f = np.exp(m - M)
    return (f[:, None] * acc).sum(axis=0) / (f * l).sum()


# ---------------------------------------------------------------------------------------------
# KV append (copy side)
# ---------------------------------------------------------------------------------------------

def kv_append(pool: OraclePool, k_new: np.ndarray, v_new: np.ndarray, seq_of_tok: Sequence[int],
              pos_of_tok: Sequence[int], tables: np.ndarray) -> List[Tuple[int, int, int]]:
    """Scatter raw rows k_new, v_new [T, Hkv, d] into the pages, in place.  Returns the slot map:
    (range, block index inside the range, slot) for every token."""
    rb = pool.range_blocks
    slots = []
    for i in range(len(seq_of_tok)):
        blk, slot = token_slot(tables[int(seq_of_tok[i])], int(pos_of_tok[i]), pool.B)
        r, local = resolve_block(rb, blk)
        mem = pool.ranges[r]
        for kvh in range(pool.Hkv):
            ko = k_elem_offset(pool, local, kvh, slot)
            mem[ko:ko + pool.d] = k_new[i, kvh]
            for j in range(pool.d):
                mem[v_elem_offset(pool, local, kvh, slot, j)] = v_new[i, kvh, j]
        slots.append((r, local, slot))
    return slots
