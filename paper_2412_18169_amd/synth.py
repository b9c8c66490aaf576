"""Seeded synthetic inputs for paged attention: layer shapes, context lengths, block tables, Q/K/V.

This module is shared by the tests, the benchmark and the CPU oracle's callers. It holds NO
attention arithmetic: it only draws request lengths, assigns physical KV blocks, produces the
values of Q, K and V, and copies K/V values into page buffers.

The workloads stand in for the paper's serving traces (Section 5.1: BurstGPT, ShareGPT and
LongBench request lengths on Qwen-2.5 GQA layers with 8 KV heads of 128 dims, Section 2.2),
which are not available here: lengths are uniform or lognormal with a heavy tail, prefill arrives
as chunks batched with decodes (Sections 2.1 and 4.3), and the pool is grown in steps the way a
parameter drop hands freed memory to the KVCache (Section 4.1, Section 5.6).

Values are keyed by LOGICAL coordinates (tensor, sequence, token, kv head, dim) through a
counter-based integer hash and a 65536-entry table of standard-normal quantiles, so the same
element has the same bytes on the host and on the device, whatever physical block it lands in.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np
import torch

# --------------------------------------------------------------------------------------------
# counter-based value generator
# --------------------------------------------------------------------------------------------

_MASK64 = (1 << 64) - 1
_GOLDEN = 0x9E3779B97F4A7C15
_C1 = 0xBF58476D1CE4E5B9
_C2 = 0x94D049BB133111EB

TENSOR_Q, TENSOR_K, TENSOR_V = 1, 2, 3


def _to_signed(x: int) -> int:
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(x: int) -> int:
    """64-bit finalizer on Python ints (reference for the tensor version below)."""
    x &= _MASK64
    x ^= x >> 30
    x = (x * _C1) & _MASK64
    x ^= x >> 27
    x = (x * _C2) & _MASK64
    x ^= x >> 31
    return x


def stream_key(seed: int, tensor_id: int, seq: int) -> int:
    """Per-(seed, tensor, sequence) 64-bit key, computed on the host."""
    k = _mix_py(seed * _GOLDEN + tensor_id)
    k = _mix_py(k ^ ((seq + 1) * _C1))
    return k


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    # logical shift right on int64 tensors
    return (x >> k) & ((1 << (64 - k)) - 1)


def hash_u16(key: int, idx: torch.Tensor) -> torch.Tensor:
    """u16 in [0, 65536) for every int64 counter in `idx` (any device); wraps modulo 2^64."""
    x = idx * _to_signed(_GOLDEN) + _to_signed(key)
    x = x ^ _lsr(x, 30)
    x = x * _to_signed(_C1)
    x = x ^ _lsr(x, 27)
    x = x * _to_signed(_C2)
    x = x ^ _lsr(x, 31)
    return _lsr(x, 48)


def hash_u16_numpy(key: int, idx: np.ndarray) -> np.ndarray:
    """Same hash with numpy uint64 arithmetic (cross-check of the int64 tensor version)."""
    with np.errstate(over="ignore"):
        x = idx.astype(np.uint64) * np.uint64(_GOLDEN) + np.uint64(key)
        x ^= x >> np.uint64(30)
        x *= np.uint64(_C1)
        x ^= x >> np.uint64(27)
        x *= np.uint64(_C2)
        x ^= x >> np.uint64(31)
        return (x >> np.uint64(48)).astype(np.int64)


_TABLES = {}


FP8 = "fp8"      # stands for "uint8 codes of OCP FP8 E4M3" where a torch dtype is expected below


def normal_table(dtype, device="cpu") -> torch.Tensor:
    """T[i] = round_to_dtype(Phi^-1((i + 1/2) / 65536)), built in fp64 on the host.  For FP8 the
    table holds the uint8 codes of the values rounded to E4M3 (round to nearest even)."""
    k = (dtype, str(device))
    if k not in _TABLES:
        from scipy.special import ndtri

        t64 = torch.from_numpy(ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0))
        if dtype == FP8:
            _TABLES[k] = t64.to(torch.float32).to(torch.float8_e4m3fn).view(torch.uint8).to(device)
        else:
            _TABLES[k] = t64.to(dtype).to(device)
    return _TABLES[k]


def normal_values(seed: int, tensor_id: int, seq: int, first: int, count: int,
                  dtype, device="cpu") -> torch.Tensor:
    """`count` N(0,1) values of stream (seed, tensor, seq), counters first .. first+count-1."""
    idx = torch.arange(first, first + count, dtype=torch.int64, device=device)
    u = hash_u16(stream_key(seed, tensor_id, seq), idx)
    return normal_table(dtype, device)[u]


# --------------------------------------------------------------------------------------------
# shapes and workloads
# --------------------------------------------------------------------------------------------

@dataclass(frozen=True)
class LayerShape:
    """One attention layer. dtype is what the KV pages hold: 'f32', 'bf16' or 'fp8' (OCP E4M3 codes;
    queries and outputs are bf16 then). B = tokens per KV block."""
    Hq: int
    Hkv: int
    d: int
    B: int
    dtype: str

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def elt(self) -> int:
        """bytes per K/V element"""
        return {"f32": 4, "bf16": 2, "fp8": 1}[self.dtype]

    @property
    def q_elt(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def torch_dtype(self) -> torch.dtype:
        """of queries and outputs"""
        return torch.float32 if self.dtype == "f32" else torch.bfloat16

    @property
    def kv_torch_dtype(self) -> torch.dtype:
        """of the page buffers and of K/V rows handed to kun_kv_append (uint8 codes for fp8)"""
        return torch.uint8 if self.dtype == "fp8" else self.torch_dtype

    @property
    def kv_value_kind(self):
        """key of the value table K/V are drawn from"""
        return FP8 if self.dtype == "fp8" else self.torch_dtype

    @property
    def block_bytes(self) -> int:
        return 2 * self.Hkv * self.B * self.d * self.elt

    @property
    def scale(self) -> float:
        return float(np.float32(1.0 / np.sqrt(self.d)))


@dataclass
class Workload:
    """A batch: decode sequences (context lengths) and prefill chunks (prior p, new c).

    Sequence ids: decodes are 0..S-1, chunk i is sequence S + i (context length p_i + c_i).
    range_blocks[r] = number of blocks in pool range r (range 0 is the first pool, later entries
    are the extensions). block_tables[s] lists the physical block ids of sequence s in logical
    order.
    """
    name: str
    cfg: int
    seed: int
    shape: LayerShape
    decode_lens: np.ndarray                      # int32 [S]
    chunks: List[Tuple[int, int]]                # (p, c) per prefill chunk
    range_blocks: List[int]
    block_tables: List[np.ndarray] = field(default_factory=list)   # int32 per sequence

    @property
    def S(self) -> int:
        return int(len(self.decode_lens))

    @property
    def n_chunks(self) -> int:
        return len(self.chunks)

    @property
    def seq_lens(self) -> np.ndarray:
        """Context length (tokens resident in pages) of every sequence, decodes then chunks."""
        cl = [p + c for p, c in self.chunks]
        return np.concatenate([self.decode_lens.astype(np.int64), np.asarray(cl, dtype=np.int64)])

    @property
    def num_blocks(self) -> int:
        return int(sum(self.range_blocks))

    def table_array(self, rows: Sequence[int], pad: int = -1) -> np.ndarray:
        """int32 [len(rows), max_blocks] block table, padded with `pad`."""
        mb = max(1, max((len(self.block_tables[r]) for r in rows), default=1))
        out = np.full((len(rows), mb), pad, dtype=np.int32)
        for i, r in enumerate(rows):
            bt = self.block_tables[r]
            out[i, : len(bt)] = bt
        return out

    @property
    def decode_kv_tokens(self) -> int:
        return int(self.decode_lens.astype(np.int64).sum())

    @property
    def prefill_pairs(self) -> int:
        """(query, key) pairs per query head over all chunks: sum of p*c + c(c+1)/2 (Eq. 1)."""
        return int(sum(p * c + c * (c + 1) // 2 for p, c in self.chunks))


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed=[seed, stream]))


def lognormal_lengths(rng, n, median=1024, sigma=0.8, lo=16, hi=16384) -> np.ndarray:
    x = np.rint(rng.lognormal(np.log(median), sigma, size=n))
    return np.clip(x, lo, hi).astype(np.int32)


def blocks_needed(lens, B: int) -> np.ndarray:
    lens = np.asarray(lens, dtype=np.int64)
    return (lens + B - 1) // B


def assign_blocks_scattered(w: Workload, stream: int = 2) -> None:
    """Give every sequence its blocks from a seeded permutation of the whole block-id space."""
    need = blocks_needed(w.seq_lens, w.shape.B)
    total = int(need.sum())
    if total > w.num_blocks:
        raise ValueError(f"pool of {w.num_blocks} blocks cannot hold {total}")
    rng = _rng(w.seed, stream)
    if total * 4 >= w.num_blocks:
        ids = rng.permutation(w.num_blocks)[:total]
    else:  # sparse draw from a very large id space
        ids = rng.choice(w.num_blocks, size=total, replace=False)
    ids = ids.astype(np.int32)
    w.block_tables = []
    o = 0
    for n in need:
        w.block_tables.append(ids[o:o + int(n)].copy())
        o += int(n)


def assign_blocks_phased(w: Workload, stream: int = 2) -> List[int]:
    """Admission in phases, one per pool range (Section 5.6: the pool grows while a burst queues).

    Phase k owns ranges 0..k. It admits the longest prefix of not-yet-admitted sequences that fits
    in the blocks still free, drawing them from a seeded shuffle of the currently free blocks.
    Returns the number of sequences resident after each phase.
    """
    need = blocks_needed(w.seq_lens, w.shape.B)
    rng = _rng(w.seed, stream)
    w.block_tables = [None] * len(need)
    resident = []
    nxt = 0
    first = 0
    free = np.zeros(0, dtype=np.int64)
    for nb in w.range_blocks:
        free = np.concatenate([free, np.arange(first, first + nb, dtype=np.int64)])
        first += nb
        free = rng.permutation(free)
        o = 0
        while nxt < len(need) and o + int(need[nxt]) <= len(free):
            w.block_tables[nxt] = free[o:o + int(need[nxt])].astype(np.int32)
            o += int(need[nxt])
            nxt += 1
        free = free[o:]
        resident.append(nxt)
    if nxt != len(need):
        raise ValueError("pool too small for the workload")
    return resident


def custom_workload(name: str, shape: LayerShape, decode_lens, chunks=(), seed=7,
                    extra_blocks=0, range_fracs=(1.0,), cfg=0) -> Workload:
    """Workload with explicit lengths; pool = needed blocks + extra, split by range_fracs."""
    w = Workload(name=name, cfg=cfg, seed=seed, shape=shape,
                 decode_lens=np.asarray(decode_lens, dtype=np.int32),
                 chunks=[(int(p), int(c)) for p, c in chunks], range_blocks=[])
    n = int(blocks_needed(w.seq_lens, shape.B).sum()) + int(extra_blocks)
    n = max(n, len(range_fracs))
    rb = [int(n * f) for f in range_fracs[:-1]]
    rb.append(n - sum(rb))
    w.range_blocks = rb
    assign_blocks_scattered(w)
    return w


SHAPE_TINY = LayerShape(Hq=8, Hkv=2, d=64, B=16, dtype="f32")
SHAPE_8B = LayerShape(Hq=32, Hkv=8, d=128, B=16, dtype="bf16")
SHAPE_70B = LayerShape(Hq=64, Hkv=8, d=128, B=16, dtype="bf16")


def config(cfg: int, block_size: int = 0, q_heads: int = 0, kv_dtype: str = "") -> Workload:
    """The five benchmark configurations (1-based). Seeds are 1000 + cfg.  `block_size` (0 = the
    configuration's own, 16) builds the same requests over KV blocks of another size (32, 64, 128), `q_heads`
    (0 = the configuration's own) with another number of query heads over the same KV heads, `kv_dtype`
    ("" = the configuration's own) with pages of another element type ("fp8": E4M3 pages, bf16 queries)."""
    import dataclasses
    seed = 1000 + cfg
    sh = {1: SHAPE_TINY, 2: SHAPE_8B, 3: SHAPE_8B, 4: SHAPE_8B, 5: SHAPE_70B}.get(cfg, SHAPE_8B)
    if block_size:
        sh = dataclasses.replace(sh, B=block_size)
    if q_heads:
        sh = dataclasses.replace(sh, Hq=q_heads)
    if kv_dtype:
        sh = dataclasses.replace(sh, dtype=kv_dtype)
    if cfg == 1:
        w = Workload("tiny-decode-f32", 1, seed, sh,
                     np.array([17, 64, 200, 513], dtype=np.int32), [], [64 * 16 // sh.B])
        assign_blocks_scattered(w)
    elif cfg == 2:
        lens = _rng(seed, 1).integers(512, 4097, size=64).astype(np.int32)
        w = Workload("8b-decode-bf16", 2, seed, sh, lens, [], [])
        w.range_blocks = [int(blocks_needed(lens, sh.B).sum())]
        assign_blocks_scattered(w)
    elif cfg == 3:
        lens = lognormal_lengths(_rng(seed, 1), 512)
        w = Workload("overload-decode-bf16", 3, seed, sh, lens, [], [])
        n = int(blocks_needed(lens, sh.B).sum())
        r0, r1 = int(0.4 * n), int(0.3 * n)
        w.range_blocks = [r0, r1, n - r0 - r1]
        w.phase_resident = assign_blocks_phased(w)
    elif cfg == 4:
        r = _rng(seed, 1)
        lens = lognormal_lengths(r, 256)
        chunks = [(int(p), 512) for p in r.integers(0, 3585, size=8)]
        w = Workload("mixed-prefill-decode-bf16", 4, seed, sh, lens, chunks, [])
        w.range_blocks = [int(blocks_needed(w.seq_lens, sh.B).sum())]
        assign_blocks_scattered(w)
    elif cfg == 5:
        r = _rng(seed, 1)
        lens = r.integers(1024, 32769, size=256).astype(np.int32)
        chunks = [(int(p), 1024) for p in r.integers(0, 8193, size=4)]
        w = Workload("70b-stage-bf16", 5, seed, sh, lens, chunks, [])
        per_range = (30 * 10**9) // w.shape.block_bytes      # 30 GB ranges: base + 4 extensions
        w.range_blocks = [per_range] * 5
        assign_blocks_scattered(w)
    else:
        raise ValueError("cfg must be 1..5")
    return w


# --------------------------------------------------------------------------------------------
# values and pages
# --------------------------------------------------------------------------------------------

def q_decode(w: Workload, device="cpu") -> torch.Tensor:
    """Decode queries [S, Hq, d]: one row per decode sequence."""
    sh = w.shape
    rows = [normal_values(w.seed, TENSOR_Q, s, 0, sh.Hq * sh.d, sh.torch_dtype, device)
            for s in range(w.S)]
    if not rows:
        return torch.empty(0, sh.Hq, sh.d, dtype=sh.torch_dtype, device=device)
    return torch.stack(rows).view(w.S, sh.Hq, sh.d)


def q_chunk(w: Workload, i: int, device="cpu") -> torch.Tensor:
    """Queries of prefill chunk i, [c, Hq, d]; counters are keyed by the token's position."""
    sh = w.shape
    p, c = w.chunks[i]
    n = sh.Hq * sh.d
    return normal_values(w.seed, TENSOR_Q, w.S + i, p * n, c * n, sh.torch_dtype,
                         device).view(c, sh.Hq, sh.d)


def kv_logical(w: Workload, seq: int, t0: int, t1: int, device="cpu"):
    """Logical K and V of sequence `seq`, tokens t0..t1-1: two tensors [t1-t0, Hkv, d]."""
    sh = w.shape
    n = sh.Hkv * sh.d
    k = normal_values(w.seed, TENSOR_K, seq, t0 * n, (t1 - t0) * n, sh.kv_value_kind, device)
    v = normal_values(w.seed, TENSOR_V, seq, t0 * n, (t1 - t0) * n, sh.kv_value_kind, device)
    return k.view(t1 - t0, sh.Hkv, sh.d), v.view(t1 - t0, sh.Hkv, sh.d)


def range_of_blocks(range_blocks: Sequence[int], ids: np.ndarray):
    """(range index, index inside the range) of every physical block id."""
    firsts = np.concatenate([[0], np.cumsum(range_blocks)])
    r = np.searchsorted(firsts, ids, side="right") - 1
    return r, ids - firsts[r]


def alloc_ranges(w: Workload, device="cpu", poison: bool = True) -> List[torch.Tensor]:
    """One buffer per pool range, [n_blocks, Hkv, 2, B*d] elements; unused space NaN-poisoned (FP8:
    the code 0x7F)."""
    sh = w.shape
    out = []
    for nb in w.range_blocks:
        if poison:
            t = torch.full((nb, sh.Hkv, 2, sh.B * sh.d), 0x7F if sh.dtype == "fp8" else float("nan"),
                           dtype=sh.kv_torch_dtype, device=device)
        else:
            t = torch.empty((nb, sh.Hkv, 2, sh.B * sh.d), dtype=sh.kv_torch_dtype, device=device)
        out.append(t)
    return out


def write_pages(w: Workload, ranges: List[torch.Tensor], seq: int, t0: int, t1: int,
                k: Optional[torch.Tensor] = None, v: Optional[torch.Tensor] = None) -> None:
    """Copy tokens t0..t1-1 of sequence `seq` into its pages.

    Page layout of one (block, kv head): a row of tiles of min(B, 16) tokens; a tile holds K as
    [tokens][d], then V as [d][tokens] (V is stored transposed inside a tile). Slots of the last
    block beyond the context are left as they are.
    """
    sh = w.shape
    B, d = sh.B, sh.d
    T = min(B, 16)
    dev = ranges[0].device
    if k is None:
        k, v = kv_logical(w, seq, t0, t1, dev)
    bt = w.block_tables[seq]
    toks = np.arange(t0, t1, dtype=np.int64)
    blk = bt[toks // B].astype(np.int64)
    tile = torch.from_numpy((toks % B) // T).to(dev)
    slot = torch.from_numpy(toks % T).to(dev)
    r_idx, local = range_of_blocks(w.range_blocks, blk)
    for r in np.unique(r_idx):
        sel = np.nonzero(r_idx == r)[0]
        selt = torch.from_numpy(sel).to(dev)
        lb = torch.from_numpy(local[sel]).to(dev)
        sl, tl = slot[selt], tile[selt]
        buf = ranges[int(r)].view(-1, sh.Hkv, B // T, 2, T * d)
        kview = buf[:, :, :, 0, :].view(-1, sh.Hkv, B // T, T, d)     # [blk, h, tile, token, d]
        vview = buf[:, :, :, 1, :].view(-1, sh.Hkv, B // T, d, T)     # [blk, h, tile, d, token]
        kview[lb, :, tl, sl, :] = k[selt]                             # [n, Hkv, d]
        vview[lb, :, tl, :, sl] = v[selt]


def fill_pool(w: Workload, ranges: List[torch.Tensor], seqs: Optional[Sequence[int]] = None,
              max_tokens_per_call: int = 1 << 15) -> None:
    """Write every resident token of the given sequences (default: all) into the pages."""
    lens = w.seq_lens
    if seqs is None:
        seqs = range(len(lens))
    for s in seqs:
        L = int(lens[s])
        for t0 in range(0, L, max_tokens_per_call):
            write_pages(w, ranges, s, t0, min(L, t0 + max_tokens_per_call))


def to_host_bits(t: torch.Tensor) -> np.ndarray:
    """Device/host tensor -> numpy array of its raw elements (float32, or uint16 for bf16)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()
