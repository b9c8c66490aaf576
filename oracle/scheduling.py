"""CPU oracle for the host-side planning routines around the attention path.  TEST INFRASTRUCTURE ONLY.

Nothing in the product path may import this module; it shares no code with the C++ library.

* Cost model (Section 4.3, Eq. 1-3): a chunk of c tokens after p prior tokens of the same request
  costs alpha * (p*c + (c*c + c)/2) + beta * c + gamma; a microbatch costs the sum over its chunks
  minus (n - 1) * gamma for its n chunks (the parameters are loaded once per microbatch).  The
  three constants are fitted by least squares to measured times.
* Lookahead batch formulation (Section 4.3): the queued tokens start as one microbatch that is
  split recursively into two microbatches of (nearly) equal cost until a microbatch would fall
  below a token threshold.
* Drop-plan generation (Section 4.1, Algorithm 1): instance groups sit in a priority queue by size; while the
  memory demand is not met the two smallest groups are merged and one redundant copy of the
  parameters is dropped.

Readings where the paper is silent (its two pseudocode listings are figures, and it leaves out the
details of `split`):
  - split walks the chunks in queue order; whole chunks go left while the left cost stays at or
    below half of the total; the chunk that crosses is cut at the token count k that makes the two
    costs closest (k = 0 or k = c mean no cut); a cut request continues on the right with prior
    p + k.  The recursion stops when either half would hold fewer than `min_tokens` tokens, or at
    `max_microbatches` (0 = no limit).
  - ties between groups of equal size go to the group created first; a merged group counts as
    created at the merge.
  - a group of g instances serves the L layers as g pipeline stages of contiguous layers, stage j
    (instances in order of their ids) holding layers floor(j*L/g) .. floor((j+1)*L/g) - 1; the
    other layers of an instance's copy are what it drops.
  - the cost model uses one gamma symbol for Eq. 1's constant and Eq. 3's correction.

Pins: tests/test_oracle_scheduling.py.
"""
from __future__ import annotations

import heapq
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import numpy as np

Chunk = Tuple[int, int, int]          # (request, prior tokens p, chunk tokens c)


# ---------------------------------------------------------------------------------------------
# cost model
# ---------------------------------------------------------------------------------------------
def attention_pairs(p: int, c: int) -> int:
    """(query, key) pairs of a chunk: prefix attention p*c plus causal self attention (Eq. 1)."""
    return p * c + (c * c + c) // 2


def chunk_cost(p: int, c: int, alpha: float, beta: float, gamma: float) -> float:
    """Eq. 1."""
    return alpha * attention_pairs(p, c) + beta * c + gamma


def microbatch_cost(chunks: Sequence[Chunk], alpha: float, beta: float, gamma: float) -> float:
    """Eq. 2-3: chunks with c > 0 only; the parameters are loaded once for all of them."""
    live = [(p, c) for _, p, c in chunks if c > 0]
    if not live:
        return 0.0
    return sum(chunk_cost(p, c, alpha, beta, gamma) for p, c in live) - (len(live) - 1) * gamma


def fit_cost_model(microbatches: Sequence[Sequence[Chunk]], times: Sequence[float]) -> Tuple[float, float, float]:
    """Least squares for (alpha, beta, gamma): a microbatch's cost is linear in
    (sum of pairs, sum of tokens, 1)."""
    rows = []
    for mb in microbatches:
        live = [(p, c) for _, p, c in mb if c > 0]
        rows.append([float(sum(attention_pairs(p, c) for p, c in live)), float(sum(c for _, c in live)), 1.0])
    sol, *_ = np.linalg.lstsq(np.asarray(rows, dtype=np.float64), np.asarray(times, dtype=np.float64), rcond=None)
    return float(sol[0]), float(sol[1]), float(sol[2])


# ---------------------------------------------------------------------------------------------
# lookahead batch formulation
# ---------------------------------------------------------------------------------------------
def split_microbatch(chunks: Sequence[Chunk], alpha: float, beta: float, gamma: float
                     ) -> Tuple[List[Chunk], List[Chunk]]:
    """Two microbatches, in queue order, whose costs are as close as a cut at a token boundary allows."""
    chunks = [ch for ch in chunks if ch[2] > 0]
    best = None
    for i, (r, p, c) in enumerate(chunks):                 # brute force over every cut position
        for k in range(0, c + 1):
            left = list(chunks[:i]) + ([(r, p, k)] if k > 0 else [])
            right = ([(r, p + k, c - k)] if k < c else []) + list(chunks[i + 1:])
            d = abs(microbatch_cost(left, alpha, beta, gamma) - microbatch_cost(right, alpha, beta, gamma))
            if best is None or d < best[0]:
                best = (d, left, right)
    if best is None:
        return [], []
    return best[1], best[2]


def tokens_of(chunks: Sequence[Chunk]) -> int:
    return sum(c for _, _, c in chunks)


def lookahead(chunks: Sequence[Chunk], alpha: float, beta: float, gamma: float, min_tokens: int,
              max_microbatches: int = 0) -> List[List[Chunk]]:
    """Recursive halving of the queued tokens into cost-balanced microbatches (breadth first, so a
    limit on the number of microbatches stops whole levels)."""
    level = [[ch for ch in chunks if ch[2] > 0]]
    while True:
        if max_microbatches and 2 * len(level) > max_microbatches:
            return level
        nxt, changed = [], False
        for b in level:
            l, r = split_microbatch(b, alpha, beta, gamma)
            if tokens_of(l) >= min_tokens and tokens_of(r) >= min_tokens:
                nxt += [l, r]
                changed = True
            else:
                nxt.append(b)
        if not changed:
            return level
        if max_microbatches and len(nxt) > max_microbatches:
            return level
        level = nxt


# ---------------------------------------------------------------------------------------------
# drop plan
# ---------------------------------------------------------------------------------------------
@dataclass
class DropPlan:
    ok: bool                              # demand met; otherwise fall back (Section 4.1)
    merges: List[Tuple[List[int], List[int]]]      # instance ids of the two groups of every merge, in order
    groups: List[List[int]]               # final groups (instance ids in ascending order)
    freed_bytes: int                      # one parameter copy per merge
    kept_layers: List[Tuple[int, int]]    # per instance: [first, end) of the layers it still holds
    dropped_bytes: List[int]              # per instance: bytes of its copy it may hand to the KVCache


def stage_layers(j: int, g: int, L: int) -> Tuple[int, int]:
    return (j * L) // g, ((j + 1) * L) // g


def drop_plan(group_sizes_or_groups, num_layers: int, layer_bytes: int, demand_bytes: int) -> DropPlan:
    """Greedy grouping: merge the two smallest groups until `demand_bytes` is freed.
    `group_sizes_or_groups`: initial groups as lists of instance ids (or just N for N single groups)."""
    if isinstance(group_sizes_or_groups, int):
        groups0 = [[i] for i in range(group_sizes_or_groups)]
    else:
        groups0 = [sorted(g) for g in group_sizes_or_groups]
    copy_bytes = num_layers * layer_bytes
    heap = [(len(g), order, g) for order, g in enumerate(groups0)]
    heapq.heapify(heap)
    order = len(heap)
    freed = 0
    merges = []
    while freed < demand_bytes and len(heap) >= 2:
        _, _, a = heapq.heappop(heap)
        _, _, b = heapq.heappop(heap)
        merges.append((a, b))
        freed += copy_bytes
        heapq.heappush(heap, (len(a) + len(b), order, sorted(a + b)))
        order += 1
    groups = [g for _, _, g in sorted(heap, key=lambda t: t[2][0])]
    n_inst = sum(len(g) for g in groups)
    kept: List[Optional[Tuple[int, int]]] = [None] * n_inst
    for g in groups:
        for j, inst in enumerate(g):
            kept[inst] = stage_layers(j, len(g), num_layers)
    dropped = [(num_layers - (e - f)) * layer_bytes for f, e in kept]
    return DropPlan(freed >= demand_bytes, merges, groups, freed, kept, dropped)
