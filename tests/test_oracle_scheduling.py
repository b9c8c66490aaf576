"""Pins of the planning oracle (cost model Eq. 1-3, lookahead split, drop-plan generation) against
what the paper and the mathematics fix: brute-force pair counts, the paper's worked examples
(tests/golden/drop_plan_examples.txt), conservation laws and special cases."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import scheduling as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "drop_plan_examples.txt")


def brute_pairs(p, c):
    """Count the visible (query, key) pairs of a chunk one by one: row r of the chunk sees keys 0 .. p + r."""
    return sum(1 for r in range(c) for k in range(p + c) if k <= p + r)


def test_pair_count_is_the_number_of_visible_query_key_pairs():
    for p, c in itertools.product([0, 1, 5, 16, 33], [0, 1, 2, 7, 16, 40]):
        assert S.attention_pairs(p, c) == brute_pairs(p, c)


def test_chunks_of_a_request_add_up_to_the_unchunked_request():
    # "the latter chunk has to additionally compute the attention with the former chunk" (Section 4.3):
    # chunking moves pairs between chunks but creates or loses none
    rng = np.random.default_rng(0)
    for _ in range(50):
        cuts = np.sort(rng.choice(np.arange(1, 200), size=rng.integers(0, 6), replace=False))
        bounds = [0] + cuts.tolist() + [200]
        total = sum(S.attention_pairs(a, b - a) for a, b in zip(bounds[:-1], bounds[1:]))
        assert total == 200 * 201 // 2
    assert S.attention_pairs(100, 100) > S.attention_pairs(0, 100)      # the later chunk is the slower one


def test_eq1_terms():
    # each constant multiplies its own term and nothing else
    assert S.chunk_cost(3, 4, 1.0, 0.0, 0.0) == brute_pairs(3, 4)
    assert S.chunk_cost(3, 4, 0.0, 1.0, 0.0) == 4
    assert S.chunk_cost(3, 4, 0.0, 0.0, 1.0) == 1
    assert S.chunk_cost(3, 4, 2.0, 3.0, 5.0) == 2 * brute_pairs(3, 4) + 12 + 5


def test_eq3_parameters_are_loaded_once_per_microbatch():
    chunks = [(0, 0, 10), (1, 5, 3), (2, 0, 0), (3, 7, 1)]              # request 2 has no tokens here
    assert S.microbatch_cost(chunks, 0.0, 0.0, 4.0) == 4.0               # three live chunks, one gamma
    assert S.microbatch_cost(chunks[:1], 1.5, 0.5, 4.0) == S.chunk_cost(0, 10, 1.5, 0.5, 4.0)
    want = sum(S.chunk_cost(p, c, 1.5, 0.5, 4.0) for _, p, c in chunks if c) - 2 * 4.0
    assert S.microbatch_cost(chunks, 1.5, 0.5, 4.0) == pytest.approx(want, rel=1e-15)
    assert S.microbatch_cost([], 1.0, 1.0, 1.0) == 0.0


def test_fit_recovers_the_constants_from_exact_times():
    rng = np.random.default_rng(1)
    a, b, g = 3.0e-9, 2.0e-6, 4.0e-4
    mbs, times = [], []
    for _ in range(40):
        n = int(rng.integers(1, 5))
        mb = [(i, int(rng.integers(0, 300)), int(rng.integers(1, 120))) for i in range(n)]
        mbs.append(mb)
        times.append(a * sum(brute_pairs(p, c) for _, p, c in mb) + b * sum(c for _, _, c in mb) + g)
    fa, fb, fg = S.fit_cost_model(mbs, times)
    assert fa == pytest.approx(a, rel=1e-6) and fb == pytest.approx(b, rel=1e-6) and fg == pytest.approx(g, rel=1e-6)


def covered(mbs):
    """request -> sorted list of (start, end) token spans over all microbatches"""
    spans = {}
    for mb in mbs:
        for r, p, c in mb:
            spans.setdefault(r, []).append((p, p + c))
    return {r: sorted(v) for r, v in spans.items()}


def check_partition(chunks, mbs):
    want = {r: (p, p + c) for r, p, c in chunks if c > 0}
    got = covered(mbs)
    assert set(got) == set(want)
    for r, spans in got.items():
        assert spans[0][0] == want[r][0] and spans[-1][1] == want[r][1]
        for (a0, a1), (b0, b1) in zip(spans[:-1], spans[1:]):
            assert a1 == b0 and a1 > a0                                   # contiguous, no overlap, no gap
    flat = [r for mb in mbs for r, _, _ in mb]
    assert flat == sorted(flat, key=lambda r: [q for q, _, _ in chunks].index(r))    # queue order kept


def test_split_conserves_tokens_and_cost_and_balances_to_within_one_token():
    rng = np.random.default_rng(2)
    for trial in range(60):
        n = int(rng.integers(1, 6))
        chunks = [(i, int(rng.integers(0, 50)), int(rng.integers(1, 60))) for i in range(n)]
        a, b, g = float(rng.uniform(0, 2)), float(rng.uniform(0, 3)), float(rng.uniform(0, 20))
        l, r = S.split_microbatch(chunks, a, b, g)
        check_partition(chunks, [m for m in (l, r) if m])
        cl, cr, cb = S.microbatch_cost(l, a, b, g), S.microbatch_cost(r, a, b, g), S.microbatch_cost(chunks, a, b, g)
        if l and r:
            assert cl + cr == pytest.approx(cb + g, rel=1e-12)            # one more parameter load, nothing else
        # moving the cut by one token cannot help: the imbalance is at most one token's largest cost
        step = a * (max(p + c for _, p, c in chunks)) + b + g
        assert abs(cl - cr) <= step + 1e-9


def test_split_with_token_costs_only_halves_the_token_count():
    chunks = [(0, 0, 7), (1, 0, 30), (2, 0, 4), (3, 0, 1)]
    l, r = S.split_microbatch(chunks, 0.0, 1.0, 0.0)
    assert S.tokens_of(l) == 21 and S.tokens_of(r) == 21
    assert l == [(0, 0, 7), (1, 0, 14)] and r == [(1, 14, 16), (2, 0, 4), (3, 0, 1)]


def test_split_of_one_long_request_gives_the_first_chunk_more_tokens():
    # attention only: the second chunk also attends to the first, so equal cost needs k > c - k;
    # k(k+1)/2 = (k(c-k) + (c-k)(c-k+1)/2) has its root near c / sqrt(2)
    c = 10000
    l, r = S.split_microbatch([(0, 0, c)], 1.0, 0.0, 0.0)
    k = l[0][2]
    assert r == [(0, k, c - k)]
    assert abs(k - c / math.sqrt(2)) <= 2


def test_lookahead_levels_thresholds_and_balance():
    chunks = [(i, 0, n) for i, n in enumerate([4000, 300, 2500, 1200, 800, 5000, 64, 900])]
    a, b, g = 1.0e-3, 1.0, 50.0
    mbs = S.lookahead(chunks, a, b, g, min_tokens=512)
    check_partition(chunks, mbs)
    assert all(S.tokens_of(m) >= 512 for m in mbs) and len(mbs) >= 8
    # nothing more can be split without going below the threshold
    for m in mbs:
        l, r = S.split_microbatch(m, a, b, g)
        assert min(S.tokens_of(l), S.tokens_of(r)) < 512
    four = S.lookahead(chunks, a, b, g, min_tokens=512, max_microbatches=4)
    assert len(four) == 4
    check_partition(chunks, four)
    costs = [S.microbatch_cost(m, a, b, g) for m in four]
    assert max(costs) / min(costs) < 1.02                                # two levels of halving stay balanced
    # token-count-based microbatches of the same requests are not: equal tokens, unequal cost
    by_tokens = S.lookahead(chunks, 0.0, 1.0, 0.0, min_tokens=512, max_microbatches=4)
    tc = [S.microbatch_cost(m, a, b, g) for m in by_tokens]
    assert max(S.tokens_of(m) for m in by_tokens) - min(S.tokens_of(m) for m in by_tokens) <= 2
    assert max(tc) / min(tc) > 1.2
    assert S.lookahead(chunks, a, b, g, min_tokens=10**6) == [list(chunks)]
    assert S.lookahead(chunks, a, b, g, min_tokens=512, max_microbatches=1) == [list(chunks)]


def golden():
    vals = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            k, *v = line.split()
            vals[k] = [float(x) if "." in x else int(x) for x in v]
    return vals


def test_drop_plan_examples_printed_in_the_paper():
    gd = golden()
    # example 1: groups of sizes 1, 2, 3 -> the groups of sizes 1 and 2 merge
    sizes = gd["groups_sizes"]
    ids = iter(range(sum(sizes)))
    groups = [[next(ids) for _ in range(n)] for n in sizes]
    plan = S.drop_plan(groups, num_layers=12, layer_bytes=10, demand_bytes=1)
    assert sorted(len(g) for g in plan.merges[0]) == gd["first_merge_sizes"] and len(plan.merges) == 1
    # example 2: 7 layers on 7 instances, everything merged: 6 of 7 layers dropped everywhere
    L, N = gd["layers"][0], gd["instances"][0]
    plan = S.drop_plan(N, num_layers=L, layer_bytes=1000, demand_bytes=(N - 1) * L * 1000)
    assert plan.ok and len(plan.groups) == 1
    assert all(e - f == L - gd["dropped_layers_per_instance"][0] for f, e in plan.kept_layers)
    frac = plan.dropped_bytes[0] / (L * 1000)
    assert math.floor(frac * 100) / 100 == gd["freed_fraction_printed"][0]


def test_drop_plan_invariants():
    rng = np.random.default_rng(4)
    for trial in range(40):
        N, L, lb = int(rng.integers(1, 20)), int(rng.integers(1, 50)), int(rng.integers(1, 1000))
        copy = L * lb
        demand = int(rng.integers(0, (N + 1) * copy))
        plan = S.drop_plan(N, L, lb, demand)
        want_merges = min(N - 1, -(-demand // copy))                      # one copy per merge, no more than needed
        assert len(plan.merges) == want_merges and plan.freed_bytes == want_merges * copy
        assert plan.ok == (plan.freed_bytes >= demand)
        assert sorted(i for g in plan.groups for i in g) == list(range(N))
        assert sum(plan.dropped_bytes) == plan.freed_bytes                # what instances hand over is what was freed
        for g in plan.groups:                                             # every group still holds one full copy
            held = sorted(plan.kept_layers[i] for i in g)
            assert held[0][0] == 0 and held[-1][1] == L
            assert all(a[1] == b[0] for a, b in zip(held[:-1], held[1:]))
        # as few instances per request as possible: group sizes differ by at most a factor of two
        # when all groups started as single instances
        sz = sorted(len(g) for g in plan.groups)
        assert sz[-1] <= 2 * max(1, sz[0]) or len(sz) == 1
    # always the two smallest, the earlier one first on ties
    plan = S.drop_plan([[0, 1, 2], [3], [4, 5], [6]], 4, 1, 3 * 4)
    assert plan.merges == [([3], [6]), ([4, 5], [3, 6]), ([0, 1, 2], [3, 4, 5, 6])]
