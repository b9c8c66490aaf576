"""CPU tests of the host-side planning entry points (cost model, lookahead, drop plan) against the
planning oracle, through the C ABI.  Integer outputs (cuts, groups, layers, bytes) must be equal;
costs and fitted constants agree to rounding."""
import itertools

import numpy as np
import pytest

from oracle import scheduling as S
from paper_2412_18169_amd import kun


def test_costs_match_oracle():
    rng = np.random.default_rng(0)
    for _ in range(200):
        m = (float(rng.uniform(0, 1e-6)), float(rng.uniform(0, 1e-3)), float(rng.uniform(0, 1e-2)))
        p, c = int(rng.integers(0, 100000)), int(rng.integers(0, 20000))
        assert kun.kun_cost_chunk(m, p, c) == pytest.approx(S.chunk_cost(p, c, *m), rel=1e-13)
        mb = [(i, int(rng.integers(0, 5000)), int(rng.integers(0, 3000))) for i in range(int(rng.integers(0, 9)))]
        assert kun.kun_cost_microbatch(m, mb) == pytest.approx(S.microbatch_cost(mb, *m), rel=1e-13, abs=0)
    assert np.isnan(kun.kun_cost_chunk((1, 1, 1), -1, 5))


def test_fit_matches_oracle_on_noisy_times():
    rng = np.random.default_rng(1)
    mbs, times = [], []
    for _ in range(60):
        mb = [(i, int(rng.integers(0, 8192)), int(rng.integers(1, 4096))) for i in range(int(rng.integers(1, 6)))]
        mbs.append(mb)
        times.append(S.microbatch_cost(mb, 2.5e-10, 3.0e-7, 2.0e-5) * float(rng.uniform(0.97, 1.03)))
    got, want = kun.kun_cost_fit(mbs, times), S.fit_cost_model(mbs, times)
    for g, w in zip(got, want):
        assert g == pytest.approx(w, rel=1e-8)
    with pytest.raises(kun.KunError):
        kun.kun_cost_fit(mbs[:2], times[:2])                              # three unknowns
    same = [[(0, 0, 64)]] * 5
    with pytest.raises(kun.KunError):
        kun.kun_cost_fit(same, [1.0] * 5)                                  # identical samples determine nothing


def test_lookahead_matches_oracle_cut_for_cut():
    rng = np.random.default_rng(2)
    for trial in range(150):
        n = int(rng.integers(1, 9))
        queue = [(i, int(rng.integers(0, 400)), int(rng.integers(0, 700))) for i in range(n)]
        kind = trial % 4
        if kind == 0:
            m = (float(rng.uniform(0, 1e-3)), float(rng.uniform(0, 1)), float(rng.uniform(0, 30)))
        elif kind == 1:
            m = (0.0, 1.0, 0.0)                                            # token counts only: exact ties happen
        elif kind == 2:
            m = (1.0, 0.0, 0.0)                                            # attention only, integer costs
        else:
            m = (0.0, 0.0, 1.0)                                            # every interior cut ties
        min_tokens = int(rng.integers(1, 300))
        limit = int(rng.choice([0, 0, 1, 2, 4, 7, 8]))
        want = S.lookahead(queue, *m, min_tokens=min_tokens, max_microbatches=limit)
        got = kun.kun_lookahead(m, queue, min_tokens, limit)
        assert got == [list(mb) for mb in want], (trial, m, min_tokens, limit, queue)
    with pytest.raises(kun.KunError):
        kun.kun_lookahead((-1.0, 0.0, 0.0), [(0, 0, 5)], 1)


def replay(n, initial, merges):
    """Member lists of every merge from (member, size) pairs, by replaying the merges."""
    groups = {}
    if initial is None:
        for i in range(n):
            groups[i] = [i]
    else:
        by = {}
        for i, g in enumerate(initial):
            by.setdefault(g, []).append(i)
        for g in by.values():
            for i in g:
                groups[i] = g
    out = []
    for (ma, sa), (mb, sb) in merges:
        a, b = groups[ma], groups[mb]
        assert len(a) == sa and len(b) == sb and a is not b
        out.append((sorted(a), sorted(b)))
        merged = sorted(a + b)
        for i in merged:
            groups[i] = merged
    return out


def test_drop_plan_matches_oracle():
    rng = np.random.default_rng(3)
    for trial in range(120):
        N = int(rng.integers(1, 40))
        L, lb = int(rng.integers(1, 90)), int(rng.integers(1, 10**9))
        demand = int(rng.integers(0, (N + 1) * L * lb))
        initial = None
        groups0 = N
        if trial % 3 == 0:
            initial = rng.integers(0, max(1, N // 2), size=N).tolist()
            by = {}
            for i, g in enumerate(initial):
                by.setdefault(g, []).append(i)
            groups0 = [by[g] for g in sorted(by)]
        want = S.drop_plan(groups0, L, lb, demand)
        got = kun.kun_drop_plan(N, initial, L, lb, demand)
        assert got["demand_met"] == want.ok and got["freed_bytes"] == want.freed_bytes
        assert got["kept"] == want.kept_layers and got["dropped_bytes"] == want.dropped_bytes
        assert replay(N, initial, got["merges"]) == [(sorted(a), sorted(b)) for a, b in want.merges]
        final = {}
        for i, g in enumerate(got["group_of_instance"]):
            final.setdefault(g, []).append(i)
        assert [final[g] for g in sorted(final)] == want.groups
    with pytest.raises(kun.KunError):
        kun.kun_drop_plan(4, [0, 1, 9, 0], 4, 1, 1)
