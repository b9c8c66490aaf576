"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (default
partitioning).  Outputs are checked against the oracle on all requests where that takes seconds,
else on a seeded sample (shortest, longest, random) that the oracle computes one by one."""
import os

import numpy as np
import pytest
import torch

from oracle import bridge, paged_attention as O
from paper_2412_18169_amd import kun, synth
from paper_2412_18169_amd.runner import DeviceWorkload

pytestmark = pytest.mark.gpu
TOL = 2e-2


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    yield
    kun.kun_set_option("KUN_DECODE_PART", None)


def decode_err(dw, out, rows):
    w, sh = dw.w, dw.w.shape
    lens = [int(w.decode_lens[s]) for s in rows]
    pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[s] for s in rows], lens, sh.Hkv,
                                    sh.d, sh.B, sh.dtype)
    ref = O.paged_decode(pool, bridge.host_bits(dw.q_dec[rows]), tab, lens, sh.Hq, sh.scale)
    got = out[rows].double().cpu().numpy()
    assert np.isfinite(got).all()
    return float(np.abs(got - ref).max())


def sample_rows(w, n_edge=16, n_rand=32):
    order = np.argsort(w.decode_lens, kind="stable")
    rng = np.random.default_rng(w.seed)
    pick = set(order[:n_edge].tolist()) | set(order[-n_edge:].tolist())
    pick |= set(rng.choice(w.S, size=min(n_rand, w.S), replace=False).tolist())
    return sorted(pick)


def test_config3_pool_extended_twice_mid_run():
    w = synth.config(3)
    dw = DeviceWorkload(w, n_ranges_at_create=1)         # pool = range 0 (40 %); data of all phases is resident
    kun.kun_validate_block_table(dw.pool, torch.from_numpy(w.table_array(range(w.phase_resident[0]))),
                                 torch.from_numpy(w.decode_lens[:w.phase_resident[0]].astype(np.int32)))
    used = np.concatenate(w.block_tables)
    r, _ = synth.range_of_blocks(w.range_blocks, used.astype(np.int64))
    assert set(np.unique(r)) == {0, 1, 2}                # the final block table mixes all three ranges
    kun.kun_set_option("KUN_DECODE_PART", "1024")               # pin the split so residents are comparable bit for bit
    outs = []
    for phase, nres in enumerate(w.phase_resident):
        if phase:
            first, nb = dw.extend_next()
            assert (first, nb) == (sum(w.range_blocks[:phase]), w.range_blocks[phase])
        out = dw.decode(nres).clone()
        torch.cuda.synchronize()
        rows = list(range(nres)) if phase == 2 else sample_rows(w)[:24]
        rows = [s for s in rows if s < nres]
        err = decode_err(dw, out, rows)
        print(f"phase {phase}: {nres} resident, max err {err:.3e}")
        assert err <= TOL
        outs.append(out)
    n0, n1 = w.phase_resident[0], w.phase_resident[1]
    assert torch.equal(outs[0][:n0], outs[1][:n0]) and torch.equal(outs[0][:n0], outs[2][:n0])
    assert torch.equal(outs[1][:n1], outs[2][:n1])
    kun.kun_set_option("KUN_DECODE_PART", None)
    out = dw.decode().clone()                            # and with the default partitioning bench.py uses
    torch.cuda.synchronize()
    assert decode_err(dw, out, sample_rows(w)) <= TOL
    dw.close()


@pytest.mark.parametrize("block_size", [16, 64])
def test_config4_mixed_batch_decode_part(block_size):
    w = synth.config(4, block_size)
    dw = DeviceWorkload(w)
    pre = dw.prefill().clone()                           # mixed batch: both calls on one stream
    out = dw.decode().clone()
    torch.cuda.synchronize()
    err = decode_err(dw, out, list(range(w.S)))
    print("cfg4 decode max err", err)
    assert err <= TOL
    if block_size == 64:                                 # (blocks of 16 tokens: the prefill tests and cfg5 below)
        sh = w.shape
        rng = np.random.default_rng(4)
        got = pre.double().cpu().numpy()
        for i, (p, c) in enumerate(w.chunks):
            q0 = int(dw.q_start_host[i])
            rws = sorted(set([0, c - 1] + rng.choice(c, size=12, replace=False).tolist()))
            pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[w.S + i]], [p + c], sh.Hkv,
                                            sh.d, sh.B, sh.dtype)
            ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq,
                                           sh.scale, rows=rws)
            assert float(np.abs(got[q0:q0 + c][rws] - ref).max()) <= TOL
    dw.close()


@pytest.mark.parametrize("Hkv,G", [(1, 8), (1, 16), (3, 4), (5, 5)])
def test_other_numbers_of_kv_heads(Hkv, G):
    # one KV head (a tensor-parallel shard of an 8-KV-head model), and counts that are not powers of two
    sh = synth.LayerShape(Hq=Hkv * G, Hkv=Hkv, d=128, B=16, dtype="bf16")
    w = synth.custom_workload("hkv", sh, [1, 17, 64, 700, 1500, 2100, 33], chunks=[(0, 70), (100, 200), (3000, 40)],
                              extra_blocks=3, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    dw.out_dec.fill_(float("nan"))
    dw.out_pre.fill_(float("nan"))
    pre = dw.prefill().clone()
    out = dw.decode().clone()
    torch.cuda.synchronize()
    assert decode_err(dw, out, list(range(w.S))) <= TOL
    got = pre.double().cpu().numpy()
    assert np.isfinite(got).all()
    for i, (p, c) in enumerate(w.chunks):
        q0 = int(dw.q_start_host[i])
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[w.S + i]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale)
        assert float(np.abs(got[q0:q0 + c] - ref).max()) <= TOL
    check_slot_map(dw, [0, 3, 5, 7], [0, 699, 2099, 50], kv_head=Hkv - 1)
    dw.close()


@pytest.mark.parametrize("seed", list(range(12)))
def test_seeded_random_shapes_lengths_and_pools(seed):
    # shape, block size, lengths, chunking and the split of the pool into ranges all drawn from the seed:
    # one decode call and one prefill call against the oracle (all decode rows, sampled prefill rows)
    rng = np.random.default_rng(1234 + seed)
    mfma = seed % 3 != 2
    G = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8] + ([16] if mfma else [])))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    B = int(rng.choice([16, 32, 64, 128]))
    d, dtype = (128, "bf16") if mfma else [(64, "f32"), (128, "f32"), (64, "bf16")][seed % 3 if seed % 3 != 2 else int(rng.integers(3))]
    sh = synth.LayerShape(Hq=Hkv * G, Hkv=Hkv, d=d, B=B, dtype=dtype)
    S = int(rng.integers(1, 24))
    lens = [int(x) for x in np.clip(rng.lognormal(5.5, 1.2, size=S), 1, 5000).astype(int)]
    if mfma:
        chunks = [(int(rng.integers(0, 3000)), int(rng.integers(0, 400))) for _ in range(int(rng.integers(1, 6)))]
    else:
        chunks = [(int(rng.integers(0, 300)), int(rng.integers(0, 40))) for _ in range(int(rng.integers(1, 4)))]
    nr = int(rng.integers(1, 5))
    fr = rng.random(nr) + 0.2
    w = synth.custom_workload(f"rnd{seed}", sh, lens, chunks=chunks, seed=100 + seed, extra_blocks=int(rng.integers(nr, 9)),
                              range_fracs=tuple((fr / fr.sum()).tolist()))
    print(f"seed {seed}: Hq={sh.Hq} Hkv={Hkv} d={d} {dtype} B={B} S={S} chunks={chunks} ranges={w.range_blocks}", flush=True)
    dw = DeviceWorkload(w)
    dw.out_dec.fill_(float("nan"))
    dw.out_pre.fill_(float("nan"))
    pre = dw.prefill().clone()
    out = dw.decode().clone()
    torch.cuda.synchronize()
    tol = 1e-5 if dtype == "f32" else TOL
    assert decode_err(dw, out, list(range(w.S))) <= tol
    got = pre.double().cpu().numpy()
    assert np.isfinite(got).all()
    for i, (p, c) in enumerate(w.chunks):
        if c == 0:
            continue
        q0 = int(dw.q_start_host[i])
        rws = sorted(set([0, c - 1] + rng.choice(c, size=min(c, 24), replace=False).tolist()))
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[w.S + i]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale,
                                       rows=rws)
        assert float(np.abs(got[q0:q0 + c][rws] - ref).max()) <= tol
    dw.close()


@pytest.mark.parametrize("kv_dtype", ["bf16", "fp8"])
def test_config5_150GB_pool_sampled(kv_dtype):
    # sample: the 16 shortest, the 16 longest and 32 random decode requests, every head; first, last and
    # 128 random rows of every chunk (FP8 pages: a quarter of that)
    w = synth.config(5, kv_dtype="" if kv_dtype == "bf16" else kv_dtype)
    dw = DeviceWorkload(w, poison=False)
    assert kun.kun_kv_pool_num_ranges(dw.pool) == 5
    assert kun.kun_kv_pool_num_blocks(dw.pool) * w.shape.block_bytes >= 149 * 10**9
    used = np.concatenate(w.block_tables).astype(np.int64)
    r, _ = synth.range_of_blocks(w.range_blocks, used)
    assert set(np.unique(r)) == {0, 1, 2, 3, 4} and used.max() > 2**21     # ids beyond 2^21: 64-bit offsets matter
    # as bench.py launches them: both plans first, then the planned calls ...
    dw.decode(steps="plan")
    dw.prefill(steps="plan")
    pre = dw.prefill(steps="planned").clone()
    out = dw.decode(steps="planned").clone()
    # ... and the one-call forms: the same bits
    dw.out_pre.fill_(float("nan"))
    dw.out_dec.fill_(float("nan"))
    pre1 = dw.prefill().clone()
    out1 = dw.decode().clone()
    torch.cuda.synchronize()
    dw.check_guards()
    assert torch.equal(pre.view(torch.int16), pre1.view(torch.int16))
    assert torch.equal(out.view(torch.int16), out1.view(torch.int16))
    rows = sample_rows(w, 16, 32) if kv_dtype == "bf16" else sample_rows(w, 4, 8)
    err = decode_err(dw, out, rows)
    print(f"cfg5 decode ({len(rows)} sampled requests) max err {err:.3e}")
    assert err <= TOL
    sh = w.shape
    rng = np.random.default_rng(5)
    got = pre.double().cpu().numpy()
    for i, (p, c) in enumerate(w.chunks):
        q0 = int(dw.q_start_host[i])
        rws = sorted(set([0, c - 1] + rng.choice(c, size=128 if kv_dtype == "bf16" else 32, replace=False).tolist()))
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[w.S + i]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale,
                                       rows=rws)
        e = float(np.abs(got[q0:q0 + c][rws] - ref).max())
        print(f"cfg5 chunk {i} (p={p}) max err {e:.3e}")
        assert e <= TOL
    # device-side resolution of 20000 sampled tokens: offsets beyond 4 GiB inside 30 GB ranges
    seqs = rng.integers(0, len(w.seq_lens), size=20000)
    poss = (rng.random(20000) * w.seq_lens[seqs]).astype(np.int64)
    check_slot_map(dw, seqs, poss, kv_head=7)
    dw.close()


def check_slot_map(dw, seqs, poss, kv_head):
    """kun_slot_map against the oracle's address arithmetic, bit-exact."""
    w, sh = dw.w, dw.w.shape
    table = w.table_array(range(len(w.seq_lens)))
    T = len(seqs)
    dev = dw.dev
    r_out = torch.empty(T, dtype=torch.int32, device=dev)
    k_out = torch.empty(T, dtype=torch.int64, device=dev)
    v_out = torch.empty(T, dtype=torch.int64, device=dev)
    kun.kun_slot_map(dw.pool, torch.from_numpy(np.asarray(seqs, dtype=np.int32)).to(dev),
                     torch.from_numpy(np.asarray(poss, dtype=np.int32)).to(dev), T, torch.from_numpy(table).to(dev),
                     table.shape[1], kv_head, r_out, k_out, v_out)
    torch.cuda.synchronize()
    geom = O.OraclePool([np.zeros(0, dtype=np.uint16)] * len(w.range_blocks), sh.Hkv, sh.d, sh.B, sh.dtype)
    exp_r, exp_k, exp_v = [], [], []
    for s_, t in zip(seqs, poss):
        blk, slot = O.token_slot(table[int(s_)], int(t), sh.B)
        r, local = O.resolve_block(w.range_blocks, blk)
        exp_r.append(r)
        exp_k.append(O.k_elem_offset(geom, local, kv_head, slot) * sh.elt)
        exp_v.append(O.v_elem_offset(geom, local, kv_head, slot, 0) * sh.elt)
    assert np.array_equal(r_out.cpu().numpy(), np.asarray(exp_r, dtype=np.int32))
    assert np.array_equal(k_out.cpu().numpy(), np.asarray(exp_k, dtype=np.int64))
    assert np.array_equal(v_out.cpu().numpy(), np.asarray(exp_v, dtype=np.int64))
    return max(exp_k)


@pytest.mark.parametrize("dtype,d,B", [("bf16", 128, 16), ("f32", 64, 16), ("bf16", 64, 16), ("f32", 128, 16),
                                       ("bf16", 128, 64), ("f32", 64, 64), ("bf16", 128, 32), ("f32", 128, 128)])
def test_slot_map_matches_oracle_for_every_token(dtype, d, B):
    sh = synth.LayerShape(Hq=8, Hkv=4, d=d, B=B, dtype=dtype)
    w = synth.custom_workload("slots", sh, [37, 1, 16, 250, 1000], chunks=[(20, 70)], extra_blocks=5,
                              range_fracs=(0.3, 0.3, 0.4))
    dw = DeviceWorkload(w, fill=False, poison=False)
    seqs, poss = [], []
    for s_, L in enumerate(w.seq_lens):
        seqs += [s_] * int(L)
        poss += list(range(int(L)))
    for h in (0, 3):
        check_slot_map(dw, seqs, poss, kv_head=h)
    dw.close()


@pytest.mark.parametrize("form", ["one-call", "plans-in-the-graph", "plans-before-the-graph"])
def test_step_captured_in_a_hip_graph_replays_bit_identically(form):
    # append + prefill + decode only enqueue kernels (no allocation, no memset nodes), so a step can be
    # captured once and replayed; every replay, with eager work in between, gives the eager bits.  The
    # two-step forms: with the plan launches captured too, or made once before the capture (every replay
    # then runs the planned calls against the same plans: the decode counters clean up after themselves)
    sh = synth.SHAPE_8B
    w = synth.custom_workload("graph", sh, [900, 3000, 17, 1500, 64] * 6, chunks=[(0, 300), (1024, 512), (300, 100)],
                              extra_blocks=4, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    ref_p = dw.prefill().clone()                          # also sizes the workspaces before the capture
    ref_d = dw.decode().clone()
    k, v = synth.kv_logical(w, 0, 899, 900, dw.dev)
    seq_of = torch.zeros(1, dtype=torch.int32, device=dw.dev)
    pos_of = torch.full((1,), 899, dtype=torch.int32, device=dw.dev)
    table = torch.from_numpy(w.table_array(range(len(w.seq_lens)))).to(dw.dev)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    if form == "plans-before-the-graph":
        dw.decode(steps="plan")
        dw.prefill(steps="plan")
        torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        if form == "plans-in-the-graph":
            dw.decode(steps="plan")
            dw.prefill(steps="plan")
        kun.kun_kv_append(dw.pool, k, v, seq_of, pos_of, 1, table, table.shape[1])
        dw.prefill(steps="both" if form == "one-call" else "planned")
        dw.decode(steps="both" if form == "one-call" else "planned")
    for rep in range(4):
        dw.out_pre.fill_(float("nan"))
        dw.out_dec.fill_(float("nan"))
        if rep % 2 and form != "plans-before-the-graph":  # (eager calls would overwrite the plans in the workspaces)
            dw.decode(5)                                  # eager work between replays, on the same buffers
            dw.out_dec.fill_(float("nan"))
        elif rep % 2:
            dw.q_dec.add_(0)                              # some eager work on the same stream
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(dw.out_pre.view(torch.int16), ref_p.view(torch.int16)), rep
        assert torch.equal(dw.out_dec.view(torch.int16), ref_d.view(torch.int16)), rep
    dw.close()


@pytest.mark.parametrize("dtype", ["bf16", "fp8"])
def test_very_long_contexts(dtype):
    """One request of 300 000 tokens next to short ones (586 split-K partitions whose records the last
    workgroup to arrive merges) and a prefill chunk behind 200 000 prior tokens (3 130 key tiles per work
    item): every decode row and a sample of the chunk's rows against the oracle."""
    from test_gpu_prefill import check_prefill
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype=dtype)
    lens = [300_000, 17, 70_001, 1]
    w = synth.custom_workload("long", sh, lens, chunks=[(200_000, 300), (0, 33)], extra_blocks=7,
                              range_fracs=(0.3, 0.5, 0.2))
    dw = DeviceWorkload(w)
    out = dw.decode().clone()
    torch.cuda.synchronize()
    dw.check_guards()
    err = decode_err(dw, out, list(range(len(lens))))
    print("decode max err", err, flush=True)
    assert err <= TOL
    perr = check_prefill(dw, rows_per_chunk=6)
    print("prefill max err", perr, flush=True)
    dw.close()


def test_very_many_small_requests():
    """50 000 decode requests of 0 to 40 tokens (the work list is built 1 024 requests at a time) and 5 000
    prefill chunks of 0 to 12 tokens (more work items than the plan sorts by cost): a seeded sample of
    requests and chunks against the oracle, and no row of a live request or chunk left unwritten."""
    from test_gpu_prefill import check_prefill
    rng = np.random.default_rng(77)
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    lens = rng.integers(0, 41, size=50_000).tolist()
    chunks = [(int(rng.integers(0, 101)), int(rng.integers(0, 13))) for _ in range(5_000)]
    w = synth.custom_workload("many", sh, lens, chunks=chunks, extra_blocks=11, range_fracs=(0.5, 0.25, 0.25))
    dw = DeviceWorkload(w)
    dw.out_dec.fill_(float("nan"))
    out = dw.decode().clone()
    torch.cuda.synchronize()
    dw.check_guards()
    live = torch.from_numpy(np.asarray(lens) > 0).to(out.device)
    assert torch.isfinite(out[live].float()).all() and torch.isnan(out[~live].float()).all()
    rows = sorted(set(rng.choice(len(lens), size=96, replace=False).tolist()) | {0, len(lens) - 1, 1023, 1024, 1025})
    rows = [r for r in rows if lens[r] > 0]
    err = decode_err(dw, out, rows)
    print("decode max err", err, flush=True)
    assert err <= TOL
    dw.out_pre.fill_(float("nan"))
    only = sorted(set(rng.choice(len(chunks), size=64, replace=False).tolist()) | {0, len(chunks) - 1, 4095, 4096, 4097})
    perr = check_prefill(dw, only=only)
    print("prefill max err", perr, flush=True)
    assert torch.isfinite(dw.out_pre.float()).all()      # rows exist for non-empty chunks only: all written
    dw.close()


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp8", 128), ("f32", 64)])
def test_pool_of_the_maximum_number_of_ranges(dtype, d):
    """A pool grown fifteen times (KUN_MAX_RANGES = 16 ranges of unequal size), every request's blocks drawn from
    all of them: decode, prefill and append against the oracle; the seventeenth range is refused."""
    from test_gpu_prefill import check_prefill
    sh = synth.LayerShape(Hq=8, Hkv=2, d=d, B=16, dtype=dtype)
    fr = np.arange(1, kun.KUN_MAX_RANGES + 1, dtype=np.float64)
    lens = [900, 1, 2500, 77, 1300, 16]
    chunks = [(700, 130), (0, 90)] if d == 128 else [(60, 20), (0, 9)]
    w = synth.custom_workload("r16", sh, lens, chunks=chunks, extra_blocks=40, range_fracs=tuple((fr / fr.sum()).tolist()))
    assert len(w.range_blocks) == kun.KUN_MAX_RANGES
    dw = DeviceWorkload(w)
    assert kun.kun_kv_pool_num_ranges(dw.pool) == kun.KUN_MAX_RANGES
    used = np.concatenate(w.block_tables)
    r, _ = synth.range_of_blocks(w.range_blocks, used.astype(np.int64))
    assert len(np.unique(r)) == kun.KUN_MAX_RANGES           # the tables name blocks of every range
    out = dw.decode().clone()
    torch.cuda.synchronize()
    err = decode_err(dw, out, list(range(len(lens))))
    assert err <= (1e-5 if dtype == "f32" else TOL)
    if dtype != "f32":
        check_prefill(dw)
    extra = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    with pytest.raises(kun.KunError):
        kun.kun_kv_pool_extend(dw.pool, extra, extra.numel())
    dw.close()
