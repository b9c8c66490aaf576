"""GPU parity of kun_paged_prefill_chunk against the CPU oracle (through the C ABI).
bf16 inputs, fp32 accumulation: max-abs error <= 2e-2 against the fp64 oracle."""
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
    kun.kun_set_option("KUN_PREFILL_SHAPE", None)


def check_prefill(dw, rows_per_chunk=None, seed=0, only=None):
    """Compare every chunk (or the chunks in `only`; all rows, or a seeded sample of rows incl. first and
    last) with the oracle."""
    w, sh = dw.w, dw.w.shape
    out = dw.prefill()
    torch.cuda.synchronize()
    dw.check_guards()                                    # nothing was written outside the workspace asked for
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all()
    rng = np.random.default_rng(seed)
    worst = 0.0
    for i, (p, c) in enumerate(w.chunks):
        if c == 0 or (only is not None and i not in only):
            continue
        seq = w.S + i
        q0 = int(dw.q_start_host[i])
        if rows_per_chunk is None or rows_per_chunk >= c:
            rows = list(range(c))
        else:
            rows = sorted(set([0, c - 1] + list(rng.choice(c, size=rows_per_chunk, replace=False))))
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[seq]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale,
                                       rows=rows)
        err = np.abs(got[q0:q0 + c][rows] - ref).max()
        worst = max(worst, err)
        assert err <= TOL, f"chunk {i} (p={p}, c={c}): max abs err {err}"
    return worst


def set_shape(shape):
    """"default": the library's own choice; else the named variant."""
    if shape != "default":
        kun.kun_set_option("KUN_PREFILL_SHAPE", shape)


@pytest.mark.parametrize("shape", ["default", "persistent", "ring", "ring-persistent"])
@pytest.mark.parametrize("G", [4, 8, 1, 2])
def test_ragged_chunks(G, shape):
    set_shape(shape)
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=128, B=16, dtype="bf16")
    # priors / sizes around block, sub-tile (32), tile (64) and workgroup-tile edges; p = 0; c = 1
    chunks = [(0, 1), (0, 17), (5, 1), (15, 16), (16, 33), (31, 64), (63, 65), (64, 129), (100, 200), (0, 300),
              (333, 77), (700, 257), (1000, 31)]
    w = synth.custom_workload("pre", sh, [3], chunks=chunks, extra_blocks=5, range_fracs=(0.4, 0.6))
    dw = DeviceWorkload(w)
    err = check_prefill(dw)
    print("max err", err)
    dw.close()


@pytest.mark.parametrize("shape", ["default", "persistent", "ring"])
@pytest.mark.parametrize("profile", ["steps", "jump", "decay"])
def test_scores_that_outgrow_the_running_maximum(profile, shape):
    # Key magnitude changes along the context, so the rows' reference maximum has to move on tiles
    # far from the first one ("jump": by more than exp2 can hold in fp32), or never again ("decay").
    set_shape(shape)
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    chunks = [(0, 700), (512, 300), (900, 64)]
    w = synth.custom_workload("grow", sh, [], chunks=chunks, extra_blocks=0)
    dw = DeviceWorkload(w, fill=False)
    for i, (p, c) in enumerate(chunks):
        L = p + c
        k, v = synth.kv_logical(w, i, 0, L, dw.dev)
        t = torch.arange(L, device=dw.dev, dtype=torch.float32)
        if profile == "steps":
            f = 0.05 * 2.0 ** torch.floor(t / 96)             # doubles every 96 tokens
        elif profile == "jump":
            f = torch.where(t < 200, 0.02, 40.0) * torch.where(t >= 640, 4.0, 1.0)
        else:
            f = 8.0 * 0.5 ** torch.floor(t / 128)
        k = (k.float() * f[:, None, None]).to(k.dtype)
        synth.write_pages(w, dw.ranges, i, 0, L, k, v)
    err = check_prefill(dw)
    print("max err", err)
    dw.close()


@pytest.mark.parametrize("shape", ["default", "persistent"])
def test_more_work_items_than_the_plan_kernel_sorts(shape):
    # 5000 chunks (the plan kernel walks them 1024 at a time and orders only the first 4096 items),
    # most of them a few tokens, some empty, a few spanning several position tiles
    set_shape(shape)
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    rng = np.random.default_rng(33)
    c = rng.integers(1, 6, size=5000)
    p = rng.integers(0, 50, size=5000)
    c[rng.choice(5000, size=30, replace=False)] = 0
    for i, (pp, cc) in {7: (100, 300), 1023: (0, 130), 1024: (64, 64), 4095: (31, 200), 4096: (500, 70), 4999: (3, 129)}.items():
        p[i], c[i] = pp, cc
    w = synth.custom_workload("manychunks", sh, [2], chunks=list(zip(p.tolist(), c.tolist())), extra_blocks=2)
    dw = DeviceWorkload(w)
    only = set(rng.choice(5000, size=400, replace=False).tolist()) | {7, 1023, 1024, 4095, 4096, 4999, 0, 4998}
    dw.out_pre.fill_(float("nan"))
    err = check_prefill(dw, only=only)
    print("max err", err)
    # rows of empty chunks do not exist and no other row may be left unwritten: all of `out` is finite
    assert torch.isfinite(dw.out_pre.float()).all()
    dw.close()


@pytest.mark.parametrize("limit", [1, 8, 20, 96, 100000])
def test_prefill_on_a_limited_number_of_workgroups(limit):
    # any number of fetching workgroups gives the bits of the plain launch (items are independent)
    sh = synth.LayerShape(Hq=16, Hkv=4, d=128, B=16, dtype="bf16")
    chunks = [(0, 300), (700, 257), (100, 200), (64, 129), (5, 1), (333, 77), (0, 17), (1000, 31)]
    w = synth.custom_workload("lim", sh, [3], chunks=chunks, extra_blocks=5, range_fracs=(0.4, 0.6))
    dw = DeviceWorkload(w)
    ref = dw.prefill().clone()
    dw.out_pre.fill_(float("nan"))
    got = dw.prefill(max_workgroups=limit)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
    check_prefill(dw)
    with pytest.raises(kun.KunError):
        kun.kun_paged_prefill_chunk_on(dw.pool, dw.q_pre, dw.out_pre, dw.q_start, dw.prior, dw.pre_table,
                                       dw.pre_table.shape[1], dw.n_chunks, sh.Hq, dw.total_new, sh.scale, 0,
                                       dw._ws_pre, dw._ws_pre.numel())
    dw.close()


def test_mixed_batch_on_two_streams_equals_the_calls_in_sequence():
    w = synth.custom_workload("mix", synth.SHAPE_8B, [900, 3000, 17, 1500, 64] * 8,
                              chunks=[(0, 512), (1024, 512), (300, 100)], extra_blocks=4, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    ref_p = dw.prefill().clone()
    ref_d = dw.decode().clone()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for rep in range(3):
        dw.out_pre.fill_(float("nan"))
        dw.out_dec.fill_(float("nan"))
        dw.mixed(s1, s2, prefill_workgroups=16)
        torch.cuda.synchronize()
        assert torch.equal(dw.out_pre.view(torch.int16), ref_p.view(torch.int16))
        assert torch.equal(dw.out_dec.view(torch.int16), ref_d.view(torch.int16))
    check_prefill(dw)
    dw.close()


@pytest.mark.parametrize("dtype,d,G", [("f32", 64, 4), ("f32", 128, 2), ("bf16", 64, 8), ("f32", 64, 1)])
def test_shapes_outside_the_mfma_kernels(dtype, d, G):
    # fp32 and head_dim 64 go through the vector-ALU kernel, row by row; fp32: 1e-5 against the oracle
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    chunks = [(0, 1), (0, 17), (5, 1), (15, 16), (31, 64), (100, 70), (0, 130), (333, 40), (20, 0)]
    w = synth.custom_workload("gen", sh, [3], chunks=chunks, extra_blocks=5, range_fracs=(0.4, 0.6))
    dw = DeviceWorkload(w)
    dw.out_pre.fill_(float("nan"))
    out = dw.prefill()
    torch.cuda.synchronize()
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all()
    tol = 1e-5 if dtype == "f32" else TOL
    for i, (p, c) in enumerate(w.chunks):
        if c == 0:
            continue
        q0 = int(dw.q_start_host[i])
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[w.S + i]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale)
        err = np.abs(got[q0:q0 + c] - ref).max()
        assert err <= tol, f"chunk {i} (p={p}, c={c}): max abs err {err}"
    dw.close()


@pytest.mark.parametrize("shape", ["default", "persistent", "on16"])
@pytest.mark.parametrize("G", [8, 4, 1])
def test_few_query_tiles_after_long_contexts_split_their_keys(G, shape):
    # launches far too small for the chip: the keys of an item are shared out over several workgroups
    # and merged (rows that see nothing of a key range, ranges of unequal length, one-tile items)
    if shape not in ("default", "on16"):
        kun.kun_set_option("KUN_PREFILL_SHAPE", shape)
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=128, B=16, dtype="bf16")
    for chunks in ([(3000, 40)], [(2047, 1)], [(5000, 200), (17, 3)], [(0, 700)], [(1500, 64), (64, 64), (9000, 5)]):
        w = synth.custom_workload("few", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.5, 0.5))
        dw = DeviceWorkload(w)
        dw.out_pre.fill_(float("nan"))
        if shape == "on16":
            out = dw.prefill(max_workgroups=16)
            torch.cuda.synchronize()
            assert torch.isfinite(out.float()).all()
        err = check_prefill(dw) if shape != "on16" else None
        if shape == "on16":
            ref = dw.prefill().clone()
            got = dw.prefill(max_workgroups=16)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
        print(chunks, "max err", err)
        dw.close()


@pytest.mark.parametrize("shape", ["default", "ring", "persistent"])
@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 4), ("fp8", 128, 8), ("f32", 64, 2)])
def test_plan_and_planned_call_equal_the_one_call_bit_for_bit(dtype, d, G, shape):
    # kun_prefill_plan + kun_paged_prefill_chunk_planned = kun_paged_prefill_chunk: launches that fill the chip
    # and launches so small that the keys are split and merged; the plan is made before the step's
    # append (it reads neither q nor the pages); the planned call runs twice on one plan, the second
    # time with other queries; without a plan, or with the plan of another batch, it computes nothing.
    if shape != "default" and dtype != "bf16":
        pytest.skip("the other launch shapes are bf16 kernels")
    set_shape(shape)
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    bits = torch.int32 if dtype == "f32" else torch.int16
    for chunks in ([(0, 1), (15, 16), (63, 65), (100, 200), (0, 300), (700, 257)], [(3000, 40)], [(5000, 200), (17, 3)]):
        w = synth.custom_workload("planned", sh, [3], chunks=chunks, extra_blocks=5, range_fracs=(0.4, 0.6))
        dw = DeviceWorkload(w, fill=False)                # pages still poison: the plan comes before the append
        dw.prefill(steps="plan")
        torch.cuda.synchronize()
        synth.fill_pool(w, dw.ranges)
        q_a = dw.q_pre.clone()
        q_b = (-1.5 * q_a.float()).to(q_a.dtype)
        for q in (q_a, q_b):
            dw.q_pre.copy_(q)
            dw.out_pre.fill_(float("nan"))
            dw.prefill(steps="planned")
            torch.cuda.synchronize()
            dw.check_guards()
            got = dw.out_pre.clone()
            check_prefill(dw)                             # kun_paged_prefill_chunk, against the oracle
            assert torch.equal(got.view(bits), dw.out_pre.view(bits))
        if dtype != "f32":                                # (row by row there is no plan to miss)
            dw._ws_pre.fill_(0x5A)
            dw.out_pre.fill_(float("nan"))
            dw.prefill(steps="planned")
            torch.cuda.synchronize()
            dw.check_guards()
            assert torch.isnan(dw.out_pre.float()).all()
        dw.close()


@pytest.mark.parametrize("B", [64, 32, 128])
@pytest.mark.parametrize("G,d,dtype", [(8, 128, "bf16"), (4, 128, "bf16"), (1, 128, "bf16"), (2, 64, "f32")])
def test_blocks_of_64_tokens(G, d, dtype, B):
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=B, dtype=dtype)
    chunks = [(0, 1), (0, 17), (5, 1), (15, 16), (31, 64), (63, 65), (64, 129), (100, 200), (0, 300), (333, 77),
              (700, 257), (1000, 31), (3000, 40)]
    w = synth.custom_workload("b64", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.4, 0.6))
    dw = DeviceWorkload(w)
    dw.out_pre.fill_(float("nan"))
    out = dw.prefill()
    torch.cuda.synchronize()
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all()
    tol = 1e-5 if dtype == "f32" else TOL
    for i, (p, c) in enumerate(w.chunks):
        q0 = int(dw.q_start_host[i])
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[w.S + i]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale)
        err = np.abs(got[q0:q0 + c] - ref).max()
        assert err <= tol, f"chunk {i} (p={p}, c={c}): max abs err {err}"
    dw.close()


@pytest.mark.parametrize("mode", ["persistent", "on16", "split"])
@pytest.mark.parametrize("G", [8, 2])
def test_blocks_of_64_tokens_other_launches(G, mode):
    # the fetching kernel, a limited number of workgroups, launches small enough to split the keys,
    # and the other tile shapes
    if mode not in ("on16", "split"):
        kun.kun_set_option("KUN_PREFILL_SHAPE", mode)
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=128, B=(64 if G == 8 else 128), dtype="bf16")
    sets = ([(3000, 40)], [(5000, 200), (17, 3)], [(1500, 64), (64, 64), (9000, 5)]) if mode == "split" else \
        ([(0, 1), (63, 65), (64, 129), (100, 200), (0, 300), (700, 257), (1000, 31), (3000, 40), (0, 2100)],)
    for chunks in sets:
        w = synth.custom_workload("b64o", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.4, 0.6))
        dw = DeviceWorkload(w)
        dw.out_pre.fill_(float("nan"))
        if mode == "on16":
            ref = dw.prefill().clone()
            dw.out_pre.fill_(float("nan"))
            got = dw.prefill(max_workgroups=16)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
        check_prefill(dw, rows_per_chunk=48)
        dw.close()


@pytest.mark.parametrize("mode", ["default", "persistent", "on16", "split"])
@pytest.mark.parametrize("G", [5, 3, 6, 7, 16])
def test_group_sizes_that_do_not_divide_32(G, mode):
    # e.g. 40 query heads over 8 KV heads (G = 5): a wave holds floor(32 / G) whole positions and its last
    # rows are dead.  Also G = 16 (64 query heads over 4 KV heads).
    if mode == "persistent":
        kun.kun_set_option("KUN_PREFILL_SHAPE", mode)
    B = 64 if G == 6 else 16
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=128, B=B, dtype="bf16")
    sets = ([(3000, 40)], [(5000, 200), (17, 3)], [(1500, 64), (64, 64), (9000, 5)]) if mode == "split" else \
        ([(0, 1), (0, 17), (5, 1), (15, 16), (31, 64), (63, 65), (64, 129), (100, 200), (0, 300), (333, 77), (700, 257),
          (1000, 31), (0, 1100)],)
    for chunks in sets:
        w = synth.custom_workload("godd", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.4, 0.6))
        dw = DeviceWorkload(w)
        dw.out_pre.fill_(float("nan"))
        if mode == "on16":
            ref = dw.prefill().clone()
            dw.out_pre.fill_(float("nan"))
            got = dw.prefill(max_workgroups=16)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
        err = check_prefill(dw, rows_per_chunk=64)
        print(chunks[:2], "max err", err)
        dw.close()


@pytest.mark.parametrize("dtype,d,G", [("f32", 64, 5), ("f32", 128, 3), ("bf16", 64, 7)])
def test_group_sizes_outside_the_mfma_kernels(dtype, d, G):
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    chunks = [(0, 1), (5, 1), (15, 16), (63, 65), (100, 40), (333, 20)]
    w = synth.custom_workload("godd2", sh, [3], chunks=chunks, extra_blocks=3)
    dw = DeviceWorkload(w)
    dw.out_pre.fill_(float("nan"))
    out = dw.prefill()
    torch.cuda.synchronize()
    got = out.double().cpu().numpy()
    assert np.isfinite(got).all()
    tol = 1e-5 if dtype == "f32" else TOL
    for i, (p, c) in enumerate(w.chunks):
        q0 = int(dw.q_start_host[i])
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[w.S + i]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale)
        assert np.abs(got[q0:q0 + c] - ref).max() <= tol
    dw.close()


def test_empty_chunk_is_skipped_and_first_row_returns_v():
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    w = synth.custom_workload("pre0", sh, [3], chunks=[(0, 5), (7, 0), (0, 40)], extra_blocks=2)
    dw = DeviceWorkload(w)
    dw.out_pre.fill_(3.0)
    out = dw.prefill()
    torch.cuda.synchronize()
    assert torch.isfinite(out).all()
    for i in (0, 2):        # first row of a chunk with no prior tokens sees only its own token
        q0 = int(dw.q_start_host[i])
        _, v = synth.kv_logical(w, w.S + i, 0, 1)
        for h in range(sh.Hq):
            assert torch.equal(out[q0, h].cpu(), v[0, h // sh.G])
    check_prefill(dw)
    dw.close()


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 4), ("fp8", 128, 2), ("f32", 64, 2)])
def test_chunks_whose_lengths_do_not_fit_together_are_left_out(dtype, d, G):
    """A prior length below zero or beyond what the table row holds, or rows beyond the call's: the kernels
    skip that chunk (no table entry, query row or page is read for it), its output rows stay as they were
    and every other chunk comes out bit for bit as before."""
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    chunks = [(0, 40), (100, 70), (33, 20), (250, 64)]
    w = synth.custom_workload("misfit", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    ref = dw.prefill().clone()
    torch.cuda.synchronize()
    row_tokens = dw.pre_table.shape[1] * sh.B
    q_start0, prior0 = dw.q_start.clone(), dw.prior.clone()
    starts = [int(x) for x in dw.q_start_host]
    misfits = [("prior beyond the table row", 1, lambda: dw.prior.__setitem__(1, row_tokens - 70 + 1)),
               ("negative prior", 2, lambda: dw.prior.__setitem__(2, -5)),
               ("rows beyond the call", 3, lambda: dw.q_start.__setitem__(4, dw.total_new + 9))]
    for what, bad, corrupt in misfits:
        print(f"[gpu-case] {dtype} {what}", flush=True)
        corrupt()
        dw.out_pre.fill_(9.0)
        for steps in (("both",) if d == 64 else ("both", "plan+planned")):
            if steps == "both":
                got = dw.prefill()
            else:
                dw.prefill(steps="plan")
                got = dw.prefill(steps="planned")
            torch.cuda.synchronize()
            for i in range(len(chunks)):
                rows = slice(starts[i], starts[i + 1])
                if i == bad:
                    assert (got[rows] == 9.0).all(), (what, i)
                else:
                    assert torch.equal(got[rows].view(torch.int16), ref[rows].view(torch.int16)), (what, i)
        dw.q_start.copy_(q_start0)
        dw.prior.copy_(prior0)
    dw.close()


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 4), ("fp8", 128, 2), ("f32", 64, 2)])
def test_table_entries_outside_the_pool_are_not_followed(dtype, d, G):
    """Block ids below zero or beyond the pool inside a chunk's context are clamped into the pool: that chunk's
    output means nothing, every other chunk comes out bit for bit as before."""
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    chunks = [(0, 40), (100, 70), (33, 20), (250, 64)]
    w = synth.custom_workload("badids", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    ref = dw.prefill().clone()
    torch.cuda.synchronize()
    starts = [int(x) for x in dw.q_start_host]
    bad = 3
    dw.pre_table[bad, 0] = -1
    dw.pre_table[bad, 7] = 1 << 30
    dw.pre_table[bad, 19] = w.num_blocks
    print(f"[gpu-case] {dtype}: block ids outside the pool in chunk {bad}", flush=True)
    got = dw.prefill()
    torch.cuda.synchronize()
    for i in range(len(chunks)):
        if i != bad:
            rows = slice(starts[i], starts[i + 1])
            assert torch.equal(got[rows].view(torch.int16), ref[rows].view(torch.int16)), i
    dw.close()


def test_chunk_rows_equal_unchunked_prefill_on_gpu():
    # a later chunk also attends to the earlier ones: rows of chunk (p, c) == rows p..p+c-1 of (0, p+c)
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    L = 333
    w = synth.custom_workload("eq", sh, [], chunks=[(0, L), (0, 100), (100, 150), (250, 83)], extra_blocks=0)
    dw = DeviceWorkload(w, fill=False)
    k, v = synth.kv_logical(w, 0, 0, L, dw.dev)
    for i in range(4):
        synth.write_pages(w, dw.ranges, i, 0, w.chunks[i][0] + w.chunks[i][1], k[:w.chunks[i][0] + w.chunks[i][1]],
                          v[:w.chunks[i][0] + w.chunks[i][1]])
    qfull = synth.q_chunk(w, 0, dw.dev)
    dw.q_pre = torch.cat([qfull, qfull[0:100], qfull[100:250], qfull[250:333]]).contiguous()
    out = dw.prefill().clone()
    torch.cuda.synchronize()
    full = out[:L].float()
    parts = out[L:].float()
    # same keys, same arithmetic per row up to tile order: well inside the bf16 output rounding
    assert (full - parts).abs().max().item() <= 1.6e-2
    check_prefill(dw)
    dw.close()


def test_decode_equals_one_token_chunk_on_gpu():
    sh = synth.SHAPE_8B
    w = synth.custom_workload("d1", sh, [500], chunks=[(499, 1)], extra_blocks=0)
    dw = DeviceWorkload(w, fill=False)
    k, v = synth.kv_logical(w, 0, 0, 500, dw.dev)
    synth.write_pages(w, dw.ranges, 0, 0, 500, k, v)
    synth.write_pages(w, dw.ranges, 1, 0, 500, k, v)
    dw.q_pre = dw.q_dec.clone()
    a = dw.decode().float()
    b = dw.prefill().float()
    torch.cuda.synchronize()
    assert (a - b).abs().max().item() <= 1.6e-2
    dw.close()


def test_config4_prefill_chunks_sampled_rows():
    w = synth.config(4)
    dw = DeviceWorkload(w)
    err = check_prefill(dw, rows_per_chunk=48)
    print("cfg4 prefill max err", err)
    dw.close()


@pytest.mark.parametrize("mode", ["default", "persistent", "on16", "split"])
@pytest.mark.parametrize("G,B", [(8, 16), (4, 64), (1, 16), (5, 32), (16, 128)])
def test_fp8_pages_on_the_matrix_cores(G, B, mode):
    # FP8 (E4M3) pages, bf16 queries: the ping-pong kernel with E4M3 tiles in the ring.  Chunks around
    # block, sub-tile, tile and workgroup-tile edges; launches small enough to split the keys; a limited
    # number of fetching workgroups (bit-identical to the plain launch)
    if mode == "persistent":
        kun.kun_set_option("KUN_PREFILL_SHAPE", "persistent")
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=128, B=B, dtype="fp8")
    sets = ([(3000, 40)], [(5000, 200), (17, 3)], [(1500, 64), (64, 64), (9000, 5)]) if mode == "split" else \
        ([(0, 1), (0, 17), (5, 1), (15, 16), (16, 33), (31, 64), (63, 65), (64, 129), (100, 200), (0, 300), (333, 77),
          (700, 257), (1000, 31), (0, 1100)],)
    for chunks in sets:
        w = synth.custom_workload("fp8-mfma", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.4, 0.6))
        dw = DeviceWorkload(w)
        dw.out_pre.fill_(float("nan"))
        if mode == "on16":
            ref = dw.prefill().clone()
            dw.out_pre.fill_(float("nan"))
            got = dw.prefill(max_workgroups=16)
            torch.cuda.synchronize()
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
        err = check_prefill(dw, rows_per_chunk=64)
        print(chunks[:2], "max err", err)
        dw.close()


def test_fp8_pages_scores_that_outgrow_the_running_maximum():
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="fp8")
    chunks = [(0, 700), (512, 300), (900, 64)]
    w = synth.custom_workload("fp8-grow", sh, [], chunks=chunks, extra_blocks=0)
    dw = DeviceWorkload(w, fill=False)
    for i, (p, c) in enumerate(chunks):
        L = p + c
        k, v = synth.kv_logical(w, i, 0, L, dw.dev)
        t = torch.arange(L, device=dw.dev, dtype=torch.float32)
        f = torch.where(t < 200, 0.05, 8.0) * torch.where(t >= 640, 4.0, 1.0)       # key magnitude jumps twice
        k = (k.view(torch.float8_e4m3fn).float() * f[:, None, None]).to(torch.float8_e4m3fn).view(torch.uint8)
        synth.write_pages(w, dw.ranges, i, 0, L, k, v)
    err = check_prefill(dw)
    print("max err", err)
    dw.close()


@pytest.mark.parametrize("G,d,B", [(2, 64, 64), (7, 64, 16)])
def test_fp8_pages_with_head_dim_64_run_on_the_vector_alu_kernel(G, d, B):
    # prefill over FP8 (E4M3) pages: queries bf16, rows served one by one (correct to the same bar, not tuned)
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=B, dtype="fp8")
    chunks = [(0, 1), (5, 1), (15, 16), (63, 65), (100, 40), (333, 20)]
    w = synth.custom_workload("fp8-pre", sh, [3], chunks=chunks, extra_blocks=3, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    dw.out_pre.fill_(float("nan"))
    err = check_prefill(dw)
    print("max err", err)
    dw.close()
