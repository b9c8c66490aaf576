"""GPU parity of kun_paged_decode and kun_kv_append against the CPU oracle (through the C ABI).

Tolerances (max-abs error against the fp64 oracle): 1e-5 for fp32 inputs, 2e-2 for bf16 inputs
with fp32 accumulation.  Indexing and copies are bit-exact.
"""
import os

import numpy as np
import pytest
import torch

from oracle import paged_attention as O
from paper_2412_18169_amd import kun, synth
from paper_2412_18169_amd.runner import DeviceWorkload

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2, "fp8": 2e-2}    # FP8 pages: bf16 queries and outputs, the same bytes on both sides


def oracle_pool(dw):
    sh = dw.w.shape
    return O.OraclePool([synth.to_host_bits(r).reshape(-1) for r in dw.ranges], sh.Hkv, sh.d, sh.B, sh.dtype)


def check_decode(dw, seqs=None, tol=None, out=None):
    w, sh = dw.w, dw.w.shape
    S = w.S if seqs is None else seqs
    if out is None:
        out = dw.decode(seqs)
    torch.cuda.synchronize()
    dw.check_guards()                                    # nothing was written outside the workspace asked for
    ref = O.paged_decode(oracle_pool(dw), synth.to_host_bits(dw.q_dec[:S]), w.table_array(range(w.S))[:S],
                         w.decode_lens[:S], sh.Hq, sh.scale)
    got = out[:S].double().cpu().numpy()
    live = w.decode_lens[:S] > 0
    err = np.abs(got[live] - ref[live]).max() if live.any() else 0.0
    assert np.isfinite(got[live]).all()
    assert err <= (tol or TOL[sh.dtype]), f"max abs err {err}"
    return err


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    yield
    kun.kun_set_option("KUN_DECODE_KERNEL", None)
    kun.kun_set_option("KUN_DECODE_PART", None)
    kun.kun_set_option("KUN_DECODE_WAVES", None)
    kun.kun_set_option("KUN_DECODE_MAP", None)
    kun.kun_set_option("KUN_DECODE_MERGE", None)


def test_config1_tiny_fp32():
    dw = DeviceWorkload(synth.config(1))
    err = check_decode(dw)
    print("cfg1 max err", err)
    dw.close()


@pytest.mark.parametrize("kernel", ["mfma", "generic"])
@pytest.mark.parametrize("G,d,dtype", [(4, 128, "bf16"), (8, 128, "bf16"), (1, 128, "bf16"), (2, 64, "bf16"),
                                       (4, 64, "f32"), (8, 128, "f32"), (1, 64, "f32"), (2, 128, "f32")])
def test_shapes_ragged_lengths(kernel, G, d, dtype):
    if kernel == "generic":
        kun.kun_set_option("KUN_DECODE_KERNEL", "generic")
    elif not (dtype == "bf16" and d == 128):
        pytest.skip("the MFMA kernel covers bf16 with head_dim 128 only")
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    # lengths around block, pair and partition edges; several partitions for the long ones
    lens = [1, 2, 15, 16, 17, 31, 32, 33, 47, 48, 49, 255, 256, 257, 300, 511, 513, 777, 1024, 1500]
    w = synth.custom_workload("ragged", sh, lens, extra_blocks=7, range_fracs=(0.3, 0.2, 0.5))
    dw = DeviceWorkload(w)
    check_decode(dw)
    dw.close()


@pytest.mark.parametrize("part", [32, 64, 256, 1024])
@pytest.mark.parametrize("waves", [1, 2, 4])
def test_result_is_invariant_to_partitioning(part, waves):
    kun.kun_set_option("KUN_DECODE_PART", str(part))
    kun.kun_set_option("KUN_DECODE_WAVES", str(waves))
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    w = synth.custom_workload("parts", sh, [5, 40, 100, 333, 1025, 2049], extra_blocks=3)
    dw = DeviceWorkload(w)
    check_decode(dw)
    dw.close()


@pytest.mark.parametrize("kernel", ["mfma", "generic"])
@pytest.mark.parametrize("profile", ["steps", "jump", "decay"])
def test_scores_that_outgrow_the_running_maximum(profile, kernel):
    # key magnitude changes along the context: the running maximum moves late and by a lot
    # ("jump": by more than exp2 can hold in fp32), or never again ("decay")
    if kernel == "generic":
        kun.kun_set_option("KUN_DECODE_KERNEL", "generic")
    kun.kun_set_option("KUN_DECODE_PART", "256")
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    lens = [700, 1300, 64, 2500, 201]
    w = synth.custom_workload("grow", sh, lens, extra_blocks=0)
    dw = DeviceWorkload(w, fill=False)
    for s_, L in enumerate(lens):
        k, v = synth.kv_logical(w, s_, 0, L, dw.dev)
        t = torch.arange(L, device=dw.dev, dtype=torch.float32)
        if profile == "steps":
            f = 0.05 * 2.0 ** torch.clamp(torch.floor(t / 96), max=10)   # scores stay well inside fp32's precision
        elif profile == "jump":
            f = torch.where(t < 200, 0.02, 40.0) * torch.where(t >= 640, 4.0, 1.0)
        else:
            f = 8.0 * 0.5 ** torch.floor(t / 128)
        k = (k.float() * f[:, None, None]).to(k.dtype)
        synth.write_pages(w, dw.ranges, s_, 0, L, k, v)
    check_decode(dw)
    dw.close()


def test_batch_larger_than_one_pass_of_the_plan_kernel():
    # 2500 requests (the plan kernel walks the batch 1024 at a time), some empty, a few long
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    rng = np.random.default_rng(21)
    lens = rng.integers(1, 200, size=2500)
    lens[rng.choice(2500, size=40, replace=False)] = 0
    lens[[5, 1023, 1024, 2047, 2048, 2499]] = [3000, 700, 1, 5000, 16, 900]
    w = synth.custom_workload("many", sh, lens, extra_blocks=3, range_fracs=(0.5, 0.25, 0.25))
    dw = DeviceWorkload(w)
    check_decode(dw)
    dw.close()


@pytest.mark.parametrize("part", [64, 0])
def test_bound_below_the_real_context_sum_computes_whole_requests_or_none(part):
    # total_ctx_upper_bound sizes the workspace; when sum(ctx_len) is above it, the partitions that do
    # not fit are dropped by request: a row of `out` is either complete and correct or untouched
    if part:
        kun.kun_set_option("KUN_DECODE_PART", str(part))
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    lens = [700, 33, 1500, 64, 900, 2100, 5, 1200, 300, 800] * 3
    w = synth.custom_workload("bound", sh, lens, extra_blocks=3, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    ref = dw.decode().clone()
    torch.cuda.synchronize()
    for bound in (sum(lens) // 2, 256, 1):
        dw._ws_dec = None
        dw.out_dec.fill_(float("nan"))
        got = dw.decode(ctx_bound=bound).clone()
        torch.cuda.synchronize()
        done = 0
        for s_ in range(len(lens)):
            if torch.isnan(got[s_].float()).all():
                continue
            assert torch.equal(got[s_].view(torch.int16), ref[s_].view(torch.int16)), (bound, s_)
            done += 1
        print("bound", bound, "of", sum(lens), ":", done, "requests computed")
        assert done < len(lens)
        if bound > 1000:
            assert done > 0
    kun.kun_set_option("KUN_DECODE_PART", None)
    dw.close()


@pytest.mark.parametrize("B", [16, 64])
def test_workgroup_order_does_not_change_a_bit(B):
    # XCD-aware order (default) against item-major order, with a number of work items that is not a
    # multiple of 8 and requests of one and of many partitions
    sh = synth.LayerShape(Hq=16, Hkv=2, d=128, B=B, dtype="bf16")
    lens = [700, 33, 1500, 64, 900, 2100, 5, 1200, 300, 800, 4100]
    w = synth.custom_workload("order", sh, lens, extra_blocks=3, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    outs = {}
    for mode in ("xcd", "flat"):
        kun.kun_set_option("KUN_DECODE_MAP", mode)
        dw.out_dec.fill_(float("nan"))
        outs[mode] = dw.decode().clone()
        torch.cuda.synchronize()
    kun.kun_set_option("KUN_DECODE_MAP", None)
    assert torch.isfinite(outs["xcd"].float()).all()
    assert torch.equal(outs["xcd"].view(torch.int16), outs["flat"].view(torch.int16))
    check_decode(dw)
    dw.close()


@pytest.mark.parametrize("dtype,d,G,B", [("bf16", 128, 5, 16), ("bf16", 128, 3, 64), ("bf16", 128, 6, 16), ("bf16", 128, 7, 16),
                                         ("f32", 64, 5, 16), ("f32", 128, 3, 16), ("bf16", 64, 7, 64),
                                         ("bf16", 128, 16, 16), ("bf16", 128, 16, 64)])
def test_any_number_of_query_heads_per_kv_head_up_to_8(dtype, d, G, B):
    # e.g. 40 query heads over 8 KV heads (G = 5); also 16 (64 over 4), on the MFMA kernel only
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=B, dtype=dtype)
    lens = [1, 15, 16, 17, 33, 64, 200, 513, 700, 1500, 2100]
    w = synth.custom_workload("gany", sh, lens, extra_blocks=3, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w)
    for part in (None, "64"):
        if part:
            kun.kun_set_option("KUN_DECODE_PART", part)
        dw._ws_dec = None
        dw.out_dec.fill_(float("nan"))
        check_decode(dw)
    dw.close()


def test_empty_calls_and_refused_arguments_leave_outputs_alone():
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    w = synth.custom_workload("empty", sh, [0, 0, 0], chunks=[(5, 0)], extra_blocks=4)
    dw = DeviceWorkload(w)
    dw.out_dec.fill_(3.0)
    out = dw.decode()                                   # every request has ctx_len 0
    torch.cuda.synchronize()
    assert torch.all(out == 3.0)
    dev = dw.dev
    ws = torch.empty(1 << 20, dtype=torch.uint8, device=dev)
    z = torch.zeros(4, dtype=torch.int32, device=dev)
    # S = 0, n_chunks = 0, T = 0: nothing is launched, nothing is dereferenced
    kun.kun_paged_decode(dw.pool, None, None, None, 1, None, 0, sh.Hq, sh.scale, 0, None, 0)
    kun.kun_paged_prefill_chunk(dw.pool, None, None, None, None, None, 1, 0, sh.Hq, 0, sh.scale, None, 0)
    kun.kun_kv_append(dw.pool, None, None, None, None, 0, None, 1)
    kun.kun_slot_map(dw.pool, None, None, 0, None, 1, 0, None, None, None)
    dw.out_pre.fill_(5.0) if dw.n_chunks and dw.out_pre.numel() else None
    dw.prefill()                                        # one chunk with c = 0
    torch.cuda.synchronize()

    def status(fn, *a):
        with pytest.raises(kun.KunError) as e:
            fn(*a)
        return e.value.status
    q, o, tab, ln = dw.q_dec, dw.out_dec, dw.dec_table, dw.dec_len
    need = kun.kun_decode_workspace_bytes(dw.pool, 3, sh.Hq, 0)
    assert need > 0 and need % 256 == 0
    assert status(kun.kun_paged_decode, dw.pool, q, o, tab, tab.shape[1], ln, 3, sh.Hq, sh.scale, 0, ws, 256) == -6
    assert status(kun.kun_paged_decode, dw.pool, q, o, tab, tab.shape[1], ln, 3, sh.Hq, sh.scale, 0, None, need) == -6
    big = torch.empty(need + 512, dtype=torch.uint8, device=dev)
    assert status(kun.kun_paged_decode, dw.pool, q, o, tab, tab.shape[1], ln, 3, sh.Hq, sh.scale, 0,
                  big.data_ptr() + 8, need) == -6                                     # misaligned workspace
    assert status(kun.kun_paged_decode, dw.pool, q, o, tab, tab.shape[1], ln, 3, 18, sh.scale, 0, big, need) == -8  # G = 9
    assert status(kun.kun_paged_decode, dw.pool, q, o, tab, tab.shape[1], ln, 3, 7, sh.scale, 0, big, need) == -1   # 7 % 2
    assert status(kun.kun_paged_decode, dw.pool, None, o, tab, tab.shape[1], ln, 3, sh.Hq, sh.scale, 0, big, need) == -1
    assert status(kun.kun_paged_prefill_chunk, dw.pool, q, o, z, z, tab, tab.shape[1], 1, 18, 4, sh.scale, big, need) == -8
    kun.kun_set_option("KUN_DECODE_KERNEL", "generic")            # 16 heads per KV head: not on the vector-ALU kernel
    assert status(kun.kun_paged_decode, dw.pool, q, o, tab, tab.shape[1], ln, 3, 32, sh.scale, 0, big, need) == -8
    kun.kun_set_option("KUN_DECODE_KERNEL", None)
    assert status(kun.kun_slot_map, dw.pool, z, z, 2, tab, tab.shape[1], 5, z, z, z) == -1           # kv head 5 of 2
    torch.cuda.synchronize()
    assert torch.all(dw.out_dec == 3.0)
    dw.close()


@pytest.mark.parametrize("B", [64, 32, 128])
@pytest.mark.parametrize("G,d,dtype", [(8, 128, "bf16"), (4, 128, "bf16"), (2, 64, "bf16"), (4, 64, "f32"), (1, 128, "f32")])
def test_blocks_of_64_tokens(G, d, dtype, B):
    # the paper's tuned block size (Section 5.1), and 32 and 128: decode, append and the slot map
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=B, dtype=dtype)
    lens = [1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 513, 777, 1024, 1500, 4100]
    w = synth.custom_workload("b64", sh, lens, extra_blocks=3, range_fracs=(0.3, 0.2, 0.5))
    dw = DeviceWorkload(w, fill=False)
    # pages written by kun_kv_append (bit-exact against the oracle's append), then decode
    seqs, poss, ks, vs = [], [], [], []
    for s_ in range(len(lens)):
        k, v = synth.kv_logical(w, s_, 0, lens[s_])
        ks.append(k); vs.append(v)
        seqs += [s_] * lens[s_]; poss += list(range(lens[s_]))
    k_new, v_new = torch.cat(ks), torch.cat(vs)
    seqs, poss = np.asarray(seqs, dtype=np.int32), np.asarray(poss, dtype=np.int32)
    table = w.table_array(range(len(lens)))
    opool = O.OraclePool([synth.to_host_bits(r).reshape(-1).copy() for r in dw.ranges], sh.Hkv, sh.d, sh.B, sh.dtype)
    O.kv_append(opool, synth.to_host_bits(k_new), synth.to_host_bits(v_new), seqs, poss, table)
    kun.kun_kv_append(dw.pool, k_new.cuda(), v_new.cuda(), torch.from_numpy(seqs).cuda(), torch.from_numpy(poss).cuda(),
                      len(seqs), torch.from_numpy(table).cuda(), table.shape[1])
    torch.cuda.synchronize()
    for r in range(len(dw.ranges)):
        assert np.array_equal(synth.to_host_bits(dw.ranges[r]).reshape(-1), opool.ranges[r], equal_nan=True)
    for kernel in ("default", "generic"):
        if kernel == "generic":
            kun.kun_set_option("KUN_DECODE_KERNEL", "generic")
        for part in (None, "64", "256"):
            if part:
                kun.kun_set_option("KUN_DECODE_PART", part)
            dw.out_dec.fill_(float("nan"))
            check_decode(dw)
            kun.kun_set_option("KUN_DECODE_PART", None)
    dw.close()


def test_length_one_returns_v_exactly_and_zero_length_is_skipped():
    for dtype, d in (("bf16", 128), ("f32", 64)):
        sh = synth.LayerShape(Hq=8, Hkv=2, d=d, B=16, dtype=dtype)
        w = synth.custom_workload("one", sh, [1, 0, 1, 5], extra_blocks=2)
        dw = DeviceWorkload(w)
        dw.out_dec.fill_(7.0)
        out = dw.decode()
        torch.cuda.synchronize()
        for s in (0, 2):
            _, v = synth.kv_logical(w, s, 0, 1)
            for h in range(sh.Hq):
                assert torch.equal(out[s, h].cpu(), v[0, h // sh.G]), (dtype, s, h)
        assert torch.all(out[1] == 7.0)           # ctx_len 0: output row untouched
        check_decode(dw, out=out)
        dw.close()


@pytest.mark.parametrize("dtype,d,merge", [("bf16", 128, "fold"), ("bf16", 128, "kernel"), ("fp8", 128, "fold"),
                                           ("f32", 64, "kernel")])
def test_a_context_longer_than_the_table_row_is_left_out(dtype, d, merge):
    """ctx_len above max_blocks * block_size cannot be served from the table row: the request is skipped
    (row untouched), the others come out bit for bit as before."""
    kun.kun_set_option("KUN_DECODE_MERGE", merge)
    kun.kun_set_option("KUN_DECODE_PART", "256")
    try:
        sh = synth.LayerShape(Hq=8, Hkv=2, d=d, B=16, dtype=dtype)
        lens = [700, 33, 1300, 5, 260]
        # (spare blocks: the bound on sum(ctx_len) is capped by the pool's capacity, and the corrupted sum must fit)
        w = synth.custom_workload("toolong", sh, lens, extra_blocks=100, range_fracs=(0.6, 0.4))
        dw = DeviceWorkload(w)
        row_tokens = dw.dec_table.shape[1] * sh.B
        bound = sum(lens) + row_tokens + 1
        ref = dw.decode(ctx_bound=bound).clone()
        torch.cuda.synchronize()
        for bad in (2, 3):
            print(f"[gpu-case] {dtype} merge={merge}: request {bad} longer than its table row", flush=True)
            keep = dw.dec_len.clone()
            dw.dec_len[bad] = row_tokens + 1
            dw.out_dec.fill_(5.0)
            got = dw.decode(ctx_bound=bound)
            torch.cuda.synchronize()
            for s_ in range(len(lens)):
                if s_ == bad:
                    assert (got[s_] == 5.0).all()
                else:
                    assert torch.equal(got[s_].view(torch.uint8), ref[s_].view(torch.uint8)), s_
            dw.dec_len.copy_(keep)
        dw.close()
    finally:
        kun.kun_set_option("KUN_DECODE_MERGE", None)
        kun.kun_set_option("KUN_DECODE_PART", None)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp8", 128), ("f32", 64)])
def test_table_entries_outside_the_pool_are_not_followed(dtype, d):
    """Block ids below zero or beyond the pool inside a request's context: the kernels clamp them into the
    pool (the request's output then means nothing) and every other request comes out bit for bit as before."""
    sh = synth.LayerShape(Hq=8, Hkv=2, d=d, B=16, dtype=dtype)
    lens = [700, 33, 1300, 5, 260]
    w = synth.custom_workload("badids", sh, lens, extra_blocks=4, range_fracs=(0.6, 0.4))
    dw = DeviceWorkload(w)
    ref = dw.decode().clone()
    torch.cuda.synchronize()
    bad = 2
    dw.dec_table[bad, 3] = -1
    dw.dec_table[bad, 40] = 1 << 30
    dw.dec_table[bad, 41] = w.num_blocks
    dw.dec_table[bad, 80] = -(1 << 31)
    print(f"[gpu-case] {dtype}: block ids outside the pool in request {bad}", flush=True)
    got = dw.decode()
    torch.cuda.synchronize()
    for s_ in range(len(lens)):
        if s_ != bad:
            assert torch.equal(got[s_].view(torch.uint8), ref[s_].view(torch.uint8)), s_
    dw.close()


def test_block_permutation_gives_bit_identical_output():
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    lens = [3, 100, 700, 1300]
    outs = []
    for seed, fracs in [(1, (1.0,)), (2, (0.5, 0.5)), (3, (0.2, 0.3, 0.5))]:
        w = synth.custom_workload("perm", sh, lens, seed=11, extra_blocks=9, range_fracs=fracs)
        rng = np.random.default_rng(seed)
        ids = rng.permutation(w.num_blocks).astype(np.int32)
        o = 0
        for i, n in enumerate(synth.blocks_needed(w.seq_lens, 16)):
            w.block_tables[i] = ids[o:o + int(n)]
            o += int(n)
        dw = DeviceWorkload(w)
        outs.append(dw.decode().clone())
        check_decode(dw)
        dw.close()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_pool_extension_keeps_resident_outputs_bit_identical():
    # three ranges (40/30/30 %), admitted in phases: decode after every extension
    sh = synth.SHAPE_8B
    rng = np.random.default_rng(5)
    lens = synth.lognormal_lengths(rng, 24, median=300, sigma=0.8, lo=16, hi=3000)
    w = synth.Workload("phased", 0, 77, sh, lens, [], [])
    n = int(synth.blocks_needed(lens, 16).sum())
    w.range_blocks = [int(0.4 * n), int(0.3 * n), n - int(0.4 * n) - int(0.3 * n)]
    resident = synth.assign_blocks_phased(w)
    dw = DeviceWorkload(w, n_ranges_at_create=1)
    used = np.concatenate(w.block_tables)
    r, _ = synth.range_of_blocks(w.range_blocks, used.astype(np.int64))
    assert set(np.unique(r)) == {0, 1, 2}
    for phase, nres in enumerate(resident):
        if phase > 0:
            first, nb = dw.extend_next()
            assert first == sum(w.range_blocks[:phase]) and nb == w.range_blocks[phase]
        assert nres > 0
        out = dw.decode(nres).clone()
        check_decode(dw, seqs=nres, out=out)
    # resident requests: bit-identical across extend (partition size pinned, so the split of a
    # request does not depend on how many requests are in the batch)
    kun.kun_set_option("KUN_DECODE_PART", "256")
    dw2 = DeviceWorkload(w, n_ranges_at_create=1)
    a = dw2.decode(resident[0]).clone()
    dw2.extend_next(); dw2.extend_next()
    b = dw2.decode(resident[0]).clone()
    c = dw2.decode(resident[2]).clone()
    torch.cuda.synchronize()
    assert torch.equal(a[:resident[0]], b[:resident[0]]) and torch.equal(a[:resident[0]], c[:resident[0]])
    dw.close(); dw2.close()


def test_extend_between_enqueued_calls_disturbs_neither():
    # the range table travels with every launch: a call enqueued before kun_kv_pool_extend keeps the
    # table it was given, a call enqueued after sees the new range, no synchronisation in between
    kun.kun_set_option("KUN_DECODE_PART", "256")
    sh = synth.SHAPE_8B
    rng = np.random.default_rng(8)
    lens = synth.lognormal_lengths(rng, 48, median=600, sigma=0.7, lo=16, hi=4000)
    w = synth.Workload("inflight", 0, 78, sh, lens, [], [])
    n = int(synth.blocks_needed(lens, 16).sum())
    w.range_blocks = [n // 2, n - n // 2]
    resident = synth.assign_blocks_phased(w)
    dw = DeviceWorkload(w, n_ranges_at_create=1)
    ref_a = dw.decode(resident[0]).clone()
    dw.extend_next()
    ref_b = dw.decode(resident[1]).clone()
    torch.cuda.synchronize()
    dw2 = DeviceWorkload(w, n_ranges_at_create=1)
    out_a = torch.empty_like(dw2.out_dec)
    dw2.decode(resident[0])
    out_a.copy_(dw2.out_dec, non_blocking=True)          # enqueued behind the first call
    dw2.extend_next()                                    # host only; the first call may still be running
    out_b = dw2.decode(resident[1])
    torch.cuda.synchronize()
    assert torch.equal(out_a[:resident[0]], ref_a[:resident[0]])
    assert torch.equal(out_b[:resident[1]], ref_b[:resident[1]])
    check_decode(dw2, seqs=resident[1], out=out_b)
    dw.close(); dw2.close()


def test_resolve_matches_oracle_on_device_pool():
    small = synth.Workload("r", 0, 1, synth.SHAPE_8B, np.array([100, 333, 20], dtype=np.int32), [], [50, 20, 30])
    synth.assign_blocks_scattered(small)
    dw = DeviceWorkload(small, fill=False, poison=False)
    for blk in range(100):
        r, off, addr = kun.kun_kv_pool_resolve(dw.pool, blk)
        assert (r, off) == O.block_byte_offset(small.range_blocks, blk, small.shape.block_bytes)
        assert addr == dw.ranges[r].data_ptr() + off
    dw.close()


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_kv_append_is_bit_exact(dtype, d):
    sh = synth.LayerShape(Hq=4, Hkv=4, d=d, B=16, dtype=dtype)
    w = synth.custom_workload("app", sh, [37, 1, 16, 250], chunks=[(20, 70)], extra_blocks=5, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w, fill=False)
    ref_ranges = synth.alloc_ranges(w, "cpu")
    synth.fill_pool(w, ref_ranges)
    # oracle-side append on a host copy, from the same rows
    seqs, poss, ks, vs = [], [], [], []
    lens = w.seq_lens
    for s in range(len(lens)):
        k, v = synth.kv_logical(w, s, 0, int(lens[s]))
        ks.append(k); vs.append(v)
        seqs += [s] * int(lens[s]); poss += list(range(int(lens[s])))
    order = np.random.default_rng(0).permutation(len(seqs))          # tokens in arbitrary order
    k_new = torch.cat(ks)[order]; v_new = torch.cat(vs)[order]
    seqs = np.asarray(seqs, dtype=np.int32)[order]; poss = np.asarray(poss, dtype=np.int32)[order]
    table = w.table_array(range(len(lens)))
    opool = O.OraclePool([synth.to_host_bits(r).reshape(-1).copy() for r in synth.alloc_ranges(w, "cpu")],
                         sh.Hkv, sh.d, sh.B, sh.dtype)
    O.kv_append(opool, synth.to_host_bits(k_new), synth.to_host_bits(v_new), seqs, poss, table)
    kun.kun_kv_append(dw.pool, k_new.cuda(), v_new.cuda(), torch.from_numpy(seqs).cuda(),
                      torch.from_numpy(poss).cuda(), len(seqs), torch.from_numpy(table).cuda(), table.shape[1])
    torch.cuda.synchronize()
    for r in range(len(dw.ranges)):
        got = synth.to_host_bits(dw.ranges[r]).reshape(-1)
        assert np.array_equal(got, opool.ranges[r], equal_nan=True)
        assert np.array_equal(got, synth.to_host_bits(ref_ranges[r]).reshape(-1), equal_nan=True)
    dw.close()


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_kv_append_leaves_out_tokens_that_the_table_cannot_place(dtype, d):
    """Rows or positions below zero, positions beyond the table row, table entries that are no block of
    the pool: nothing is written for such tokens, every other token lands bit-exactly (the oracle appends
    the placeable tokens only), and the slot map reports -1 for the others."""
    sh = synth.LayerShape(Hq=4, Hkv=4, d=d, B=16, dtype=dtype)
    w = synth.custom_workload("app-bad", sh, [37, 1, 16, 250], chunks=[(20, 70)], extra_blocks=5, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w, fill=False)
    lens = w.seq_lens
    seqs, poss, ks, vs = [], [], [], []
    for s in range(len(lens)):
        k, v = synth.kv_logical(w, s, 0, int(lens[s]))
        ks.append(k); vs.append(v)
        seqs += [s] * int(lens[s]); poss += list(range(int(lens[s])))
    k_new = torch.cat(ks); v_new = torch.cat(vs)
    seqs = np.asarray(seqs, dtype=np.int32); poss = np.asarray(poss, dtype=np.int32)
    table = w.table_array(range(len(lens))).copy()
    row_tokens = table.shape[1] * sh.B
    rng = np.random.default_rng(4)
    bad = rng.choice(len(seqs), size=24, replace=False)
    poss[bad[:8]] = -1 - rng.integers(0, 50, size=8)              # positions below zero
    poss[bad[8:16]] = row_tokens + rng.integers(0, 50, size=8)    # positions beyond the table row
    seqs[bad[16:24]] = -1 - rng.integers(0, 3, size=8)            # rows below zero
    table[3, 2] = -1                                              # tokens 32..47 of request 3: no block
    table[3, 7] = w.num_blocks                                    # tokens 112..127: one past the last block
    table[4, 1] = -7                                              # the chunk's request, tokens 16..31
    placeable = np.array([seqs[i] >= 0 and 0 <= poss[i] < row_tokens and 0 <= table[seqs[i], poss[i] // sh.B] < w.num_blocks
                          for i in range(len(seqs))])
    assert 50 < (~placeable).sum() < len(seqs) // 2
    opool = O.OraclePool([synth.to_host_bits(r).reshape(-1).copy() for r in dw.ranges], sh.Hkv, sh.d, sh.B, sh.dtype)
    O.kv_append(opool, synth.to_host_bits(k_new)[placeable], synth.to_host_bits(v_new)[placeable], seqs[placeable],
                poss[placeable], table)
    dseq, dpos, dtab = torch.from_numpy(seqs).cuda(), torch.from_numpy(poss).cuda(), torch.from_numpy(table).cuda()
    print(f"[gpu-case] append with {int((~placeable).sum())} unplaceable tokens of {len(seqs)}, {dtype}", flush=True)
    kun.kun_kv_append(dw.pool, k_new.cuda(), v_new.cuda(), dseq, dpos, len(seqs), dtab, table.shape[1])
    torch.cuda.synchronize()
    for r in range(len(dw.ranges)):
        assert np.array_equal(synth.to_host_bits(dw.ranges[r]).reshape(-1), opool.ranges[r], equal_nan=True)
    rng_out = torch.empty(len(seqs), dtype=torch.int32, device="cuda")
    k_off = torch.empty(len(seqs), dtype=torch.int64, device="cuda")
    v_off = torch.empty(len(seqs), dtype=torch.int64, device="cuda")
    kun.kun_slot_map(dw.pool, dseq, dpos, len(seqs), dtab, table.shape[1], 1, rng_out, k_off, v_off)
    torch.cuda.synchronize()
    gone = torch.from_numpy(~placeable).cuda()
    assert (rng_out[gone] == -1).all() and (k_off[gone] == -1).all() and (v_off[gone] == -1).all()
    assert (rng_out[~gone] >= 0).all() and (k_off[~gone] >= 0).all() and (v_off[~gone] > 0).all()
    dw.close()


def test_generator_is_identical_on_device_and_host():
    a = synth.normal_values(1003, synth.TENSOR_K, 17, 12345, 100000, torch.bfloat16, "cuda")
    b = synth.normal_values(1003, synth.TENSOR_K, 17, 12345, 100000, torch.bfloat16, "cpu")
    assert torch.equal(a.cpu(), b)


def test_config2_8b_decode_full_parity():
    w = synth.config(2)
    dw = DeviceWorkload(w)
    kun.kun_validate_block_table(dw.pool, torch.from_numpy(w.table_array(range(w.S))),
                                 torch.from_numpy(w.decode_lens.astype(np.int32)))
    err = check_decode(dw)
    print("cfg2 max err", err)
    dw.close()


def test_merged_records_are_fresh_when_the_workspace_is_reused():
    # The last workgroup of a (request, kv head) to finish merges the partial records that the other
    # partitions -- on other XCDs, behind other L2 caches -- have written.  A stale read would pick up
    # the records of the call before: so the same workspace serves calls with different queries in
    # turn, many multi-partition requests each, and every output is checked against the oracle.
    sh = synth.LayerShape(Hq=32, Hkv=8, d=128, B=16, dtype="bf16")
    rng = np.random.default_rng(5)
    lens = rng.integers(600, 5000, size=96).tolist()
    w = synth.custom_workload("fresh", sh, lens, extra_blocks=3, range_fracs=(0.5, 0.5))
    kun.kun_set_option("KUN_DECODE_PART", "256")         # 3 to 20 partitions per request
    kun.kun_set_option("KUN_DECODE_MERGE", "fold")
    dw = DeviceWorkload(w)
    q_a = dw.q_dec.clone()
    q_b = (-2.0 * q_a.float()).to(q_a.dtype)
    outs = {}
    for name, q in (("a", q_a), ("b", q_b), ("a", q_a), ("b", q_b)):
        dw.q_dec.copy_(q)
        dw.out_dec.fill_(float("nan"))
        check_decode(dw)
        got = dw.out_dec.clone()
        if name in outs:
            assert torch.equal(got.view(torch.int16), outs[name].view(torch.int16))
        outs[name] = got
    assert not torch.equal(outs["a"].view(torch.int16), outs["b"].view(torch.int16))
    dw.close()


@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 4), ("f32", 64, 2)])
def test_merge_inside_the_partial_kernel_and_as_a_launch_of_its_own_give_the_same_bits(dtype, d, G):
    # small batches merge the split-K records in the partial kernel (last workgroup to arrive), large
    # ones in a separate launch; both combine the records in partition order with the same arithmetic
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    lens = [1, 255, 256, 257, 700, 1025, 2049, 3000, 64, 0, 513]
    w = synth.custom_workload("merge-modes", sh, lens, extra_blocks=3, range_fracs=(0.4, 0.6))
    kun.kun_set_option("KUN_DECODE_PART", "256")
    dw = DeviceWorkload(w)
    outs = []
    for mode in ("fold", "kernel", "auto"):
        kun.kun_set_option("KUN_DECODE_MERGE", mode)
        dw.out_dec.fill_(float("nan"))
        check_decode(dw)
        outs.append(dw.out_dec.clone())
    live = torch.tensor([L > 0 for L in lens], device=outs[0].device)
    bits = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(outs[0][live].view(bits), outs[1][live].view(bits))
    assert torch.equal(outs[0][live].view(bits), outs[2][live].view(bits))
    dw.close()


@pytest.mark.parametrize("merge", ["fold", "kernel"])
@pytest.mark.parametrize("dtype,d,G", [("bf16", 128, 4), ("fp8", 128, 8), ("f32", 64, 2)])
def test_one_plan_serves_many_calls_bit_for_bit(dtype, d, G, merge):
    # kun_decode_plan + kun_paged_decode_planned = kun_paged_decode: the work list depends on the context
    # lengths only, so one plan serves every layer of a step.  The planned call runs three times on one
    # plan (the arrival counters of the folded merge go back to zero by themselves), the second time with
    # other queries, and once against another pool of the same shape (another layer's cache: other
    # contents, other block ids) through the first pool's workspace.
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=16, dtype=dtype)
    lens = [1, 255, 256, 257, 700, 1025, 2049, 3000, 64, 0, 513]
    w = synth.custom_workload("planned", sh, lens, extra_blocks=3, range_fracs=(0.4, 0.6))
    w2 = synth.custom_workload("planned-layer-2", sh, lens, seed=11, extra_blocks=9, range_fracs=(0.7, 0.3))
    kun.kun_set_option("KUN_DECODE_PART", "256")
    kun.kun_set_option("KUN_DECODE_MERGE", merge)
    dw, dw2 = DeviceWorkload(w), DeviceWorkload(w2)
    bits = torch.int32 if dtype == "f32" else torch.int16
    live = torch.tensor([L > 0 for L in lens], device=dw.dev)
    q_a = dw.q_dec.clone()
    q_b = (-2.0 * q_a.float()).to(q_a.dtype)
    want = {}
    for name, q in (("a", q_a), ("b", q_b)):
        dw.q_dec.copy_(q)
        dw.out_dec.fill_(float("nan"))
        check_decode(dw)
        want[name] = dw.out_dec.clone()
    dw2.out_dec.fill_(float("nan"))
    check_decode(dw2)
    want2 = dw2.out_dec.clone()

    dw.decode(steps="plan")
    for name, q in (("a", q_a), ("b", q_b), ("a", q_a)):
        dw.q_dec.copy_(q)
        dw.out_dec.fill_(float("nan"))
        dw.decode(steps="planned")
        torch.cuda.synchronize()
        dw.check_guards()
        assert torch.equal(dw.out_dec[live].view(bits), want[name][live].view(bits)), name
        assert torch.isnan(dw.out_dec[~live].float()).all()            # the request of length 0 is left alone
    # the other pool, through the first one's plan and workspace
    sh2 = w2.shape
    ctx_bound = int(np.asarray(lens, dtype=np.int64).sum())
    dw2.out_dec.fill_(float("nan"))
    kun.kun_paged_decode_planned(dw2.pool, dw2.q_dec, dw2.out_dec, dw2.dec_table, dw2.dec_table.shape[1], dw.dec_len,
                                 len(lens), sh2.Hq, sh2.scale, ctx_bound, dw._ws_dec, dw._ws_dec.numel())
    torch.cuda.synchronize()
    dw.check_guards()
    assert torch.equal(dw2.out_dec[live].view(bits), want2[live].view(bits))
    # and the first pool once more on the same plan
    dw.q_dec.copy_(q_b)
    dw.out_dec.fill_(float("nan"))
    dw.decode(steps="planned")
    torch.cuda.synchronize()
    assert torch.equal(dw.out_dec[live].view(bits), want["b"][live].view(bits))
    dw.close()
    dw2.close()


def test_a_planned_call_without_its_plan_computes_nothing():
    # kun_paged_decode_planned on a workspace that holds no plan, or the plan of another batch shape,
    # finds the wrong tag behind the list length and leaves the outputs alone (no list entry is followed)
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="bf16")
    lens = [300, 17, 1025, 64]
    w = synth.custom_workload("no-plan", sh, lens, extra_blocks=2)
    kun.kun_set_option("KUN_DECODE_PART", "256")
    dw = DeviceWorkload(w)
    dw.decode()                                           # sizes the workspace
    torch.cuda.synchronize()
    want = dw.out_dec.clone()
    for fill in (0x00, 0xFF, 0x5A):                       # no plan at all: arbitrary bytes
        dw._ws_dec.fill_(fill)
        dw.out_dec.fill_(float("nan"))
        dw.decode(steps="planned")
        torch.cuda.synchronize()
        dw.check_guards()
        assert torch.isnan(dw.out_dec.float()).all()
    dw.decode(seqs=3, steps="plan")                       # the plan of another batch (3 requests)
    dw.out_dec.fill_(float("nan"))
    dw.decode(steps="planned")
    torch.cuda.synchronize()
    assert torch.isnan(dw.out_dec.float()).all()
    dw.decode(steps="plan")                               # its own plan: the result of the one-call form
    dw.decode(steps="planned")
    torch.cuda.synchronize()
    assert torch.equal(dw.out_dec.view(torch.int16), want.view(torch.int16))
    dw.close()


# ------------------------------------------------------------------------------------------
# FP8 (E4M3) pages: half the bytes per token; queries and outputs bf16; same tolerance (the
# oracle reads the same bytes)
# ------------------------------------------------------------------------------------------

@pytest.mark.parametrize("kernel", ["mfma", "generic"])
@pytest.mark.parametrize("G,d,B", [(4, 128, 16), (8, 128, 16), (1, 128, 64), (5, 128, 32), (16, 128, 16), (2, 64, 16), (8, 64, 128)])
def test_fp8_pages_ragged_lengths(kernel, G, d, B):
    if kernel == "generic":
        if G == 16:
            pytest.skip("16 query heads per KV head: the matrix-core kernel only")
        kun.kun_set_option("KUN_DECODE_KERNEL", "generic")
    elif d != 128:
        pytest.skip("the matrix-core kernel covers head_dim 128 only")
    sh = synth.LayerShape(Hq=2 * G, Hkv=2, d=d, B=B, dtype="fp8")
    # lengths around tile (16), quad (64) and partition edges; several partitions for the long ones
    lens = [1, 2, 15, 16, 17, 47, 48, 49, 63, 64, 65, 127, 128, 129, 255, 256, 257, 300, 511, 513, 777, 1024, 1500, 0]
    w = synth.custom_workload("fp8-ragged", sh, lens, extra_blocks=7, range_fracs=(0.3, 0.2, 0.5))
    dw = DeviceWorkload(w)
    for part in (None, "64", "96"):
        kun.kun_set_option("KUN_DECODE_PART", part)
        for waves in ((4, 1, 2) if kernel == "mfma" else (4,)):
            kun.kun_set_option("KUN_DECODE_WAVES", waves)
            dw.out_dec.fill_(float("nan"))
            dw._ws_dec = None
            check_decode(dw)
    dw.close()


def test_fp8_append_is_bit_exact_and_length_one_returns_v_exactly():
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="fp8")
    lens = [1, 40, 17]
    w = synth.custom_workload("fp8-append", sh, lens, extra_blocks=2, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w, fill=False)
    opool = oracle_pool(dw)                            # NaN codes everywhere
    ks, vs, seqs, poss = [], [], [], []
    for s_, L in enumerate(lens):
        k, v = synth.kv_logical(w, s_, 0, L, "cpu")
        ks.append(k); vs.append(v); seqs += [s_] * L; poss += list(range(L))
    k_new, v_new = torch.cat(ks).contiguous(), torch.cat(vs).contiguous()
    order = np.random.default_rng(3).permutation(len(seqs))
    k_new, v_new = k_new[order], v_new[order]
    seqs, poss = np.asarray(seqs, dtype=np.int32)[order], np.asarray(poss, dtype=np.int32)[order]
    table = w.table_array(range(w.S))
    O.kv_append(opool, k_new.numpy(), v_new.numpy(), seqs, poss, table)
    kun.kun_kv_append(dw.pool, k_new.cuda(), v_new.cuda(), torch.from_numpy(seqs).cuda(), torch.from_numpy(poss).cuda(),
                      len(seqs), torch.from_numpy(table).cuda(), table.shape[1])
    torch.cuda.synchronize()
    for r in range(len(dw.ranges)):
        assert np.array_equal(synth.to_host_bits(dw.ranges[r]).reshape(-1), opool.ranges[r])
    out = dw.decode()
    torch.cuda.synchronize()
    check_decode(dw, out=out)
    # a context of one token: the output is that token's V, exactly (E4M3 values are bf16 values)
    _, v0 = synth.kv_logical(w, 0, 0, 1, "cpu")
    want = v0.view(torch.float8_e4m3fn).to(torch.bfloat16)[0]           # [Hkv, d]
    got = out[0].cpu().view(sh.Hkv, sh.G, sh.d)
    for g in range(sh.G):
        assert torch.equal(got[:, g].view(torch.int16), want.view(torch.int16))
    dw.close()


def test_fp8_scores_that_outgrow_the_running_maximum():
    kun.kun_set_option("KUN_DECODE_PART", "256")
    sh = synth.LayerShape(Hq=8, Hkv=2, d=128, B=16, dtype="fp8")
    lens = [700, 1300, 64, 2500, 201]
    w = synth.custom_workload("fp8-grow", sh, lens, extra_blocks=0)
    dw = DeviceWorkload(w, fill=False)
    for s_, L in enumerate(lens):
        k, v = synth.kv_logical(w, s_, 0, L, dw.dev)
        t = torch.arange(L, device=dw.dev, dtype=torch.float32)
        f = torch.where(t < 200, 0.05, 8.0) * torch.where(t >= 640, 4.0, 1.0)     # key magnitude jumps twice
        k = (k.view(torch.float8_e4m3fn).float() * f[:, None, None]).to(torch.float8_e4m3fn).view(torch.uint8)
        synth.write_pages(w, dw.ranges, s_, 0, L, k, v)
    check_decode(dw)
    dw.close()


@pytest.mark.parametrize("dtype,d,B", [("bf16", 128, 16), ("bf16", 128, 64), ("f32", 64, 16), ("fp8", 128, 32), ("fp8", 64, 16)])
@pytest.mark.parametrize("order", ["chunks", "reversed-blocks", "interleaved"])
def test_kv_append_of_runs_is_bit_exact(dtype, d, B, order):
    # Tokens that follow each other in the input and in a page tile are moved as one run (whole V^T rows
    # when the run fills its tile).  Chunks that begin and end inside a tile, chunks shorter than a
    # tile, decode tokens between them, input offsets that are no multiple of 16, runs cut by the order.
    sh = synth.LayerShape(Hq=4, Hkv=4, d=d, B=B, dtype=dtype)
    chunks = [(5, 40), (16, 16), (31, 70), (0, 3), (64, 129), (7, 1)]
    w = synth.custom_workload("runs", sh, [37, 1, 16, 250, 99], chunks=chunks, extra_blocks=5, range_fracs=(0.5, 0.5))
    dw = DeviceWorkload(w, fill=False)
    pieces = []                                        # (seq, first position, count): tokens in input order
    for s_ in range(w.S):
        pieces.append((s_, int(w.decode_lens[s_]) - 1, 1))          # the decode requests' newest token
    for i, (p, c) in enumerate(chunks):
        pieces.append((w.S + i, p, c))
    if order == "interleaved":                         # a decode token after every chunk, and one chunk cut in two
        pieces = [pieces[5], pieces[0], pieces[6], pieces[1], (w.S + 2, 31, 33), pieces[2], (w.S + 2, 64, 37), pieces[3],
                  pieces[8], pieces[9], pieces[4], pieces[10]]
    seqs, poss = [], []
    for s_, p0, c in pieces:
        seqs += [s_] * c
        poss += list(range(p0, p0 + c))
    seqs, poss = np.asarray(seqs, dtype=np.int32), np.asarray(poss, dtype=np.int32)
    if order == "reversed-blocks":                     # blocks of 5 tokens in reverse order: short runs, odd offsets
        idx = np.concatenate([np.arange(i, min(i + 5, len(seqs))) for i in range(0, len(seqs), 5)][::-1])
        seqs, poss = seqs[idx], poss[idx]
    ks, vs = [], []
    for s_, t in zip(seqs.tolist(), poss.tolist()):
        k, v = synth.kv_logical(w, s_, t, t + 1)
        ks.append(k); vs.append(v)
    k_new, v_new = torch.cat(ks).contiguous(), torch.cat(vs).contiguous()
    table = w.table_array(range(len(w.seq_lens)))
    opool = oracle_pool(dw)                            # poisoned pages
    O.kv_append(opool, synth.to_host_bits(k_new), synth.to_host_bits(v_new), seqs, poss, table)
    kun.kun_kv_append(dw.pool, k_new.cuda(), v_new.cuda(), torch.from_numpy(seqs).cuda(), torch.from_numpy(poss).cuda(),
                      len(seqs), torch.from_numpy(table).cuda(), table.shape[1])
    torch.cuda.synchronize()
    for r in range(len(dw.ranges)):
        assert np.array_equal(synth.to_host_bits(dw.ranges[r]).reshape(-1), opool.ranges[r], equal_nan=True)
    dw.close()
