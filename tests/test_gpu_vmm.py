"""GPU tests of the KVCache region as one growing virtual range: kun_vmm_region_* and
kun_kv_pool_resize_tail, with decode over the grown pool checked against the CPU oracle."""
import os

import numpy as np
import pytest
import torch

from oracle import paged_attention as O
from paper_2412_18169_amd import kun, synth
from paper_2412_18169_amd.runner import DeviceWorkload

pytestmark = pytest.mark.gpu
TOL = 2e-2


@pytest.fixture(autouse=True)
def _announce(request):
    print(f"\n[gpu-case] {request.node.nodeid}", flush=True)
    yield
    kun.kun_set_option("KUN_DECODE_PART", None)


def status_of(fn, *a):
    with pytest.raises(kun.KunError) as e:
        fn(*a)
    return e.value.status


def test_regions_grow_move_their_tail_without_a_copy_and_shrink():
    torch.cuda.init()
    kv = kun.kun_vmm_region_create((1 << 30) + 5)
    par = kun.kun_vmm_region_create(1 << 28)
    base, mapped, reserved, gran = kun.kun_vmm_region_info(kv)
    assert mapped == 0 and reserved >= (1 << 30) + 5 and reserved % gran == 0 and base % gran == 0
    g = max(gran, 1 << 21)                                 # chunk unit of this test
    kun.kun_vmm_region_grow(kv, 4 * g)
    kun.kun_vmm_region_grow(kv, 2 * g)
    assert kun.kun_vmm_region_info(kv)[1] == 6 * g
    kv_bytes = kun.device_bytes(base, 6 * g)
    kv_bytes.copy_(torch.arange(6 * g, device="cuda", dtype=torch.int64).remainder(251).to(torch.uint8))
    pbase = kun.kun_vmm_region_info(par)[0]
    for i in range(3):                                     # three "layers" of parameters, one chunk each
        kun.kun_vmm_region_grow(par, 3 * g)
        kun.device_bytes(pbase + i * 3 * g, 3 * g).fill_(10 + i)
    torch.cuda.synchronize()
    assert status_of(kun.kun_vmm_region_grow, kv, g + 1) == -2                 # not a multiple of the granularity
    assert status_of(kun.kun_vmm_region_move_tail, par, kv, 4 * g) == -2       # not whole chunks
    assert status_of(kun.kun_vmm_region_grow, par, 1 << 28) == -3              # beyond the reservation
    # drop two layers: their physical memory becomes the KV region's tail, contents and order intact
    kun.kun_vmm_region_move_tail(par, kv, 6 * g)
    assert kun.kun_vmm_region_info(par)[1] == 3 * g and kun.kun_vmm_region_info(kv)[1] == 12 * g
    whole = kun.device_bytes(base, 12 * g)
    assert torch.equal(whole[:6 * g], kv_bytes)
    assert bool((whole[6 * g:9 * g] == 11).all()) and bool((whole[9 * g:] == 12).all())
    assert bool((kun.device_bytes(pbase, 3 * g) == 10).all())
    whole[6 * g:].fill_(99)
    torch.cuda.synchronize()
    # restoration: the same memory goes back behind the remaining parameters
    kun.kun_vmm_region_move_tail(kv, par, 6 * g)
    assert kun.kun_vmm_region_info(par)[1] == 9 * g and kun.kun_vmm_region_info(kv)[1] == 6 * g
    assert bool((kun.device_bytes(pbase + 3 * g, 6 * g) == 99).all())
    assert torch.equal(kun.device_bytes(base, 6 * g), kv_bytes)
    assert status_of(kun.kun_vmm_region_move_tail, par, kv, 4 * g) == -2       # chunks keep their sizes: 3 g each
    # chunks of many different sizes next to each other
    for k in (1, 5, 2, 7, 3):
        kun.kun_vmm_region_grow(kv, k * g)
    kun.device_bytes(base, 24 * g).fill_(5)
    torch.cuda.synchronize()
    kun.kun_vmm_region_shrink(kv, 18 * g)
    kun.kun_vmm_region_shrink(kv, 2 * g)
    assert kun.kun_vmm_region_info(kv)[1] == 4 * g
    torch.cuda.synchronize()
    kun.kun_vmm_region_destroy(kv)
    kun.kun_vmm_region_destroy(par)


def test_decode_over_a_pool_that_grows_in_place_and_gives_the_memory_back():
    kun.kun_set_option("KUN_DECODE_PART", "256")         # partitions depend on lengths only: bit-identical outputs
    sh = synth.SHAPE_8B
    bb = sh.block_bytes
    kv = kun.kun_vmm_region_create(1 << 30)
    par = kun.kun_vmm_region_create(1 << 28)
    base, _, _, gran = kun.kun_vmm_region_info(kv)
    per = max(gran, 1 << 21) // bb                 # blocks per 2 MiB (or per granule if that is larger)
    n0, n1, n2 = 8 * per, 4 * per, 4 * per
    kun.kun_vmm_region_grow(kv, n0 * bb)
    for _ in range(2):
        kun.kun_vmm_region_grow(par, n1 * bb)      # two droppable parameter chunks
    rng = np.random.default_rng(3)
    total_tokens = (n0 + n1 + n2) * sh.B
    lens = synth.lognormal_lengths(rng, 64, median=total_tokens // 80, sigma=0.7, lo=16, hi=total_tokens // 8)
    w = synth.Workload("vmm", 0, 41, sh, lens, [], [n0, n1, n2])
    keep = int(np.searchsorted(np.cumsum(synth.blocks_needed(lens, sh.B)), n0 + n1 + n2, side="right"))
    w = synth.Workload("vmm", 0, 41, sh, lens[:keep], [], [n0, n1, n2])
    resident = synth.assign_blocks_phased(w)       # phase k draws from the first k + 1 spans only
    assert 0 < resident[0] < resident[1] < resident[2] == keep
    w.range_blocks = [n0 + n1 + n2]                # ... which the pool sees as ONE range that grows
    full = kun.device_bytes(base, (n0 + n1 + n2) * bb).view(sh.torch_dtype).view(-1, sh.Hkv, 2, sh.B * sh.d)
    dw = DeviceWorkload(w, ranges=[full], create_bytes=n0 * bb, fill=False)

    def oracle_check(n_req, n_blocks, out):
        bits = synth.to_host_bits(kun.device_bytes(base, n_blocks * bb).view(sh.torch_dtype)).reshape(-1)
        pool = O.OraclePool([bits], sh.Hkv, sh.d, sh.B, sh.dtype)
        ref = O.paged_decode(pool, synth.to_host_bits(dw.q_dec[:n_req]), w.table_array(range(w.S))[:n_req],
                             w.decode_lens[:n_req], sh.Hq, sh.scale)
        err = float(np.abs(out[:n_req].double().cpu().numpy() - ref).max())
        assert err <= TOL, err

    def admit(lo, hi):
        for s in range(lo, hi):
            synth.write_pages(w, [full], s, 0, int(w.seq_lens[s]))

    admit(0, resident[0])
    a = dw.decode(resident[0]).clone()
    torch.cuda.synchronize()
    oracle_check(resident[0], n0, a)
    have = n0
    for phase, nb in ((1, n1), (2, n2)):
        kun.kun_vmm_region_move_tail(par, kv, nb * bb)                       # a parameter chunk is dropped
        first, delta = kun.kun_kv_pool_resize_tail(dw.pool, (have + nb) * bb)
        assert (first, delta) == (have, nb) and kun.kun_kv_pool_num_ranges(dw.pool) == 1
        have += nb
        assert kun.kun_kv_pool_num_blocks(dw.pool) == have
        r, off, addr = kun.kun_kv_pool_resolve(dw.pool, have - 1)
        assert (r, off, addr) == (0, (have - 1) * bb, base + (have - 1) * bb)
        admit(resident[phase - 1], resident[phase])
        out = dw.decode(resident[phase]).clone()
        torch.cuda.synchronize()
        oracle_check(resident[phase], have, out)
        assert torch.equal(out[:resident[0]], a[:resident[0]])               # residents: same bits as before
    b = out
    # restoration: the requests of the last phase have finished; the chunk returns to the parameters
    kun.kun_vmm_region_move_tail(kv, par, n2 * bb)
    first, delta = kun.kun_kv_pool_resize_tail(dw.pool, (have - n2) * bb)
    assert (first, delta) == (have - n2, -n2)
    assert status_of(kun.kun_kv_pool_resolve, dw.pool, have - n2) == -5
    c = dw.decode(resident[1]).clone()
    torch.cuda.synchronize()
    assert torch.equal(c[:resident[1]], b[:resident[1]])
    assert kun.kun_vmm_region_info(par)[1] == n2 * bb and kun.kun_vmm_region_info(kv)[1] == (n0 + n1) * bb
    dw.close()
    kun.kun_vmm_region_destroy(kv)
    kun.kun_vmm_region_destroy(par)
