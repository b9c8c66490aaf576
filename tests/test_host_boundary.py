"""CPU-only tests of the C-ABI boundary: the library loads, exports every declared symbol, and the
host-side pool logic (growth, block resolution, validation, error codes) is bit-exact against the
oracle's own resolver.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest
import torch

from oracle import paged_attention as O
from paper_2412_18169_amd import kun

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BASE = 0x7F0000000000          # fake, 256-aligned "device" addresses: never dereferenced on the host
BB = 65536                     # block bytes of 8 kv heads x 128 dims x 16 tokens in bf16


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "kun.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kun_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 14
    L = kun.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(kun.SYMBOLS) == names


def make_pool(nbytes=BB * 5, base=BASE):
    return kun.kun_kv_pool_create(base, nbytes, kun.KUN_BF16, 8, 128, 16)


def test_block_bytes_formula():
    p = make_pool()
    assert kun.kun_kv_pool_block_bytes(p) == 2 * 8 * 16 * 128 * 2 == BB
    kun.kun_kv_pool_destroy(p)
    p = kun.kun_kv_pool_create(BASE, 1 << 20, kun.KUN_F32, 2, 64, 16)
    assert kun.kun_kv_pool_block_bytes(p) == 16384 and kun.kun_kv_pool_num_blocks(p) == 64
    kun.kun_kv_pool_destroy(p)
    p = kun.kun_kv_pool_create(BASE, 1 << 22, kun.KUN_BF16, 8, 128, 64)       # 64-token blocks
    assert kun.kun_kv_pool_block_bytes(p) == 4 * BB and kun.kun_kv_pool_num_blocks(p) == 16
    kun.kun_kv_pool_destroy(p)


def test_growth_and_resolve_match_oracle_bit_exact():
    sizes = [BB * 5 + 100, BB * 1, BB * 7 + BB - 1, BB * 3]       # remainders are unused
    bases = [BASE, BASE + (1 << 30), BASE + (2 << 30), BASE + (3 << 30)]
    p = make_pool(sizes[0], bases[0])
    rb = [O.usable_blocks(sizes[0], BB)]
    assert kun.kun_kv_pool_num_blocks(p) == 5
    before = [kun.kun_kv_pool_resolve(p, b) for b in range(5)]
    for sz, base in zip(sizes[1:], bases[1:]):
        first, n = kun.kun_kv_pool_extend(p, base, sz)
        assert first == sum(rb) and n == O.usable_blocks(sz, BB)
        rb.append(n)
        # ids and addresses of existing blocks are stable across an extension
        assert [kun.kun_kv_pool_resolve(p, b) for b in range(5)] == before
    assert kun.kun_kv_pool_num_ranges(p) == 4 and kun.kun_kv_pool_num_blocks(p) == sum(rb) == 16
    for blk in range(sum(rb)):
        r, off, addr = kun.kun_kv_pool_resolve(p, blk)
        assert (r, off) == O.block_byte_offset(rb, blk, BB)
        assert addr == bases[r] + off
    for bad in (-1, 16, 1 << 40):
        with pytest.raises(kun.KunError) as e:
            kun.kun_kv_pool_resolve(p, bad)
        assert e.value.status == -5
    kun.kun_kv_pool_destroy(p)


def test_large_pool_offsets_are_64_bit():
    # 150 GB in five ranges: byte offsets exceed 2^32 and block ids exceed 2^15
    per = 30 * 10**9
    p = make_pool(per, BASE)
    for i in range(1, 5):
        kun.kun_kv_pool_extend(p, BASE + i * (1 << 36), per)
    nb = per // BB
    assert kun.kun_kv_pool_num_blocks(p) == 5 * nb
    for blk in (0, 32768, nb - 1, nb, 3 * nb + 12345, 5 * nb - 1):
        r, off, addr = kun.kun_kv_pool_resolve(p, blk)
        assert (r, off) == O.block_byte_offset([nb] * 5, blk, BB)
        assert addr == BASE + r * (1 << 36) + off
    kun.kun_kv_pool_destroy(p)


def test_error_paths():
    def status(fn, *a):
        with pytest.raises(kun.KunError) as e:
            fn(*a)
        return e.value.status
    assert status(kun.kun_kv_pool_create, BASE + 8, BB * 4, kun.KUN_BF16, 8, 128, 16) == -2    # misaligned
    assert status(kun.kun_kv_pool_create, BASE, BB - 1, kun.KUN_BF16, 8, 128, 16) == -3        # too small
    assert status(kun.kun_kv_pool_create, 0, BB * 4, kun.KUN_BF16, 8, 128, 16) == -1           # null base
    assert status(kun.kun_kv_pool_create, BASE, BB * 4, 7, 8, 128, 16) == -1                   # bad dtype
    assert status(kun.kun_kv_pool_create, BASE, BB * 4, kun.KUN_BF16, 8, 128, 48) == -8        # block size
    assert status(kun.kun_kv_pool_create, BASE, BB * 4, kun.KUN_BF16, 8, 96, 16) == -8         # head dim
    p = make_pool()
    assert status(kun.kun_kv_pool_extend, p, BASE + 17, BB * 2) == -2
    assert status(kun.kun_kv_pool_extend, p, BASE + (1 << 30), 100) == -3
    assert status(kun.kun_kv_pool_extend, p, BASE + BB, BB * 2) == -9                          # overlaps range 0
    assert status(kun.kun_kv_pool_extend, 0, BASE + (1 << 30), BB * 2) == -1                   # null handle
    for i in range(1, kun.KUN_MAX_RANGES):
        kun.kun_kv_pool_extend(p, BASE + i * (1 << 30), BB)
    assert status(kun.kun_kv_pool_extend, p, BASE + 17 * (1 << 30), BB) == -4                  # too many ranges
    assert kun.kun_kv_pool_num_ranges(p) == kun.KUN_MAX_RANGES
    # decode argument checks happen before any launch
    assert kun.kun_decode_workspace_bytes(p, 4, 30, 0) == 0                                    # 30 % 8 != 0
    assert status(kun.kun_paged_decode, p, BASE, BASE, BASE, 4, BASE, 2, 30, 1.0, 0, BASE, 1 << 30, 0) == -1
    assert status(kun.kun_paged_decode, p, BASE, BASE, BASE, 4, BASE, 2, 72, 1.0, 0, BASE, 1 << 30, 0) == -8  # G = 9
    assert status(kun.kun_paged_decode, p, BASE, BASE, BASE, 4, BASE, 2, 32, 1.0, 0, BASE, 16, 0) == -6       # workspace small
    assert status(kun.kun_paged_decode, p, BASE, BASE, BASE, 4, BASE, 2, 32, 1.0, 0, BASE + 4, 1 << 30, 0) == -6
    assert status(kun.kun_paged_decode, p, 0, BASE, BASE, 4, BASE, 2, 32, 1.0, 0, BASE, 1 << 30, 0) == -1
    # ... and so do those of the two-step form
    assert status(kun.kun_decode_plan, p, 0, 2, 32, 0, BASE, 1 << 30, 0) == -1                  # no lengths
    assert status(kun.kun_decode_plan, p, BASE, 2, 30, 0, BASE, 1 << 30, 0) == -1               # 30 % 8 != 0
    assert status(kun.kun_decode_plan, p, BASE, 2, 32, 0, BASE, 16, 0) == -6                    # workspace small
    assert status(kun.kun_paged_decode_planned, p, 0, BASE, BASE, 4, BASE, 2, 32, 1.0, 0, BASE, 1 << 30, 0) == -1
    assert status(kun.kun_paged_decode_planned, p, BASE, BASE, BASE, 4, BASE, 2, 32, 1.0, 0, BASE, 16, 0) == -6
    kun.kun_decode_plan(p, 0, 0, 32, 0, 0, 0, 0)                                               # S == 0: no-op
    kun.kun_paged_decode_planned(p, 0, 0, 0, 0, 0, 0, 32, 1.0, 0, 0, 0, 0)
    # prefill: the same checks, in one call and in two
    assert kun.kun_prefill_workspace_bytes(p, 2, 30, 64, 8) == 0                               # 30 % 8 != 0
    for fn in (kun.kun_paged_prefill_chunk, kun.kun_paged_prefill_chunk_planned):
        assert status(fn, p, BASE, BASE, BASE, BASE, BASE, 8, 2, 30, 64, 1.0, BASE, 1 << 30, 0) == -1
        assert status(fn, p, BASE, BASE, BASE, BASE, BASE, 8, 2, 72, 64, 1.0, BASE, 1 << 30, 0) == -8   # G = 9
        assert status(fn, p, 0, BASE, BASE, BASE, BASE, 8, 2, 32, 64, 1.0, BASE, 1 << 30, 0) == -1      # no q
        assert status(fn, p, BASE, BASE, BASE, BASE, BASE, 8, 2, 32, 64, 1.0, BASE, 16, 0) == -6        # workspace small
        fn(p, 0, 0, 0, 0, 0, 0, 0, 32, 0, 1.0, 0, 0, 0)                                        # nothing to do
    assert status(kun.kun_prefill_plan, p, 0, BASE, BASE, 8, 2, 32, 64, BASE, 1 << 30, 0) == -1    # no q_start
    assert status(kun.kun_prefill_plan, p, BASE, BASE, BASE, 8, 2, 32, 64, BASE + 8, 1 << 30, 0) == -6
    kun.kun_prefill_plan(p, 0, 0, 0, 0, 0, 32, 0, 0, 0, 0)
    assert status(kun.kun_kv_append, p, 0, BASE, BASE, BASE, 3, BASE, 4, 0) == -1
    kun.kun_kv_append(p, 0, 0, 0, 0, 0, 0, 0, 0)                                               # T == 0: no-op
    kun.kun_paged_decode(p, 0, 0, 0, 0, 0, 0, 32, 1.0, 0, 0, 0, 0)                             # S == 0: no-op
    kun.kun_kv_pool_destroy(p)
    assert kun.status_string(-5) == "KUN_ERR_BLOCK_OOB" and kun.status_string(0) == "KUN_OK"


def test_validate_block_table():
    p = make_pool(BB * 10)
    tab = torch.tensor([[3, 9, -1, -1], [0, 1, 2, 4]], dtype=torch.int32)
    kun.kun_validate_block_table(p, tab, torch.tensor([20, 64], dtype=torch.int32))
    kun.kun_validate_block_table(p, tab, torch.tensor([32, 49], dtype=torch.int32))   # -1 beyond ctx ignored
    for lens, code in [([33, 64], -5), ([20, 65], -1), ([-1, 3], -1)]:
        with pytest.raises(kun.KunError) as e:
            kun.kun_validate_block_table(p, tab, torch.tensor(lens, dtype=torch.int32))
        assert e.value.status == code
    tab[1, 3] = 10
    with pytest.raises(kun.KunError) as e:
        kun.kun_validate_block_table(p, tab, torch.tensor([20, 64], dtype=torch.int32))
    assert e.value.status == -5
    kun.kun_kv_pool_destroy(p)


def test_workspace_size_is_monotone_in_the_bound():
    p = make_pool(30 * 10**9)
    prev = 0
    for ub in [1, 1000, 100000, 131071, 131072, 262143, 262144, 600000, 1048575, 1048576, 2097151, 2097152, 5000000]:
        need = kun.kun_decode_workspace_bytes(p, 256, 64, ub)
        assert need >= prev and need % 256 == 0
        prev = need
    kun.kun_kv_pool_destroy(p)


def test_resize_of_the_last_range_matches_oracle_bit_exact():
    # the pool as ONE growing range, and as a first range plus a growing second one
    for lead in ([], [BB * 4]):
        sizes = lead + [BB * 3 + 17]
        p = make_pool(sizes[0], BASE)
        if lead:
            kun.kun_kv_pool_extend(p, BASE + (1 << 32), sizes[1])
        tail_base = BASE + ((1 << 32) if lead else 0)
        n_lead = sum(O.usable_blocks(x, BB) for x in lead)
        seen = {}
        for new_bytes in [BB * 3 + 17, BB * 9, BB * 9 + BB - 1, BB * 70000, BB * 6 + 5, BB * 1, BB * 2]:
            old = kun.kun_kv_pool_num_blocks(p) - n_lead
            first, delta = kun.kun_kv_pool_resize_tail(p, new_bytes)
            nb = O.usable_blocks(new_bytes, BB)
            assert delta == nb - old and first == n_lead + min(nb, old)
            rb = [O.usable_blocks(x, BB) for x in lead] + [nb]
            assert kun.kun_kv_pool_num_blocks(p) == sum(rb) and kun.kun_kv_pool_num_ranges(p) == len(rb)
            for blk in sorted(set([0, n_lead, sum(rb) - 1, n_lead + nb // 2, n_lead + nb - 1])):
                r, off, addr = kun.kun_kv_pool_resolve(p, blk)
                assert (r, off) == O.block_byte_offset(rb, blk, BB)
                assert addr == (BASE if r == 0 and lead else tail_base) + off
                assert seen.setdefault(blk, addr) == addr          # a block that exists keeps its address
            with pytest.raises(kun.KunError) as e:
                kun.kun_kv_pool_resolve(p, sum(rb))
            assert e.value.status == -5
        with pytest.raises(kun.KunError) as e:
            kun.kun_kv_pool_resize_tail(p, BB - 1)
        assert e.value.status == -3
        kun.kun_kv_pool_destroy(p)
    # growing the last range into an earlier one is refused
    p = make_pool(BB * 4, BASE + BB * 100)
    kun.kun_kv_pool_extend(p, BASE, BB * 10)
    with pytest.raises(kun.KunError) as e:
        kun.kun_kv_pool_resize_tail(p, BB * 101)
    assert e.value.status == -9
    kun.kun_kv_pool_destroy(p)


def test_header_and_host_entry_points_from_plain_c(tmp_path):
    # include/kun.h compiles as C99 with warnings as errors, and a C program linked against the
    # library gets the documented results from the host-only calls (tests/c_abi_client.c)
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    libdir = os.path.join(ROOT, "paper_2412_18169_amd")
    exe = str(tmp_path / "c_abi_client")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi_client.c"), "-o", exe, "-L", libdir, "-lkun", "-lm",
                    "-Wl,-rpath," + libdir], check=True, capture_output=True, text=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert run.returncode == 0 and "c abi ok" in run.stdout, run.stdout + run.stderr


def test_static_scratch_decode_refuses_what_does_not_fit_before_touching_the_device():
    # The entry point for callers that cannot allocate keeps its split-K records in a fixed array of
    # KUN_STATIC_SCRATCH_BYTES; a call that needs more is refused on the host (no HIP call is made, so
    # this runs without a GPU) with a status of its own.
    p = make_pool(200 << 30)                       # 200 GB of fake addresses
    need = kun.kun_decode_workspace_bytes(p, 4096, 32, 0)
    assert need > kun.KUN_STATIC_SCRATCH_BYTES
    with pytest.raises(kun.KunError) as e:
        kun.kun_paged_decode_static(p, BASE, BASE, BASE, 8, BASE, 4096, 32, 0.1, 0, stream=0)
    assert e.value.status == -10 and "SCRATCH_LIMIT" in str(e.value)
    text = open(os.path.join(ROOT, "include", "kun.h")).read()
    assert re.search(r"#define KUN_STATIC_SCRATCH_BYTES \(32u << 20\)", text) and kun.KUN_STATIC_SCRATCH_BYTES == 32 << 20
    # bad shapes are still argument errors, and an empty batch is a no-op
    with pytest.raises(kun.KunError) as e:
        kun.kun_paged_decode_static(p, BASE, BASE, BASE, 8, BASE, 4, 33, 0.1, 0, stream=0)
    assert e.value.status == -1
    kun.kun_paged_decode_static(p, BASE, BASE, BASE, 8, BASE, 0, 32, 0.1, 0, stream=0)
    kun.kun_kv_pool_destroy(p)


def test_vmm_region_bookkeeping_survives_driver_failures(tmp_path):
    # kun_vmm_region_move_tail is all or nothing, and when the driver also refuses the undoing both
    # regions still list exactly what is mapped: the bookkeeping template behind the entry points, run
    # on the host against a driver that fails the n-th call (tests/vmm_bookkeeping_test.cpp)
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("no g++")
    exe = str(tmp_path / "vmm_bookkeeping_test")
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Wextra", "-Werror", "-I",
                    os.path.join(ROOT, "paper_2412_18169_amd", "csrc"),
                    os.path.join(ROOT, "tests", "vmm_bookkeeping_test.cpp"), "-o", exe],
                   check=True, capture_output=True, text=True)
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and "vmm bookkeeping ok" in run.stdout, run.stdout + run.stderr
