"""Seeded random workloads against the CPU oracle through the C ABI: every page type, head_dim, block
size and group size the library takes, ragged lengths (zero included), one to three pool ranges, any
split-K partition size and merge mode, the one-call and the planned forms of decode and prefill, decode
out of the library's fixed scratch array and prefill on a capped number of workgroups.
Tolerances as in the other GPU tests (1e-5 fp32, 2e-2 bf16 and FP8 pages)."""
import numpy as np
import pytest
import torch

from paper_2412_18169_amd import kun, synth
from paper_2412_18169_amd.runner import DeviceWorkload
from test_gpu_decode import check_decode
from test_gpu_prefill import check_prefill

pytestmark = pytest.mark.gpu
CASES_PER_SEED = 12


@pytest.fixture(autouse=True)
def _reset_options():
    yield
    kun.kun_set_option("KUN_DECODE_PART", None)
    kun.kun_set_option("KUN_DECODE_MERGE", None)


def random_workload(rng, name):
    dtype = str(rng.choice(["bf16", "bf16", "fp8", "f32"]))
    d = int(rng.choice([64, 128])) if dtype == "f32" else int(rng.choice([128, 128, 64]))
    B = int(rng.choice([16, 16, 32, 64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    on_matrix_cores = dtype in ("bf16", "fp8") and d == 128
    G = int(rng.choice([g for g in (1, 2, 3, 4, 5, 6, 7, 8, 16) if g <= (16 if on_matrix_cores else 8)]))
    sh = synth.LayerShape(Hq=Hkv * G, Hkv=Hkv, d=d, B=B, dtype=dtype)
    hi = {"short": 200, "mixed": 3000, "long": 9000}[str(rng.choice(["short", "mixed", "long"]))]
    lens = rng.integers(0, hi, size=int(rng.integers(1, 24))).tolist()
    # (the row-by-row prefill of the other shapes is slow: short chunks there)
    chunks = [(int(rng.integers(0, hi if on_matrix_cores else 300)), int(rng.integers(0, 400 if on_matrix_cores else 40)))
              for _ in range(int(rng.integers(0, 5)))]
    nr = int(rng.integers(1, 4))
    fracs = (0.15 + rng.dirichlet(np.ones(nr)) * (1 - 0.15 * nr)).tolist()
    w = synth.custom_workload(name, sh, lens, chunks=chunks, seed=int(rng.integers(1, 1 << 30)),
                              extra_blocks=int(rng.integers(8, 20)), range_fracs=tuple(fracs))
    return w, on_matrix_cores


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_workloads(seed):
    for case in range(CASES_PER_SEED):
        rng = np.random.default_rng(seed * 1000 + case)
        w, on_matrix_cores = random_workload(rng, f"random-{seed}-{case}")
        sh = w.shape
        part = rng.choice([None, "64", "256", "1024"])
        merge = rng.choice([None, "fold", "kernel"])
        planned = bool(rng.integers(0, 2))
        print(f"[case {seed}/{case}] {sh} decode_lens={w.decode_lens.tolist()} chunks={w.chunks} part={part} "
              f"merge={merge} planned={planned}", flush=True)
        kun.kun_set_option("KUN_DECODE_PART", part)
        kun.kun_set_option("KUN_DECODE_MERGE", merge)
        dw = DeviceWorkload(w)
        if planned:
            dw.decode(steps="plan")
            check_decode(dw, out=dw.decode(steps="planned"))
        else:
            check_decode(dw)
        if any(c > 0 for _, c in w.chunks) and sh.dtype != "f32":
            if planned and on_matrix_cores:
                dw.prefill(steps="plan")
                got = dw.prefill(steps="planned").clone()
                check_prefill(dw)                          # the one-call form, against the oracle
                assert torch.equal(got.view(torch.int16), dw.out_pre.view(torch.int16))
            else:
                check_prefill(dw)
            if on_matrix_cores and bool(rng.integers(0, 2)):        # fetching workgroups: the bits of the plain launch
                ref = dw.out_pre.clone()
                got = dw.prefill(max_workgroups=int(rng.choice([8, 24, 64, 512])))
                torch.cuda.synchronize()
                assert torch.equal(got.view(torch.int16), ref.view(torch.int16))
        if bool(rng.integers(0, 2)):                                # no workspace argument: same kernels, same bits
            bound = int(w.decode_lens.astype(np.int64).sum())
            if 0 < kun.kun_decode_workspace_bytes(dw.pool, w.S, sh.Hq, bound) <= kun.KUN_STATIC_SCRATCH_BYTES:
                ref = dw.decode().clone()
                out = torch.full_like(dw.q_dec, 3.0)
                kun.kun_paged_decode_static(dw.pool, dw.q_dec, out, dw.dec_table, dw.dec_table.shape[1], dw.dec_len,
                                            w.S, sh.Hq, sh.scale, bound)
                torch.cuda.synchronize()
                live = torch.tensor(w.decode_lens > 0, device=out.device)
                assert torch.equal(out[live].view(torch.uint8), ref[live].view(torch.uint8))
                assert (out[~live] == 3.0).all()
        dw.close()
