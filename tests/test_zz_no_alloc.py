"""kun_paged_decode_static (decode for callers that cannot allocate: split-K records in the library's
fixed device array) against kun_paged_decode, through the C ABI: two calls in a row, the second with
a smaller input, each bit-identical to the workspace entry point and within the bf16 bar (max-abs
2e-2) of the CPU oracle.  Collected last, so that a failure here hides no other test."""
import numpy as np
import pytest
import torch

from oracle import paged_attention as O
from paper_2412_18169_amd import kun, synth
from paper_2412_18169_amd.runner import DeviceWorkload

pytestmark = pytest.mark.gpu


def _both(dw, S, bound):
    """(workspace entry point, static entry point) outputs for the first S requests."""
    sh = dw.w.shape
    ref = dw.decode(S, ctx_bound=bound).clone()
    out = torch.full_like(dw.q_dec, 7.0)               # stale contents: untouched rows must stay
    kun.kun_paged_decode_static(dw.pool, dw.q_dec, out, dw.dec_table, dw.dec_table.shape[1], dw.dec_len, S,
                                sh.Hq, sh.scale, bound)
    torch.cuda.synchronize()
    return ref, out


def test_static_scratch_decode_matches_workspace_decode_twice_in_a_row():
    print("\n[gpu-case] static scratch decode, large then small", flush=True)
    sh = synth.LayerShape(Hq=32, Hkv=8, d=128, B=16, dtype="bf16")
    # several partitions per long request (records in scratch), single-partition ones, an empty one
    lens = [4100, 1, 17, 2500, 0, 300, 9000, 1025, 64, 5000, 333, 2049]
    w = synth.custom_workload("noalloc", sh, lens, extra_blocks=5, range_fracs=(0.4, 0.3, 0.3))
    dw = DeviceWorkload(w)
    pool = O.OraclePool([synth.to_host_bits(r).reshape(-1) for r in dw.ranges], sh.Hkv, sh.d, sh.B, sh.dtype)
    for S in (len(lens), 5):                           # the second call is the smaller one
        bound = int(np.asarray(lens[:S], dtype=np.int64).sum())
        assert kun.kun_decode_workspace_bytes(dw.pool, S, sh.Hq, bound) <= kun.KUN_STATIC_SCRATCH_BYTES
        ref, out = _both(dw, S, bound)
        live = torch.tensor([L > 0 for L in lens[:S]], device=out.device)
        assert torch.equal(out[:S][live].view(torch.int16), ref[:S][live].view(torch.int16))
        assert (out[:S][~live] == 7.0).all() and (out[S:] == 7.0).all()
        want = O.paged_decode(pool, synth.to_host_bits(dw.q_dec[:S]), w.table_array(range(w.S))[:S],
                              np.asarray(lens[:S]), sh.Hq, sh.scale)
        got = out[:S].double().cpu().numpy()
        lv = np.asarray(lens[:S]) > 0
        assert np.abs(got[lv] - want[lv]).max() <= 2e-2
    dw.close()
