"""Thin ctypes binding of the C-ABI library declared in include/kun.h.

Argument marshalling only: every function here has the name of the C entry point it forwards to,
takes torch tensors (or raw integers) for the pointer arguments, and raises KunError on a
non-zero status.  All computation happens in the HIP kernels of libkun.so.  There is no CPU
fallback: if the library is missing or cannot be loaded, importing this module's functions fails
with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkun.so")

KUN_F32, KUN_BF16, KUN_FP8_E4M3 = 0, 1, 2
KUN_MAX_RANGES = 16

SYMBOLS = [
    "kun_status_string", "kun_last_hip_error", "kun_set_option", "kun_kv_pool_create", "kun_kv_pool_extend", "kun_kv_pool_num_blocks",
    "kun_kv_pool_num_ranges", "kun_kv_pool_block_bytes", "kun_kv_pool_resolve",
    "kun_kv_pool_destroy", "kun_validate_block_table", "kun_slot_map", "kun_kv_append",
    "kun_decode_workspace_bytes", "kun_paged_decode", "kun_decode_plan", "kun_paged_decode_planned", "kun_paged_decode_static",
    "kun_prefill_workspace_bytes",
    "kun_paged_prefill_chunk", "kun_prefill_plan", "kun_paged_prefill_chunk_planned", "kun_paged_prefill_chunk_on", "kun_kv_pool_resize_tail",
    "kun_vmm_region_create", "kun_vmm_region_info", "kun_vmm_region_grow", "kun_vmm_region_move_tail",
    "kun_vmm_region_shrink", "kun_vmm_region_destroy",
    "kun_cost_chunk", "kun_cost_microbatch", "kun_cost_fit", "kun_lookahead", "kun_drop_plan",
]


class CostModel(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_double), ("beta", ctypes.c_double), ("gamma", ctypes.c_double)]


class Chunk(ctypes.Structure):
    _fields_ = [("request", ctypes.c_int32), ("prior", ctypes.c_int32), ("tokens", ctypes.c_int32)]


class KunError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = f": {last_hip_error()}" if status == -7 else ""
        super().__init__(f"{where}: {status_string(status)} ({status}){detail}")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libkun.so once.  Fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2412_18169_amd.build` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, sz, i32, i64, f32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_int64, ctypes.c_float
    P = ctypes.POINTER
    L.kun_status_string.restype = ctypes.c_char_p
    L.kun_status_string.argtypes = [i32]
    L.kun_last_hip_error.restype = ctypes.c_char_p
    L.kun_last_hip_error.argtypes = []
    L.kun_set_option.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    L.kun_kv_pool_create.argtypes = [P(vp), vp, sz, i32, i32, i32, i32]
    L.kun_kv_pool_extend.argtypes = [vp, vp, sz, P(i64), P(i64)]
    L.kun_kv_pool_num_blocks.argtypes = [vp, P(i64)]
    L.kun_kv_pool_resize_tail.argtypes = [vp, sz, P(i64), P(i64)]
    L.kun_vmm_region_create.argtypes = [P(vp), sz]
    L.kun_vmm_region_info.argtypes = [vp, P(vp), P(sz), P(sz), P(sz)]
    L.kun_vmm_region_grow.argtypes = [vp, sz]
    L.kun_vmm_region_move_tail.argtypes = [vp, vp, sz]
    L.kun_vmm_region_shrink.argtypes = [vp, sz]
    L.kun_vmm_region_destroy.argtypes = [vp]
    f64 = ctypes.c_double
    L.kun_cost_chunk.restype = f64
    L.kun_cost_chunk.argtypes = [P(CostModel), i64, i64]
    L.kun_cost_microbatch.restype = f64
    L.kun_cost_microbatch.argtypes = [P(CostModel), vp, i32]
    L.kun_cost_fit.argtypes = [vp, vp, i32, vp, P(CostModel)]
    L.kun_lookahead.argtypes = [P(CostModel), vp, i32, i32, i32, vp, i32, vp, i32, P(i32), P(i32)]
    L.kun_drop_plan.argtypes = [i32, vp, i32, i64, i64, vp, vp, vp, vp, vp, vp, P(i32), P(i64), P(i32)]
    L.kun_kv_pool_num_ranges.argtypes = [vp, P(i32)]
    L.kun_kv_pool_block_bytes.argtypes = [vp, P(sz)]
    L.kun_kv_pool_resolve.argtypes = [vp, i64, P(i32), P(sz), P(vp)]
    L.kun_kv_pool_destroy.argtypes = [vp]
    L.kun_validate_block_table.argtypes = [vp, vp, i32, i32, vp]
    L.kun_kv_append.argtypes = [vp, vp, vp, vp, vp, i32, vp, i32, vp]
    L.kun_slot_map.argtypes = [vp, vp, vp, i32, vp, i32, i32, vp, vp, vp, vp]
    L.kun_decode_workspace_bytes.restype = sz
    L.kun_decode_workspace_bytes.argtypes = [vp, i32, i32, i64]
    L.kun_paged_decode.argtypes = [vp, vp, vp, vp, i32, vp, i32, i32, f32, i64, vp, sz, vp]
    L.kun_decode_plan.argtypes = [vp, vp, i32, i32, i64, vp, sz, vp]
    L.kun_paged_decode_planned.argtypes = [vp, vp, vp, vp, i32, vp, i32, i32, f32, i64, vp, sz, vp]
    L.kun_paged_decode_static.argtypes = [vp, vp, vp, vp, i32, vp, i32, i32, f32, i64, vp]
    L.kun_prefill_workspace_bytes.restype = sz
    L.kun_prefill_workspace_bytes.argtypes = [vp, i32, i32, i32, i32]
    L.kun_paged_prefill_chunk.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, vp, sz, vp]
    L.kun_prefill_plan.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]
    L.kun_paged_prefill_chunk_planned.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, vp, sz, vp]
    L.kun_paged_prefill_chunk_on.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, f32, i32, vp, sz, vp]
    for name in SYMBOLS:
        if name not in ("kun_status_string", "kun_last_hip_error", "kun_decode_workspace_bytes",
                        "kun_prefill_workspace_bytes", "kun_cost_chunk", "kun_cost_microbatch"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def last_hip_error() -> str:
    return lib().kun_last_hip_error().decode()


def status_string(status: int) -> str:
    return lib().kun_status_string(int(status)).decode()


OPTION_NAMES = ("KUN_DECODE_PART", "KUN_DECODE_WAVES", "KUN_DECODE_KERNEL", "KUN_DECODE_MAP", "KUN_DECODE_MERGE",
                "KUN_PREFILL_SHAPE")


def kun_set_option(name: str, value=None) -> None:
    """value None = back to the default."""
    _check(lib().kun_set_option(name.encode(), None if value is None else str(value).encode()),
           f"kun_set_option({name}={value})")


def _check(st: int, where: str) -> None:
    if st != 0:
        raise KunError(st, where)


def _ptr(x) -> Optional[int]:
    """Device/host address of a tensor, or a raw integer address, or None."""
    if x is None:
        return None
    if isinstance(x, torch.Tensor):
        return x.data_ptr()
    return int(x)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream if torch.cuda.is_available() else None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def kun_kv_pool_create(base, nbytes: int, dtype: int, num_kv_heads: int, head_dim: int,
                       block_size: int) -> int:
    """Returns the opaque pool handle (an integer address)."""
    h = ctypes.c_void_p()
    _check(lib().kun_kv_pool_create(ctypes.byref(h), _ptr(base), int(nbytes), dtype, num_kv_heads,
                                    head_dim, block_size), "kun_kv_pool_create")
    return h.value


def kun_kv_pool_extend(pool: int, base, nbytes: int):
    """Returns (first_new_block, num_new_blocks)."""
    first, n = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().kun_kv_pool_extend(pool, _ptr(base), int(nbytes), ctypes.byref(first),
                                    ctypes.byref(n)), "kun_kv_pool_extend")
    return first.value, n.value


def kun_kv_pool_resize_tail(pool: int, new_bytes: int):
    """Returns (first_changed_block, num_blocks_delta)."""
    first, delta = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().kun_kv_pool_resize_tail(pool, int(new_bytes), ctypes.byref(first), ctypes.byref(delta)),
           "kun_kv_pool_resize_tail")
    return first.value, delta.value


def kun_vmm_region_create(reserve_bytes: int) -> int:
    h = ctypes.c_void_p()
    _check(lib().kun_vmm_region_create(ctypes.byref(h), int(reserve_bytes)), "kun_vmm_region_create")
    return h.value


def kun_vmm_region_info(region: int):
    """Returns (base address, mapped bytes, reserved bytes, granularity)."""
    base, mapped, reserved, gran = ctypes.c_void_p(), ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().kun_vmm_region_info(region, ctypes.byref(base), ctypes.byref(mapped), ctypes.byref(reserved),
                                     ctypes.byref(gran)), "kun_vmm_region_info")
    return base.value, mapped.value, reserved.value, gran.value


def kun_vmm_region_grow(region: int, nbytes: int) -> None:
    _check(lib().kun_vmm_region_grow(region, int(nbytes)), "kun_vmm_region_grow")


def kun_vmm_region_move_tail(src: int, dst: int, nbytes: int) -> None:
    _check(lib().kun_vmm_region_move_tail(src, dst, int(nbytes)), "kun_vmm_region_move_tail")


def kun_vmm_region_shrink(region: int, nbytes: int) -> None:
    _check(lib().kun_vmm_region_shrink(region, int(nbytes)), "kun_vmm_region_shrink")


def kun_vmm_region_destroy(region: int) -> None:
    _check(lib().kun_vmm_region_destroy(region), "kun_vmm_region_destroy")


def device_bytes(address: int, nbytes: int) -> torch.Tensor:
    """uint8 tensor over [address, address + nbytes) of device memory the caller keeps mapped (no copy,
    no ownership)."""
    class _Span:
        __cuda_array_interface__ = {"shape": (int(nbytes),), "typestr": "|u1", "data": (int(address), False),
                                    "version": 3}
    return torch.as_tensor(_Span(), device="cuda")


def kun_kv_pool_num_blocks(pool: int) -> int:
    n = ctypes.c_int64()
    _check(lib().kun_kv_pool_num_blocks(pool, ctypes.byref(n)), "kun_kv_pool_num_blocks")
    return n.value


def kun_kv_pool_num_ranges(pool: int) -> int:
    n = ctypes.c_int()
    _check(lib().kun_kv_pool_num_ranges(pool, ctypes.byref(n)), "kun_kv_pool_num_ranges")
    return n.value


def kun_kv_pool_block_bytes(pool: int) -> int:
    n = ctypes.c_size_t()
    _check(lib().kun_kv_pool_block_bytes(pool, ctypes.byref(n)), "kun_kv_pool_block_bytes")
    return n.value


def kun_kv_pool_resolve(pool: int, block: int):
    """Returns (range index, byte offset inside the range, device address)."""
    r, off, addr = ctypes.c_int(), ctypes.c_size_t(), ctypes.c_void_p()
    _check(lib().kun_kv_pool_resolve(pool, int(block), ctypes.byref(r), ctypes.byref(off),
                                     ctypes.byref(addr)), "kun_kv_pool_resolve")
    return r.value, off.value, addr.value


def kun_kv_pool_destroy(pool: int) -> None:
    _check(lib().kun_kv_pool_destroy(pool), "kun_kv_pool_destroy")


def kun_validate_block_table(pool: int, host_table: torch.Tensor, host_ctx_len: torch.Tensor) -> None:
    """host_table: CPU int32 [rows, max_blocks]; host_ctx_len: CPU int32 [rows]."""
    assert host_table.device.type == "cpu" and host_table.dtype == torch.int32 and host_table.is_contiguous()
    assert host_ctx_len.device.type == "cpu" and host_ctx_len.dtype == torch.int32
    rows, mb = host_table.shape
    _check(lib().kun_validate_block_table(pool, _ptr(host_table), rows, mb, _ptr(host_ctx_len)),
           "kun_validate_block_table")


def kun_slot_map(pool: int, seq_of_tok, pos_of_tok, T: int, block_table, max_blocks: int, kv_head: int,
                 range_out, k_off_out, v_off_out, stream=None) -> None:
    _check(lib().kun_slot_map(pool, _ptr(seq_of_tok), _ptr(pos_of_tok), int(T), _ptr(block_table),
                              int(max_blocks), int(kv_head), _ptr(range_out), _ptr(k_off_out), _ptr(v_off_out),
                              _stream(stream)), "kun_slot_map")


def kun_kv_append(pool: int, k_new, v_new, seq_of_tok, pos_of_tok, T: int, block_table,
                  max_blocks: int, stream=None) -> None:
    _check(lib().kun_kv_append(pool, _ptr(k_new), _ptr(v_new), _ptr(seq_of_tok), _ptr(pos_of_tok),
                               int(T), _ptr(block_table), int(max_blocks), _stream(stream)),
           "kun_kv_append")


def kun_decode_workspace_bytes(pool: int, S: int, num_q_heads: int, total_ctx_upper_bound: int = 0) -> int:
    return lib().kun_decode_workspace_bytes(pool, int(S), int(num_q_heads), int(total_ctx_upper_bound))


def kun_paged_decode(pool: int, q, out, block_table, max_blocks: int, ctx_len, S: int,
                     num_q_heads: int, scale: float, total_ctx_upper_bound: int, workspace,
                     workspace_bytes: int, stream=None) -> None:
    _check(lib().kun_paged_decode(pool, _ptr(q), _ptr(out), _ptr(block_table), int(max_blocks),
                                  _ptr(ctx_len), int(S), int(num_q_heads), float(scale),
                                  int(total_ctx_upper_bound), _ptr(workspace), int(workspace_bytes),
                                  _stream(stream)), "kun_paged_decode")


def kun_decode_plan(pool: int, ctx_len, S: int, num_q_heads: int, total_ctx_upper_bound: int, workspace,
                    workspace_bytes: int, stream=None) -> None:
    _check(lib().kun_decode_plan(pool, _ptr(ctx_len), int(S), int(num_q_heads), int(total_ctx_upper_bound),
                                 _ptr(workspace), int(workspace_bytes), _stream(stream)), "kun_decode_plan")


def kun_paged_decode_planned(pool: int, q, out, block_table, max_blocks: int, ctx_len, S: int,
                             num_q_heads: int, scale: float, total_ctx_upper_bound: int, workspace,
                             workspace_bytes: int, stream=None) -> None:
    _check(lib().kun_paged_decode_planned(pool, _ptr(q), _ptr(out), _ptr(block_table), int(max_blocks),
                                          _ptr(ctx_len), int(S), int(num_q_heads), float(scale),
                                          int(total_ctx_upper_bound), _ptr(workspace), int(workspace_bytes),
                                          _stream(stream)), "kun_paged_decode_planned")


KUN_STATIC_SCRATCH_BYTES = 32 << 20


def kun_paged_decode_static(pool: int, q, out, block_table, max_blocks: int, ctx_len, S: int,
                            num_q_heads: int, scale: float, total_ctx_upper_bound: int, stream=None) -> None:
    _check(lib().kun_paged_decode_static(pool, _ptr(q), _ptr(out), _ptr(block_table), int(max_blocks),
                                         _ptr(ctx_len), int(S), int(num_q_heads), float(scale),
                                         int(total_ctx_upper_bound), _stream(stream)), "kun_paged_decode_static")


def kun_prefill_workspace_bytes(pool: int, n_chunks: int, num_q_heads: int, total_new_tokens: int,
                                max_blocks: int) -> int:
    return lib().kun_prefill_workspace_bytes(pool, int(n_chunks), int(num_q_heads), int(total_new_tokens),
                                             int(max_blocks))


def kun_paged_prefill_chunk(pool: int, q, out, q_start, prior_len, block_table, max_blocks: int,
                            n_chunks: int, num_q_heads: int, total_new_tokens: int, scale: float,
                            workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib().kun_paged_prefill_chunk(pool, _ptr(q), _ptr(out), _ptr(q_start), _ptr(prior_len),
                                         _ptr(block_table), int(max_blocks), int(n_chunks),
                                         int(num_q_heads), int(total_new_tokens), float(scale),
                                         _ptr(workspace), int(workspace_bytes), _stream(stream)),
           "kun_paged_prefill_chunk")


def kun_prefill_plan(pool: int, q_start, prior_len, block_table, max_blocks: int, n_chunks: int,
                     num_q_heads: int, total_new_tokens: int, workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib().kun_prefill_plan(pool, _ptr(q_start), _ptr(prior_len), _ptr(block_table), int(max_blocks),
                                  int(n_chunks), int(num_q_heads), int(total_new_tokens), _ptr(workspace),
                                  int(workspace_bytes), _stream(stream)), "kun_prefill_plan")


def kun_paged_prefill_chunk_planned(pool: int, q, out, q_start, prior_len, block_table, max_blocks: int,
                                    n_chunks: int, num_q_heads: int, total_new_tokens: int, scale: float,
                                    workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib().kun_paged_prefill_chunk_planned(pool, _ptr(q), _ptr(out), _ptr(q_start), _ptr(prior_len),
                                                 _ptr(block_table), int(max_blocks), int(n_chunks),
                                                 int(num_q_heads), int(total_new_tokens), float(scale),
                                                 _ptr(workspace), int(workspace_bytes), _stream(stream)),
           "kun_paged_prefill_chunk_planned")


def kun_paged_prefill_chunk_on(pool: int, q, out, q_start, prior_len, block_table, max_blocks: int,
                               n_chunks: int, num_q_heads: int, total_new_tokens: int, scale: float,
                               max_workgroups: int, workspace, workspace_bytes: int, stream=None) -> None:
    _check(lib().kun_paged_prefill_chunk_on(pool, _ptr(q), _ptr(out), _ptr(q_start), _ptr(prior_len),
                                            _ptr(block_table), int(max_blocks), int(n_chunks),
                                            int(num_q_heads), int(total_new_tokens), float(scale),
                                            int(max_workgroups), _ptr(workspace), int(workspace_bytes),
                                            _stream(stream)),
           "kun_paged_prefill_chunk_on")


# ---- host-side planning (no device work) ---------------------------------------------------------
def _chunk_array(chunks):
    arr = (Chunk * max(len(chunks), 1))()
    for i, (r, p, c) in enumerate(chunks):
        arr[i] = Chunk(int(r), int(p), int(c))
    return arr


def kun_cost_chunk(model, prior: int, tokens: int) -> float:
    return lib().kun_cost_chunk(ctypes.byref(CostModel(*model)), int(prior), int(tokens))


def kun_cost_microbatch(model, chunks) -> float:
    return lib().kun_cost_microbatch(ctypes.byref(CostModel(*model)), _chunk_array(chunks), len(chunks))


def kun_cost_fit(microbatches, seconds):
    """microbatches: list of lists of (request, prior, tokens); returns (alpha, beta, gamma)."""
    flat = [ch for mb in microbatches for ch in mb]
    starts = (ctypes.c_int32 * (len(microbatches) + 1))()
    o = 0
    for k, mb in enumerate(microbatches):
        starts[k] = o
        o += len(mb)
    starts[len(microbatches)] = o
    t = (ctypes.c_double * max(len(seconds), 1))(*[float(x) for x in seconds])
    out = CostModel()
    _check(lib().kun_cost_fit(_chunk_array(flat), starts, len(microbatches), t, ctypes.byref(out)), "kun_cost_fit")
    return out.alpha, out.beta, out.gamma


def kun_lookahead(model, queue, min_tokens: int, max_microbatches: int = 0):
    """Returns the microbatches as lists of (request, prior, tokens)."""
    total = sum(c for _, _, c in queue)
    mb_cap = max(1, min(total // max(min_tokens, 1) + 1, max_microbatches or (1 << 30)))
    ch_cap = len(queue) + mb_cap
    out = (Chunk * ch_cap)()
    starts = (ctypes.c_int32 * (mb_cap + 1))()
    n_mb, n_ch = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().kun_lookahead(ctypes.byref(CostModel(*model)), _chunk_array(queue), len(queue), int(min_tokens),
                               int(max_microbatches), out, ch_cap, starts, mb_cap, ctypes.byref(n_mb),
                               ctypes.byref(n_ch)), "kun_lookahead")
    return [[(out[i].request, out[i].prior, out[i].tokens) for i in range(starts[k], starts[k + 1])]
            for k in range(n_mb.value)]


def kun_drop_plan(n_instances: int, initial_group, num_layers: int, layer_bytes: int, demand_bytes: int):
    """Returns a dict: group_of_instance, kept (list of (first, end)), dropped_bytes, merges (list of
    ((member, size), (member, size))), freed_bytes, demand_met."""
    N = int(n_instances)
    i32a, i64a = ctypes.c_int32 * N, ctypes.c_int64 * N
    grp, kf, ke, db = i32a(), i32a(), i32a(), i64a()
    mm, ms = (ctypes.c_int32 * (2 * max(N - 1, 1)))(), (ctypes.c_int32 * (2 * max(N - 1, 1)))()
    init = None if initial_group is None else i32a(*[int(g) for g in initial_group])
    n_m, freed, met = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_int32()
    _check(lib().kun_drop_plan(N, init, int(num_layers), int(layer_bytes), int(demand_bytes), grp, kf, ke, db, mm, ms,
                               ctypes.byref(n_m), ctypes.byref(freed), ctypes.byref(met)), "kun_drop_plan")
    return {"group_of_instance": list(grp), "kept": list(zip(kf, ke)), "dropped_bytes": list(db),
            "merges": [((mm[2 * k], ms[2 * k]), (mm[2 * k + 1], ms[2 * k + 1])) for k in range(n_m.value)],
            "freed_bytes": freed.value, "demand_met": bool(met.value)}
