"""Device-side plumbing that turns a synthetic Workload into library calls.

Owns the torch buffers (pool ranges, tables, q, out, workspaces) and the pool handle; every
attention step goes through the C-ABI binding in `kun`.  Used by the GPU tests, the smoke check
and the benchmark.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import kun, synth


class DeviceWorkload:
    def __init__(self, w: synth.Workload, device="cuda:0", poison: bool = True,
                 n_ranges_at_create: Optional[int] = None, fill: bool = True,
                 ranges: Optional[List[torch.Tensor]] = None, create_bytes: Optional[int] = None):
        """Allocates one buffer per pool range, creates the pool on range 0 and extends it with the
        others (all of them unless n_ranges_at_create limits it; call extend_next() later).
        `ranges`: use these buffers (shaped like synth.alloc_ranges') instead of allocating;
        `create_bytes`: create the pool on the first create_bytes of range 0 only (a range that grows
        in place: kun_kv_pool_resize_tail)."""
        self.w = w
        self.dev = torch.device(device)
        sh = w.shape
        self.ranges: List[torch.Tensor] = (ranges if ranges is not None
                                           else synth.alloc_ranges(w, self.dev, poison=poison))
        dt = {"f32": kun.KUN_F32, "bf16": kun.KUN_BF16, "fp8": kun.KUN_FP8_E4M3}[sh.dtype]
        r0 = self.ranges[0]
        r0_bytes = r0.numel() * r0.element_size() if create_bytes is None else int(create_bytes)
        self.pool = kun.kun_kv_pool_create(r0, r0_bytes, dt, sh.Hkv, sh.d, sh.B)
        self.n_attached = 1
        want = len(self.ranges) if n_ranges_at_create is None else n_ranges_at_create
        while self.n_attached < want:
            self.extend_next()
        if fill:
            synth.fill_pool(w, self.ranges)
        # decode side
        self.S = w.S
        if self.S:
            self.dec_table = torch.from_numpy(w.table_array(range(self.S))).to(self.dev)
            self.dec_len = torch.from_numpy(w.decode_lens.astype(np.int32)).to(self.dev)
            self.q_dec = synth.q_decode(w, self.dev)
            self.out_dec = torch.zeros_like(self.q_dec)
        # prefill side
        self.n_chunks = w.n_chunks
        if self.n_chunks:
            rows = [w.S + i for i in range(self.n_chunks)]
            self.pre_table = torch.from_numpy(w.table_array(rows)).to(self.dev)
            cs = [c for _, c in w.chunks]
            self.q_start_host = np.concatenate([[0], np.cumsum(cs)]).astype(np.int32)
            self.q_start = torch.from_numpy(self.q_start_host).to(self.dev)
            self.prior = torch.tensor([p for p, _ in w.chunks], dtype=torch.int32, device=self.dev)
            self.q_pre = torch.cat([synth.q_chunk(w, i, self.dev) for i in range(self.n_chunks)])
            self.out_pre = torch.zeros_like(self.q_pre)
            self.total_new = int(self.q_start_host[-1])
        self._ws_dec = None
        self._ws_pre = None

    # ---- pool growth -------------------------------------------------------------------------
    def extend_next(self):
        r = self.ranges[self.n_attached]
        first, n = kun.kun_kv_pool_extend(self.pool, r, r.numel() * r.element_size())
        self.n_attached += 1
        return first, n

    # ---- decode ------------------------------------------------------------------------------
    def decode(self, seqs: Optional[Sequence[int]] = None, ctx_bound: Optional[int] = None,
               stream=None, steps: str = "both") -> torch.Tensor:
        """One decode step over all decode requests (or the first `seqs` ones given as a count).
        steps: "both" (kun_paged_decode), "plan" (kun_decode_plan only) or "planned"
        (kun_paged_decode_planned, after a "plan" call with the same arguments)."""
        sh = self.w.shape
        S = self.S if seqs is None else int(seqs)
        if ctx_bound is None:
            ctx_bound = int(self.w.decode_lens[:S].astype(np.int64).sum())
        need = kun.kun_decode_workspace_bytes(self.pool, S, sh.Hq, ctx_bound)
        if self._ws_dec is None or self._ws_dec.numel() < need:
            self._ws_dec = self._guarded(need, "dec")
        if steps == "plan":
            kun.kun_decode_plan(self.pool, self.dec_len, S, sh.Hq, ctx_bound, self._ws_dec, self._ws_dec.numel(),
                                stream)
            return self.out_dec
        fn = kun.kun_paged_decode_planned if steps == "planned" else kun.kun_paged_decode
        fn(self.pool, self.q_dec, self.out_dec, self.dec_table, self.dec_table.shape[1], self.dec_len, S, sh.Hq,
           sh.scale, ctx_bound, self._ws_dec, self._ws_dec.numel(), stream)
        return self.out_dec

    # ---- prefill -----------------------------------------------------------------------------
    def prefill(self, stream=None, max_workgroups: int = 0, steps: str = "both") -> torch.Tensor:
        """All prefill chunks; max_workgroups > 0 runs them on that many workgroups (mixed batches).
        steps: "both" (kun_paged_prefill_chunk), "plan" (kun_prefill_plan only) or "planned"
        (kun_paged_prefill_chunk_planned, after a "plan" call)."""
        sh = self.w.shape
        need = kun.kun_prefill_workspace_bytes(self.pool, self.n_chunks, sh.Hq, self.total_new,
                                               self.pre_table.shape[1])
        if self._ws_pre is None or self._ws_pre.numel() < need:
            self._ws_pre = self._guarded(max(need, 256), "pre")
        if steps == "plan":
            kun.kun_prefill_plan(self.pool, self.q_start, self.prior, self.pre_table, self.pre_table.shape[1],
                                 self.n_chunks, sh.Hq, self.total_new, self._ws_pre, self._ws_pre.numel(), stream)
            return self.out_pre
        if steps == "planned":
            kun.kun_paged_prefill_chunk_planned(self.pool, self.q_pre, self.out_pre, self.q_start, self.prior,
                                                self.pre_table, self.pre_table.shape[1], self.n_chunks, sh.Hq,
                                                self.total_new, sh.scale, self._ws_pre, self._ws_pre.numel(),
                                                stream)
            return self.out_pre
        if max_workgroups > 0:
            kun.kun_paged_prefill_chunk_on(self.pool, self.q_pre, self.out_pre, self.q_start, self.prior,
                                           self.pre_table, self.pre_table.shape[1], self.n_chunks, sh.Hq,
                                           self.total_new, sh.scale, max_workgroups, self._ws_pre,
                                           self._ws_pre.numel(), stream)
        else:
            kun.kun_paged_prefill_chunk(self.pool, self.q_pre, self.out_pre, self.q_start, self.prior,
                                        self.pre_table, self.pre_table.shape[1], self.n_chunks, sh.Hq,
                                        self.total_new, sh.scale, self._ws_pre, self._ws_pre.numel(),
                                        stream)
        return self.out_pre

    def mixed(self, prefill_stream, decode_stream, prefill_workgroups: int) -> None:
        """Prefill on `prefill_workgroups` compute units and the decode step side by side: both start
        after the work already on the current stream, which in turn waits for both."""
        cur = torch.cuda.current_stream()
        start = torch.cuda.Event()
        start.record(cur)
        prefill_stream.wait_event(start)
        decode_stream.wait_event(start)
        self.prefill(stream=prefill_stream, max_workgroups=prefill_workgroups)
        self.decode(stream=decode_stream)
        for st in (prefill_stream, decode_stream):
            done = torch.cuda.Event()
            done.record(st)
            cur.wait_event(done)

    # ---- workspaces with guard words -----------------------------------------------------------
    GUARD = 256          # bytes in front of and behind every workspace, filled with 0xA5

    def _guarded(self, nbytes: int, name: str) -> torch.Tensor:
        """A workspace of exactly nbytes (256-byte aligned) between two guard areas; check_guards()
        tells whether a kernel wrote outside the size the library asked for."""
        raw = torch.empty(nbytes + 2 * self.GUARD, dtype=torch.uint8, device=self.dev)
        assert raw.data_ptr() % 256 == 0
        raw[:self.GUARD] = 0xA5
        raw[self.GUARD + nbytes:] = 0xA5
        if not hasattr(self, "_guards"):
            self._guards = {}
        self._guards[name] = (raw, nbytes)
        return raw[self.GUARD:self.GUARD + nbytes]

    def check_guards(self) -> None:
        for name, (raw, nbytes) in getattr(self, "_guards", {}).items():
            ok = bool((raw[:self.GUARD] == 0xA5).all()) and bool((raw[self.GUARD + nbytes:] == 0xA5).all())
            assert ok, f"a kernel wrote outside the {name} workspace of {nbytes} bytes"

    def close(self):
        """Destroys the pool object and lets go of the device buffers (the ranges are the caller's memory: here
        the caller is this object)."""
        if self.pool is not None:
            kun.kun_kv_pool_destroy(self.pool)
            self.pool = None
        self.ranges = []
        self._ws_dec = self._ws_pre = None
        self._guards = {}
