#!/usr/bin/env python3
"""Benchmark of the paged-attention hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic batch, with every input already
resident in HBM: KV append of the step's new tokens, chunked prefill of the batch's prefill chunks
and the decode step of its decode requests, all enqueued on one stream through the C ABI.

Prints ONE JSON line.  `value` is the achieved HBM bandwidth of the decode step (algorithmic bytes
of the batch / average duration of the decode call measured with HIP events on the launch stream);
the prefill rate, the per-part times and the oracle timed on the host cores are in the same line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config {2,3,4,5}]

Without --config the line describes configuration 5 (the largest one-GPU workload) and carries, under
"others", the decode and prefill rates of configurations 3, 4 and 2 measured the same way, and of the
default workload over FP8 (E4M3) pages and over blocks of 64 tokens.
"""
import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=0, help="workload 2..5 (default: the largest supported)")
    ap.add_argument("--block-size", type=int, default=0, choices=[0, 16, 32, 64, 128],
                    help="tokens per KV block (default: the configuration's own, 16)")
    ap.add_argument("--q-heads", type=int, default=0,
                    help="query heads (default: the configuration's own); e.g. 40 over the 8 KV heads of cfg 2-4")
    ap.add_argument("--kv-dtype", default="", choices=["", "fp8"],
                    help="element type of the KV pages (default: the configuration's own, bf16); fp8 = E4M3 pages "
                         "with bf16 queries: 2 048 instead of 4 096 algorithmic bytes per token")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--plan-per-call", action="store_true",
                    help="kun_paged_decode and kun_paged_prefill_chunk (plan launch inside every call) instead "
                         "of the plans at the step's start and the planned calls")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the shorter runs of configurations 3, 4 and 2 that follow the default workload")
    ap.add_argument("--no-mixed", action="store_true",
                    help="skip the side-by-side prefill + decode measurement (keeps profiles to the K timed steps)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (known HBM traffic) to scale rocprofv3 --pmc counters")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--cost-model", action="store_true",
                    help="also fit the chunk cost model (prefix + self attention pairs, tokens, constant) to "
                         "measured prefill calls and report its error on held-out microbatches")
    ap.add_argument("--prefill-scaling", action="store_true",
                    help="also run long equal prefill items on all, 128 and 64 compute units and report the rate "
                         "per compute unit and the shader clock (rocm-smi) of each: is the chip power-limited?")
    ap.add_argument("--vmm", action="store_true",
                    help="also time the decode step over the same pool built as ONE virtual range that grew "
                         "chunk by chunk, and the mapping calls themselves")
    return ap.parse_args()


def decode_bytes(w):
    sh = w.shape
    L = w.decode_lens.astype(np.int64)
    kv = int(L.sum()) * 2 * sh.Hkv * sh.d * sh.elt
    qo = w.S * sh.Hq * sh.d * sh.q_elt * 2
    tab = 4 * int(((L + sh.B - 1) // sh.B).sum())
    return kv + qo + tab


def prefill_flops(w):
    sh = w.shape
    return 4 * sh.d * sh.Hq * w.prefill_pairs


def time_steps(cfg, args, block_size=0, q_heads=0, kv_dtype="", settle_ms=0.0):
    """Builds configuration `cfg` on the device and times args.steps steps (after args.warmup untimed
    ones).  A step = KV append of the step's new tokens + chunked prefill + decode on one stream, inputs
    resident in HBM.  Returns (report, dw, dws): the per-part figures, the first DeviceWorkload (kept
    for the follow-up measurements) and all of them (to close)."""
    import torch
    from paper_2412_18169_amd import kun, synth
    from paper_2412_18169_amd.runner import DeviceWorkload
    t_setup = time.time()
    w = synth.config(cfg, block_size, q_heads, kv_dtype)
    sh = w.shape
    dw = DeviceWorkload(w, poison=(cfg != 5))
    torch.cuda.synchronize()
    t_setup = time.time() - t_setup

    # the step's new tokens: the last token of every decode request and every token of every chunk
    seqs, poss, ks, vs = [], [], [], []
    for s in range(w.S):
        L = int(w.decode_lens[s])
        k, v = synth.kv_logical(w, s, L - 1, L, dw.dev)
        ks.append(k); vs.append(v); seqs.append(s); poss.append(L - 1)
    for i, (p, c) in enumerate(w.chunks):
        k, v = synth.kv_logical(w, w.S + i, p, p + c, dw.dev)
        ks.append(k); vs.append(v); seqs += [w.S + i] * c; poss += list(range(p, p + c))
    k_new = torch.cat(ks).contiguous(); v_new = torch.cat(vs).contiguous()
    seq_of = torch.tensor(seqs, dtype=torch.int32, device=dw.dev)
    pos_of = torch.tensor(poss, dtype=torch.int32, device=dw.dev)
    all_table = torch.from_numpy(w.table_array(range(len(w.seq_lens)))).to(dw.dev)
    T_new = len(seqs)
    has_prefill = w.n_chunks > 0 and PREFILL_SUPPORTED

    # A working set below 1 GB could be served in part by the 256 MB last-level cache when the same
    # pool is read step after step: such configurations alternate between two pools (same requests and
    # contents, separate buffers), so every step reads pages that the step before did not touch.
    dws = [dw]
    if decode_bytes(w) < 10**9:
        dws.append(DeviceWorkload(w, poison=True))
    step_no = [0]

    # The decode work list depends on the context lengths only: a serving step makes it once
    # (kun_decode_plan) and every layer's decode call runs against it (kun_paged_decode_planned); the
    # prefill plan (work list + resolved block table) needs neither q nor the pages and can be made
    # ahead of the append.  The step does the same: both plans first, then append and the two planned
    # calls, so the plan launches are part of the step but not of the calls they serve.
    # --plan-per-call: kun_paged_decode and kun_paged_prefill_chunk instead.
    planned = not args.plan_per_call

    def step(ev=None):
        d = dws[step_no[0] % len(dws)]
        step_no[0] += 1
        if ev: ev[0].record()
        if planned:
            d.decode(steps="plan")
            if has_prefill:
                d.prefill(steps="plan")
        kun.kun_kv_append(d.pool, k_new, v_new, seq_of, pos_of, T_new, all_table, all_table.shape[1])
        if ev: ev[1].record()
        if has_prefill:
            d.prefill(steps="planned" if planned else "both")
        if ev: ev[2].record()
        d.decode(steps="planned" if planned else "both")
        if ev: ev[3].record()

    if args.pmc_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dw.dev).zero_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    warmup_steps = args.warmup
    if settle_ms > 0:
        # The configurations reported under "others" have steps of 0.1 to 0.5 ms and start right after a
        # setup phase of host work: three warm-up steps are over before the card has raised its clocks
        # (measured: cfg4's prefill call 0.200 ms after 3 warm-up steps, 0.173 ms after 200).  They warm up
        # for settle_ms of steps instead; the default workload keeps exactly args.warmup.
        t0 = time.time()
        step()
        torch.cuda.synchronize()
        extra = int(settle_ms * 1e-3 / max(time.time() - t0, 1e-5))
        for _ in range(min(extra, 2000)):
            step()
        torch.cuda.synchronize()
        warmup_steps += 1 + min(extra, 2000)
    # HIP events on the stream the kernels are launched on (torch's current stream)
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    t_app = float(np.mean([e[0].elapsed_time(e[1]) for e in evs]))
    t_pre = float(np.mean([e[1].elapsed_time(e[2]) for e in evs]))
    t_dec = float(np.mean([e[2].elapsed_time(e[3]) for e in evs]))
    t_dec_med = float(np.median([e[2].elapsed_time(e[3]) for e in evs]))

    dbytes = decode_bytes(w)
    gbps = dbytes / (t_dec * 1e-3) / 1e9
    rep = {
        "ms_per_step": round(ms_per_step, 4), "dtype": sh.dtype, "warmup_steps": warmup_steps,
        "config": {"workload": f"cfg{cfg}:{w.name}", "block_size": w.shape.B, "pools_alternated": len(dws),
                   "decode_requests": w.S, "prefill_chunks": w.n_chunks if has_prefill else 0,
                   "Hq": sh.Hq, "Hkv": sh.Hkv, "head_dim": sh.d, "kv_dtype": sh.dtype,
                   "pool_ranges": len(w.range_blocks), "pool_GB": round(w.num_blocks * sh.block_bytes / 1e9, 2),
                   "decode_kv_tokens": w.decode_kv_tokens, "seed": w.seed},
        "decode": {"ms": round(t_dec, 4), "ms_median": round(t_dec_med, 4), "algorithmic_bytes": dbytes,
                   "GB_per_s": round(gbps, 1), "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBPS, 4),
                   "requests_per_s": round(w.S / (t_dec * 1e-3), 1),
                   "kv_tokens_per_s": round(w.decode_kv_tokens / (t_dec * 1e-3), 1),
                   "plan": "once per step (kun_decode_plan at the step's start, timed with the append; "
                           "kun_paged_decode_planned is the call)" if planned else "in every call (kun_paged_decode)"},
        "append": {"ms": round(t_app, 4), "tokens": T_new, "with_the_plan_launches": planned},
        "setup_s": round(t_setup, 1),
    }
    if has_prefill:
        fl = prefill_flops(w)
        tf = fl / (t_pre * 1e-3) / 1e12
        rep["prefill"] = {"ms": round(t_pre, 4), "flops": fl, "TFLOP_per_s": round(tf, 1),
                          "frac_of_mfma_peak": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                          "new_tokens_per_s": round(dw.total_new / (t_pre * 1e-3), 1),
                          "plan": "at the step's start (kun_prefill_plan, timed with the append; "
                                  "kun_paged_prefill_chunk_planned is the call)" if planned
                                  else "in every call (kun_paged_prefill_chunk)"}
    return rep, dw, dws


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2412_18169_amd import kun

    kun.lib()   # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    cfg = args.config or DEFAULT_CONFIG
    rep, dw, dws = time_steps(cfg, args, args.block_size, args.q_heads, args.kv_dtype)
    w, sh = dw.w, dw.w.shape
    has_prefill = "prefill" in rep
    gbps = rep["decode"]["GB_per_s"]
    traffic = TRAFFIC.get((cfg, sh.B, sh.Hq, sh.dtype))
    out = {
        "metric": "paged_decode_hbm_bandwidth", "value": gbps, "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": rep["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (fp8 e4m3 pages)" if sh.dtype == "fp8" else sh.dtype,
        "data": "synthetic",
        "config": rep["config"], "decode": rep["decode"], "append": rep["append"],
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(gbps / HBM_PEAK_GBPS, 4),
                     "traffic": traffic[0] if traffic else None,
                     "traffic_source": traffic[1] if traffic else None,
                     "kernel": ("decode_partial_mfma_fp8" if sh.dtype == "fp8" else "decode_partial_mfma") +
                               (" (the planned call: the kernel, and the merge launch behind it when the batch is "
                                "large enough to have one; the step's plan launch is timed with the append)"
                                if not args.plan_per_call else
                                " (timed with the plan launch in front of it and the merge behind it)")},
        "setup_s": rep["setup_s"],
    }
    if has_prefill:
        out["prefill"] = rep["prefill"]

    if has_prefill and not args.pmc_calibration and not args.no_mixed:
        out["mixed"] = mixed_batch(dw, args.steps)

    if args.prefill_scaling:
        out["prefill_scaling"] = prefill_scaling_report(sh)
    if args.vmm:
        out["vmm"] = vmm_report(dw, args.steps)
    if args.cost_model:
        out["cost_model"] = cost_model_report(sh)

    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["max_abs_err_vs_oracle"] = cpu_baseline(dw, args.cpu_seconds)
        if has_prefill:
            out["prefill_max_abs_err_vs_oracle"] = prefill_check(dw)
    for d in dws:
        d.close()
    del dw, dws
    gc.collect()
    torch.cuda.empty_cache()

    # The other configurations the targets are quoted on, same number of steps each: the metric, value,
    # roofline and config above stay those of the default workload.
    if not args.config and not args.no_others and not args.pmc_calibration:
        out["others"] = {}
        runs = [(f"cfg{c}", c, args.block_size, args.kv_dtype) for c in OTHER_CONFIGS]
        if not args.block_size and not args.kv_dtype and not args.q_heads:
            # the default workload in the two variants of the page format: FP8 (E4M3) pages, blocks of 64 tokens
            runs += [(f"cfg{DEFAULT_CONFIG}_fp8_pages", DEFAULT_CONFIG, 0, "fp8"),
                     (f"cfg{DEFAULT_CONFIG}_block_size_64", DEFAULT_CONFIG, 64, "")]
        for name, c, block_size, kv_dtype in runs:
            r, d0, ds = time_steps(c, args, block_size, args.q_heads, kv_dtype,
                                   settle_ms=0.0 if c == DEFAULT_CONFIG else SETTLE_MS)
            o = {"decode_ms": r["decode"]["ms"], "GB_per_s": r["decode"]["GB_per_s"],
                 "frac": r["decode"]["frac_of_hbm_peak"], "decode_kv_tokens": r["config"]["decode_kv_tokens"],
                 "kv_tokens_per_s": r["decode"]["kv_tokens_per_s"], "block_size": r["config"]["block_size"],
                 "kv_dtype": r["config"]["kv_dtype"], "ms_per_step": r["ms_per_step"],
                 "warmup_steps": r["warmup_steps"]}
            if "prefill" in r:
                o.update({"prefill_ms": r["prefill"]["ms"], "TFLOP_per_s": r["prefill"]["TFLOP_per_s"],
                          "prefill_frac": r["prefill"]["frac_of_mfma_peak"]})
            out["others"][name] = o
            for d in ds:
                d.close()
            del d0, ds
            gc.collect()
            torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)


def mixed_batch(dw, steps, prefill_workgroups=256):
    """Prefill (on `prefill_workgroups` workgroups that fetch their items) and decode enqueued side by
    side on two streams, against the same two calls back to back on one stream."""
    import torch
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

    def timed(f):
        for _ in range(2):
            f()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            f()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    def back_to_back():
        dw.prefill()
        dw.decode()

    t_seq = timed(back_to_back)
    t_mix = timed(lambda: dw.mixed(s1, s2, prefill_workgroups))
    return {"ms_back_to_back": round(t_seq, 4), "ms_two_streams": round(t_mix, 4),
            "prefill_workgroups": prefill_workgroups}


def prefill_scaling_report(sh, seconds=2.0):
    """Four chunks of 1024 tokens after 30 000 prior tokens each (long, equal work items: the tile loop
    in steady state) through kun_paged_prefill_chunk_on with 256, 128 and 64 fetching workgroups (one per
    compute unit): Tflop/s, the same scaled to 256 compute units, and the shader clock rocm-smi shows
    while the kernel loops.  Equal rates per compute unit would mean the tile loop sets the pace; a rate
    that rises as compute units go idle, with the clock, means the chip's power limit does."""
    import json as _json
    import subprocess
    import threading
    import torch
    from paper_2412_18169_amd import synth
    from paper_2412_18169_amd.runner import DeviceWorkload
    w = synth.custom_workload("prefill-scaling", sh, [16], chunks=[(30000, 1024)] * 4, seed=78, extra_blocks=2)
    dw = DeviceWorkload(w, poison=False)
    fl = prefill_flops(w)
    clocks, stop = [], [False]

    def poll():
        while not stop[0]:
            try:
                o = subprocess.run(["rocm-smi", "--showclocks", "--json"], capture_output=True, text=True, timeout=5).stdout
                c = _json.loads(o).get("card0", {})
                mhz = [int("".join(ch for ch in v if ch.isdigit())) for k, v in c.items() if k.startswith("sclk clock speed")]
                if mhz:
                    clocks.append((time.time(), mhz[0]))
            except Exception:
                pass
            time.sleep(0.05)

    th = threading.Thread(target=poll, daemon=True)
    th.start()
    rows = []
    for wgs in (0, 256, 128, 64):
        for _ in range(3):
            dw.prefill(max_workgroups=wgs)
        torch.cuda.synchronize()
        t0 = time.time()
        n = 0
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        while time.time() - t0 < seconds:
            for _ in range(10):
                dw.prefill(max_workgroups=wgs)
            torch.cuda.synchronize()
            n += 10
        b.record()
        torch.cuda.synchronize()
        t1 = time.time()
        ms = a.elapsed_time(b) / n
        mid = sorted(m for t, m in clocks if t0 + 0.5 < t < t1)
        cus = wgs or 256
        rows.append({"workgroups": wgs or "one per item", "ms": round(ms, 4),
                     "TFLOP_per_s": round(fl / ms / 1e9, 1),
                     "TFLOP_per_s_per_256_CUs": round(fl / ms / 1e9 * 256 / cus, 1),
                     "sclk_MHz_median": mid[len(mid) // 2] if mid else None})
    stop[0] = True
    dw.close()
    return {"chunks": "4 x (30000 prior, 1024 new)", "flops": fl, "runs": rows}


def cost_model_report(sh, reps=10):
    """Times kun_paged_prefill_chunk on microbatches of 1-4 chunks over a grid of (prior, chunk) sizes,
    fits the three constants of the chunk cost model with kun_cost_fit on two thirds of them and
    reports the relative error of the fitted model, and of a model that counts tokens only, on the
    held-out third."""
    import torch
    from paper_2412_18169_amd import kun, synth
    from paper_2412_18169_amd.runner import DeviceWorkload
    rng = np.random.default_rng(77)
    priors = [0, 1024, 2048, 4096, 8192, 12288, 16384]
    sizes = [1024, 2048, 4096]
    combos = [(p, c) for p in priors for c in sizes]
    w = synth.custom_workload("cost-model", sh, [1], chunks=combos, seed=77, extra_blocks=0)
    dw = DeviceWorkload(w, poison=False)
    # microbatches of 3-8 chunks: enough query tiles to fill every compute unit several times, as the
    # lookahead formulation assumes of a microbatch (a launch that leaves compute units idle is bound
    # by its longest workgroup instead, which no work-based model describes)
    idx_sets = []
    for _ in range(75):
        idx_sets.append(sorted(rng.choice(len(combos), size=int(rng.integers(3, 9)), replace=False).tolist()))
    table_all = dw.pre_table
    times, mbs = [], []
    for ids in idx_sets:
        cs = [combos[i][1] for i in ids]
        q_start = torch.tensor(np.concatenate([[0], np.cumsum(cs)]).astype(np.int32), device=dw.dev)
        prior = torch.tensor([combos[i][0] for i in ids], dtype=torch.int32, device=dw.dev)
        table = table_all[ids].contiguous()
        total = int(sum(cs))
        q = torch.cat([dw.q_pre[int(dw.q_start_host[i]):int(dw.q_start_host[i + 1])] for i in ids]).contiguous()
        o = torch.empty_like(q)
        need = kun.kun_prefill_workspace_bytes(dw.pool, len(ids), sh.Hq, total, table.shape[1])
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dw.dev)

        def call():
            kun.kun_paged_prefill_chunk(dw.pool, q, o, q_start, prior, table, table.shape[1], len(ids), sh.Hq,
                                        total, sh.scale, ws, ws.numel())
        for _ in range(2):
            call()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            call()
        b.record()
        torch.cuda.synchronize()
        times.append(a.elapsed_time(b) / reps * 1e-3)
        mbs.append([(i, combos[i][0], combos[i][1]) for i in ids])
    dw.close()
    order = rng.permutation(len(mbs))
    test = set(order[: len(mbs) // 3].tolist())
    train = [k for k in range(len(mbs)) if k not in test]
    model = kun.kun_cost_fit([mbs[k] for k in train], [times[k] for k in train])
    # token-count model: time = b * tokens + g, fitted on the same samples
    X = np.array([[sum(c for _, _, c in mbs[k]), 1.0] for k in train])
    tb, tg = np.linalg.lstsq(X, np.array([times[k] for k in train]), rcond=None)[0]
    err, err_tok = [], []
    for k in sorted(test):
        pred = kun.kun_cost_microbatch(model, mbs[k])
        err.append(abs(pred - times[k]) / times[k])
        err_tok.append(abs(tb * sum(c for _, _, c in mbs[k]) + tg - times[k]) / times[k])
    ktest = sorted(test)
    worst = ktest[int(np.argmax(err))]
    return {"alpha_s_per_pair": model[0], "beta_s_per_token": model[1], "gamma_s": model[2],
            "fitted_on": len(train), "held_out": len(test),
            "rel_err_mean": round(float(np.mean(err)), 4), "rel_err_max": round(float(np.max(err)), 4),
            "held_out_within_5_percent": int(sum(e < 0.05 for e in err)),
            "worst_held_out": {"chunks_prior_tokens": [(p_, c_) for _, p_, c_ in mbs[worst]],
                               "measured_ms": round(times[worst] * 1e3, 4),
                               "predicted_ms": round(kun.kun_cost_microbatch(model, mbs[worst]) * 1e3, 4)},
            "token_count_model_rel_err_mean": round(float(np.mean(err_tok)), 4),
            "token_count_model_rel_err_max": round(float(np.max(err_tok)), 4),
            "shape": {"Hq": sh.Hq, "Hkv": sh.Hkv, "head_dim": sh.d}}


def vmm_report(dw, steps):
    """The workload's pool built twice with the same block ids and contents -- as the range table (one
    buffer per range) and as ONE virtual range that grew range by range, each range a chunk of physical
    memory that starts life in another region (as parameter memory would) and is moved to the tail:
    decode time of both, bit-identity of the outputs, and the host time of the mapping calls.
    Ranges are rounded up to 2 MiB (32 blocks) so that chunk and range boundaries coincide."""
    import copy
    import torch
    from paper_2412_18169_amd import kun, synth
    from paper_2412_18169_amd.runner import DeviceWorkload
    sh = dw.w.shape
    bb = sh.block_bytes
    unit = (1 << 21) // bb
    if sum(dw.w.range_blocks) * bb > 40 * 10**9:
        return {"skipped": "two more copies of this pool do not fit next to it"}
    w = copy.copy(dw.w)
    w.range_blocks = [(nb + unit - 1) // unit * unit for nb in dw.w.range_blocks]
    if getattr(dw.w, "phase_resident", None) is not None:
        synth.assign_blocks_phased(w)
    else:
        synth.assign_blocks_scattered(w)
    torch.cuda.synchronize()

    def host_us(f):
        t0 = time.perf_counter()
        f()
        return (time.perf_counter() - t0) * 1e6

    def dec_ms(d):
        for _ in range(3):
            d.decode()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(steps):
            d.decode()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / steps

    d0 = DeviceWorkload(w)
    t_table = dec_ms(d0)
    ref = d0.decode().clone()
    torch.cuda.synchronize()
    sizes = [nb * bb for nb in w.range_blocks]
    region = kun.kun_vmm_region_create(sum(sizes))
    scratch = kun.kun_vmm_region_create(max(sizes))
    base, _, _, gran = kun.kun_vmm_region_info(region)
    calls = []
    for sz in sizes:
        t_create = host_us(lambda: kun.kun_vmm_region_grow(scratch, sz))
        t_move = host_us(lambda: kun.kun_vmm_region_move_tail(scratch, region, sz))
        calls.append({"MiB": sz >> 20, "create_and_map_us": round(t_create, 1), "move_tail_us": round(t_move, 1)})
    full = kun.device_bytes(base, sum(sizes)).view(sh.torch_dtype).view(-1, sh.Hkv, 2, sh.B * sh.d)
    o = 0
    for r in d0.ranges:                               # same contents at the same block ids
        full[o:o + r.shape[0]].copy_(r)
        o += r.shape[0]
    w1 = copy.copy(w)
    w1.range_blocks = [sum(w.range_blocks)]
    d1 = DeviceWorkload(w1, ranges=[full], create_bytes=sizes[0], fill=False)
    have = sizes[0]
    for sz in sizes[1:]:
        have += sz
        kun.kun_kv_pool_resize_tail(d1.pool, have)
    t_one = dec_ms(d1)
    same = bool(torch.equal(d1.decode(), ref))
    torch.cuda.synchronize()
    t_back = host_us(lambda: kun.kun_vmm_region_move_tail(region, scratch, sizes[-1]))
    d0.close()
    d1.close()
    kun.kun_vmm_region_destroy(region)
    kun.kun_vmm_region_destroy(scratch)
    return {"decode_ms_range_table": round(t_table, 4), "decode_ms_one_virtual_range": round(t_one, 4),
            "ranges": len(sizes), "bit_identical": same, "mapping_calls": calls,
            "move_last_chunk_back_us": round(t_back, 1), "granularity": gran}


def cpu_baseline(dw, target_s):
    """Time the oracle (as it stands) on a bounded sample of the same batch's decode requests and
    check the GPU output of those requests against it."""
    import torch
    from oracle import bridge, paged_attention as O
    w, sh = dw.w, dw.w.shape
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    out_gpu = dw.decode().double().cpu().numpy()
    torch.cuda.synchronize()
    # sample: requests in batch order until about ORACLE_TOKENS_PER_S * target_s KV tokens
    budget = int(ORACLE_TOKENS_PER_S * (0.15 if sh.dtype == "fp8" else 1.0) * target_s)   # (widening E4M3 codes is slower)
    rows, tot = [], 0
    for s in range(w.S):
        rows.append(s)
        tot += int(w.decode_lens[s])
        if tot >= budget:
            break
    lens = [int(w.decode_lens[s]) for s in rows]
    pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[s] for s in rows], lens,
                                    sh.Hkv, sh.d, sh.B, sh.dtype)
    qb = bridge.host_bits(dw.q_dec[rows])
    t0 = time.perf_counter()
    ref = O.paged_decode(pool, qb, tab, lens, sh.Hq, sh.scale)
    dt = time.perf_counter() - t0
    err = float(np.abs(out_gpu[rows] - ref).max())
    nbytes = tot * 2 * sh.Hkv * sh.d * sh.elt + len(rows) * sh.Hq * sh.d * sh.q_elt * 2
    return ({"value": round(nbytes / dt / 1e9, 4), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
             "seconds": round(dt, 2),
             "sample": f"decode of the first {len(rows)} of {w.S} requests ({tot} KV tokens) of the same batch, "
                       f"fp64 numpy oracle"}, err)


def prefill_check(dw, rows_per_chunk=6):
    """GPU prefill output of a few rows of every chunk (first, last, seeded random) against the oracle."""
    import torch
    from oracle import bridge, paged_attention as O
    w, sh = dw.w, dw.w.shape
    got = dw.prefill().double().cpu().numpy()
    torch.cuda.synchronize()
    rng = np.random.default_rng(w.seed)
    worst = 0.0
    for i, (p, c) in enumerate(w.chunks):
        seq = w.S + i
        q0 = int(dw.q_start_host[i])
        rows = sorted(set([0, c - 1] + list(rng.choice(c, size=min(c, rows_per_chunk), replace=False))))
        pool, tab = bridge.compact_pool(dw.ranges, w.range_blocks, [w.block_tables[seq]], [p + c], sh.Hkv, sh.d,
                                        sh.B, sh.dtype)
        ref, _ = O.paged_prefill_chunk(pool, bridge.host_bits(dw.q_pre[q0:q0 + c]), tab[0], p, c, sh.Hq, sh.scale,
                                       rows=rows)
        worst = max(worst, float(np.abs(got[q0:q0 + c][rows] - ref).max()))
    return worst


# Largest workload every part of which is implemented; chunked prefill joins when its kernel lands.
DEFAULT_CONFIG = 5
PREFILL_SUPPORTED = True
ORACLE_TOKENS_PER_S = 80000.0      # rough speed of the numpy oracle, only used to size its sample
OTHER_CONFIGS = (3, 4, 2)          # reported under "others" after the default workload
SETTLE_MS = 100.0                  # ... after this much warm-up (their steps are 0.1 to 0.5 ms long)
# HBM bytes per decode launch from rocprofv3 --pmc runs of an EARLIER session (not of this run), keyed by
# (config, block size, query heads, page dtype): (bytes, where the figure comes from).
TRAFFIC = {
    (5, 16, 64, "bf16"): (17134246810, "profiles/bench_cfg5_70b_stage_kernels.md: rocprofv3 --pmc FETCH_SIZE (x2.0) + WRITE_SIZE of "
                                       "decode_partial_mfma in an earlier session of this build, 1.004 x the algorithmic bytes; not "
                                       "measured in this run"),
    (5, 16, 64, "fp8"): (8612556800, "profiles/bench_cfg5_fp8_pages_kernels.md: rocprofv3 --pmc FETCH_SIZE (x2.0) of "
                                     "decode_partial_mfma_fp8 in an earlier session of this build (reads only), 1.009 x the "
                                     "algorithmic bytes; not measured in this run"),
}

if __name__ == "__main__":
    main()
