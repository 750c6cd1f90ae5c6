#!/usr/bin/env python3
"""Benchmark of the fused-RoPE paged-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--only NAME[,NAME..]] [--no-cpu-baseline]

With no flags it measures every benchmark workload that fits a roofline (configs 2, 3, 4, 5), the commit step
(prompt shape in bf16 and bf16 -> e4m3, decode-step shape) and the matrix-instruction-only calibration kernel, and
prints ONE JSON line. A step is one call of the library over the whole batch of the workload (gather through the
block tables, rotary embedding of K and Q on chip, online softmax, PV, split-K combine), every input already
resident in HBM. Block tables come from the library's own aligner before the timed region (the scheduling path runs
once per request, not once per decode step); its cost is reported separately.

The top level of the line (`value`, `ms_per_step`, `config`, `roofline`, `cpu_baseline`) describes ONE run: the
Llama-3-8B-shaped decode workload laid out with one page per logical block, so that every byte has to come from HBM,
with the caller's read-once hint — a rate that can be held against the 8 TB/s peak. What the page-sharing layout
delivers (pages served from L2 / Infinity Cache: a cache rate, not an HBM rate) is under `layouts`, the other
workloads under `configs`. `--only` restricts the run to some records (names: cfg2 cfg3 cfg4 cfg5 commit_bf16
commit_fp8 commit_decode mfma_probe), e.g. for a profiler; the top level then describes the first of them.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
N_LAYERS = 32            # layers that share one decode plan (block tables are per request, not per layer)
PLAN_HORIZON = 32        # decode steps one plan built ahead serves

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command
# (counter readings in KiB, each scaled by what the same counter reads for a 1 GiB device copy: FETCH_SIZE x2.000,
# WRITE_SIZE x1.000). Summaries with the commands are under profiles/.
MEASURED_TRAFFIC = {
    ("cfg2", "decode_mfma_bf16"): int((552111.8 * 2.0 + 5236.3) * 1024),
    ("cfg4", "decode_mfma_bf16"): int((1050328.9 * 2.0 + 4266.7) * 1024),
    ("cfg5", "decode_mfma_fp8"): int((1111731.1 * 2.0 + 9313.1) * 1024),
    ("cfg3", "prefill_mfma_bf16"): int((374300.0 * 2.0 + 32770.0) * 1024),
    ("commit_bf16", "kv_commit"): int((131422.6 * 2.0 + 265693.8) * 1024),
    ("commit_fp8", "kv_commit"): int((131432.1 * 2.0 + 131072.0) * 1024),
    ("commit_bf16_unaligned", "kv_commit"): int((131422.3 * 2.0 + 276860.1) * 1024),
    ("commit_fp8_unaligned", "kv_commit"): int((131385.7 * 2.0 + 174081.0) * 1024),
    ("commit_decode", "kv_commit"): int((8283.7 * 2.0 + 147456.0) * 1024),
}
ALL = ["cfg2", "cfg3", "cfg4", "cfg5", "commit_bf16", "commit_fp8", "commit_decode", "mfma_probe"]


def algorithmic_bytes(case) -> int:
    """Bytes the method must move per call: K and V of every addressed slot, block-table entries,
    per-page scales (fp8), q in and out. No rotated copy of K, no cos/sin table."""
    st = case.st
    qb = 4 if st.q_dtype == "f32" else 2
    n = case.kv_bytes_logical()
    n += int(case.n_blocks.sum()) * 4
    if st.kv_dtype == "f8e4m3":
        n += int(case.n_blocks.sum()) * 8
    n += 2 * case.n_q * st.Hq * st.D * qb
    return n


def visible_pairs(case) -> int:
    """(query, key) pairs that take part, per query head (prefill: causal by position)."""
    import numpy as np
    if case.cu_q_lens is None:
        return int(case.kv_lens.astype(np.int64).sum())
    total = 0
    for b in range(case.st.B):
        pos = case.q_positions[case.cu_q_lens[b]:case.cu_q_lens[b + 1]].astype(np.int64)
        total += int(np.minimum(pos + 1, int(case.kv_lens[b])).sum())
    return total


def time_steps(dc, steps: int, warmup: int, batched: bool = False):
    """Run warmup + 2 x steps calls on torch's current stream. After the warmup, a pass of `steps` calls with HIP
    events, handed to the library through timing_start / timing_stop, that bracket the main kernel of every call
    alone (on the stream the library launches on). Then the timed pass: the same `steps` calls with nothing between
    them, bracketed by two events and a synchronize on both sides (an event recorded between calls costs several
    microseconds of a 60-200 us step, so the pass that carries them is not the one that is timed).
    Returns (ms per call of the timed pass, mean main-kernel ms of the pass with events)."""
    import torch
    M = dc.M
    run = M.attn_prefill if dc.prefill else M.attn_decode
    if batched:
        run = lambda params: M.attn_decode_batched(params, dc.plan, dc.plan_info)
    for _ in range(warmup):
        run(dc.params)
    torch.cuda.synchronize()
    k0 = [M.HipEvent() for _ in range(steps)]
    k1 = [M.HipEvent() for _ in range(steps)]
    for i in range(steps):
        dc.params.timing_start, dc.params.timing_stop = k0[i].handle, k1[i].handle
        run(dc.params)
    torch.cuda.synchronize()
    dc.params.timing_start = dc.params.timing_stop = None
    kern = [k0[i].elapsed_ms(k1[i]) for i in range(steps)]
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0.record()
    for _ in range(steps):
        run(dc.params)
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1) / steps, sum(kern) / len(kern)


def time_cold(dc, n: int = 5) -> float:
    """Per-call ms with cold caches: a 1 GiB memset (four times the Infinity Cache) runs before every call."""
    import torch
    run = dc.M.attn_prefill if dc.prefill else dc.M.attn_decode
    flush = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    ms = []
    for _ in range(n):
        flush.zero_()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        run(dc.params)
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1))
    del flush
    return sum(ms) / len(ms)


def oracle_sample(case, got, n_rows_total, cpu_seconds, prefill, flops, abytes):
    """The oracle as it stands on this machine's host cores, on a bounded random sample of (query token, head) rows of the
    same workload; also a live parity check of the timed output."""
    import numpy as np
    from oracle import attn as oracle_attn
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from harness import oracle_out
    st = case.st
    # ~0.15 us per (row, key) at D = 128 on the 16 host cores of a GPU machine
    per_row = 0.15e-6 * max(1.0, float(case.kv_lens.mean()))
    n_rows = max(8, min(n_rows_total, int(cpu_seconds / per_row)))
    if n_rows >= n_rows_total:
        rows = [(t, h) for t in range(case.n_q) for h in range(st.Hq)]
    else:
        rng = np.random.default_rng(0)
        rows = sorted({(int(rng.integers(case.n_q)), int(rng.integers(st.Hq))) for _ in range(n_rows)})
    t0 = time.perf_counter()
    want = oracle_out(oracle_attn, case, rows=rows)
    cpu_s = time.perf_counter() - t0
    err = float(np.abs(np.stack([got[t, h] for t, h in rows]) - want).max())
    whole = cpu_s * n_rows_total / len(rows)
    return dict(value=(flops / whole / 1e12) if prefill else (abytes / whole / 1e9), unit="TFLOP/s" if prefill else "GB/s",
                cores=oracle_attn.num_threads(), kind="oracle",
                sample=f"{len(rows)} of {n_rows_total} (query token, head) rows in {cpu_s:.2f} s, scaled to the whole job",
                max_abs_err_of_gpu_on_sample=err)


def bench_attention(cfg: int, args, mfma_measured=None, ref_mhz=None) -> dict:
    """One benchmark attention workload: every layout and call variant, its roofline record, the oracle beside it."""
    import numpy as np
    import torch
    import paper_2512_16822_amd as M
    import workloads as W
    from paper_2512_16822_amd.device_case import DeviceCase, align_with_library

    st = W.config(cfg)
    t0 = time.perf_counter()
    aligned, pool = align_with_library(M, st)
    align_s = time.perf_counter() - t0
    stats = pool.stats()
    case = W.assemble(st, aligned, poison=False)
    prefill = st.mode == "prefill"
    abytes, ubytes = algorithmic_bytes(case), case.kv_bytes_unique()
    flops = 4 * st.D * visible_pairs(case) * st.Hq
    rec = dict(workload=st.name, B=st.B, Hq=st.Hq, Hkv=st.Hkv, D=st.D, P=st.P, kv_len_mean=float(case.kv_lens.mean()),
               kv_len_max=int(case.kv_lens.max()), n_q_tokens=case.n_q, algorithmic_bytes=abytes,
               unique_kv_bytes=ubytes, useful_flops=flops,
               dtype={"f32": "f32", "bf16": "bf16", "f8e4m3": "bf16 (fp8 e4m3 KV)"}[st.kv_dtype],
               accounting=dict(pages_unique=stats["pages_in_use_unique"], pages_duplicated=stats["pages_logical_duplicated"],
                               ratio=stats["pages_logical_duplicated"] / max(1, stats["pages_in_use_unique"]),
                               aligner_us_per_request=align_s / max(1, st.B) * 1e6))
    gbs = lambda nbytes, ms: nbytes / (ms * 1e-3) / 1e9
    layouts = {}

    # ---- page-sharing layout (the workload as named): pages shared between requests come from the caches ----
    dc = DeviceCase(M, case)
    call_ms, kern_ms = time_steps(dc, args.steps, args.warmup)
    kernel = M.last_kernel()
    shared_out = dc.out.float().cpu()
    clock_ghz = None
    if prefill:
        layouts["shared"] = dict(call_ms=call_ms, kernel_ms=kern_ms, kernel=kernel, tflops=flops / (call_ms * 1e-3) / 1e12)
        if kernel == "prefill_mfma_bf16" and ref_mhz:
            # the kernel's own clock sample (workgroup 0; the last 16 bytes of the workspace size the library reports)
            torch.cuda.synchronize()
            off = M.attn_workspace_size(dc.params, True) - 16
            clocks, ticks = [int(x) for x in dc.ws[off:off + 16].view(torch.int64).cpu()]
            if 0 < ticks < 10 ** 9 and 0 < clocks < 10 ** 12:
                clock_ghz = clocks / (ticks / (ref_mhz * 1e6)) / 1e9
        if not args.no_cold:
            layouts["shared"]["cold_call_ms"] = time_cold(dc)
    else:
        layouts["shared"] = dict(call_ms=call_ms, kernel_ms=kern_ms, kernel=kernel, bound="cache",
                                 gbs_logical=gbs(abytes, call_ms), gbs_unique=gbs(ubytes, call_ms),
                                 note="pages many requests alias are served from L2 / Infinity Cache: not an HBM rate")
        if not args.no_cold:
            layouts["shared"]["cold_call_ms"] = time_cold(dc)
        if kernel.startswith("decode_mfma"):
            # the same job with one pass over shared pages for several requests (plan built on the host)
            fmt = M.F8E4M3 if st.kv_dtype == "f8e4m3" else M.BF16
            info = dc.prepare_batched()
            plan_s = min(_timed(lambda: M.decode_plan_build(case.block_tables, case.kv_lens, st.P, st.Hq, st.Hkv, fmt))
                         for _ in range(3))
            b_ms, b_kern = time_steps(dc, args.steps, args.warmup, batched=True)
            diff = (dc.out.float().cpu() - shared_out).abs().max().item()
            assert diff <= 4e-2, f"batched and plain decode disagree by {diff}"
            batched = dict(call_ms=b_ms, kernel_ms=b_kern, kernel=M.last_kernel(), bound="cache",
                           gbs_logical=gbs(abytes, b_ms), gbs_unique=gbs(ubytes, b_ms), plan=info.as_dict(),
                           plan_build_ms=plan_s * 1e3)
            # A plan built ahead serves PLAN_HORIZON decode steps of all N_LAYERS layers. Measured half-way through its
            # horizon: built from kv_lens - H/2, used at kv_lens.
            half = PLAN_HORIZON // 2
            early = np.maximum(case.kv_lens - half, 0).astype(np.int32)
            build = lambda: M.decode_plan_build(case.block_tables, early, st.P, st.Hq, st.Hkv, fmt, horizon_tokens=PLAN_HORIZON)
            ahead_s = min(_timed(build) for _ in range(3))
            plan, ainfo = build()
            dc.plan_info, dc.plan = ainfo, torch.from_numpy(plan).to(dc.q.device)
            nbytes = M.attn_decode_batched_workspace_size(dc.params, ainfo)
            if nbytes > dc.ws.numel():
                dc.ws = torch.empty(nbytes, dtype=torch.uint8, device=dc.q.device)
                dc.params.workspace, dc.params.workspace_bytes = dc.ws.data_ptr(), nbytes
            a_ms, _ = time_steps(dc, args.steps, args.warmup, batched=True)
            diff = (dc.out.float().cpu() - shared_out).abs().max().item()
            assert diff <= 4e-2, f"batched decode with a plan built ahead and plain decode disagree by {diff}"
            amort_us = ahead_s * 1e6 / (PLAN_HORIZON * N_LAYERS)
            batched["plan_ahead"] = dict(horizon_steps=PLAN_HORIZON, layers_sharing_a_plan=N_LAYERS, build_ms=ahead_s * 1e3,
                                         call_ms=a_ms, amortised_plan_us_per_call=amort_us,
                                         end_to_end_us_per_call=a_ms * 1e3 + amort_us, plain_call_us=call_ms * 1e3,
                                         gain_us_per_call=call_ms * 1e3 - (a_ms * 1e3 + amort_us))
            layouts["shared_batched"] = batched
    del dc
    torch.cuda.empty_cache()

    # ---- one page per logical block: every byte comes from HBM (decode: the layout the HBM roofline is quoted on) ----
    if prefill:
        traffic = MEASURED_TRAFFIC.get((f"cfg{cfg}", kernel))
        ach = flops / (kern_ms * 1e-3) / 1e12
        roofline = dict(bound="mfma", achieved=ach, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s", frac=ach / MFMA_BF16_PEAK_TFLOPS,
                        traffic=traffic, layout="shared", kernel=kernel, kernel_ms=kern_ms, call_ms=call_ms,
                        frac_call=flops / (call_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS)
        if mfma_measured:
            roofline["peak_measured"] = mfma_measured
            roofline["frac_of_measured"] = ach / mfma_measured
        if clock_ghz:
            # what the matrix cores could do at the clock the kernel actually ran at (the nominal peak is at 2.4 GHz)
            roofline["clock_ghz"] = clock_ghz
            roofline["peak_at_clock"] = MFMA_BF16_PEAK_TFLOPS * clock_ghz / 2.4
            roofline["frac_at_clock"] = ach / roofline["peak_at_clock"]
        main = dict(value=flops / (call_ms * 1e-3) / 1e12, unit="TFLOP/s", ms=call_ms, layout="shared",
                    metric="fused-RoPE paged prefill attention throughput")
    else:
        dup = W.to_duplicated(case)
        dch = DeviceCase(M, dup, flags=M.FLAG_KV_READ_ONCE)   # no page is shared: the caller says so
        h_ms, h_kern = time_steps(dch, args.steps, args.warmup)
        assert torch.equal(dch.out.float().cpu(), shared_out), "layouts disagree"
        layouts["duplicated_read_once_hint"] = dict(call_ms=h_ms, kernel_ms=h_kern, kernel=M.last_kernel(), bound="hbm",
                                                    gbs=gbs(abytes, h_ms), frac_call=gbs(abytes, h_ms) / HBM_PEAK_GBS,
                                                    frac_kernel=gbs(abytes, h_kern) / HBM_PEAK_GBS)
        if not args.no_cold:
            layouts["duplicated_read_once_hint"]["cold_call_ms"] = time_cold(dch)
        del dch
        dcn = DeviceCase(M, dup)
        n_ms, n_kern = time_steps(dcn, args.steps, args.warmup)
        layouts["duplicated"] = dict(call_ms=n_ms, kernel_ms=n_kern, kernel=M.last_kernel(), bound="hbm", gbs=gbs(abytes, n_ms),
                                     frac_call=gbs(abytes, n_ms) / HBM_PEAK_GBS, frac_kernel=gbs(abytes, n_kern) / HBM_PEAK_GBS)
        del dcn, dup
        torch.cuda.empty_cache()
        ach = gbs(abytes, h_kern)
        roofline = dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                        traffic=MEASURED_TRAFFIC.get((f"cfg{cfg}", kernel)), layout="duplicated_read_once_hint",
                        kernel=kernel, kernel_ms=h_kern, call_ms=h_ms, frac_call=gbs(abytes, h_ms) / HBM_PEAK_GBS,
                        frac_without_hint=gbs(abytes, n_kern) / HBM_PEAK_GBS)
        main = dict(value=gbs(abytes, h_ms), unit="GB/s", ms=h_ms, layout="duplicated_read_once_hint",
                    metric="fused-RoPE paged decode attention KV throughput")
    rec.update(layouts=layouts, roofline=roofline, main=main)
    rec["cpu_baseline"] = None if args.no_cpu_baseline else oracle_sample(
        case, shared_out.double().numpy(), case.n_q * st.Hq, args.cpu_seconds, prefill, flops, abytes)
    return rec


def _timed(f) -> float:
    t0 = time.perf_counter()
    f()
    return time.perf_counter() - t0


def bench_commit(kind: str, args) -> dict:
    """The commit step alone (scatter of new un-rotated K/V into their pages), Llama-3-8B KV shape (Hkv 8, D 128):
    `bf16` / `fp8`: 64 requests x 1024 new tokens into bf16 pages of 16 slots / e4m3 pages of 32 slots (prompt commit;
    every run starts on a page boundary, as every segment of an aligned prompt does, §3.2.1);
    `bf16_unaligned` / `fp8_unaligned` (only on request): the same with runs that start at slot 0, 8 or 16 of a page;
    `decode`: 4096 requests x one token into bf16 pages (what a decode step of a large batch commits per layer).
    HBM roofline on source bytes read + page bytes written."""
    import numpy as np
    import torch
    import paper_2512_16822_amd as M
    import workloads as W
    unaligned = kind.endswith("_unaligned")
    kind = kind.replace("_unaligned", "")
    fp8 = kind == "fp8"
    kv_dtype, P = ("f8e4m3", 32) if fp8 else ("bf16", 16)
    Hkv, D = 8, 128
    B, T = (4096, 1) if kind == "decode" else (64, 1024)
    MB = 2 if kind == "decode" else T // P + 2
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(10)
    pages = W.gen_pages(25, B * MB, Hkv, P, D, kv_dtype)
    bt = rng.permutation(B * MB).reshape(B, MB).astype(np.int32)
    i32 = lambda a: torch.tensor(np.asarray(a, dtype=np.int32), dtype=torch.int32, device=dev)
    src_cpu = lambda: torch.from_numpy(rng.standard_normal((B * T, Hkv, D)).astype(np.float32)).to(torch.bfloat16)
    k_cpu, v_cpu = src_cpu(), src_cpu()
    k_new, v_new = k_cpu.to(dev), v_cpu.to(dev)
    k_dev, v_dev = pages.k.to(dev), pages.v.to(dev)
    ks = None if pages.k_scales is None else pages.k_scales.to(dev)
    vs = None if pages.v_scales is None else pages.v_scales.to(dev)
    first = ([int(rng.integers(P)) for _ in range(B)] if kind == "decode" else
             [(b % 3) * 8 for b in range(B)] if unaligned else [(b % 2) * P for b in range(B)])
    p = M.make_commit_params(k_new, v_new, k_dev, v_dev, i32(bt), i32(np.arange(B)), i32(first), i32(np.arange(B + 1) * T),
                             k_scales=ks, v_scales=vs)
    for _ in range(args.warmup):
        M.kv_commit(p)
    torch.cuda.synchronize()
    k0 = [M.HipEvent() for _ in range(args.steps)]
    k1 = [M.HipEvent() for _ in range(args.steps)]
    for i in range(args.steps):
        p.timing_start, p.timing_stop = k0[i].handle, k1[i].handle
        M.kv_commit(p)
    torch.cuda.synchronize()
    p.timing_start = p.timing_stop = None
    kern_ms = sum(a.elapsed_ms(b) for a, b in zip(k0, k1)) / args.steps
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        M.kv_commit(p)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    n_el = 2 * B * T * Hkv * D
    blocks_touched = B * (-(-(max(first) + T) // P))
    abytes = n_el * 2 + n_el * (1 if fp8 else 2) + blocks_touched * 4 + (blocks_touched * 8 if fp8 else 0) + (3 * B + 1) * 4
    ach = abytes / (kern_ms * 1e-3) / 1e9
    rec = dict(workload=f"commit_{kind}{'_unaligned' if unaligned else ''}_{B}x{T}_llama3_8b_{kv_dtype}", B=B, new_tokens=B * T, Hkv=Hkv, D=D, P=P,
               dtype="bf16 -> e4m3" if fp8 else "bf16", algorithmic_bytes=abytes, call_ms=ms,
               main=dict(value=abytes / (ms * 1e-3) / 1e9, unit="GB/s", ms=ms, layout="private pages",
                         metric="KV commit throughput (source read + page write)"),
               roofline=dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                             traffic=MEASURED_TRAFFIC.get((f"commit_{kind}{'_unaligned' if unaligned else ''}", "kv_commit")), kernel="kv_commit",
                             kernel_ms=kern_ms, call_ms=ms, frac_call=abytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS))
    rec["cpu_baseline"] = None
    if not args.no_cpu_baseline:
        from oracle import commit as oracle_commit
        n_runs = {"bf16": 32, "fp8": 16, "decode": B}[kind]     # a bounded share of the runs, scaled to the whole job
        raw = lambda t: t.view(torch.uint8 if t.dtype == torch.float8_e4m3fn else torch.uint16).numpy().reshape(-1).copy()
        k_ref, v_ref = raw(pages.k), raw(pages.v)
        cu = np.arange(n_runs + 1) * T
        t0 = time.perf_counter()
        oracle_commit.kv_commit(k_ref, v_ref, None if not fp8 else pages.k_scales.numpy(),
                                None if not fp8 else pages.v_scales.numpy(),
                                k_cpu.view(torch.uint16).numpy()[: n_runs * T], v_cpu.view(torch.uint16).numpy()[: n_runs * T],
                                bt, list(range(n_runs)), first[:n_runs], cu, Hkv=Hkv, D=D, P=P, kv_dtype=kv_dtype)
        cpu_s = time.perf_counter() - t0
        whole = cpu_s * B / n_runs
        rec["cpu_baseline"] = dict(value=abytes / whole / 1e9, unit="GB/s", cores=1, kind="oracle",
                                   sample=f"{n_runs} of {B} runs ({n_runs * T} tokens) in {cpu_s:.2f} s, scaled to the whole job")
    return rec


def bench_mfma_probe(args) -> dict:
    """The matrix-instruction-only kernel: what the chip sustains on v_mfma_f32_32x32x16_bf16 with every CU busy."""
    import torch
    import paper_2512_16822_amd as M
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    iters = 20000
    ref_mhz = M.device_counter_khz() / 1e3
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def rate(random_operands: bool):
        for _ in range(2):
            M.probe_mfma_bf16(iters, sink, random_operands=random_operands)
        torch.cuda.synchronize()
        e0.record()
        flop = 0.0
        for _ in range(5):
            flop += M.probe_mfma_bf16(iters, sink, random_operands=random_operands)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        # first wave of workgroup 0 of the last launch: core clocks and ticks of the constant-rate counter it ran for
        clocks, ticks = float(sink[1]), float(sink[2])
        return flop / (ms * 1e-3) / 1e12, ms, (clocks / (ticks / (ref_mhz * 1e6)) / 1e9 if ticks > 0 else None)

    tf_const, _, clock_const = rate(False)     # a few constant operand values: little toggling, the optimistic figure
    tf, ms, clock_ghz = rate(True)             # pseudo-random operands: what the chip sustains on real data
    # the prefill tile's instruction mix as synthetic in-order streams, in three arrangements (us per tile and CU)
    buf = torch.zeros(1 << 14, dtype=torch.float32, device="cuda")
    streams = {}
    for structure, name in enumerate(("phases_all_waves_alike", "phases_two_groups", "uniform_stream")):
        M.probe_tile_stream(structure, 500, buf)
        torch.cuda.synchronize()
        n_tiles = 4000
        e0.record()
        M.probe_tile_stream(structure, n_tiles, buf)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / n_tiles
        c, t = float(buf[1]), float(buf[2])
        streams[name] = dict(us_per_tile=us, clock_ghz=c / (t / (ref_mhz * 1e6)) / 1e9 if t > 0 else None,
                             matrix_tflops=256 * 8 * 32 * 32768 / (us * 1e-6) / 1e12)   # 256 CUs x 8 waves x 32 products of 32 x 32 x 16
    return dict(workload="mfma_only_bf16_32x32x16_random_operands", tflops=tf, frac_of_nominal=tf / MFMA_BF16_PEAK_TFLOPS, ms=ms / 5,
                clock_ghz=clock_ghz, tflops_constant_operands=tf_const, clock_ghz_constant_operands=clock_const,
                ref_counter_mhz=ref_mhz, tile_streams=streams,
                main=dict(value=tf, unit="TFLOP/s", ms=ms / 5, layout="registers only", metric="matrix-instruction-only rate"),
                roofline=dict(bound="mfma", achieved=tf, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s", frac=tf / MFMA_BF16_PEAK_TFLOPS,
                              traffic=None, kernel="mfma_rate", kernel_ms=ms / 5), cpu_baseline=None)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--only", default="", help="comma-separated records to run (default: all): " + " ".join(ALL))
    ap.add_argument("--config", type=int, default=0, help="shorthand for --only cfgN")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold-cache timings")
    ap.add_argument("--cpu-seconds", type=float, default=4.0, help="oracle time per attention record, about")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy three times (calibrates the FETCH_SIZE / WRITE_SIZE "
                         "counters of a rocprofv3 --pmc run of this same command)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2
    names = [n for n in (args.only.split(",") if args.only else ([f"cfg{args.config}"] if args.config else ALL)) if n]
    bad = [n for n in names if n not in ALL + ["commit_bf16_unaligned", "commit_fp8_unaligned"]]
    if bad:
        print(f"bench.py: unknown record(s) {bad}; known: {ALL}", file=sys.stderr)
        return 2

    import torch
    import paper_2512_16822_amd as M
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    M.load()
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    t_all = time.perf_counter()
    records = {}
    mfma = ref_mhz = None
    if "mfma_probe" in names or "cfg3" in names:
        records["mfma_probe"] = bench_mfma_probe(args)
        mfma = records["mfma_probe"]["tflops"]
        ref_mhz = records["mfma_probe"]["ref_counter_mhz"]
    for n in names:
        t0 = time.perf_counter()
        if n.startswith("cfg"):
            records[n] = bench_attention(int(n[3:]), args, mfma_measured=mfma, ref_mhz=ref_mhz)
        elif n.startswith("commit_"):
            records[n] = bench_commit(n[len("commit_"):], args)
        if n in records:
            records[n]["bench_wall_s"] = round(time.perf_counter() - t0, 2)
    first = records[names[0]]
    m = first.pop("main")
    for r in records.values():
        r.pop("main", None)
    line = dict(metric=m["metric"], value=m["value"], unit=m["unit"], n_gpus=1, steps=args.steps, warmup=args.warmup,
                ms_per_step=m["ms"], higher_is_better=True, scaling="weak", vs_baseline=None,
                dtype=first.get("dtype", "bf16"), data="synthetic",
                config={"workload": first["workload"], "layout": m["layout"],
                        **{k: first[k] for k in ("B", "Hq", "Hkv", "D", "P", "kv_len_mean", "kv_len_max", "n_q_tokens",
                                                 "algorithmic_bytes", "unique_kv_bytes", "useful_flops", "new_tokens") if k in first}},
                roofline=first["roofline"], cpu_baseline=first.get("cpu_baseline"),
                layouts=first.get("layouts"), accounting=first.get("accounting"),
                mfma_peak=dict(nominal_tflops=MFMA_BF16_PEAK_TFLOPS, measured_tflops=mfma, clock_ghz_measured=records["mfma_probe"]["clock_ghz"],
                               measured_tflops_constant_operands=records["mfma_probe"]["tflops_constant_operands"],
                               clock_ghz_constant_operands=records["mfma_probe"]["clock_ghz_constant_operands"]) if mfma else None,
                configs={k: v for k, v in records.items() if k != names[0]},
                bench_wall_s=round(time.perf_counter() - t_all, 1))
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
