#!/usr/bin/env python3
"""Benchmark of the fused-RoPE paged-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--layout both|shared|duplicated]

A step is one attention call of the library over the whole batch of the workload (gather through the
block tables, rotary embedding of K and Q on chip, online softmax, PV, split-K combine), with every
input already resident in HBM. Block tables come from the library's own aligner before the timed
region (the scheduling path runs once per request, not once per decode step); its cost is reported
separately. The default workload is the Llama-3-8B-shaped decode configuration of the benchmark spec.

Prints ONE JSON line. `value` is logical KV bytes per second on the page-sharing (MEPIC) layout;
`roofline` is measured on the same logical workload laid out with one page per logical block, where
every byte has to come from HBM (shared pages can be served from the caches).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# command (counter readings in KiB, each scaled by what the same counter reads for a 1 GiB device copy:
# FETCH_SIZE x2.000, WRITE_SIZE x1.000). Summaries with the commands are under profiles/.
MEASURED_TRAFFIC = {
    ("cfg2_llama3_8b_decode_bf16", "duplicated", "decode_mfma_bf16"): int((583510.4 * 2.0 + 5221.6) * 1024),
    ("cfg4_long_decode_bf16", "duplicated", "decode_mfma_bf16"): int((1112407.2 * 2.0 + 4236.3) * 1024),
    ("cfg5_mixed_decode_fp8", "duplicated", "decode_mfma_fp8"): int((1119965.7 * 2.0 + 9261.2) * 1024),
    ("cfg3_question_prefill_bf16", "shared", "prefill_mfma_bf16"): int((320040.3 * 2.0 + 32768.0) * 1024),
}


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
    """Run warmup + 2 x steps calls on torch's current stream. After the warmup, a pass of `steps` calls with
    events after every step and HIP events, handed to the library through timing_start / timing_stop, that
    bracket the main kernel of every call alone (on the stream the library launches on). Then the timed pass:
    the same `steps` calls with nothing between them, bracketed by two events and a synchronize on both sides
    (an event recorded between calls costs several microseconds of a 60-200 us step, so the pass that carries
    them is not the one that is timed).
    Returns (total ms of the timed pass, per-step ms and per-step main-kernel ms of the pass with events)."""
    import torch
    M = dc.M
    run = M.attn_prefill if dc.prefill else M.attn_decode
    if batched:
        run = lambda params: M.attn_decode_batched(params, dc.plan, dc.plan_info)
    for _ in range(warmup):
        run(dc.params)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    k0 = [M.HipEvent() for _ in range(steps)]
    k1 = [M.HipEvent() for _ in range(steps)]
    ev[0].record()
    for i in range(steps):
        dc.params.timing_start, dc.params.timing_stop = k0[i].handle, k1[i].handle
        run(dc.params)
        ev[i + 1].record()
    torch.cuda.synchronize()
    dc.params.timing_start = dc.params.timing_stop = None
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    kern = [k0[i].elapsed_ms(k1[i]) for i in range(steps)]
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0.record()
    for _ in range(steps):
        run(dc.params)
    t1.record()
    torch.cuda.synchronize()
    return t0.elapsed_time(t1), per, kern


def bench_commit(args) -> int:
    """`--commit`: the commit step alone (scatter of new un-rotated K/V into their pages) on the prompt-commit
    workload: 64 requests x 1024 new tokens of Llama-3-8B KV shape (Hkv 8, D 128), bf16 pages of 16 slots
    (`--commit fp8`: e4m3 pages of 32 slots). One JSON line, HBM roofline on source bytes read + page bytes
    written."""
    import numpy as np
    import torch
    import paper_2512_16822_amd as M
    import workloads as W
    M.load()
    fp8 = args.commit == "fp8"
    kv_dtype, P = ("f8e4m3", 32) if fp8 else ("bf16", 16)
    Hkv, D, B, T = 8, 128, 64, 1024
    MB = T // P + 1
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(10)
    pages = W.gen_pages(25, B * MB, Hkv, P, D, kv_dtype)
    bt = rng.permutation(B * MB).reshape(B, MB).astype(np.int32)
    i32 = lambda a: torch.tensor(np.asarray(a, dtype=np.int32), dtype=torch.int32, device=dev)
    src = lambda: torch.from_numpy(rng.standard_normal((B * T, Hkv, D)).astype(np.float32)).to(torch.bfloat16).to(dev)
    k_new, v_new = src(), src()
    k_dev, v_dev = pages.k.to(dev), pages.v.to(dev)
    ks = None if pages.k_scales is None else pages.k_scales.to(dev)
    vs = None if pages.v_scales is None else pages.v_scales.to(dev)
    p = M.make_commit_params(k_new, v_new, k_dev, v_dev, i32(bt), i32(np.arange(B)), i32([(b % 3) * 8 for b in range(B)]),
                             i32(np.arange(B + 1) * T), k_scales=ks, v_scales=vs)
    for _ in range(args.warmup):
        M.kv_commit(p)
    torch.cuda.synchronize()
    k0 = [M.HipEvent() for _ in range(args.steps)]
    k1 = [M.HipEvent() for _ in range(args.steps)]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        p.timing_start, p.timing_stop = k0[i].handle, k1[i].handle
        M.kv_commit(p)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    kern_ms = sum(a.elapsed_ms(b) for a, b in zip(k0, k1)) / args.steps
    n_el = 2 * B * T * Hkv * D
    abytes = n_el * 2 + n_el * (1 if fp8 else 2) + B * MB * 4 + (B * MB * 8 if fp8 else 0) + (3 * B + 1) * 4
    ach = abytes / (kern_ms * 1e-3) / 1e9
    print(json.dumps(dict(metric="KV commit throughput (source read + page write)", value=abytes / (ms * 1e-3) / 1e9,
                          unit="GB/s", n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms,
                          higher_is_better=True, scaling="weak", vs_baseline=None,
                          dtype="bf16 -> e4m3" if fp8 else "bf16", data="synthetic",
                          config=dict(workload=f"prompt_commit_64x1024_llama3_8b_{kv_dtype}", B=B, new_tokens=B * T,
                                      Hkv=Hkv, D=D, P=P, algorithmic_bytes=abytes),
                          roofline=dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                                        traffic=None, kernel="kv_commit", kernel_ms=kern_ms), cpu_baseline=None)))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=2, help="BASELINE.json config (1-based); default 2")
    ap.add_argument("--layout", default="both", choices=["both", "shared", "duplicated"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=0, help="oracle sample size in (token, head) rows")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 1 GiB device copy three times (calibrates the FETCH_SIZE / WRITE_SIZE "
                         "counters of a rocprofv3 --pmc run of this same command)")
    ap.add_argument("--commit", nargs="?", const="bf16", default=None, choices=["bf16", "fp8"],
                    help="benchmark the commit step (mepic_kv_commit) instead of attention")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    if args.commit:
        return bench_commit(args)

    import numpy as np
    import torch
    import paper_2512_16822_amd as M
    import workloads as W
    from paper_2512_16822_amd.device_case import DeviceCase, align_with_library

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    M.load()
    st = W.config(args.config)

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    # ---- scheduling path (host): align every request, report the accounting ----
    t0 = time.perf_counter()
    aligned, pool = align_with_library(M, st)
    align_s = time.perf_counter() - t0
    stats = pool.stats()
    case = W.assemble(st, aligned, poison=False)
    prefill = st.mode == "prefill"

    results = {}
    layouts = ["shared", "duplicated"] if args.layout == "both" else [args.layout]
    for layout in layouts:
        c = case if layout == "shared" else W.to_duplicated(case)
        # one page per logical block: no page is shared, which the caller tells the library (MEPIC_FLAG_KV_READ_ONCE)
        dc = DeviceCase(M, c, flags=0 if layout == "shared" else M.FLAG_KV_READ_ONCE)
        total_ms, per, kern = time_steps(dc, args.steps, args.warmup)
        results[layout] = dict(ms=total_ms / args.steps, min_ms=min(per), kernel=M.last_kernel(),
                               kernel_ms=sum(kern) / len(kern), ms_instr=sum(per) / len(per),
                               pages=c.pages.num_pages, out=dc.out.float().cpu())
        if layout == "shared" and not prefill and M.last_kernel().startswith("decode_mfma"):
            # the same job with one pass over shared pages for several requests (plan built on the host)
            info = dc.prepare_batched()
            plan_s = 1e9
            for _ in range(3):   # the host planner alone (the upload and the workspace are not part of it)
                t0 = time.perf_counter()
                M.decode_plan_build(c.block_tables, c.kv_lens, st.P, st.Hq, st.Hkv,
                                    M.F8E4M3 if st.kv_dtype == "f8e4m3" else M.BF16)
                plan_s = min(plan_s, time.perf_counter() - t0)
            total_ms, per, kern = time_steps(dc, args.steps, args.warmup, batched=True)
            results["shared_batched"] = dict(ms=total_ms / args.steps, min_ms=min(per), kernel=M.last_kernel(),
                                             kernel_ms=sum(kern) / len(kern), ms_instr=sum(per) / len(per),
                                             pages=c.pages.num_pages,
                                             out=dc.out.float().cpu(), plan=info.as_dict(), plan_build_ms=plan_s * 1e3)
        del dc
        torch.cuda.empty_cache()
    if "shared_batched" in results:
        diff = (results["shared_batched"]["out"] - results["shared"]["out"]).abs().max().item()
        assert diff <= 4e-2, f"batched and plain decode disagree by {diff}"
    if len(layouts) == 2:
        assert torch.equal(results["shared"]["out"], results["duplicated"]["out"]), "layouts disagree"

    abytes = algorithmic_bytes(case)
    flops = 4 * st.D * visible_pairs(case) * st.Hq
    main_layout = "shared" if "shared" in results else layouts[0]
    roof_layout = "duplicated" if "duplicated" in results else layouts[0]
    ms = results[main_layout]["ms"]
    if prefill:
        value, unit, metric = flops / (ms * 1e-3) / 1e12, "TFLOP/s", "fused-RoPE paged prefill attention throughput"
        roof_layout = main_layout          # bound by the matrix cores: where the pages come from does not matter
        rms = results[roof_layout]["kernel_ms"]
        ach = flops / (rms * 1e-3) / 1e12
        traffic = MEASURED_TRAFFIC.get((st.name, roof_layout, results[roof_layout]["kernel"]))
        roofline = dict(bound="mfma", achieved=ach, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=ach / MFMA_BF16_PEAK_TFLOPS, traffic=traffic, layout=roof_layout,
                        kernel=results[roof_layout]["kernel"], kernel_ms=rms, call_ms=results[roof_layout]["ms"])
    else:
        value, unit, metric = abytes / (ms * 1e-3) / 1e9, "GB/s", "fused-RoPE paged decode attention KV throughput"
        rms = results[roof_layout]["kernel_ms"]
        ach = abytes / (rms * 1e-3) / 1e9
        traffic = MEASURED_TRAFFIC.get((st.name, roof_layout, results[roof_layout]["kernel"]))
        roofline = dict(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                        traffic=traffic, layout=roof_layout, kernel=results[roof_layout]["kernel"], kernel_ms=rms,
                        call_ms=results[roof_layout]["ms"])

    # ---- the oracle on this machine's host cores, on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import attn as oracle_attn
        from oracle import align as oracle_align
        from harness import oracle_out
        opool = oracle_align.PoolOracle(1 << 20, st.P)
        o_aligned = [opool.align(segs, st.extra_tail) for segs in st.requests]
        assert all(a["block_table"] == b["block_table"].tolist() for a, b in zip(o_aligned, aligned))
        n_rows_total = case.n_q * st.Hq
        # 10-20 CPU-seconds of oracle work: ~0.15 us per (row, key) at D = 128 on the 16 host cores of a GPU machine
        n_rows = args.cpu_rows or max(8, min(n_rows_total, int(1.0e8 / max(1, int(case.kv_lens.mean())))))
        if n_rows >= n_rows_total:                    # the whole job is within the budget: no sampling
            rows = [(t, h) for t in range(case.n_q) for h in range(st.Hq)]
        else:
            rng = np.random.default_rng(0)
            rows = sorted({(int(rng.integers(case.n_q)), int(rng.integers(st.Hq))) for _ in range(n_rows)})
        t0 = time.perf_counter()
        want = oracle_out(oracle_attn, case, rows=rows)
        cpu_s = time.perf_counter() - t0
        got = results[main_layout]["out"].double().numpy()
        err = float(np.abs(np.stack([got[t, h] for t, h in rows]) - want).max())
        scale = n_rows_total / len(rows)
        whole = cpu_s * scale
        cpu = dict(value=(flops / whole / 1e12) if prefill else (abytes / whole / 1e9), unit=unit,
                   cores=oracle_attn.num_threads(), kind="oracle",
                   sample=f"{len(rows)} of {n_rows_total} (query token, head) rows in {cpu_s:.2f} s, scaled to the whole job",
                   max_abs_err_of_gpu_on_sample=err)

    line = dict(metric=metric, value=value, unit=unit, n_gpus=1, steps=args.steps, warmup=args.warmup,
                ms_per_step=ms, higher_is_better=True, scaling="weak", vs_baseline=None,
                dtype={"f32": "f32", "bf16": "bf16", "f8e4m3": "bf16 (fp8 e4m3 KV)"}[st.kv_dtype],
                data="synthetic",
                config=dict(workload=st.name, layout=main_layout, B=st.B, Hq=st.Hq, Hkv=st.Hkv, D=st.D, P=st.P,
                            kv_len_mean=float(case.kv_lens.mean()), kv_len_max=int(case.kv_lens.max()),
                            n_q_tokens=case.n_q, algorithmic_bytes=abytes, useful_flops=flops),
                roofline=roofline, cpu_baseline=cpu,
                layouts={k: dict(ms_per_step=v["ms"], ms_per_step_with_events=v["ms_instr"], min_ms=v["min_ms"],
                                 kernel_ms=v["kernel_ms"], pages=v["pages"],
                                 kernel=v["kernel"], gbs=abytes / (v["ms"] * 1e-3) / 1e9,
                                 **({"plan": v["plan"], "plan_build_ms": v["plan_build_ms"]} if "plan" in v else {}))
                         for k, v in results.items()},
                accounting=dict(pages_unique=stats["pages_in_use_unique"],
                                pages_duplicated=stats["pages_logical_duplicated"],
                                ratio=stats["pages_logical_duplicated"] / max(1, stats["pages_in_use_unique"]),
                                aligner_us_per_request=align_s / max(1, st.B) * 1e6))
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
