"""Page-accounting sweep with the library's aligner only (no GPU): how many KV pages a page-sharing pool
holds at peak versus a pool in which every request owns all of its blocks, as the number of chunks per
prompt and the load grow. This mirrors the shape of the paper's context-length study (§4.4: 2 to 16 chunks
per prompt at fixed QPS) and load study (§4.3: QPS sweep) on synthetic traffic; it reproduces none of the
paper's datasets or numbers.

    python -m paper_2512_16822_amd.accounting_sweep [--requests 200] [--seed 0]

Traffic: requests arrive as a Poisson process of the given rate, each holds its pages for a service time
proportional to its length, then is released. A request = 64-token private prefix + n chunks of 512 tokens
drawn Zipf(1.1) with replacement from a pool of 64 chunks + 128-token private question. Page size 16.
The pool is large enough that nothing is evicted or rejected; zero-reference chunks stay resident (they are
what the next request reuses), so `unique` counts them.
"""
from __future__ import annotations

import argparse
import heapq
from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np

PROMPT, CHUNK = 0, 1
P = 16


def make_trace(n_requests: int, n_chunks: int, qps: float, seed: int, pool_chunks: int = 64,
               chunk_tokens: int = 512, zipf_s: float = 1.1) -> List[Tuple[float, float, List[Tuple[int, int, int]]]]:
    """(arrival time, departure time, segments) per request, seeded."""
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, n_chunks, int(qps * 1000)])))
    w = np.arange(1, pool_chunks + 1, dtype=np.float64) ** (-zipf_s)
    cdf = np.cumsum(w / w.sum())
    t = 0.0
    out = []
    for _ in range(n_requests):
        t += float(rng.exponential(1.0 / qps))
        keys = np.minimum(np.searchsorted(cdf, rng.random(n_chunks), side="right"), pool_chunks - 1)
        segs = [(PROMPT, 64, 0)] + [(CHUNK, chunk_tokens, 0xC0DE0000 + int(k)) for k in keys] + [(PROMPT, 128, 0)]
        tokens = 64 + n_chunks * chunk_tokens + 128
        service = 0.5 + tokens / 4000.0          # seconds a request keeps its KV
        out.append((t, t + service, segs))
    return out


def replay(trace, align: Callable, release: Callable, stats: Callable) -> Dict[str, int]:
    """Replay a trace through an aligner (the library's or any object with the same three calls)."""
    live: List[Tuple[float, int]] = []
    for arrive, depart, segs in trace:
        while live and live[0][0] <= arrive:
            release(heapq.heappop(live)[1])
        heapq.heappush(live, (depart, align(segs)))
    s = stats()
    while live:
        release(heapq.heappop(live)[1])
    return dict(peak_unique=s["peak_pages_in_use_unique"], peak_duplicated=s["peak_pages_logical_duplicated"])


def run_library(trace, num_pages: int = 1 << 20) -> Dict[str, int]:
    from . import Pool
    pool = Pool(num_pages, P)
    return replay(trace, lambda segs: pool.align_request(segs, 1)["handle"], pool.release_request, pool.stats)


def sweep(n_requests: int, seed: int):
    rows = []
    for n_chunks in (2, 4, 8, 12, 16):
        r = run_library(make_trace(n_requests, n_chunks, 15.0, seed))
        rows.append(("chunks", n_chunks, 15.0, r["peak_unique"], r["peak_duplicated"]))
    for qps in (2.0, 5.0, 10.0, 15.0, 25.0):
        r = run_library(make_trace(n_requests, 8, qps, seed))
        rows.append(("qps", 8, qps, r["peak_unique"], r["peak_duplicated"]))
    return rows


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=200)
    ap.add_argument("--seed", type=int, default=0)
    a = ap.parse_args()
    print("| sweep | chunks/prompt | QPS | peak pages, sharing pool | peak pages, every request owns its blocks | ratio |")
    print("|---|---|---|---|---|---|")
    for kind, n_chunks, qps, u, d in sweep(a.requests, a.seed):
        print(f"| {kind} | {n_chunks} | {qps:g} | {u} | {d} | {d / u:.2f}x |")


if __name__ == "__main__":
    main()
