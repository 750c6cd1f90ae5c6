"""Accounting sweep (page counts only, no GPU): the library's pool against the oracle pool on seeded arrival
traces, bit-exact peaks, plus the properties the paper's context-length study rests on (§4.4)."""
import pytest

from oracle import align as OA
from paper_2512_16822_amd import accounting_sweep as S


def run_oracle(trace):
    pool = OA.PoolOracle(1 << 20, S.P)
    return S.replay(trace, lambda segs: pool.align(segs, 1)["handle"], pool.release, pool.stats)


@pytest.mark.parametrize("n_chunks,qps", [(2, 15.0), (8, 5.0), (16, 15.0), (8, 25.0)])
def test_library_and_oracle_agree_on_traces(n_chunks, qps):
    trace = S.make_trace(120, n_chunks, qps, seed=3)
    assert S.run_library(trace) == run_oracle(trace)


def test_sharing_saves_more_for_longer_prompts_and_higher_load():
    by_chunks = [S.run_library(S.make_trace(150, n, 15.0, seed=1)) for n in (2, 8, 16)]
    ratios = [r["peak_duplicated"] / r["peak_unique"] for r in by_chunks]
    assert ratios[0] < ratios[1] < ratios[2] and ratios[2] > 4.0      # more reusable chunks -> larger saving
    by_qps = [S.run_library(S.make_trace(150, 8, q, seed=1)) for q in (2.0, 25.0)]
    r_lo, r_hi = (r["peak_duplicated"] / r["peak_unique"] for r in by_qps)
    assert r_hi > r_lo                                                  # more concurrent requests -> more aliasing
    # the sharing pool can never hold more than the duplicated one plus the resident zero-reference chunks
    for r in by_chunks + by_qps:
        assert r["peak_unique"] <= r["peak_duplicated"] + 64 * 31
