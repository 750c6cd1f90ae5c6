"""The host planner of the batched decode (mepic_decode_plan_build): structural properties of the plan on seeded
workloads. No GPU needed; the numerical result of the batched kernel is checked against the attention oracle in
the GPU tests."""
import numpy as np
import pytest

import workloads as W
from harness import align_with_oracle

HEADER, MAXR = 8, 16
RUN_WORDS = 1 + 3 * MAXR


def parse(plan, info):
    n, B = info.n_runs, info.B
    assert plan[0] == 0x4D455049 and plan[1] == n and plan[5] == B
    cum = plan[HEADER: HEADER + n + 1]
    runs = plan[HEADER + n + 1: HEADER + n + 1 + n * RUN_WORDS].reshape(n, RUN_WORDS)
    n_part = plan[HEADER + n + 1 + n * RUN_WORDS:]
    assert n_part.size == B
    return cum, runs, n_part


def check_plan(M, bt, kv_lens, P, Hq, Hkv, kv_dtype):
    plan, info = M.decode_plan_build(bt, kv_lens, P, Hq, Hkv, kv_dtype)
    cum, runs, n_part = parse(plan, info)
    bps, G = 32 // P, Hq // Hkv
    B = bt.shape[0]
    nst = [(-(-int(L) // P) + bps - 1) // bps for L in kv_lens]
    assert info.steps_unbatched == sum(nst) and info.r_cap == 16 // G
    seen = [np.zeros(n, dtype=np.int32) for n in nst]
    used = [0] * B
    pos = 0
    for i, w in enumerate(runs):
        R = int(w[0])
        req, step0, slot = w[1:1 + R], w[1 + MAXR:1 + MAXR + R], w[1 + 2 * MAXR:1 + 2 * MAXR + R]
        n = int(cum[i + 1] - cum[i])
        assert cum[i] == pos and n >= 1 and 1 <= R <= info.r_cap and len(set(req.tolist())) == R
        pieces = (pos + n - 1) // info.chunk - pos // info.chunk + 1
        for k in range(R):
            b, s0 = int(req[k]), int(step0[k])
            seen[b][s0:s0 + n] += 1
            assert slot[k] == used[b]                       # slots of a request are handed out in run order
            used[b] += pieces
        for j in range(n):                                  # identical pages, and whole steps when shared
            tuples = {tuple(bt[int(req[k]), (int(step0[k]) + j) * bps:(int(step0[k]) + j + 1) * bps].tolist()) for k in range(R)}
            assert len(tuples) == 1
            if R > 1:
                assert all((int(step0[k]) + j + 1) * 32 <= int(kv_lens[int(req[k])]) for k in range(R))
        pos += n
    assert pos == info.total_steps == cum[-1]
    assert all((s == 1).all() for s in seen), "every (request, step) exactly once"
    assert used == n_part.tolist() and info.n_splits == max(1, max(used, default=1))
    return info


@pytest.mark.parametrize("cfg", [2, 5])
def test_plan_of_baseline_decode_configs(mepic, cfg):
    st = W.config(cfg)
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned, poison=False)
    info = check_plan(mepic, case.block_tables, case.kv_lens, st.P, st.Hq, st.Hkv,
                      mepic.F8E4M3 if st.kv_dtype == "f8e4m3" else mepic.BF16)
    ratio = info.steps_unbatched / info.total_steps
    assert ratio > (2.5 if cfg == 2 else 1.6), ratio          # shared chunk pages are walked once per group


def test_plan_edge_cases(mepic):
    rng = np.random.default_rng(5)
    # identical block tables with different lengths, empty requests, a page repeated inside one request
    bt = np.tile(np.arange(12, dtype=np.int32), (5, 1))
    bt[4, 6:8] = bt[4, 2:4]
    kv = np.array([192, 170, 0, 33, 192], dtype=np.int32)
    info = check_plan(mepic, bt, kv, 16, 8, 2, mepic.BF16)
    assert info.total_steps < info.steps_unbatched
    # nothing shared: one run per request
    bt = rng.permutation(40).reshape(4, 10).astype(np.int32)
    info = check_plan(mepic, bt, np.array([160, 1, 159, 320], dtype=np.int32), 32, 14, 2, mepic.F8E4M3)
    assert info.n_runs == 4 and info.total_steps == info.steps_unbatched
    # group size 16: one request per run even when everything is shared
    bt = np.tile(np.arange(6, dtype=np.int32), (3, 1))
    info = check_plan(mepic, bt, np.array([96, 96, 96], dtype=np.int32), 16, 16, 1, mepic.BF16)
    assert info.r_cap == 1 and info.total_steps == info.steps_unbatched
    with pytest.raises(mepic.MepicError):
        mepic.decode_plan_build(bt, np.array([96, 97, 96], dtype=np.int32), 16, 16, 1, mepic.BF16)   # kv_len beyond the table
    with pytest.raises(mepic.MepicError):
        mepic.decode_plan_build(bt, np.array([96, 96, 96], dtype=np.int32), 32, 16, 1, mepic.BF16)   # bf16 needs P = 16
