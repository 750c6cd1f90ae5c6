"""The host planner of the batched decode (mepic_decode_plan_build): structural properties of the plan on seeded
workloads. No GPU needed; the numerical result of the batched kernel is checked against the attention oracle in
the GPU tests."""
import numpy as np
import pytest

import workloads as W
from harness import align_with_oracle

HEADER, MAXR = 8, 16
RUN_WORDS = 2 + 3 * MAXR


GATHER_WORDS, GATHER_MAX, GATHER_BELOW = 3, 64, 4


def parse(plan, info):
    n, B, n_gather = info.n_runs, info.B, int(plan[7])
    assert plan[0] == 0x4D455049 and plan[1] == n and plan[5] == B
    cum = plan[HEADER: HEADER + n + 1]
    runs = plan[HEADER + n + 1: HEADER + n + 1 + n * RUN_WORDS].reshape(n, RUN_WORDS)
    off = HEADER + n + 1 + n * RUN_WORDS
    n_part = plan[off: off + B]
    gather = plan[off + B:]
    cuts = plan[off + B + n_gather * GATHER_WORDS:]
    gather = plan[off + B: off + B + n_gather * GATHER_WORDS]
    assert cuts.size == info.n_waves + 1 == plan[3] + 1 and plan.size == info.n_int32
    return cum, runs, n_part, gather.reshape(n_gather, GATHER_WORDS), cuts


def check_plan(M, bt, kv_lens, P, Hq, Hkv, kv_dtype, horizon=0):
    plan, info = M.decode_plan_build(bt, kv_lens, P, Hq, Hkv, kv_dtype, horizon_tokens=horizon)
    planned = [min(int(L) + horizon, bt.shape[1] * P) for L in kv_lens]      # lengths the plan reaches
    cum, runs, n_part, gather, cuts = parse(plan, info)
    listed = 0
    # the waves' ranges tile the sequence of steps; wave_of(p) = the wave whose range holds position p
    assert cuts[0] == 0 and cuts[-1] == info.total_steps and (np.diff(cuts) >= 0).all()
    wave_of = lambda p: int(np.searchsorted(cuts, p, side="right")) - 1
    # cut by estimated time, not by count, but no wave gets more than twice its even share of steps
    assert int(np.diff(cuts).max(initial=0)) <= 2 * -(-info.total_steps // info.n_waves) + 2
    bps, G = 32 // P, Hq // Hkv
    B = bt.shape[0]
    nst = [(-(-int(L) // P) + bps - 1) // bps for L in planned]
    assert info.steps_unbatched == sum(nst) and info.r_cap == 16 // G
    seen = [np.zeros(n, dtype=np.int32) for n in nst]
    used = [0] * B
    pos = 0
    chain_base, chain_head_wave = None, None
    for i, w in enumerate(runs):
        R, cont, is_gather = int(w[0]) & 0xFF, bool(int(w[0]) & 0x100), bool(int(w[0]) & 0x200)
        req, step0, slot = w[1:1 + R], w[1 + MAXR:1 + MAXR + R], w[1 + 2 * MAXR:1 + 2 * MAXR + R]
        n = int(cum[i + 1] - cum[i])
        assert cum[i] == pos and n >= 1 and 1 <= R <= info.r_cap and len(set(req.tolist())) == R
        if cont:                                            # continues the previous one-request run of the same request
            prev = runs[i - 1]
            assert R == 1 and (int(prev[0]) & 0xFF) == 1 and prev[1] == req[0]
        else:                                               # head of a chain: its slots cover every wave the chain touches
            j, length = i + 1, n
            while j < len(runs) and int(runs[j][0]) & 0x100:
                length += int(cum[j + 1] - cum[j])
                j += 1
            pieces = wave_of(pos + length - 1) - wave_of(pos) + 1
            chain_base = [used[int(b)] for b in req]
            chain_head_wave = wave_of(pos)
            for b in req:
                used[int(b)] += pieces
        for k in range(R):
            assert slot[k] == chain_base[k] - chain_head_wave       # the kernel adds its wave index
        if is_gather:                                       # one request; listed steps, ascending, with their pages
            b, L = int(req[0]), planned[int(req[0])]
            assert R == 1 and n <= GATHER_MAX and step0[0] == listed
            entries = gather[listed:listed + n]
            listed += n
            assert (np.diff(entries[:, 0]) > 0).all()
            for st, p0, p1 in entries.tolist():
                seen[b][st] += 1
                assert p0 == bt[b, st * bps]
                second = bps == 2 and st * bps + 1 < -(-L // P)
                assert p1 == (bt[b, st * bps + 1] if second else p0)
            pos += n
            continue
        if R == 1:                                          # short one-request runs were gathered
            assert n >= GATHER_BELOW
        if horizon:                                         # planned ahead: only gather runs hold steps that reach past kv_len
            assert all((int(step0[k]) + n) * 32 <= int(kv_lens[int(req[k])]) for k in range(R))
        for k in range(R):
            b, s0 = int(req[k]), int(step0[k])
            seen[b][s0:s0 + n] += 1
        for j in range(n):                                  # identical pages, and whole steps when shared
            tuples = {tuple(bt[int(req[k]), (int(step0[k]) + j) * bps:(int(step0[k]) + j + 1) * bps].tolist()) for k in range(R)}
            assert len(tuples) == 1
            if R > 1:
                assert all((int(step0[k]) + j + 1) * 32 <= int(kv_lens[int(req[k])]) for k in range(R))
        pos += n
    assert pos == info.total_steps == cum[-1] and listed == len(gather)
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


@pytest.mark.parametrize("horizon", [1, 32, 100])
def test_plan_built_ahead(mepic, horizon):
    """Planned for growth: the steps a request reaches within `horizon` tokens are covered, each exactly once, and
    sit in gather runs (whose steps are masked one by one against the kv_len of the call)."""
    st = W.decode_structure("ahead", 71, B=9, Hq=8, Hkv=2, D=128, P=16, theta=5e5, q_dtype="bf16", kv_dtype="bf16",
                            prefix=40, n_chunks=(1, 5), chunk_tokens=300, pool=3, question=45)
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned, poison=False)
    bt = np.concatenate([case.block_tables, np.full((st.B, 8), 7, dtype=np.int32)], axis=1)   # room to grow: 128 slots
    info0 = check_plan(mepic, bt, case.kv_lens, st.P, st.Hq, st.Hkv, mepic.BF16)
    info = check_plan(mepic, bt, case.kv_lens, st.P, st.Hq, st.Hkv, mepic.BF16, horizon=horizon)
    extra = sum(-(-(int(L) + horizon) // 32) - -(-int(L) // 32) for L in case.kv_lens)
    assert info.steps_unbatched == info0.steps_unbatched + extra
    # the table bounds the plan: no room, no steps ahead
    info = check_plan(mepic, case.block_tables, case.kv_lens, st.P, st.Hq, st.Hkv, mepic.BF16, horizon=1000)
    with pytest.raises(mepic.MepicError):
        mepic.decode_plan_build(bt, case.kv_lens, st.P, st.Hq, st.Hkv, mepic.BF16, horizon_tokens=-1)


def test_plan_edge_cases(mepic):
    rng = np.random.default_rng(5)
    # identical block tables with different lengths, empty requests, a page repeated inside one request
    bt = np.tile(np.arange(12, dtype=np.int32), (5, 1))
    bt[4, 6:8] = bt[4, 2:4]
    kv = np.array([192, 170, 0, 33, 192], dtype=np.int32)
    info = check_plan(mepic, bt, kv, 16, 8, 2, mepic.BF16)
    assert info.total_steps < info.steps_unbatched
    # alternating shared / own steps: more loose steps per request than one gather run holds
    bt = np.arange(2 * 300, dtype=np.int32).reshape(2, 300)
    bt[1, 0::4] = bt[0, 0::4]
    bt[1, 1::4] = bt[0, 1::4]                                 # steps 0, 2, 4, .. (two pages each) coincide
    plan, info = mepic.decode_plan_build(bt, np.array([4800, 4790], dtype=np.int32), 16, 8, 2, mepic.BF16)
    _, runs, _, gather, _ = parse(plan, info)
    n_gather_runs = sum(1 for w in runs if int(w[0]) & 0x200)
    assert len(gather) == 150 and n_gather_runs == 4          # 75 loose steps per request: 64 + 11
    check_plan(mepic, bt, np.array([4800, 4790], dtype=np.int32), 16, 8, 2, mepic.BF16)
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
