"""GPU parity of mepic_attn_decode_batched (one pass over shared pages for several requests) against the fp64
attention oracle, and against the plain decode call."""
import numpy as np
import pytest
import torch

import workloads as W
from harness import DeviceCase, align_with_oracle, oracle_out

pytestmark = pytest.mark.gpu
TOL = 2e-2


def check_batched(M, oracle_attn, case, rows=None):
    dc = DeviceCase(M, case)
    info = dc.prepare_batched()
    got = dc.run_batched()
    name = M.last_kernel()
    assert name == ("decode_mfma_fp8_batched" if case.st.kv_dtype == "f8e4m3" else "decode_mfma_bf16_batched")
    plain = dc.run()
    want = oracle_out(oracle_attn, case, rows=rows)
    sel = (lambda x: np.stack([x[t, h] for t, h in rows])) if rows is not None else (lambda x: x)
    assert np.isfinite(got).all()
    err = np.abs(sel(got) - want).max()
    assert err <= TOL, f"max abs err {err:.3e} ({name})"
    assert np.abs(got - plain).max() <= 2 * TOL           # the two library paths agree as well
    return info


@pytest.mark.parametrize("kv_dtype,P", [("bf16", 16), ("f8e4m3", 32)])
@pytest.mark.parametrize("G", [1, 2, 4, 7, 8, 16])
def test_shared_chunks_all_group_sizes(mepic, oracle_attn, kv_dtype, P, G):
    st = W.decode_structure(f"batched_{kv_dtype}_{G}", 90 + G, B=11, Hq=2 * G, Hkv=2, D=128, P=P, theta=5e5, q_dtype="bf16",
                            kv_dtype=kv_dtype, prefix=40, n_chunks=(1, 5), chunk_tokens=300, pool=3, question=45)
    aligned, _ = align_with_oracle(st)
    info = check_batched(mepic, oracle_attn, W.assemble(st, aligned))
    if G <= 8:
        assert info.total_steps < info.steps_unbatched     # something was actually batched


def test_identical_tables_different_lengths_and_empty_requests(mepic, oracle_attn):
    """All requests alias the same pages from slot 0 (a shared prompt), with different kv_len: whole steps are
    batched, each request's ragged last step is not."""
    st = W.decode_structure("same_prompt", 91, B=9, Hq=8, Hkv=2, D=128, P=16, theta=1e4, q_dtype="bf16", kv_dtype="bf16",
                            prefix=700, n_chunks=0, chunk_tokens=16, pool=1, question=0)
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned)
    case.block_tables[:] = case.block_tables[0]
    case.kv_lens[:] = np.array([701, 640, 33, 0, 1, 512, 700, 31, 96], dtype=np.int32)
    case.q_positions[:] = np.maximum(case.kv_lens - 1, 0)
    info = check_batched(mepic, oracle_attn, case)
    assert info.total_steps < info.steps_unbatched


@pytest.mark.parametrize("kv_dtype,P", [("bf16", 16), ("f8e4m3", 32)])
def test_many_scattered_unshared_steps(mepic, oracle_attn, kv_dtype, P):
    """Every other step of three long requests aliases the first request's pages, the steps in between are their
    own: each request has more unshared one-step stretches than one gather run holds, and its shared steps never
    form runs longer than one step."""
    st = W.decode_structure(f"scattered_{kv_dtype}", 95, B=4, Hq=8, Hkv=2, D=128, P=P, theta=5e5, q_dtype="bf16",
                            kv_dtype=kv_dtype, prefix=4700, n_chunks=0, chunk_tokens=16, pool=1, question=0)
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned)
    bps = 32 // P
    for b in range(1, 4):
        for step in range(b, 140, 2):                     # from a different first step per request
            case.block_tables[b, step * bps:(step + 1) * bps] = case.block_tables[0, step * bps:(step + 1) * bps]
    info = check_batched(mepic, oracle_attn, case)
    assert info.total_steps < info.steps_unbatched


@pytest.mark.parametrize("seed", range(12))
def test_random_structures(mepic, oracle_attn, seed):
    rng = np.random.default_rng(3000 + seed)
    fp8 = bool(seed & 1)
    G, Hkv = int(rng.choice([1, 2, 4, 7])), int(rng.choice([1, 2, 4]))
    st = W.decode_structure(f"rand_batched_{seed}", 700 + seed, B=int(rng.integers(2, 50)), Hq=G * Hkv, Hkv=Hkv, D=128,
                            P=32 if fp8 else 16, theta=5e5, q_dtype="bf16", kv_dtype="f8e4m3" if fp8 else "bf16",
                            prefix=int(rng.integers(0, 100)), n_chunks=(0, int(rng.integers(1, 7))),
                            chunk_tokens=int(rng.integers(33, 600)), pool=int(rng.integers(1, 4)),
                            question=int(rng.integers(0, 120)))
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned)
    n_rows = case.n_q * st.Hq
    rows = None
    if n_rows > 256:
        r = np.random.default_rng(seed)
        rows = sorted({(int(r.integers(case.n_q)), int(r.integers(st.Hq))) for _ in range(256)})
    check_batched(mepic, oracle_attn, case, rows=rows)


@pytest.mark.parametrize("kv_dtype,P,G", [("bf16", 16, 4), ("f8e4m3", 32, 7), ("bf16", 16, 1)])
def test_plan_built_ahead_serves_later_decode_steps(mepic, oracle_attn, kv_dtype, P, G):
    """One plan built with a horizon of 40 tokens, then decode calls at kv_len + 0, 1, 17, 31, 32, 40 with the
    device-side kv_lens and query positions of each step: every call against the oracle. The pages of the slots
    ahead exist (the requests were aligned with that many tail tokens); what lies past the kv_len of a call is
    poisoned with NaN for that call."""
    H = 40
    st = W.decode_structure(f"ahead_{kv_dtype}", 73 + G, B=10, Hq=2 * G, Hkv=2, D=128, P=P, theta=5e5, q_dtype="bf16",
                            kv_dtype=kv_dtype, prefix=40, n_chunks=(1, 5), chunk_tokens=300, pool=3, question=45)
    st.extra_tail = 1 + H                                       # the decode token and the H after it
    aligned, _ = align_with_oracle(st)
    full = W.assemble(st, aligned, poison=False)                # values for every slot up to the horizon
    L0 = full.kv_lens - H
    fmt = mepic.F8E4M3 if kv_dtype == "f8e4m3" else mepic.BF16
    plan, info = mepic.decode_plan_build(full.block_tables, L0, P, st.Hq, st.Hkv, fmt, horizon_tokens=H)
    for k in (0, 1, 17, 31, 32, 40):
        case = W.Case(st, full.block_tables, full.n_blocks, (L0 + k).astype(np.int32), (L0 + k - 1).astype(np.int32),
                      None, W.gen_pages(st.seed, full.pages.num_pages, st.Hkv, P, st.D, kv_dtype), full.q)
        W.poison_tail(case.pages, case.block_tables, case.kv_lens)
        for b in range(st.B):                                   # whole blocks past kv_len as well
            for j in range(-(-int(case.kv_lens[b]) // P), int(case.n_blocks[b])):
                page = int(case.block_tables[b, j])
                if kv_dtype == "f8e4m3":
                    case.pages.k.view(torch.uint8)[page] = 0x7F
                    case.pages.v.view(torch.uint8)[page] = 0x7F
                    case.pages.k_scales[page] = float("nan")
                    case.pages.v_scales[page] = float("nan")
                else:
                    case.pages.k[page] = float("nan")
                    case.pages.v[page] = float("nan")
        dc = DeviceCase(mepic, case)
        dc.plan_info, dc.plan = info, torch.from_numpy(plan).to(dc.q.device)
        nbytes = mepic.attn_decode_batched_workspace_size(dc.params, info)
        dc.ws = torch.empty(max(nbytes, dc.ws.numel()), dtype=torch.uint8, device=dc.q.device)
        dc.params.workspace, dc.params.workspace_bytes = dc.ws.data_ptr(), dc.ws.numel()
        got = dc.run_batched()
        want = oracle_out(oracle_attn, case)
        assert np.isfinite(got).all(), k
        err = np.abs(got - want).max()
        assert err <= TOL, (k, err)


@pytest.mark.parametrize("cfg,n_rows", [(2, 2048), (4, 256), (5, 512)])
def test_full_size_configs_sampled(mepic, oracle_attn, cfg, n_rows):
    st = W.config(cfg)
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned)
    rows = None                                   # configs 2 and 4: every (request, head) row
    if n_rows < case.n_q * st.Hq:
        r = np.random.default_rng(cfg)
        rows = sorted({(int(r.integers(case.n_q)), int(r.integers(st.Hq))) for _ in range(n_rows)})
    info = check_batched(mepic, oracle_attn, case, rows=rows)
    assert info.steps_unbatched / info.total_steps > (2.5 if cfg == 2 else 1.6)


def test_long_runs_cross_several_page_id_windows(mepic, oracle_attn):
    """Three unshared requests of 46 001 slots with 32 KV heads (few waves per head): each request is one run of
    1438 steps, and a wave's piece of it spans more blocks than the two windows of page ids it starts with."""
    st = W.decode_structure("long_unshared", 96, B=3, Hq=32, Hkv=32, D=128, P=16, theta=5e5, q_dtype="bf16",
                            kv_dtype="bf16", prefix=46000, n_chunks=0, chunk_tokens=16, pool=1, question=0)
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned)
    r = np.random.default_rng(44)
    rows = sorted({(int(r.integers(case.n_q)), int(r.integers(st.Hq))) for _ in range(12)})
    info = check_batched(mepic, oracle_attn, case, rows=rows)
    assert info.n_runs == st.B and info.total_steps == info.steps_unbatched
    assert info.total_steps // info.n_waves > 64            # more than 128 blocks per piece
