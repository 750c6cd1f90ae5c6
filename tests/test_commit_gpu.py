"""GPU parity of mepic_kv_commit (§3.3.2) against oracle/commit.py: page bytes must be identical, including
every byte the call must not touch."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import commit as OC

pytestmark = pytest.mark.gpu

_VIEW = {"f32": torch.float32, "bf16": torch.uint16, "f8e4m3": torch.uint8}
_SRC = {"f32": torch.float32, "bf16": torch.bfloat16, "f8e4m3": torch.bfloat16}


def _src(rng, n, Hkv, D, kv_dtype, amp=1.5):
    x = torch.from_numpy(rng.standard_normal((n, Hkv, D)).astype(np.float32) * amp)
    return x.to(_SRC[kv_dtype])


def _raw_src(t):
    return t.numpy() if t.dtype == torch.float32 else t.view(torch.uint16).numpy()


def run_both(M, pages, bt, runs, k_new, v_new, oracle_runs=None):
    """Commit `runs` = [(request, first slot, tokens)] on the GPU and with the oracle; return both page sets
    as flat byte arrays. `oracle_runs` (default: the same runs, with their token offsets) lets a test hand the
    oracle only the tokens the library must not skip: [(request, first slot, first token, tokens)]."""
    dev = torch.device("cuda:0")
    dt = pages.kv_dtype
    cu = np.cumsum([0] + [c for _, _, c in runs]).astype(np.int32)
    k_ref = pages.k.view(_VIEW[dt]).numpy().reshape(-1).copy()
    v_ref = pages.v.view(_VIEW[dt]).numpy().reshape(-1).copy()
    ks = None if pages.k_scales is None else pages.k_scales.numpy()
    vs = None if pages.v_scales is None else pages.v_scales.numpy()
    if oracle_runs is None:
        oracle_runs = [(r, f, int(cu[i]), c) for i, (r, f, c) in enumerate(runs)]
    for r, f, t0, c in oracle_runs:
        OC.kv_commit(k_ref, v_ref, ks, vs, _raw_src(k_new)[t0:t0 + c], _raw_src(v_new)[t0:t0 + c], bt, [r], [f], [0, c],
                     Hkv=pages.Hkv, D=pages.D, P=pages.P, kv_dtype=dt)
    k_dev, v_dev = pages.k.to(dev), pages.v.to(dev)
    i32 = lambda a: torch.tensor(np.asarray(a, dtype=np.int32), dtype=torch.int32, device=dev)
    p = M.make_commit_params(k_new.to(dev), v_new.to(dev), k_dev, v_dev, i32(bt), i32([r for r, _, _ in runs]),
                             i32([f for _, f, _ in runs]), i32(cu),
                             k_scales=None if ks is None else pages.k_scales.to(dev),
                             v_scales=None if vs is None else pages.v_scales.to(dev))
    M.kv_commit(p)
    torch.cuda.synchronize()
    got_k = k_dev.cpu().view(torch.uint8).numpy().reshape(-1)
    got_v = v_dev.cpu().view(torch.uint8).numpy().reshape(-1)
    return got_k, got_v, k_ref.view(np.uint8), v_ref.view(np.uint8)


def assert_same(got_k, got_v, want_k, want_v):
    bad_k, bad_v = np.flatnonzero(got_k != want_k), np.flatnonzero(got_v != want_v)
    assert bad_k.size == 0, f"{bad_k.size} K bytes differ, first at {bad_k[:4]}"
    assert bad_v.size == 0, f"{bad_v.size} V bytes differ, first at {bad_v[:4]}"


@pytest.mark.parametrize("kv_dtype,D,P", [("bf16", 128, 16), ("bf16", 128, 32), ("bf16", 64, 16), ("bf16", 64, 32),
                                          ("f32", 64, 16), ("f32", 128, 32), ("f8e4m3", 128, 32), ("f8e4m3", 128, 16),
                                          ("f8e4m3", 64, 32)])
def test_ragged_runs_match_the_oracle_byte_for_byte(mepic, kv_dtype, D, P):
    Hkv, N, B, MB = 3, 40, 3, 12
    rng = np.random.default_rng(hash((kv_dtype, D, P)) % 1000)
    pages = W.gen_pages(21, N, Hkv, P, D, kv_dtype)
    bt = rng.permutation(N)[: B * MB].reshape(B, MB).astype(np.int32)
    # aligned and unaligned starts, a one-token run, an empty run, several runs of one request, a run that
    # ends exactly on a page boundary, a long run over several tiles
    runs = [(0, 0, 3 * P), (1, 5, 2 * P + 3), (2, P - 1, 1), (2, 3 * P, 0), (2, 4 * P + 8, 8), (1, 6 * P + 2, P - 2),
            (0, 4 * P, 5 * P + 7)]
    n = sum(c for _, _, c in runs)
    assert_same(*run_both(mepic, pages, bt, runs, _src(rng, n, Hkv, D, kv_dtype), _src(rng, n, Hkv, D, kv_dtype)))


def test_decode_step_shape_one_token_per_request(mepic):
    Hkv, D, P, B, MB = 8, 128, 16, 64, 6
    rng = np.random.default_rng(7)
    pages = W.gen_pages(22, B * MB, Hkv, P, D, "bf16")
    bt = rng.permutation(B * MB).reshape(B, MB).astype(np.int32)
    runs = [(b, int(rng.integers(0, MB * P)), 1) for b in range(B)]
    assert_same(*run_both(mepic, pages, bt, runs, _src(rng, B, Hkv, D, "bf16"), _src(rng, B, Hkv, D, "bf16")))


def test_fp8_ties_saturation_zero_and_tiny_values(mepic):
    Hkv, D, P = 1, 128, 32
    pages = W.gen_pages(23, 4, Hkv, P, D, "f8e4m3")
    pages.k_scales[:] = torch.tensor([1.0, 0.5, 3.0, 2.0 ** -20])
    pages.v_scales[:] = torch.tensor([2.0, 1.0, 0.37, 1e4])
    mags = OC.e4m3_magnitudes()
    mids = (mags[1:] + mags[:-1]) / 2                    # every tie; all fit bf16 exactly (at most 5 significant bits)
    special = np.concatenate([mids, -mids, mags, -mags, [0.0, -0.0, 448.0, 449.0, 464.0, 1e6, -1e6, 2.0 ** -11, -2.0 ** -11,
                                                          1e-30, -1e-30, 1e-36, -1e-36, 3.0e38, -3.0e38]])
    special = torch.from_numpy(special.astype(np.float32)).to(torch.bfloat16)
    assert torch.equal(special.float()[: 2 * len(mids)], torch.from_numpy(np.concatenate([mids, -mids]).astype(np.float32)))
    n = 4 * P
    reps = (n * Hkv * D + len(special) - 1) // len(special)
    src = special.repeat(reps)[: n * Hkv * D].reshape(n, Hkv, D).contiguous()
    bt = np.array([[0, 1, 2, 3]], dtype=np.int32)
    assert_same(*run_both(mepic, pages, bt, [(0, 0, n)], src, src.flip(0).contiguous()))


def test_out_of_range_requests_blocks_and_pages_are_skipped(mepic):
    Hkv, D, P, N = 2, 128, 16, 8
    rng = np.random.default_rng(9)
    pages = W.gen_pages(24, N, Hkv, P, D, "bf16")
    bt = np.array([[3, -1, 5, N], [6, 2, 0, 1]], dtype=np.int32)     # request 0: block 1 unassigned, block 3 beyond the pool
    runs = [(0, 4, 3 * P + 20), (2, 0, 5), (-1, 0, 3), (1, 3 * P + 10, 20), (1, 0, 4)]
    n = sum(c for _, _, c in runs)
    # what must land: request 0 slots [4, P) and [2P, 3P); request 1 slots [3P+10, 4P) (the rest is past the table)
    oracle_runs = [(0, 4, 0, P - 4), (0, 2 * P, 2 * P - 4, P), (1, 3 * P + 10, 3 * P + 20 + 5 + 3, P - 10),
                   (1, 0, 3 * P + 20 + 5 + 3 + 20, 4)]
    assert_same(*run_both(mepic, pages, bt, runs, _src(rng, n, Hkv, D, "bf16"), _src(rng, n, Hkv, D, "bf16"),
                          oracle_runs=oracle_runs))


@pytest.mark.parametrize("kv_dtype,P", [("bf16", 16), ("f8e4m3", 32)])
def test_full_size_prompt_commit(mepic, kv_dtype, P):
    """The measured workload: 64 requests x 1024 new tokens, Llama-3-8B KV shape; every byte compared."""
    Hkv, D, B, T = 8, 128, 64, 1024
    MB = T // P + 1
    rng = np.random.default_rng(10)
    pages = W.gen_pages(25, B * MB, Hkv, P, D, kv_dtype)
    bt = rng.permutation(B * MB).reshape(B, MB).astype(np.int32)
    runs = [(b, (b % 3) * 8, T) for b in range(B)]                   # starts at slot 0, 8 or 16
    k_new, v_new = _src(rng, B * T, Hkv, D, kv_dtype), _src(rng, B * T, Hkv, D, kv_dtype)
    assert_same(*run_both(mepic, pages, bt, runs, k_new, v_new))


def test_commit_then_attend_equals_the_oracle_on_the_original_pages(mepic, oracle_attn):
    """Wipe the private tail of every request, put it back through mepic_kv_commit, run decode attention."""
    from harness import DeviceCase, align_with_oracle, oracle_out
    st = W.decode_structure("commit_then_attend", 77, B=6, Hq=8, Hkv=2, D=128, P=16, theta=1e4,
                            q_dtype="bf16", kv_dtype="bf16", prefix=20, n_chunks=2, chunk_tokens=100, pool=3,
                            question=50)
    aligned, _ = align_with_oracle(st)
    case = W.assemble(st, aligned)
    want = oracle_out(oracle_attn, case)
    dc = DeviceCase(mepic, case)
    P, dev = st.P, torch.device("cuda:0")
    kl, vl = W.unpack_k(case.pages.k), W.unpack_v(case.pages.v)     # [N, Hkv, P, D]
    runs, k_rows, v_rows = [], [], []
    for b in range(st.B):
        n1 = int(case.kv_lens[b])
        n0 = max(0, n1 - 40)
        runs.append((b, n0, n1 - n0))
        for n in range(n0, n1):
            p = int(case.block_tables[b, n // P])
            k_rows.append(kl[p, :, n % P, :]); v_rows.append(vl[p, :, n % P, :])
            dc.k.view(torch.int16)[p, :, :, n % P, :] = 0x7FC0           # NaN
            dc.v.view(torch.int16)[p, :, :, n % P] = 0x7FC0
    assert not (np.abs(dc.run() - want).max() <= 2e-2)            # the wipe is visible (NaN or far off)
    i32 = lambda a: torch.tensor(a, dtype=torch.int32, device=dev)
    cu = np.cumsum([0] + [c for _, _, c in runs])
    # the params struct holds raw pointers: keep every tensor it points at alive for as long as it is used
    held = (torch.stack(k_rows).to(dev), torch.stack(v_rows).to(dev), i32([r for r, _, _ in runs]),
            i32([f for _, f, _ in runs]), i32(cu))
    p = mepic.make_commit_params(held[0], held[1], dc.k, dc.v, dc.bt, held[2], held[3], held[4])
    mepic.kv_commit(p)
    got = dc.run()
    assert np.abs(got - want).max() <= 2e-2
    # the same right after another commit, with the attention reading the pages past the caches
    mepic.kv_commit(p)
    dc.params.flags |= mepic.FLAG_KV_READ_ONCE
    assert np.array_equal(dc.run(), got)
