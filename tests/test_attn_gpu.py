"""GPU parity: the library's attention (through the C-ABI) against the fp64 oracle, element by element,
on the same seeded inputs. Block tables come from the oracle's aligner and are also checked against
the library's aligner. Tolerances: 1e-4 max-abs for fp32 storage, 2e-2 for bf16 and bf16+fp8."""
import numpy as np
import pytest
import torch

import workloads as W
from harness import DeviceCase, align_with_library, align_with_oracle, oracle_out

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2, "f8e4m3": 2e-2}


def build_case(M, st, **kw):
    aligned, _ = align_with_oracle(st)
    lib_aligned, _ = align_with_library(M, st)
    for a, b in zip(aligned, lib_aligned):                      # page-table parity is bit-exact
        assert b["block_table"].tolist() == a["block_table"] and b["info"] == a["info"]
    return W.assemble(st, aligned, **kw)


def check(M, oracle_attn, case, flags=0, rows=None, expect_kernel=None, **okw):
    dc = DeviceCase(M, case, flags=flags | (M.FLAG_ROPE_INTERLEAVED if okw.get("interleaved") else 0),
                    sm_scale=okw.get("sm_scale", 0.0))
    got = dc.run()
    if expect_kernel is not None:
        assert M.last_kernel() == expect_kernel, M.last_kernel()
    want = oracle_out(oracle_attn, case, rows=rows, **okw)
    if rows is not None:
        got = np.stack([got[t, h] for t, h in rows])
    assert got.shape == want.shape
    assert np.isfinite(got).all(), "non-finite output (a poisoned slot or page leaked in)"
    err = np.abs(got - want).max() if got.size else 0.0
    assert err <= TOL[case.st.kv_dtype], f"max abs err {err:.3e} ({M.last_kernel()})"
    return err, dc


def small_decode(kv_dtype, seed=7, **kw):
    base = dict(B=5, Hq=8, Hkv=2, D=128, P=16, theta=5e5, q_dtype="f32" if kv_dtype == "f32" else "bf16",
                kv_dtype=kv_dtype, prefix=48, n_chunks=(1, 4), chunk_tokens=160, pool=4, question=37)
    base.update(kw)
    return W.decode_structure(f"small_decode_{kv_dtype}", seed, **base)


BOTH_PATHS = [0, 2]  # 2 = FLAG_FORCE_GENERAL


def test_config1_tiny_decode_fp32(mepic, oracle_attn):
    case = build_case(mepic, W.config(1))
    assert case.kv_lens.tolist() == [289] and case.n_blocks.tolist() == [19]
    check(mepic, oracle_attn, case)


@pytest.mark.parametrize("flags", BOTH_PATHS)
@pytest.mark.parametrize("kv_dtype", ["f32", "bf16", "f8e4m3"])
def test_small_decode_all_dtypes(mepic, oracle_attn, kv_dtype, flags):
    P = 32 if kv_dtype == "f8e4m3" else 16
    check(mepic, oracle_attn, build_case(mepic, small_decode(kv_dtype, P=P)), flags=flags)


@pytest.mark.parametrize("kv_dtype,P", [("bf16", 16), ("f8e4m3", 32), ("f32", 16)])
def test_read_once_hint_changes_no_result(mepic, oracle_attn, kv_dtype, P):
    """MEPIC_FLAG_KV_READ_ONCE only changes how the matrix-core decode kernels load pages (other kernels ignore it):
    same bits as without it, on shared pages and on one page per logical block, and within tolerance of the oracle."""
    case = build_case(mepic, small_decode(kv_dtype, P=P, B=9, n_chunks=(2, 6)))
    for c in (case, W.to_duplicated(case)):
        _, plain = check(mepic, oracle_attn, c)
        want = plain.out.clone()
        _, hinted = check(mepic, oracle_attn, c, flags=mepic.FLAG_KV_READ_ONCE)
        assert torch.equal(hinted.out, want)


@pytest.mark.parametrize("flags", BOTH_PATHS)
def test_decode_gqa7_fp8_page32(mepic, oracle_attn, flags):
    """Head shapes of the mixed-length config: 28 query heads on 4 KV heads, page 32, theta 1e6."""
    st = W.decode_structure("small_cfg5", 11, B=9, Hq=28, Hkv=4, D=128, P=32, theta=1e6, q_dtype="bf16",
                            kv_dtype="f8e4m3", prefix=0, n_chunks=(1, 9), chunk_tokens=512, pool=6, question=0)
    check(mepic, oracle_attn, build_case(mepic, st), flags=flags)


@pytest.mark.parametrize("flags", BOTH_PATHS)
def test_decode_long_context_many_splits(mepic, oracle_attn, flags):
    """One long request next to short ones: several splits, ragged last split, positions up to ~20K."""
    st = W.decode_structure("long_short", 13, B=3, Hq=32, Hkv=8, D=128, P=16, theta=5e5, q_dtype="bf16",
                            kv_dtype="bf16", prefix=0, n_chunks=(1, 20), chunk_tokens=1024, pool=5, question=19)
    check(mepic, oracle_attn, build_case(mepic, st), flags=flags)


@pytest.mark.parametrize("D,P", [(64, 16), (64, 32), (128, 32)])
@pytest.mark.parametrize("kv_dtype", ["f32", "bf16"])
def test_decode_other_shapes(mepic, oracle_attn, kv_dtype, D, P):
    st = small_decode(kv_dtype, D=D, P=P, Hq=6, Hkv=3, theta=1e4, chunk_tokens=96)
    check(mepic, oracle_attn, build_case(mepic, st))


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16"])
def test_interleaved_pairing_and_explicit_scale(mepic, oracle_attn, kv_dtype):
    case = build_case(mepic, small_decode(kv_dtype, seed=3))
    check(mepic, oracle_attn, case, interleaved=True)
    check(mepic, oracle_attn, case, sm_scale=0.05)


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16", "f8e4m3"])
@pytest.mark.parametrize("pads_are_positions", [True, False])
def test_ragged_segments_with_pads_both_readings(mepic, oracle_attn, kv_dtype, pads_are_positions):
    """Segment lengths that are not multiples of the page: leading pads in chunks, trailing pads in prompts.
    Reading 1: pads are ordinary slots. Reading 2: the aligner's valid masks and pad-free positions are used."""
    P = 32 if kv_dtype == "f8e4m3" else 16
    st = W.Structure("ragged", "decode", 3, 8, 2, 128, P, 1e4, "f32" if kv_dtype == "f32" else "bf16", kv_dtype, 21)
    C = W.CHUNK_KEY_BASE
    st.requests = [[(0, 35, 0), (1, 100, C + 1), (0, 7, 0), (1, 45, C + 2), (0, 20, 0)],
                   [(1, 45, C + 2), (1, 100, C + 1)],
                   [(0, 3, 0)]]
    st.n_q = [1, 1, 1]
    case = build_case(mepic, st, pads_are_positions=pads_are_positions)
    assert (case.block_valid_mask is None) == pads_are_positions
    check(mepic, oracle_attn, case)


@pytest.mark.parametrize("kv_dtype", ["f32", "bf16", "f8e4m3"])
def test_masked_pad_slots_may_hold_nan(mepic, oracle_attn, kv_dtype):
    """Under the reading in which pad slots do not take part (valid masks), nobody ever writes them: the commit step
    leaves the pad slots of a request-private block as they were. Poison them with NaN in K and V; the result must
    not change (a probability of zero times a NaN would)."""
    P = 32 if kv_dtype == "f8e4m3" else 16
    st = W.Structure("ragged_nan", "decode", 3, 8, 2, 128, P, 1e4, "f32" if kv_dtype == "f32" else "bf16", kv_dtype, 22)
    C = W.CHUNK_KEY_BASE
    st.requests = [[(0, 35, 0), (1, 100, C + 1), (0, 7, 0), (1, 45, C + 2), (0, 20, 0)],
                   [(1, 45, C + 2), (1, 100, C + 1)],
                   [(0, 3, 0)]]
    st.n_q = [1, 1, 1]
    case = build_case(mepic, st, pads_are_positions=False)
    pg, n_poisoned = case.pages, 0
    for b in range(st.B):
        for j in range(int(case.n_blocks[b])):
            for sl in range(P):
                if j * P + sl < int(case.kv_lens[b]) and not (int(case.block_valid_mask[b, j]) >> sl) & 1:
                    page = int(case.block_tables[b, j])
                    if kv_dtype == "f8e4m3":
                        pg.k.view(torch.uint8)[page, :, :, sl, :] = 0x7F
                        pg.v.view(torch.uint8)[page, :, :, sl] = 0x7F
                    else:
                        pg.k[page, :, :, sl, :] = float("nan")
                        pg.v[page, :, :, sl] = float("nan")
                    n_poisoned += 1
    assert n_poisoned > 20
    check(mepic, oracle_attn, case)


def test_prefill_small_fp32_and_bf16(mepic, oracle_attn):
    for kv_dtype, flags in (("f32", 0), ("bf16", 0), ("bf16", 2)):
        st = W.prefill_structure("small_prefill", 17, B=3, Hq=8, Hkv=2, D=128, P=16, theta=5e5, n_chunks=3,
                                 chunk_tokens=144, pool=4, q_tokens=70, max_gap_pages=2,
                                 q_dtype="f32" if kv_dtype == "f32" else "bf16", kv_dtype=kv_dtype)
        check(mepic, oracle_attn, build_case(mepic, st), flags=flags)


def test_prefill_ragged_query_counts(mepic, oracle_attn):
    st = W.prefill_structure("ragged_prefill", 19, B=4, Hq=32, Hkv=8, D=128, P=16, theta=5e5, n_chunks=2,
                             chunk_tokens=256, pool=3, q_tokens=1)
    st.n_q = [1, 33, 64, 7]
    for b, n in enumerate(st.n_q):
        st.requests[b][-1] = (0, n + 5 * b, 0)          # the question segment is longer than the query count
    check(mepic, oracle_attn, build_case(mepic, st))


def test_empty_and_degenerate_requests(mepic, oracle_attn):
    """kv_len 0 (all-zero output row), kv_len 1 (output = that V row), and an empty batch."""
    st = W.Structure("degenerate", "decode", 3, 8, 2, 128, 16, 1e4, "bf16", "bf16", 23)
    st.requests = [[(0, 1, 0)], [(0, 1, 0)], [(0, 40, 0)]]
    st.extra_tail = 0
    st.n_q = [1, 1, 1]
    case = build_case(mepic, st)
    case.kv_lens[0] = 0
    err, dc = check(mepic, oracle_attn, case)
    out = dc.out.float().cpu().numpy()
    assert (out[0] == 0).all()
    v_row = W.unpack_v(case.pages.v)[case.block_tables[1, 0], :, 0, :].float().numpy()   # [Hkv, D], slot 0
    assert np.array_equal(out[1], np.repeat(v_row, 4, axis=0))
    # B = 0: nothing to do, no launch, no error
    z = torch.zeros((0, 8, 128), dtype=torch.bfloat16, device="cuda")
    zi = torch.zeros((0,), dtype=torch.int32, device="cuda")
    p = mepic.make_params(z, z.clone(), dc.k, dc.v, torch.zeros((0, 4), dtype=torch.int32, device="cuda"), zi, zi,
                          rope_theta=1e4, workspace=dc.ws)
    mepic.attn_decode(p)


@pytest.mark.parametrize("kv_dtype", ["bf16", "f8e4m3"])
def test_shared_and_duplicated_layouts_agree_bitwise(mepic, oracle_attn, kv_dtype):
    """Sharing pages changes nothing numerically: the work split depends on the logical shape only."""
    P = 32 if kv_dtype == "f8e4m3" else 16
    case = build_case(mepic, small_decode(kv_dtype, P=P, B=8, pool=2), poison=False)
    dup = W.to_duplicated(case)
    assert dup.pages.num_pages == int(case.n_blocks.sum()) > case.pages.num_pages
    a = DeviceCase(mepic, case).run()
    b = DeviceCase(mepic, dup).run()
    assert np.array_equal(a, b)
    assert np.abs(a - oracle_out(oracle_attn, dup)).max() <= TOL[kv_dtype]


def test_chunk_twice_in_one_request_uses_request_positions(mepic, oracle_attn):
    """The same shared pages at two offsets of one block table: rotation must follow the request's positions."""
    st = W.Structure("twice", "decode", 1, 8, 2, 128, 16, 5e5, "bf16", "bf16", 29)
    C = W.CHUNK_KEY_BASE
    st.requests = [[(1, 256, C + 1), (0, 16, 0), (1, 256, C + 1), (1, 256, C + 1)]]
    st.n_q = [1]
    case = build_case(mepic, st)
    bt = case.block_tables[0]
    assert bt[1:16].tolist() == bt[18:33].tolist() == bt[34:49].tolist()
    check(mepic, oracle_attn, case)


# ------------------------------------------------------------------ the benchmark configurations at full size
def sample_rows(case, n, seed=0):
    rng = np.random.default_rng(seed)
    nq, Hq = case.n_q, case.st.Hq
    rows = {(0, 0), (nq - 1, Hq - 1)}
    while len(rows) < min(n, nq * Hq):
        rows.add((int(rng.integers(nq)), int(rng.integers(Hq))))
    return sorted(rows)


@pytest.mark.parametrize("cfg", [2, 4, 5])
def test_full_size_decode_configs_every_row(mepic, oracle_attn, cfg):
    """Configs 2, 4, 5 at full size in the launch configuration the bench times: EVERY (request, head) row against
    the oracle (a few seconds of oracle time each), shared vs duplicated layout bitwise equal."""
    case = build_case(mepic, W.config(cfg))
    err, dc = check(mepic, oracle_attn, case)
    out = dc.out.float()
    assert torch.isfinite(out).all()
    if cfg == 2:
        dup = DeviceCase(mepic, W.to_duplicated(case))
        assert torch.equal(torch.from_numpy(dup.run()), out.double().cpu())


def test_full_size_prefill_config3_every_workgroup(mepic, oracle_attn):
    """Config 3 at full size: one row out of every workgroup's tile, i.e. per (request, tile of 64 query tokens, KV
    head) a random token of the tile and a random head of the KV head's group (512 rows), plus the first and last
    row of every request, which sit on the causal edge."""
    st = W.config(3)
    case = build_case(mepic, st)
    rng = np.random.default_rng(3)
    G, tok_per_wg = st.Hq // st.Hkv, 256 // (st.Hq // st.Hkv)
    rows = set()
    for b in range(st.B):
        q0, q1 = int(case.cu_q_lens[b]), int(case.cu_q_lens[b + 1])
        for t0 in range(q0, q1, tok_per_wg):
            for hk in range(st.Hkv):
                rows.add((int(rng.integers(t0, min(t0 + tok_per_wg, q1))), hk * G + int(rng.integers(G))))
        rows.add((q0, 0))
        rows.add((q1 - 1, st.Hq - 1))
    assert len(rows) >= st.B * (256 // tok_per_wg) * st.Hkv
    check(mepic, oracle_attn, case, rows=sorted(rows), expect_kernel="prefill_mfma_bf16")


# ------------------------------------------------------------------ more shapes for the matrix-core paths
@pytest.mark.parametrize("kv_dtype,P,kernel", [("bf16", 16, "decode_mfma_bf16"), ("f8e4m3", 32, "decode_mfma_fp8")])
@pytest.mark.parametrize("G", [1, 2, 8, 16])
def test_decode_matrix_core_group_sizes(mepic, oracle_attn, kv_dtype, P, kernel, G):
    st = small_decode(kv_dtype, seed=31 + G, P=P, B=6, Hq=2 * G, Hkv=2, n_chunks=(1, 6), chunk_tokens=192, question=21)
    check(mepic, oracle_attn, build_case(mepic, st), expect_kernel=kernel)


@pytest.mark.parametrize("kv_dtype,P", [("bf16", 16), ("f8e4m3", 32)])
def test_decode_many_requests_skewed_lengths(mepic, oracle_attn, kv_dtype, P):
    """More requests than one wave scans at once, one very long request among short and empty ones: the
    equal-chunk cut crosses many request boundaries and the long request is cut into many pieces."""
    st = W.Structure("skewed", "decode", 150, 8, 2, 128, P, 5e5, "bf16", kv_dtype, 37)
    rng = np.random.default_rng(37)
    C = W.CHUNK_KEY_BASE
    for b in range(st.B):
        if b == 77:
            segs = [(1, 4096, C + 1)] * 6 + [(0, 333, 0)]
        else:
            segs = [(0, int(rng.integers(1, 90)), 0)]
            if rng.random() < 0.3:
                segs.insert(0, (1, 256, C + 2))
        st.requests.append(segs)
        st.n_q.append(1)
    case = build_case(mepic, st)
    case.kv_lens[[3, 40, 149]] = 0                        # empty requests in between
    rows = [(b, h) for b in (0, 3, 40, 76, 77, 78, 148, 149) for h in range(8)]
    err, dc = check(mepic, oracle_attn, case, rows=rows)
    assert mepic.last_kernel().startswith("decode_mfma")
    out = dc.out.float()
    assert torch.isfinite(out).all() and (out[[3, 40, 149]] == 0).all()


def test_dispatch_names(mepic, oracle_attn):
    """Which kernel serves which case (the general kernel must stay reachable for everything else)."""
    for st, want in ((small_decode("bf16"), "decode_mfma_bf16"), (small_decode("f8e4m3", P=32), "decode_mfma_fp8"),
                     (small_decode("f32"), "general"), (small_decode("bf16", P=32), "general"),
                     (small_decode("f8e4m3", P=16), "general"), (small_decode("bf16", D=64), "general")):
        check(mepic, oracle_attn, build_case(mepic, st), expect_kernel=want)


@pytest.mark.parametrize("G", [1, 2, 8])
def test_prefill_matrix_core_group_sizes_and_ragged_kv(mepic, oracle_attn, G):
    """kv_len not a multiple of the 64-slot tile, query counts not a multiple of the row tile."""
    st = W.prefill_structure("prefill_g", 41 + G, B=3, Hq=2 * G, Hkv=2, D=128, P=16, theta=5e5, n_chunks=3,
                             chunk_tokens=208, pool=3, q_tokens=1, max_gap_pages=1)
    st.n_q = [37, 300, 5]
    for b, n in enumerate(st.n_q):
        st.requests[b][-1] = (0, n + 11 * b, 0)
    check(mepic, oracle_attn, build_case(mepic, st), expect_kernel="prefill_mfma_bf16")


@pytest.mark.parametrize("ctx", [17, 64, 65, 129, 193, 260])
def test_prefill_contexts_of_one_to_five_tiles(mepic, oracle_attn, ctx):
    """The tile loop's start-up and tail: loads run two tiles ahead and staging is unconditional past the last tile,
    so contexts of one to five 64-slot tiles (odd and even counts, ragged ends) each take a different path."""
    st = W.prefill_structure(f"prefill_ctx_{ctx}", 47, B=2, Hq=8, Hkv=2, D=128, P=16, theta=5e5, n_chunks=1,
                             chunk_tokens=ctx, pool=2, q_tokens=1, max_gap_pages=0)
    st.n_q = [9, 70]
    for b, n in enumerate(st.n_q):
        st.requests[b][-1] = (0, n + 3 * b, 0)
    check(mepic, oracle_attn, build_case(mepic, st), expect_kernel="prefill_mfma_bf16")


def test_prefill_queries_in_the_middle_and_far_positions(mepic, oracle_attn):
    """Query positions well inside the context (most of the KV is causally hidden) and positions around 40K."""
    st = W.prefill_structure("prefill_mid", 43, B=2, Hq=8, Hkv=2, D=128, P=16, theta=5e5, n_chunks=40,
                             chunk_tokens=1024, pool=4, q_tokens=40, max_gap_pages=0)
    case = build_case(mepic, st)
    case.q_positions[:40] = np.arange(1000, 1040)         # request 0: sees only the first ~1000 slots
    rows = [(t, h) for t in (0, 17, 39, 40, 61, 79) for h in (0, 3, 7)]
    check(mepic, oracle_attn, case, rows=rows, expect_kernel="prefill_mfma_bf16")


@pytest.mark.parametrize("order", ["random", "rising", "falling"])
def test_fp8_page_scales_spread_over_four_decades(mepic, oracle_attn, order):
    """Per-page V (and K) scales that differ by up to 10^4 between the pages of one request, in random, rising and
    falling order along the request: the matrix-core kernel keeps its output accumulator in units of a reference
    V scale that it raises on the way, which this exercises; the stored value of a slot is code * scale either way."""
    st = W.decode_structure("fp8_scale_spread", 13, B=6, Hq=28, Hkv=4, D=128, P=32, theta=1e6, q_dtype="bf16",
                            kv_dtype="f8e4m3", prefix=40, n_chunks=(2, 6), chunk_tokens=512, pool=5, question=70)
    case = build_case(mepic, st)
    rng = np.random.default_rng(17)
    n = case.pages.num_pages
    f = 10.0 ** rng.uniform(-4, 0, size=n)
    if order != "random":                     # pages are handed out in rising order along a request
        f = np.sort(f) if order == "rising" else np.sort(f)[::-1].copy()
    case.pages.v_scales *= torch.from_numpy(f.astype(np.float32)) / case.pages.v_scales.max()
    case.pages.k_scales *= torch.from_numpy((10.0 ** rng.uniform(-1, 0, size=n)).astype(np.float32))
    check(mepic, oracle_attn, case, expect_kernel="decode_mfma_fp8")
    check(mepic, oracle_attn, case, flags=2)


# ------------------------------------------------------------------ seeded random structures
@pytest.mark.parametrize("seed", range(16))
def test_random_decode_structures(mepic, oracle_attn, seed):
    """Random batch sizes, group sizes, chunk mixes and lengths on both matrix-core decode kernels."""
    rng = np.random.default_rng(1000 + seed)
    fp8 = bool(seed & 1)
    G = int(rng.choice([1, 2, 3, 4, 7, 8]))
    Hkv = int(rng.choice([1, 2, 4]))
    st = W.decode_structure(f"rand_decode_{seed}", 500 + seed, B=int(rng.integers(1, 40)), Hq=G * Hkv, Hkv=Hkv, D=128,
                            P=32 if fp8 else 16, theta=float(rng.choice([1e4, 5e5, 1e6])), q_dtype="bf16",
                            kv_dtype="f8e4m3" if fp8 else "bf16", prefix=int(rng.integers(0, 200)),
                            n_chunks=(0, int(rng.integers(1, 9))), chunk_tokens=int(rng.integers(17, 700)),
                            pool=int(rng.integers(1, 6)), question=int(rng.integers(0, 150)))
    case = build_case(mepic, st)
    n_rows = case.n_q * st.Hq
    rows = None if n_rows <= 256 else sample_rows(case, 256, seed)
    check(mepic, oracle_attn, case, rows=rows, expect_kernel="decode_mfma_fp8" if fp8 else "decode_mfma_bf16")


@pytest.mark.parametrize("seed", range(8))
def test_random_prefill_structures(mepic, oracle_attn, seed):
    rng = np.random.default_rng(2000 + seed)
    G = int(rng.choice([1, 2, 4, 8]))
    Hkv = int(rng.choice([1, 2]))
    B = int(rng.integers(1, 5))
    st = W.prefill_structure(f"rand_prefill_{seed}", 600 + seed, B=B, Hq=G * Hkv, Hkv=Hkv, D=128, P=16, theta=5e5,
                             n_chunks=int(rng.integers(1, 6)), chunk_tokens=int(rng.integers(30, 500)),
                             pool=int(rng.integers(1, 4)), q_tokens=1, max_gap_pages=int(rng.integers(0, 3)))
    st.n_q = [int(rng.integers(1, 400)) for _ in range(B)]
    for b, n in enumerate(st.n_q):
        st.requests[b][-1] = (0, n + int(rng.integers(0, 40)), 0)
    case = build_case(mepic, st)
    n_rows = case.n_q * st.Hq
    rows = None if n_rows <= 512 else sample_rows(case, 512, seed)
    check(mepic, oracle_attn, case, rows=rows, expect_kernel="prefill_mfma_bf16")
