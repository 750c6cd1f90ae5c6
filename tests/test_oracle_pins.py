"""Pins of the fp64 attention oracle against facts that do not come from the oracle itself.

Each test plants nothing in the product: it checks oracle/mepic_oracle.c against brute force written
here in another formulation (complex-number RoPE over contiguous, pre-rotated K/V — the
rotate-then-store path that §3.3.3 says the fused operator must equal), against closed forms, against
invariants of rotary embedding, and against a library's dtype conversions.
"""
import math

import numpy as np
import pytest
import torch

F32, BF16, F8 = "f32", "bf16", "f8e4m3"


# --------------------------------------------------------------------------------------------
# helpers written independently of the oracle
# --------------------------------------------------------------------------------------------
def rope_complex(x, pos, theta, interleaved=False):
    """RoPE as multiplication of complex pairs by e^{i pos f}. x: [..., D] float64."""
    D = x.shape[-1]
    f = theta ** (-np.arange(D // 2, dtype=np.float64) * 2.0 / D)
    ph = np.exp(1j * pos * f)
    if interleaved:
        z = x[..., 0::2] + 1j * x[..., 1::2]
        z = z * ph
        out = np.empty_like(x)
        out[..., 0::2], out[..., 1::2] = z.real, z.imag
        return out
    z = x[..., : D // 2] + 1j * x[..., D // 2:]
    z = z * ph
    return np.concatenate([z.real, z.imag], axis=-1)


def brute_attention(q, K, V, pos_q, pos_k, G, theta, causal, interleaved=False, visible=None):
    """q [Hq, D]; K, V [L, Hkv, D] contiguous and UN-rotated; returns [Hq, D]. Three plain loops."""
    Hq, D = q.shape
    L = K.shape[0]
    Khat = np.stack([rope_complex(K[n], pos_k[n], theta, interleaved) for n in range(L)]) if L else K
    out = np.zeros((Hq, D))
    for h in range(Hq):
        qh = rope_complex(q[h], pos_q, theta, interleaved)
        idx = [n for n in range(L) if (visible is None or visible[n]) and (not causal or pos_k[n] <= pos_q)]
        if not idx:
            continue
        s = np.array([qh @ Khat[n, h // G] for n in idx]) / math.sqrt(D)
        w = np.exp(s - s.max())
        w /= w.sum()
        for wi, n in zip(w, idx):
            out[h] += wi * V[n, h // G]
    return out


def scatter_to_pages(K, V, table, P, X, num_pages):
    """Write contiguous K, V [L, Hkv, D] into pages by the index formulas of the C-ABI header."""
    L, Hkv, D = K.shape
    kp = np.full((num_pages, Hkv, D // X, P, X), np.nan, dtype=np.float32)
    vp = np.full((num_pages, Hkv, D, P), np.nan, dtype=np.float32)
    for n in range(L):
        p, s = table[n // P], n % P
        for h in range(Hkv):
            for d in range(D):
                kp[p, h, d // X, s, d % X] = K[n, h, d]
                vp[p, h, d, s] = V[n, h, d]
    return kp, vp


def run_oracle(oracle_attn, q, kp, vp, tables, kv_lens, q_pos, Hq, Hkv, D, P, theta, **kw):
    return oracle_attn.attention(np.asarray(q, np.float32), F32, kp, vp, F32, tables, kv_lens, q_pos,
                                 Hq=Hq, Hkv=Hkv, D=D, P=P, theta=theta, **kw)


def small_case(seed, L, Hq=4, Hkv=2, D=8, P=4, extra_pages=3):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((L, Hkv, D)).astype(np.float32).astype(np.float64)
    V = rng.standard_normal((L, Hkv, D)).astype(np.float32).astype(np.float64)
    q = rng.standard_normal((Hq, D)).astype(np.float32).astype(np.float64)
    nb = -(-L // P)
    table = rng.permutation(nb + extra_pages)[:nb]
    kp, vp = scatter_to_pages(K, V, table, P, 4, nb + extra_pages)
    return q, K, V, table, kp, vp


# --------------------------------------------------------------------------------------------
# P1: gather + rotate-on-the-fly == standard attention over contiguous pre-rotated K/V
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("L,interleaved", [(1, False), (5, False), (13, False), (16, True), (23, True)])
def test_decode_equals_bruteforce_over_prerotated_kv(oracle_attn, L, interleaved):
    Hq, Hkv, D, P, theta = 4, 2, 8, 4, 100.0
    q, K, V, table, kp, vp = small_case(L, L, Hq, Hkv, D, P)
    pos_q = L - 1
    want = brute_attention(q, K, V, pos_q, np.arange(L), Hq // Hkv, theta, causal=False, interleaved=interleaved)
    got = run_oracle(oracle_attn, q[None], kp, vp, table[None], [L], [pos_q], Hq, Hkv, D, P, theta,
                     interleaved=interleaved)[0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_decode_matches_torch_sdpa_fp64(oracle_attn):
    """Library special case: rotate K and q outside, then scaled_dot_product_attention in fp64."""
    Hq, Hkv, D, P, theta, L = 4, 2, 8, 4, 10000.0, 19
    q, K, V, table, kp, vp = small_case(7, L, Hq, Hkv, D, P)
    G = Hq // Hkv
    Khat = np.stack([rope_complex(K[n], n, theta) for n in range(L)])           # [L, Hkv, D]
    qhat = rope_complex(q, L - 1, theta)                                          # [Hq, D]
    kt = torch.from_numpy(Khat).permute(1, 0, 2).repeat_interleave(G, dim=0)      # [Hq, L, D]
    vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, dim=0)
    want = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(qhat)[:, None, :], kt, vt)[:, 0].numpy()
    got = run_oracle(oracle_attn, q[None], kp, vp, table[None], [L], [L - 1], Hq, Hkv, D, P, theta)[0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_prefill_causal_equals_bruteforce(oracle_attn):
    """Two requests, ragged query counts, causal by absolute position."""
    Hq, Hkv, D, P, theta = 4, 2, 8, 4, 50.0
    Ls, nqs = [11, 6], [3, 2]
    cases = [small_case(40 + i, L, Hq, Hkv, D, P, extra_pages=0) for i, L in enumerate(Ls)]
    nb = [len(c[3]) for c in cases]
    kp = np.concatenate([c[4] for c in cases])
    vp = np.concatenate([c[5] for c in cases])
    tables = np.zeros((2, max(nb)), dtype=np.int32)
    tables[0, : nb[0]] = cases[0][3]
    tables[1, : nb[1]] = cases[1][3] + nb[0]
    rng = np.random.default_rng(5)
    q = rng.standard_normal((sum(nqs), Hq, D)).astype(np.float32).astype(np.float64)
    q_pos, want = [], []
    t = 0
    for b, (L, nq) in enumerate(zip(Ls, nqs)):
        for i in range(nq):
            pq = L - nq + i                      # the question tokens are the last nq slots
            q_pos.append(pq)
            want.append(brute_attention(q[t], cases[b][1], cases[b][2], pq, np.arange(L), Hq // Hkv, theta, causal=True))
            t += 1
    got = run_oracle(oracle_attn, q, kp, vp, tables, Ls, q_pos, Hq, Hkv, D, P, theta, cu_q_lens=[0, 3, 5])
    np.testing.assert_allclose(got, np.stack(want), rtol=0, atol=1e-12)


def test_block_positions_and_valid_mask_equal_bruteforce(oracle_attn):
    Hq, Hkv, D, P, theta, L = 2, 1, 8, 4, 30.0, 14
    q, K, V, table, kp, vp = small_case(11, L, Hq, Hkv, D, P)
    rng = np.random.default_rng(3)
    nb = len(table)
    block_pos = rng.integers(-3, 60, size=nb)
    masks = rng.integers(1, 16, size=nb).astype(np.uint32)
    pos_k = np.array([block_pos[n // P] + n % P for n in range(L)])
    visible = np.array([(masks[n // P] >> (n % P)) & 1 for n in range(L)], dtype=bool)
    want = brute_attention(q, K, V, 77, pos_k, Hq // Hkv, theta, causal=False, visible=visible)
    got = run_oracle(oracle_attn, q[None], kp, vp, table[None], [L], [77], Hq, Hkv, D, P, theta,
                     block_positions=block_pos[None], block_valid_mask=masks[None])[0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


# --------------------------------------------------------------------------------------------
# P2: relative-position property — shifting every position by a constant changes nothing
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("shift", [1, 977, 40000])
def test_shift_invariance(oracle_attn, shift):
    Hq, Hkv, D, P, theta, L = 4, 2, 16, 4, 10000.0, 21
    q, K, V, table, kp, vp = small_case(2, L, Hq, Hkv, D, P)
    nb = len(table)
    base = run_oracle(oracle_attn, q[None], kp, vp, table[None], [L], [L + 5], Hq, Hkv, D, P, theta)[0]
    bp = (np.arange(nb) * P + shift)[None]
    moved = run_oracle(oracle_attn, q[None], kp, vp, table[None], [L], [L + 5 + shift], Hq, Hkv, D, P, theta,
                       block_positions=bp)[0]
    np.testing.assert_allclose(moved, base, rtol=0, atol=1e-10)


# --------------------------------------------------------------------------------------------
# P3: a layout that shares pages and one that duplicates them give the same result
# --------------------------------------------------------------------------------------------
def test_shared_equals_duplicated_layout(oracle_attn):
    Hq, Hkv, D, P, theta = 4, 2, 8, 4, 100.0
    rng = np.random.default_rng(9)
    num_pages = 6
    kp = rng.standard_normal((num_pages, Hkv, D // 4, P, 4)).astype(np.float32)
    vp = rng.standard_normal((num_pages, Hkv, D, P)).astype(np.float32)
    # two requests alias pages 1 and 2 at different logical positions; request 1 uses page 1 twice
    tables = np.array([[0, 1, 2, 3], [4, 2, 1, 1]], dtype=np.int32)
    kv_lens = [15, 16]
    q = rng.standard_normal((2, Hq, D)).astype(np.float32)
    shared = run_oracle(oracle_attn, q, kp, vp, tables, kv_lens, [14, 15], Hq, Hkv, D, P, theta)
    flat = tables.reshape(-1)
    dup_tables = np.arange(8, dtype=np.int32).reshape(2, 4)
    dup = run_oracle(oracle_attn, q, kp[flat], vp[flat], dup_tables, kv_lens, [14, 15], Hq, Hkv, D, P, theta)
    assert np.array_equal(shared, dup)
    # and the aliased page really was rotated at the request's own positions: swapping the two aliases of
    # request 1 into different logical blocks changes request 1's result
    other = run_oracle(oracle_attn, q, kp, vp, np.array([[0, 1, 2, 3], [4, 1, 2, 1]], np.int32), kv_lens, [14, 15],
                       Hq, Hkv, D, P, theta)
    assert np.array_equal(other[0], shared[0]) and not np.allclose(other[1], shared[1])


# --------------------------------------------------------------------------------------------
# P4: closed forms for D = 2 (one frequency, f_0 = 1)
# --------------------------------------------------------------------------------------------
def test_closed_form_d2(oracle_attn):
    """One rotary pair with f = 1, query (1,0) at m, two keys at positions n: the softmax weights (read back
    through one-hot V rows) must be those of scores cos(m-n)/sqrt(D) for k=(1,0) and sin(m-n)/sqrt(D) for k=(0,1)."""
    P, m = 4, 9
    for kvec, fn in (((1.0, 0.0), math.cos), ((0.0, 1.0), math.sin)):
        positions = [2, 5]
        # D must be a multiple of the 4-element fp32 granule, so the D=2 problem sits in D=4: dim 0 pairs with
        # dim 2 (half-split), f_0 = 1; the second frequency multiplies zeros only. Keys at slots 2 and 5.
        kp2 = np.zeros((2, 1, 1, P, 4), np.float32)
        vp2 = np.zeros((2, 1, 4, P), np.float32)
        for idx, n in enumerate(positions):
            kp2[n // P, 0, 0, n % P, 0], kp2[n // P, 0, 0, n % P, 2] = kvec
            vp2[n // P, 0, idx, n % P] = 1.0
        masks = np.array([[1 << 2, 1 << 1]], np.uint32)
        q = np.zeros((1, 1, 4), np.float32)
        q[0, 0, 0] = 1.0
        got = oracle_attn.attention(q, F32, kp2, vp2, F32, np.array([[0, 1]], np.int32), [8], [m], Hq=1, Hkv=1, D=4,
                                    P=P, theta=1e4, block_valid_mask=masks)[0, 0]
        s = np.array([fn(m - n) for n in positions]) / math.sqrt(4)
        w = np.exp(s - s.max())
        w /= w.sum()
        np.testing.assert_allclose(got[:2], w, rtol=0, atol=1e-14)


def test_frequency_law(oracle_attn):
    """Second frequency of D=4 is theta^(-1/2): q=e_1, k=e_1 at distance m-n gives cos((m-n)/sqrt(theta))."""
    P, theta, m, n0, n1 = 4, 400.0, 30, 3, 1
    kp = np.zeros((1, 1, 1, P, 4), np.float32)
    vp = np.zeros((1, 1, 4, P), np.float32)
    for idx, n in enumerate((n0, n1)):
        kp[0, 0, 0, n, 1] = 1.0
        vp[0, 0, idx, n] = 1.0
    q = np.zeros((1, 1, 4), np.float32)
    q[0, 0, 1] = 1.0
    got = oracle_attn.attention(q, F32, kp, vp, F32, np.array([[0]], np.int32), [4], [m], Hq=1, Hkv=1, D=4, P=P,
                                theta=theta, block_valid_mask=np.array([[(1 << n0) | (1 << n1)]], np.uint32))[0, 0]
    s = np.array([math.cos((m - n) / 20.0) for n in (n0, n1)]) / 2.0
    w = np.exp(s - s.max())
    w /= w.sum()
    np.testing.assert_allclose(got[:2], w, rtol=0, atol=1e-14)


# --------------------------------------------------------------------------------------------
# P5: q = 0 gives uniform weights, so the output tells exactly which slots were gathered
# --------------------------------------------------------------------------------------------
def test_uniform_softmax_reveals_gather(oracle_attn):
    Hq, Hkv, D, P = 2, 2, 8, 4
    num_pages = 7
    kp = np.random.default_rng(0).standard_normal((num_pages, Hkv, D // 4, P, 4)).astype(np.float32)
    vp = np.zeros((num_pages, Hkv, D, P), np.float32)
    for p in range(num_pages):
        for h in range(Hkv):
            for s in range(P):
                vp[p, h, 0, s] = p           # dim 0: page id
                vp[p, h, 1, s] = s           # dim 1: slot
                vp[p, h, 2, s] = h           # dim 2: kv head
    tables = np.array([[5, 2, 6, 0]], np.int32)
    L = 14
    q = np.zeros((1, Hq, D), np.float32)
    got = oracle_attn.attention(q, F32, kp, vp, F32, tables, [L], [L], Hq=Hq, Hkv=Hkv, D=D, P=P, theta=1e4)[0]
    slots = [(tables[0, n // P], n % P) for n in range(L)]
    for h in range(Hq):
        assert got[h, 0] == pytest.approx(np.mean([p for p, _ in slots]), abs=1e-14)
        assert got[h, 1] == pytest.approx(np.mean([s for _, s in slots]), abs=1e-14)
        assert got[h, 2] == pytest.approx(h, abs=1e-14)          # G = 1: q head h reads kv head h
    # causal prefill: a query at position 5 sees slots 0..5 only
    got = oracle_attn.attention(q, F32, kp, vp, F32, tables, [L], [5], Hq=Hq, Hkv=Hkv, D=D, P=P, theta=1e4,
                                cu_q_lens=[0, 1])[0]
    assert got[0, 0] == pytest.approx(np.mean([p for p, _ in slots[:6]]), abs=1e-14)
    # GQA mapping: 4 q heads on 2 kv heads -> heads 0,1 read kv head 0 and heads 2,3 read kv head 1
    q4 = np.zeros((1, 4, D), np.float32)
    got = oracle_attn.attention(q4, F32, kp, vp, F32, tables, [L], [L], Hq=4, Hkv=2, D=D, P=P, theta=1e4)[0]
    assert [round(x) for x in got[:, 2]] == [0, 0, 1, 1]


# --------------------------------------------------------------------------------------------
# P6: edge cases with exact answers
# --------------------------------------------------------------------------------------------
def test_single_key_returns_its_value_and_empty_returns_zero(oracle_attn):
    Hq, Hkv, D, P = 2, 1, 8, 4
    rng = np.random.default_rng(4)
    kp = rng.standard_normal((2, Hkv, D // 4, P, 4)).astype(np.float32)
    vp = rng.standard_normal((2, Hkv, D, P)).astype(np.float32)
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    got = oracle_attn.attention(q, F32, kp, vp, F32, np.array([[1, 0]], np.int32), [1], [123], Hq=Hq, Hkv=Hkv, D=D,
                                P=P, theta=1e4)[0]
    for h in range(Hq):
        assert np.array_equal(got[h], vp[1, 0, :, 0].astype(np.float64))
    got = oracle_attn.attention(q, F32, kp, vp, F32, np.array([[1, 0]], np.int32), [0], [0], Hq=Hq, Hkv=Hkv, D=D,
                                P=P, theta=1e4)[0]
    assert np.array_equal(got, np.zeros((Hq, D)))


def test_scale_and_norm_properties(oracle_attn):
    """Rotation preserves norms: with k = c*q_dir placed so that q^.k^ depends only on |q||k| and the angle
    difference, position 0 for both leaves vectors untouched: scores = q.k/sqrt(D) exactly."""
    Hq, Hkv, D, P = 1, 1, 8, 4
    rng = np.random.default_rng(12)
    kp = rng.standard_normal((1, 1, D // 4, P, 4)).astype(np.float32)
    vp = np.zeros((1, 1, D, P), np.float32)
    for s in range(P):
        vp[0, 0, s, s] = 1.0
    q = rng.standard_normal((1, 1, D)).astype(np.float32)
    # all four keys at position 0 (block_positions = -s is impossible per block, so mask one slot at a time)
    for s in range(P):
        got = oracle_attn.attention(q, F32, kp, vp, F32, np.array([[0]], np.int32), [P], [0], Hq=1, Hkv=1, D=D, P=P,
                                    theta=1e4, block_positions=np.array([[-s]], np.int32),
                                    block_valid_mask=np.array([[1 << s]], np.uint32))[0, 0]
        assert got[s] == 1.0 and got.sum() == 1.0
    # explicit sm_scale is honoured: scale 0+ -> nearly uniform weights
    got = oracle_attn.attention(q, F32, kp, vp, F32, np.array([[0]], np.int32), [P], [9], Hq=1, Hkv=1, D=D, P=P,
                                theta=1e4, sm_scale=1e-12)[0, 0]
    np.testing.assert_allclose(got[:P], 0.25, atol=1e-10)


# --------------------------------------------------------------------------------------------
# P8: the position belongs to the request, not to the page
# --------------------------------------------------------------------------------------------
def test_permuting_blocks_with_their_positions_changes_nothing(oracle_attn):
    Hq, Hkv, D, P, theta, nb = 4, 2, 8, 4, 1000.0, 5
    rng = np.random.default_rng(21)
    kp = rng.standard_normal((nb, Hkv, D // 4, P, 4)).astype(np.float32)
    vp = rng.standard_normal((nb, Hkv, D, P)).astype(np.float32)
    q = rng.standard_normal((1, Hq, D)).astype(np.float32)
    table = np.arange(nb, dtype=np.int32)
    bp = np.arange(nb, dtype=np.int32) * P
    base = oracle_attn.attention(q, F32, kp, vp, F32, table[None], [nb * P], [nb * P], Hq=Hq, Hkv=Hkv, D=D, P=P,
                                 theta=theta, block_positions=bp[None])[0]
    perm = rng.permutation(nb)
    got = oracle_attn.attention(q, F32, kp, vp, F32, table[perm][None], [nb * P], [nb * P], Hq=Hq, Hkv=Hkv, D=D, P=P,
                                theta=theta, block_positions=bp[perm][None])[0]
    np.testing.assert_allclose(got, base, rtol=0, atol=1e-13)
    # same pages in another order WITHOUT moving their positions is a different context
    got = oracle_attn.attention(q, F32, kp, vp, F32, table[::-1].copy()[None], [nb * P], [nb * P], Hq=Hq, Hkv=Hkv,
                                D=D, P=P, theta=theta, block_positions=bp[None])[0]
    assert not np.allclose(got, base)


# --------------------------------------------------------------------------------------------
# storage decoders against a library and the format's defining values
# --------------------------------------------------------------------------------------------
def test_e4m3_decoder_matches_torch_and_format(oracle_attn):
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    want = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy().astype(np.float64)
    got = np.array([oracle_attn.decode_elem(F8, c) for c in range(256)])
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[~np.isnan(got)], want[~np.isnan(want)])
    assert oracle_attn.decode_elem(F8, 0x7E) == 448.0 and oracle_attn.decode_elem(F8, 0x01) == 2.0 ** -9
    assert oracle_attn.decode_elem(F8, 0x08) == 2.0 ** -6 and oracle_attn.decode_elem(F8, 0xB8) == -1.0
    assert math.isnan(oracle_attn.decode_elem(F8, 0x7F))


def test_bf16_decoder_matches_torch(oracle_attn):
    rng = np.random.default_rng(1)
    bits = rng.integers(0, 1 << 16, size=2000).astype(np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([oracle_attn.decode_elem(BF16, int(b)) for b in bits])
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])


def test_fp8_and_bf16_storage_equal_f32_storage_of_the_decoded_values(oracle_attn):
    """Feeding codes + scales must equal feeding the decoded, scaled fp32 values."""
    import workloads as W
    Hq, Hkv, D, P, theta = 4, 2, 32, 4, 1e4
    tables = np.array([[2, 0, 1]], np.int32)
    q = W.gen_q(3, 1, Hq, D, "bf16")
    for kvd in (BF16, F8):
        pages = W.gen_pages(3, 3, Hkv, P, D, kvd)
        kl = W.unpack_k(pages.k).to(torch.float32)
        vl = W.unpack_v(pages.v).to(torch.float32)
        if kvd == F8:
            kl = kl * pages.k_scales.view(-1, 1, 1, 1)
            vl = vl * pages.v_scales.view(-1, 1, 1, 1)
        ref = oracle_attn.attention(q.to(torch.float32).numpy(), F32, W.pack_k(kl, F32).numpy(), W.pack_v(vl).numpy(),
                                    F32, tables, [11], [10], Hq=Hq, Hkv=Hkv, D=D, P=P, theta=theta)
        got = oracle_attn.attention(W.raw_numpy(q), BF16, W.raw_numpy(pages.k), W.raw_numpy(pages.v), kvd, tables,
                                    [11], [10], Hq=Hq, Hkv=Hkv, D=D, P=P, theta=theta,
                                    k_scales=W.raw_numpy(pages.k_scales), v_scales=W.raw_numpy(pages.v_scales))
        np.testing.assert_allclose(got, ref, rtol=0, atol=1e-6 if kvd == F8 else 0)


def test_bad_page_id_is_an_error(oracle_attn):
    kp = np.zeros((2, 1, 2, 4, 4), np.float32)
    vp = np.zeros((2, 1, 8, 4), np.float32)
    q = np.zeros((1, 1, 8), np.float32)
    with pytest.raises(ValueError):
        oracle_attn.attention(q, F32, kp, vp, F32, np.array([[2]], np.int32), [3], [3], Hq=1, Hkv=1, D=8, P=4, theta=1e4)
