"""Pins of the commit-step oracle (oracle/commit.py; §3.3.2) against facts it does not compute itself:
the e4m3fn format's printed values, a library cast, the page generator's own packing, and invariants."""
import numpy as np
import pytest
import torch

import workloads as W
from oracle import commit as OC


# ---- fp8 encoder -------------------------------------------------------------------------------
def test_e4m3_table_values_of_the_format():
    m = OC.e4m3_magnitudes()
    assert len(m) == 127 and m[0] == 0.0
    assert m[1] == 2.0 ** -9 and m[7] == 7 * 2.0 ** -9            # subnormals
    assert m[8] == 2.0 ** -6                                       # smallest normal
    assert m[0x38] == 1.0 and m[0x39] == 1.125 and m[0x40] == 2.0
    assert m[0x7E] == 448.0                                        # largest finite
    assert np.all(np.diff(m) > 0)


def test_encode_exact_ties_saturation_and_sign():
    enc = lambda *v: OC.encode_e4m3(np.array(v, dtype=np.float32)).tolist()
    assert enc(0.0, 1.0, 448.0, 2.0 ** -9) == [0x00, 0x38, 0x7E, 0x01]
    assert enc(-1.0, -448.0, -0.0) == [0xB8, 0xFE, 0x80]
    # midpoints go to the even code: 1.0625 between 0x38 / 0x39, 1.1875 between 0x39 / 0x3A
    assert enc(1.0625, 1.1875, -1.0625) == [0x38, 0x3A, 0xB8]
    assert enc(np.nextafter(np.float32(1.0625), np.float32(2)), np.nextafter(np.float32(1.0625), np.float32(0))) == [0x39, 0x38]
    # half the smallest subnormal is a tie with zero (even); just above it rounds up
    assert enc(2.0 ** -10, 2.0 ** -10 * 1.0001, 3 * 2.0 ** -10) == [0x00, 0x01, 0x02]
    # saturation instead of NaN
    assert enc(449.0, 464.0, 1e9, -1e9, np.inf) == [0x7E, 0x7E, 0x7E, 0xFE, 0x7E]


def test_encode_roundtrips_every_code_and_matches_library_cast():
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)
    vals = torch.from_numpy(codes).view(torch.float8_e4m3fn).float().numpy()
    assert np.array_equal(OC.encode_e4m3(vals), codes)
    rng = np.random.default_rng(5)
    y = np.concatenate([rng.standard_normal(200000).astype(np.float32) * s for s in (1e-3, 0.05, 1.0, 30.0, 150.0)])
    mags = OC.e4m3_magnitudes()
    mids = ((mags[1:] + mags[:-1]) / 2).astype(np.float32)        # every tie, exactly representable in fp32
    y = np.concatenate([y, mids, -mids])
    y = y[np.abs(y) <= 448.0]
    lib = torch.from_numpy(y).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(OC.encode_e4m3(y), lib)


# ---- the scatter -------------------------------------------------------------------------------
def _flat(pages: W.KVPages):
    view = {"f32": torch.float32, "bf16": torch.uint16, "f8e4m3": torch.uint8}[pages.kv_dtype]
    k = pages.k.view(view).numpy().reshape(-1).copy()
    v = pages.v.view(view).numpy().reshape(-1).copy()
    ks = None if pages.k_scales is None else pages.k_scales.numpy()
    vs = None if pages.v_scales is None else pages.v_scales.numpy()
    return k, v, ks, vs


def _source_rows(pages: W.KVPages, page_slot):
    """Values the model would hand to the commit step so that the page content is reproduced: the stored
    value itself (fp8: code * scale rounded to bf16 would not round-trip, so fp8 sources are drawn fresh)."""
    kl, vl = W.unpack_k(pages.k), W.unpack_v(pages.v)              # [N, Hkv, P, D], the generator's own unpacking
    k = torch.stack([kl[p, :, s, :] for p, s in page_slot])
    v = torch.stack([vl[p, :, s, :] for p, s in page_slot])
    view = {"f32": torch.float32, "bf16": torch.uint16}[pages.kv_dtype]
    return k.view(view).numpy(), v.view(view).numpy()


@pytest.mark.parametrize("kv_dtype,P", [("f32", 16), ("bf16", 16), ("bf16", 32)])
def test_commit_reproduces_pages_packed_by_the_generator(kv_dtype, P):
    Hkv, D, N = 3, 64, 12
    pages = W.gen_pages(11, N, Hkv, P, D, kv_dtype)
    k0, v0, _, _ = _flat(pages)
    bt = np.array([[5, 2, 9, 0], [7, 1, 3, 11]], dtype=np.int32)
    runs = [(0, 3, 2 * P + 5), (1, P - 1, 2), (1, 2 * P, P), (0, 3 * P + 1, 0)]     # (request, first slot, tokens)
    page_slot = [(int(bt[r, n // P]), n % P) for r, f, c in runs for n in range(f, f + c)]
    k_new, v_new = _source_rows(pages, page_slot)
    cu = np.cumsum([0] + [c for _, _, c in runs])
    k, v = k0.copy(), v0.copy()
    # wipe the destination slots, then commit: every byte must come back, and nothing else may change
    wipe_k, wipe_v = k0.copy(), v0.copy()
    OC.kv_commit(wipe_k, wipe_v, None, None, np.zeros_like(k_new), np.zeros_like(v_new), bt,
                 [r for r, _, _ in runs], [f for _, f, _ in runs], cu, Hkv=Hkv, D=D, P=P, kv_dtype=kv_dtype)
    assert not np.array_equal(wipe_k.view(np.uint8), k0.view(np.uint8))
    n_changed = int((wipe_k.view(np.uint8).reshape(-1, k0.itemsize) != k0.view(np.uint8).reshape(-1, k0.itemsize)).any(1).sum())
    assert n_changed <= len(page_slot) * Hkv * D
    k, v = wipe_k.copy(), wipe_v.copy()
    OC.kv_commit(k, v, None, None, k_new, v_new, bt, [r for r, _, _ in runs], [f for _, f, _ in runs], cu,
                 Hkv=Hkv, D=D, P=P, kv_dtype=kv_dtype)
    assert np.array_equal(k.view(np.uint8), k0.view(np.uint8)) and np.array_equal(v.view(np.uint8), v0.view(np.uint8))


def test_commit_fp8_codes_dequantise_to_nearest_and_keep_other_slots():
    Hkv, D, P, N = 2, 128, 32, 6
    pages = W.gen_pages(12, N, Hkv, P, D, "f8e4m3")
    k0, v0, ks, vs = _flat(pages)
    bt = np.array([[4, 1, 3]], dtype=np.int32)
    first, count = 20, 50
    rng = np.random.default_rng(3)
    src = lambda: torch.from_numpy(rng.standard_normal((count, Hkv, D)).astype(np.float32) * 2).to(torch.bfloat16)
    kn, vn = src(), src()
    k, v = k0.copy(), v0.copy()
    OC.kv_commit(k, v, ks, vs, kn.view(torch.uint16).numpy(), vn.view(torch.uint16).numpy(), bt, [0], [first], [0, count],
                 Hkv=Hkv, D=D, P=P, kv_dtype="f8e4m3")
    kl = W.unpack_k(torch.from_numpy(k).view(torch.float8_e4m3fn).reshape(pages.k.shape))   # [N, Hkv, P, D]
    vl = W.unpack_v(torch.from_numpy(v).view(torch.float8_e4m3fn).reshape(pages.v.shape))
    kl0, vl0 = W.unpack_k(pages.k), W.unpack_v(pages.v)
    touched = np.zeros((N, P), dtype=bool)
    grid = OC.e4m3_magnitudes()
    for i in range(count):
        n = first + i
        p, s = int(bt[0, n // P]), n % P
        touched[p, s] = True
        for got, want, sc in ((kl[p, :, s, :], kn[i], ks[p]), (vl[p, :, s, :], vn[i], vs[p])):
            y = np.clip(want.float().numpy().astype(np.float64) / float(sc), -448, 448)
            err = np.abs(got.float().numpy().astype(np.float64) - y)
            best = np.abs(np.abs(y)[..., None] - grid).min(-1)
            assert np.all(err <= best + 2e-7 * np.abs(y) + 1e-12)   # as close as any code (fp32 quotient rounding aside)
    same = ~torch.from_numpy(touched)
    by_slot = lambda t: t.view(torch.uint8).permute(0, 2, 1, 3)                    # [N, P, Hkv, D]
    assert torch.equal(by_slot(kl)[same], by_slot(kl0)[same])
    assert torch.equal(by_slot(vl)[same], by_slot(vl0)[same])
    assert not torch.equal(by_slot(kl)[~same], by_slot(kl0)[~same])


def test_commit_in_pieces_equals_commit_at_once():
    Hkv, D, P, N = 2, 64, 16, 8
    pages = W.gen_pages(13, N, Hkv, P, D, "bf16")
    k0, v0, _, _ = _flat(pages)
    bt = np.array([[6, 0, 2, 5]], dtype=np.int32)
    rng = np.random.default_rng(4)
    kn = rng.integers(0, 0x7F00, size=(40, Hkv, D), dtype=np.uint16)
    vn = rng.integers(0, 0x7F00, size=(40, Hkv, D), dtype=np.uint16)
    a_k, a_v = k0.copy(), v0.copy()
    OC.kv_commit(a_k, a_v, None, None, kn, vn, bt, [0], [9], [0, 40], Hkv=Hkv, D=D, P=P, kv_dtype="bf16")
    b_k, b_v = k0.copy(), v0.copy()
    OC.kv_commit(b_k, b_v, None, None, kn, vn, bt, [0, 0, 0], [9, 9 + 7, 9 + 7 + 20], [0, 7, 27, 40],
                 Hkv=Hkv, D=D, P=P, kv_dtype="bf16")
    assert np.array_equal(a_k, b_k) and np.array_equal(a_v, b_v)
