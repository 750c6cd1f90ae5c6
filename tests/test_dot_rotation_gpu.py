"""Guard for the hand-scheduled dot-product block with which the bf16 decode kernel rotates K: the block alone
(mepic_selftest_dot_rotation, through the C-ABI) against the two-term sums computed here in fp64 from the same
bf16 bit patterns. The block's correctness rests on instruction-hazard rules the compiler does not check, so this
test is what fails if a toolchain starts to schedule around it differently."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def bf16_val(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16 values in any int array) -> float64, exactly."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float -> nearest bf16 bit pattern (ties to even), as uint32 in [0, 65535]."""
    u = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint32)


def pack(lo_bits, hi_bits):
    return (lo_bits.astype(np.uint32) | (hi_bits.astype(np.uint32) << 16)).astype(np.uint32)


def make_words(rng, n):
    """[n, 12] uint32: e0..e3 = (low, high) element words, then (cos, -sin), (sin, cos) words of each pair."""
    kinds = rng.integers(0, 6, size=(n, 4))
    # element bit patterns: finite only (exponent field < 0xFF), magnitudes capped so that sums stay finite
    exp = rng.integers(1, 0xBE, size=(n, 4, 2))                   # up to ~2^62
    bits = (rng.integers(0, 2, size=(n, 4, 2)) << 15) | (exp << 7) | rng.integers(0, 128, size=(n, 4, 2))
    bits = np.where(kinds[..., None] == 0, rng.integers(0, 2, size=(n, 4, 2)) << 15, bits)            # signed zeros
    bits = np.where(kinds[..., None] == 1, (rng.integers(0, 2, size=(n, 4, 2)) << 15) | rng.integers(1, 128, size=(n, 4, 2)),
                    bits)                                                                              # denormals
    bits = np.where(kinds[..., None] == 2, (rng.integers(0, 2, size=(n, 4, 2)) << 15) | (0x7F << 7)
                    | rng.integers(0, 128, size=(n, 4, 2)), bits)                                      # magnitudes in [1, 2)
    # kinds 3-5: anything finite in range
    ang = rng.uniform(0, 2 * np.pi, size=(n, 4))
    ang = np.where(rng.random((n, 4)) < 0.1, rng.integers(0, 8, size=(n, 4)) * (np.pi / 4), ang)      # axes and diagonals
    c, s = to_bf16_bits(np.cos(ang)), to_bf16_bits(np.sin(ang))
    ms = s ^ 0x8000
    words = np.empty((n, 12), dtype=np.uint32)
    words[:, 0:4] = pack(bits[..., 0], bits[..., 1])
    words[:, 4::2] = pack(c, ms)                                  # (cos, -sin)
    words[:, 5::2] = pack(s, c)                                   # (sin, cos)
    return words


def expected(words):
    lo, hi = bf16_val(words[:, 0:4] & 0xFFFF), bf16_val(words[:, 0:4] >> 16)
    ca, cb = words[:, 4::2], words[:, 5::2]
    t = [lo * bf16_val(ca & 0xFFFF), hi * bf16_val(ca >> 16), lo * bf16_val(cb & 0xFFFF), hi * bf16_val(cb >> 16)]
    want = np.concatenate([t[0] + t[1], t[2] + t[3]], axis=1)
    size = np.concatenate([np.abs(t[0]) + np.abs(t[1]), np.abs(t[2]) + np.abs(t[3])], axis=1)
    return want, size


@pytest.mark.parametrize("seed", [0, 1])
def test_dot_rotation_block_matches_exact_two_term_sums(mepic, seed):
    rng = np.random.default_rng(seed)
    n = 200_000
    words = make_words(rng, n)
    dev = torch.device("cuda:0")
    w = torch.from_numpy(words.view(np.int32)).to(dev)
    out = torch.full((n, 8), float("nan"), dtype=torch.float32, device=dev)
    mepic.selftest_dot_rotation(w, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want, size = expected(words)
    assert np.isfinite(got).all()
    # fp32 accumulation of two exactly representable products: a few units in the last place of the larger term;
    # products of denormal elements with |constant| <= 1 may be flushed to zero (they are below 1.2e-38)
    tol = size * 2.0 ** -22 + 1.2e-38
    bad = np.abs(got - want) > tol
    assert not bad.any(), (int(bad.sum()), words[np.argwhere(bad)[0][0]], got[bad][:4], want[bad][:4])


def test_dot_rotation_block_identities(mepic):
    """Rotation by 0 and by a quarter turn on elements whose results are exact."""
    one, zero, mone = 0x3F80, 0x0000, 0xBF80
    rows = []
    for lo, hi in ((0x4000, 0x4040), (0xC2F7, 0x3DCD), (0x0000, 0x7F7F), (0x8000, 0x0080)):   # (2, 3), (-123.5, 0.1), ...
        e = (lo | (hi << 16))
        rows.append([e] * 4 + [one | (zero << 16), zero | (one << 16)] * 2                     # angle 0: (1, -0), (0, 1)
                    + [zero | (mone << 16), one | (zero << 16)] * 2)                           # quarter turn: (0, -1), (1, 0)
    words = np.array(rows, dtype=np.uint32)
    dev = torch.device("cuda:0")
    out = torch.zeros((len(rows), 8), dtype=torch.float32, device=dev)
    mepic.selftest_dot_rotation(torch.from_numpy(words.view(np.int32)).to(dev), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    lo = bf16_val(words[:, 0] & 0xFFFF).astype(np.float32)
    hi = bf16_val(words[:, 0] >> 16).astype(np.float32)
    for i in range(len(rows)):
        assert got[i, 0] == lo[i] and got[i, 1] == lo[i] and got[i, 4] == hi[i] and got[i, 5] == hi[i]      # identity
        assert got[i, 2] == -hi[i] and got[i, 3] == -hi[i] and got[i, 6] == lo[i] and got[i, 7] == lo[i]    # quarter turn
