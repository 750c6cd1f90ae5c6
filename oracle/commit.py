"""CPU oracle for the commit step (§3.3.2 "Commit to Paged KV") — TEST INFRASTRUCTURE ONLY.

Freshly computed, un-rotated K and V of new tokens are written straight into the pages the scheduling
path assigned: no indirection beyond the request's block table, no positional encoding (pages stay
position-free for §3.3.3). This file is that definition written out with numpy: one token at a time, one
index formula per tensor, no blocking or fusion.

Storage representation (numpy): fp32 pages are float32 arrays, bf16 pages are uint16 bit patterns, fp8
pages are uint8 e4m3fn codes; all flat, in the page layout of the library's header:
    K element (page p, head h, slot s, dim d) at (((p*Hkv + h)*(D/X) + d//X)*P + s)*X + d%X, X = 16 // bytes
    V element (page p, head h, slot s, dim d) at ((p*Hkv + h)*D + d)*P + s

fp8 quantisation (a reading: the paper names no low-precision format): the caller supplies the page's
scale; code = e4m3fn value nearest to fp32(x) / fp32(scale) (the quotient rounded once to fp32, which is
the precision the kernel divides in), ties to the even code, magnitudes beyond 448 saturate to 448, the
sign of the quotient is kept (also for zero). `encode_e4m3` is that definition as a search over the 127
finite magnitudes; it is pinned against the format's printed values and a library cast in the tests.
"""
from __future__ import annotations

import numpy as np

_BYTES = {"f32": 4, "bf16": 2, "f8e4m3": 1}


def e4m3_magnitudes() -> np.ndarray:
    """Values of the codes 0x00..0x7E of OCP e4m3fn (bias 7, subnormals at exponent field 0, 0x7F = NaN)."""
    vals = []
    for code in range(0x7F):
        e, m = code >> 3, code & 7
        vals.append(m * 2.0 ** -9 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7))
    return np.array(vals, dtype=np.float64)


def encode_e4m3(y: np.ndarray) -> np.ndarray:
    """Nearest e4m3fn code of each fp32 value, ties to the even code, saturating; sign bit = sign of y."""
    y = np.asarray(y, dtype=np.float32)
    mags = e4m3_magnitudes()
    a = np.abs(y.astype(np.float64))
    hi = np.searchsorted(mags, a, side="left")           # first code whose value >= a
    hi = np.minimum(hi, len(mags) - 1)
    lo = np.maximum(hi - 1, 0)
    d_lo, d_hi = a - mags[lo], mags[hi] - a              # exact in fp64: fp32 inputs, 4-bit table values
    pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    code = np.where(a >= mags[-1], len(mags) - 1, np.where(pick_hi, hi, lo)).astype(np.uint8)
    return code | (np.signbit(y).astype(np.uint8) << 7)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def kv_commit(k_pages: np.ndarray, v_pages: np.ndarray, k_scales, v_scales, k_new: np.ndarray,
              v_new: np.ndarray, block_tables: np.ndarray, run_request, run_first_slot, cu_run_tokens,
              *, Hkv: int, D: int, P: int, kv_dtype: str) -> None:
    """Write the new tokens' K/V into the pages, in place.

    k_new / v_new: [n_tokens][Hkv][D] in the model's dtype (float32 for fp32 pages, bf16 bit patterns as
    uint16 for bf16 and fp8 pages). Run r holds tokens cu_run_tokens[r] .. cu_run_tokens[r+1]; they go to the
    consecutive logical slots run_first_slot[r] .. of request run_request[r]; logical slot n lives in page
    block_tables[request][n // P] at slot n % P. Slots not named by any run keep their contents.
    """
    X = 16 // _BYTES[kv_dtype]
    d = np.arange(D)
    h = np.arange(Hkv)[:, None]
    for r in range(len(run_request)):
        req, first = int(run_request[r]), int(run_first_slot[r])
        for i, t in enumerate(range(int(cu_run_tokens[r]), int(cu_run_tokens[r + 1]))):
            n = first + i
            p, s = int(block_tables[req, n // P]), n % P
            k_idx = (((p * Hkv + h) * (D // X) + d // X) * P + s) * X + d % X      # [Hkv][D]
            v_idx = ((p * Hkv + h) * D + d) * P + s
            if kv_dtype == "f8e4m3":
                with np.errstate(over="ignore"):             # a quotient beyond fp32 becomes inf and saturates
                    k_pages[k_idx] = encode_e4m3(bf16_bits_to_f32(k_new[t]) / np.float32(k_scales[p]))
                    v_pages[v_idx] = encode_e4m3(bf16_bits_to_f32(v_new[t]) / np.float32(v_scales[p]))
            else:                                                                   # same dtype: a copy
                k_pages[k_idx] = k_new[t]
                v_pages[v_idx] = v_new[t]
