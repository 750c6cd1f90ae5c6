"""The decode entry point that allocates nothing (mepic_attn_decode_noalloc: split-K partials in a fixed array
inside the library's device image) against the existing entry point (caller's workspace), through the C-ABI:
two calls in a row, the second on a smaller input, so that whatever the first call left in the shared array is
there when the second runs. Same kernels, so the outputs must be identical bit for bit; the existing entry
point's output is also held to the oracle's tolerance."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as W
from harness import DeviceCase, align_with_oracle, oracle_out

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2, "f8e4m3": 2e-2}


def _case(name, seed, **kw):
    st = W.decode_structure(name, seed, **kw)
    aligned, _ = align_with_oracle(st)
    return W.assemble(st, aligned)


def _both(M, oracle_attn, case, rows=None):
    dc = DeviceCase(M, case)
    want_dev = dc.run()                       # existing entry point, caller's workspace
    kernel = M.last_kernel()
    got = dc.run_noalloc()                    # fixed array inside the library
    assert M.last_kernel() == kernel
    assert np.isfinite(got).all()
    assert np.array_equal(got, want_dev), f"no-alloc entry point differs from mepic_attn_decode ({kernel})"
    want = oracle_out(oracle_attn, case, rows=rows)
    sel = got if rows is None else np.stack([got[t, h] for t, h in rows])
    err = float(np.abs(sel - want).max())
    assert err <= TOL[case.st.kv_dtype], err
    return kernel


def test_noalloc_matches_workspace_entry_point_twice_second_smaller(mepic, oracle_attn):
    big = _case("noalloc_big_bf16", 31, B=24, Hq=32, Hkv=8, D=128, P=16, theta=5e5, q_dtype="bf16", kv_dtype="bf16",
                prefix=64, n_chunks=(2, 6), chunk_tokens=512, pool=6, question=77)
    small = _case("noalloc_small_bf16", 32, B=3, Hq=32, Hkv=8, D=128, P=16, theta=5e5, q_dtype="bf16",
                  kv_dtype="bf16", prefix=16, n_chunks=(1, 2), chunk_tokens=160, pool=3, question=21)
    rng = np.random.default_rng(5)
    rows = sorted({(int(rng.integers(big.n_q)), int(rng.integers(32))) for _ in range(96)})
    assert _both(mepic, oracle_attn, big, rows=rows) == "decode_mfma_bf16"
    assert _both(mepic, oracle_attn, small) == "decode_mfma_bf16"


def test_noalloc_other_kernels_back_to_back(mepic, oracle_attn):
    """fp8 pages (matrix-core kernel) and then the tiny fp32 configuration (general kernel), which shares the array."""
    fp8 = _case("noalloc_fp8", 33, B=9, Hq=28, Hkv=4, D=128, P=32, theta=1e6, q_dtype="bf16", kv_dtype="f8e4m3",
                prefix=0, n_chunks=(2, 5), chunk_tokens=512, pool=5, question=0)
    assert _both(mepic, oracle_attn, fp8) == "decode_mfma_fp8"
    st = W.config(1)
    aligned, _ = align_with_oracle(st)
    assert _both(mepic, oracle_attn, W.assemble(st, aligned)) == "general"


def test_noalloc_rejects_what_does_not_fit(mepic):
    """Shapes whose partials exceed the fixed array: MEPIC_ERR_CAPACITY from the host check, nothing launched."""
    p = mepic.AttnParams()
    p.B = p.n_q_tokens = 4096
    p.Hq, p.Hkv, p.D, p.P, p.max_blocks, p.num_pages = 64, 8, 128, 16, 4096, 1 << 20
    p.max_kv_len = 65536
    p.q_dtype = p.kv_dtype = mepic.BF16
    p.rope_theta = 5e5
    assert mepic.attn_workspace_size(p, False) > mepic.NOALLOC_SCRATCH_BYTES
    rc = mepic.load().mepic_attn_decode_noalloc(ctypes.byref(p), None)
    assert rc == mepic.ERR_CAPACITY
