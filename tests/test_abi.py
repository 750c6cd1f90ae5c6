"""The C-ABI library loads, exports every symbol include/mepic.h declares, and rejects bad arguments on
the host before anything is launched (so these run without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mepic.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mepic_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(mepic):
    lib = mepic.load()
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), f"{n} declared in mepic.h but not exported"
    assert sorted(mepic.EXPORTS) == names, "the binding's list and the header disagree"
    assert mepic.version() >= 100
    assert mepic.strerror(0) == "ok" and "reject" in mepic.strerror(mepic.ERR_NOMEM).lower()
    assert mepic.last_kernel() == "" or isinstance(mepic.last_kernel(), str)


def test_every_entry_point_with_arguments_declares_their_types(mepic):
    """ctypes passes an undeclared Python int as a 32-bit C int: a device pointer handed to an entry point whose
    argument types the binding forgot to declare would arrive truncated. Every export that takes arguments must
    declare them, and the declaration must have as many entries as the header's parameter list."""
    lib = mepic.load()
    text = open(os.path.join(ROOT, "include", "mepic.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    for name in mepic.EXPORTS:
        m = re.search(r"\b" + name + r"\s*\(([^;]*?)\)\s*;", text, flags=re.S)
        assert m, name
        params = m.group(1).strip()
        n_params = 0 if params in ("", "void") else params.count(",") + 1
        fn = getattr(lib, name)
        if n_params == 0:
            continue
        assert fn.argtypes is not None, f"{name}: argument types not declared in the binding"
        assert len(fn.argtypes) == n_params, f"{name}: {len(fn.argtypes)} declared, {n_params} in the header"


def test_probe_argument_errors_are_rejected_before_any_launch(mepic):
    lib = mepic.load()
    assert lib.mepic_probe_tile_stream(3, 10, ctypes.c_void_p(0x1000), 65536, None) == mepic.ERR_INVALID
    assert lib.mepic_probe_tile_stream(0, 10, None, 65536, None) == mepic.ERR_INVALID
    assert lib.mepic_probe_tile_stream(0, 10, ctypes.c_void_p(0x1000), 1024, None) == mepic.ERR_INVALID
    assert lib.mepic_probe_tile_stream(0, -1, ctypes.c_void_p(0x1000), 65536, None) == mepic.ERR_INVALID
    assert lib.mepic_probe_mfma_bf16(-1, 0, ctypes.c_void_p(0x1000), ctypes.byref(ctypes.c_double()), None) == mepic.ERR_INVALID
    assert lib.mepic_device_counter_khz(None) == mepic.ERR_INVALID


def test_product_does_not_import_the_oracle():
    """The product path may not route through the oracle or any CPU fallback."""
    pkg = os.path.join(ROOT, "paper_2512_16822_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("not import the oracle", ""), f"{f} mentions the oracle"


def params(mepic, **over):
    p = mepic.AttnParams()
    base = dict(B=2, n_q_tokens=2, Hq=8, Hkv=2, D=128, P=16, max_blocks=4, num_pages=8, q_dtype=mepic.BF16,
                kv_dtype=mepic.BF16, rope_theta=1e4)
    base.update(over)
    for k, v in base.items():
        setattr(p, k, v)
    return p


def test_workspace_size_and_shape_errors(mepic):
    n = mepic.attn_workspace_size(params(mepic), False)
    assert n > 0 and n % 4 == 0
    for bad, status in ((dict(D=96), mepic.ERR_UNSUPPORTED), (dict(P=8), mepic.ERR_UNSUPPORTED),
                        (dict(Hq=7), mepic.ERR_INVALID), (dict(q_dtype=mepic.F32), mepic.ERR_UNSUPPORTED),
                        (dict(kv_dtype=mepic.F32), mepic.ERR_UNSUPPORTED), (dict(Hq=68, Hkv=2), mepic.ERR_UNSUPPORTED),
                        (dict(n_q_tokens=3), mepic.ERR_INVALID)):
        with pytest.raises(mepic.MepicError) as e:
            mepic.attn_workspace_size(params(mepic, **bad), False)
        assert e.value.status == status, bad
    # prefill may have more query tokens than requests
    # matrix-core prefill: the rotary table the call builds, 32 entries of 16 bytes per position, whole tiles of 64
    assert mepic.attn_workspace_size(params(mepic, n_q_tokens=40), True) == 64 * 16 * 16 + 16
    assert mepic.attn_workspace_size(params(mepic, n_q_tokens=40, flags=mepic.FLAG_FORCE_GENERAL), True) > 0


def test_null_pointers_are_rejected_before_any_launch(mepic):
    lib = mepic.load()
    p = params(mepic)
    assert lib.mepic_attn_decode(ctypes.byref(p), None) == mepic.ERR_INVALID       # q, out, pages ... are NULL
    assert lib.mepic_attn_decode(None, None) == mepic.ERR_INVALID
    assert lib.mepic_attn_workspace_size(ctypes.byref(p), 0, None) == mepic.ERR_INVALID
    assert lib.mepic_pool_create(4, 16, None) == mepic.ERR_INVALID
    assert lib.mepic_pool_get_stats(None, None) == mepic.ERR_INVALID


def test_commit_shape_errors_are_rejected_before_any_launch(mepic):
    lib = mepic.load()

    def cp(**over):
        p = mepic.CommitParams()
        base = dict(B=1, n_runs=1, n_tokens=4, Hkv=2, D=128, P=16, max_blocks=2, num_pages=4,
                    src_dtype=mepic.BF16, kv_dtype=mepic.BF16)
        base.update(over)
        for k, v in base.items():
            setattr(p, k, v)
        return p
    for bad, status in ((dict(D=96), mepic.ERR_UNSUPPORTED), (dict(P=8), mepic.ERR_UNSUPPORTED),
                        (dict(src_dtype=mepic.F32), mepic.ERR_UNSUPPORTED),
                        (dict(src_dtype=mepic.F8E4M3, kv_dtype=mepic.F8E4M3), mepic.ERR_UNSUPPORTED),
                        (dict(n_tokens=-1), mepic.ERR_INVALID), (dict(Hkv=0), mepic.ERR_INVALID),
                        (dict(), mepic.ERR_INVALID)):               # all pointers null
        assert lib.mepic_kv_commit(ctypes.byref(cp(**bad)), None) == status, bad
    assert lib.mepic_kv_commit(ctypes.byref(cp(n_tokens=0)), None) == mepic.OK     # nothing to do: ok without pointers
    assert lib.mepic_kv_commit(None, None) == mepic.ERR_INVALID


def test_batched_decode_argument_errors_are_rejected_before_any_launch(mepic):
    import numpy as np
    lib = mepic.load()
    bt = np.tile(np.arange(4, dtype=np.int32), (2, 1))
    kv = np.array([64, 40], dtype=np.int32)
    plan, info = mepic.decode_plan_build(bt, kv, 16, 8, 2, mepic.BF16)
    p = params(mepic)
    need = mepic.attn_decode_batched_workspace_size(p, info)
    assert need == p.n_q_tokens * p.Hq * info.n_splits * (p.D + 2) * 4

    def status(pp, ii, plan_ptr=None):
        return lib.mepic_attn_decode_batched(ctypes.byref(pp), plan_ptr, ctypes.byref(ii), None)

    def changed(**over):
        i2 = mepic.DecodePlanInfo()
        ctypes.memmove(ctypes.byref(i2), ctypes.byref(info), ctypes.sizeof(info))
        for k, v in over.items():
            setattr(i2, k, v)
        return i2
    assert status(p, info) == mepic.ERR_INVALID                                   # plan, q, out, pages ... are NULL
    assert status(params(mepic, B=3, n_q_tokens=3), info) == mepic.ERR_INVALID    # a plan for another batch
    assert status(params(mepic, Hq=4), info) == mepic.ERR_INVALID                 # ... for another group size
    assert status(p, changed(n_waves=info.n_waves + 1)) == mepic.ERR_INVALID      # ... cut for another device
    assert status(p, changed(n_runs=1 << 20)) == mepic.ERR_UNSUPPORTED            # run prefix sums would not fit in LDS
    assert status(params(mepic, kv_dtype=mepic.F8E4M3, P=16), info) == mepic.ERR_UNSUPPORTED
    assert status(params(mepic, D=64), info) == mepic.ERR_UNSUPPORTED
    assert status(params(mepic, flags=mepic.FLAG_FORCE_GENERAL), info) == mepic.ERR_UNSUPPORTED
    assert lib.mepic_attn_decode_batched(ctypes.byref(p), None, None, None) == mepic.ERR_INVALID
    # the planner's own checks
    cap = ctypes.c_size_t()
    assert lib.mepic_decode_plan_capacity(2, 4, 8, ctypes.byref(cap)) == mepic.ERR_INVALID      # page size
    assert lib.mepic_decode_plan_capacity(2, 4, 16, None) == mepic.ERR_INVALID
    out = np.empty(64, dtype=np.int32)
    i3 = mepic.DecodePlanInfo()
    args = (bt.ctypes.data, kv.ctypes.data, 2, 4, 16, 8, 2, mepic.BF16, out.ctypes.data)
    assert lib.mepic_decode_plan_build(*args, ctypes.c_size_t(out.size), ctypes.byref(i3)) == mepic.ERR_CAPACITY
    assert lib.mepic_decode_plan_build(*args, ctypes.c_size_t(out.size), None) == mepic.ERR_INVALID
    assert lib.mepic_decode_plan_build(bt.ctypes.data, kv.ctypes.data, 2, 4, 16, 34, 2, mepic.BF16, out.ctypes.data,
                                       ctypes.c_size_t(out.size), ctypes.byref(i3)) == mepic.ERR_UNSUPPORTED  # G = 17
