"""ctypes front end of the fp64 C oracle (mepic_oracle.c) — test infrastructure only.

`build()` compiles the C file with gcc; `attention(...)` marshals numpy arrays and returns the fp64
output rows. No arithmetic of the method happens in this file.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mepic_oracle.c")
_LIB = os.path.join(_HERE, "libmepic_oracle.so")
_DT = {"f32": 0, "bf16": 1, "f8e4m3": 2}
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle (gcc, -O2, OpenMP). Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_attn.restype = ctypes.c_int
        _lib.oracle_decode_elem.restype = ctypes.c_double
        _lib.oracle_decode_elem.argtypes = [ctypes.c_int, ctypes.c_uint32]
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def decode_elem(dtype: str, bits: int) -> float:
    return float(_load().oracle_decode_elem(_DT[dtype], bits))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def attention(q: np.ndarray, q_dtype: str, k_pages: np.ndarray, v_pages: np.ndarray, kv_dtype: str,
              block_tables, kv_lens, q_positions, *, Hq: int, Hkv: int, D: int, P: int, theta: float,
              cu_q_lens=None, k_scales=None, v_scales=None, block_positions=None, block_valid_mask=None,
              sm_scale: float = 0.0, interleaved: bool = False, rows=None) -> np.ndarray:
    """Run the C oracle.

    q, k_pages, v_pages are arrays of storage words (float32, or uint16 for bf16, or uint8 for e4m3) in
    the layouts of the C-ABI header. Returns float64 [n_q, Hq, D], or [len(rows), D] when `rows`
    (a list of (token, head) pairs) is given."""
    lib = _load()
    q = np.ascontiguousarray(q)
    k_pages = np.ascontiguousarray(k_pages)
    v_pages = np.ascontiguousarray(v_pages)
    bt = _i32(block_tables)
    B, max_blocks = bt.shape
    kv_lens = _i32(kv_lens)
    q_positions = _i32(q_positions)
    n_q = q_positions.shape[0]
    cu = _i32(cu_q_lens)
    bp = _i32(block_positions)
    bm = None if block_valid_mask is None else np.ascontiguousarray(block_valid_mask, dtype=np.uint32)
    ks = None if k_scales is None else np.ascontiguousarray(k_scales, dtype=np.float32)
    vs = None if v_scales is None else np.ascontiguousarray(v_scales, dtype=np.float32)
    num_pages = k_pages.shape[0]
    if rows is None:
        r, n_rows = None, 0
        out = np.zeros((n_q, Hq, D), dtype=np.float64)
    else:
        r = _i32(rows).reshape(-1, 2)
        n_rows = r.shape[0]
        out = np.zeros((n_rows, D), dtype=np.float64)
    rc = lib.oracle_attn(_ptr(q), _DT[q_dtype], _ptr(k_pages), _ptr(v_pages), _DT[kv_dtype], _ptr(ks), _ptr(vs),
                         _ptr(bt), _ptr(kv_lens), _ptr(q_positions), _ptr(cu), _ptr(bp), _ptr(bm),
                         ctypes.c_int(B), ctypes.c_int(n_q), ctypes.c_int(Hq), ctypes.c_int(Hkv),
                         ctypes.c_int(D), ctypes.c_int(P), ctypes.c_int(max_blocks), ctypes.c_int(num_pages),
                         ctypes.c_double(theta), ctypes.c_double(sm_scale), ctypes.c_int(int(interleaved)),
                         _ptr(r), ctypes.c_int(n_rows), _ptr(out))
    if rc != 0:
        raise ValueError("oracle_attn: bad argument or page id out of range")
    return out
