"""Glue used by the GPU parity tests: run one case through the fp64 oracle (here) and through the library
(paper_2512_16822_amd.device_case)."""
from __future__ import annotations

import numpy as np
import torch

import workloads as W
from oracle import align as OA
from paper_2512_16822_amd.device_case import DeviceCase, align_with_library  # noqa: F401  (re-exported for the tests)


def align_with_oracle(st: W.Structure, num_pages: int = 1 << 20):
    pool = OA.PoolOracle(num_pages, st.P)
    return [pool.align(segs, st.extra_tail) for segs in st.requests], pool


def oracle_out(attn, case: W.Case, rows=None, interleaved=False, sm_scale=0.0) -> np.ndarray:
    st, pg = case.st, case.pages
    return attn.attention(W.raw_numpy(case.q), st.q_dtype, W.raw_numpy(pg.k), W.raw_numpy(pg.v), st.kv_dtype,
                          case.block_tables, case.kv_lens, case.q_positions, Hq=st.Hq, Hkv=st.Hkv, D=st.D, P=st.P,
                          theta=st.theta, cu_q_lens=case.cu_q_lens, k_scales=W.raw_numpy(pg.k_scales),
                          v_scales=W.raw_numpy(pg.v_scales), block_positions=case.block_positions,
                          block_valid_mask=case.block_valid_mask, rows=rows, interleaved=interleaved,
                          sm_scale=sm_scale)
