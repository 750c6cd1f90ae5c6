"""Device-side plumbing shared by the tests, the benchmark and the smoke run: put a generated case (any object
with the fields of workloads.Case) on the GPU and fill the params struct that points at it. Argument marshalling
only; nothing is computed here, and nothing here knows of any CPU checker."""
from __future__ import annotations

import numpy as np
import torch


def align_with_library(M, st, num_pages: int = 1 << 20):
    """Block tables of every request of the structure `st` from the library's own aligner."""
    pool = M.Pool(num_pages, st.P)
    return [pool.align_request(segs, st.extra_tail) for segs in st.requests], pool


class DeviceCase:
    """A case resident on the GPU plus the params struct that points at it."""

    def __init__(self, M, case, flags: int = 0, sm_scale: float = 0.0):
        dev = torch.device("cuda:0")
        st, pg = case.st, case.pages
        self.M, self.case = M, case
        t = lambda a, dt=None: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.q = case.q.to(dev)
        self.out = torch.full_like(self.q, float("nan"))
        self.k, self.v = pg.k.to(dev), pg.v.to(dev)
        self.ks = None if pg.k_scales is None else pg.k_scales.to(dev)
        self.vs = None if pg.v_scales is None else pg.v_scales.to(dev)
        self.bt, self.kv_lens, self.q_pos = t(case.block_tables), t(case.kv_lens), t(case.q_positions)
        self.cu = t(case.cu_q_lens)
        self.bp = t(case.block_positions)
        self.bm = None if case.block_valid_mask is None else torch.from_numpy(
            case.block_valid_mask.view(np.int32)).to(dev)
        self.prefill = st.mode == "prefill"
        mk = lambda ws: M.make_params(self.q, self.out, self.k, self.v, self.bt, self.kv_lens, self.q_pos,
                                      rope_theta=st.theta, cu_q_lens=self.cu, k_scales=self.ks, v_scales=self.vs,
                                      block_positions=self.bp, block_valid_mask=self.bm, sm_scale=sm_scale,
                                      flags=flags, max_kv_len=int(case.kv_lens.max()) if st.B else 0,
                                      max_q_len=max(st.n_q) if st.n_q else 0, workspace=ws)
        nbytes = M.attn_workspace_size(mk(None), self.prefill)
        self.ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
        self.params = mk(self.ws)

    def prepare_batched(self):
        """Build the batched-decode plan from the host copies of the block tables and lengths; upload it."""
        M, st = self.M, self.case.st
        plan, info = M.decode_plan_build(self.case.block_tables, self.case.kv_lens, st.P, st.Hq, st.Hkv,
                                         M.F8E4M3 if st.kv_dtype == "f8e4m3" else M.BF16)
        self.plan_info = info
        self.plan = torch.from_numpy(plan).to(self.q.device)
        nbytes = M.attn_decode_batched_workspace_size(self.params, info)
        if nbytes > self.ws.numel():
            self.ws = torch.empty(nbytes, dtype=torch.uint8, device=self.q.device)
            self.params.workspace, self.params.workspace_bytes = self.ws.data_ptr(), nbytes
        return info

    def run_batched(self) -> np.ndarray:
        if not hasattr(self, "plan"):
            self.prepare_batched()
        self.out.fill_(float("nan"))
        self.M.attn_decode_batched(self.params, self.plan, self.plan_info)
        torch.cuda.synchronize()
        return self.out.to(torch.float64).cpu().numpy()

    def run(self) -> np.ndarray:
        (self.M.attn_prefill if self.prefill else self.M.attn_decode)(self.params)
        torch.cuda.synchronize()
        return self.out.to(torch.float64).cpu().numpy()

    def run_noalloc(self) -> np.ndarray:
        """The decode entry point that takes its scratch from the library's own fixed array: no workspace."""
        ws, nbytes = self.params.workspace, self.params.workspace_bytes
        self.params.workspace, self.params.workspace_bytes = None, 0
        self.out.fill_(float("nan"))
        try:
            self.M.attn_decode_noalloc(self.params)
            torch.cuda.synchronize()
        finally:
            self.params.workspace, self.params.workspace_bytes = ws, nbytes
        return self.out.to(torch.float64).cpu().numpy()
