"""Python binding of libmepic.so (argument marshalling only — every step of the path runs in the
library's C++/HIP code). Names follow include/mepic.h.

The library must have been built (`python paper_2512_16822_amd/build.py` or `__graft_entry__.build()`);
`load()` raises if it is missing. There is no fallback of any kind.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmepic.so")

OK, ERR_INVALID, ERR_NOMEM, ERR_CAPACITY, ERR_UNSUPPORTED, ERR_LAUNCH = 0, -1, -2, -3, -4, -5
SEG_PROMPT, SEG_CHUNK = 0, 1
BLOCK_PRIVATE, BLOCK_SHARED_HIT, BLOCK_SHARED_NEW = 0, 1, 2
F32, BF16, F8E4M3 = 0, 1, 2
FLAG_ROPE_INTERLEAVED, FLAG_FORCE_GENERAL, FLAG_KV_READ_ONCE = 1, 2, 4
NOALLOC_SCRATCH_BYTES = 48 << 20

EXPORTS = ["mepic_strerror", "mepic_version", "mepic_pool_create", "mepic_pool_destroy", "mepic_align_request",
           "mepic_release_request", "mepic_pool_get_stats", "mepic_pool_lookup_chunk", "mepic_attn_workspace_size",
           "mepic_attn_decode", "mepic_attn_prefill", "mepic_last_kernel", "mepic_kv_commit",
           "mepic_decode_plan_capacity", "mepic_decode_plan_build", "mepic_attn_decode_batched_workspace_size",
           "mepic_attn_decode_batched", "mepic_attn_decode_noalloc", "mepic_selftest_dot_rotation",
           "mepic_decode_plan_build_ahead", "mepic_probe_mfma_bf16", "mepic_device_counter_khz",
           "mepic_probe_tile_stream"]


class MepicError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} ({status})")


class Segment(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_uint32), ("n_tokens", ctypes.c_uint32), ("chunk_key", ctypes.c_uint64)]


class AlignInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint32) for n in ("n_blocks", "n_private", "n_shared_hit", "n_shared_new",
                                               "n_pad_slots", "kv_len", "n_evicted_chunks")]

    def as_dict(self) -> dict:
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class PoolStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_uint64) for n in ("pages_total", "pages_free", "pages_in_use_unique",
                                               "pages_logical_duplicated", "chunks_resident", "chunks_zero_ref",
                                               "requests_live", "peak_pages_in_use_unique",
                                               "peak_pages_logical_duplicated")]

    def as_dict(self) -> dict:
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class AttnParams(ctypes.Structure):
    _fields_ = ([(n, ctypes.c_void_p) for n in ("q", "out", "k_pages", "v_pages", "k_scales", "v_scales",
                                                "block_tables", "kv_lens", "q_positions", "cu_q_lens",
                                                "block_positions", "block_valid_mask")]
                + [(n, ctypes.c_int32) for n in ("B", "n_q_tokens", "Hq", "Hkv", "D", "P", "max_blocks", "num_pages",
                                                 "max_kv_len", "max_q_len", "q_dtype", "kv_dtype")]
                + [("rope_theta", ctypes.c_float), ("sm_scale", ctypes.c_float), ("flags", ctypes.c_uint32),
                   ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                   ("timing_start", ctypes.c_void_p), ("timing_stop", ctypes.c_void_p)])


class CommitParams(ctypes.Structure):
    _fields_ = ([(n, ctypes.c_void_p) for n in ("k_new", "v_new", "k_pages", "v_pages", "k_scales", "v_scales",
                                                "block_tables", "run_request", "run_first_slot", "cu_run_tokens")]
                + [(n, ctypes.c_int32) for n in ("B", "n_runs", "n_tokens", "Hkv", "D", "P", "max_blocks", "num_pages",
                                                 "src_dtype", "kv_dtype")]
                + [("timing_start", ctypes.c_void_p), ("timing_stop", ctypes.c_void_p)])


class DecodePlanInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_runs", "total_steps", "steps_unbatched", "n_waves", "n_splits", "r_cap",
                                              "n_int32", "B")]

    def as_dict(self) -> dict:
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


_lib = None


def load() -> ctypes.CDLL:
    """Load libmepic.so; fails loudly when it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python paper_2512_16822_amd/build.py`")
    lib = ctypes.CDLL(LIB_PATH)
    lib.mepic_strerror.restype = ctypes.c_char_p
    lib.mepic_strerror.argtypes = [ctypes.c_int]
    lib.mepic_last_kernel.restype = ctypes.c_char_p
    lib.mepic_version.restype = ctypes.c_int
    lib.mepic_pool_create.argtypes = [ctypes.c_uint32, ctypes.c_uint32, ctypes.POINTER(ctypes.c_void_p)]
    lib.mepic_pool_destroy.argtypes = [ctypes.c_void_p]
    lib.mepic_pool_destroy.restype = None
    lib.mepic_align_request.argtypes = [ctypes.c_void_p, ctypes.POINTER(Segment), ctypes.c_uint32, ctypes.c_uint32,
                                        ctypes.c_void_p, ctypes.c_uint32, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(AlignInfo)]
    lib.mepic_release_request.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
    lib.mepic_pool_get_stats.argtypes = [ctypes.c_void_p, ctypes.POINTER(PoolStats)]
    lib.mepic_pool_lookup_chunk.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.POINTER(ctypes.c_int),
                                            ctypes.POINTER(ctypes.c_uint32)]
    lib.mepic_attn_workspace_size.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_int,
                                              ctypes.POINTER(ctypes.c_size_t)]
    lib.mepic_attn_decode.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_void_p]
    lib.mepic_attn_prefill.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_void_p]
    lib.mepic_attn_decode_noalloc.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_void_p]
    lib.mepic_probe_mfma_bf16.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
    lib.mepic_selftest_dot_rotation.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
    lib.mepic_probe_tile_stream.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    lib.mepic_device_counter_khz.argtypes = [ctypes.POINTER(ctypes.c_int32)]
    lib.mepic_kv_commit.argtypes = [ctypes.POINTER(CommitParams), ctypes.c_void_p]
    lib.mepic_decode_plan_capacity.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                               ctypes.POINTER(ctypes.c_size_t)]
    lib.mepic_decode_plan_build.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int32] * 6 + [
        ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(DecodePlanInfo)]
    lib.mepic_decode_plan_build_ahead.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int32] * 7 + [
        ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(DecodePlanInfo)]
    lib.mepic_attn_decode_batched_workspace_size.argtypes = [ctypes.POINTER(AttnParams), ctypes.POINTER(DecodePlanInfo),
                                                             ctypes.POINTER(ctypes.c_size_t)]
    lib.mepic_attn_decode_batched.argtypes = [ctypes.POINTER(AttnParams), ctypes.c_void_p,
                                              ctypes.POINTER(DecodePlanInfo), ctypes.c_void_p]
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().mepic_strerror(status).decode()


def version() -> int:
    return int(load().mepic_version())


def last_kernel() -> str:
    return load().mepic_last_kernel().decode()


# ------------------------------------------------------------------------------------------------
# page pool / aligner
# ------------------------------------------------------------------------------------------------
class Pool:
    """mepic_pool_* : host-side page pool and chunk-to-page aligner."""

    def __init__(self, num_pages: int, page_size: int):
        self._h = ctypes.c_void_p()
        rc = load().mepic_pool_create(num_pages, page_size, ctypes.byref(self._h))
        if rc != OK:
            raise MepicError(rc, "mepic_pool_create")
        self.page_size = page_size

    def close(self) -> None:
        if self._h:
            load().mepic_pool_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def align_request(self, segs: Sequence[Tuple[int, int, int]], extra_tail_tokens: int = 0,
                      capacity: Optional[int] = None) -> dict:
        """mepic_align_request. segs: (kind, n_tokens, chunk_key). Returns numpy arrays + info + handle."""
        n = len(segs)
        arr = (Segment * max(n, 1))()
        for i, (kind, ntok, key) in enumerate(segs):
            arr[i].kind, arr[i].n_tokens, arr[i].chunk_key = kind, ntok, key
        if capacity is None:
            P = self.page_size
            capacity = sum(-(-s[1] // P) for s in segs) + -(-extra_tail_tokens // P) + 1
        table = np.zeros(capacity, dtype=np.int32)
        kind = np.zeros(capacity, dtype=np.uint8)
        valid = np.zeros(capacity, dtype=np.uint32)
        pos = np.zeros(capacity, dtype=np.int32)
        handle = ctypes.c_uint64()
        info = AlignInfo()
        rc = load().mepic_align_request(self._h, arr, n, extra_tail_tokens, table.ctypes.data, capacity,
                                        kind.ctypes.data, valid.ctypes.data, pos.ctypes.data,
                                        ctypes.byref(handle), ctypes.byref(info))
        if rc != OK:
            raise MepicError(rc, "mepic_align_request")
        nb = info.n_blocks
        return dict(block_table=table[:nb], block_kind=kind[:nb], block_valid=valid[:nb], block_pos=pos[:nb],
                    handle=int(handle.value), info=info.as_dict())

    def release_request(self, handle: int) -> None:
        rc = load().mepic_release_request(self._h, handle)
        if rc != OK:
            raise MepicError(rc, "mepic_release_request")

    def stats(self) -> dict:
        st = PoolStats()
        rc = load().mepic_pool_get_stats(self._h, ctypes.byref(st))
        if rc != OK:
            raise MepicError(rc, "mepic_pool_get_stats")
        return st.as_dict()

    def lookup_chunk(self, key: int) -> Tuple[bool, int]:
        res, ref = ctypes.c_int(), ctypes.c_uint32()
        rc = load().mepic_pool_lookup_chunk(self._h, key, ctypes.byref(res), ctypes.byref(ref))
        if rc != OK:
            raise MepicError(rc, "mepic_pool_lookup_chunk")
        return bool(res.value), int(ref.value)


# ------------------------------------------------------------------------------------------------
# attention (torch tensors carry the device memory; nothing is computed here)
# ------------------------------------------------------------------------------------------------
def _dt(t) -> int:
    import torch
    return {torch.float32: F32, torch.bfloat16: BF16, torch.float8_e4m3fn: F8E4M3}[t.dtype]


def _p(t) -> Optional[int]:
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous and on the GPU"
    return t.data_ptr()


def make_params(q, out, k_pages, v_pages, block_tables, kv_lens, q_positions, *, rope_theta: float,
                cu_q_lens=None, k_scales=None, v_scales=None, block_positions=None, block_valid_mask=None,
                sm_scale: float = 0.0, flags: int = 0, max_kv_len: int = 0, max_q_len: int = 0,
                workspace=None) -> AttnParams:
    """Fill a mepic_attn_params from torch tensors laid out as include/mepic.h states."""
    n_q, Hq, D = q.shape
    num_pages, Hkv = k_pages.shape[0], k_pages.shape[1]
    P = v_pages.shape[3]
    B, max_blocks = block_tables.shape
    p = AttnParams()
    p.q, p.out, p.k_pages, p.v_pages = _p(q), _p(out), _p(k_pages), _p(v_pages)
    p.k_scales, p.v_scales = _p(k_scales), _p(v_scales)
    p.block_tables, p.kv_lens, p.q_positions, p.cu_q_lens = _p(block_tables), _p(kv_lens), _p(q_positions), _p(cu_q_lens)
    p.block_positions, p.block_valid_mask = _p(block_positions), _p(block_valid_mask)
    p.B, p.n_q_tokens, p.Hq, p.Hkv, p.D, p.P, p.max_blocks, p.num_pages = B, n_q, Hq, Hkv, D, P, max_blocks, num_pages
    p.max_kv_len, p.max_q_len = max_kv_len, max_q_len
    p.q_dtype, p.kv_dtype = _dt(q), _dt(k_pages)
    p.rope_theta, p.sm_scale, p.flags = rope_theta, sm_scale, flags
    if workspace is not None:
        p.workspace, p.workspace_bytes = _p(workspace), workspace.numel() * workspace.element_size()
    # the struct holds raw device pointers: keep the tensors alive for as long as it is
    p._tensors = (q, out, k_pages, v_pages, block_tables, kv_lens, q_positions, cu_q_lens, k_scales, v_scales,
                  block_positions, block_valid_mask, workspace)
    return p


def attn_workspace_size(params: AttnParams, is_prefill: bool) -> int:
    n = ctypes.c_size_t()
    rc = load().mepic_attn_workspace_size(ctypes.byref(params), int(is_prefill), ctypes.byref(n))
    if rc != OK:
        raise MepicError(rc, "mepic_attn_workspace_size")
    return int(n.value)


def _stream_handle(stream) -> int:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def attn_decode(params: AttnParams, stream=None) -> None:
    """mepic_attn_decode on `stream` (default: torch's current stream)."""
    rc = load().mepic_attn_decode(ctypes.byref(params), _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_attn_decode")


def attn_decode_noalloc(params: AttnParams, stream=None) -> None:
    """mepic_attn_decode_noalloc on `stream` (default: torch's current stream); params.workspace is ignored."""
    rc = load().mepic_attn_decode_noalloc(ctypes.byref(params), _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_attn_decode_noalloc")


def probe_mfma_bf16(iters: int, sink, stream=None, random_operands: bool = False) -> float:
    """mepic_probe_mfma_bf16: launches the matrix-instruction-only kernel; returns the flop it executes.
    sink: float32 tensor of 4 on the GPU; [1], [2] receive workgroup 0's core clocks and constant-rate ticks."""
    flop = ctypes.c_double()
    rc = load().mepic_probe_mfma_bf16(iters, int(random_operands), _p(sink), ctypes.byref(flop), _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_probe_mfma_bf16")
    return float(flop.value)


def probe_tile_stream(structure: int, iters: int, buf, stream=None) -> None:
    """mepic_probe_tile_stream: buf = float32 tensor of >= 16384 elements on the GPU."""
    rc = load().mepic_probe_tile_stream(structure, iters, _p(buf), ctypes.c_size_t(buf.numel() * buf.element_size()),
                                        _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_probe_tile_stream")


def device_counter_khz() -> int:
    """mepic_device_counter_khz: rate of the constant-rate counter behind the kernels' tick samples."""
    khz = ctypes.c_int32()
    rc = load().mepic_device_counter_khz(ctypes.byref(khz))
    if rc != OK:
        raise MepicError(rc, "mepic_device_counter_khz")
    return int(khz.value)


def selftest_dot_rotation(words, out, stream=None) -> None:
    """mepic_selftest_dot_rotation: words uint32 [n, 12] (int32 tensor), out float32 [n, 8], both on the GPU."""
    rc = load().mepic_selftest_dot_rotation(_p(words), _p(out), words.shape[0], _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_selftest_dot_rotation")


def attn_prefill(params: AttnParams, stream=None) -> None:
    """mepic_attn_prefill on `stream` (default: torch's current stream)."""
    rc = load().mepic_attn_prefill(ctypes.byref(params), _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_attn_prefill")


def decode_plan_build(block_tables, kv_lens, P: int, Hq: int, Hkv: int, kv_dtype: int, horizon_tokens: int = 0):
    """mepic_decode_plan_build (horizon_tokens = 0) or mepic_decode_plan_build_ahead on host arrays (numpy int32).
    Returns (plan words as a numpy int32 array, info)."""
    import numpy as np
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    kl = np.ascontiguousarray(kv_lens, dtype=np.int32)
    B, max_blocks = bt.shape
    cap = ctypes.c_size_t()
    rc = load().mepic_decode_plan_capacity(B, max_blocks, P, ctypes.byref(cap))
    if rc != OK:
        raise MepicError(rc, "mepic_decode_plan_capacity")
    plan = np.empty(max(int(cap.value), 1), dtype=np.int32)  # worst case; the library writes the words it uses
    info = DecodePlanInfo()
    if horizon_tokens:
        rc = load().mepic_decode_plan_build_ahead(bt.ctypes.data, kl.ctypes.data, B, max_blocks, P, Hq, Hkv, kv_dtype,
                                                  horizon_tokens, plan.ctypes.data, plan.size, ctypes.byref(info))
    else:
        rc = load().mepic_decode_plan_build(bt.ctypes.data, kl.ctypes.data, B, max_blocks, P, Hq, Hkv, kv_dtype,
                                            plan.ctypes.data, plan.size, ctypes.byref(info))
    if rc != OK:
        raise MepicError(rc, "mepic_decode_plan_build")
    return plan[: info.n_int32].copy(), info


def attn_decode_batched_workspace_size(params: AttnParams, info: DecodePlanInfo) -> int:
    n = ctypes.c_size_t()
    rc = load().mepic_attn_decode_batched_workspace_size(ctypes.byref(params), ctypes.byref(info), ctypes.byref(n))
    if rc != OK:
        raise MepicError(rc, "mepic_attn_decode_batched_workspace_size")
    return int(n.value)


def attn_decode_batched(params: AttnParams, plan_device, info: DecodePlanInfo, stream=None) -> None:
    """mepic_attn_decode_batched on `stream` (default: torch's current stream); plan_device: int32 device tensor."""
    rc = load().mepic_attn_decode_batched(ctypes.byref(params), _p(plan_device), ctypes.byref(info),
                                          _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_attn_decode_batched")


def make_commit_params(k_new, v_new, k_pages, v_pages, block_tables, run_request, run_first_slot, cu_run_tokens,
                       *, k_scales=None, v_scales=None) -> CommitParams:
    """Fill a mepic_commit_params from torch tensors laid out as include/mepic.h states."""
    n_tokens, Hkv, D = k_new.shape
    B, max_blocks = block_tables.shape
    p = CommitParams()
    p.k_new, p.v_new, p.k_pages, p.v_pages = _p(k_new), _p(v_new), _p(k_pages), _p(v_pages)
    p.k_scales, p.v_scales = _p(k_scales), _p(v_scales)
    p.block_tables, p.run_request, p.run_first_slot, p.cu_run_tokens = (_p(block_tables), _p(run_request),
                                                                       _p(run_first_slot), _p(cu_run_tokens))
    p.B, p.n_runs, p.n_tokens, p.Hkv, p.D, p.P = B, run_request.numel(), n_tokens, Hkv, D, v_pages.shape[3]
    p.max_blocks, p.num_pages = max_blocks, k_pages.shape[0]
    p.src_dtype, p.kv_dtype = _dt(k_new), _dt(k_pages)
    # the struct holds raw device pointers: keep the tensors alive for as long as it is
    p._tensors = (k_new, v_new, k_pages, v_pages, block_tables, run_request, run_first_slot, cu_run_tokens,
                  k_scales, v_scales)
    return p


def kv_commit(params: CommitParams, stream=None) -> None:
    """mepic_kv_commit on `stream` (default: torch's current stream)."""
    rc = load().mepic_kv_commit(ctypes.byref(params), _stream_handle(stream))
    if rc != OK:
        raise MepicError(rc, "mepic_kv_commit")


# ------------------------------------------------------------------------------------------------
# HIP events for mepic_attn_params.timing_start / timing_stop (plain runtime calls, nothing computed)
# ------------------------------------------------------------------------------------------------
_hip = None


def _hiprt() -> ctypes.CDLL:
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        _hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        _hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        _hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    return _hip


class HipEvent:
    """A hipEvent_t whose handle can be put into AttnParams.timing_start / timing_stop."""

    def __init__(self):
        self.handle = ctypes.c_void_p()
        if _hiprt().hipEventCreate(ctypes.byref(self.handle)) != 0:
            raise RuntimeError("hipEventCreate failed")

    def __del__(self):
        try:
            if self.handle:
                _hiprt().hipEventDestroy(self.handle)
        except Exception:
            pass

    def synchronize(self) -> None:
        if _hiprt().hipEventSynchronize(self.handle) != 0:
            raise RuntimeError("hipEventSynchronize failed")

    def elapsed_ms(self, later: "HipEvent") -> float:
        ms = ctypes.c_float()
        if _hiprt().hipEventElapsedTime(ctypes.byref(ms), self.handle, later.handle) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return float(ms.value)
