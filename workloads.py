"""Seeded synthetic inputs for the fused-RoPE paged-attention path.

This module serves both the CPU oracle's tests and the HIP path's tests / bench. It holds none of the
method's arithmetic: no padding rule, no rotary embedding, no softmax. It only

  * draws request *structures* (segment lists: private prompt text and reusable chunks with Zipfian
    popularity, the request mix the paper motivates in its introduction and evaluates in §4),
  * draws N(0,1) values keyed by physical page id and rounds them to the storage dtype,
  * moves bytes between the slot-major "logical" view [page][Hkv][P][D] and the page layout of the
    C-ABI header (K: [page][Hkv][D/X][P][X], V: [page][Hkv][D][P]),
  * copies pages into a layout in which every logical block owns a page (the layout of systems
    that do not share chunk pages).

Block tables are NOT made here: they come from an aligner (the oracle's or the library's) and are
passed in where needed.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Tuple

import numpy as np
import torch

PROMPT, CHUNK = 0, 1
CHUNK_KEY_BASE = 0xC0DE_0000_0000

_TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f8e4m3": torch.float8_e4m3fn}
_ELEM_BYTES = {"f32": 4, "bf16": 2, "f8e4m3": 1}
E4M3_MAX = 448.0


@dataclass
class Structure:
    """Shapes plus the per-request segment lists of one workload."""
    name: str
    mode: str                 # "decode" | "prefill"
    B: int
    Hq: int
    Hkv: int
    D: int
    P: int
    theta: float
    q_dtype: str              # "f32" | "bf16"
    kv_dtype: str             # "f32" | "bf16" | "f8e4m3"
    seed: int
    requests: List[List[Tuple[int, int, int]]] = field(default_factory=list)  # (kind, n_tokens, key)
    extra_tail: int = 1       # tokens appended after the last segment (the token being decoded)
    n_q: List[int] = field(default_factory=list)  # query tokens per request


def _rng(seed: int, stream: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, stream, *key])))


def zipf_draw(rng: np.random.Generator, pool: int, n: int, s: float = 1.1) -> np.ndarray:
    """n draws with replacement from {0..pool-1}, P(k) proportional to (k+1)^-s (inverse CDF)."""
    w = np.arange(1, pool + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w / w.sum())
    idx = np.searchsorted(cdf, rng.random(n), side="right")
    return np.minimum(idx, pool - 1)


# ---------------------------------------------------------------------------------------------
# structures
# ---------------------------------------------------------------------------------------------
def decode_structure(name: str, seed: int, *, B: int, Hq: int, Hkv: int, D: int, P: int, theta: float,
                     q_dtype: str, kv_dtype: str, prefix: int, n_chunks, chunk_tokens: int, pool: int,
                     question: int, zipf_s: float = 1.1) -> Structure:
    """Decode workload: [private prefix] + chunks drawn Zipf(s) from a pool + [private question] +
    the token being decoded. `n_chunks` is an int or an inclusive (lo, hi) range drawn uniformly."""
    rs = _rng(seed, 1)
    st = Structure(name, "decode", B, Hq, Hkv, D, P, theta, q_dtype, kv_dtype, seed, extra_tail=1)
    for _ in range(B):
        nc = n_chunks if isinstance(n_chunks, int) else int(rs.integers(n_chunks[0], n_chunks[1] + 1))
        segs = []
        if prefix:
            segs.append((PROMPT, prefix, 0))
        for k in zipf_draw(rs, pool, nc, zipf_s):
            segs.append((CHUNK, chunk_tokens, CHUNK_KEY_BASE + int(k)))
        if question:
            segs.append((PROMPT, question, 0))
        st.requests.append(segs)
        st.n_q.append(1)
    return st


def prefill_structure(name: str, seed: int, *, B: int, Hq: int, Hkv: int, D: int, P: int, theta: float,
                      n_chunks: int, chunk_tokens: int, pool: int, q_tokens: int, max_gap_pages: int = 4,
                      q_dtype: str = "bf16", kv_dtype: str = "bf16", zipf_s: float = 1.1) -> Structure:
    """Question-token prefill: chunks at random offsets (a private gap of 0..max_gap_pages pages of
    prompt text before each chunk), then `q_tokens` question tokens whose K/V are already committed."""
    rs = _rng(seed, 1)
    st = Structure(name, "prefill", B, Hq, Hkv, D, P, theta, q_dtype, kv_dtype, seed, extra_tail=0)
    for _ in range(B):
        segs = []
        keys = zipf_draw(rs, pool, n_chunks, zipf_s)
        gaps = rs.integers(0, max_gap_pages + 1, size=n_chunks)
        for k, g in zip(keys, gaps):
            if g:
                segs.append((PROMPT, int(g) * P, 0))
            segs.append((CHUNK, chunk_tokens, CHUNK_KEY_BASE + int(k)))
        segs.append((PROMPT, q_tokens, 0))
        st.requests.append(segs)
        st.n_q.append(q_tokens)
    return st


def config(idx: int) -> Structure:
    """The five benchmark workloads, by 1-based index (seed = 1000 + index)."""
    seed = 1000 + idx
    if idx == 1:
        st = Structure("cfg1_tiny_decode_f32", "decode", 1, 8, 8, 64, 16, 1e4, "f32", "f32", seed)
        st.requests = [[(PROMPT, 32, 0), (CHUNK, 128, CHUNK_KEY_BASE + 1), (CHUNK, 128, CHUNK_KEY_BASE + 2)]]
        st.n_q = [1]
        return st
    if idx == 2:
        return decode_structure("cfg2_llama3_8b_decode_bf16", seed, B=64, Hq=32, Hkv=8, D=128, P=16,
                                theta=5e5, q_dtype="bf16", kv_dtype="bf16", prefix=64, n_chunks=8,
                                chunk_tokens=512, pool=32, question=128)
    if idx == 3:
        return prefill_structure("cfg3_question_prefill_bf16", seed, B=16, Hq=32, Hkv=8, D=128, P=16,
                                 theta=5e5, n_chunks=16, chunk_tokens=1024, pool=64, q_tokens=256)
    if idx == 4:
        return decode_structure("cfg4_long_decode_bf16", seed, B=8, Hq=32, Hkv=8, D=128, P=16,
                                theta=5e5, q_dtype="bf16", kv_dtype="bf16", prefix=0, n_chunks=64,
                                chunk_tokens=1024, pool=256, question=0)
    if idx == 5:
        return decode_structure("cfg5_mixed_decode_fp8", seed, B=128, Hq=28, Hkv=4, D=128, P=32,
                                theta=1e6, q_dtype="bf16", kv_dtype="f8e4m3", prefix=0, n_chunks=(4, 64),
                                chunk_tokens=512, pool=128, question=0)
    raise ValueError(f"no config {idx}")


# ---------------------------------------------------------------------------------------------
# values
# ---------------------------------------------------------------------------------------------
@dataclass
class KVPages:
    """K/V pages in the storage layout of the C-ABI header, on the CPU."""
    k: torch.Tensor                    # [num_pages, Hkv, D/X, P, X] storage dtype
    v: torch.Tensor                    # [num_pages, Hkv, D, P]      storage dtype
    k_scales: Optional[torch.Tensor]   # [num_pages] fp32 (fp8 only)
    v_scales: Optional[torch.Tensor]
    kv_dtype: str
    Hkv: int
    D: int
    P: int

    @property
    def num_pages(self) -> int:
        return self.k.shape[0]

    def nbytes_per_page(self) -> int:
        return 2 * self.Hkv * self.D * self.P * _ELEM_BYTES[self.kv_dtype]


def granule(kv_dtype: str) -> int:
    """Elements per 16-byte granule."""
    return 16 // _ELEM_BYTES[kv_dtype]


def pack_k(k_logical: torch.Tensor, kv_dtype: str) -> torch.Tensor:
    """[N, Hkv, P, D] -> [N, Hkv, D/X, P, X] (pure data movement)."""
    N, H, P, D = k_logical.shape
    X = granule(kv_dtype)
    return k_logical.reshape(N, H, P, D // X, X).permute(0, 1, 3, 2, 4).contiguous()


def pack_v(v_logical: torch.Tensor) -> torch.Tensor:
    """[N, Hkv, P, D] -> [N, Hkv, D, P] (pure data movement)."""
    return v_logical.permute(0, 1, 3, 2).contiguous()


def unpack_k(k_packed: torch.Tensor) -> torch.Tensor:
    N, H, DX, P, X = k_packed.shape
    return k_packed.permute(0, 1, 3, 2, 4).reshape(N, H, P, DX * X).contiguous()


def unpack_v(v_packed: torch.Tensor) -> torch.Tensor:
    return v_packed.permute(0, 1, 3, 2).contiguous()


def store_round(x: torch.Tensor, kv_dtype: str):
    """Round fp32 logical pages [N, Hkv, P, D] to the storage dtype.

    Returns (stored tensor of the storage dtype, per-page fp32 scales or None). For fp8 the scale of a
    page is amax/448 over the whole page (all heads and slots; 1.0 for an all-zero page), the code is the
    round-to-nearest-even e4m3fn of x/scale (|x/scale| <= 448 by construction, clamped against fp32
    rounding)."""
    if kv_dtype == "f32":
        return x.contiguous(), None
    if kv_dtype == "bf16":
        return x.to(torch.bfloat16), None
    amax = x.abs().amax(dim=(1, 2, 3))
    scale = torch.where(amax > 0, amax / E4M3_MAX, torch.ones_like(amax)).to(torch.float32)
    y = (x / scale.view(-1, 1, 1, 1)).clamp_(-E4M3_MAX, E4M3_MAX)
    return y.to(torch.float8_e4m3fn), scale


def gen_pages(seed: int, num_pages: int, Hkv: int, P: int, D: int, kv_dtype: str,
              used: Optional[np.ndarray] = None, group: int = 256) -> KVPages:
    """N(0,1) K/V for pages [0, num_pages), keyed by (seed, page group) so the values of a page do not
    depend on how many pages exist. Pages with used[p] == False are filled with NaN (fp8: the NaN
    code) so that a wrong gather shows up in the output."""
    X = granule(kv_dtype)
    dt = _TORCH_DT[kv_dtype]
    k = torch.empty((num_pages, Hkv, D // X, P, X), dtype=dt)
    v = torch.empty((num_pages, Hkv, D, P), dtype=dt)
    ks = vs = None
    if kv_dtype == "f8e4m3":
        ks = torch.empty(num_pages, dtype=torch.float32)
        vs = torch.empty(num_pages, dtype=torch.float32)
    for g0 in range(0, num_pages, group):
        g1 = min(g0 + group, num_pages)
        rng = _rng(seed, 2, g0 // group)
        kv = rng.standard_normal((2, group, Hkv, P, D), dtype=np.float32)[:, : g1 - g0]
        kl, kscale = store_round(torch.from_numpy(np.ascontiguousarray(kv[0])), kv_dtype)
        vl, vscale = store_round(torch.from_numpy(np.ascontiguousarray(kv[1])), kv_dtype)
        k[g0:g1] = pack_k(kl, kv_dtype)
        v[g0:g1] = pack_v(vl)
        if ks is not None:
            ks[g0:g1] = kscale
            vs[g0:g1] = vscale
    if used is not None:
        dead = torch.from_numpy(~np.asarray(used, dtype=bool))
        if dead.any():
            if kv_dtype == "f8e4m3":
                k.view(torch.uint8)[dead] = 0x7F
                v.view(torch.uint8)[dead] = 0x7F
            else:
                k[dead] = float("nan")
                v[dead] = float("nan")
    return KVPages(k, v, ks, vs, kv_dtype, Hkv, D, P)


def gen_q(seed: int, n_q: int, Hq: int, D: int, q_dtype: str) -> torch.Tensor:
    x = _rng(seed, 4).standard_normal((n_q, Hq, D), dtype=np.float32)
    return torch.from_numpy(x).to(_TORCH_DT[q_dtype])


def poison_tail(pages: KVPages, block_tables: np.ndarray, kv_lens: np.ndarray) -> None:
    """Overwrite the slots at or beyond kv_len in each request's last block with NaN (fp8: NaN code).
    Only call when those last blocks are request-private pages."""
    P = pages.P
    for b, L in enumerate(np.asarray(kv_lens)):
        if L % P == 0:
            continue
        page = int(block_tables[b][(L - 1) // P])
        s0 = int(L % P)
        if pages.kv_dtype == "f8e4m3":
            pages.k.view(torch.uint8)[page, :, :, s0:, :] = 0x7F
            pages.v.view(torch.uint8)[page, :, :, s0:] = 0x7F
        else:
            pages.k[page, :, :, s0:, :] = float("nan")
            pages.v[page, :, :, s0:] = float("nan")


def duplicate_layout(pages: KVPages, block_tables: np.ndarray, n_blocks: np.ndarray, shuffle_seed=None):
    """Materialise the same logical KV with one page per logical block (no sharing).

    Pages are handed out in request order, or in a seeded random order when `shuffle_seed` is given (a pool
    that has been in use for a while). Returns (KVPages with sum(n_blocks) pages, block table of the same
    shape pointing at them)."""
    B, max_blocks = block_tables.shape
    src_logical = np.concatenate([block_tables[b, : n_blocks[b]] for b in range(B)]).astype(np.int64)
    total = int(src_logical.size)
    place = np.arange(total, dtype=np.int64)          # logical block i lives in physical page place[i]
    if shuffle_seed is not None:
        place = _rng(shuffle_seed, 5).permutation(total)
    src = np.empty(total, dtype=np.int64)             # physical page p holds the content of old page src[p]
    src[place] = src_logical
    bt = np.zeros_like(block_tables)
    o = 0
    for b in range(B):
        bt[b, : n_blocks[b]] = place[o:o + n_blocks[b]].astype(block_tables.dtype)
        o += int(n_blocks[b])
    idx = torch.from_numpy(src)
    ks = pages.k_scales[idx].contiguous() if pages.k_scales is not None else None
    vs = pages.v_scales[idx].contiguous() if pages.v_scales is not None else None
    dup = KVPages(pages.k[idx].contiguous(), pages.v[idx].contiguous(), ks, vs, pages.kv_dtype,
                  pages.Hkv, pages.D, pages.P)
    return dup, bt


def raw_numpy(t: Optional[torch.Tensor]) -> Optional[np.ndarray]:
    """View a CPU tensor as a numpy array of its storage words (bf16 -> uint16, fp8 -> uint8)."""
    if t is None:
        return None
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float8_e4m3fn:
        return t.view(torch.uint8).numpy()
    return t.numpy()


# ---------------------------------------------------------------------------------------------
# a complete attention case: structure + block tables (from an aligner) + values
# ---------------------------------------------------------------------------------------------
@dataclass
class Case:
    st: Structure
    block_tables: np.ndarray            # [B, max_blocks] int32
    n_blocks: np.ndarray                # [B]
    kv_lens: np.ndarray                 # [B] int32
    q_positions: np.ndarray             # [n_q] int32
    cu_q_lens: Optional[np.ndarray]     # [B+1] int32, prefill only
    pages: KVPages
    q: torch.Tensor                     # [n_q, Hq, D]
    block_positions: Optional[np.ndarray] = None
    block_valid_mask: Optional[np.ndarray] = None

    @property
    def n_q(self) -> int:
        return int(self.q.shape[0])

    def kv_bytes_logical(self) -> int:
        """Bytes of K and V the requests address: sum of kv_len * Hkv * D * 2 * elem size."""
        st = self.st
        return int(self.kv_lens.astype(np.int64).sum()) * st.Hkv * st.D * 2 * _ELEM_BYTES[st.kv_dtype]

    def kv_bytes_unique(self) -> int:
        """Bytes of the distinct pages the block tables touch."""
        used = np.unique(np.concatenate([self.block_tables[b, : self.n_blocks[b]] for b in range(self.st.B)]))
        return int(used.size) * self.pages.nbytes_per_page()


def assemble(st: Structure, aligned: List[dict], *, pads_are_positions: bool = True, poison: bool = True,
             num_pages: Optional[int] = None) -> Case:
    """Put a case together from a structure and the aligner's result per request (dicts with
    block_table, block_valid, block_pos, info). The query tokens are the last n_q slots of each request
    (decode: the token being decoded). With pads_are_positions=False the aligner's valid masks and
    pad-free positions are passed on and query positions count real tokens only."""
    B = st.B
    nb = np.array([len(a["block_table"]) for a in aligned], dtype=np.int32)
    max_blocks = int(nb.max()) if B else 0
    bt = np.zeros((B, max_blocks), dtype=np.int32)
    for b, a in enumerate(aligned):
        bt[b, : nb[b]] = np.asarray(a["block_table"], dtype=np.int32)
    kv_lens = np.array([a["info"]["kv_len"] for a in aligned], dtype=np.int32)
    bp = bm = None
    q_pos, cu = [], [0]
    if not pads_are_positions:
        bp = np.zeros((B, max_blocks), dtype=np.int32)
        bm = np.zeros((B, max_blocks), dtype=np.uint32)
        for b, a in enumerate(aligned):
            bp[b, : nb[b]] = np.asarray(a["block_pos"], dtype=np.int32)
            bm[b, : nb[b]] = np.asarray(a["block_valid"], dtype=np.uint32)
    for b, a in enumerate(aligned):
        last = int(kv_lens[b]) - 1
        if not pads_are_positions:  # position of the last real token = number of real tokens - 1
            last = int(kv_lens[b]) - int(a["info"]["n_pad_slots"]) - 1
        q_pos += [last - st.n_q[b] + 1 + i for i in range(st.n_q[b])]
        cu.append(cu[-1] + st.n_q[b])
    n_pages = int(bt.max()) + 1 if num_pages is None else num_pages
    used = np.zeros(n_pages, dtype=bool)
    for b in range(B):
        used[bt[b, : nb[b]]] = True
    pages = gen_pages(st.seed, n_pages, st.Hkv, st.P, st.D, st.kv_dtype, used=used if poison else None)
    if poison:
        poison_tail(pages, bt, kv_lens)
    q = gen_q(st.seed, cu[-1], st.Hq, st.D, st.q_dtype)
    return Case(st, bt, nb, kv_lens, np.array(q_pos, dtype=np.int32),
                np.array(cu, dtype=np.int32) if st.mode == "prefill" else None, pages, q, bp, bm)


def to_duplicated(case: Case, shuffle_seed=None) -> Case:
    """The same logical case with one page per logical block."""
    pages, bt = duplicate_layout(case.pages, case.block_tables, case.n_blocks, shuffle_seed)
    return Case(case.st, bt, case.n_blocks, case.kv_lens, case.q_positions, case.cu_q_lens, pages, case.q,
                case.block_positions, case.block_valid_mask)
