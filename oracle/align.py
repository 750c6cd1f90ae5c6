"""Chunk-to-page aligner and pool accounting, plain Python — TEST INFRASTRUCTURE ONLY.

Follows the paper's scheduling path (§3.2, Alg. 1) step by step: lay the request out slot by slot
under the padding rule of §3.2.1, resolve which chunks are resident, check admission, evict
zero-reference chunks if needed, assign pages. It shares no code with the library's C++ pool.

Layout rule (§3.2.1): a chunk gets LEADING pad so that it ends on a block boundary and starts on one;
a prompt segment gets TRAILING pad; the final prompt segment is left unpadded. First-block rule
(§3.2.3, §3.3.1): block 0 of every chunk occurrence is request-private, blocks 1.. are the chunk's
canonical shared pages.

Readings where the paper is silent: lowest-numbered free page first; segments left to right; a chunk's
private first block before its shared pages; every occurrence of a chunk holds one reference; the
LRU clock ticks once per chunk occurrence at align and at release; eviction takes whole chunks,
oldest stamp first, only as many as needed, never a chunk the request itself uses.

Pins (tests/test_aligner.py): the paper's worked example (block 16, a chunk after 32 vs 35 tokens,
§2 challenge 2), closed-form page counts, refcounts back to zero after release, Reject when demand
exceeds free + evictable.
"""
from __future__ import annotations

import heapq
from typing import Dict, List, Sequence, Tuple

PROMPT, CHUNK = 0, 1
PRIVATE, SHARED_HIT, SHARED_NEW = 0, 1, 2


class Reject(Exception):
    """Alg. 1: not enough free or evictable pages."""


class Invalid(Exception):
    pass


class Capacity(Exception):
    pass


def layout_slots(segs: Sequence[Tuple[int, int, int]], P: int, extra_tail: int):
    """T_align slot by slot. Returns a list of (is_real, position_without_pads, owner) per slot where
    owner is ('p',) for private slots or ('c', key, block_index_in_chunk) for shared chunk slots."""
    slots = []
    real = 0  # real tokens laid out so far
    for si, (kind, n, key) in enumerate(segs):
        last = si == len(segs) - 1
        if n <= 0 or kind not in (PROMPT, CHUNK):
            raise Invalid("bad segment")
        if kind == PROMPT:
            for _ in range(n):
                slots.append((True, real, ("p",)))
                real += 1
            if not last:
                while len(slots) % P:
                    slots.append((False, None, ("p",)))
        else:
            assert len(slots) % P == 0, "a chunk always starts on a block boundary"
            lead = (-n) % P
            for _ in range(lead):
                slots.append((False, None, ("p",)))
            for i in range(n):
                blk = (lead + i) // P
                slots.append((True, real, ("p",) if blk == 0 else ("c", key, blk)))
                real += 1
    for _ in range(extra_tail):
        slots.append((True, real, ("p",)))
        real += 1
    return slots


class PoolOracle:
    def __init__(self, num_pages: int, page_size: int):
        self.P = page_size
        self.total = num_pages
        self.free: List[int] = list(range(num_pages))
        heapq.heapify(self.free)
        self.chunks: Dict[int, dict] = {}    # key -> {n, pages, ref, stamp}
        self.requests: Dict[int, dict] = {}  # handle -> {private, occ, n_blocks}
        self.clock = 0
        self.next_handle = 1
        self.peak_unique = 0
        self.peak_dup = 0

    # ---- accounting (the paper's HBM-usage metric, §4.1) ----
    def stats(self) -> dict:
        dup = sum(r["n_blocks"] for r in self.requests.values())
        return dict(pages_total=self.total, pages_free=len(self.free),
                    pages_in_use_unique=self.total - len(self.free), pages_logical_duplicated=dup,
                    chunks_resident=len(self.chunks),
                    chunks_zero_ref=sum(1 for c in self.chunks.values() if c["ref"] == 0),
                    requests_live=len(self.requests), peak_pages_in_use_unique=self.peak_unique,
                    peak_pages_logical_duplicated=self.peak_dup)

    def align(self, segs: Sequence[Tuple[int, int, int]], extra_tail: int = 0, capacity: int = 1 << 30) -> dict:
        P = self.P
        # --- segmentation and canonicalisation ---
        slots = layout_slots(segs, P, extra_tail)
        for kind, n, key in segs:
            if kind == CHUNK and key in self.chunks and self.chunks[key]["n"] != n:
                raise Invalid("chunk key reused with another length")
        seen = {}
        for kind, n, key in segs:
            if kind == CHUNK and seen.setdefault(key, n) != n:
                raise Invalid("chunk key reused with another length")
        n_blocks = -(-len(slots) // P)
        if capacity < n_blocks:
            raise Capacity("block table too small")
        blocks = [slots[j * P:(j + 1) * P] for j in range(n_blocks)]
        owners = []
        for blk in blocks:
            own = {s[2] for s in blk}
            assert len(own) == 1, "a block never mixes private and shared slots"
            owners.append(own.pop())
        # --- residency resolution ---
        used_keys = {o[1] for o in owners if o[0] == "c"}
        missing = {k for k in used_keys if k not in self.chunks}
        # --- admission check ---
        demand = sum(1 for o in owners if o[0] == "p")
        for k in missing:
            demand += len({o[2] for o in owners if o[0] == "c" and o[1] == k})
        evictable = [(c["stamp"], k) for k, c in self.chunks.items() if c["ref"] == 0 and k not in used_keys]
        if demand > len(self.free) + sum(len(self.chunks[k]["pages"]) for _, k in evictable):
            raise Reject()
        n_evicted = 0
        for _, k in sorted(evictable):
            if len(self.free) >= demand:
                break
            for p in self.chunks.pop(k)["pages"]:
                heapq.heappush(self.free, p)
            n_evicted += 1
        # --- block allocation, left to right ---
        table, kinds = [], []
        private, occ = [], []
        j = 0
        while j < n_blocks:
            o = owners[j]
            if o[0] == "p":
                pg = heapq.heappop(self.free)
                private.append(pg)
                table.append(pg)
                kinds.append(PRIVATE)
                j += 1
                continue
            key = o[1]
            run = 0
            while j + run < n_blocks and owners[j + run][:2] == ("c", key) and owners[j + run][2] == run + 1:
                run += 1
            self.clock += 1
            if key in self.chunks:
                c = self.chunks[key]
                c["ref"] += 1
                kind = SHARED_HIT
            else:
                c = dict(n=seen[key], pages=[heapq.heappop(self.free) for _ in range(run)], ref=1, stamp=0)
                self.chunks[key] = c
                kind = SHARED_NEW
            c["stamp"] = self.clock
            assert len(c["pages"]) == run
            table += c["pages"]
            kinds += [kind] * run
            occ.append(key)
            j += run
        valid = [sum(1 << s for s, sl in enumerate(blk) if sl[0]) for blk in blocks]
        pos0 = []
        for blk in blocks:
            s, sl = next((s, sl) for s, sl in enumerate(blk) if sl[0])
            pos0.append(sl[1] - s)
        handle = self.next_handle
        self.next_handle += 1
        self.requests[handle] = dict(private=private, occ=occ, n_blocks=n_blocks)
        st = self.stats()
        self.peak_unique = max(self.peak_unique, st["pages_in_use_unique"])
        self.peak_dup = max(self.peak_dup, st["pages_logical_duplicated"])
        info = dict(n_blocks=n_blocks, n_private=kinds.count(PRIVATE), n_shared_hit=kinds.count(SHARED_HIT),
                    n_shared_new=kinds.count(SHARED_NEW), n_pad_slots=sum(1 for s in slots if not s[0]),
                    kv_len=len(slots), n_evicted_chunks=n_evicted)
        return dict(block_table=table, block_kind=kinds, block_valid=valid, block_pos=pos0, handle=handle, info=info)

    def release(self, handle: int) -> None:
        if handle not in self.requests:
            raise Invalid("unknown handle")
        r = self.requests.pop(handle)
        for p in r["private"]:
            heapq.heappush(self.free, p)
        for key in r["occ"]:
            self.clock += 1
            c = self.chunks[key]
            c["ref"] -= 1
            c["stamp"] = self.clock

    def lookup(self, key: int):
        c = self.chunks.get(key)
        return (False, 0) if c is None else (True, c["ref"])
