"""The chunk-to-page aligner: the plain-Python oracle against facts of the paper and closed forms,
and the library's C++ pool against the oracle, bit for bit (block tables, kinds, masks, positions,
accounting). No GPU needed: the pool is host code."""
import os

import numpy as np
import pytest

import workloads as W
from oracle import align as OA

HERE = os.path.dirname(os.path.abspath(__file__))
PROMPT, CHUNK = 0, 1


def read_golden():
    rows = []
    with open(os.path.join(HERE, "golden", "aligner_worked_example.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(tuple(int(x) for x in line.split()))
    return rows


# ---------------------------------------------------------------- oracle pins
def test_oracle_worked_example_from_paper():
    """§2 challenge 2: block 16, chunk after a 32- vs a 35-token prompt."""
    rows = read_golden()
    pool = OA.PoolOracle(64, rows[0][0])
    shared_pages = []
    for P, prompt, first_block, pad in rows:
        r = pool.align([(PROMPT, prompt, 0), (CHUNK, 64, 7)], 0)
        kinds = r["block_kind"]
        assert kinds.index(OA.SHARED_NEW if not shared_pages else OA.SHARED_HIT) == first_block + 1
        assert kinds[first_block] == OA.PRIVATE          # first block of the chunk is request-private
        assert r["info"]["n_pad_slots"] == pad
        shared_pages.append(r["block_table"][first_block + 1:first_block + 4])
    assert shared_pages[0] == shared_pages[1]            # identical chunk -> identical physical blocks


def test_oracle_padding_rule_slot_by_slot():
    """§3.2.1: chunk gets leading pad, prompt trailing pad, final prompt none."""
    slots = OA.layout_slots([(PROMPT, 5, 0), (CHUNK, 6, 9), (PROMPT, 3, 0)], 4, 1)
    real = "".join("x" if s[0] else "." for s in slots)
    #        prompt 5 -> 8      chunk 6 -> lead 2   final prompt 3 + 1 tail token
    assert real == "xxxxx..." + "..xxxxxx" + "xxxx"
    assert [s[1] for s in slots if s[0]] == list(range(15))
    owners = [s[2] for s in slots]
    assert owners[8:12] == [("p",)] * 4 and owners[12:16] == [("c", 9, 1)] * 4


def closed_form_counts(requests, P, tail):
    """Page counts straight from the rule: duplicated = all blocks; unique = private blocks + (ceil(n/P)-1)
    per distinct chunk."""
    dup = priv = 0
    keys = {}
    for segs in requests:
        slots = 0
        for i, (kind, n, key) in enumerate(segs):
            nb = -(-n // P)
            if kind == PROMPT:
                priv += nb
                slots += n if i == len(segs) - 1 else nb * P
            else:
                priv += 1
                keys[key] = nb - 1
                slots += nb * P
        total = -(-(slots + tail) // P)
        priv += total - -(-slots // P)
        dup += total
    return dup, priv + sum(keys.values())


@pytest.mark.parametrize("cfg", [1, 2, 4, 5])
def test_oracle_closed_form_page_counts(cfg):
    st = W.config(cfg)
    pool = OA.PoolOracle(1 << 20, st.P)
    for segs in st.requests:
        pool.align(segs, st.extra_tail)
    dup, uniq = closed_form_counts(st.requests, st.P, st.extra_tail)
    s = pool.stats()
    assert (s["pages_logical_duplicated"], s["pages_in_use_unique"]) == (dup, uniq)
    if cfg == 2:
        assert dup == 64 * 269                       # 17 216 logical blocks of the 64 requests
    if cfg == 4:
        assert dup == 8 * 4097


def test_oracle_refcounts_reject_and_eviction():
    pool = OA.PoolOracle(12, 4)
    a = pool.align([(CHUNK, 16, 1)], 0)              # 1 private + 3 shared
    b = pool.align([(CHUNK, 16, 1), (CHUNK, 16, 1)], 0)   # same chunk twice in one request
    assert pool.lookup(1) == (True, 3)
    assert b["block_table"][1:4] == b["block_table"][5:8] == a["block_table"][1:4]
    assert pool.stats()["pages_in_use_unique"] == 1 + 3 + 2
    with pytest.raises(OA.Reject):
        pool.align([(PROMPT, 28, 0)], 0)             # 7 pages wanted, 6 free, nothing evictable
    assert pool.stats()["pages_free"] == 6           # a rejected request leaves the pool unchanged
    pool.release(a["handle"])
    pool.release(b["handle"])
    assert pool.lookup(1) == (True, 0) and pool.stats()["chunks_zero_ref"] == 1
    assert pool.stats()["pages_free"] == 9           # zero-ref chunk stays resident
    c = pool.align([(PROMPT, 40, 0)], 0)             # 10 pages: must evict the zero-ref chunk
    assert c["info"]["n_evicted_chunks"] == 1 and pool.lookup(1) == (False, 0)
    with pytest.raises(OA.Invalid):
        pool.align([(CHUNK, 0, 3)], 0)
    with pytest.raises(OA.Invalid):
        pool.align([(CHUNK, 8, 5), (CHUNK, 12, 5)], 0)


def test_oracle_lru_order():
    pool = OA.PoolOracle(9, 4)
    h = [pool.align([(CHUNK, 12, k)], 0)["handle"] for k in (1, 2, 3)]   # 1 private + 2 shared pages each
    for i in (1, 0, 2):                                                # release order: 2, 1, 3
        pool.release(h[i])
    pool.align([(PROMPT, 16, 0)], 0)                                   # 4 pages, 3 free: evicts chunk 2 (oldest)
    assert [pool.lookup(k)[0] for k in (1, 2, 3)] == [True, False, True]
    r = pool.align([(CHUNK, 12, 1)], 0)                                # touch chunk 1 -> chunk 3 is now oldest
    pool.release(r["handle"])
    pool.align([(PROMPT, 12, 0)], 0)                                   # 3 pages, 1 free -> evicts chunk 3 only
    assert [pool.lookup(k)[0] for k in (1, 2, 3)] == [True, False, False]


# ---------------------------------------------------------------- library vs oracle, bit-exact
def both(num_pages, P):
    import paper_2512_16822_amd as M
    return M, M.Pool(num_pages, P), OA.PoolOracle(num_pages, P)


def assert_same(r_lib, r_or):
    assert r_lib["block_table"].tolist() == r_or["block_table"]
    assert r_lib["block_kind"].tolist() == r_or["block_kind"]
    assert r_lib["block_valid"].tolist() == r_or["block_valid"]
    assert r_lib["block_pos"].tolist() == r_or["block_pos"]
    assert r_lib["info"] == r_or["info"]


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_library_matches_oracle_on_baseline_configs(cfg):
    st = W.config(cfg)
    M, lib, orc = both(1 << 17, st.P)
    for segs in st.requests:
        assert_same(lib.align_request(segs, st.extra_tail), orc.align(segs, st.extra_tail))
    assert lib.stats() == orc.stats()


def test_library_matches_oracle_on_random_traffic():
    """Ragged lengths (pads everywhere), arrivals and departures, evictions and rejections."""
    rng = np.random.default_rng(77)
    for P in (16, 32, 5):
        M, lib, orc = both(1600 // P, P)
        live = []
        n_reject = n_evict = 0
        for step in range(400):
            if live and rng.random() < 0.45:
                hl, ho = live.pop(int(rng.integers(len(live))))
                lib.release_request(hl)
                orc.release(ho)
            else:
                segs = []
                for _ in range(int(rng.integers(0, 6))):
                    if rng.random() < 0.6:
                        key = int(rng.integers(0, 12))
                        segs.append((CHUNK, 7 + 13 * key, key))      # length is a function of the key
                    else:
                        segs.append((PROMPT, int(rng.integers(1, 70)), 0))
                tail = int(rng.integers(0, 3))
                try:
                    ro = orc.align(segs, tail)
                except OA.Reject:
                    with pytest.raises(M.MepicError) as e:
                        lib.align_request(segs, tail)
                    assert e.value.status == M.ERR_NOMEM
                    n_reject += 1
                else:
                    rl = lib.align_request(segs, tail)
                    assert_same(rl, ro)
                    n_evict += ro["info"]["n_evicted_chunks"]
                    live.append((rl["handle"], ro["handle"]))
            assert lib.stats() == orc.stats()
        assert n_reject > 0 and n_evict > 0, "the traffic must exercise Reject and eviction"
        for hl, ho in live:
            lib.release_request(hl)
            orc.release(ho)
        s = lib.stats()
        assert s == orc.stats() and s["requests_live"] == 0 and s["pages_logical_duplicated"] == 0
        assert s["chunks_zero_ref"] == s["chunks_resident"]
        for k in range(12):
            assert lib.lookup_chunk(k) == orc.lookup(k)


def test_library_error_paths():
    M, lib, orc = both(8, 16)
    for bad in ([(CHUNK, 0, 1)], [(7, 5, 1)], [(CHUNK, 40, 2), (CHUNK, 41, 2)]):
        with pytest.raises(M.MepicError) as e:
            lib.align_request(bad, 0)
        assert e.value.status == M.ERR_INVALID
    with pytest.raises(M.MepicError) as e:
        lib.align_request([(PROMPT, 100, 0)], 0, capacity=3)
    assert e.value.status == M.ERR_CAPACITY
    with pytest.raises(M.MepicError) as e:
        lib.align_request([(PROMPT, 16 * 9, 0)], 0)
    assert e.value.status == M.ERR_NOMEM
    assert lib.stats()["pages_free"] == 8
    with pytest.raises(M.MepicError):
        lib.release_request(12345)
    r = lib.align_request([(CHUNK, 40, 2)], 0)
    with pytest.raises(M.MepicError) as e:                    # resident key, other length
        lib.align_request([(CHUNK, 48, 2)], 0)
    assert e.value.status == M.ERR_INVALID
    lib.release_request(r["handle"])
    with pytest.raises(M.MepicError):
        M.Pool(4, 33)


def test_expected_sharing_ratios_of_the_synthetic_configs():
    """Accounting row: unique vs duplicated pages (the paper's HBM-usage effect, §4) on the benchmark shapes."""
    import paper_2512_16822_amd as M
    got = {}
    for cfg in (2, 3, 4):
        st = W.config(cfg)
        pool = M.Pool(1 << 17, st.P)
        for segs in st.requests:
            pool.align_request(segs, st.extra_tail)
        s = pool.stats()
        got[cfg] = s["pages_logical_duplicated"] / s["pages_in_use_unique"]
    assert got[2] > 4 and got[3] > 3 and got[4] > 2.5, got
