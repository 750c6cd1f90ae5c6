// Host-side page pool and chunk-to-page aligner: the metadata half of the path (scheduling path of
// §3.2 and Alg. 1). Integer-only; owns no device memory.
//
// A request is laid out in closed form, block by block, from the padding rule of §3.2.1 (chunks get
// leading pad, prompts trailing pad, the final prompt none) and the first-block rule of §3.2.3 /
// §3.3.1 (block 0 of each chunk occurrence is request-private, blocks 1.. are the chunk's canonical
// shared pages). Residency, admission, eviction and allocation then follow the order of Alg. 1.
#include <algorithm>
#include <cstdint>
#include <functional>
#include <new>
#include <queue>
#include <unordered_map>
#include <utility>
#include <memory>
#include <new>
#include <vector>

#include "mepic.h"

namespace {

struct Chunk {
  uint32_t n_tokens = 0;
  std::vector<int32_t> pages;  // canonical pages of blocks 1..
  uint32_t ref = 0;            // one per live occurrence
  uint64_t stamp = 0;          // LRU clock of the last occurrence aligned or released
};

struct Request {
  std::vector<int32_t> private_pages;
  std::vector<uint64_t> occurrences;  // chunk keys, one per occurrence that holds shared pages
  uint32_t n_blocks = 0;
};

// One logical block of the aligned request before pages are assigned.
struct BlockPlan {
  bool shared;
  uint64_t key;        // shared only
  uint32_t index;      // shared only: block index inside the chunk (>= 1)
  uint32_t valid;      // bit s = slot s holds a real token
  int32_t pos0;        // position of slot 0 when pads are not counted
};

inline uint32_t bits(uint32_t lo, uint32_t hi) {  // bits [lo, hi), hi <= 32
  const uint64_t m = ((uint64_t{1} << hi) - 1) & ~((uint64_t{1} << lo) - 1);
  return static_cast<uint32_t>(m);
}

}  // namespace

struct mepic_pool {
  uint32_t P = 0, total = 0;
  std::priority_queue<int32_t, std::vector<int32_t>, std::greater<int32_t>> free_pages;
  std::unordered_map<uint64_t, Chunk> chunks;
  std::unordered_map<uint64_t, Request> requests;
  uint64_t clock = 0, next_handle = 1;
  uint64_t dup_pages = 0, peak_unique = 0, peak_dup = 0;

  int32_t take_page() {
    const int32_t p = free_pages.top();
    free_pages.pop();
    return p;
  }
};

namespace {
// Nothing may throw across the C boundary: a failed host allocation (std::bad_alloc from a container) or any other
// exception becomes a status code.
template <class F>
int guarded(F&& body) noexcept {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return MEPIC_ERR_NOMEM;
  } catch (...) {
    return MEPIC_ERR_INVALID;
  }
}
}  // namespace

extern "C" {

const char* mepic_strerror(int status) {
  switch (status) {
    case MEPIC_OK: return "ok";
    case MEPIC_ERR_INVALID: return "invalid argument";
    case MEPIC_ERR_NOMEM: return "rejected: free and evictable pages cannot cover the demand";
    case MEPIC_ERR_CAPACITY: return "output buffer or workspace too small";
    case MEPIC_ERR_UNSUPPORTED: return "unsupported shape or dtype combination";
    case MEPIC_ERR_LAUNCH: return "HIP launch error";
    default: return "unknown status";
  }
}

int mepic_version(void) { return 100; }

int mepic_pool_create(uint32_t num_pages, uint32_t page_size, mepic_pool** out) {
  if (!out || page_size == 0 || page_size > 32 || num_pages > 0x7fffffffu) return MEPIC_ERR_INVALID;
  return guarded([&]() -> int {
    std::unique_ptr<mepic_pool> p(new mepic_pool());
    p->P = page_size;
    p->total = num_pages;
    std::vector<int32_t> ids(num_pages);
    for (uint32_t i = 0; i < num_pages; ++i) ids[i] = static_cast<int32_t>(i);
    p->free_pages = decltype(p->free_pages)(std::greater<int32_t>(), std::move(ids));
    *out = p.release();
    return MEPIC_OK;
  });
}

void mepic_pool_destroy(mepic_pool* pool) { delete pool; }

int mepic_align_request(mepic_pool* pool, const mepic_segment* segs, uint32_t n_segs,
                        uint32_t extra_tail_tokens, int32_t* block_table_out, uint32_t capacity,
                        uint8_t* block_kind_out, uint32_t* block_valid_out, int32_t* block_pos_out,
                        uint64_t* request_handle_out, mepic_align_info* info_out) {
  return guarded([&]() -> int {
    if (!pool || (!segs && n_segs) || !request_handle_out || !info_out) return MEPIC_ERR_INVALID;
    const uint32_t P = pool->P;
  
    // ---- segmentation and canonicalisation: plan every block in closed form ----
    std::vector<BlockPlan> plan;
    std::unordered_map<uint64_t, uint32_t> key_len;  // chunk keys of this request -> n_tokens
    uint64_t real = 0, pads = 0, kv_len = 0;
    uint32_t open_fill = 0;  // real slots in a final prompt's partly filled last block (0 = none open)
    for (uint32_t i = 0; i < n_segs; ++i) {
      const mepic_segment& s = segs[i];
      const uint32_t n = s.n_tokens;
      if (n == 0 || (s.kind != MEPIC_SEG_PROMPT && s.kind != MEPIC_SEG_CHUNK)) return MEPIC_ERR_INVALID;
      const uint32_t nb = (n + P - 1) / P;
      if (s.kind == MEPIC_SEG_PROMPT) {
        const bool last = (i + 1 == n_segs);
        for (uint32_t j = 0; j < nb; ++j) {
          const uint32_t cnt = std::min(P, n - j * P);
          plan.push_back({false, 0, 0, bits(0, cnt), static_cast<int32_t>(real + uint64_t{j} * P)});
        }
        if (last) {
          kv_len += n;
          open_fill = n % P;
        } else {
          kv_len += uint64_t{nb} * P;
          pads += uint64_t{nb} * P - n;
        }
      } else {
        auto seen = key_len.find(s.chunk_key);
        if (seen != key_len.end() && seen->second != n) return MEPIC_ERR_INVALID;
        auto res = pool->chunks.find(s.chunk_key);
        if (res != pool->chunks.end() && res->second.n_tokens != n) return MEPIC_ERR_INVALID;
        key_len[s.chunk_key] = n;
        const uint32_t lead = nb * P - n;
        const int64_t base = static_cast<int64_t>(real) - lead;
        plan.push_back({false, 0, 0, bits(lead, P), static_cast<int32_t>(base)});
        for (uint32_t j = 1; j < nb; ++j)
          plan.push_back({true, s.chunk_key, j, bits(0, P), static_cast<int32_t>(base + int64_t{j} * P)});
        kv_len += uint64_t{nb} * P;
        pads += lead;
      }
      real += n;
    }
    // the tokens after the last segment: fill the open block first, then fresh private blocks
    uint32_t tail = extra_tail_tokens;
    if (tail && open_fill) {
      const uint32_t add = std::min(tail, P - open_fill);
      plan.back().valid = bits(0, open_fill + add);
      tail -= add;
      real += add;
      kv_len += add;
    }
    while (tail) {
      const uint32_t cnt = std::min(tail, P);
      plan.push_back({false, 0, 0, bits(0, cnt), static_cast<int32_t>(real)});
      tail -= cnt;
      real += cnt;
      kv_len += cnt;
    }
    const uint32_t n_blocks = static_cast<uint32_t>(plan.size());
    if (n_blocks > capacity) return MEPIC_ERR_CAPACITY;
    if (n_blocks && !block_table_out) return MEPIC_ERR_INVALID;
    if (kv_len > 0x7fffffffu) return MEPIC_ERR_INVALID;
  
    // ---- residency resolution and admission check ----
    uint64_t demand = 0;
    for (const BlockPlan& b : plan)
      if (!b.shared) ++demand;
    for (const auto& kl : key_len) {
      const uint32_t nb = (kl.second + P - 1) / P;
      if (nb > 1 && !pool->chunks.count(kl.first)) demand += nb - 1;
    }
    std::vector<std::pair<uint64_t, uint64_t>> evictable;  // (stamp, key), unused by this request
    uint64_t evictable_pages = 0;
    for (const auto& kc : pool->chunks)
      if (kc.second.ref == 0 && !key_len.count(kc.first)) {
        evictable.emplace_back(kc.second.stamp, kc.first);
        evictable_pages += kc.second.pages.size();
      }
    if (demand > pool->free_pages.size() + evictable_pages) return MEPIC_ERR_NOMEM;
    uint32_t n_evicted = 0;
    if (demand > pool->free_pages.size()) {
      std::sort(evictable.begin(), evictable.end());
      for (const auto& e : evictable) {
        if (pool->free_pages.size() >= demand) break;
        auto it = pool->chunks.find(e.second);
        for (int32_t pg : it->second.pages) pool->free_pages.push(pg);
        pool->chunks.erase(it);
        ++n_evicted;
      }
    }
  
    // ---- block allocation, left to right ----
    Request req;
    req.n_blocks = n_blocks;
    mepic_align_info info = {};
    for (uint32_t j = 0; j < n_blocks;) {
      const BlockPlan& b = plan[j];
      if (!b.shared) {
        const int32_t pg = pool->take_page();
        req.private_pages.push_back(pg);
        block_table_out[j] = pg;
        if (block_kind_out) block_kind_out[j] = MEPIC_BLOCK_PRIVATE;
        ++info.n_private;
        ++j;
        continue;
      }
      // blocks 1.. of one chunk occurrence are consecutive in the plan
      const uint32_t run = (key_len[b.key] + P - 1) / P - 1;
      auto it = pool->chunks.find(b.key);
      uint8_t kind;
      if (it != pool->chunks.end()) {
        it->second.ref += 1;
        kind = MEPIC_BLOCK_SHARED_HIT;
        info.n_shared_hit += run;
      } else {
        Chunk c;
        c.n_tokens = key_len[b.key];
        c.ref = 1;
        c.pages.reserve(run);
        for (uint32_t r = 0; r < run; ++r) c.pages.push_back(pool->take_page());
        it = pool->chunks.emplace(b.key, std::move(c)).first;
        kind = MEPIC_BLOCK_SHARED_NEW;
        info.n_shared_new += run;
      }
      it->second.stamp = ++pool->clock;
      for (uint32_t r = 0; r < run; ++r) {
        block_table_out[j + r] = it->second.pages[r];
        if (block_kind_out) block_kind_out[j + r] = kind;
      }
      req.occurrences.push_back(b.key);
      j += run;
    }
    for (uint32_t j = 0; j < n_blocks; ++j) {
      if (block_valid_out) block_valid_out[j] = plan[j].valid;
      if (block_pos_out) block_pos_out[j] = plan[j].pos0;
    }
    info.n_blocks = n_blocks;
    info.n_pad_slots = static_cast<uint32_t>(pads);
    info.kv_len = static_cast<uint32_t>(kv_len);
    info.n_evicted_chunks = n_evicted;
    *info_out = info;
  
    const uint64_t handle = pool->next_handle++;
    pool->requests.emplace(handle, std::move(req));
    *request_handle_out = handle;
    pool->dup_pages += n_blocks;
    pool->peak_dup = std::max(pool->peak_dup, pool->dup_pages);
    pool->peak_unique = std::max<uint64_t>(pool->peak_unique, pool->total - pool->free_pages.size());
    return MEPIC_OK;
  });
}

int mepic_release_request(mepic_pool* pool, uint64_t request_handle) {
  return guarded([&]() -> int {
    if (!pool) return MEPIC_ERR_INVALID;
    auto it = pool->requests.find(request_handle);
    if (it == pool->requests.end()) return MEPIC_ERR_INVALID;
    for (int32_t pg : it->second.private_pages) pool->free_pages.push(pg);
    for (uint64_t key : it->second.occurrences) {
      Chunk& c = pool->chunks.at(key);
      c.ref -= 1;
      c.stamp = ++pool->clock;
    }
    pool->dup_pages -= it->second.n_blocks;
    pool->requests.erase(it);
    return MEPIC_OK;
  });
}

int mepic_pool_get_stats(const mepic_pool* pool, mepic_pool_stats* out) {
  if (!pool || !out) return MEPIC_ERR_INVALID;
  mepic_pool_stats s = {};
  s.pages_total = pool->total;
  s.pages_free = pool->free_pages.size();
  s.pages_in_use_unique = pool->total - pool->free_pages.size();
  s.pages_logical_duplicated = pool->dup_pages;
  s.chunks_resident = pool->chunks.size();
  for (const auto& kc : pool->chunks)
    if (kc.second.ref == 0) ++s.chunks_zero_ref;
  s.requests_live = pool->requests.size();
  s.peak_pages_in_use_unique = pool->peak_unique;
  s.peak_pages_logical_duplicated = pool->peak_dup;
  *out = s;
  return MEPIC_OK;
}

int mepic_pool_lookup_chunk(const mepic_pool* pool, uint64_t chunk_key, int* resident_out,
                            uint32_t* refcount_out) {
  if (!pool || !resident_out) return MEPIC_ERR_INVALID;
  auto it = pool->chunks.find(chunk_key);
  *resident_out = it != pool->chunks.end();
  if (refcount_out) *refcount_out = it != pool->chunks.end() ? it->second.ref : 0;
  return MEPIC_OK;
}

}  // extern "C"
