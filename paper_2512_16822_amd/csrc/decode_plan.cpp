// Host planner of the batched decode: groups the (request, step) pairs that read identical pages so that the
// kernel passes over shared pages once for up to 16/G requests (the related-work discussion of the paper, §6,
// names shared-KV attention kernels as the complement of MEPIC's page sharing: the pages many requests alias
// are then read and rotated once instead of once per request).
#include <algorithm>
#include <cstring>
#include <unordered_map>
#include <vector>

#include "attn_common.h"
#include "decode_plan.h"

namespace mepic {
namespace {

struct StepRef {
  int32_t b, s;
};

inline uint64_t key_of(const int32_t* pages, int bps) {
  return bps == 2 ? ((uint64_t)(uint32_t)pages[0] | ((uint64_t)(uint32_t)pages[1] << 32)) : (uint64_t)(uint32_t)pages[0];
}

}  // namespace
}  // namespace mepic

extern "C" {

int mepic_decode_plan_capacity(int32_t B, int32_t max_blocks, int32_t P, size_t* n_int32_out) {
  using namespace mepic;
  if (!n_int32_out || B < 0 || max_blocks < 0 || (P != 16 && P != 32)) return MEPIC_ERR_INVALID;
  const int bps = 32 / P;
  const long steps = (long)B * ((max_blocks + bps - 1) / bps);  // every step its own run at worst
  *n_int32_out = plan_words((int)std::min<long>(steps, 0x3fffffff / kPlanRunWords), B);
  return MEPIC_OK;
}

int mepic_decode_plan_build(const int32_t* block_tables, const int32_t* kv_lens, int32_t B, int32_t max_blocks,
                            int32_t P, int32_t Hq, int32_t Hkv, int32_t kv_dtype, int32_t* plan_out,
                            size_t capacity_int32, mepic_decode_plan_info* info_out) {
  using namespace mepic;
  if (!block_tables || !kv_lens || !plan_out || !info_out || B < 0 || max_blocks < 0 || Hq <= 0 || Hkv <= 0 ||
      Hq % Hkv)
    return MEPIC_ERR_INVALID;
  const bool fp8 = kv_dtype == MEPIC_F8E4M3;
  if (!((kv_dtype == MEPIC_BF16 && P == 16) || (fp8 && P == 32))) return MEPIC_ERR_UNSUPPORTED;
  const int G = Hq / Hkv;
  if (G > kPlanMaxR) return MEPIC_ERR_UNSUPPORTED;
  const int bps = 32 / P, r_cap = kPlanMaxR / G;

  // steps per request; where each request's steps start in one flat numbering
  std::vector<int> nst(B), first(B + 1, 0);
  for (int b = 0; b < B; ++b) {
    const int L = kv_lens[b];
    if (L < 0 || L > max_blocks * P) return MEPIC_ERR_INVALID;
    nst[b] = ((L + P - 1) / P + bps - 1) / bps;
    first[b + 1] = first[b] + nst[b];
  }
  const int total = first[B];

  // group id of every step: steps wholly below kv_len whose pages coincide are grouped, at most r_cap requests
  // per group and a request at most once per group
  std::vector<int> gid(total, -1);
  std::vector<std::vector<StepRef>> groups;
  {
    std::unordered_map<uint64_t, std::vector<StepRef>> by_key;
    by_key.reserve((size_t)total * 2);
    for (int b = 0; b < B; ++b)
      for (int s = 0; s < nst[b]; ++s)
        if ((s + 1) * 32 <= kv_lens[b]) by_key[key_of(block_tables + (size_t)b * max_blocks + (size_t)s * bps, bps)].push_back({b, s});
    for (int b = 0; b < B; ++b)  // deterministic order: by first member
      for (int s = 0; s < nst[b]; ++s) {
        if (gid[first[b] + s] >= 0 || (s + 1) * 32 > kv_lens[b]) continue;
        auto it = by_key.find(key_of(block_tables + (size_t)b * max_blocks + (size_t)s * bps, bps));
        std::vector<StepRef>& members = it->second;  // ascending (b, s)
        std::vector<StepRef> cur;
        for (const StepRef& m : members) {
          if (gid[first[m.b] + m.s] >= 0) continue;
          bool dup = false;
          for (const StepRef& c : cur) dup = dup || c.b == m.b;
          if (dup) continue;  // a second occurrence in the same request waits for a later group
          cur.push_back(m);
          if ((int)cur.size() == r_cap) break;
        }
        for (const StepRef& c : cur) gid[first[c.b] + c.s] = (int)groups.size();
        groups.push_back(std::move(cur));
      }
    for (int b = 0; b < B; ++b)
      for (int s = 0; s < nst[b]; ++s)
        if (gid[first[b] + s] < 0) {  // ragged last steps
          gid[first[b] + s] = (int)groups.size();
          groups.push_back({{b, s}});
        }
  }

  // runs: follow a group while all of its members step forward together into one and the same group
  struct Run {
    int n;
    std::vector<StepRef> at;
  };
  std::vector<Run> runs;
  std::vector<char> done(total, 0);
  for (int b = 0; b < B; ++b)
    for (int s = 0; s < nst[b]; ++s) {
      if (done[first[b] + s]) continue;
      const std::vector<StepRef>& g0 = groups[gid[first[b] + s]];
      Run r{1, g0};
      for (const StepRef& m : g0) done[first[m.b] + m.s] = 1;
      for (;;) {
        const StepRef lead{g0[0].b, g0[0].s + r.n};
        if (lead.s >= nst[lead.b] || done[first[lead.b] + lead.s]) break;
        const std::vector<StepRef>& g = groups[gid[first[lead.b] + lead.s]];
        bool same = g.size() == g0.size();
        for (size_t i = 0; same && i < g.size(); ++i) same = g[i].b == g0[i].b && g[i].s == g0[i].s + r.n;
        if (!same) break;
        for (const StepRef& m : g) done[first[m.b] + m.s] = 1;
        ++r.n;
      }
      runs.push_back(std::move(r));
    }

  const int n_runs = (int)runs.size();
  if (plan_words(n_runs, B) > capacity_int32) return MEPIC_ERR_CAPACITY;
  int T = 0;
  for (const Run& r : runs) T += r.n;
  const int W = decode_mfma_waves_per_head(Hkv, fp8);
  const int chunk = std::max((T + W - 1) / W, 1);

  std::memset(plan_out, 0, plan_words(n_runs, B) * sizeof(int32_t));
  int32_t* cum = plan_out + plan_off_cum(n_runs);
  int32_t* rw = plan_out + plan_off_runs(n_runs);
  int32_t* n_part = plan_out + plan_off_npart(n_runs);
  int pos = 0, n_splits = 1;
  for (int i = 0; i < n_runs; ++i) {
    const Run& r = runs[i];
    cum[i] = pos;
    const int pieces = (pos + r.n - 1) / chunk - pos / chunk + 1;  // chunks of the head's sequence the run touches
    int32_t* w = rw + (size_t)i * kPlanRunWords;
    w[0] = (int32_t)r.at.size();
    for (size_t k = 0; k < r.at.size(); ++k) {
      w[1 + k] = r.at[k].b;
      w[1 + kPlanMaxR + k] = r.at[k].s;
      w[1 + 2 * kPlanMaxR + k] = n_part[r.at[k].b];
      n_part[r.at[k].b] += pieces;
      n_splits = std::max(n_splits, (int)n_part[r.at[k].b]);
    }
    pos += r.n;
  }
  cum[n_runs] = pos;
  plan_out[0] = kPlanMagic; plan_out[1] = n_runs; plan_out[2] = T; plan_out[3] = chunk; plan_out[4] = n_splits;
  plan_out[5] = B; plan_out[6] = r_cap; plan_out[7] = 0;

  info_out->n_runs = n_runs; info_out->total_steps = T; info_out->chunk = chunk; info_out->n_splits = n_splits;
  info_out->r_cap = r_cap; info_out->steps_unbatched = total; info_out->n_int32 = (int32_t)plan_words(n_runs, B);
  info_out->B = B;
  return MEPIC_OK;
}

}  // extern "C"
