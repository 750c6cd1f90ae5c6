// Host planner of the batched decode: groups the (request, step) pairs that read identical pages so that the
// kernel passes over shared pages once for up to 16/G requests (the related-work discussion of the paper, §6,
// names shared-KV attention kernels as the complement of MEPIC's page sharing: the pages many requests alias
// are then read and rotated once instead of once per request).
#include <algorithm>
#include <cstring>
#include <new>
#include <vector>

#include "attn_common.h"
#include "decode_plan.h"

// Cost of a gather step and of starting a piece of a run, in 1/16 of an ordinary step (from timings of the kernel
// on runs of known structure).
#ifndef MEPIC_PLAN_COST_GATHER_BF16
#define MEPIC_PLAN_COST_GATHER_BF16 23
#endif
#ifndef MEPIC_PLAN_COST_START_BF16
#define MEPIC_PLAN_COST_START_BF16 12
#endif
#ifndef MEPIC_PLAN_COST_GATHER_FP8
#define MEPIC_PLAN_COST_GATHER_FP8 28
#endif
#ifndef MEPIC_PLAN_COST_START_FP8
#define MEPIC_PLAN_COST_START_FP8 16
#endif

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
  const int n = (int)std::min<long>(steps, 0x3fffffff / kPlanRunWords);
  *n_int32_out = plan_words(n, B, n, kPlanMaxWaves);
  return MEPIC_OK;
}

int mepic_decode_plan_build(const int32_t* block_tables, const int32_t* kv_lens, int32_t B, int32_t max_blocks,
                            int32_t P, int32_t Hq, int32_t Hkv, int32_t kv_dtype, int32_t* plan_out,
                            size_t capacity_int32, mepic_decode_plan_info* info_out) {
  return mepic_decode_plan_build_ahead(block_tables, kv_lens, B, max_blocks, P, Hq, Hkv, kv_dtype, 0, plan_out,
                                       capacity_int32, info_out);
}

int mepic_decode_plan_build_ahead(const int32_t* block_tables, const int32_t* kv_lens, int32_t B, int32_t max_blocks,
                                  int32_t P, int32_t Hq, int32_t Hkv, int32_t kv_dtype, int32_t horizon_tokens,
                                  int32_t* plan_out, size_t capacity_int32, mepic_decode_plan_info* info_out) {
  try {
    using namespace mepic;
    if (!block_tables || !kv_lens || !plan_out || !info_out || B < 0 || max_blocks < 0 || Hq <= 0 || Hkv <= 0 ||
        Hq % Hkv || horizon_tokens < 0)
      return MEPIC_ERR_INVALID;
    const int horizon = horizon_tokens;
    const bool fp8 = kv_dtype == MEPIC_F8E4M3;
    if (!((kv_dtype == MEPIC_BF16 && P == 16) || (fp8 && P == 32))) return MEPIC_ERR_UNSUPPORTED;
    const int G = Hq / Hkv;
    if (G > kPlanMaxR) return MEPIC_ERR_UNSUPPORTED;
    const int bps = 32 / P, r_cap = kPlanMaxR / G;
  
    // steps per request; where each request's steps start in one flat numbering
    // (planned for growth: the steps a request reaches within `horizon` more tokens are in the plan already, as steps
    // of its own whose slots the kernel masks against the kv_len of the call)
    std::vector<int> nst(B), first(B + 1, 0), lp(B);
    for (int b = 0; b < B; ++b) {
      const int L = kv_lens[b];
      if (L < 0 || (long)L > (long)max_blocks * P) return MEPIC_ERR_INVALID;
      lp[b] = (int)std::min<long>((long)L + horizon, (long)max_blocks * P);
      nst[b] = ((lp[b] + P - 1) / P + bps - 1) / bps;
      first[b + 1] = first[b] + nst[b];
    }
    // a step that is not wholly below the kv_len the plan is built from: the ragged last step and what lies ahead
    auto is_tail = [&](int b, int st) { return (st + 1) * 32 > kv_lens[b]; };
    const int total = first[B];
  
    // group id of every step: steps wholly below kv_len whose pages coincide are grouped, at most r_cap requests
    // per group and a request at most once per group. Groups are stored back to back: group g = members
    // gm[goff[g] .. goff[g + 1]), ascending in (request, step).
    std::vector<int> gid(total, -1), goff{0};
    std::vector<StepRef> gm;
    gm.reserve(total);
    goff.reserve(total + 1);
    {
      // steps with the same pages, as singly linked lists in ascending (request, step) order; the lists' heads sit in
      // an open-addressing table keyed by the pages
      size_t cap = 64;
      while (cap < 2 * (size_t)total) cap <<= 1;
      std::vector<uint64_t> slot_key(cap);
      std::vector<int> slot_head(cap, -1), next(total, -1);
      std::vector<StepRef> ref(total);
      for (int b = B - 1; b >= 0; --b)
        for (int s = nst[b] - 1; s >= 0; --s) {
          const int me = first[b] + s;
          ref[me] = {b, s};
          if ((s + 1) * 32 > kv_lens[b]) continue;
          const uint64_t key = key_of(block_tables + (size_t)b * max_blocks + (size_t)s * bps, bps);
          size_t h = (size_t)((key * 0x9e3779b97f4a7c15ull) >> 20) & (cap - 1);
          while (slot_head[h] >= 0 && slot_key[h] != key) h = (h + 1) & (cap - 1);
          slot_key[h] = key;
          next[me] = slot_head[h];  // -1 for the first of its kind
          slot_head[h] = me;
        }
      for (int b = 0; b < B; ++b)  // deterministic order: by first member
        for (int s = 0; s < nst[b]; ++s) {
          const int me = first[b] + s;
          if (gid[me] >= 0) continue;
          const int g = (int)goff.size() - 1;
          if ((s + 1) * 32 > kv_lens[b]) {  // a ragged last step is a group of its own
            gid[me] = g;
            gm.push_back({b, s});
            goff.push_back((int)gm.size());
            continue;
          }
          // the ungrouped steps of the list from here on (everything before `me` is grouped already); a step that
          // joins the group is unlinked, so that later walks pass over ungrouped steps only
          const size_t at = gm.size();
          int last_b = -1;  // the list is ascending in request: a request's second occurrence follows its first
          for (int m = me, prev = -1; m >= 0 && (int)(gm.size() - at) < r_cap;) {
            const int nx = next[m];
            if (ref[m].b == last_b) {  // a second occurrence in one request waits for a later group
              prev = m;
            } else {
              gid[m] = g;
              gm.push_back(ref[m]);
              last_b = ref[m].b;
              if (prev >= 0) next[prev] = nx;
            }
            m = nx;
          }
          goff.push_back((int)gm.size());
        }
    }
    auto group_size = [&](int g) { return goff[g + 1] - goff[g]; };
  
    // runs: follow a group while all of its members step forward together into one and the same group
    struct Run {
      int n;
      std::vector<StepRef> at;
      std::vector<int> steps;  // gather run: its steps, ascending
    };
    std::vector<Run> runs;
    std::vector<char> done(total, 0);
    for (int b = 0; b < B; ++b)
      for (int s = 0; s < nst[b]; ++s) {
        if (done[first[b] + s]) continue;
        const int g0 = gid[first[b] + s], n0 = group_size(g0);
        const StepRef* m0 = gm.data() + goff[g0];
        Run r{1, std::vector<StepRef>(m0, m0 + n0), {}};
        for (int k = 0; k < n0; ++k) done[first[m0[k].b] + m0[k].s] = 1;
        // With a horizon, every tail step is a run of its own (and so ends up in a gather run, the only kind whose
        // steps are each masked against the call's kv_len); without one, a request's single ragged step may close a
        // longer run, which masks its last step.
        const bool tail_alone = horizon > 0 && is_tail(b, s);
        for (; !tail_alone;) {
          const StepRef lead{m0[0].b, m0[0].s + r.n};
          if (lead.s >= nst[lead.b] || done[first[lead.b] + lead.s]) break;
          if (horizon > 0 && is_tail(lead.b, lead.s)) break;
          const int g = gid[first[lead.b] + lead.s];
          const StepRef* m = gm.data() + goff[g];
          bool same = group_size(g) == n0;
          for (int k = 0; same && k < n0; ++k) same = m[k].b == m0[k].b && m[k].s == m0[k].s + r.n;
          if (!same) break;
          for (int k = 0; k < n0; ++k) done[first[m[k].b] + m[k].s] = 1;
          ++r.n;
        }
        runs.push_back(std::move(r));
      }
  
    // order: per request first the runs it walks alone (a chain: consecutive in the sequence, so that one wave can
    // keep accumulating into one partial result across them), then the shared runs it leads. The short ones among
    // the runs it walks alone are merged into gather runs, whose steps need not be consecutive: a start-up per
    // run costs the kernel about as much as a step.
    int n_gather = 0;
    {
      std::vector<Run> ordered;
      ordered.reserve(runs.size());
      std::vector<std::vector<int>> alone(B), led(B);
      for (int i = 0; i < (int)runs.size(); ++i) (runs[i].at.size() == 1 ? alone : led)[runs[i].at[0].b].push_back(i);
      for (int b = 0; b < B; ++b) {
        std::vector<int> loose;  // ascending: runs were formed in step order
        for (int i : alone[b])
          if (runs[i].n < kPlanGatherBelow)
            for (int j = 0; j < runs[i].n; ++j) loose.push_back(runs[i].at[0].s + j);
        for (size_t o = 0; o < loose.size(); o += kPlanGatherMax) {
          const size_t e = std::min(loose.size(), o + (size_t)kPlanGatherMax);
          ordered.push_back(Run{(int)(e - o), {{b, loose[o]}}, std::vector<int>(loose.begin() + o, loose.begin() + e)});
        }
        n_gather += (int)loose.size();
        for (int i : alone[b])
          if (runs[i].n >= kPlanGatherBelow) ordered.push_back(std::move(runs[i]));
        for (int i : led[b]) ordered.push_back(std::move(runs[i]));
      }
      runs.swap(ordered);
    }
    const int n_runs = (int)runs.size();
    const int W = decode_mfma_waves_per_head(Hkv, fp8);
    if (W > kPlanMaxWaves) return MEPIC_ERR_UNSUPPORTED;
    if (plan_words(n_runs, B, n_gather, W) > capacity_int32) return MEPIC_ERR_CAPACITY;
    int T = 0;
    for (const Run& r : runs) T += r.n;
  
    // Where the W waves of a KV head cut the sequence: by estimated time (unit: 1/16 of an ordinary step), not by
    // step count. A gather step sets Q' up from scratch, and every piece of a run a wave starts costs a start-up.
    // The smallest bound on a wave's time that W waves can meet, by bisection over a greedy fill.
    std::vector<int> cuts(W + 1, T);
    {
      const int c_step = 16, c_gather = fp8 ? MEPIC_PLAN_COST_GATHER_FP8 : MEPIC_PLAN_COST_GATHER_BF16;
      const int c_start = fp8 ? MEPIC_PLAN_COST_START_FP8 : MEPIC_PLAN_COST_START_BF16;
      auto fill = [&](long bound, int* out) {  // waves needed under this bound; out: their first positions
        int w = 0, pos = 0;
        long acc = 0;
        for (const Run& r : runs) {
          const int c = r.steps.empty() ? c_step : c_gather;
          for (int left = r.n; left > 0;) {
            const long room = bound - acc - c_start;
            int fit = room >= c ? (int)std::min<long>(left, room / c) : 0;
            if (fit == 0) {
              if (acc > 0) {  // this wave is full: the run goes to the next one
                if (++w <= W && out) out[w] = pos;
                acc = 0;
                continue;
              }
              fit = 1;  // a bound below one step's cost cannot be met; move on all the same
            }
            acc += c_start + (long)fit * c;
            pos += fit;
            left -= fit;
          }
        }
        return w + (acc > 0 ? 1 : 0);
      };
      long lo = c_start + c_step, hi = (long)T * std::max(c_step, c_gather) + (long)n_runs * c_start + lo;
      while (lo < hi) {
        const long mid = (lo + hi) / 2;
        if (fill(mid, nullptr) <= W) hi = mid; else lo = mid + 1;
      }
      cuts[0] = 0;
      fill(lo, cuts.data());  // waves past the last one needed keep the empty range [T, T)
    }
    auto wave_of = [&](int p) { return (int)(std::upper_bound(cuts.begin(), cuts.end(), p) - cuts.begin()) - 1; };
  
    std::memset(plan_out, 0, plan_words(n_runs, B, n_gather, W) * sizeof(int32_t));
    int32_t* cum = plan_out + plan_off_cum(n_runs);
    int32_t* rw = plan_out + plan_off_runs(n_runs);
    int32_t* n_part = plan_out + plan_off_npart(n_runs);
    int32_t* gather = plan_out + plan_off_gather(n_runs, B);
    int pos = 0, n_splits = 1, n_listed = 0;
    for (int i = 0; i < n_runs;) {
      // a chain: a maximal stretch of consecutive one-request runs of the same request (or one shared run)
      int j = i + 1, len = runs[i].n;
      if (runs[i].at.size() == 1)
        while (j < n_runs && runs[j].at.size() == 1 && runs[j].at[0].b == runs[i].at[0].b) len += runs[j++].n;
      const int head_wave = wave_of(pos);
      const int pieces = wave_of(pos + len - 1) - head_wave + 1;  // waves that touch the chain: one partial result each
      std::vector<int> base(runs[i].at.size());
      for (size_t k = 0; k < runs[i].at.size(); ++k) {
        base[k] = n_part[runs[i].at[k].b];
        n_part[runs[i].at[k].b] += pieces;
        n_splits = std::max(n_splits, (int)n_part[runs[i].at[k].b]);
      }
      for (int q = i; q < j; ++q) {
        const Run& r = runs[q];
        cum[q] = pos;
        int32_t* w = rw + (size_t)q * kPlanRunWords;
        w[0] = (int32_t)r.at.size() | (q > i ? kPlanContinues : 0) | (r.steps.empty() ? 0 : kPlanGather);
        w[kPlanRunWords - 1] = std::max((lp[r.at[0].b] + P - 1) / P - 1, 0);  // clamp for the page-id loads
        for (size_t k = 0; k < r.at.size(); ++k) {
          w[1 + k] = r.at[k].b;
          w[1 + kPlanMaxR + k] = r.steps.empty() ? r.at[k].s : n_listed;
          // the kernel adds its wave index: every run of a chain lands on the chain's slots
          w[1 + 2 * kPlanMaxR + k] = base[k] - head_wave;
        }
        for (int st : r.steps) {
          const int32_t* pages = block_tables + (size_t)r.at[0].b * max_blocks + (size_t)st * bps;
          int32_t* g = gather + (size_t)n_listed++ * kPlanGatherWords;
          // the second block of a request's last step may lie past its blocks: the kernel masks those slots, the
          // page it reads them from only has to exist
          const bool second = bps == 2 && st * bps + 1 < (lp[r.at[0].b] + P - 1) / P;
          g[0] = st; g[1] = pages[0]; g[2] = second ? pages[1] : pages[0];
        }
        pos += r.n;
      }
      i = j;
    }
    cum[n_runs] = pos;
    std::copy(cuts.begin(), cuts.end(), plan_out + plan_off_cuts(n_runs, B, n_gather));
    plan_out[0] = kPlanMagic; plan_out[1] = n_runs; plan_out[2] = T; plan_out[3] = W; plan_out[4] = n_splits;
    plan_out[5] = B; plan_out[6] = r_cap; plan_out[7] = n_gather;
  
    info_out->n_runs = n_runs; info_out->total_steps = T; info_out->n_waves = W; info_out->n_splits = n_splits;
    info_out->r_cap = r_cap; info_out->steps_unbatched = total; info_out->n_int32 = (int32_t)plan_words(n_runs, B, n_gather, W);
    info_out->B = B;
    return MEPIC_OK;
  } catch (const std::bad_alloc&) {  // nothing may throw across the C boundary
    return MEPIC_ERR_NOMEM;
  } catch (...) {
    return MEPIC_ERR_INVALID;
  }
}

}  // extern "C"
