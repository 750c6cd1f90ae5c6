// Layout of the plan blob of the batched decode (int32 words), shared by the host planner and the kernel.
//
// A "step" is 32 consecutive slots of a request (two pages of 16 or one page of 32). Steps of different
// requests that read exactly the same pages, and lie wholly below their request's kv_len, can be served by one
// pass over those pages: the matrix-core tile has 16 rows and a request needs only G of them. A "run" is a
// sequence of consecutive steps over which the same group of up to 16/G requests moves in lockstep (request i of
// the group is at step step0[i] + j when the run is at its j-th step). Every (request, step) belongs to exactly
// one run; steps nobody shares form runs of one request. Short stretches of those (a request's private first
// blocks between shared chunks, its ragged last step) are collected into "gather" runs: one request, steps in
// ascending order but not consecutive, listed with their pages in the blob's gather section.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mepic {

constexpr int kPlanMagic = 0x4d455049;  // "MEPI"
constexpr int kPlanHeader = 8;          // magic, n_runs, total_steps, n_waves, n_splits, B, r_cap, n_gather
constexpr int kPlanMaxWaves = 4096;     // bound on n_waves (waves that share one KV head's sequence)
constexpr int kPlanMaxR = 16;
// A run: R | flags, req[16], step0[16], slot[16], last block of req[0]. The wave with index w among the waves of
// its KV head writes the partial result of request req[i] to slot slot[i] + w of that request.
constexpr int kPlanRunWords = 2 + 3 * kPlanMaxR;
constexpr int kPlanContinues = 0x100;  // flag in word 0: this one-request run continues the previous run's partial result
constexpr int kPlanGather = 0x200;     // flag in word 0: a gather run; step0[0] is the index of its first gather entry
constexpr int kPlanGatherWords = 3;    // a gather entry: step, its first page, its second page (= the first when a step is one page)
constexpr int kPlanGatherMax = 64;     // steps per gather run at most
constexpr int kPlanGatherBelow = 4;    // one-request runs shorter than this are gathered

// word offsets inside the blob
__host__ __device__ inline int plan_off_cum(int) { return kPlanHeader; }                                    // run_cum[n_runs + 1]
__host__ __device__ inline int plan_off_runs(int n_runs) { return kPlanHeader + n_runs + 1; }               // runs[n_runs][kPlanRunWords]
__host__ __device__ inline int plan_off_npart(int n_runs) { return plan_off_runs(n_runs) + n_runs * kPlanRunWords; }  // n_part[B]
__host__ __device__ inline int plan_off_gather(int n_runs, int B) { return plan_off_npart(n_runs) + B; }  // gather[n_gather][kPlanGatherWords]
// cuts[n_waves + 1]: wave w walks positions cuts[w] .. cuts[w + 1] of the sequence of runs; the planner places the
// cuts so that the waves' estimated times, not their step counts, come out equal
__host__ __device__ inline size_t plan_off_cuts(int n_runs, int B, int n_gather) {
  return (size_t)plan_off_gather(n_runs, B) + (size_t)n_gather * kPlanGatherWords;
}
__host__ __device__ inline size_t plan_words(int n_runs, int B, int n_gather, int n_waves) {
  return plan_off_cuts(n_runs, B, n_gather) + (size_t)n_waves + 1;
}

}  // namespace mepic
