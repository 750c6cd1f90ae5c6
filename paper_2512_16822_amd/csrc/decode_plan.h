// Layout of the plan blob of the batched decode (int32 words), shared by the host planner and the kernel.
//
// A "step" is 32 consecutive slots of a request (two pages of 16 or one page of 32). Steps of different
// requests that read exactly the same pages, and lie wholly below their request's kv_len, can be served by one
// pass over those pages: the matrix-core tile has 16 rows and a request needs only G of them. A "run" is a
// sequence of consecutive steps over which the same group of up to 16/G requests moves in lockstep (request i of
// the group is at step step0[i] + j when the run is at its j-th step). Every (request, step) belongs to exactly
// one run; steps nobody shares form runs of one request.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mepic {

constexpr int kPlanMagic = 0x4d455049;  // "MEPI"
constexpr int kPlanHeader = 8;          // magic, n_runs, total_steps, chunk, n_splits, B, r_cap, 0
constexpr int kPlanMaxR = 16;
constexpr int kPlanRunWords = 1 + 3 * kPlanMaxR;  // R, req[16], step0[16], slot[16]

// word offsets inside the blob
__host__ __device__ inline int plan_off_cum(int) { return kPlanHeader; }                                    // run_cum[n_runs + 1]
__host__ __device__ inline int plan_off_runs(int n_runs) { return kPlanHeader + n_runs + 1; }               // runs[n_runs][kPlanRunWords]
__host__ __device__ inline int plan_off_npart(int n_runs) { return plan_off_runs(n_runs) + n_runs * kPlanRunWords; }  // n_part[B]
__host__ __device__ inline size_t plan_words(int n_runs, int B) { return (size_t)plan_off_npart(n_runs) + B; }

}  // namespace mepic
