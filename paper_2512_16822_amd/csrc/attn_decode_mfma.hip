// Matrix-core decode kernels of fused-RoPE paged attention (§3.3.3), D = 128:
//   bf16 K/V pages of 16 slots (a step = two pages), and
//   fp8 e4m3 K/V pages of 32 slots with one fp32 scale per page for K and for V (a step = one page).
// The text below describes the bf16 kernel; the fp8 variant differs where noted at the end.
//
// Persistent waves, stream-K over pages. The grid is two workgroups of four waves per compute unit (two waves
// per SIMD). Workgroup g serves KV head g % Hkv (consecutive workgroups land on consecutive
// XCDs, so one KV head's pages stay in one XCD's L2). For one KV head the "steps" (two pages = 32
// slots) of all requests form one sequence of length T; the waves of that head cut it into equal
// contiguous chunks, regardless of request boundaries. A wave writes one partial (max, sum,
// un-normalised output) per request it touched; a second kernel merges the partials of each
// (request, head).
//
// Everything a step needs comes straight from HBM into registers as aligned 16-byte loads that
// already are matrix-core operands (that is what the page layouts are for):
//
//   S^T[32 slots x 16 heads] = Khat[32 x 128] * Q'^T[128 x 16]     2 x 4 v_mfma_f32_16x16x32_bf16
//   O  [16 heads x 128]     += P[16 x 32 slots] * V[32 x 128]      8     v_mfma_f32_16x16x32_bf16
//
// fp8: K and V of the next step are in flight in a second register buffer while a step is computed; bf16 has
// room for one buffer only (two waves per SIMD leave 256 registers each) and counts on the SIMD's other wave.
//
// Rotary embedding without per-key trigonometry: a key at position n0 + s (n0 = first slot of the
// step) has  q^.k^ = (R(pos_q - n0) q) . (R(s) k).  R(s), s in [0, 32), is a per-lane constant (each
// lane always handles the same two slot offsets and the same 16 frequencies) read from LDS, so a key
// costs one constant 2x2 rotation per element pair (in the plain walker two two-term dot products per pair,
// v_dot2_f32_bf16, on words that v_perm_b32 assembles from the pair's two granules); Q' = R(pos_q - n0) q is
// advanced by a constant rotation (with two tables of slot rotations, R(s) and R(s + 32), only every second
// step, by R(-64)).
//
// The 16 matrix rows of the QK product are the slots {0-3, 8-11, 16-19, 24-27} (+4 for the second
// product), which makes each lane end up with the scores of 8 consecutive slots of one page for one
// head — exactly the A operand of the PV product, so probabilities never leave their lane, and the
// matching V operand is one contiguous 16-byte piece of a V page row.
//
// fp8 variant: a lane owns dims 16kg..16kg+15 and 64+16kg.. (two 16-byte K granules per row). K codes are
// widened to packed fp16 (v_cvt_scalef32_pk_f16_fp8, exact), rotated with packed fp16 arithmetic (two element
// pairs per instruction; the rotation constants are stored as fp16 pairs) and go into fp16 QK products
// (v_mfma_f32_16x16x32_f16) against Q' rounded to fp16; the page's K scale multiplies the scores. There are
// four slot-rotation tables, R(s), R(s+32), R(s+64), R(s+96): step j uses table j mod 4 and Q' advances by
// R(-128) once every four steps, because in this variant the advance sits on the critical path of an otherwise
// memory-bound loop. V is never widened: PV runs on v_mfma_f32_16x16x32_fp8_fp8 with the V bytes as loaded
// (8 bytes per lane and column tile) and the probabilities split into two e4m3 terms (p*4 = hi + lo, 8
// significant bits together); the page's V scale rides on the probabilities, O being kept in units of a
// reference scale that is raised (with a rescale of O) only when a page's scale exceeds it by 1.75 x.
//
// Batched variant (kBatched): the sequence a KV head's waves share is not the list of requests but a host-built
// plan of "runs", groups of up to 16/G requests that read identical pages for a number of consecutive steps (the
// tile's 16 rows then hold G heads of each of them: K is loaded and rotated once for all, every request has its
// own Q'), plus "gather runs" that collect a request's scattered unshared steps. Its walker prefetches the plan
// words, page ids and first K/V loads of the next piece of work while the current one is computed, and the
// planner, not the kernel, places the cuts between the waves.
#include <type_traits>

#include "attn_common.h"
#include "decode_plan.h"

namespace mepic {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128;
constexpr int kWaves = 4;             // waves per workgroup
// Workgroups resident per compute unit: two, i.e. two waves per SIMD, which fill the issue slots each other leaves
// while waiting on matrix-core, LDS and memory results. For that a wave has to fit 256 registers: the fp8 kernel
// does with two register buffers of K and V (the next step's pages in flight while a step is computed); the bf16
// kernel, whose buffers are twice as large, keeps one (a step's loads are issued, then waited for: the other
// wave computes meanwhile). Measured against one wave per SIMD with two buffers (bf16): 84 instead of 105 us on
// the page-sharing layout of the Llama-3-8B decode workload, the same on the layout where every byte comes from
// HBM, 347 instead of 421 us on the 8 x 65 537-slot workload.
#ifndef MEPIC_DECODE_WG_PER_CU_BF16
#define MEPIC_DECODE_WG_PER_CU_BF16 2
#endif
#ifndef MEPIC_DECODE_WG_PER_CU_FP8
#define MEPIC_DECODE_WG_PER_CU_FP8 2
#endif
#ifndef MEPIC_DECODE_WG_PER_CU_FP8_BATCHED
#define MEPIC_DECODE_WG_PER_CU_FP8_BATCHED 2
#endif
constexpr int wg_per_cu(bool fp8, bool batched = false) {
  return fp8 ? (batched ? MEPIC_DECODE_WG_PER_CU_FP8_BATCHED : MEPIC_DECODE_WG_PER_CU_FP8) : MEPIC_DECODE_WG_PER_CU_BF16;
}
#ifndef MEPIC_DECODE_NBUF_BF16
#define MEPIC_DECODE_NBUF_BF16 1
#endif
#ifndef MEPIC_DECODE_NBUF_FP8
#define MEPIC_DECODE_NBUF_FP8 2
#endif
// register buffers of K and V per wave of the plain walker (prefetch depth + 1)
constexpr int n_buf(bool fp8) { return fp8 ? MEPIC_DECODE_NBUF_FP8 : MEPIC_DECODE_NBUF_BF16; }
constexpr float kRescaleSlack = 6.f;  // the running maximum may lag the true one by this much (log2 units)

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

union Frag {  // one 16-byte operand fragment
  uint4 u;
  bf16x8 v;
  f16x8 hv;
  uint32_t w[4];
};

// Two fp32 -> packed fp16 pair, round to nearest even.
__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// Two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// A page id as the kernels use it: forced into [0, num_pages) so that a corrupt block table reads a wrong page
// instead of faulting (the result of that request is then unspecified, nothing else is affected).
__device__ __forceinline__ int safe_page(int id, int num_pages) { return max(min(id, num_pages - 1), 0); }

// 16- and 8-byte loads of page data, optionally with the non-temporal hint (the line is not kept in the caches):
// right when every page is read by one request only, wrong when pages are shared between requests.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
template <bool kNT>
__device__ __forceinline__ uint4 load_page(const uint4* p) {
  if constexpr (kNT) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v[0], v[1], v[2], v[3]);
  } else {
    return *p;
  }
}
template <bool kNT>
__device__ __forceinline__ uint2 load_page(const uint2* p) {
  if constexpr (kNT) {
    const u32x2_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
    return make_uint2(v[0], v[1]);
  } else {
    return *p;
  }
}

// Wave-uniform read of a read-only int32 input through the scalar unit (s_load): unlike a vector load it
// does not share the vector-memory counter, so waiting for it never drains the K/V loads in flight.
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
__device__ __forceinline__ int sload(const int32_t* p, size_t idx) {
  return ((const_i32_ptr)(uintptr_t)p)[idx];
}

typedef const __attribute__((address_space(4))) float* const_f32_ptr;
__device__ __forceinline__ float sloadf(const float* p, size_t idx) { return ((const_f32_ptr)(uintptr_t)p)[idx]; }

// Maximum over the four lanes l, l^16, l^32, l^48 (the four k-groups of one head), in every lane.
__device__ __forceinline__ float max_over_kgroups(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const uint32_t v = __float_as_uint(y);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float sum_over_kgroups(float x) {
  const uint32_t u = __float_as_uint(x);
  const auto a = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const float y = __uint_as_float(a[0]) + __uint_as_float(a[1]);
  const uint32_t v = __float_as_uint(y);
  const auto b = __builtin_amdgcn_permlane32_swap(v, v, false, false);
  return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Eight two-term dot products on packed bf16 words, fp32 results: l_i = e_i . ca_i, h_i = e_i . cb_i, where
// e_i = (low element, high element) of a rotary pair and ca = (cos, -sin), cb = (sin, cos) as packed bf16.
// One block of eight v_dot2_f32_bf16 closed by four wait states: another vector instruction may neither read the
// result of a dot instruction for three wait states nor rewrite its register for four, and the compiler places those
// only around its own builtin. Within the block no dot reads or rewrites another's result; the outputs are
// early-clobber, so none shares a register with an input. Validated on ROCm 7.2 (AMD clang 22, gfx950); the
// library's self-test entry point runs this block alone against fp32 arithmetic so that a toolchain that breaks the
// rule shows up as a failed test and not as slightly wrong attention.
__device__ __forceinline__ void dot_rotate_block(uint32_t e0, uint32_t e1, uint32_t e2, uint32_t e3, uint32_t ca0,
                                                 uint32_t cb0, uint32_t ca1, uint32_t cb1, uint32_t ca2, uint32_t cb2,
                                                 uint32_t ca3, uint32_t cb3, float& l0, float& l1, float& l2, float& l3,
                                                 float& h0, float& h1, float& h2, float& h3) {
  asm("v_dot2_f32_bf16 %0, %8, %12, 0\n\t"
      "v_dot2_f32_bf16 %1, %9, %14, 0\n\t"
      "v_dot2_f32_bf16 %2, %10, %16, 0\n\t"
      "v_dot2_f32_bf16 %3, %11, %18, 0\n\t"
      "v_dot2_f32_bf16 %4, %8, %13, 0\n\t"
      "v_dot2_f32_bf16 %5, %9, %15, 0\n\t"
      "v_dot2_f32_bf16 %6, %10, %17, 0\n\t"
      "v_dot2_f32_bf16 %7, %11, %19, 0\n\t"
      "s_nop 3"
      : "=&v"(l0), "=&v"(l1), "=&v"(l2), "=&v"(l3), "=&v"(h0), "=&v"(h1), "=&v"(h2), "=&v"(h3)
      : "v"(e0), "v"(e1), "v"(e2), "v"(e3), "v"(ca0), "v"(cb0), "v"(ca1), "v"(cb1), "v"(ca2), "v"(cb2), "v"(ca3),
        "v"(cb3));
}

constexpr float kPScaleFp8 = 4.f;     // probabilities (< 2^slack = 64) are multiplied by this before the e4m3 split

// kBatched: the sequence a KV head's waves cut into chunks is the plan's list of runs (groups of up to 16/G
// requests stepping through identical pages together) instead of the list of requests; a lane's matrix row then
// belongs to request row / G of the run.
// kReadOnce: the caller's hint that pages are not shared between the requests of the call. V is then loaded
// non-temporally (every V load instruction consumes whole 128-byte lines, so nothing is lost by not keeping them).
// K keeps ordinary loads: the slot order that makes a lane's scores eight consecutive slots of a page lets one K load
// instruction touch only half of each line it addresses and the next one the other half - with the hint a line was
// sometimes gone in between and came from HBM twice (6-7 % more traffic, and slower than hinting V alone).
template <bool kFp8, bool kBatched, bool kReadOnce = false>
__global__ __launch_bounds__(64 * kWaves, wg_per_cu(kFp8, kBatched)) void decode_mfma_kernel(const AttnArgs a) {
  constexpr int kP = kFp8 ? 32 : 16;          // slots per page
  constexpr int kBps = kFp8 ? 1 : 2;          // blocks (pages) per step of 32 slots
  constexpr int kNK = kFp8 ? 2 : 4;           // 16-byte K fragments per lane and product
  typedef typename std::conditional<kFp8, uint2, uint4>::type VRaw;  // V fragment per lane and column tile
  // Rotation constants, identical for every wave: one float4 {c0, s0, c1, s1} per lane and element pair.
  // kNV tables R(slot32 + 32 v), v < kNV (fp8 entries: {packed fp16 cos pair, sin pair}); step j uses table
  // j mod kNV and Q' advances by R(-32 kNV) once every kNV steps only: fewer vector instructions per step, which
  // is what limits the loop whenever the pages come from the caches (shared pages) rather than from HBM.
  // bf16 keeps fp32 constants, so two tables are what fits beside the rest in 64 KB of static LDS.
  constexpr int kNV = kFp8 ? 4 : 2;
  // bf16, plain walker: keys are rotated with two-term dot products (v_dot2_f32_bf16) on (low, high) element pairs,
  // 9 instead of 14 vector instructions per two pairs; the batched walker, short of registers, keeps fp32 arithmetic
  constexpr bool kDotRot = !kFp8 && !kBatched;
  typedef typename std::conditional<kFp8, float2, float4>::type RotK;
  __shared__ RotK rotK[kNV * 16][64];  // slot rotation: index v*16 + (u*2 + h)*4 + w
  __shared__ float4 rotS[8][64];       // step rotation R(-32 kNV): index h*4 + w
  __shared__ float2 freq_lds[kBatched ? 64 : 1];  // batched: {hi, lo} of the frequencies, index kg*16 + pair
  __shared__ uint4 q_lds[kBatched ? kWaves * 4 : 1][64];  // batched: q of the current piece, [wave*4 + fragment][lane]
  extern __shared__ int cum[];     // cum[b] = steps of the requests before b; B + 1 entries

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n16 = lane & 15, kg = lane >> 4;
  const int G = a.G, Hkv = a.Hkv;

  // ---- cum[]: steps before each item of the sequence (requests, or the plan's runs) ----
  const int n_items = kBatched ? sload(a.plan, 1) : a.B;
  if constexpr (kBatched) {
    for (int i = tid; i <= n_items; i += 64 * kWaves) cum[i] = a.plan[plan_off_cum(n_items) + i];
  } else if (wave == 0) {
    // from kv_lens (a step = two blocks); one wave scans
    int carry = 0;
    for (int base = 0; base < a.B; base += 64) {
      const int b = base + lane;
      int x = 0;
      if (b < a.B) x = ((a.kv_lens[b] + kP - 1) / kP + kBps - 1) / kBps;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(x, o);
        if (lane >= o) x += y;
      }
      if (b < a.B) cum[b + 1] = carry + x;
      carry += __shfl(x, 63);
    }
    if (lane == 0) cum[0] = 0;
  }
  // ---- rotation constants. As holder of K rows, row n16 of product u is slot32 = 8*(n16/4) + 4u + n16%4 of
  // the step. A lane owns 16 rotary pairs p = 8h + e (h in {0,1}, e < 8): frequency i(p) = 32h + 8kg + e for
  // bf16 (dims i and i + 64 sit in k-steps h and h + 2), i(p) = 16kg + p for fp8. ----
  auto freq_of = [&](int pidx) { return kFp8 ? 16 * kg + pidx : 32 * (pidx >> 3) + 8 * kg + (pidx & 7); };
  const int slot_u0 = 8 * (n16 >> 2) + (n16 & 3);
  if constexpr (kBatched) {
    // a piece of a run starts every few steps: its Q' set-up reads the frequencies from LDS, not from memory
    if (wave == 0) {
      const int i = freq_of(n16);  // lane (kg, n16) fills entry kg*16 + n16
      freq_lds[lane] = make_float2(a.freq_hi[i], a.freq_lo[i]);
    }
  }
  for (int idx = wave; idx < kNV * 16 + 8; idx += kWaves) {
    const bool is_k = idx < kNV * 16;
    const int h = (idx >> 2) & 1, w = idx & 3;  // idx = v*16 + (u*2 + h)*4 + w for rotK, kNV*16 + h*4 + w for rotS
    const float pos = is_k ? (float)(slot_u0 + 4 * ((idx >> 3) & 1) + 32 * (idx >> 4)) : -32.0f * kNV;
    const int i = freq_of(8 * h + 2 * w);     // pairs 8h + 2w and 8h + 2w + 1 have consecutive frequencies
    const float t0 = turns_frac(pos, a.freq_hi[i], a.freq_lo[i]);
    const float t1 = turns_frac(pos, a.freq_hi[i + 1], a.freq_lo[i + 1]);
    const float4 r = make_float4(__builtin_amdgcn_cosf(t0), __builtin_amdgcn_sinf(t0), __builtin_amdgcn_cosf(t1),
                                 __builtin_amdgcn_sinf(t1));
    if (!is_k) {
      rotS[idx - kNV * 16][lane] = r;
    } else if constexpr (kFp8) {  // fp8 keys are rotated in packed fp16: {cos pair, sin pair} as two words
      rotK[idx][lane] = make_float2(__uint_as_float(pack_f16x2(r.x, r.z)), __uint_as_float(pack_f16x2(r.y, r.w)));
    } else if constexpr (kDotRot) {
      // per pair the two constant words (cos, -sin) and (sin, cos) as packed bf16
      rotK[idx][lane] = make_float4(__uint_as_float(pack_bf16x2(r.x, -r.y)), __uint_as_float(pack_bf16x2(r.y, r.x)),
                                    __uint_as_float(pack_bf16x2(r.z, -r.w)), __uint_as_float(pack_bf16x2(r.w, r.z)));
    } else {
      rotK[idx][lane] = r;
    }
  }
  __syncthreads();

  const int T = uni(cum[n_items]);
  const int hk = (int)blockIdx.x % Hkv;
  const int wk = ((int)blockIdx.x / Hkv) * kWaves + wave, n_k = ((int)gridDim.x / Hkv) * kWaves;
  // blocks_per_split carries the minimum chunk
  const int chunk = kBatched ? 0 : max((T + n_k - 1) / n_k, a.blocks_per_split);
  if (!kBatched && blockIdx.x == 0 && wave == 0) {  // what the merge kernel needs to find each request's partials
    for (int i = lane; i <= a.B; i += 64) a.part_meta[i] = cum[i];
    if (lane == 0) a.part_meta[a.B + 1] = chunk;
  }
  int pos_begin = wk * chunk, pos_end = min(pos_begin + chunk, T);
  if constexpr (kBatched) {  // the planner placed the cuts between the waves (the host checked n_k against the plan)
    const int32_t* cuts = a.plan + plan_off_cuts(n_items, a.B, sload(a.plan, 7));
    pos_begin = sload(cuts, wk);
    pos_end = sload(cuts, wk + 1);
  }
  if (pos_begin >= pos_end) return;

  const uint4* kpages = reinterpret_cast<const uint4*>(a.k_pages);
  const VRaw* vpages = reinterpret_cast<const VRaw*>(a.v_pages);
  const uint4* q4 = reinterpret_cast<const uint4*>(a.q);

  floatx4 o[8];
  float m_run, l_part;
  float v_ref = 0.f;  // fp8: O is kept in units of this reference V scale (wave-uniform), raised lazily
  float qlo[2][8], qhi[2][8];  // Q' of head n16 for the lane's 16 rotary pairs [h][e], in log2 units

  // K fragments of product u (row = slot slot_u0 + 4u of the step):
  //   bf16: kf[u][j] = granule (4j + kg) of the row, j < 4 (page p0 for rows 0-7, p1 for rows 8-15);
  //   fp8:  kf[u][0] = granule kg (dims 16kg..), kf[u][1] = granule kg + 4 (dims 64 + 16kg..) of page p0.
  auto issue_k = [&](Frag (&kf)[2][kNK], int p0, int p1) __attribute__((always_inline)) {
    if constexpr (kFp8) {
      const size_t kb = ((size_t)p0 * Hkv + hk) * (kD / 16 * kP) + (size_t)kg * kP + slot_u0;
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int j = 0; j < 2; ++j) kf[u][j].u = load_page<false>(&kpages[kb + (size_t)(4 * j) * kP + 4 * u]);
    } else {
      const int pk = (n16 < 8) ? p0 : p1;
      const size_t kb = ((size_t)pk * Hkv + hk) * (kD / 8 * kP) + (size_t)kg * kP + (slot_u0 & 15);
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int j = 0; j < 4; ++j) kf[u][j].u = load_page<false>(&kpages[kb + (size_t)(4 * j) * kP + 4 * u]);
    }
  };
  // V fragments, column tile nt = dim 16nt + n16: bf16: slots 8*(kg&1).. of page kg/2 (16 bytes);
  // fp8: slots 8kg.. of the page (8 bytes).
  auto issue_v = [&](VRaw (&vf)[8], int p0, int p1) __attribute__((always_inline)) {
    if constexpr (kFp8) {
      const size_t vb = (((size_t)p0 * Hkv + hk) * kD + n16) * 4 + kg;
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) vf[nt] = load_page<kReadOnce>(&vpages[vb + (size_t)nt * 64]);
    } else {
      const int pv = (kg < 2) ? p0 : p1;
      const size_t vb = (((size_t)pv * Hkv + hk) * kD + n16) * 2 + (kg & 1);
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) vf[nt] = load_page<kReadOnce>(&vpages[vb + (size_t)nt * 32]);
    }
  };

  // One step: 32 slots starting at logical slot n0. `ragged` marks the request's last step when it reaches
  // past kv_len L. ksc / vsc: the page's K and V scales (fp8; 1 for bf16).
  auto compute = [&](Frag (&kf)[2][kNK], VRaw (&vf)[8], int n0, int st, int L, bool ragged, float ksc, float vsc)
      __attribute__((always_inline)) {
    // Q' as the B operand of the QK products
    Frag bq[4];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        bq[h].w[e / 2] = kFp8 ? pack_f16x2(qlo[h][e], qlo[h][e + 1]) : pack_bf16x2(qlo[h][e], qlo[h][e + 1]);
        bq[h + 2].w[e / 2] = kFp8 ? pack_f16x2(qhi[h][e], qhi[h][e + 1]) : pack_bf16x2(qhi[h][e], qhi[h][e + 1]);
      }
    // Rotate the K rows by their constant slot rotation and run the two QK products, then advance Q' by
    // R(-32). Six groups of four constants each; the constants of the next group are fetched from LDS while a
    // group is computed, and scheduling barriers keep the groups apart so that only two sets are ever live.
    floatx4 sc[2];
    const int tv = kNV > 1 ? (st & (kNV - 1)) * 16 : 0;  // which slot-rotation table this step uses
    RotK rc[2][4];
#pragma unroll
    for (int w = 0; w < 4; ++w) rc[0][w] = rotK[tv + w][lane];
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
      RotK (&r)[4] = rc[grp & 1];
      if (grp + 1 < 4) {
#pragma unroll
        for (int w = 0; w < 4; ++w) rc[(grp + 1) & 1][w] = rotK[tv + (grp + 1) * 4 + w][lane];
      }
      {
        const int u = grp >> 1, h = grp & 1;
        if (h == 0) sc[u] = floatx4{0.f, 0.f, 0.f, 0.f};
        Frag klo, khi;
        if constexpr (kFp8) {
          // e4m3 codes -> packed fp16 (exact), rotated with packed fp16 arithmetic (two pairs per instruction;
          // fp16 keeps 11 significant bits, more than the bf16 operands of the bf16 path), fp16 products
#pragma unroll
          for (int w = 0; w < 4; ++w) {  // pairs 8h + 2w and 8h + 2w + 1
            const uint32_t wl = kf[u][0].w[2 * h + (w >> 1)], wh = kf[u][1].w[2 * h + (w >> 1)];
            const f16x2 lo = (w & 1) ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wl, 1.0f, true)
                                     : __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wl, 1.0f, false);
            const f16x2 hi = (w & 1) ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wh, 1.0f, true)
                                     : __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(wh, 1.0f, false);
            const f16x2 c2 = __builtin_bit_cast(f16x2, __float_as_uint(r[w].x));
            const f16x2 s2 = __builtin_bit_cast(f16x2, __float_as_uint(r[w].y));
            klo.w[w] = __builtin_bit_cast(uint32_t, lo * c2 - hi * s2);
            khi.w[w] = __builtin_bit_cast(uint32_t, hi * c2 + lo * s2);
          }
          sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(klo.hv, bq[h].hv, sc[u], 0, 0, 0);
          sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_f16(khi.hv, bq[h + 2].hv, sc[u], 0, 0, 0);
        } else if constexpr (kDotRot) {
#pragma unroll
          for (int w = 0; w < 4; w += 2) {  // pairs 8h + 2w .. 8h + 2w + 3
            // Bring the low and the high element of a pair into one word (v_perm_b32); each rotated element is then
            // one two-term dot product with a constant word, (cos, -sin) or (sin, cos), accumulated in fp32.
            const uint32_t la = kf[u][h].w[w], ha = kf[u][h + 2].w[w], lb = kf[u][h].w[w + 1], hb = kf[u][h + 2].w[w + 1];
            const uint32_t e0 = __builtin_amdgcn_perm(ha, la, 0x05040100u), e1 = __builtin_amdgcn_perm(ha, la, 0x07060302u);
            const uint32_t e2 = __builtin_amdgcn_perm(hb, lb, 0x05040100u), e3 = __builtin_amdgcn_perm(hb, lb, 0x07060302u);
            float l0, l1, l2, l3, h0, h1, h2, h3;
            dot_rotate_block(e0, e1, e2, e3, __float_as_uint(r[w].x), __float_as_uint(r[w].y), __float_as_uint(r[w].z),
                             __float_as_uint(r[w].w), __float_as_uint(r[w + 1].x), __float_as_uint(r[w + 1].y),
                             __float_as_uint(r[w + 1].z), __float_as_uint(r[w + 1].w), l0, l1, l2, l3, h0, h1, h2, h3);
            klo.w[w] = pack_bf16x2(l0, l1);
            klo.w[w + 1] = pack_bf16x2(l2, l3);
            khi.w[w] = pack_bf16x2(h0, h1);
            khi.w[w + 1] = pack_bf16x2(h2, h3);
          }
          sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(klo.v, bq[h].v, sc[u], 0, 0, 0);
          sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(khi.v, bq[h + 2].v, sc[u], 0, 0, 0);
        } else {
#pragma unroll
          for (int w = 0; w < 4; ++w) {  // pairs 8h + 2w and 8h + 2w + 1
            const uint32_t lo2 = kf[u][h].w[w], hi2 = kf[u][h + 2].w[w];
            const float l0 = bf16_bits_to_f32(lo2 & 0xffffu), l1 = __uint_as_float(lo2 & 0xffff0000u);
            const float h0 = bf16_bits_to_f32(hi2 & 0xffffu), h1 = __uint_as_float(hi2 & 0xffff0000u);
            klo.w[w] = pack_bf16x2(l0 * r[w].x - h0 * r[w].y, l1 * r[w].z - h1 * r[w].w);  // r = {c0, s0, c1, s1}
            khi.w[w] = pack_bf16x2(h0 * r[w].x + l0 * r[w].y, h1 * r[w].z + l1 * r[w].w);
          }
          sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(klo.v, bq[h].v, sc[u], 0, 0, 0);
          sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(khi.v, bq[h + 2].v, sc[u], 0, 0, 0);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // advance Q' by R(-32 kNV) after the last step that uses it
    if (kNV == 1 || (st & (kNV - 1)) == kNV - 1) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float4 r[4];
#pragma unroll
        for (int w = 0; w < 4; ++w) r[w] = rotS[h * 4 + w][lane];
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float a0 = qlo[h][2 * w], b0 = qhi[h][2 * w], a1 = qlo[h][2 * w + 1], b1 = qhi[h][2 * w + 1];
          qlo[h][2 * w] = a0 * r[w].x - b0 * r[w].y;
          qhi[h][2 * w] = b0 * r[w].x + a0 * r[w].y;
          qlo[h][2 * w + 1] = a1 * r[w].z - b1 * r[w].w;
          qhi[h][2 * w + 1] = b1 * r[w].z + a1 * r[w].w;
        }
      }
    }
    if constexpr (kFp8) {
      sc[0] *= ksc;
      sc[1] *= ksc;
    }
    // lane (head n16, kg) now holds the scores of slots n0 + 8kg + 4u + e
    // (a step wholly past kv_len, which a plan built ahead can hold, may read a page nobody has written yet: its V scale
    // must not reach the arithmetic; its scores and V bytes are masked below like any slot past kv_len)
    if (kFp8 && ragged && n0 >= L) vsc = v_ref;
    if (ragged) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n0 + 8 * kg + 4 * u + e >= L) sc[u][e] = -INFINITY;
      // slots at or past kv_len may hold anything (even NaN): zero them in V
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) {
        if constexpr (kFp8) {
          uint32_t keep[2];
#pragma unroll
          for (int w = 0; w < 2; ++w) {
            keep[w] = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) keep[w] |= (n0 + 8 * kg + 4 * w + e < L) ? (0xffu << (8 * e)) : 0u;
          }
          vf[nt].x &= keep[0];
          vf[nt].y &= keep[1];
        } else {
          uint32_t* vw = reinterpret_cast<uint32_t*>(&vf[nt]);
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const int n = n0 + 8 * kg + 2 * w;
            vw[w] &= (n < L ? 0x0000ffffu : 0u) | (n + 1 < L ? 0xffff0000u : 0u);
          }
        }
      }
    }
    const float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                           fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    // The reference maximum only has to bound the scores from above up to a fixed slack (probabilities stay
    // below 2^slack); it is raised, and everything accumulated so far rescaled, only when some score gets
    // past that. Rare after the first steps, so the cross-lane work sits inside the branch.
    if (__any(mx > m_run + kRescaleSlack)) {
      const float m_new = fmaxf(m_run, max_over_kgroups(mx));
      const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_part *= alpha;
      // accumulator rows of this lane are heads 4kg + e; their factors live in lanes 4kg + e
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float ar = __shfl(alpha, 4 * kg + e);
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) o[nt][e] *= ar;
      }
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    float pf[8];  // probabilities of slots n0 + 8kg + e', e' = 4u + e
    float psum = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        pf[4 * u + e] = __builtin_amdgcn_exp2f(sc[u][e] - m_use);
        psum += pf[4 * u + e];
      }
    l_part += psum;
    if constexpr (kFp8) {
      // The page's V scale rides on the probabilities: O accumulates in units of a reference scale v_ref that is
      // at least vsc / 1.75, raised (with a rescale of O) only when a page's scale exceeds that; then
      // p * 4 * vsc / v_ref = hi + lo, both e4m3: p < 2^slack = 64, so the product stays below 448, the largest
      // e4m3 value. Pages with a much smaller scale lose relative precision in proportion to how little they add.
      if (vsc > 1.75f * v_ref) {  // wave-uniform
        const float f = v_ref / vsc;  // 0 on the first page
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) o[nt] *= f;
        v_ref = vsc;
      }
      // (one v_rcp_f32, good to an ulp, instead of a correctly rounded division: this runs every step)
      const float ps = v_ref > 0.f ? kPScaleFp8 * vsc * __builtin_amdgcn_rcpf(v_ref) : 0.f;  // a zero scale means an all-zero page
      uint32_t hi[2], lo[2];
#pragma unroll
      for (int w = 0; w < 2; ++w) {
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) x[e] = pf[4 * w + e] * ps;
        int hw = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], 0, false);
        hw = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], hw, true);
        const f32x2 b0 = __builtin_amdgcn_cvt_pk_f32_fp8(hw, false), b1 = __builtin_amdgcn_cvt_pk_f32_fp8(hw, true);
        int lw = __builtin_amdgcn_cvt_pk_fp8_f32(x[0] - b0[0], x[1] - b0[1], 0, false);
        lw = __builtin_amdgcn_cvt_pk_fp8_f32(x[2] - b1[0], x[3] - b1[1], lw, true);
        hi[w] = (uint32_t)hw;
        lo[w] = (uint32_t)lw;
      }
      const long a_hi = (long)(((uint64_t)hi[1] << 32) | hi[0]), a_lo = (long)(((uint64_t)lo[1] << 32) | lo[0]);
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) {
        const long vb = (long)(((uint64_t)vf[nt].y << 32) | vf[nt].x);
        o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a_hi, vb, o[nt], 0, 0, 0);
        o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_fp8_fp8(a_lo, vb, o[nt], 0, 0, 0);
      }
    } else {
      Frag pa;
#pragma unroll
      for (int w = 0; w < 4; ++w) pa.w[w] = pack_bf16x2(pf[2 * w], pf[2 * w + 1]);
#pragma unroll
      for (int nt = 0; nt < 8; ++nt) {
        Frag vb;
        vb.u = vf[nt];
        o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa.v, vb.v, o[nt], 0, 0, 0);
      }
    }
  };

  // ---- batched variant: walk the runs of the plan with the metadata of the next piece fetched during the current
  // one, and the first K/V loads of the next piece issued right after the last step of the current one (pieces are
  // short — a handful of steps — so their start-up latency would otherwise dominate) ----
  if constexpr (kBatched) {
    const int32_t* runs = a.plan + plan_off_runs(n_items);
    const int32_t* gather_list = a.plan + plan_off_gather(n_items, a.B);
    struct Meta {
      int b, c0, c1, pos, seg_end, n_st;              // run index, its range in the sequence, this piece of it
      int w0, req0, step0, jlast, vreq, vstep, vslot;  // plan words (w0 .. jlast the same in every lane)
      int bt0, bt1, L;                                 // first two windows of page ids of the leader, its kv_len
      int gs;                                          // gather run: lane i holds step i of the piece (bt0 / bt1: its pages)
      int posq;                                        // position of the request of this lane's row
    };
    auto find = [&](Meta& m, int pos, int b) __attribute__((always_inline)) {
      while (uni(cum[b + 1]) <= pos) ++b;
      m.b = b; m.c0 = uni(cum[b]); m.c1 = uni(cum[b + 1]); m.pos = pos;
      m.seg_end = min(pos_end, m.c1); m.n_st = m.seg_end - pos;
    };
    auto stage_a = [&](Meta& m) __attribute__((always_inline)) {  // plan words: vector loads, nothing waits here
      const int32_t* w = runs + (size_t)m.b * kPlanRunWords;
      const int r = n16 / G;       // rows past the run's requests read zero-filled words
      m.w0 = w[0]; m.req0 = w[1]; m.step0 = w[1 + kPlanMaxR]; m.jlast = w[kPlanRunWords - 1];
      m.vreq = w[1 + r]; m.vstep = w[1 + kPlanMaxR + r]; m.vslot = w[1 + 2 * kPlanMaxR + r];
    };
    auto stage_b = [&](Meta& m) __attribute__((always_inline)) {  // page ids of the piece's first 128 blocks and the leader's kv_len
      const int req0 = uni(m.req0);
      if (uni(m.w0) & kPlanGather) {  // the piece's steps and their pages from the gather section (64 at most)
        const int32_t* g = gather_list + (size_t)(uni(m.step0) + (m.pos - m.c0) + min(lane, m.n_st - 1)) * kPlanGatherWords;
        m.gs = g[0]; m.bt0 = safe_page(g[1], a.num_pages); m.bt1 = safe_page(g[2], a.num_pages);
      } else {
        const int j0 = kBps * (uni(m.step0) + (m.pos - m.c0)), jl = uni(m.jlast);
        const size_t row = (size_t)req0 * a.max_blocks;
        m.bt0 = safe_page(a.block_tables[row + min(j0 + lane, jl)], a.num_pages);
        m.bt1 = safe_page(a.block_tables[row + min(j0 + 64 + lane, jl)], a.num_pages);
        m.gs = 0;
      }
      m.L = a.kv_lens[req0];
      m.posq = a.q_positions[m.vreq];  // rows past the run's requests read request 0's and are zeroed later
    };
    Meta cur, nxt;
    {
      int lo = 0, hi = n_items - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (uni(cum[mid]) <= pos_begin) lo = mid; else hi = mid - 1;
      }
      find(cur, pos_begin, lo);
    }
    stage_a(cur);
    bool have_nxt = cur.seg_end < pos_end;
    if (have_nxt) { find(nxt, cur.seg_end, cur.b); stage_a(nxt); }
    stage_b(cur);
    // One register buffer of K and V for both formats (measured faster than two for fp8 here, unlike in the plain
    // walker): a step's loads are issued as soon as the step before it has been computed, also across pieces, so
    // that they are in flight during the next piece's set-up; the SIMD's other wave computes meanwhile.
    Frag kbuf[2][kNK];
    VRaw vbuf[8];
    float ks_cur = 1.f, vs_cur = 1.f;
    auto issue_pages = [&](int p0, int p1) __attribute__((always_inline)) {
      if constexpr (kFp8) { ks_cur = a.k_scales[p0]; vs_cur = a.v_scales[p0]; }
      issue_k(kbuf, p0, p1);
      issue_v(vbuf, p0, p1);
    };
    bool pre = false;       // the current piece's first step was issued during the previous piece
    bool carry_open = false;
    for (;;) {
      const int word0 = uni(cur.w0), R = word0 & 0xff, n_rows = R * G, n_st = cur.n_st;
      const bool cont = carry_open && (word0 & kPlanContinues);
      const bool gather = (word0 & kPlanGather) != 0;  // one request, listed steps: Q' is set up anew for every step
      const int req0 = uni(cur.req0), step_first = uni(cur.step0) + (cur.pos - cur.c0), jl = uni(cur.jlast);
      const int my_req = cur.vreq, my_slot = cur.vslot;
      const int my_step = gather ? __builtin_amdgcn_readlane(cur.gs, 0) : cur.vstep + (cur.pos - cur.c0);
      const bool row_ok = n16 < n_rows;
      const int g_row = n16 % G;
      const int L = uni(cur.L), j0 = kBps * step_first;
      const bool ragged_end = (step_first + n_st) * 32 > L;  // only a run of one request can reach past kv_len
      const size_t bt_row = (size_t)req0 * a.max_blocks;
      auto bt_load = [&](int win) { return safe_page(a.block_tables[bt_row + min(j0 + 64 * win + lane, jl)], a.num_pages); };
      int bt_win = 0, bt_cur = cur.bt0, bt_nxt = cur.bt1;
      auto page = [&](int st, int k) __attribute__((always_inline)) {  // page k of step st; called with non-decreasing st
        if (gather) return __builtin_amdgcn_readlane(k ? bt_nxt : bt_cur, st);
        const int rel = kBps * st + k;
        if ((rel >> 6) != bt_win) {
          ++bt_win;
          bt_cur = bt_nxt;
          bt_nxt = bt_load(bt_win + 1);
        }
        return __builtin_amdgcn_readlane(bt_cur, rel & 63);
      };
      if (!pre) {
        const int p0 = page(0, 0), p1 = kBps > 1 ? page(0, kBps - 1) : p0;
        issue_pages(p0, p1);
      }
      if (have_nxt) stage_b(nxt);  // its plan words were requested a piece ago
      if (!cont) {
#pragma unroll
        for (int nt = 0; nt < 8; ++nt) o[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
        m_run = -INFINITY;
        l_part = 0.f;
        v_ref = 0.f;
      }
      auto setup_q = [&](int first_slot) __attribute__((always_inline)) {  // Q' = R(pos_q - first_slot) q in log2 units
        const float delta = (float)(cur.posq - first_slot);
        const float qs = row_ok ? a.qk_scale_log2 : 0.f;
        // A gather run comes here once per step. Everything below but delta is the same every time, and left to
        // itself the compiler keeps it all (scaled q, frequencies: 64 values) in registers across the steps, which
        // the step loop cannot afford: q waits in LDS (each lane reads back what it wrote itself), and the opaque
        // zero in the addresses makes each call read and convert again.
        int again = 0;
        asm volatile("" : "+v"(again));
        Frag qf[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) qf[i].u = q_lds[wave * 4 + i][lane + again];
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float2 f = freq_lds[kg * 16 + again + 8 * h + e];
            const uint32_t wl = qf[h].w[e >> 1], wh = qf[h + 2].w[e >> 1];
            const float x0 = qs * ((e & 1) ? __uint_as_float(wl & 0xffff0000u) : bf16_bits_to_f32(wl & 0xffffu));
            const float x1 = qs * ((e & 1) ? __uint_as_float(wh & 0xffff0000u) : bf16_bits_to_f32(wh & 0xffffu));
            const float t = turns_frac(delta, f.x, f.y);
            const float c = __builtin_amdgcn_cosf(t), sn = __builtin_amdgcn_sinf(t);
            qlo[h][e] = x0 * c - x1 * sn;
            qhi[h][e] = x1 * c + x0 * sn;
          }
      };
      {  // q of this lane's row into LDS: pairs 0-7 and 8-15 low dims, then their high dims (fetching it a piece
         // ahead, like the page ids, measured no faster and costs 16 registers)
        const size_t qrow = ((size_t)my_req * a.Hq + (size_t)hk * G + (row_ok ? g_row : 0)) * (kD / 8);
        const int g0 = kFp8 ? 2 * kg : kg, g1 = kFp8 ? 2 * kg + 1 : 4 + kg;
        q_lds[wave * 4 + 0][lane] = q4[qrow + g0]; q_lds[wave * 4 + 1][lane] = q4[qrow + g1];
        q_lds[wave * 4 + 2][lane] = q4[qrow + 8 + g0]; q_lds[wave * 4 + 3][lane] = q4[qrow + 8 + g1];
      }
      setup_q(my_step * 32);
      pre = false;
      for (int st = 0; st < n_st; ++st) {
        const int n0 = gather ? 32 * __builtin_amdgcn_readlane(cur.gs, st) : (j0 + kBps * st) * kP;
        if (gather && st > 0) setup_q(n0);
        // a gather step always uses slot table 0 and leaves Q' alone
        compute(kbuf, vbuf, n0, gather ? 0 : st, L, gather ? n0 + 32 > L : ragged_end && st == n_st - 1, ks_cur, vs_cur);
        // loads of the step after this one: the next step of this piece, or the first step of the next piece
        if (st + 1 < n_st) {
          const int p0 = page(st + 1, 0), p1 = kBps > 1 ? page(st + 1, kBps - 1) : p0;
          issue_pages(p0, p1);
        } else if (have_nxt) {
          const int p0 = __builtin_amdgcn_readlane(nxt.bt0, 0);
          const int p1 = kBps == 1 ? p0 : (uni(nxt.w0) & kPlanGather) ? __builtin_amdgcn_readlane(nxt.bt1, 0)
                                                                     : __builtin_amdgcn_readlane(nxt.bt0, 1);
          issue_pages(p0, p1);
          pre = true;
        }
      }

      carry_open = have_nxt && (uni(nxt.w0) & kPlanContinues) != 0;
      if (!carry_open) {
        const float l_tot = sum_over_kgroups(l_part);
        auto slot_of = [&](int req, int g, int base) {  // the plan's slot words are relative to the wave index
          return ((size_t)req * a.Hq + (size_t)hk * G + g) * a.n_splits + base + wk;
        };
        if (kg == 0 && row_ok) {
          const size_t sl = slot_of(my_req, g_row, my_slot);
          a.part_ml[sl * 2] = m_run;
          a.part_ml[sl * 2 + 1] = l_tot;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int rr = 4 * kg + e;  // the accumulator element's matrix row
          const int req = __shfl(my_req, rr), base = __shfl(my_slot, rr);
          if (rr < n_rows) {
            float* dst = a.part_o + slot_of(req, rr % G, base) * kD + n16;
#pragma unroll
            for (int nt = 0; nt < 8; ++nt) dst[16 * nt] = kFp8 ? o[nt][e] * (v_ref * (1.f / kPScaleFp8)) : o[nt][e];
          }
        }
      }
      if (!have_nxt) break;
      cur = nxt;
      have_nxt = cur.seg_end < pos_end;
      if (have_nxt) { find(nxt, cur.seg_end, cur.b); stage_a(nxt); }
    }
    return;
  }

  // ---- walk the wave's chunk request by request ----
  int pos = pos_begin, b = 0;
  {  // request that owns the first step: largest b with cum[b] <= pos_begin
    int lo = 0, hi = n_items - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (uni(cum[mid]) <= pos_begin) lo = mid; else hi = mid - 1;
    }
    b = lo;
  }
  while (pos < pos_end) {
    int c0 = uni(cum[b]), c1 = uni(cum[b + 1]);
    while (c1 <= pos) {  // skip requests without steps
      ++b;
      c0 = c1;
      c1 = uni(cum[b + 1]);
    }
    const int seg_end = min(pos_end, c1), n_st = seg_end - pos;
    const int step_first = pos - c0;
    const bool row_ok = n16 < G;  // matrix row n16 is query head n16 of the KV head's group
    const int L = sload(a.kv_lens, b), jend = (L + kP - 1) / kP;
    const int j0 = kBps * step_first;
    const bool ragged_end = (step_first + n_st) * 32 > L;
    const size_t bt_row = (size_t)b * a.max_blocks;
    // Page ids of the run: lane i of bt_cur holds the page of block j0 + 64*bt_win + i (clamped to the
    // request's last block), bt_nxt the 64 after those; a step reads its ids with v_readlane. Vector loads on
    // purpose: scalar loads share a counter with the LDS reads, so every wait for a rotation constant would
    // also wait for them. The next window is fetched a whole window ahead.
    auto bt_load = [&](int win) { return safe_page(a.block_tables[bt_row + min(j0 + 64 * win + lane, jend - 1)], a.num_pages); };
    int bt_win = 0, bt_cur = bt_load(0), bt_nxt = bt_load(1);
    auto page = [&](int st, int k) {  // page k of step st; called with non-decreasing st
      const int rel = kBps * st + k;
      if ((rel >> 6) != bt_win) {
        ++bt_win;
        bt_cur = bt_nxt;
        bt_nxt = bt_load(bt_win + 1);
      }
      return __builtin_amdgcn_readlane(bt_cur, rel & 63);
    };

    // q of head n16: the lane's four 8-element chunks (rows >= G are zeroed through the scale):
    // qf[h] = pairs 8h.. low dims, qf[h + 2] = the same pairs' high dims (+64)
    Frag qf[4];
    {
      const size_t qrow = ((size_t)b * a.Hq + (size_t)hk * G + (row_ok ? n16 : 0)) * (kD / 8);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int glo = kFp8 ? 2 * kg + h : 4 * h + kg;
        qf[h].u = q4[qrow + glo];
        qf[h + 2].u = q4[qrow + 8 + glo];
      }
    }
    // Ring of kNBuf register buffers: while a step is computed the K and V of the next kNBuf-1 steps are in
    // flight.
    constexpr int kNBuf = n_buf(kFp8);
    Frag kbuf[kNBuf][2][kNK];
    VRaw vbuf[kNBuf][8];
    float ks_of[kNBuf], vs_of[kNBuf];  // page scales (fp8), loaded with the step's K and V
    auto issue_step = [&](int rb, int st) {
      const int p0 = page(st, 0), p1 = kBps > 1 ? page(st, kBps - 1) : p0;
      if constexpr (kFp8) {
        ks_of[rb] = a.k_scales[p0];
        vs_of[rb] = a.v_scales[p0];
      } else {
        ks_of[rb] = vs_of[rb] = 1.f;
      }
      issue_k(kbuf[rb], p0, p1);
      issue_v(vbuf[rb], p0, p1);
    };
#pragma unroll
    for (int r = 0; r < kNBuf - 1; ++r)
      if (r < n_st) issue_step(r, r);

    // Q' = R(pos_q - n0) q, scaled into log2 units; reset the accumulators
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) o[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    m_run = -INFINITY;
    l_part = 0.f;
    v_ref = 0.f;
    {
      const float delta = (float)(sload(a.q_positions, b) - step_first * 32);
      const float qs = row_ok ? a.qk_scale_log2 : 0.f;
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int i = freq_of(8 * h + e);
          const uint32_t wl = qf[h].w[e >> 1], wh = qf[h + 2].w[e >> 1];
          const float x0 = qs * ((e & 1) ? __uint_as_float(wl & 0xffff0000u) : bf16_bits_to_f32(wl & 0xffffu));
          const float x1 = qs * ((e & 1) ? __uint_as_float(wh & 0xffff0000u) : bf16_bits_to_f32(wh & 0xffffu));
          const float t = turns_frac(delta, a.freq_hi[i], a.freq_lo[i]);
          const float c = __builtin_amdgcn_cosf(t), sn = __builtin_amdgcn_sinf(t);
          qlo[h][e] = x0 * c - x1 * sn;
          qhi[h][e] = x1 * c + x0 * sn;
        }
    }

    for (int s0 = 0; s0 < n_st; s0 += kNBuf) {
#pragma unroll
      for (int r = 0; r < kNBuf; ++r) {
        const int st = s0 + r;
        if (st < n_st) {
          constexpr int kLead = kNBuf - 1;
          const int rn = (r + kLead) % kNBuf;  // buffer of step st + kLead (free: step st - 1 used it)
          if (st + kLead < n_st) issue_step(rn, st + kLead);
          compute(kbuf[r], vbuf[r], (j0 + kBps * st) * kP, st, L, ragged_end && st == n_st - 1, ks_of[r], vs_of[r]);
        }
      }
    }

    // the partial of this (request, wave): un-normalised rows, reference max (log2 units), sum
    {
      const int split = wk - c0 / chunk;
      const size_t row0 = ((size_t)b * a.Hq + (size_t)hk * G) * a.n_splits + split;  // + g * n_splits
      const float l_tot = sum_over_kgroups(l_part);
      if (kg == 0 && n16 < G) {
        a.part_ml[(row0 + (size_t)n16 * a.n_splits) * 2] = m_run;
        a.part_ml[(row0 + (size_t)n16 * a.n_splits) * 2 + 1] = l_tot;
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int g = 4 * kg + e;
        if (g < G) {
          float* dst = a.part_o + (row0 + (size_t)g * a.n_splits) * kD + n16;
#pragma unroll
          for (int nt = 0; nt < 8; ++nt) dst[16 * nt] = kFp8 ? o[nt][e] * (v_ref * (1.f / kPScaleFp8)) : o[nt][e];
        }
      }
    }
    pos = seg_end;
  }
}

// Merge ns partials (reference max in log2 units, sum, un-normalised row of 128) into one bf16 output row.
// 128 threads: four groups of 32 take every fourth partial, a thread four dims of it, so that enough loads are in
// flight for the merge to run at memory speed when a request has tens of partials; LDS adds the groups up.
__device__ __forceinline__ void merge_row(const float* ml, const float* po, int ns, uint16_t* out_row) {
  __shared__ float4 num_s[4][32];
  __shared__ float den_s[4];
  const int part = threadIdx.x >> 5, dq = threadIdx.x & 31;
  float m = -INFINITY;
  for (int s = 0; s < ns; ++s) m = fmaxf(m, ml[2 * s]);
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
  float den = 0.f;
  if (m != -INFINITY) {
    const float4* po4 = reinterpret_cast<const float4*>(po);
    int s = part;
    for (; s + 4 < ns; s += 8) {  // two partials per turn
      const float w0 = __builtin_amdgcn_exp2f(ml[2 * s] - m), w1 = __builtin_amdgcn_exp2f(ml[2 * s + 8] - m);
      const float4 x0 = po4[(size_t)s * (kD / 4) + dq], x1 = po4[(size_t)(s + 4) * (kD / 4) + dq];
      num.x += w0 * x0.x + w1 * x1.x; num.y += w0 * x0.y + w1 * x1.y;
      num.z += w0 * x0.z + w1 * x1.z; num.w += w0 * x0.w + w1 * x1.w;
      den += w0 * ml[2 * s + 1] + w1 * ml[2 * s + 9];
    }
    if (s < ns) {
      const float w0 = __builtin_amdgcn_exp2f(ml[2 * s] - m);
      const float4 x0 = po4[(size_t)s * (kD / 4) + dq];
      num.x += w0 * x0.x; num.y += w0 * x0.y; num.z += w0 * x0.z; num.w += w0 * x0.w;
      den += w0 * ml[2 * s + 1];
    }
  }
  num_s[part][dq] = num;
  if (dq == 0) den_s[part] = den;
  __syncthreads();
  if (part == 0) {
    const float4 a1 = num_s[1][dq], a2 = num_s[2][dq], a3 = num_s[3][dq];
    // the same order of additions in every thread
    const float d = (den_s[0] + den_s[1]) + (den_s[2] + den_s[3]);
    const float inv = d > 0.f ? 1.f / d : 0.f;
    const float o0 = ((num.x + a1.x) + (a2.x + a3.x)) * inv, o1 = ((num.y + a1.y) + (a2.y + a3.y)) * inv;
    const float o2 = ((num.z + a1.z) + (a2.z + a3.z)) * inv, o3 = ((num.w + a1.w) + (a2.w + a3.w)) * inv;
    uint2 packed;
    packed.x = f32_to_bf16_bits(o0) | (f32_to_bf16_bits(o1) << 16);
    packed.y = f32_to_bf16_bits(o2) | (f32_to_bf16_bits(o3) << 16);
    reinterpret_cast<uint2*>(out_row)[dq] = packed;
  }
}

// Merge the partials of one (request, query head). Request b owns steps [cum[b], cum[b+1]) of its KV
// head's sequence; the waves that cut that range wrote partials 0 .. (cum[b+1]-1)/chunk - cum[b]/chunk.
__global__ __launch_bounds__(128) void combine_streamk_kernel(const AttnArgs a) {
  const int row = blockIdx.x;
  const int b = row / a.Hq;
  const int c0 = a.part_meta[b], c1 = a.part_meta[b + 1], chunk = a.part_meta[a.B + 1];
  const int ns = c1 > c0 ? (c1 - 1) / chunk - c0 / chunk + 1 : 0;
  merge_row(a.part_ml + (size_t)row * a.n_splits * 2, a.part_o + (size_t)row * a.n_splits * kD, ns,
            reinterpret_cast<uint16_t*>(a.out) + (size_t)row * kD);
}

// Merge for the batched variant: request b has n_part[b] partials per head, in slots 0 .. n_part[b]-1.
__global__ __launch_bounds__(128) void combine_batched_kernel(const AttnArgs a) {
  const int row = blockIdx.x;
  const int b = row / a.Hq;
  const int n_runs = a.plan[1];
  const int ns = a.plan[plan_off_npart(n_runs) + b];
  merge_row(a.part_ml + (size_t)row * a.n_splits * 2, a.part_o + (size_t)row * a.n_splits * kD, ns,
            reinterpret_cast<uint16_t*>(a.out) + (size_t)row * kD);
}

// Self-test of dot_rotate_block: words[i] = {e0..e3, ca0, cb0, ca1, cb1, ca2, cb2, ca3, cb3}; out[i] = {l0..l3, h0..h3}.
__global__ __launch_bounds__(256) void dot_rotate_selftest_kernel(const uint32_t* words, float* out, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint32_t* w = words + (size_t)i * 12;
  float r[8];
  dot_rotate_block(w[0], w[1], w[2], w[3], w[4], w[5], w[6], w[7], w[8], w[9], w[10], w[11], r[0], r[1], r[2], r[3], r[4],
                   r[5], r[6], r[7]);
#pragma unroll
  for (int k = 0; k < 8; ++k) out[(size_t)i * 8 + k] = r[k];
}

int compute_units() {
  static const int cus = [] {  // initialised once, thread-safely (function-local static)
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    return n;
  }();
  return cus;
}

}  // namespace

hipError_t launch_decode_mfma(const AttnArgs& a, hipStream_t s) {
  // a fixed number of workgroups per compute unit, a whole number of them per KV head
  const bool fp8 = a.kv_dtype == MEPIC_F8E4M3;
  const int n_wg = max(wg_per_cu(fp8) * compute_units() / a.Hkv, 1) * a.Hkv;
  const size_t lds = (size_t)(a.B + 1) * sizeof(int);
  if (a.timing_start) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_start), s);
  if (fp8 && a.kv_read_once)
    hipLaunchKernelGGL((decode_mfma_kernel<true, false, true>), dim3(n_wg), dim3(64 * kWaves), lds, s, a);
  else if (fp8)
    hipLaunchKernelGGL((decode_mfma_kernel<true, false>), dim3(n_wg), dim3(64 * kWaves), lds, s, a);
  else if (a.kv_read_once)
    hipLaunchKernelGGL((decode_mfma_kernel<false, false, true>), dim3(n_wg), dim3(64 * kWaves), lds, s, a);
  else
    hipLaunchKernelGGL((decode_mfma_kernel<false, false>), dim3(n_wg), dim3(64 * kWaves), lds, s, a);
  hipError_t e = hipGetLastError();
  if (a.timing_stop) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_stop), s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(combine_streamk_kernel, dim3(a.n_q * a.Hq), dim3(kD), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_decode_mfma_batched(const AttnArgs& a, int n_runs, hipStream_t s) {
  const bool fp8 = a.kv_dtype == MEPIC_F8E4M3;
  const int n_wg = max(wg_per_cu(fp8, true) * compute_units() / a.Hkv, 1) * a.Hkv;
  const size_t lds = (size_t)(n_runs + 1) * sizeof(int);
  // static + dynamic LDS may pass 64 KB (the caller bounds n_runs): ask for it, once per process
  static const hipError_t lds_limit_status = [] {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_mfma_kernel<true, true>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 48 * 1024);
    if (e == hipSuccess)
      e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_mfma_kernel<false, true>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 48 * 1024);
    return e;
  }();
  if (lds_limit_status != hipSuccess) return lds_limit_status;
  if (a.timing_start) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_start), s);
  if (fp8)
    hipLaunchKernelGGL((decode_mfma_kernel<true, true>), dim3(n_wg), dim3(64 * kWaves), lds, s, a);
  else
    hipLaunchKernelGGL((decode_mfma_kernel<false, true>), dim3(n_wg), dim3(64 * kWaves), lds, s, a);
  hipError_t e = hipGetLastError();
  if (a.timing_stop) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_stop), s);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(combine_batched_kernel, dim3(a.n_q * a.Hq), dim3(kD), 0, s, a);
  return hipGetLastError();
}

// Requests one plain decode call can take: the per-request step counts (B + 1 ints of dynamic LDS) must fit beside the
// kernel's static tables in the 64 KB a workgroup gets without asking for more.
int decode_mfma_max_requests() { return (64 * 1024 - 44 * 1024) / (int)sizeof(int) - 1; }

int device_compute_units() { return compute_units(); }

hipError_t launch_dot_rotate_selftest(const uint32_t* words, float* out, int n, hipStream_t s) {
  hipLaunchKernelGGL(dot_rotate_selftest_kernel, dim3((n + 255) / 256), dim3(256), 0, s, words, out, n);
  return hipGetLastError();
}

int decode_mfma_waves_per_head(int Hkv, bool fp8) {  // of the batched variant: its planner cuts the sequence
  return max(wg_per_cu(fp8, true) * compute_units() / Hkv, 1) * kWaves;
}

// Upper bound on the partials per request and the matching minimum chunk (in steps of 32 slots), from
// host-known sizes only: with W waves per KV head and B requests a request needs about W/B pieces for an even
// cut; allow four times that for skewed length mixes, never more than W.
void decode_mfma_plan(int B, int Hkv, int max_kv_len, bool fp8, int* max_splits, int* min_chunk) {
  const int W = max(wg_per_cu(fp8) * compute_units() / Hkv, 1) * kWaves;
  const int max_steps = max((max_kv_len + 31) / 32, 1);
  int pieces = 4 * ((W + max(B, 1) - 1) / max(B, 1));
  if (pieces > W) pieces = W;
  if (pieces > max_steps) pieces = max_steps;
  *min_chunk = (max_steps + pieces - 1) / pieces;
  *max_splits = (max_steps + *min_chunk - 1) / *min_chunk + 1;
}

}  // namespace mepic
