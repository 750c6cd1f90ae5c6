// Matrix-core decode kernel of fused-RoPE paged attention (§3.3.3) for bf16 K/V, D = 128, P = 16.
//
// Persistent waves, stream-K over pages. The grid is one workgroup of four waves per compute unit (one
// wave per SIMD: measured faster than two, whose smaller register budget costs prefetch depth). Workgroup g serves KV head g % Hkv (consecutive workgroups land on consecutive
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
// K of the next step and V of the current step are in flight while a step is computed.
//
// Rotary embedding without per-key trigonometry: a key at position n0 + s (n0 = first slot of the
// step) has  q^.k^ = (R(pos_q - n0) q) . (R(s) k).  R(s), s in [0, 32), is a per-lane constant (each
// lane always handles the same two slot offsets and the same 16 frequencies) read from LDS, so a key
// costs one constant 2x2 rotation per element pair; Q' = R(pos_q - n0) q is advanced from step to step
// by the constant rotation R(-32).
//
// The 16 matrix rows of the QK product are the slots {0-3, 8-11, 16-19, 24-27} (+4 for the second
// product), which makes each lane end up with the scores of 8 consecutive slots of one page for one
// head — exactly the A operand of the PV product, so probabilities never leave their lane, and the
// matching V operand is one contiguous 16-byte piece of a V page row.
#include "attn_common.h"

namespace mepic {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128, kP = 16;
constexpr int kWaves = 4;             // waves per workgroup
#ifndef MEPIC_DECODE_WG_PER_CU
#define MEPIC_DECODE_WG_PER_CU 1
#endif
constexpr int kWgPerCu = MEPIC_DECODE_WG_PER_CU;  // workgroups resident per compute unit
constexpr float kRescaleSlack = 6.f;  // the running maximum may lag the true one by this much (log2 units)

union Frag {  // one 16-byte operand fragment
  uint4 u;
  bf16x8 v;
  uint32_t w[4];
};

// Two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Wave-uniform read of a read-only int32 input through the scalar unit (s_load): unlike a vector load it
// does not share the vector-memory counter, so waiting for it never drains the K/V loads in flight.
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
__device__ __forceinline__ int sload(const int32_t* p, size_t idx) {
  return ((const_i32_ptr)(uintptr_t)p)[idx];
}

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

__global__ __launch_bounds__(64 * kWaves, kWgPerCu) void decode_mfma_bf16_kernel(const AttnArgs a) {
  // Rotation constants, identical for every wave: one float4 {c0, s0, c1, s1} per lane and element pair.
  __shared__ float4 rotK[16][64];  // slot rotation R(slot32): index (u*2 + jj)*4 + w
  __shared__ float4 rotS[8][64];   // step rotation R(-32):    index jj*4 + w
  extern __shared__ int cum[];     // cum[b] = steps of the requests before b; B + 1 entries

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n16 = lane & 15, kg = lane >> 4;
  const int G = a.G, Hkv = a.Hkv;

  // ---- cum[] from kv_lens (a step = two blocks); one wave scans ----
  if (wave == 0) {
    int carry = 0;
    for (int base = 0; base < a.B; base += 64) {
      const int b = base + lane;
      int x = 0;
      if (b < a.B) x = ((a.kv_lens[b] + kP - 1) / kP + 1) / 2;
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
  // the step; as holder of 8-element column chunks a lane owns frequencies i = 32*jj + 8*kg + e (dims i and
  // i + 64 are the rotary pair and sit in k-steps jj and jj + 2 of the same lane). ----
  const int slot_u0 = 8 * (n16 >> 2) + (n16 & 3);
  for (int idx = wave; idx < 24; idx += kWaves) {
    const int jj = (idx >> 2) & 1, w = idx & 3;  // idx = (u*2 + jj)*4 + w for rotK, 16 + jj*4 + w for rotS
    const float pos = idx < 16 ? (float)(slot_u0 + 4 * (idx >> 3)) : -32.0f;
    const int i = 32 * jj + 8 * kg + 2 * w;
    const float t0 = turns_frac(pos, a.freq_hi[i], a.freq_lo[i]);
    const float t1 = turns_frac(pos, a.freq_hi[i + 1], a.freq_lo[i + 1]);
    const float4 r = make_float4(__builtin_amdgcn_cosf(t0), __builtin_amdgcn_sinf(t0), __builtin_amdgcn_cosf(t1),
                                 __builtin_amdgcn_sinf(t1));
    if (idx < 16) rotK[idx][lane] = r; else rotS[idx - 16][lane] = r;
  }
  __syncthreads();

  const int T = uni(cum[a.B]);
  const int hk = (int)blockIdx.x % Hkv;
  const int wk = ((int)blockIdx.x / Hkv) * kWaves + wave, n_k = ((int)gridDim.x / Hkv) * kWaves;
  const int chunk = max((T + n_k - 1) / n_k, a.blocks_per_split);  // blocks_per_split carries the minimum chunk
  if (blockIdx.x == 0 && wave == 0) {  // what the merge kernel needs to find each request's partials
    for (int i = lane; i <= a.B; i += 64) a.part_meta[i] = cum[i];
    if (lane == 0) a.part_meta[a.B + 1] = chunk;
  }
  const int pos_begin = wk * chunk, pos_end = min(pos_begin + chunk, T);
  if (pos_begin >= pos_end) return;

  const uint4* kpages = reinterpret_cast<const uint4*>(a.k_pages);
  const uint4* vpages = reinterpret_cast<const uint4*>(a.v_pages);
  const uint4* q4 = reinterpret_cast<const uint4*>(a.q);

  floatx4 o[8];
  float m_run, l_part;
  float qlo[2][8], qhi[2][8];  // Q' of head n16 for the lane's 16 rotary pairs, in log2 units

  // K: product u, k-step j: granule (4j + kg) of slot slot_u0 + 4u (page p0 for rows 0-7, p1 for rows 8-15).
  auto issue_k = [&](Frag (&kf)[2][4], int p0, int p1) {
    const int pk = (n16 < 8) ? p0 : p1;
    const size_t kb = ((size_t)pk * Hkv + hk) * (kD / 8 * kP) + (size_t)kg * kP + (slot_u0 & 15);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) kf[u][j].u = kpages[kb + (size_t)(4 * j) * kP + 4 * u];
  };
  // V: column tile nt: dim 16nt + n16, slots 8*(kg&1).. of page kg/2.
  auto issue_v = [&](Frag (&vf)[8], int p0, int p1) {
    const int pv = (kg < 2) ? p0 : p1;
    const size_t vb = (((size_t)pv * Hkv + hk) * kD + n16) * 2 + (kg & 1);
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) vf[nt].u = vpages[vb + (size_t)nt * 32];
  };

  // One step: 32 slots starting at logical slot n0. `ragged` marks the request's last step when it reaches
  // past kv_len L.
  auto compute = [&](Frag (&kf)[2][4], Frag (&vf)[8], int n0, int L, bool ragged) {
    // Q' as the B operand of the QK products
    Frag bq[4];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        bq[jj].w[e / 2] = pack_bf16x2(qlo[jj][e], qlo[jj][e + 1]);
        bq[jj + 2].w[e / 2] = pack_bf16x2(qhi[jj][e], qhi[jj][e + 1]);
      }
    // Rotate the K rows by their constant slot rotation and run the two QK products, then advance Q' by
    // R(-32). Six groups of four constants each; the constants of the next group are fetched from LDS while a
    // group is computed, and scheduling barriers keep the groups apart so that only two sets are ever live.
    floatx4 sc[2];
    float4 rc[2][4];
#pragma unroll
    for (int w = 0; w < 4; ++w) rc[0][w] = rotK[w][lane];
#pragma unroll
    for (int grp = 0; grp < 6; ++grp) {
      float4 (&r)[4] = rc[grp & 1];
      if (grp + 1 < 6) {
#pragma unroll
        for (int w = 0; w < 4; ++w)
          rc[(grp + 1) & 1][w] = (grp + 1 < 4) ? rotK[(grp + 1) * 4 + w][lane] : rotS[(grp + 1 - 4) * 4 + w][lane];
      }
      if (grp < 4) {
        const int u = grp >> 1, jj = grp & 1;
        if (jj == 0) sc[u] = floatx4{0.f, 0.f, 0.f, 0.f};
        Frag klo, khi;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t lo2 = kf[u][jj].w[w], hi2 = kf[u][jj + 2].w[w];
          const float l0 = bf16_bits_to_f32(lo2 & 0xffffu), l1 = __uint_as_float(lo2 & 0xffff0000u);
          const float h0 = bf16_bits_to_f32(hi2 & 0xffffu), h1 = __uint_as_float(hi2 & 0xffff0000u);
          klo.w[w] = pack_bf16x2(l0 * r[w].x - h0 * r[w].y, l1 * r[w].z - h1 * r[w].w);  // r = {c0, s0, c1, s1}
          khi.w[w] = pack_bf16x2(h0 * r[w].x + l0 * r[w].y, h1 * r[w].z + l1 * r[w].w);
        }
        sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(klo.v, bq[jj].v, sc[u], 0, 0, 0);
        sc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(khi.v, bq[jj + 2].v, sc[u], 0, 0, 0);
      } else {
        const int jj = grp - 4;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const float a0 = qlo[jj][2 * w], b0 = qhi[jj][2 * w], a1 = qlo[jj][2 * w + 1], b1 = qhi[jj][2 * w + 1];
          qlo[jj][2 * w] = a0 * r[w].x - b0 * r[w].y;
          qhi[jj][2 * w] = b0 * r[w].x + a0 * r[w].y;
          qlo[jj][2 * w + 1] = a1 * r[w].z - b1 * r[w].w;
          qhi[jj][2 * w + 1] = b1 * r[w].z + a1 * r[w].w;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    // lane (head n16, kg) now holds the scores of slots n0 + 8kg + 4u + e
    if (ragged) {
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n0 + 8 * kg + 4 * u + e >= L) sc[u][e] = -INFINITY;
      // slots at or past kv_len may hold anything (even NaN): zero them in V
#pragma unroll
      for (int nt = 0; nt < 8; ++nt)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int n = n0 + 8 * kg + 2 * w;
          const uint32_t keep = (n < L ? 0x0000ffffu : 0u) | (n + 1 < L ? 0xffff0000u : 0u);
          vf[nt].w[w] &= keep;
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
    Frag pa;
    float psum = 0.f;
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int e = 0; e < 4; e += 2) {
        const float p0 = __builtin_amdgcn_exp2f(sc[u][e] - m_use), p1 = __builtin_amdgcn_exp2f(sc[u][e + 1] - m_use);
        psum += p0 + p1;
        pa.w[2 * u + e / 2] = pack_bf16x2(p0, p1);
      }
    l_part += psum;
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) o[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa.v, vf[nt].v, o[nt], 0, 0, 0);
  };

  // ---- walk the wave's chunk request by request ----
  int pos = pos_begin, b = 0;
  {  // request that owns the first step: largest b with cum[b] <= pos_begin
    int lo = 0, hi = a.B - 1;
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
    const int L = sload(a.kv_lens, b), jend = (L + kP - 1) / kP;
    const int j0 = 2 * (pos - c0);
    const bool ragged_end = (seg_end == c1) && (L & 31);
    const size_t bt_row = (size_t)b * a.max_blocks;
    auto page = [&](int j) { return sload(a.block_tables, bt_row + min(j, jend - 1)); };

    // q of head n16: the lane's four 8-element chunks (rows >= G are zeroed through the scale)
    Frag qf[4];
    {
      const size_t qb = ((size_t)b * a.Hq + (size_t)hk * G + (n16 < G ? n16 : 0)) * (kD / 8) + kg;
#pragma unroll
      for (int j = 0; j < 4; ++j) qf[j].u = q4[qb + 4 * j];
    }
    Frag kA[2][4], kB[2][4], vf[8];
    int pa0 = page(j0), pa1 = page(j0 + 1);      // pages of the step being computed
    int pb0 = page(j0 + 2), pb1 = page(j0 + 3);  // pages of the step after it
    issue_k(kA, pa0, pa1);

    // Q' = R(pos_q - n0) q, scaled into log2 units; reset the accumulators
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) o[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    m_run = -INFINITY;
    l_part = 0.f;
    {
      const float delta = (float)(sload(a.q_positions, b) - j0 * kP);
      const float qs = n16 < G ? a.qk_scale_log2 : 0.f;
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int i = 32 * jj + 8 * kg + e;
          const uint32_t wl = qf[jj].w[e >> 1], wh = qf[jj + 2].w[e >> 1];
          const float x0 = qs * ((e & 1) ? __uint_as_float(wl & 0xffff0000u) : bf16_bits_to_f32(wl & 0xffffu));
          const float x1 = qs * ((e & 1) ? __uint_as_float(wh & 0xffff0000u) : bf16_bits_to_f32(wh & 0xffffu));
          const float t = turns_frac(delta, a.freq_hi[i], a.freq_lo[i]);
          const float c = __builtin_amdgcn_cosf(t), sn = __builtin_amdgcn_sinf(t);
          qlo[jj][e] = x0 * c - x1 * sn;
          qhi[jj][e] = x1 * c + x0 * sn;
        }
    }

    // steps i and i+1 per iteration; K of the next step and V of this step are in flight during a step
    for (int i = 0; i < n_st; i += 2) {
      issue_v(vf, pa0, pa1);
      if (i + 1 < n_st) issue_k(kB, pb0, pb1);
      pa0 = page(j0 + 2 * i + 4);
      pa1 = page(j0 + 2 * i + 5);
      compute(kA, vf, (j0 + 2 * i) * kP, L, ragged_end && i == n_st - 1);
      if (i + 1 >= n_st) break;
      issue_v(vf, pb0, pb1);
      if (i + 2 < n_st) issue_k(kA, pa0, pa1);
      pb0 = page(j0 + 2 * i + 6);
      pb1 = page(j0 + 2 * i + 7);
      compute(kB, vf, (j0 + 2 * i + 2) * kP, L, ragged_end && i + 1 == n_st - 1);
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
          for (int nt = 0; nt < 8; ++nt) dst[16 * nt] = o[nt][e];
        }
      }
    }
    pos = seg_end;
  }
}

// Merge the partials of one (request, query head). Request b owns steps [cum[b], cum[b+1]) of its KV
// head's sequence; the waves that cut that range wrote partials 0 .. (cum[b+1]-1)/chunk - cum[b]/chunk.
__global__ __launch_bounds__(128) void combine_streamk_kernel(const AttnArgs a) {
  const int row = blockIdx.x, d = threadIdx.x;
  const int b = row / a.Hq;
  const int c0 = a.part_meta[b], c1 = a.part_meta[b + 1], chunk = a.part_meta[a.B + 1];
  const int ns = c1 > c0 ? (c1 - 1) / chunk - c0 / chunk + 1 : 0;
  const float* ml = a.part_ml + (size_t)row * a.n_splits * 2;
  const float* po = a.part_o + (size_t)row * a.n_splits * kD;
  float m = -INFINITY;
  for (int s = 0; s < ns; ++s) m = fmaxf(m, ml[2 * s]);
  float num = 0.f, den = 0.f;
  if (m != -INFINITY) {
    for (int s = 0; s < ns; ++s) {
      const float w = __builtin_amdgcn_exp2f(ml[2 * s] - m);
      num += w * po[(size_t)s * kD + d];
      den += w * ml[2 * s + 1];
    }
  }
  const float o = den > 0.f ? num / den : 0.f;
  reinterpret_cast<uint16_t*>(a.out)[(size_t)row * kD + d] = (uint16_t)f32_to_bf16_bits(o);
}

int compute_units() {
  static int cus = 0;
  if (!cus) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cus = n;
  }
  return cus;
}

}  // namespace

hipError_t launch_decode_mfma_bf16(const AttnArgs& a, hipStream_t s) {
  // kWgPerCu workgroups per compute unit, a whole number of them per KV head
  const int n_wg = max(kWgPerCu * compute_units() / a.Hkv, 1) * a.Hkv;
  const size_t lds = (size_t)(a.B + 1) * sizeof(int);
  hipLaunchKernelGGL(decode_mfma_bf16_kernel, dim3(n_wg), dim3(64 * kWaves), lds, s, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(combine_streamk_kernel, dim3(a.n_q * a.Hq), dim3(kD), 0, s, a);
  return hipGetLastError();
}

// Upper bound on the partials per request and the matching minimum chunk (in steps), from host-known sizes
// only: with W waves per KV head and B requests a request needs about W/B pieces for an even cut; allow four
// times that for skewed length mixes, never more than W.
void decode_mfma_plan(int B, int Hkv, int max_kv_len, int* max_splits, int* min_chunk) {
  const int W = max(kWgPerCu * compute_units() / Hkv, 1) * kWaves;
  const int max_steps = max(((max_kv_len + kP - 1) / kP + 1) / 2, 1);
  int pieces = 4 * ((W + max(B, 1) - 1) / max(B, 1));
  if (pieces > W) pieces = W;
  if (pieces > max_steps) pieces = max_steps;
  *min_chunk = (max_steps + pieces - 1) / pieces;
  *max_splits = (max_steps + *min_chunk - 1) / *min_chunk + 1;
}

}  // namespace mepic
