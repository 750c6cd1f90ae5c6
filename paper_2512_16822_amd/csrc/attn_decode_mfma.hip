// Matrix-core decode kernel of fused-RoPE paged attention (§3.3.3) for bf16 K/V, D = 128, P = 16.
//
// One 64-lane wave serves one (request, KV head, split) and streams the split's pages two at a time
// ("step" = 32 slots). Everything a step needs comes straight from HBM into registers as aligned
// 16-byte loads that already are matrix-core operands (that is what the page layouts are for):
//
//   S^T[32 slots x 16 heads] = Khat[32 x 128] * Q'^T[128 x 16]     2 x 4 v_mfma_f32_16x16x32_bf16
//   O  [16 heads x 128]     += P[16 x 32 slots] * V[32 x 128]      8     v_mfma_f32_16x16x32_bf16
//
// Rotary embedding without per-key trigonometry: a key at position n0 + s (n0 = first slot of the
// step) has  q^.k^ = (R(pos_q - n0) q) . (R(s) k).  R(s), s in [0, 32), is a per-lane constant held in
// registers (each lane always handles the same two slot offsets and the same 16 frequencies), so a
// key costs one constant 2x2 rotation per element pair; Q' = R(pos_q - n0) q is advanced from step
// to step by the constant rotation R(-32).
//
// The 16 matrix rows of the QK product are the slots {0-3, 8-11, 16-19, 24-27} (+4 for the second
// product), which makes each lane end up with the scores of 8 consecutive slots of one page for one
// head — exactly the A operand of the PV product, so probabilities never leave their lane, and the
// matching V operand is one contiguous 16-byte piece of a V page row.
#include "attn_common.h"

namespace mepic {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kD = 128, kP = 16;

struct StepPages { int p0, p1; };

union Frag {  // one 16-byte operand fragment
  uint4 u;
  bf16x8 v;
  uint32_t w[4];
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

__global__ __launch_bounds__(64) void decode_mfma_bf16_kernel(const AttnArgs a) {
  const int lane = threadIdx.x, n16 = lane & 15, kg = lane >> 4;
  const int G = a.G, Hkv = a.Hkv;
  // consecutive workgroups go to consecutive XCDs: keep one KV head on one XCD's L2
  const int hk = blockIdx.x % Hkv;
  const int rest = blockIdx.x / Hkv;
  const int split = rest % a.n_splits, b = rest / a.n_splits;

  const int L = a.kv_lens[b];
  const int pos_q = a.q_positions[b];
  const int n_blocks = (L + kP - 1) / kP;
  const int j_begin = split * a.blocks_per_split;
  const int j_end = min(n_blocks, j_begin + a.blocks_per_split);

  const size_t row0 = ((size_t)b * a.Hq + (size_t)hk * G) * a.n_splits + split;  // + g * n_splits
  if (j_begin >= j_end) {  // nothing in this split: an empty partial
    if (kg == 0 && n16 < G) {
      a.part_ml[(row0 + (size_t)n16 * a.n_splits) * 2] = -INFINITY;
      a.part_ml[(row0 + (size_t)n16 * a.n_splits) * 2 + 1] = 0.f;
    }
    return;
  }

  // ---- per-lane rotary constants ----
  // As holder of K rows: row n16 of product u is slot32 = 8*(n16/4) + 4u + n16%4 of the step.
  // As holder of 8-element column chunks: frequencies i = 32*jj + 8*kg + e, jj in {0,1}, e < 8
  // (dims i and i + 64 are the rotary pair; they sit in k-steps jj and jj + 2 of the same lane).
  float cK[2][2][8], sK[2][2][8], cS[2][8], sS[2][8];
  const int slot_u0 = 8 * (n16 >> 2) + (n16 & 3);
#pragma unroll
  for (int jj = 0; jj < 2; ++jj)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int i = 32 * jj + 8 * kg + e;
      const float fh = a.freq_hi[i], fl = a.freq_lo[i];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const float t = turns_frac((float)(slot_u0 + 4 * u), fh, fl);
        cK[u][jj][e] = __builtin_amdgcn_cosf(t);
        sK[u][jj][e] = __builtin_amdgcn_sinf(t);
      }
      const float t = turns_frac(-32.0f, fh, fl);
      cS[jj][e] = __builtin_amdgcn_cosf(t);
      sS[jj][e] = __builtin_amdgcn_sinf(t);
    }

  // ---- Q' = R(pos_q - n0) q for head n16 (zero rows for n16 >= G), scaled into log2 units ----
  float qlo[2][8], qhi[2][8];
  {
    const float delta = (float)(pos_q - j_begin * kP);
    const uint16_t* qrow = reinterpret_cast<const uint16_t*>(a.q) + ((size_t)b * a.Hq + (size_t)hk * G + n16) * kD;
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int i = 32 * jj + 8 * kg + e;
        float x0 = 0.f, x1 = 0.f;
        if (n16 < G) {
          x0 = bf16_bits_to_f32(qrow[i]) * a.qk_scale_log2;
          x1 = bf16_bits_to_f32(qrow[i + 64]) * a.qk_scale_log2;
        }
        const float t = turns_frac(delta, a.freq_hi[i], a.freq_lo[i]);
        const float c = __builtin_amdgcn_cosf(t), s = __builtin_amdgcn_sinf(t);
        qlo[jj][e] = x0 * c - x1 * s;
        qhi[jj][e] = x1 * c + x0 * s;
      }
  }

  const uint4* kpages = reinterpret_cast<const uint4*>(a.k_pages);
  const uint4* vpages = reinterpret_cast<const uint4*>(a.v_pages);
  const int32_t* bt = a.block_tables + (size_t)b * a.max_blocks;

  auto step_pages = [&](int s) {
    const int jb = j_begin + 2 * s;
    StepPages sp;
    sp.p0 = bt[min(jb, j_end - 1)];
    sp.p1 = bt[min(jb + 1, j_end - 1)];
    return sp;
  };
  // K: product u, k-step j: granule (4j + kg) of slot slot_u0 + 4u (page 0 for rows 0-7, page 1 for rows 8-15).
  // V: column tile nt: dim 16nt + n16, slots 8*(kg&1).. of page kg/2.
  auto issue = [&](Frag (&kf)[2][4], Frag (&vf)[8], const StepPages sp) {
    const int pk = (n16 < 8) ? sp.p0 : sp.p1;
    const size_t kb = ((size_t)pk * Hkv + hk) * (kD / 8 * kP) + (size_t)kg * kP + (slot_u0 & 15);
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j) kf[u][j].u = kpages[kb + (size_t)(4 * j) * kP + 4 * u];
    const int pv = (kg < 2) ? sp.p0 : sp.p1;
    const size_t vb = (((size_t)pv * Hkv + hk) * kD + n16) * 2 + (kg & 1);
#pragma unroll
    for (int nt = 0; nt < 8; ++nt) vf[nt].u = vpages[vb + (size_t)nt * 32];
  };

  floatx4 o[8];
#pragma unroll
  for (int nt = 0; nt < 8; ++nt) o[nt] = floatx4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_part = 0.f;

  auto compute = [&](Frag (&kf)[2][4], Frag (&vf)[8], int s) {
    const int n0 = (j_begin + 2 * s) * kP;
    // Q' as the B operand of the QK products
    Frag bq[4];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int e = 0; e < 8; e += 2) {
        bq[jj].w[e / 2] = pack_bf16x2(qlo[jj][e], qlo[jj][e + 1]);
        bq[jj + 2].w[e / 2] = pack_bf16x2(qhi[jj][e], qhi[jj][e + 1]);
      }
    // rotate the K rows by their constant slot rotation and run the two QK products
    floatx4 sc[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      Frag ak[4];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t lo2 = kf[u][jj].w[w], hi2 = kf[u][jj + 2].w[w];
          const float l0 = bf16_bits_to_f32(lo2 & 0xffffu), l1 = __uint_as_float(lo2 & 0xffff0000u);
          const float h0 = bf16_bits_to_f32(hi2 & 0xffffu), h1 = __uint_as_float(hi2 & 0xffff0000u);
          const float c0 = cK[u][jj][2 * w], s0 = sK[u][jj][2 * w], c1 = cK[u][jj][2 * w + 1], s1 = sK[u][jj][2 * w + 1];
          ak[jj].w[w] = pack_bf16x2(l0 * c0 - h0 * s0, l1 * c1 - h1 * s1);
          ak[jj + 2].w[w] = pack_bf16x2(h0 * c0 + l0 * s0, h1 * c1 + l1 * s1);
        }
      floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ak[j].v, bq[j].v, acc, 0, 0, 0);
      sc[u] = acc;
    }
    // lane (head n16, kg) now holds the scores of slots n0 + 8kg + 4u + e
    const bool tail = n0 + 32 > L;
    if (tail) {
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
    float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                     fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    if (__any(mx > m_run)) {  // rare after the first steps: rescale what has been accumulated
      const float m_new = fmaxf(m_run, mx);
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
    // advance Q' to the next step: 32 positions further from the query
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float lo = qlo[jj][e], hi = qhi[jj][e];
        qlo[jj][e] = lo * cS[jj][e] - hi * sS[jj][e];
        qhi[jj][e] = hi * cS[jj][e] + lo * sS[jj][e];
      }
  };

  // ---- stream the split: loads of step s+1 are in flight while step s is computed ----
  const int n_steps = (j_end - j_begin + 1) / 2;
  Frag kA[2][4], vA[8], kB[2][4], vB[8];
  StepPages pa_ = step_pages(0), pb_ = step_pages(1);
  issue(kA, vA, pa_);
  for (int s = 0; s < n_steps; s += 2) {
    if (s + 1 < n_steps) issue(kB, vB, pb_);
    pa_ = step_pages(s + 2);
    compute(kA, vA, s);
    if (s + 1 >= n_steps) break;
    if (s + 2 < n_steps) issue(kA, vA, pa_);
    pb_ = step_pages(s + 3);
    compute(kB, vB, s + 1);
  }

  // ---- write the split's partial: un-normalised rows, running max (log2 units), sum ----
  float l_tot = l_part + __shfl_xor(l_part, 16);
  l_tot += __shfl_xor(l_tot, 32);
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

}  // namespace

hipError_t launch_decode_mfma_bf16(const AttnArgs& a, hipStream_t s) {
  const unsigned grid = (unsigned)a.B * a.Hkv * a.n_splits;
  hipLaunchKernelGGL(decode_mfma_bf16_kernel, dim3(grid), dim3(64), 0, s, a);
  return hipGetLastError();
}

}  // namespace mepic
