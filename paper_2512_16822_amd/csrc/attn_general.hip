// General-path kernel of fused-RoPE paged attention (§3.3.3) and the split-K combine kernel.
//
// Handles every dtype combination, both rotary pairings, decode and causal prefill, the optional
// per-block positions and valid masks. The matrix-core kernels cover the common fast cases; this one
// is the path for everything else (fp32 storage, masks, renumbered positions).
//
// One workgroup of 256 threads serves one (query token, KV head, split): the G query heads that share
// the KV head reuse every rotated key. Per tile of 256 slots:
//   phase A  thread = slot: gather the K row through the block table, rotate it at the slot's
//            absolute position, dot it with the G rotated queries (LDS broadcast) -> scores in LDS;
//   softmax  online max / sum per head with wave shuffles + one LDS exchange;
//   phase B  thread = (dim, part): walk the tile's V rows (contiguous per dim in the V page layout)
//            and accumulate p * v for the G heads.
// Partial (max, sum, un-normalised output) per split go to the workspace; combine_kernel merges them.
#include "attn_common.h"

namespace mepic {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

template <int KV> struct Store;
template <> struct Store<MEPIC_F32> { using T = float; static constexpr int X = 4; };
template <> struct Store<MEPIC_BF16> { using T = uint16_t; static constexpr int X = 8; };
template <> struct Store<MEPIC_F8E4M3> { using T = uint8_t; static constexpr int X = 16; };

// Load one 16-byte granule and widen it to fp32.
template <int KV>
__device__ __forceinline__ void load_granule(const void* base, size_t granule_index, float* x) {
  const uint4 w = reinterpret_cast<const uint4*>(base)[granule_index];
  const uint32_t u[4] = {w.x, w.y, w.z, w.w};
  if constexpr (KV == MEPIC_F32) {
#pragma unroll
    for (int i = 0; i < 4; ++i) x[i] = __uint_as_float(u[i]);
  } else if constexpr (KV == MEPIC_BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = bf16_bits_to_f32(u[i] & 0xffffu);
      x[2 * i + 1] = bf16_bits_to_f32(u[i] >> 16);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int k = 0; k < 4; ++k) x[4 * i + k] = e4m3_to_f32((u[i] >> (8 * k)) & 0xffu);
  }
}

__device__ __forceinline__ float load_q(const void* q, int q_dtype, size_t idx) {
  return q_dtype == MEPIC_F32 ? reinterpret_cast<const float*>(q)[idx]
                              : bf16_bits_to_f32(reinterpret_cast<const uint16_t*>(q)[idx]);
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// GM: compile-time bound on G (query heads per KV head) so the per-head arrays stay in registers.
template <int KV, int GM>
__global__ __launch_bounds__(kThreads) void attn_general_kernel(const AttnArgs a) {
  constexpr int X = Store<KV>::X;
  using T = typename Store<KV>::T;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int t = blockIdx.x, hk = blockIdx.y, split = blockIdx.z;
  const int D = a.D, P = a.P, G = a.G, half = D / 2;

  __shared__ float qhat[GM * 2 * kMaxHalfD];  // [G][D], rotated, pre-multiplied by the score scale
  __shared__ float sc[GM * kThreads];         // [G][256] scores, then probabilities, of the tile
  __shared__ float red[kWaves * GM];
  __shared__ unsigned char took[kThreads];    // does the slot of the tile take part (valid, visible, below kv_len)?
  __shared__ int s_req;

  // which request owns this query token
  if (tid == 0) {
    int b = t;
    if (a.cu_q_lens) {
      int lo = 0, hi = a.B - 1;
      while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (a.cu_q_lens[mid] <= t) lo = mid; else hi = mid - 1;
      }
      b = lo;
    }
    s_req = b;
  }
  __syncthreads();
  const int b = s_req;
  const int L = a.kv_lens[b];
  const int pos_q = a.q_positions[t];
  const int n_begin = split * a.blocks_per_split * P;
  const int n_end = min(L, (split + 1) * a.blocks_per_split * P);

  // rotate the G queries of this KV head at the query's own position
  for (int idx = tid; idx < G * half; idx += kThreads) {
    const int g = idx / half, i = idx % half;
    const int i0 = a.interleaved ? 2 * i : i, i1 = a.interleaved ? 2 * i + 1 : i + half;
    const size_t base = ((size_t)t * a.Hq + (size_t)hk * G + g) * D;
    const float x0 = load_q(a.q, a.q_dtype, base + i0), x1 = load_q(a.q, a.q_dtype, base + i1);
    float sn, cs;
    sincospif(2.0f * turns_frac((float)pos_q, a.freq_hi[i], a.freq_lo[i]), &sn, &cs);
    qhat[g * D + i0] = (x0 * cs - x1 * sn) * a.qk_scale_log2;
    qhat[g * D + i1] = (x1 * cs + x0 * sn) * a.qk_scale_log2;
  }
  __syncthreads();

  // phase-B ownership: dim d, and every `parts`-th block of the tile
  const int d_own = tid % D, part = tid / D, parts = kThreads / D;
  float acc[GM], m_run[GM], l_run[GM];
#pragma unroll
  for (int g = 0; g < GM; ++g) { acc[g] = 0.f; m_run[g] = -INFINITY; l_run[g] = 0.f; }

  const T* kp = reinterpret_cast<const T*>(a.k_pages);
  const T* vp = reinterpret_cast<const T*>(a.v_pages);
  const size_t bt_row = (size_t)b * a.max_blocks;

  for (int n0 = n_begin; n0 < n_end; n0 += kThreads) {
    // ---- phase A: one slot per thread ----
    const int n = n0 + tid;
    float s[GM];
#pragma unroll
    for (int g = 0; g < GM; ++g) s[g] = -INFINITY;
    bool take = n < n_end;
    int pos_k = n, page = 0;
    const int j = n / P, sl = n % P;
    if (take) {
      page = max(min(a.block_tables[bt_row + j], a.num_pages - 1), 0);  // a corrupt id reads a wrong page, never faults
      if (a.block_valid_mask) take = (a.block_valid_mask[bt_row + j] >> sl) & 1u;
      if (a.block_positions) pos_k = a.block_positions[bt_row + j] + sl;
      if (a.causal && pos_k > pos_q) take = false;
    }
    if (take) {
      float dot[GM];
#pragma unroll
      for (int g = 0; g < GM; ++g) dot[g] = 0.f;
      const size_t head_granules = ((size_t)page * a.Hkv + hk) * (size_t)(D / X) * P;  // in granules
      const float fpos = (float)pos_k;
      if (!a.interleaved) {
        for (int c = 0; c < half / X; ++c) {
          float x0[X], x1[X];
          load_granule<KV>(kp, head_granules + (size_t)c * P + sl, x0);
          load_granule<KV>(kp, head_granules + (size_t)(c + half / X) * P + sl, x1);
#pragma unroll
          for (int e = 0; e < X; ++e) {
            const int i = c * X + e;
            float sn, cs;
            sincospif(2.0f * turns_frac(fpos, a.freq_hi[i], a.freq_lo[i]), &sn, &cs);
            const float k0 = x0[e] * cs - x1[e] * sn, k1 = x1[e] * cs + x0[e] * sn;
            _Pragma("unroll") for (int g = 0; g < GM; ++g)
              if (g < G) dot[g] += qhat[g * D + i] * k0 + qhat[g * D + i + half] * k1;
          }
        }
      } else {
        for (int c = 0; c < D / X; ++c) {
          float x[X];
          load_granule<KV>(kp, head_granules + (size_t)c * P + sl, x);
#pragma unroll
          for (int e = 0; e < X; e += 2) {
            const int i = (c * X + e) / 2;
            float sn, cs;
            sincospif(2.0f * turns_frac(fpos, a.freq_hi[i], a.freq_lo[i]), &sn, &cs);
            const float k0 = x[e] * cs - x[e + 1] * sn, k1 = x[e + 1] * cs + x[e] * sn;
            _Pragma("unroll") for (int g = 0; g < GM; ++g)
              if (g < G) dot[g] += qhat[g * D + 2 * i] * k0 + qhat[g * D + 2 * i + 1] * k1;
          }
        }
      }
      const float ksc = KV == MEPIC_F8E4M3 ? a.k_scales[page] : 1.f;
      _Pragma("unroll") for (int g = 0; g < GM; ++g)
        if (g < G) s[g] = dot[g] * ksc;
    }

    // ---- online softmax over the tile, per head ----
    _Pragma("unroll") for (int g = 0; g < GM; ++g) {
      if (g >= G) continue;
      const float wm = wave_max(s[g]);
      if (lane == 0) red[wave * GM + g] = wm;
    }
    __syncthreads();
    float alpha[GM];
    _Pragma("unroll") for (int g = 0; g < GM; ++g) {
      if (g >= G) continue;
      float tm = red[g];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) tm = fmaxf(tm, red[w * GM + g]);
      const float m_new = fmaxf(m_run[g], tm);
      alpha[g] = m_new == -INFINITY ? 1.f : exp2f(m_run[g] - m_new);
      m_run[g] = m_new;
      const float p = take ? exp2f(s[g] - m_new) : 0.f;
      sc[g * kThreads + tid] = p;
      s[g] = p;
    }
    took[tid] = take ? 1 : 0;
    __syncthreads();  // red fully read, sc and took fully written
    _Pragma("unroll") for (int g = 0; g < GM; ++g) {
      if (g >= G) continue;
      const float ws = wave_sum(s[g]);
      if (lane == 0) red[wave * GM + g] = ws;
    }
    __syncthreads();
    _Pragma("unroll") for (int g = 0; g < GM; ++g) {
      if (g >= G) continue;
      float ts = red[g];
#pragma unroll
      for (int w = 1; w < kWaves; ++w) ts += red[w * GM + g];
      l_run[g] = l_run[g] * alpha[g] + ts;
      acc[g] *= alpha[g];
    }

    // ---- phase B: p * V. Thread owns dim d_own and blocks part, part+parts, ... of the tile ----
    const int tile_blocks = (min(n0 + kThreads, n_end) - n0 + P - 1) / P;
    for (int jb = part; jb < tile_blocks; jb += parts) {
      const int nb0 = n0 + jb * P;  // first slot of the block; n0 is a multiple of P
      const int pg = max(min(a.block_tables[bt_row + nb0 / P], a.num_pages - 1), 0);
      const float vsc = KV == MEPIC_F8E4M3 ? a.v_scales[pg] : 1.f;
      const size_t row = (((size_t)pg * a.Hkv + hk) * D + d_own) * (size_t)P;  // in elements
      for (int c = 0; c < P / X; ++c) {
        float v[X];
        load_granule<KV>(vp, row / X + c, v);
#pragma unroll
        for (int e = 0; e < X; ++e) {
          const int rel = jb * P + c * X + e;  // slot index inside the tile
          // a slot that does not take part (at or past kv_len, a pad slot the valid mask drops, a key the causal rule
          // hides) may hold anything, even NaN, and 0 x NaN is NaN: never let its V into the sum
          const float vv = took[rel] ? v[e] * vsc : 0.f;
          _Pragma("unroll") for (int g = 0; g < GM; ++g)
            if (g < G) acc[g] += sc[g * kThreads + rel] * vv;
        }
      }
    }
    __syncthreads();  // sc and red are rewritten by the next tile
  }

  // ---- fold the `parts` partial sums of each dim and write the split's partial result ----
  _Pragma("unroll") for (int g = 0; g < GM; ++g)
    if (g < G) sc[g * kThreads + tid] = acc[g];
  __syncthreads();
  if (part == 0) {
    _Pragma("unroll") for (int g = 0; g < GM; ++g) {
      if (g >= G) continue;
      float o = 0.f;
      for (int pp = 0; pp < parts; ++pp) o += sc[g * kThreads + pp * D + d_own];
      const size_t row = ((size_t)t * a.Hq + (size_t)hk * G + g) * a.n_splits + split;
      a.part_o[row * D + d_own] = o;
      if (d_own == 0) {
        a.part_ml[row * 2] = m_run[g];
        a.part_ml[row * 2 + 1] = l_run[g];
      }
    }
  }
}

// Merge the per-split partials of one (query token, query head): with m* the largest split maximum,
// out = sum_s 2^(m_s - m*) o_s / sum_s 2^(m_s - m*) l_s (all zeros when no slot took part).
__global__ __launch_bounds__(128) void combine_kernel(const AttnArgs a) {
  const int row = blockIdx.x, d = threadIdx.x;
  if (d >= a.D) return;
  const float* ml = a.part_ml + (size_t)row * a.n_splits * 2;
  const float* po = a.part_o + (size_t)row * a.n_splits * a.D;
  float m = -INFINITY;
  for (int s = 0; s < a.n_splits; ++s) m = fmaxf(m, ml[2 * s]);
  float num = 0.f, den = 0.f;
  if (m != -INFINITY) {
    for (int s = 0; s < a.n_splits; ++s) {
      const float ms = ml[2 * s];
      if (ms == -INFINITY) continue;
      const float w = exp2f(ms - m);
      num += w * po[(size_t)s * a.D + d];
      den += w * ml[2 * s + 1];
    }
  }
  const float o = den > 0.f ? num / den : 0.f;
  const size_t idx = (size_t)row * a.D + d;
  if (a.q_dtype == MEPIC_F32) reinterpret_cast<float*>(a.out)[idx] = o;
  else reinterpret_cast<uint16_t*>(a.out)[idx] = (uint16_t)f32_to_bf16_bits(o);
}

}  // namespace

template <int KV>
static void launch_general_kv(const AttnArgs& a, hipStream_t s) {
  const dim3 grid(a.n_q, a.Hkv, a.n_splits), block(kThreads);
  if (a.G <= 1) hipLaunchKernelGGL((attn_general_kernel<KV, 1>), grid, block, 0, s, a);
  else if (a.G <= 2) hipLaunchKernelGGL((attn_general_kernel<KV, 2>), grid, block, 0, s, a);
  else if (a.G <= 4) hipLaunchKernelGGL((attn_general_kernel<KV, 4>), grid, block, 0, s, a);
  else if (a.G <= 8) hipLaunchKernelGGL((attn_general_kernel<KV, 8>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((attn_general_kernel<KV, 16>), grid, block, 0, s, a);
}

hipError_t launch_general(const AttnArgs& a, hipStream_t s) {
  switch (a.kv_dtype) {
    case MEPIC_F32: launch_general_kv<MEPIC_F32>(a, s); break;
    case MEPIC_BF16: launch_general_kv<MEPIC_BF16>(a, s); break;
    default: launch_general_kv<MEPIC_F8E4M3>(a, s); break;
  }
  return hipGetLastError();
}

hipError_t launch_combine(const AttnArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(combine_kernel, dim3(a.n_q * a.Hq), dim3(128), 0, s, a);
  return hipGetLastError();
}

}  // namespace mepic
