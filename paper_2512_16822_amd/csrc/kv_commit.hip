// Commit step (§3.3.2): scatter the un-rotated K/V of new tokens into their assigned pages.
//
// One workgroup takes a tile of 32 or 64 consecutive source tokens and one KV head. The destination of every
// token of the tile (run by binary search over the run prefix sums, then request, logical slot, page id and
// the page's scales) is resolved once into LDS. K needs no transposition at 16-byte granularity: the granule
// (token, 16 bytes of dims) of the source is the granule (16 bytes of dims, slot) of the page, so each thread
// moves granules directly. V is transposed through LDS: a page row holds the P slots of one dim, so a thread
// collects one dim of eight consecutive tokens and, when those land on eight consecutive slots of one page
// starting at a multiple of eight (always the case for runs that start on a multiple of eight slots), writes
// them with one store; otherwise element by element. fp8 pages are quantised on the way (one fp32 division by
// the page's scale, clamp to the largest finite e4m3 magnitude, hardware round-to-nearest-even conversion).
//
// HBM-bound: reads n_tokens*Hkv*D*2 source elements once, writes as many page elements once.
#include <type_traits>

#include "attn_common.h"

namespace mepic {
namespace {

// Source tokens per workgroup: 64 for the same-format copy, 32 for the quantising one (measured on 64 x 1024 tokens:
// 98.5 -> 95.0 us and 82.3 <- 86.0 us respectively).
constexpr int kThreads = 256;

struct CommitArgs {
  const void* k_new;
  const void* v_new;
  void* k_pages;
  void* v_pages;
  const float* k_scales;
  const float* v_scales;
  const int32_t* block_tables;
  const int32_t* run_request;
  const int32_t* run_first_slot;
  const int32_t* cu_run_tokens;
  int32_t B, n_runs, n_tokens, Hkv, D, P, max_blocks, num_pages;
};

struct alignas(16) Granule { uint32_t w[4]; };

__device__ __forceinline__ uint32_t quant4(const float* x, float scale) {
  // four values -> four e4m3 codes in one word; the quotient is the correctly rounded fp32 division
  float y[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) y[e] = __builtin_fminf(__builtin_fmaxf(x[e] / scale, -448.f), 448.f);
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(y[0], y[1], 0, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(y[2], y[3], w, true);
  return (uint32_t)w;
}

// Source rows are read once and pages are written once, so one side of the copy goes past the caches with the
// non-temporal hint. Which side is a measured choice (64 x 1024 tokens): the same-format copy gains from
// non-temporal loads (123 -> 98 us) and loses with non-temporal stores, alone or on top (110 / 137 us); the
// quantising commit gains from non-temporal stores (101 -> 85 us) and not from the loads.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
template <bool kNT>
__device__ __forceinline__ Granule load_granule(const void* src) {
  if constexpr (kNT) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src));
    return Granule{{v[0], v[1], v[2], v[3]}};
  } else {
    return *reinterpret_cast<const Granule*>(src);
  }
}
template <bool kNT>
__device__ __forceinline__ void store_granule(void* dst, const Granule& g) {
  if constexpr (kNT) {
    const u32x4_t v = {g.w[0], g.w[1], g.w[2], g.w[3]};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(dst));
  } else {
    *reinterpret_cast<Granule*>(dst) = g;
  }
}
template <bool kNT>
__device__ __forceinline__ void store_half_granule(void* dst, const uint2& g) {
  if constexpr (kNT) {
    const u32x2_t v = {g.x, g.y};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2_t*>(dst));
  } else {
    *reinterpret_cast<uint2*>(dst) = g;
  }
}

// The source elements that make one destination granule: 16 bytes, or 32 when bf16 is narrowed to e4m3.
template <typename Src, typename Dst>
struct Raw {
  Granule g[std::is_same_v<Src, Dst> ? 1 : 2];
};

template <typename Src, typename Dst>
__device__ __forceinline__ Raw<Src, Dst> load_raw(const Src* src) {
  Raw<Src, Dst> r;
  constexpr bool kSame = std::is_same_v<Src, Dst>;
  r.g[0] = load_granule<kSame>(src);
  if constexpr (!kSame) r.g[1] = load_granule<kSame>(reinterpret_cast<const Granule*>(src) + 1);
  return r;
}

template <typename Src, typename Dst>
__device__ __forceinline__ Granule convert(const Raw<Src, Dst>& r, float scale) {
  if constexpr (std::is_same_v<Src, Dst>) {
    return r.g[0];
  } else {  // bf16 -> e4m3: 16 elements
    Granule g;
    float x[16];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[2 * e] = bf16_bits_to_f32(r.g[0].w[e] & 0xffffu);
      x[2 * e + 1] = __uint_as_float(r.g[0].w[e] & 0xffff0000u);
      x[8 + 2 * e] = bf16_bits_to_f32(r.g[1].w[e] & 0xffffu);
      x[8 + 2 * e + 1] = __uint_as_float(r.g[1].w[e] & 0xffff0000u);
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) g.w[e] = quant4(x + 4 * e, scale);
    return g;
  }
}

template <typename Src, typename Dst, int D, int P, int kTile>
__global__ __launch_bounds__(kThreads) void kv_commit_kernel(const CommitArgs a) {
  constexpr int X = 16 / (int)sizeof(Dst);        // elements per 16-byte destination granule
  constexpr int DX = D / X;
  constexpr int kPitch = D * (int)sizeof(Dst) + 16;  // bytes per staged V row (keeps 16-byte alignment)
  constexpr int kGroups = kTile / 8;
  // the V pass below enumerates the groups of eight tokens page by page: a tile must hold whole pages' worth of them
  static_assert(kTile % P == 0 && kTile % 8 == 0 && kTile <= kThreads, "tile size does not fit the V pass");
  constexpr bool kNtStore = !std::is_same_v<Src, Dst>;  // see load_granule / store_granule
  __shared__ int s_page[kTile];                   // -1: nothing to write for this token
  __shared__ int s_slot[kTile];
  __shared__ float s_ksc[kTile], s_vsc[kTile];
  __shared__ int s_fast[kGroups];
  __shared__ __attribute__((aligned(16))) unsigned char s_v[kTile * kPitch];

  const int tid = threadIdx.x;
  const int t0 = blockIdx.x * kTile;
  const int h = blockIdx.y;
  const Src* k_new = static_cast<const Src*>(a.k_new);
  const Src* v_new = static_cast<const Src*>(a.v_new);
  Dst* k_pages = static_cast<Dst*>(a.k_pages);
  Dst* v_pages = static_cast<Dst*>(a.v_pages);

  // The source addresses do not depend on the destination: issue every load of this thread first, so that
  // the dependent chain that resolves the destinations (prefix sums -> run -> block table -> scales) runs
  // under their latency.
  constexpr int kUnits = (kTile * DX + kThreads - 1) / kThreads;
  Raw<Src, Dst> rk[kUnits], rv[kUnits];
#pragma unroll
  for (int j = 0; j < kUnits; ++j) {
    const int u = tid + j * kThreads;
    const int i = u / DX, dc = u % DX;
    if (u < kTile * DX && t0 + i < a.n_tokens) {
      const long src_off = ((long)(t0 + i) * a.Hkv + h) * D + dc * X;
      rk[j] = load_raw<Src, Dst>(k_new + src_off);
      rv[j] = load_raw<Src, Dst>(v_new + src_off);
    }
  }

  if (tid < kTile) {
    const int t = t0 + tid;
    int page = -1, slot = 0;
    float ks = 1.f, vs = 1.f;
    if (t < a.n_tokens && t < a.cu_run_tokens[a.n_runs]) {
      int lo = 0, hi = a.n_runs;                  // last run r with cu[r] <= t (it is not empty: cu[r+1] > t)
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.cu_run_tokens[mid] <= t) lo = mid; else hi = mid;
      }
      const int req = a.run_request[lo];
      const long n = (long)a.run_first_slot[lo] + (t - a.cu_run_tokens[lo]);
      const long blk = n / P;
      if (req >= 0 && req < a.B && n >= 0 && blk < a.max_blocks) {
        const int p = a.block_tables[(long)req * a.max_blocks + blk];
        if (p >= 0 && p < a.num_pages) {
          page = p;
          slot = (int)(n % P);
          if constexpr (!std::is_same_v<Src, Dst>) { ks = a.k_scales[p]; vs = a.v_scales[p]; }
        }
      }
    }
    s_page[tid] = page; s_slot[tid] = slot; s_ksc[tid] = ks; s_vsc[tid] = vs;
  }
  __syncthreads();
  if (tid < kGroups) {
    const int p = s_page[8 * tid], s = s_slot[8 * tid];
    bool ok = p >= 0 && (s & 7) == 0;
    for (int j = 1; j < 8; ++j) ok = ok && s_page[8 * tid + j] == p && s_slot[8 * tid + j] == s + j;
    s_fast[tid] = ok ? 1 : 0;
  }

  // K: granule (token i, dims X*dc ..) -> page granule (dc, slot); V: same granule converted into the LDS tile
#pragma unroll
  for (int j = 0; j < kUnits; ++j) {
    const int u = tid + j * kThreads;
    const int i = u / DX, dc = u % DX;
    if (u >= kTile * DX) continue;
    const int p = s_page[i];                      // >= 0 implies t0 + i < n_tokens, i.e. rk[j] / rv[j] were loaded
    if (p < 0) continue;
    store_granule<kNtStore>(k_pages + ((((long)p * a.Hkv + h) * DX + dc) * P + s_slot[i]) * X,
                            convert<Src, Dst>(rk[j], s_ksc[i]));
    *reinterpret_cast<Granule*>(s_v + i * kPitch + dc * 16) = convert<Src, Dst>(rv[j], s_vsc[i]);
  }
  __syncthreads();

  // V: (dim d, eight tokens) -> eight slots of the page row of d
  constexpr int kInner = P / 8;                   // groups per page when the tile is page-aligned
  for (int u = tid; u < D * kGroups; u += kThreads) {
    const int g = (u / (kInner * D)) * kInner + u % kInner;
    const int d = (u / kInner) % D;
    alignas(16) Dst e[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) e[j] = *reinterpret_cast<const Dst*>(s_v + (8 * g + j) * kPitch + d * (int)sizeof(Dst));
    if (s_fast[g]) {
      Dst* dst = v_pages + (((long)s_page[8 * g] * a.Hkv + h) * D + d) * P + s_slot[8 * g];
      if constexpr (sizeof(Dst) == 4) {
        store_granule<kNtStore>(dst, *reinterpret_cast<Granule*>(&e[0]));
        store_granule<kNtStore>(dst + 4, *reinterpret_cast<Granule*>(&e[4]));
      } else if constexpr (sizeof(Dst) == 2) {
        store_granule<kNtStore>(dst, *reinterpret_cast<Granule*>(&e[0]));
      } else {
        store_half_granule<kNtStore>(dst, *reinterpret_cast<uint2*>(&e[0]));
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int p = s_page[8 * g + j];
        if (p >= 0) v_pages[(((long)p * a.Hkv + h) * D + d) * P + s_slot[8 * g + j]] = e[j];
      }
    }
  }
}

template <typename Src, typename Dst>
hipError_t launch(const CommitArgs& a, hipStream_t s) {
  constexpr int kTile = std::is_same_v<Src, Dst> && sizeof(Src) == 2 ? 64 : 32;
  const dim3 grid((a.n_tokens + kTile - 1) / kTile, a.Hkv);
  if (a.D == 128 && a.P == 16) kv_commit_kernel<Src, Dst, 128, 16, kTile><<<grid, kThreads, 0, s>>>(a);
  else if (a.D == 128 && a.P == 32) kv_commit_kernel<Src, Dst, 128, 32, kTile><<<grid, kThreads, 0, s>>>(a);
  else if (a.D == 64 && a.P == 16) kv_commit_kernel<Src, Dst, 64, 16, kTile><<<grid, kThreads, 0, s>>>(a);
  else kv_commit_kernel<Src, Dst, 64, 32, kTile><<<grid, kThreads, 0, s>>>(a);
  return hipGetLastError();
}

}  // namespace
}  // namespace mepic

extern "C" int mepic_kv_commit(const mepic_commit_params* p, void* hip_stream) {
  using namespace mepic;
  if (!p) return MEPIC_ERR_INVALID;
  if (p->B < 0 || p->n_runs < 0 || p->n_tokens < 0 || p->Hkv <= 0 || p->max_blocks < 0 || p->num_pages < 0)
    return MEPIC_ERR_INVALID;
  const bool same = (p->src_dtype == MEPIC_F32 && p->kv_dtype == MEPIC_F32) ||
                    (p->src_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_BF16);
  const bool quant = p->src_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_F8E4M3;
  if (!same && !quant) return MEPIC_ERR_UNSUPPORTED;
  if ((p->D != 64 && p->D != 128) || (p->P != 16 && p->P != 32) || p->Hkv > 65535) return MEPIC_ERR_UNSUPPORTED;
  if ((p->timing_start == nullptr) != (p->timing_stop == nullptr)) return MEPIC_ERR_INVALID;
  if (p->n_tokens == 0 || p->n_runs == 0) return MEPIC_OK;
  if (!p->k_new || !p->v_new || !p->k_pages || !p->v_pages || !p->block_tables || !p->run_request ||
      !p->run_first_slot || !p->cu_run_tokens)
    return MEPIC_ERR_INVALID;
  if (quant && (!p->k_scales || !p->v_scales)) return MEPIC_ERR_INVALID;

  CommitArgs a{};
  a.k_new = p->k_new; a.v_new = p->v_new; a.k_pages = p->k_pages; a.v_pages = p->v_pages;
  a.k_scales = p->k_scales; a.v_scales = p->v_scales; a.block_tables = p->block_tables;
  a.run_request = p->run_request; a.run_first_slot = p->run_first_slot; a.cu_run_tokens = p->cu_run_tokens;
  a.B = p->B; a.n_runs = p->n_runs; a.n_tokens = p->n_tokens; a.Hkv = p->Hkv; a.D = p->D; a.P = p->P;
  a.max_blocks = p->max_blocks; a.num_pages = p->num_pages;

  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  if (p->timing_start) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(p->timing_start), s);
  hipError_t e;
  if (quant) e = launch<uint16_t, uint8_t>(a, s);
  else if (p->kv_dtype == MEPIC_BF16) e = launch<uint16_t, uint16_t>(a, s);
  else e = launch<float, float>(a, s);
  if (p->timing_stop) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(p->timing_stop), s);
  return e == hipSuccess ? MEPIC_OK : MEPIC_ERR_LAUNCH;
}
