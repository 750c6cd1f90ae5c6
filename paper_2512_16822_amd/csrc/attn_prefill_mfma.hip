// Matrix-core prefill kernel of fused-RoPE paged attention (§3.3.3) for bf16, D = 128, P = 16:
// question tokens attend causally (by absolute position) to their request's paged, un-rotated KV.
//
// One workgroup of 8 waves serves 256 query rows (a row = one query token x one of the G query heads
// that share a KV head; 256/G tokens) of one (request, KV head) and walks the request's KV in tiles of
// 64 slots (4 pages). Per tile:
//   stage   every thread pulls two 16-byte granules of K and two of V from the pages; K is rotated in
//           registers at the slot's absolute position (each thread keeps cos/sin of "its" slot and 8
//           frequencies and advances them by the constant rotation R(64) per tile — no trigonometry in
//           the loop) and written to LDS as bf16 in matrix-operand order; V goes to LDS as is. The
//           rotated tile is shared by all 256 rows, so the rotation costs 1/256 per row.
//   QK      S^T[64 slots x 32 rows] per wave = Khat (LDS) x Qhat^T (registers), v_mfma_f32_32x32x16_bf16.
//           Transposed so that a lane owns one query row: row max / sum are register-local.
//   softmax online, reference maximum raised lazily; causal / length mask only on tiles that need it.
//   PV      O^T[128 x 32 rows] += V^T (LDS) x P^T (the S^T registers, re-packed in place).
// LDS tiles are double-buffered: one barrier per tile, the next tile's global loads are in flight during
// the products.
#include <type_traits>

#include "attn_common.h"

namespace mepic {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kD = 128, kP = 16;
constexpr int kThreads = 512;
constexpr int kRows = 256;   // query rows per workgroup (32 per wave)
constexpr int kTile = 64;    // KV slots per tile
constexpr float kSlack = 6.f;

union Frag {
  uint4 u;
  bf16x8 v;
  uint32_t w[4];
  uint2 h[2];
};

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
__device__ __forceinline__ int sload(const int32_t* p, size_t idx) { return ((const_i32_ptr)(uintptr_t)p)[idx]; }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// LDS tile layouts (per buffer):
//   K: [16 chunks of 8 dims][64 slots] granules of 16 bytes -> granule (c, s) at c*64 + s
//   V: [4 pages][128 dims] rows of 32 bytes = two 16-byte halves; half h of dim d holds the slot quads
//      {h, h+2} (slots 4h..4h+3 and 8+4h..8+4h+3) and sits at granule d*2 + (h ^ ((d >> 2) & 1)) so that the
//      lanes of one matrix-operand read hit distinct banks.
struct __align__(16) Tile {
  uint4 k[16 * kTile];
  uint4 v[4 * kD * 2];
};

__global__ __launch_bounds__(kThreads, 1) void prefill_mfma_bf16_kernel(const AttnArgs a) {
  __shared__ Tile tiles[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int G = a.G, Hkv = a.Hkv;
  const int hk = blockIdx.x % Hkv;
  const int qt = (blockIdx.x / Hkv) % a.n_splits;  // n_splits carries the number of query tiles per request
  const int b = blockIdx.x / Hkv / a.n_splits;

  const int q_begin = sload(a.cu_q_lens, b), q_end = sload(a.cu_q_lens, b + 1);
  const int tok_per_wg = kRows / G;
  const int tok0 = q_begin + qt * tok_per_wg;
  if (tok0 >= q_end) return;
  const int L = sload(a.kv_lens, b);

  // ---- this lane's query row: token and head, causal limit, rotated query as B operands ----
  const int row = wave * 32 + l32;          // row of the workgroup tile
  const int tok = tok0 + row / G, g = row % G;
  const bool row_ok = tok < q_end;
  const int pos_q = row_ok ? a.q_positions[tok] : -1;
  const int lim = min(pos_q, L - 1);        // last visible slot of this row (-1: none)

  Frag bq[8];  // k-step ks: dims 16ks + 8half + e
  {
    const uint4* q4 = reinterpret_cast<const uint4*>(a.q);
    const size_t qb = ((size_t)(row_ok ? tok : q_begin) * a.Hq + (size_t)hk * G + g) * (kD / 8);
    const float qs = row_ok ? a.qk_scale_log2 : 0.f;
    Frag raw[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) raw[ks].u = q4[qb + 2 * ks + half];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        float lo[2], hi[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int i = 16 * ks + 8 * half + 2 * w + e;
          const uint32_t wl = raw[ks].w[w], wh = raw[ks + 4].w[w];
          const float x0 = qs * (e ? __uint_as_float(wl & 0xffff0000u) : bf16_bits_to_f32(wl & 0xffffu));
          const float x1 = qs * (e ? __uint_as_float(wh & 0xffff0000u) : bf16_bits_to_f32(wh & 0xffffu));
          const float t = turns_frac((float)pos_q, a.freq_hi[i], a.freq_lo[i]);
          const float c = __builtin_amdgcn_cosf(t), s = __builtin_amdgcn_sinf(t);
          lo[e] = x0 * c - x1 * s;
          hi[e] = x1 * c + x0 * s;
        }
        bq[ks].w[w] = pack2(lo[0], lo[1]);
        bq[ks + 4].w[w] = pack2(hi[0], hi[1]);
      }
  }

  // ---- KV range of the workgroup: up to the largest visible slot of any of its rows ----
  const int last_tok = min(tok0 + tok_per_wg, q_end) - 1;
  int pos_max = -1, pos_min = 0x7fffffff;
  for (int t = tok0 + lane; t <= last_tok; t += 64) {
    const int p = a.q_positions[t];
    pos_max = max(pos_max, p);
    pos_min = min(pos_min, p);
  }
#pragma unroll
  for (int o = 32; o; o >>= 1) {
    pos_max = max(pos_max, __shfl_xor(pos_max, o));
    pos_min = min(pos_min, __shfl_xor(pos_min, o));
  }
  pos_max = uni(pos_max);
  pos_min = uni(pos_min);
  const int n_hi = min(L, pos_max + 1);              // slots [0, n_hi) are visible to some row
  const int n_tiles = (n_hi + kTile - 1) / kTile;
  const int n_blocks = (L + kP - 1) / kP;

  // ---- staging role: thread = (slot s_st of the tile, pair-chunk pc); dims 8pc.. and 64 + 8pc.. ----
  const int s_st = tid & 63, pc = tid >> 6;
  float rc[8], rs[8], stc[8], sts[8];  // cos/sin of (tile start + s_st) * f_i, and of 64 * f_i, i = 8pc + e
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int i = 8 * pc + e;
    const float t0 = turns_frac((float)s_st, a.freq_hi[i], a.freq_lo[i]);
    const float t1 = turns_frac((float)kTile, a.freq_hi[i], a.freq_lo[i]);
    rc[e] = __builtin_amdgcn_cosf(t0);
    rs[e] = __builtin_amdgcn_sinf(t0);
    stc[e] = __builtin_amdgcn_cosf(t1);
    sts[e] = __builtin_amdgcn_sinf(t1);
  }
  const uint4* kpages = reinterpret_cast<const uint4*>(a.k_pages);
  const uint4* vpages = reinterpret_cast<const uint4*>(a.v_pages);
  const size_t bt_row = (size_t)b * a.max_blocks;
  // the four pages of tile t (block indices clamped to the request's last block; clamped slots are masked)
  auto tile_page = [&](int t, int k) { return sload(a.block_tables, bt_row + min(4 * t + k, max(n_blocks - 1, 0))); };

  Frag gk[2], gv[2];
  auto load_tile = [&](int p0, int p1, int p2, int p3) __attribute__((always_inline)) {
    const int pg_k = (s_st < 32) ? (s_st < 16 ? p0 : p1) : (s_st < 48 ? p2 : p3);
    const size_t kb = ((size_t)pg_k * Hkv + hk) * (kD / 8 * kP) + (size_t)pc * kP + (s_st & 15);
    gk[0].u = kpages[kb];
    gk[1].u = kpages[kb + 8 * kP];
    // V: granule gi of the tile = page gi/256, granule gi%256 of the page; this thread: gi = tid, tid + 512
    const int pg_v0 = (tid < 256) ? p0 : p1, pg_v1 = (tid < 256) ? p2 : p3;
    gv[0].u = vpages[((size_t)pg_v0 * Hkv + hk) * (kD * 2) + (tid & 255)];
    gv[1].u = vpages[((size_t)pg_v1 * Hkv + hk) * (kD * 2) + (tid & 255)];
  };
  // rotate the staged K granules at position (tile start + s_st), write K and V into LDS buffer `buf`
  auto stage_tile = [&](int buf, int n0) __attribute__((always_inline)) {
    Frag klo, khi;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t lo2 = gk[0].w[w], hi2 = gk[1].w[w];
      const float l0 = bf16_bits_to_f32(lo2 & 0xffffu), l1 = __uint_as_float(lo2 & 0xffff0000u);
      const float h0 = bf16_bits_to_f32(hi2 & 0xffffu), h1 = __uint_as_float(hi2 & 0xffff0000u);
      klo.w[w] = pack2(l0 * rc[2 * w] - h0 * rs[2 * w], l1 * rc[2 * w + 1] - h1 * rs[2 * w + 1]);
      khi.w[w] = pack2(h0 * rc[2 * w] + l0 * rs[2 * w], h1 * rc[2 * w + 1] + l1 * rs[2 * w + 1]);
    }
    tiles[buf].k[pc * kTile + s_st] = klo.u;
    tiles[buf].k[(pc + 8) * kTile + s_st] = khi.u;
    // advance the rotation to the next tile
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float c = rc[e], s = rs[e];
      rc[e] = c * stc[e] - s * sts[e];
      rs[e] = s * stc[e] + c * sts[e];
    }
    // V granule (page pgi, dim d, slot half sh): quads 2sh, 2sh+1 -> halves (2sh)&1.. : quad q goes to half q&1,
    // position q>>1 inside the half
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int pgi = (tid >> 8) + 2 * r, d = (tid & 255) >> 1, sh = tid & 1;
      Frag x = gv[r];
      if (n0 + kTile > L && n0 + pgi * kP + 8 * sh + 8 > L) {  // slots at or past kv_len may hold anything: zero them
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int n = n0 + pgi * kP + 8 * sh + 2 * w;
          x.w[w] &= (n < L ? 0x0000ffffu : 0u) | (n + 1 < L ? 0xffff0000u : 0u);
        }
      }
      uint2* vrow = reinterpret_cast<uint2*>(&tiles[buf].v[(pgi * kD + d) * 2]);
      const int swz = (d >> 2) & 1;
      // quad 2sh (even) -> half 0, quad 2sh+1 (odd) -> half 1; inside a half the quads {h, h+2} are in order
      vrow[((0 ^ swz) << 1) + sh] = x.h[0];
      vrow[((1 ^ swz) << 1) + sh] = x.h[1];
    }
  };

  floatx16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
  float m_run = -INFINITY, l_part = 0.f;

  if (n_tiles > 0) {
    load_tile(tile_page(0, 0), tile_page(0, 1), tile_page(0, 2), tile_page(0, 3));
  }
  int np0 = tile_page(1, 0), np1 = tile_page(1, 1), np2 = tile_page(1, 2), np3 = tile_page(1, 3);

  auto tile_step = [&](int t, auto buf_tag) __attribute__((always_inline)) {
    constexpr int buf = decltype(buf_tag)::value;  // compile-time, so that LDS addresses fold into offsets
    const int n0 = t * kTile;
    stage_tile(buf, n0);
    __syncthreads();
    if (t + 1 < n_tiles) load_tile(np0, np1, np2, np3);
    np0 = tile_page(t + 2, 0); np1 = tile_page(t + 2, 1); np2 = tile_page(t + 2, 2); np3 = tile_page(t + 2, 3);

    const bool need_mask = n0 + kTile - 1 > min(pos_min, L - 1);  // some row cannot see the whole tile
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      // S^T block: slots n0 + 32sb + {8blk + 4half + e}, row l32
      floatx16 sc;
#pragma unroll
      for (int e = 0; e < 16; ++e) sc[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        Frag ka;
        ka.u = tiles[buf].k[(2 * ks + half) * kTile + 32 * sb + l32];
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, bq[ks].v, sc, 0, 0, 0);
      }
      if (need_mask) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (n0 + 32 * sb + 8 * (e >> 2) + 4 * half + (e & 3) > lim) sc[e] = -INFINITY;
      }
      float mx = sc[0];
#pragma unroll
      for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sc[e]);
      {
        // the two lanes of a row (l32, half 0/1) keep one common reference maximum, raised lazily: it only has
        // to bound the scores up to a fixed slack
        const uint32_t u = __float_as_uint(mx);
        const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        const float mrow = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        if (mrow > m_run + kSlack) {
          const float alpha = __builtin_amdgcn_exp2f(m_run - mrow);  // m_run = -inf -> 0
          m_run = mrow;
          l_part *= alpha;
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
        }
      }
      const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
      float psum = 0.f;
      Frag pb[2];  // page 2sb + pp of the tile: k index e -> slots 4half + e (e < 4), 8 + 4half + e - 4
#pragma unroll
      for (int pp = 0; pp < 2; ++pp)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int e0 = 8 * pp + 4 * (w >> 1) + 2 * (w & 1);  // sc index: blk = 2pp + (w>>1), e = 2(w&1)
          const float p0 = __builtin_amdgcn_exp2f(sc[e0] - m_use), p1 = __builtin_amdgcn_exp2f(sc[e0 + 1] - m_use);
          psum += p0 + p1;
          pb[pp].w[w] = pack2(p0, p1);
        }
      l_part += psum;
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) {
        const int pgi = 2 * sb + pp;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const int d = 32 * db + l32;
          Frag va;
          va.u = tiles[buf].v[(pgi * kD + d) * 2 + (half ^ ((d >> 2) & 1))];
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pb[pp].v, o[db], 0, 0, 0);
        }
      }
    }
  };
  for (int t = 0; t < n_tiles; t += 2) {
    tile_step(t, std::integral_constant<int, 0>{});
    if (t + 1 < n_tiles) tile_step(t + 1, std::integral_constant<int, 1>{});
  }

  // ---- normalise and store: lane (row l32, half) holds dims 32db + 8blk + 4half + e of its row ----
  {
    const uint32_t u = __float_as_uint(l_part);
    const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const float l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (row_ok) {
      uint2* orow = reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(a.out) +
                                             ((size_t)tok * a.Hq + (size_t)hk * G + g) * kD);
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk) {
          uint2 w;
          w.x = pack2(o[db][4 * blk] * inv, o[db][4 * blk + 1] * inv);
          w.y = pack2(o[db][4 * blk + 2] * inv, o[db][4 * blk + 3] * inv);
          orow[(32 * db + 8 * blk + 4 * half) / 4] = w;
        }
    }
  }
}

}  // namespace

hipError_t launch_prefill_mfma_bf16(const AttnArgs& a, hipStream_t s) {
  const unsigned grid = (unsigned)a.B * a.Hkv * a.n_splits;
  hipLaunchKernelGGL(prefill_mfma_bf16_kernel, dim3(grid), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

int prefill_mfma_rows_per_workgroup() { return kRows; }

}  // namespace mepic
