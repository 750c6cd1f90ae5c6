// Matrix-core prefill kernel of fused-RoPE paged attention (§3.3.3) for bf16, D = 128, P = 16:
// question tokens attend causally (by absolute position) to their request's paged, un-rotated KV.
//
// One workgroup of 8 waves serves 256 query rows (a row = one query token x one of the G query heads
// that share a KV head; 256/G tokens) of one (request, KV head) and walks the request's KV in tiles of
// 64 slots (4 pages). The vector pipe, not the matrix pipe, is what a tile waits for, so everything is
// arranged to need few vector instructions per tile:
//   stage   every thread pulls two 16-byte granules of K from the pages and rotates them in registers at the
//           slot's absolute position with cos/sin read from a per-position table (built once per call by
//           rope_table_kernel: no trigonometry and no rotation state to advance in the loop), then writes them
//           to LDS as bf16 in matrix-operand order. The rotated tile is shared by all 256 rows, so the rotation
//           costs 1/256 per row. V never passes through registers: the four page-heads of the tile are copied
//           from HBM straight into LDS (global_load_lds_dwordx4) as they are.
//   QK      S^T[64 slots x 32 rows] per wave = Khat (LDS) x Qhat^T (registers), v_mfma_f32_32x32x16_bf16.
//           Transposed so that a lane owns one query row: row sums are register-local. The accumulator starts
//           at minus the row's reference maximum, so the scores come out of the products already shifted.
//           The matrix rows are assigned to the tile's slots in an order that leaves a lane with the
//           probabilities of eight consecutive slots of one page: exactly the 16-byte piece of a V page row.
//   softmax online; the reference maximum is a lower bound raised only when a probability would get huge (the
//           test is on the row sum that is needed anyway), causal / length mask only on tiles that need it.
//   PV      O^T[128 x 32 rows] += V^T (LDS, as stored in the page) x P^T (the S^T registers, packed in place).
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
// A probability may grow to 2^kBigLog2 before the reference maximum is raised (fp32 sums and bf16 operands keep
// their relative precision at any scale; only overflow has to be kept away).
constexpr float kBig = 0x1p40f;

union Frag {
  uint4 u;
  bf16x8 v;
  uint32_t w[4];
  float f[4];
};

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
__device__ __forceinline__ int sload(const int32_t* p, size_t idx) { return ((const_i32_ptr)(uintptr_t)p)[idx]; }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// 16 bytes per lane from global memory straight into LDS: lane i's piece lands at lds_base + 16 i (lds_base is
// wave-uniform). Counted by vmcnt like any other vector-memory load; the data never touches a register.
__device__ __forceinline__ void load_to_lds(const uint4* src, uint4* lds_base) {
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                   (__attribute__((address_space(3))) void*)lds_base, 16, 0, 0);
}

// Per-position rotary table: for position p and frequency pair (i0, i0 + 1), i0 = 8 pc + 2 j, one 16-byte entry
// {cos(p f_i0), sin(p f_i0), cos(p f_i0+1), sin(p f_i0+1)} at entry index
//   (((p / 64) * 8 + pc) * 4 + j) * 64 + p % 64,
// so that the 64 lanes of a wave, which stage 64 consecutive positions for one (pc, j), read 1 KB in one piece.
__device__ __forceinline__ size_t rope_entry(int p, int pc, int j) {
  return ((((size_t)(p >> 6) * 8 + pc) * 4 + j) << 6) + (p & 63);
}

__global__ __launch_bounds__(256) void rope_table_kernel(const AttnArgs a, int n_pos) {
  const int idx = blockIdx.x * 256 + threadIdx.x;   // (p / 64, pc, j, p % 64), the entry index itself
  if (idx >= n_pos * 32) return;
  const int p = ((idx >> 11) << 6) + (idx & 63), pc = (idx >> 8) & 7, j = (idx >> 6) & 3;
  const int i0 = 8 * pc + 2 * j;
  const float t0 = turns_frac((float)p, a.freq_hi[i0], a.freq_lo[i0]);
  const float t1 = turns_frac((float)p, a.freq_hi[i0 + 1], a.freq_lo[i0 + 1]);
  a.rope_table[idx] = make_float4(__builtin_amdgcn_cosf(t0), __builtin_amdgcn_sinf(t0), __builtin_amdgcn_cosf(t1),
                                  __builtin_amdgcn_sinf(t1));
}

// LDS tile layouts (per buffer):
//   K: [16 chunks of 8 dims][64 slots] granules of 16 bytes -> granule (c, s) at c*64 + s, rotated, bf16
//   V: the tile's four page-heads as they lie in HBM, [4 pages][128 dims][2 halves of 8 slots] granules
struct __align__(16) Tile {
  uint4 k[16 * kTile];
  uint4 v[4 * kD * 2];
};

__global__ __launch_bounds__(kThreads, 1) void prefill_mfma_bf16_kernel(const AttnArgs a) {
  __shared__ Tile tiles[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int G = a.G, Hkv = a.Hkv;
  const int hk = blockIdx.x % Hkv;
  const int qt = (blockIdx.x / Hkv) % a.n_splits;  // n_splits carries the number of query tiles per request
  const int b = blockIdx.x / Hkv / a.n_splits;

  const int q_begin = sload(a.cu_q_lens, b), q_end = sload(a.cu_q_lens, b + 1);
  const int tok_per_wg = kRows / G;
  const int tok0 = q_begin + qt * tok_per_wg;
  if (tok0 >= q_end) return;
  const int L = min(sload(a.kv_lens, b), a.blocks_per_split * kP);  // blocks_per_split: blocks the host sized the rotary table for

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
  const int s_st = tid & 63, pc = wave;
  const uint4* kpages = reinterpret_cast<const uint4*>(a.k_pages);
  const uint4* vpages = reinterpret_cast<const uint4*>(a.v_pages);
  const float4* table = a.rope_table + rope_entry(s_st, pc, 0);   // + 2048 entries per tile, + 64 per j
  const size_t bt_row = (size_t)b * a.max_blocks;
  // the four pages of tile t (block indices clamped to the request's last block; clamped slots are masked)
  auto tile_page = [&](int t, int k) { return sload(a.block_tables, bt_row + min(4 * t + k, max(n_blocks - 1, 0))); };

  // V of a tile goes from the pages straight into LDS: wave w copies half w%2 (64 dims = 2 KB) of page-head w/2
  const int v_page_sel = wave >> 1, v_gran0 = (wave & 1) * 128 + lane;

  Frag gk[2];
  float4 gt[4];
  auto load_tile = [&](int t, int buf, int p0, int p1, int p2, int p3) __attribute__((always_inline)) {
    const int pg_k = (s_st < 32) ? (s_st < 16 ? p0 : p1) : (s_st < 48 ? p2 : p3);
    const size_t kb = ((size_t)pg_k * Hkv + hk) * (kD / 8 * kP) + (size_t)pc * kP + (s_st & 15);
    gk[0].u = kpages[kb];
    gk[1].u = kpages[kb + 8 * kP];
#pragma unroll
    for (int j = 0; j < 4; ++j) gt[j] = table[(size_t)t * 2048 + j * 64];
    const int pg_v = v_page_sel < 2 ? (v_page_sel == 0 ? p0 : p1) : (v_page_sel == 2 ? p2 : p3);  // wave-uniform
    const uint4* vsrc = vpages + ((size_t)pg_v * Hkv + hk) * (kD * 2) + v_gran0;
    uint4* vdst = &tiles[buf].v[v_page_sel * (kD * 2) + (wave & 1) * 128];
    load_to_lds(vsrc, vdst);
    load_to_lds(vsrc + 64, vdst + 64);
  };
  // rotate the staged K granules at position (tile start + s_st), write them into LDS buffer `buf`; make sure this
  // wave's share of the tile's V has landed in LDS and holds no garbage past kv_len
  auto stage_tile = [&](int buf, int n0) __attribute__((always_inline)) {
    Frag klo, khi;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t lo2 = gk[0].w[w], hi2 = gk[1].w[w];
      const float l0 = bf16_bits_to_f32(lo2), l1 = __uint_as_float(lo2 & 0xffff0000u);
      const float h0 = bf16_bits_to_f32(hi2), h1 = __uint_as_float(hi2 & 0xffff0000u);
      const float4 r = gt[w];  // {cos, sin} of frequencies 8pc + 2w and 8pc + 2w + 1 at this slot's position
      klo.w[w] = pack2(l0 * r.x - h0 * r.y, l1 * r.z - h1 * r.w);
      khi.w[w] = pack2(h0 * r.x + l0 * r.y, h1 * r.z + l1 * r.w);
    }
    tiles[buf].k[pc * kTile + s_st] = klo.u;
    tiles[buf].k[(pc + 8) * kTile + s_st] = khi.u;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the direct-to-LDS copies of V are not tied to any register
    if (n0 + kTile > L) {
      // Slots at or past kv_len may hold anything, NaN included, and 0 x NaN would poison the row: zero them.
      // Each wave patches the 2 KB it copied itself (two granules per lane: dim, half of the page's slots).
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int gi = v_gran0 + 64 * i;              // granule of the page-head: dim gi / 2, slots 8 (gi & 1)..
        const int nbase = n0 + v_page_sel * kP + 8 * (gi & 1);
        if (nbase + 8 > L) {
          uint4* cell = &tiles[buf].v[v_page_sel * (kD * 2) + gi];
          Frag x;
          x.u = *cell;
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const int n = nbase + 2 * w;
            x.w[w] &= (n < L ? 0x0000ffffu : 0u) | (n + 1 < L ? 0xffff0000u : 0u);
          }
          *cell = x.u;
        }
      }
    }
  };

  floatx16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[db][e] = 0.f;
  // Reference maximum of the row (log2 units). -inf until the row has seen a visible slot; rows that do not exist
  // (past the last query token: zero query, everything masked) start at 0 so that they never ask for attention.
  float m_run = row_ok ? -INFINITY : 0.f, l_part = 0.f;
  floatx16 negm;  // minus the reference maximum in all sixteen elements: where the QK accumulators start
#pragma unroll
  for (int e = 0; e < 16; ++e) negm[e] = 0.f;

  if (n_tiles > 0) load_tile(0, 0, tile_page(0, 0), tile_page(0, 1), tile_page(0, 2), tile_page(0, 3));
  int np0 = tile_page(1, 0), np1 = tile_page(1, 1), np2 = tile_page(1, 2), np3 = tile_page(1, 3);

  // Matrix row m of a 32-slot block holds slot (m & 16) + 8 * bit2(m) + 4 * bit3(m) + (m & 3) of the block: a lane
  // of the score tile (row l32, half) then owns, in accumulator order, slots 8 half .. 8 half + 7 of the block's first
  // page and the same of its second page.
  const int k_read = (l32 & 16) + ((l32 & 4) << 1) + ((l32 & 8) >> 1) + (l32 & 3);

  auto tile_step = [&](int t, auto buf_tag) __attribute__((always_inline)) {
    constexpr int buf = decltype(buf_tag)::value;  // compile-time, so that LDS addresses fold into offsets
    const int n0 = t * kTile;
    stage_tile(buf, n0);
    __syncthreads();
    if (t + 1 < n_tiles) load_tile(t + 1, buf ^ 1, np0, np1, np2, np3);
    np0 = tile_page(t + 2, 0); np1 = tile_page(t + 2, 1); np2 = tile_page(t + 2, 2); np3 = tile_page(t + 2, 3);

    const bool need_mask = n0 + kTile - 1 > min(pos_min, L - 1);  // some row cannot see the whole tile
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      // S^T block: accumulator element e of lane (row l32, half) is slot n0 + 32sb + 16(e>>3) + 8half + (e&7)
      floatx16 sc = negm;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        Frag ka;
        ka.u = tiles[buf].k[(2 * ks + half) * kTile + 32 * sb + k_read];
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka.v, bq[ks].v, sc, 0, 0, 0);
      }
      if (need_mask) {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (n0 + 32 * sb + 16 * (e >> 3) + 8 * half + (e & 7) > lim) sc[e] = -INFINITY;
      }
      float p[16];
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        p[e] = __builtin_amdgcn_exp2f(sc[e]);
        psum += p[e];
      }
      // Raise the reference maximum only when a probability got huge (or overflowed), or on the first visible slots of
      // the row; both lanes of a row (l32, half 0/1) must agree on it, so the decision and the new value are common.
      if (__any(!(psum <= kBig) || m_run == -INFINITY)) {
        float mx = sc[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) mx = fmaxf(mx, sc[e]);
        const uint32_t u = __float_as_uint(mx);
        const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
        const float mrow = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));  // relative to the old reference
        if (mrow > -INFINITY) {
          const bool first = m_run == -INFINITY;
          const float delta = first ? mrow : fmaxf(mrow, 0.f);
          const float alpha = first ? 1.f : __builtin_amdgcn_exp2f(-delta);
          m_run = (first ? 0.f : m_run) + delta;
          l_part *= alpha;
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
#pragma unroll
          for (int e = 0; e < 16; ++e) negm[e] = -m_run;
          psum = 0.f;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            p[e] = __builtin_amdgcn_exp2f(sc[e] - delta);
            psum += p[e];
          }
        }
      }
      l_part += psum;
      Frag pb[2];  // page 2sb + pp of the tile: k index e -> slot 8half + e of the page
#pragma unroll
      for (int pp = 0; pp < 2; ++pp)
#pragma unroll
        for (int w = 0; w < 4; ++w) pb[pp].w[w] = pack2(p[8 * pp + 2 * w], p[8 * pp + 2 * w + 1]);
#pragma unroll
      for (int pp = 0; pp < 2; ++pp) {
        const int pgi = 2 * sb + pp;
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const int d = 32 * db + l32;
          Frag va;
          va.u = tiles[buf].v[(pgi * kD + d) * 2 + half];
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

// Rotary table, then the attention kernel. The optional timing events bracket the attention kernel alone.
hipError_t launch_prefill_mfma_bf16(const AttnArgs& a, hipStream_t s) {
  const int n_pos = prefill_mfma_table_positions(a.blocks_per_split * a.P);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n_pos * 32 + 255) / 256), dim3(256), 0, s, a, n_pos);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const unsigned grid = (unsigned)a.B * a.Hkv * a.n_splits;
  if (a.timing_start) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_start), s);
  hipLaunchKernelGGL(prefill_mfma_bf16_kernel, dim3(grid), dim3(kThreads), 0, s, a);
  e = hipGetLastError();
  if (a.timing_stop) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_stop), s);
  return e;
}

int prefill_mfma_rows_per_workgroup() { return kRows; }

// Positions the rotary table covers for contexts of up to max_kv_len slots: whole tiles of 64.
int prefill_mfma_table_positions(int max_kv_len) { return (max_kv_len + kTile - 1) / kTile * kTile; }

}  // namespace mepic
