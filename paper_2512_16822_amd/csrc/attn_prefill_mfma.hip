// Matrix-core prefill kernel of fused-RoPE paged attention (§3.3.3) for bf16, D = 128, P = 16:
// question tokens attend causally (by absolute position) to their request's paged, un-rotated KV.
//
// One workgroup of 8 waves serves 256 query rows (a row = one query token x one of the G query heads
// that share a KV head; 256/G tokens) of one (request, KV head) and walks the request's KV in tiles of
// 64 slots (4 pages). What a tile costs is not matrix-pipe time but the waits of its two waves per SIMD (for
// global loads, for LDS operands, for each other at the barrier), so the kernel is arranged around those:
//   stage   every thread pulls two 16-byte granules of K and two of V from the pages (issued two whole tiles before
//           they are needed, into two alternating register sets) and rotates K in registers at the slot's absolute
//           position with cos/sin read from a per-position half-precision table (built once per call by
//           rope_table_kernel: no trigonometry and no rotation state to advance in the loop), then writes both to
//           LDS: K as bf16 in matrix-operand order, V as it lies in the page (16-byte pieces swapped pairwise so that
//           operand reads hit every bank once). The rotated tile is shared by all 256 rows, so the rotation costs
//           1/256 per row.
//   QK      S^T[64 slots x 32 rows] per wave = Khat (LDS) x Qhat^T (registers), v_mfma_f32_32x32x16_bf16.
//           Transposed so that a lane owns one query row: row sums are register-local. The accumulator starts
//           at minus the row's reference maximum, so the scores come out of the products already shifted.
//           The matrix rows are assigned to the tile's slots in an order that leaves a lane with the
//           probabilities of eight consecutive slots of one page: exactly the 16-byte piece of a V page row.
//   softmax online; the reference maximum is a lower bound raised only when a probability would get huge (the
//           test is on the row sum that is needed anyway), causal / length mask only on tiles that need it.
//   PV      O^T[128 x 32 rows] += V^T (LDS) x P^T (the S^T registers, packed in place).
// Matrix operands come from LDS through a ring of four register quadruples: the read for the product four places
// ahead is issued right behind each product, so products do not wait for LDS. Three LDS tile buffers and ONE
// barrier per tile; the waves of a SIMD belong to two groups that stage the next tile before, respectively after,
// that barrier, which keeps them one segment apart. Page ids come 64 at a time through a vector load and
// v_readlane: nothing in the loop uses the scalar-memory counter the LDS waits share.
#include <mutex>
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

typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;  // scalar loads: set-up only, never in the loop
__device__ __forceinline__ int sload(const int32_t* p, size_t idx) { return ((const_i32_ptr)(uintptr_t)p)[idx]; }
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// Per-position rotary table in half precision (11 significant bits: eight times finer than the bf16 rounding of the
// rotated keys): for position p and the four frequencies i0 .. i0 + 3, i0 = 8 pc + 4 e, one 16-byte entry
// {cos, sin}(p f_i0), {cos, sin}(p f_i0+1), ... at entry index
//   (((p / 64) * 8 + pc) * 2 + e) * 64 + p % 64,
// so that the 64 lanes of a wave, which stage 64 consecutive positions for one (pc, e), read 1 KB in one piece.
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
union HFrag {
  uint4 u;
  half8 h;
};
__host__ __device__ constexpr int prefill_table_positions(int max_kv_len) { return (max_kv_len + 63) / 64 * 64; }  // whole tiles
__device__ __forceinline__ size_t rope_entry(int p, int pc, int e) {
  return ((((size_t)(p >> 6) * 8 + pc) * 2 + e) << 6) + (p & 63);
}

__global__ __launch_bounds__(256) void rope_table_kernel(const AttnArgs a, int n_pos) {
  const int idx = blockIdx.x * 256 + threadIdx.x;   // (p / 64, pc, e, p % 64), the entry index itself
  if (idx >= n_pos * 16) return;
  const int p = ((idx >> 10) << 6) + (idx & 63), pc = (idx >> 7) & 7, e = (idx >> 6) & 1;
  HFrag r;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int i = 8 * pc + 4 * e + j;
    const float t = turns_frac((float)p, a.freq_hi[i], a.freq_lo[i]);
    r.h[2 * j] = (_Float16)__builtin_amdgcn_cosf(t);
    r.h[2 * j + 1] = (_Float16)__builtin_amdgcn_sinf(t);
  }
  reinterpret_cast<uint4*>(a.rope_table)[idx] = r.u;
}

// LDS tile layouts (per buffer):
//   K: [16 chunks of 8 dims][64 slots] granules of 16 bytes -> granule (c, s) at c*64 + s, rotated, bf16
//   V: the tile's four page-heads, [4 pages][128 dims][2 halves of 8 slots] granules, the two halves of a dim
//      swapped when bit 3 of the dim is set (16 consecutive lanes of an operand read then cover all 64 banks)
constexpr int kNBuf = 3;
// Workgroup barrier that orders LDS traffic only: global loads issued before it stay in flight across it.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
struct __align__(16) Tile {
  uint4 k[16 * kTile];
  uint4 v[4 * kD * 2];
};

__global__ __launch_bounds__(kThreads, 1) void prefill_mfma_bf16_kernel(const AttnArgs a) {
  extern __shared__ uint4 lds_all[];
  Tile* const tiles = reinterpret_cast<Tile*>(lds_all);   // kNBuf tiles
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int l32 = lane & 31, half = lane >> 5;
  const int G = a.G, Hkv = a.Hkv;
  const int hk = blockIdx.x % Hkv;
  const int qt = (blockIdx.x / Hkv) % a.n_splits;  // n_splits carries the number of query tiles per request
  const int b = blockIdx.x / Hkv / a.n_splits;

  // Workgroup 0 reports how long it ran in core clocks and in ticks of the constant-rate counter (16 bytes behind
  // the rotary table): the ratio is the clock the kernel actually ran at, which power management sets well below
  // the nominal one under this instruction mix.
  unsigned long long clk0 = 0, rt0 = 0;
  if (blockIdx.x == 0) {
    clk0 = __builtin_readcyclecounter();
    rt0 = __builtin_amdgcn_s_memrealtime();
  }
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
  const uint4* table = reinterpret_cast<const uint4*>(a.rope_table) + rope_entry(s_st, pc, 0);   // + 1024 entries per tile, + 64 per e
  const size_t bt_row = (size_t)b * a.max_blocks;
  // V of a tile: wave w moves half w%2 (64 dims = 2 KB) of page-head w/2
  const int v_page_sel = wave >> 1, v_gran0 = (wave & 1) * 128 + lane;

  // What a thread has in flight for one tile: two K granules, the table entries of its eight frequencies, two V
  // granules. Two such sets: the loads of a tile are issued two tiles before they are staged.
  struct Staged {
    Frag gk[2], gv[2];
    HFrag gt[2];
  };
  Staged set_a, set_b;
  auto load_tile = [&](Staged& S, int t, int p0, int p1, int p2, int p3) __attribute__((always_inline)) {
    const int pg_k = (s_st < 32) ? (s_st < 16 ? p0 : p1) : (s_st < 48 ? p2 : p3);
    const size_t kb = ((size_t)pg_k * Hkv + hk) * (kD / 8 * kP) + (size_t)pc * kP + (s_st & 15);
    S.gk[0].u = kpages[kb];
    S.gk[1].u = kpages[kb + 8 * kP];
    S.gt[0].u = table[(size_t)t * 1024];
    S.gt[1].u = table[(size_t)t * 1024 + 64];
    const int pg_v = v_page_sel < 2 ? (v_page_sel == 0 ? p0 : p1) : (v_page_sel == 2 ? p2 : p3);  // wave-uniform
    const uint4* vsrc = vpages + ((size_t)pg_v * Hkv + hk) * (kD * 2) + v_gran0;
    S.gv[0].u = vsrc[0];
    S.gv[1].u = vsrc[64];
  };
  // rotate the staged K granules at position (tile start + s_st) and write them into LDS buffer `buf`; V goes there as
  // loaded, except that slots at or past kv_len, which may hold anything (NaN included: 0 x NaN would poison the
  // row), are zeroed
  auto stage_tile = [&](Staged& S, int buf, int n0) __attribute__((always_inline)) {
    Frag klo, khi;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t lo2 = S.gk[0].w[w], hi2 = S.gk[1].w[w];
      const float l0 = bf16_bits_to_f32(lo2), l1 = __uint_as_float(lo2 & 0xffff0000u);
      const float h0 = bf16_bits_to_f32(hi2), h1 = __uint_as_float(hi2 & 0xffff0000u);
      // {cos, sin} of frequencies 8pc + 2w and 8pc + 2w + 1 at this slot's position; the half-precision values feed
      // mixed-precision multiply-adds directly (fma with a zero addend instead of a multiply keeps them unconverted)
      const half8 r = S.gt[w >> 1].h;
      const float c0 = (float)r[4 * (w & 1)], s0 = (float)r[4 * (w & 1) + 1];
      const float c1 = (float)r[4 * (w & 1) + 2], s1 = (float)r[4 * (w & 1) + 3];
      klo.w[w] = pack2(__builtin_fmaf(l0, c0, -__builtin_fmaf(h0, s0, 0.f)), __builtin_fmaf(l1, c1, -__builtin_fmaf(h1, s1, 0.f)));
      khi.w[w] = pack2(__builtin_fmaf(h0, c0, __builtin_fmaf(l0, s0, 0.f)), __builtin_fmaf(h1, c1, __builtin_fmaf(l1, s1, 0.f)));
    }
    tiles[buf].k[pc * kTile + s_st] = klo.u;
    tiles[buf].k[(pc + 8) * kTile + s_st] = khi.u;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int gi = v_gran0 + 64 * i;              // granule of the page-head: dim gi / 2, slots 8 (gi & 1)..
      const int nbase = n0 + v_page_sel * kP + 8 * (gi & 1);
      Frag x = S.gv[i];
      if (nbase + 8 > L) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int n = nbase + 2 * w;
          x.w[w] &= (n < L ? 0x0000ffffu : 0u) | (n + 1 < L ? 0xffff0000u : 0u);
        }
      }
      tiles[buf].v[v_page_sel * (kD * 2) + (gi ^ ((gi >> 4) & 1))] = x.u;
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
  float negm = 0.f;   // minus the reference maximum: where the score accumulators start

  // Page ids of 16 tiles at a time: lane i of bt_cur holds the page of block 64 * bt_win + i (clamped to the
  // request's last block), bt_nxt the 64 after those; a tile reads its four ids with v_readlane. Vector loads on
  // purpose: scalar loads share a counter with the LDS reads and return out of order, so one in flight would turn
  // every wait for an LDS operand into a full drain.
  // (ids forced into [0, num_pages): a corrupt table reads a wrong page instead of faulting)
  auto bt_load = [&](int win) {
    return max(min(a.block_tables[bt_row + min(64 * win + lane, max(n_blocks - 1, 0))], a.num_pages - 1), 0);
  };
  int bt_win = 0, bt_cur = 0, bt_nxt = 0;
  if (n_tiles > 0) {   // (a request without visible slots has nothing to read, possibly not even a block table)
    bt_cur = bt_load(0);
    bt_nxt = bt_load(1);
  }
  auto pages_of = [&](int t, int& p0, int& p1, int& p2, int& p3) __attribute__((always_inline)) {  // non-decreasing t
    if ((t >> 4) != bt_win) {
      ++bt_win;
      bt_cur = bt_nxt;
      bt_nxt = bt_load(bt_win + 1);
    }
    const int l0 = (4 * t) & 63;
    p0 = __builtin_amdgcn_readlane(bt_cur, l0);
    p1 = __builtin_amdgcn_readlane(bt_cur, l0 + 1);
    p2 = __builtin_amdgcn_readlane(bt_cur, l0 + 2);
    p3 = __builtin_amdgcn_readlane(bt_cur, l0 + 3);
  };
  int np0 = 0, np1 = 0, np2 = 0, np3 = 0;

  // Matrix row m of a 32-slot block holds slot (m & 16) + 8 * bit2(m) + 4 * bit3(m) + (m & 3) of the block: a lane
  // of the score tile (row l32, half) then owns, in accumulator order, slots 8 half .. 8 half + 7 of the block's first
  // page and the same of its second page.
  const int k_read = (l32 & 16) + ((l32 & 4) << 1) + ((l32 & 8) >> 1) + (l32 & 3);

  // Operand j of a tile's 32 products: 0-7 K rows of slots 0-31, 8-15 K rows of slots 32-63, 16-23 V of pages 0, 1,
  // 24-31 V of pages 2, 3.
  constexpr int kRing = 4;
  auto tile_step = [&](int t, int buf) __attribute__((always_inline)) {
    const int n0 = t * kTile;
    const bool need_mask = n0 + kTile - 1 > min(pos_min, L - 1);  // some row cannot see the whole tile
    // Operand ring: the LDS read of the operand that the product kRing places later needs is issued right after
    // a product has consumed the ring entry, so that no product waits for LDS.
    Frag ring[kRing];
    const uint4* kt = tiles[buf].k + half * kTile + k_read;
    const uint4* vt = tiles[buf].v + l32 * 2 + (half ^ ((l32 >> 3) & 1));
    auto operand = [&](int j) __attribute__((always_inline)) {
      if (j < 16) return kt[2 * (j & 7) * kTile + 32 * (j >> 3)];
      const int jj = j - 16;
      return vt[((jj >> 2) * kD + 32 * (jj & 3)) * 2];
    };
#pragma unroll
    for (int i = 0; i < kRing; ++i) ring[i].u = operand(i);
    floatx16 sc2[2];
    {
      float nm = negm;
      asm volatile("" : "+v"(nm));   // a value of this tile: keeps sixteen copies of it from living across tiles
#pragma unroll
      for (int e = 0; e < 16; ++e) sc2[0][e] = sc2[1][e] = nm;
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      sc2[i >> 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[i % kRing].v, bq[i & 7].v, sc2[i >> 3], 0, 0, 0);
      ring[i % kRing].u = operand(i + kRing);
    }
    // pin the order: kRing reads, then sixteen times (product, read of the operand kRing products ahead)
    __builtin_amdgcn_sched_group_barrier(0x100, kRing, 0);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int sb = 0; sb < 2; ++sb) {
      floatx16 sc = sc2[sb];
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
          negm = -m_run;
          if (sb == 0) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sc2[1][e] -= delta;   // the second block's scores were shifted by the old reference
          }
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
      int n_reads = 0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int j = 16 + 8 * sb + i;
        o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[j % kRing].v, pb[i >> 2].v, o[i & 3], 0, 0, 0);
        if (j + kRing < 32) {
          ring[j % kRing].u = operand(j + kRing);
          ++n_reads;
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (i < n_reads) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Two groups of waves (one wave of each per SIMD) run the same sequence one segment apart, so that the matrix
  // segments of one fall on the vector segments of the other: group 0 stages the next tile BEFORE the tile's one
  // barrier, group 1 AFTER it. Three LDS buffers, so that staging tile t+1 never touches what tile t-1's products
  // still read. The global loads of tile t+3 are issued when tile t+1 has been staged out of their registers.
  // Staging and loading are unconditional in the loop (past the last tile they repeat the last tile into a buffer
  // nobody reads): the counts behind the compiler's waits for in-flight loads are then the same on every path.
  const int grp = wave >> 2;
  const int t_last = n_tiles - 1;
  int bi = 0;
  auto iteration = [&](Staged& S, int t) __attribute__((always_inline)) {   // S: the set that holds tile t + 1
    const int bn = bi + 1 == kNBuf ? 0 : bi + 1;
    if (grp) lds_barrier();
    stage_tile(S, bn, min(t + 1, t_last) * kTile);
    {
      const int tn = min(t + 3, t_last);
      pages_of(tn, np0, np1, np2, np3);
      load_tile(S, tn, np0, np1, np2, np3);
    }
    if (!grp) lds_barrier();
    if (t < n_tiles) tile_step(t, bi);
    bi = bn;
  };
  if (n_tiles > 0) {
    pages_of(0, np0, np1, np2, np3);
    load_tile(set_a, 0, np0, np1, np2, np3);
    pages_of(min(1, t_last), np0, np1, np2, np3);
    load_tile(set_b, min(1, t_last), np0, np1, np2, np3);
    stage_tile(set_a, 0, 0);
    pages_of(min(2, t_last), np0, np1, np2, np3);
    load_tile(set_a, min(2, t_last), np0, np1, np2, np3);
    lds_barrier();
    for (int t = 0; t < n_tiles; t += 2) {
      iteration(set_b, t);
      iteration(set_a, t + 1);
    }
  }

  if (blockIdx.x == 0 && tid == 0) {
    unsigned long long* sample = reinterpret_cast<unsigned long long*>(
        reinterpret_cast<uint4*>(a.rope_table) + (size_t)prefill_table_positions(a.blocks_per_split * kP) * 16);
    sample[0] = __builtin_readcyclecounter() - clk0;
    sample[1] = __builtin_amdgcn_s_memrealtime() - rt0;
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
  hipLaunchKernelGGL(rope_table_kernel, dim3((n_pos * 16 + 255) / 256), dim3(256), 0, s, a, n_pos);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const unsigned grid = (unsigned)a.B * a.Hkv * a.n_splits;
  if (a.timing_start) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_start), s);
  // three tile buffers are more LDS than a kernel gets by default: ask once per process (the attribute sticks)
  static std::once_flag lds_once;
  static hipError_t lds_status = hipSuccess;
  std::call_once(lds_once, [] {
    lds_status = hipFuncSetAttribute(reinterpret_cast<const void*>(&prefill_mfma_bf16_kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kNBuf * sizeof(Tile)));
  });
  if (lds_status != hipSuccess) return lds_status;
  hipLaunchKernelGGL(prefill_mfma_bf16_kernel, dim3(grid), dim3(kThreads), kNBuf * sizeof(Tile), s, a);
  e = hipGetLastError();
  if (a.timing_stop) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(a.timing_stop), s);
  return e;
}

int prefill_mfma_rows_per_workgroup() { return kRows; }

// Positions the rotary table covers for contexts of up to max_kv_len slots: whole tiles of 64.
int prefill_mfma_table_positions(int max_kv_len) { return prefill_table_positions(max_kv_len); }

}  // namespace mepic
