/*
 * mepic_oracle.c — TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, fp64 CPU statement of what fused-RoPE paged attention computes (§3.3.3 of the
 * paper): K is stored without positional encoding in pages; for every query row the oracle gathers
 * each key through the request's block table, rotates it explicitly at its absolute position, and
 * runs textbook max-subtracted softmax attention. The paper states that this reaches the same result
 * as rotating before storing (standard paged attention), so the oracle is that definition written
 * out; there is no tiling, fusion or reordering here.
 *
 * It shares no code with the HIP library: own page indexing, own bf16 / e4m3 decoding, own RoPE,
 * own softmax. Only tests, the smoke check and the bench's cpu_baseline leg may call it.
 *
 * Readings the paper leaves open (it prints no formula): frequency f_i = theta^(-2i/D); half-split
 * pairing (i, i+D/2) unless `interleaved`; V is not rotated; query head h uses KV head h/(Hq/Hkv);
 * softmax scale 1/sqrt(D) unless given; pad slots are ordinary slots unless masked out.
 *
 * Pins (tests/test_oracle_pins.py): brute force over contiguous pre-rotated K/V, position-shift
 * invariance, shared == duplicated page layouts, the D=2 closed form cos(m-n), uniform softmax
 * gather accounting, norm preservation / single key, chunk permutation. The pairing convention and
 * the pad treatment are readings, not facts of the paper: "parity unpinned" for those two choices.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { OR_F32 = 0, OR_BF16 = 1, OR_F8E4M3 = 2 };

/* bf16 is the upper half of an IEEE binary32. */
static double bf16_to_double(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* OCP 8-bit float E4M3 ("fn" flavour): 1 sign, 4 exponent (bias 7), 3 mantissa bits; no infinity;
 * S.1111.111 is NaN; exponent field 0 is subnormal: value = m/8 * 2^-6. Largest finite = 448. */
static double e4m3_to_double(uint8_t c) {
  int sign = c >> 7, e = (c >> 3) & 0xF, m = c & 7;
  double v;
  if (e == 0xF && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m / 8.0, -6);
  else v = ldexp(1.0 + (double)m / 8.0, e - 7);
  return sign ? -v : v;
}

static double load_elem(const void* base, int dtype, size_t idx) {
  switch (dtype) {
    case OR_F32: return (double)((const float*)base)[idx];
    case OR_BF16: return bf16_to_double(((const uint16_t*)base)[idx]);
    default: return e4m3_to_double(((const uint8_t*)base)[idx]);
  }
}

static int granule_elems(int dtype) { return dtype == OR_F32 ? 4 : dtype == OR_BF16 ? 8 : 16; }

/* Exposed so a test can pin the decoders against a library's conversion. */
double oracle_decode_elem(int dtype, uint32_t bits) {
  if (dtype == OR_BF16) return bf16_to_double((uint16_t)bits);
  if (dtype == OR_F8E4M3) return e4m3_to_double((uint8_t)bits);
  float f;
  memcpy(&f, &bits, 4);
  return (double)f;
}

/* Rotate x[0..D) in place at integer position pos: RoPE with base theta. */
static void rope(double* x, int D, long pos, double theta, int interleaved) {
  int half = D / 2;
  for (int i = 0; i < half; ++i) {
    double f = pow(theta, -2.0 * (double)i / (double)D);
    double a = (double)pos * f, c = cos(a), s = sin(a);
    int i0 = interleaved ? 2 * i : i, i1 = interleaved ? 2 * i + 1 : i + half;
    double x0 = x[i0], x1 = x[i1];
    x[i0] = x0 * c - x1 * s;
    x[i1] = x1 * c + x0 * s;
  }
}

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/*
 * Attention for a list of (query token, query head) rows.
 *
 *   rows[2*r] = query token t, rows[2*r+1] = query head h; out[r*D .. r*D+D) receives the row.
 *   rows == NULL means all n_q*Hq rows in (t, h) order (n_rows is then ignored).
 *   cu_q_lens == NULL means decode: token t belongs to request t, no causal mask.
 *   Otherwise token t belongs to the request b with cu_q_lens[b] <= t < cu_q_lens[b+1] and a key
 *   takes part only if its position <= the query's position.
 * Returns 0, or -1 for a page id outside [0, num_pages) / a bad argument.
 */
int oracle_attn(const void* q, int q_dtype, const void* k_pages, const void* v_pages, int kv_dtype,
                const float* k_scales, const float* v_scales, const int32_t* block_tables,
                const int32_t* kv_lens, const int32_t* q_positions, const int32_t* cu_q_lens,
                const int32_t* block_positions, const uint32_t* block_valid_mask, int B, int n_q,
                int Hq, int Hkv, int D, int P, int max_blocks, int num_pages, double theta,
                double sm_scale, int interleaved, const int32_t* rows, int n_rows, double* out) {
  if (Hkv <= 0 || Hq % Hkv || D % 2 || P <= 0) return -1;
  if (!rows) n_rows = n_q * Hq;
  if (sm_scale <= 0) sm_scale = 1.0 / sqrt((double)D);
  const int G = Hq / Hkv, X = granule_elems(kv_dtype);
  int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
  for (int r = 0; r < n_rows; ++r) {
    const int t = rows ? rows[2 * r] : r / Hq, h = rows ? rows[2 * r + 1] : r % Hq;
    int b = t;
    if (cu_q_lens) {
      b = 0;
      while (b < B - 1 && t >= cu_q_lens[b + 1]) ++b;
    }
    const int hk = h / G;
    const long pos_q = q_positions[t];
    const int L = kv_lens[b];
    double* qr = (double*)malloc(sizeof(double) * (size_t)D);
    double* kr = (double*)malloc(sizeof(double) * (size_t)D);
    double* score = (double*)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
    char* take = (char*)malloc((size_t)(L > 0 ? L : 1));
    double* o = out + (size_t)r * D;

    for (int d = 0; d < D; ++d) qr[d] = load_elem(q, q_dtype, ((size_t)t * Hq + h) * D + d);
    rope(qr, D, pos_q, theta, interleaved);

    /* scores over every logical slot of the request */
    for (int n = 0; n < L; ++n) {
      const int j = n / P, s = n % P;
      const int32_t page = block_tables[(size_t)b * max_blocks + j];
      take[n] = 0;
      if (page < 0 || page >= num_pages) {
#pragma omp atomic write
        bad = 1;
        continue;
      }
      if (block_valid_mask && !((block_valid_mask[(size_t)b * max_blocks + j] >> s) & 1u)) continue;
      const long pos_k = block_positions ? (long)block_positions[(size_t)b * max_blocks + j] + s : (long)n;
      if (cu_q_lens && pos_k > pos_q) continue;
      const size_t head_base = ((size_t)page * Hkv + hk) * (size_t)D * P;
      const double ksc = kv_dtype == OR_F8E4M3 ? (double)k_scales[page] : 1.0;
      for (int d = 0; d < D; ++d)
        kr[d] = ksc * load_elem(k_pages, kv_dtype, head_base + ((size_t)(d / X) * P + s) * X + d % X);
      rope(kr, D, pos_k, theta, interleaved);
      double acc = 0.0;
      for (int d = 0; d < D; ++d) acc += qr[d] * kr[d];
      score[n] = sm_scale * acc;
      take[n] = 1;
    }

    /* softmax over the slots that take part, then the weighted sum of their V rows */
    double mx = -INFINITY;
    for (int n = 0; n < L; ++n)
      if (take[n] && score[n] > mx) mx = score[n];
    double denom = 0.0;
    for (int n = 0; n < L; ++n)
      if (take[n]) denom += exp(score[n] - mx);
    for (int d = 0; d < D; ++d) o[d] = 0.0;
    for (int n = 0; n < L; ++n) {
      if (!take[n]) continue;
      const int j = n / P, s = n % P;
      const int32_t page = block_tables[(size_t)b * max_blocks + j];
      const size_t head_base = ((size_t)page * Hkv + hk) * (size_t)D * P;
      const double vsc = kv_dtype == OR_F8E4M3 ? (double)v_scales[page] : 1.0;
      const double p = exp(score[n] - mx) / denom;
      for (int d = 0; d < D; ++d)
        o[d] += p * vsc * load_elem(v_pages, kv_dtype, head_base + (size_t)d * P + s);
    }
    free(qr); free(kr); free(score); free(take);
  }
  return bad ? -1 : 0;
}
