// Shared declarations of the attention kernels (device side of §3.3.3: fused-RoPE paged attention).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mepic.h"

namespace mepic {

constexpr int kMaxHalfD = 64;   // D <= 128
constexpr int kMaxG = 16;       // query heads per KV head the kernels are built for
constexpr float kLog2e = 1.4426950408889634f;

// Kernel arguments: the caller's pointers and shapes plus what the host derived from them.
struct AttnArgs {
  const void* q;
  void* out;
  const void* k_pages;
  const void* v_pages;
  const float* k_scales;
  const float* v_scales;
  const int32_t* block_tables;
  const int32_t* kv_lens;
  const int32_t* q_positions;
  const int32_t* cu_q_lens;          // null for decode
  const int32_t* block_positions;    // nullable
  const uint32_t* block_valid_mask;  // nullable
  float* part_o;                     // [n_q][Hq][n_splits][D] un-normalised partial outputs
  float* part_ml;                    // [n_q][Hq][n_splits][2] running max (log2 units) and sum
  void* timing_start;                // optional hipEvent_t pair around the main kernel
  void* timing_stop;
  int32_t* part_meta;                // stream-K decode: steps before each request [B+1], then the chunk
  const int32_t* plan;               // batched decode: the plan blob (device), see decode_plan.h
  float4* rope_table;                // matrix-core prefill: per-position cos/sin entries (built by the call itself)
  int32_t B, n_q, Hq, Hkv, D, P, max_blocks, num_pages, G;
  int32_t q_dtype, kv_dtype;
  int32_t interleaved, causal;
  int32_t kv_read_once;  // hint: pages are not shared between requests (matrix-core decode: non-temporal loads)
  int32_t n_splits, blocks_per_split;
  float qk_scale_log2;               // sm_scale * log2(e): scores are kept in log2 units
  // Rotary frequencies in turns per position, f_i / (2 pi), split into two floats whose sum carries
  // ~48 bits, so that position * frequency can be reduced modulo one turn without fp64.
  float freq_hi[kMaxHalfD];
  float freq_lo[kMaxHalfD];
};

// Fraction of a turn of pos * f_i, in [-0.5, 0.5], accurate to ~1e-7 turns for |pos| < 2^24.
__device__ __forceinline__ float turns_frac(float pos, float fhi, float flo) {
  const float p = pos * fhi;
  const float e = __builtin_fmaf(pos, fhi, -p);  // exact error of the product
  const float r = p - __builtin_rintf(p);        // exact
  return r + (e + pos * flo);
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// OCP e4m3fn code -> fp32 (exact). Exponent field 0 is subnormal: m * 2^-9.
__device__ __forceinline__ float e4m3_to_f32(uint32_t c) {
  const uint32_t em = c & 0x7fu;
  const float mag = em < 8u ? (float)em * 0x1p-9f : __uint_as_float((em << 20) + (120u << 23));
  return (c & 0x80u) ? -mag : mag;
}

// Round-to-nearest-even fp32 -> bf16 bits (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Launchers (host). Each returns a hipError_t from the launch.
hipError_t launch_general(const AttnArgs& a, hipStream_t s);
hipError_t launch_combine(const AttnArgs& a, hipStream_t s);
hipError_t launch_decode_mfma(const AttnArgs& a, hipStream_t s);  // bf16 or fp8 pages; includes its merge kernel
hipError_t launch_prefill_mfma_bf16(const AttnArgs& a, hipStream_t s);  // n_splits = query tiles per request
int prefill_mfma_rows_per_workgroup();
int prefill_mfma_table_positions(int max_kv_len);                    // positions its rotary table covers (16 bytes x 16 each)
void decode_mfma_plan(int B, int Hkv, int max_kv_len, bool fp8, int* max_splits, int* min_chunk);
hipError_t launch_dot_rotate_selftest(const uint32_t* words, float* out, int n, hipStream_t s);
hipError_t launch_mfma_rate_probe(int iters, bool random_operands, float* sink, int n_workgroups, hipStream_t s);  // 512 threads each
hipError_t launch_tile_stream_probe(int structure, int iters, float* buf, int n_workgroups, hipStream_t s);
int device_compute_units();
int decode_mfma_max_requests();                                       // B the plain walker's LDS has room for
int decode_mfma_waves_per_head(int Hkv, bool fp8);                   // waves that share one KV head's steps
hipError_t launch_decode_mfma_batched(const AttnArgs& a, int n_runs, hipStream_t s);  // plan-driven variant

}  // namespace mepic
