// C-ABI entry points of the attention half of the library: argument checks, the split-K plan, the
// rotary frequency table, and dispatch to the kernels. No device memory is allocated here.
#include <cmath>
#include <cstring>
#include <mutex>

#include "attn_common.h"

// Scratch of mepic_attn_decode_noalloc: the split-K partials and their metadata live here instead of in a
// caller-supplied workspace. Every GPU the library runs on holds its own copy of the array, at its own address,
// until the process ends. In host code the name below is only a handle for hipGetSymbolAddress: the device
// address it yields (kept per device in g_scratch_ptr) is what kernels and runtime calls get.
static __device__ __align__(256) unsigned char scratch[MEPIC_NOALLOC_SCRATCH_BYTES];

namespace mepic {
namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device, with that device current).
int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MEPIC_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return MEPIC_ERR_LAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return MEPIC_OK;
}

thread_local const char* g_last_kernel = "";

enum Kernel { K_GENERAL = 0, K_DECODE_MFMA_BF16 = 1, K_DECODE_MFMA_F8 = 2, K_PREFILL_MFMA_BF16 = 3 };

struct Plan {
  Kernel kernel;
  int n_splits, blocks_per_split;
  size_t workspace_bytes;
};

int check_shapes(const mepic_attn_params* p, bool prefill) {
  if (!p) return MEPIC_ERR_INVALID;
  if (p->B < 0 || p->n_q_tokens < 0 || p->Hq <= 0 || p->Hkv <= 0 || p->max_blocks < 0 || p->num_pages < 0)
    return MEPIC_ERR_INVALID;
  if (p->Hq % p->Hkv) return MEPIC_ERR_INVALID;
  if (!prefill && p->n_q_tokens != p->B) return MEPIC_ERR_INVALID;
  const bool combo = (p->q_dtype == MEPIC_F32 && p->kv_dtype == MEPIC_F32) ||
                     (p->q_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_BF16) ||
                     (p->q_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_F8E4M3);
  if (!combo) return MEPIC_ERR_UNSUPPORTED;
  if (p->D != 64 && p->D != 128) return MEPIC_ERR_UNSUPPORTED;
  if (p->P != 16 && p->P != 32) return MEPIC_ERR_UNSUPPORTED;
  if (p->Hq / p->Hkv > kMaxG) return MEPIC_ERR_UNSUPPORTED;
  if (p->Hkv > 65535) return MEPIC_ERR_UNSUPPORTED;
  return MEPIC_OK;
}

Plan make_plan(const mepic_attn_params* p, bool prefill) {
  Plan pl{};
  const int G = p->Hq / p->Hkv;
  int max_kv = p->max_kv_len > 0 ? p->max_kv_len : p->max_blocks * p->P;
  if (max_kv > p->max_blocks * p->P) max_kv = p->max_blocks * p->P;
  const int n_blocks = (max_kv + p->P - 1) / p->P;
  const bool plain = !p->block_positions && !p->block_valid_mask &&
                     !(p->flags & (MEPIC_FLAG_ROPE_INTERLEAVED | MEPIC_FLAG_FORCE_GENERAL));
  pl.kernel = K_GENERAL;

  const bool mfma_bf16 = p->q_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_BF16 && p->D == 128 && p->P == 16;
  const bool mfma_fp8 = p->q_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_F8E4M3 && p->D == 128 && p->P == 32;
  if (!prefill && plain && G <= 16 && (mfma_bf16 || mfma_fp8) && p->B <= decode_mfma_max_requests()) {
    // Matrix-core decode: persistent waves cut each KV head's sequence of steps into equal chunks; here only
    // the bound on partials per request (sizes the workspace) and the minimum chunk are fixed.
    pl.kernel = mfma_fp8 ? K_DECODE_MFMA_F8 : K_DECODE_MFMA_BF16;
    decode_mfma_plan(p->B, p->Hkv, max_kv, mfma_fp8, &pl.n_splits, &pl.blocks_per_split);
    pl.workspace_bytes = (size_t)p->n_q_tokens * p->Hq * pl.n_splits * (p->D + 2) * sizeof(float) +
                         (size_t)(p->B + 2) * sizeof(int32_t);
    return pl;
  }

  if (prefill && plain && mfma_bf16 && prefill_mfma_rows_per_workgroup() % G == 0) {
    // Matrix-core prefill: one workgroup per (request, KV head, tile of 256 query rows); no split over KV, the
    // output is written directly. The workspace holds the rotary table.
    pl.kernel = K_PREFILL_MFMA_BF16;
    const int max_q = p->max_q_len > 0 && p->max_q_len < p->n_q_tokens ? p->max_q_len : p->n_q_tokens;
    const int tok_per_wg = prefill_mfma_rows_per_workgroup() / G;
    pl.n_splits = (max_q + tok_per_wg - 1) / tok_per_wg;
    if (pl.n_splits < 1) pl.n_splits = 1;
    pl.blocks_per_split = n_blocks;
    // the per-position rotary table the call builds for itself: 32 entries of 16 bytes per position
    pl.workspace_bytes = (size_t)prefill_mfma_table_positions(n_blocks * p->P) * 16 * sizeof(uint4) + 16;  // table + clock sample
    return pl;
  }

  // General path: one workgroup per (query token, KV head, split); a split is a whole number of
  // 256-slot tiles. Enough splits to put ~8 workgroups on each of the 256 compute units.
  const int tile_blocks = 256 / p->P;
  const long rows = (long)p->n_q_tokens * p->Hkv;
  int want = rows > 0 ? (int)((2048 + rows - 1) / rows) : 1;
  const int max_splits = (n_blocks + tile_blocks - 1) / tile_blocks;
  if (want > max_splits) want = max_splits;
  if (want > 1024) want = 1024;
  if (want < 1) want = 1;
  int bps = (n_blocks + want - 1) / want;
  bps = (bps + tile_blocks - 1) / tile_blocks * tile_blocks;
  if (bps < tile_blocks) bps = tile_blocks;
  pl.blocks_per_split = bps;
  pl.n_splits = n_blocks > 0 ? (n_blocks + bps - 1) / bps : 1;
  pl.workspace_bytes = (size_t)p->n_q_tokens * p->Hq * pl.n_splits * (p->D + 2) * sizeof(float);
  return pl;
}

void mark(void* ev, hipStream_t s) {
  if (ev) (void)hipEventRecord(reinterpret_cast<hipEvent_t>(ev), s);
}

int run(const mepic_attn_params* p, void* hip_stream, bool prefill) {
  const int rc = check_shapes(p, prefill);
  if (rc != MEPIC_OK) return rc;
  if (p->n_q_tokens == 0) return MEPIC_OK;
  if (!p->q || !p->out || !p->k_pages || !p->v_pages || !p->block_tables || !p->kv_lens || !p->q_positions)
    return MEPIC_ERR_INVALID;
  if (prefill && !p->cu_q_lens) return MEPIC_ERR_INVALID;
  if (p->kv_dtype == MEPIC_F8E4M3 && (!p->k_scales || !p->v_scales)) return MEPIC_ERR_INVALID;
  if (!(p->rope_theta > 0.f)) return MEPIC_ERR_INVALID;
  if ((p->timing_start == nullptr) != (p->timing_stop == nullptr)) return MEPIC_ERR_INVALID;

  const Plan pl = make_plan(p, prefill);
  if (pl.workspace_bytes && (!p->workspace || p->workspace_bytes < pl.workspace_bytes)) return MEPIC_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(p->workspace) & 255u) return MEPIC_ERR_INVALID;

  AttnArgs a{};
  a.timing_start = p->timing_start; a.timing_stop = p->timing_stop;
  a.q = p->q; a.out = p->out; a.k_pages = p->k_pages; a.v_pages = p->v_pages;
  a.k_scales = p->k_scales; a.v_scales = p->v_scales;
  a.block_tables = p->block_tables; a.kv_lens = p->kv_lens; a.q_positions = p->q_positions;
  a.cu_q_lens = prefill ? p->cu_q_lens : nullptr;
  a.block_positions = p->block_positions; a.block_valid_mask = p->block_valid_mask;
  a.B = p->B; a.n_q = p->n_q_tokens; a.Hq = p->Hq; a.Hkv = p->Hkv; a.D = p->D; a.P = p->P;
  a.max_blocks = p->max_blocks; a.num_pages = p->num_pages; a.G = p->Hq / p->Hkv;
  a.q_dtype = p->q_dtype; a.kv_dtype = p->kv_dtype;
  a.interleaved = (p->flags & MEPIC_FLAG_ROPE_INTERLEAVED) ? 1 : 0;
  a.kv_read_once = (p->flags & MEPIC_FLAG_KV_READ_ONCE) ? 1 : 0;
  a.causal = prefill ? 1 : 0;
  a.n_splits = pl.n_splits; a.blocks_per_split = pl.blocks_per_split;
  const double sm = p->sm_scale > 0.f ? (double)p->sm_scale : 1.0 / std::sqrt((double)p->D);
  a.qk_scale_log2 = (float)(sm * 1.4426950408889634);
  // frequencies in turns per position, f_i / (2 pi), as a two-float sum
  for (int i = 0; i < p->D / 2; ++i) {
    const double f = std::pow((double)p->rope_theta, -2.0 * i / (double)p->D) / 6.283185307179586476925;
    a.freq_hi[i] = (float)f;
    a.freq_lo[i] = (float)(f - (double)a.freq_hi[i]);
  }
  float* ws = reinterpret_cast<float*>(p->workspace);
  a.part_o = ws;
  a.part_ml = ws + (size_t)a.n_q * a.Hq * a.n_splits * a.D;
  a.part_meta = reinterpret_cast<int32_t*>(a.part_ml + (size_t)a.n_q * a.Hq * a.n_splits * 2);

  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  hipError_t e = hipSuccess;
  switch (pl.kernel) {
    case K_DECODE_MFMA_BF16:
    case K_DECODE_MFMA_F8:
      g_last_kernel = pl.kernel == K_DECODE_MFMA_F8 ? "decode_mfma_fp8" : "decode_mfma_bf16";
      e = launch_decode_mfma(a, s);
      break;
    case K_PREFILL_MFMA_BF16:
      g_last_kernel = "prefill_mfma_bf16";
      a.rope_table = reinterpret_cast<float4*>(p->workspace);
      e = launch_prefill_mfma_bf16(a, s);
      break;
    default:
      g_last_kernel = "general";
      mark(a.timing_start, s);
      e = launch_general(a, s);
      mark(a.timing_stop, s);
      if (e == hipSuccess) e = launch_combine(a, s);
      break;
  }
  return e == hipSuccess ? MEPIC_OK : MEPIC_ERR_LAUNCH;
}

// Batched decode: same checks as run(), then the plan-driven launch.
int run_batched(const mepic_attn_params* p, const int32_t* plan, const mepic_decode_plan_info* info, void* hip_stream,
                size_t* bytes_only) {
  const int rc = check_shapes(p, false);
  if (rc != MEPIC_OK) return rc;
  if (!info) return MEPIC_ERR_INVALID;
  const bool plain = !p->block_positions && !p->block_valid_mask &&
                     !(p->flags & (MEPIC_FLAG_ROPE_INTERLEAVED | MEPIC_FLAG_FORCE_GENERAL));
  const bool mfma_bf16 = p->q_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_BF16 && p->D == 128 && p->P == 16;
  const bool mfma_fp8 = p->q_dtype == MEPIC_BF16 && p->kv_dtype == MEPIC_F8E4M3 && p->D == 128 && p->P == 32;
  if (!plain || !(mfma_bf16 || mfma_fp8)) return MEPIC_ERR_UNSUPPORTED;
  if (info->B != p->B || info->n_splits < 1 || info->n_runs < 0 || info->r_cap != 16 / (p->Hq / p->Hkv))
    return MEPIC_ERR_INVALID;
  if ((size_t)(info->n_runs + 1) * sizeof(int) > 48 * 1024) return MEPIC_ERR_UNSUPPORTED;  // run prefix sums live in LDS
  // the plan cut the work for the waves of the device it was built on
  if (info->n_waves != decode_mfma_waves_per_head(p->Hkv, mfma_fp8)) return MEPIC_ERR_INVALID;
  const size_t need = (size_t)p->n_q_tokens * p->Hq * info->n_splits * (p->D + 2) * sizeof(float);
  if (bytes_only) {
    *bytes_only = need;
    return MEPIC_OK;
  }
  if (p->n_q_tokens == 0) return MEPIC_OK;
  if (!plan || !p->q || !p->out || !p->k_pages || !p->v_pages || !p->block_tables || !p->kv_lens || !p->q_positions)
    return MEPIC_ERR_INVALID;
  if (mfma_fp8 && (!p->k_scales || !p->v_scales)) return MEPIC_ERR_INVALID;
  if (!(p->rope_theta > 0.f)) return MEPIC_ERR_INVALID;
  if ((p->timing_start == nullptr) != (p->timing_stop == nullptr)) return MEPIC_ERR_INVALID;
  if (!p->workspace || p->workspace_bytes < need) return MEPIC_ERR_CAPACITY;
  if (reinterpret_cast<uintptr_t>(p->workspace) & 255u) return MEPIC_ERR_INVALID;

  AttnArgs a{};
  a.timing_start = p->timing_start; a.timing_stop = p->timing_stop;
  a.q = p->q; a.out = p->out; a.k_pages = p->k_pages; a.v_pages = p->v_pages;
  a.k_scales = p->k_scales; a.v_scales = p->v_scales;
  a.block_tables = p->block_tables; a.kv_lens = p->kv_lens; a.q_positions = p->q_positions;
  a.B = p->B; a.n_q = p->n_q_tokens; a.Hq = p->Hq; a.Hkv = p->Hkv; a.D = p->D; a.P = p->P;
  a.max_blocks = p->max_blocks; a.num_pages = p->num_pages; a.G = p->Hq / p->Hkv;
  a.q_dtype = p->q_dtype; a.kv_dtype = p->kv_dtype;
  a.n_splits = info->n_splits; a.blocks_per_split = 0;
  a.plan = plan;
  const double sm = p->sm_scale > 0.f ? (double)p->sm_scale : 1.0 / std::sqrt((double)p->D);
  a.qk_scale_log2 = (float)(sm * 1.4426950408889634);
  for (int i = 0; i < p->D / 2; ++i) {
    const double f = std::pow((double)p->rope_theta, -2.0 * i / (double)p->D) / 6.283185307179586476925;
    a.freq_hi[i] = (float)f;
    a.freq_lo[i] = (float)(f - (double)a.freq_hi[i]);
  }
  float* ws = reinterpret_cast<float*>(p->workspace);
  a.part_o = ws;
  a.part_ml = ws + (size_t)a.n_q * a.Hq * a.n_splits * a.D;
  g_last_kernel = mfma_fp8 ? "decode_mfma_fp8_batched" : "decode_mfma_bf16_batched";
  const hipError_t e = launch_decode_mfma_batched(a, info->n_runs, reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MEPIC_OK : MEPIC_ERR_LAUNCH;
}

}  // namespace
}  // namespace mepic

extern "C" {

int mepic_attn_decode_batched_workspace_size(const mepic_attn_params* params, const mepic_decode_plan_info* info,
                                             size_t* bytes_out) {
  if (!bytes_out) return MEPIC_ERR_INVALID;
  return mepic::run_batched(params, nullptr, info, nullptr, bytes_out);
}

int mepic_attn_decode_batched(const mepic_attn_params* params, const int32_t* plan_device,
                              const mepic_decode_plan_info* info, void* hip_stream) {
  return mepic::run_batched(params, plan_device, info, hip_stream, nullptr);
}

int mepic_attn_workspace_size(const mepic_attn_params* params, int is_prefill, size_t* bytes_out) {
  if (!bytes_out) return MEPIC_ERR_INVALID;
  const int rc = mepic::check_shapes(params, is_prefill != 0);
  if (rc != MEPIC_OK) return rc;
  *bytes_out = mepic::make_plan(params, is_prefill != 0).workspace_bytes;
  return MEPIC_OK;
}

int mepic_attn_decode(const mepic_attn_params* params, void* hip_stream) {
  return mepic::run(params, hip_stream, false);
}

int mepic_attn_decode_noalloc(const mepic_attn_params* params, void* hip_stream) {
  if (!params) return MEPIC_ERR_INVALID;
  const int rc = mepic::check_shapes(params, false);
  if (rc != MEPIC_OK) return rc;
  // same plan as mepic_attn_decode, so the same partials; they must fit the fixed array
  if (mepic::make_plan(params, false).workspace_bytes > (size_t)MEPIC_NOALLOC_SCRATCH_BYTES) return MEPIC_ERR_CAPACITY;
  void* ptr = nullptr;
  const int rs = mepic::scratch_of_current_device(&ptr);
  if (rs != MEPIC_OK) return rs;
  // Nothing in the array has to start at zero: the kernels write every partial and every metadata word the merge
  // kernel reads, so the contents a previous call left behind are never looked at.
  mepic_attn_params p = *params;
  p.workspace = ptr;
  p.workspace_bytes = (size_t)MEPIC_NOALLOC_SCRATCH_BYTES;
  return mepic::run(&p, hip_stream, false);
}

int mepic_attn_prefill(const mepic_attn_params* params, void* hip_stream) {
  return mepic::run(params, hip_stream, true);
}

const char* mepic_last_kernel(void) { return mepic::g_last_kernel; }

int mepic_probe_mfma_bf16(int32_t iters, int32_t random_operands, float* sink_device, double* flop_out, void* hip_stream) {
  if (iters < 0 || !sink_device || !flop_out) return MEPIC_ERR_INVALID;
  const int n_wg = mepic::device_compute_units();
  // per workgroup: 8 waves x iters x 4 products of 32 x 32 x 16 multiply-adds
  *flop_out = (double)n_wg * 8.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
  const hipError_t e = mepic::launch_mfma_rate_probe(iters, random_operands != 0, sink_device, n_wg, reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MEPIC_OK : MEPIC_ERR_LAUNCH;
}

int mepic_probe_tile_stream(int32_t structure, int32_t iters, float* buf_device, size_t buf_bytes, void* hip_stream) {
  if (structure < 0 || structure > 2 || iters < 0 || !buf_device || buf_bytes < 65536) return MEPIC_ERR_INVALID;
  const hipError_t e = mepic::launch_tile_stream_probe(structure, iters, buf_device, mepic::device_compute_units(),
                                                        reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MEPIC_OK : MEPIC_ERR_LAUNCH;
}

int mepic_device_counter_khz(int32_t* khz_out) {
  if (!khz_out) return MEPIC_ERR_INVALID;
  int dev = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess) return MEPIC_ERR_LAUNCH;
  if (hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || khz <= 0) return MEPIC_ERR_LAUNCH;
  *khz_out = khz;
  return MEPIC_OK;
}

int mepic_selftest_dot_rotation(const uint32_t* words_device, float* out_device, int32_t n, void* hip_stream) {
  if (n < 0 || (n && (!words_device || !out_device))) return MEPIC_ERR_INVALID;
  if (n == 0) return MEPIC_OK;
  const hipError_t e = mepic::launch_dot_rotate_selftest(words_device, out_device, n, reinterpret_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? MEPIC_OK : MEPIC_ERR_LAUNCH;
}

}  // extern "C"
