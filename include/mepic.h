/*
 * mepic.h — C-ABI boundary of the MI355X (gfx950) implementation of the hot path of MEPIC's
 * position-independent KV caching: paged-KV attention with rotary embedding fused into the kernel,
 * plus the host-side page pool / chunk-to-page aligner that produces the block tables.
 *
 * Paper passages each call follows are cited per declaration (section / algorithm / figure only).
 *
 * Conventions that hold for every call:
 *   - returns a mepic_status (0 = ok, negative = error); nothing throws or aborts across the ABI (a host
 *     allocation that fails inside the pool or the planner comes back as MEPIC_ERR_NOMEM; a pool that reported it
 *     from mepic_align_request or mepic_release_request is in an unspecified state and can only be destroyed);
 *   - the caller owns every buffer. "device" pointers are HIP device memory reachable from the
 *     current device; "host" pointers are ordinary host memory. The library never allocates or frees
 *     device memory; the pool owns only its own host metadata;
 *   - attention calls are asynchronous on the given HIP stream; the params struct is read on the host
 *     during the call and may be freed as soon as the call returns;
 *   - outputs are undefined after an error;
 *   - the pool is not thread-safe (one scheduler thread, as in the paper's scheduling path, §3.2).
 */
#ifndef MEPIC_H
#define MEPIC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MEPIC_OK = 0,
  MEPIC_ERR_INVALID = -1,     /* null pointer, zero-length segment, inconsistent shapes, key/length clash */
  MEPIC_ERR_NOMEM = -2,       /* Alg. 1 "Reject": free + evictable pages cannot cover the demand          */
  MEPIC_ERR_CAPACITY = -3,    /* a caller-supplied output buffer or workspace is too small                */
  MEPIC_ERR_UNSUPPORTED = -4, /* shape / dtype combination no kernel is built for                         */
  MEPIC_ERR_LAUNCH = -5       /* the HIP runtime reported an error at launch                              */
} mepic_status;

/* Static, human-readable text for a status code (never NULL). */
const char* mepic_strerror(int status);

/* Library version as major*10000 + minor*100 + patch. */
int mepic_version(void);

/* ------------------------------------------------------------------------------------------------
 * Host-side page pool and chunk-to-page aligner (metadata only; §3.2, Alg. 1).
 *
 * The pool tracks `num_pages` physical KV pages of `page_size` token slots each. One pool serves
 * request-private pages and shared chunk pages alike (§3.2.3 "shared paged-KV block pool").
 *
 * Allocation policy is deterministic so block tables are reproducible bit for bit:
 *   - the lowest-numbered free page is handed out first;
 *   - segments are processed left to right; for a chunk occurrence the private first block is
 *     allocated before the chunk's shared pages.
 * ---------------------------------------------------------------------------------------------- */
typedef struct mepic_pool mepic_pool; /* opaque */

enum { MEPIC_SEG_PROMPT = 0, MEPIC_SEG_CHUNK = 1 };

/* One segment of a request (§3.2.1): request-specific prompt text, or an immutable reusable chunk. */
typedef struct {
  uint32_t kind;      /* MEPIC_SEG_PROMPT or MEPIC_SEG_CHUNK                                        */
  uint32_t n_tokens;  /* > 0                                                                        */
  uint64_t chunk_key; /* identity of the chunk's padded token sequence (§3.2.3); ignored for prompts.
                         Two segments with equal key must have equal n_tokens.                      */
} mepic_segment;

/* Per-block provenance written by mepic_align_request. */
enum { MEPIC_BLOCK_PRIVATE = 0, MEPIC_BLOCK_SHARED_HIT = 1, MEPIC_BLOCK_SHARED_NEW = 2 };

typedef struct {
  uint32_t n_blocks;     /* logical blocks of the aligned request (= block-table entries written)   */
  uint32_t n_private;    /* request-private blocks (prompt blocks + the first block of every chunk) */
  uint32_t n_shared_hit; /* shared blocks whose chunk was already resident                          */
  uint32_t n_shared_new; /* shared blocks allocated for a chunk seen for the first time             */
  uint32_t n_pad_slots;  /* pad slots inserted (leading pads of chunks + trailing pads of prompts)   */
  uint32_t kv_len;       /* length of the padded sequence T_align, including extra_tail_tokens      */
  uint32_t n_evicted_chunks; /* zero-reference chunks evicted to admit this request                 */
} mepic_align_info;

typedef struct {
  uint64_t pages_total;
  uint64_t pages_free;
  uint64_t pages_in_use_unique;      /* pages currently allocated (private + resident shared)       */
  uint64_t pages_logical_duplicated; /* sum of n_blocks over live requests: what a layout in which
                                        every request owns all of its blocks would occupy           */
  uint64_t chunks_resident;          /* chunks whose shared pages are in the pool                   */
  uint64_t chunks_zero_ref;          /* resident chunks no live request references (evictable)      */
  uint64_t requests_live;
  uint64_t peak_pages_in_use_unique; /* high-water marks since creation                              */
  uint64_t peak_pages_logical_duplicated;
} mepic_pool_stats;

/* Create a pool of `num_pages` pages with `page_size` slots (1..32) each. *out receives the pool. */
int mepic_pool_create(uint32_t num_pages, uint32_t page_size, mepic_pool** out);
void mepic_pool_destroy(mepic_pool* pool);

/*
 * Align one request to pages and assign its blocks (Alg. 1: segmentation and canonicalisation,
 * residency resolution, admission check, block allocation; padding rule of §3.2.1; first-block rule
 * of §3.2.3 / §3.3.1).
 *
 *   segs[n_segs]       host, the request's segments in order.
 *   extra_tail_tokens  tokens appended after the last segment in request-private pages (1 for the
 *                      token being decoded). They continue in a final prompt segment's partial block.
 *   block_table_out    host int32[capacity]: physical page of each logical block.
 *   block_kind_out     host uint8[capacity] or NULL: MEPIC_BLOCK_* of each block.
 *   block_valid_out    host uint32[capacity] or NULL: bit s set iff slot s of the block holds a real
 *                      token (pad slots and the unused tail of the last block are 0).
 *   block_pos_out      host int32[capacity] or NULL: position of slot 0 of the block when pad slots
 *                      are NOT counted as positions (may be negative for a leading pad at the start).
 *   request_handle_out host, handle to pass to mepic_release_request.
 *
 * Layout rule: a prompt segment of n tokens takes ceil(n/P) private blocks with trailing pad, except
 * that the last segment of the request, if a prompt, keeps a partially filled last block; a chunk of n
 * tokens takes ceil(n/P) blocks with ceil(n/P)*P - n leading pad slots, block 0 private and blocks
 * 1.. shared by key. A chunk of at most P tokens owns no shared page and is not registered.
 *
 * Admission: the demand is the private blocks plus the shared blocks of chunks not resident. If it
 * exceeds the free pages plus the pages of zero-reference chunks this request does not itself use,
 * MEPIC_ERR_NOMEM is returned and the pool is unchanged. Otherwise zero-reference chunks are evicted
 * whole, least recently used first, only as far as needed (§3.2.3 eviction policy).
 *
 * Errors: MEPIC_ERR_INVALID (null pointers, zero-length segment, bad kind, key reused with another
 * length), MEPIC_ERR_CAPACITY (capacity < n_blocks; pool unchanged), MEPIC_ERR_NOMEM.
 */
int mepic_align_request(mepic_pool* pool, const mepic_segment* segs, uint32_t n_segs,
                        uint32_t extra_tail_tokens, int32_t* block_table_out, uint32_t capacity,
                        uint8_t* block_kind_out, uint32_t* block_valid_out, int32_t* block_pos_out,
                        uint64_t* request_handle_out, mepic_align_info* info_out);

/* Drop a request (§3.2.3, reference counts of the shared block pool): its private pages return to the free
 * list, each chunk occurrence gives back one reference; chunks that reach zero stay resident, as candidates of
 * the lazy eviction, until admission needs their pages. MEPIC_ERR_INVALID for an unknown handle. */
int mepic_release_request(mepic_pool* pool, uint64_t request_handle);

/* Page accounting (the HBM-usage metric of §4.1 and the comparison of §4.3 / §4.4 in pages): what the sharing
 * pool holds now and at its peak, next to what a layout in which every request owns all of its blocks would
 * hold. MEPIC_ERR_INVALID for null pointers. */
int mepic_pool_get_stats(const mepic_pool* pool, mepic_pool_stats* out);

/* Is the chunk resident, and with how many references? Returns MEPIC_OK and writes 0/1 to
 * *resident_out (and the count to *refcount_out if not NULL). (Chunk Matcher lookup, §3.2.2.) */
int mepic_pool_lookup_chunk(const mepic_pool* pool, uint64_t chunk_key, int* resident_out,
                            uint32_t* refcount_out);

/* ------------------------------------------------------------------------------------------------
 * Fused-RoPE paged attention (§3.3.3): K is stored WITHOUT positional encoding; the kernels gather
 * pages through the block table, rotate K and Q at the request's own absolute positions on chip and
 * run online-softmax attention. V is never rotated.
 *
 * Rotary convention (the paper prints no formula): frequency f_i = theta^(-2i/D), i in [0, D/2);
 * angle a = position * f_i; pair (x[i], x[i+D/2]) -> (x[i] cos a - x[i+D/2] sin a,
 * x[i+D/2] cos a + x[i] sin a). With MEPIC_FLAG_ROPE_INTERLEAVED the pair is (x[2i], x[2i+1]).
 *
 * Page layout (a choice of this library; the paper fixes none). Let E = bytes per KV element and
 * X = 16 / E elements (one 16-byte granule: 4 fp32, 8 bf16, 16 fp8). For page p and KV head h:
 *   K: element (slot s, dim d) at  k_pages[(((p*Hkv + h)*(D/X) + d/X)*P + s)*X + d%X]
 *      i.e. [num_pages][Hkv][D/X][P][X] — for a fixed granule the P slots are contiguous;
 *   V: element (slot s, dim d) at  v_pages[((p*Hkv + h)*D + d)*P + s]
 *      i.e. [num_pages][Hkv][D][P] — for a fixed dim the P slots are contiguous.
 * Both make every matrix-core operand a single aligned 16-byte load straight from the page.
 *
 * Logical slot n of request b lives in block j = n / P, slot s = n % P, page block_tables[b][j]; its
 * position is block_positions[b][j] + s, or n when block_positions is NULL (the index in T_align).
 * Slot n takes part iff n < kv_lens[b], its bit in block_valid_mask is set (when given) and, for
 * prefill, position(n) <= position of the query token (causal by absolute position).
 * Query head h reads KV head h / (Hq / Hkv). If no slot takes part the output row is all zeros.
 * ---------------------------------------------------------------------------------------------- */
typedef enum { MEPIC_F32 = 0, MEPIC_BF16 = 1, MEPIC_F8E4M3 = 2 } mepic_dtype;

enum {
  MEPIC_FLAG_ROPE_INTERLEAVED = 1u, /* pair (x[2i], x[2i+1]) instead of (x[i], x[i+D/2])              */
  MEPIC_FLAG_FORCE_GENERAL = 2u,    /* run the general kernel even where a matrix-core kernel exists
                                       (for tests: both must agree with the oracle)                  */
  MEPIC_FLAG_KV_READ_ONCE = 4u      /* a hint, never a change of the result: (almost) no page is read by
                                       more than one request of this call (the pool's unique and logical
                                       page counts nearly agree). The matrix-core decode kernels then load
                                       V with the non-temporal hint: faster when every byte comes from
                                       HBM once anyway, slower when requests do share pages, whose reuse
                                       from the caches it defeats. Other kernels ignore it.            */
};

typedef struct {
  const void* q;                    /* device [n_q_tokens][Hq][D], q_dtype, UN-rotated                */
  void* out;                        /* device [n_q_tokens][Hq][D], q_dtype                            */
  const void* k_pages;              /* device, K page layout above, kv_dtype, UN-rotated              */
  const void* v_pages;              /* device, V page layout above, kv_dtype                          */
  const float* k_scales;            /* device [num_pages] fp32; required iff kv_dtype == F8E4M3:      */
  const float* v_scales;            /*   stored value = e4m3fn code * scale of its page; scales are
                                       magnitudes (amax / 448): finite and >= 0                       */
  const int32_t* block_tables;      /* device [B][max_blocks] physical page ids in [0, num_pages); an id
                                       outside that range is forced into it on the device (no fault; the
                                       result of that request is unspecified)                           */
  const int32_t* kv_lens;           /* device [B] valid KV slots per request (<= max_blocks * P)      */
  const int32_t* q_positions;       /* device [n_q_tokens] absolute position of each query token      */
  const int32_t* cu_q_lens;         /* device [B+1] prefix sums of query tokens per request; prefill
                                       only. Decode has one query token per request: n_q_tokens == B  */
  const int32_t* block_positions;   /* device [B][max_blocks] or NULL                                 */
  const uint32_t* block_valid_mask; /* device [B][max_blocks] or NULL                                 */
  int32_t B, n_q_tokens, Hq, Hkv, D, P, max_blocks, num_pages;
  int32_t max_kv_len;               /* host-known upper bound on kv_lens[] (sizes the split-K grid);
                                       <= 0 means max_blocks * P                                      */
  int32_t max_q_len;                /* prefill: host-known upper bound on query tokens per request;
                                       <= 0 means n_q_tokens                                          */
  int32_t q_dtype, kv_dtype;        /* (F32,F32) | (BF16,BF16) | (BF16,F8E4M3)                        */
  float rope_theta;
  float sm_scale;                   /* <= 0 means 1/sqrt(D)                                           */
  uint32_t flags;                   /* MEPIC_FLAG_*                                                   */
  void* workspace;                  /* device scratch (split-K partials; rotary table of the matrix-core
                                       prefill), 256-byte aligned                                       */
  size_t workspace_bytes;
  void* timing_start;               /* optional hipEvent_t pair (both or neither): recorded on the stream     */
  void* timing_stop;                /*   right before / after the call's main kernel, i.e. without the small  */
                                    /*   merge kernel that follows it in decode. A profiling aid; NULL = off.  */
} mepic_attn_params;

/* Bytes of workspace mepic_attn_decode / mepic_attn_prefill need. Read: the shape, dtype and max_* fields, the
 * flags, and WHETHER block_positions / block_valid_mask are NULL (they and the flags select the kernel, and the
 * kernels differ in what they need: split-K partials in decode, the per-position rotary table in the matrix-core
 * prefill). Query with the same flags and the same NULL-ness of those two pointers as the call will have;
 * a size queried otherwise can be too small, which the call reports as MEPIC_ERR_CAPACITY.
 * A measurement aid of the matrix-core prefill: the last 16 bytes of the size it reports receive two uint64, the
 * core clocks and the ticks of the device's constant-rate counter (s_memrealtime) that workgroup 0 of the attention
 * kernel ran for (written only if that workgroup has query tokens); their ratio tells the clock rate the kernel ran
 * at, which the device's power management lowers under load. */
int mepic_attn_workspace_size(const mepic_attn_params* params, int is_prefill, size_t* bytes_out);

/* Decode: one query token per request attends to all of the request's valid slots (§3.3.3). */
int mepic_attn_decode(const mepic_attn_params* params, void* hip_stream);

/*
 * mepic_attn_decode for callers that cannot supply (or allocate) a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid allocation. The split-K partials go to a fixed array of
 * MEPIC_NOALLOC_SCRATCH_BYTES inside the library's device image (one copy per GPU, held until the process
 * ends); params->workspace and workspace_bytes are ignored. Same kernels, same result bit for bit as
 * mepic_attn_decode with a workspace. Calls no hipMalloc / hipFree nor any allocating routine.
 * MEPIC_ERR_CAPACITY when mepic_attn_workspace_size for these shapes exceeds MEPIC_NOALLOC_SCRATCH_BYTES
 * (the decode batches of the benchmark workloads need 17-32 MB); otherwise the errors of mepic_attn_decode.
 * All calls on one GPU share that GPU's array: two such calls that overlap in time on one GPU (different
 * streams, different threads) race; calls on one stream are ordered and safe.
 */
#define MEPIC_NOALLOC_SCRATCH_BYTES (48u << 20)
int mepic_attn_decode_noalloc(const mepic_attn_params* params, void* hip_stream);

/* Prefill of question tokens: the tokens cu_q_lens[b]..cu_q_lens[b+1] of request b attend causally,
 * by absolute position, to the request's slots; their own K/V are already committed to the request's
 * private pages (§3.3.2 precedes §3.3.3). */
int mepic_attn_prefill(const mepic_attn_params* params, void* hip_stream);

/* Name of the kernel variant the last attention call on this thread dispatched to (static string;
 * "" before any call). For tests and reports. */
const char* mepic_last_kernel(void);

/*
 * Calibration of the matrix-core roofline, for benchmarks (not part of the method): launches a kernel that does
 * nothing but the bf16 matrix instruction of the prefill kernel (v_mfma_f32_32x32x16_bf16; four independent
 * accumulators per wave, two waves per SIMD, one workgroup per compute unit, `iters` rounds of four products) and
 * writes the floating-point operations it executes to *flop_out (host). The caller times it with events on the
 * stream: flop / time is the rate the device sustains on that instruction, to be read next to the nominal peak.
 * random_operands != 0: the operands are pseudo-random bf16 values instead of a few constants, so that the datapaths
 * toggle as on real data; the device then settles at a lower clock (power), i.e. this is the fairer figure.
 * sink_device: device float[4]; [0] is never written in practice, [1] and [2] receive the core clocks and the ticks
 * of the constant-rate counter (s_memrealtime) that the first wave of workgroup 0 ran for, as floats:
 * clocks / ticks x the counter's rate (mepic_device_counter_khz) is the clock rate under this load. (Of the two
 * waves of a SIMD the older one is served first, so workgroup 0's first waves run for about half the launch.)
 * Errors: MEPIC_ERR_INVALID, MEPIC_ERR_LAUNCH.
 */
int mepic_probe_mfma_bf16(int32_t iters, int32_t random_operands, float* sink_device, double* flop_out, void* hip_stream);

/*
 * Second calibration kernel, for benchmarks (not part of the method): the instruction mix of one tile of the
 * matrix-core prefill kernel as a synthetic in-order stream (per wave and tile: 32 matrix products with their A
 * operand through an LDS ring, 112 vector instructions in the staging's mix, the softmax's 32 exponentials, 32 adds
 * and 16 packs, four LDS writes, six cached global loads, one barrier; eight waves per workgroup, one workgroup per
 * compute unit, `iters` tiles), in one of three arrangements: structure 0 = phases, all waves alike; 1 = phases, two
 * groups of waves half a tile apart (the prefill kernel's arrangement); 2 = one uniform stream. The caller times the
 * launch with events: time / iters is the time per tile this mix needs in that arrangement, to be read next to the
 * prefill kernel's own time per tile.
 * buf_device: device memory of buf_bytes >= 65536 that the kernel's loads read (any content); its floats [1], [2]
 * receive the core clocks and constant-rate ticks of the first wave of workgroup 0, [0] is never written in practice.
 * Errors: MEPIC_ERR_INVALID (structure not 0..2, iters < 0, NULL, buffer too small), MEPIC_ERR_LAUNCH.
 */
int mepic_probe_tile_stream(int32_t structure, int32_t iters, float* buf_device, size_t buf_bytes, void* hip_stream);

/* Rate, in kHz, of the device's constant-rate counter (the one s_memrealtime reads; hipDeviceAttributeWallClockRate
 * of the current device): what turns the tick counts above into seconds. Errors: MEPIC_ERR_INVALID (NULL),
 * MEPIC_ERR_LAUNCH (the runtime's query failed). */
int mepic_device_counter_khz(int32_t* khz_out);

/*
 * Self-test of one building block, for the test suite (a guard against toolchain changes, not part of the method):
 * the bf16 decode kernel rotates K (§3.3.3) with two-term dot-product instructions issued as a hand-written block
 * whose hazard rules the compiler does not see. This call runs that block alone. words_device: device uint32
 * [n][12] = four words (low element, high element) of rotary pairs as packed bf16, then for each of the four the
 * constant words (cos, -sin) and (sin, cos) as packed bf16; out_device: device float [n][8] = the four rotated low
 * elements, then the four rotated high elements, in fp32. Errors: MEPIC_ERR_INVALID, MEPIC_ERR_LAUNCH.
 */
int mepic_selftest_dot_rotation(const uint32_t* words_device, float* out_device, int32_t n, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Commit to paged KV (§3.3.2): the K and V vectors just computed for new tokens (prompt tokens, the
 * recomputed first block of a cached chunk, a newly seen chunk, the token a decode step produced) are
 * written straight into the pages the aligner assigned, WITHOUT positional encoding, in the page layout
 * above. The token-to-page mapping is the block table itself; nothing else is translated.
 *
 * New tokens arrive packed, [n_tokens][Hkv][D], as a list of runs: run r holds the tokens
 * cu_run_tokens[r] .. cu_run_tokens[r+1]-1, which occupy the consecutive logical slots
 * run_first_slot[r], run_first_slot[r]+1, ... of request run_request[r] (logical slot n -> page
 * block_tables[request][n / P], slot n % P). A decode step is B runs of one token. Slots no run names
 * keep their contents. Two runs (in one call, or in calls that overlap on the GPU) that name the same
 * slot race.
 *
 * dtypes: (src F32 -> pages F32), (BF16 -> BF16): a copy; (BF16 -> F8E4M3): quantised with the
 * destination page's scale, which the caller supplies (the paper names no low-precision format):
 * code = e4m3fn value nearest to fp32(x) / scale (one fp32 division), ties to even, magnitudes beyond
 * 448 saturate, the sign is kept. Scales are read, never written.
 *
 * A token whose request index, block index or page id is out of range is skipped (nothing is written
 * for it); the host checks only shapes and null pointers. Asynchronous on the stream; allocates
 * nothing; needs no workspace.
 * Errors: MEPIC_ERR_INVALID (null pointers, negative sizes, one timing event without the other),
 * MEPIC_ERR_UNSUPPORTED (dtype pair, D not 64/128, P not 16/32), MEPIC_ERR_LAUNCH.
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  const void* k_new;               /* device [n_tokens][Hkv][D], src_dtype, UN-rotated                */
  const void* v_new;               /* device [n_tokens][Hkv][D], src_dtype                            */
  void* k_pages;                   /* device, K page layout, kv_dtype (written)                       */
  void* v_pages;                   /* device, V page layout, kv_dtype (written)                       */
  const float* k_scales;           /* device [num_pages] fp32 > 0; required iff kv_dtype == F8E4M3    */
  const float* v_scales;
  const int32_t* block_tables;     /* device [B][max_blocks]                                          */
  const int32_t* run_request;      /* device [n_runs] request index of each run, in [0, B)            */
  const int32_t* run_first_slot;   /* device [n_runs] logical slot of the run's first token           */
  const int32_t* cu_run_tokens;    /* device [n_runs+1] prefix sums of tokens per run; [0] = 0 and
                                      [n_runs] = n_tokens                                             */
  int32_t B, n_runs, n_tokens, Hkv, D, P, max_blocks, num_pages;
  int32_t src_dtype, kv_dtype;     /* (F32,F32) | (BF16,BF16) | (BF16,F8E4M3)                         */
  void* timing_start;              /* optional hipEvent_t pair around the kernel, as for attention    */
  void* timing_stop;
} mepic_commit_params;

int mepic_kv_commit(const mepic_commit_params* params, void* hip_stream);

/* ------------------------------------------------------------------------------------------------
 * Batched decode over shared pages. The paper's related-work discussion (§6, operator-level acceleration)
 * names shared-KV attention kernels as the complement of MEPIC: the chunk pages that many requests alias
 * are then read (and, here, rotated) once for several requests instead of once per request. This pair of
 * calls does that for the matrix-core decode kernels: a host planner groups the 32-slot steps of
 * different requests that read exactly the same pages (and lie wholly below their request's kv_len) into
 * runs served by one pass for up to 16 / (Hq/Hkv) requests; the kernel walks the runs. Results are those
 * of mepic_attn_decode (same oracle, same tolerance); only the order of summation differs.
 *
 * mepic_decode_plan_build reads HOST copies of the block tables and kv_lens (the aligner wrote them to
 * host memory in the first place) and writes the plan, a buffer of int32 words whose layout is private to
 * the library, to host memory; the caller copies its first info.n_int32 words to the device and passes
 * that pointer to mepic_attn_decode_batched together with the info struct. A plan is valid for exactly the
 * block tables, kv_lens, head counts and dtype it was built from, on the device that was current when it
 * was built (it is cut for that device's number of waves: MEPIC_ERR_INVALID on another). In a decode loop
 * that is one plan per decode step, shared by the attention calls of all layers, whose block tables are
 * the same. Supported: (bf16 pages, P = 16) and (fp8 pages, P = 32), D = 128, Hq/Hkv <= 16, no
 * block_positions / block_valid_mask / interleaved pairing; otherwise MEPIC_ERR_UNSUPPORTED.
 * Errors: MEPIC_ERR_INVALID (null pointers, kv_len beyond the table), MEPIC_ERR_CAPACITY (plan buffer or
 * workspace too small; mepic_decode_plan_capacity gives the worst case for the plan).
 * ---------------------------------------------------------------------------------------------- */
typedef struct {
  int32_t n_runs;          /* runs in the plan                                                        */
  int32_t total_steps;     /* 32-slot steps the kernel executes per KV head                           */
  int32_t steps_unbatched; /* steps per KV head without batching (sum over requests)                  */
  int32_t n_waves;         /* waves per KV head the plan cuts the work for (fixed by the device)      */
  int32_t n_splits;        /* partial results per (request, head) the workspace must hold             */
  int32_t r_cap;           /* requests per run at most: 16 / (Hq/Hkv)                                 */
  int32_t n_int32;         /* words of the plan buffer in use                                         */
  int32_t B;
} mepic_decode_plan_info;

int mepic_decode_plan_capacity(int32_t B, int32_t max_blocks, int32_t P, size_t* n_int32_out);

int mepic_decode_plan_build(const int32_t* block_tables_host, const int32_t* kv_lens_host, int32_t B,
                            int32_t max_blocks, int32_t P, int32_t Hq, int32_t Hkv, int32_t kv_dtype,
                            int32_t* plan_out_host, size_t capacity_int32, mepic_decode_plan_info* info_out);

/*
 * The same planner, planning ahead so that one plan serves several decode steps: every request is planned as if
 * it were `horizon_tokens` longer. The steps it will grow into are in the plan as steps of its own, masked in the
 * kernel against the kv_lens of the call, so the plan stays valid for any call with
 *     kv_lens_host[b] <= kv_lens[b] <= kv_lens_host[b] + horizon_tokens   for every request b
 * and the block tables it was built from. Those tables must therefore already hold the pages of the slots ahead
 * (align the request with extra_tail_tokens >= horizon_tokens), and max_blocks * P must cover them (lengths are
 * planned up to that bound only). In a decode loop this is one plan per horizon_tokens decode steps, shared by all
 * layers; horizon_tokens = 0 is mepic_decode_plan_build. Errors as there; horizon_tokens < 0 is MEPIC_ERR_INVALID.
 */
int mepic_decode_plan_build_ahead(const int32_t* block_tables_host, const int32_t* kv_lens_host, int32_t B,
                                  int32_t max_blocks, int32_t P, int32_t Hq, int32_t Hkv, int32_t kv_dtype,
                                  int32_t horizon_tokens, int32_t* plan_out_host, size_t capacity_int32,
                                  mepic_decode_plan_info* info_out);

/* Workspace bytes mepic_attn_decode_batched needs for this plan. */
int mepic_attn_decode_batched_workspace_size(const mepic_attn_params* params, const mepic_decode_plan_info* info,
                                             size_t* bytes_out);

/* Decode as mepic_attn_decode, walking the runs of `plan_device` (device copy of the planner's output). */
int mepic_attn_decode_batched(const mepic_attn_params* params, const int32_t* plan_device,
                              const mepic_decode_plan_info* info, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MEPIC_H */
