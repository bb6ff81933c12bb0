/*
 * fineserve.h -- C ABI of the KV-slab decode-attention library for AMD MI355X (gfx950).
 *
 * The library implements the data-parallel hot path implied by FineServe's KV Slab
 * (arXiv 2509.06261, Sec. 5): one pre-allocated shared KV tensor per GPU, carved into
 * fixed-byte slabs; every co-located model formats slabs into blocks of its own token
 * layout (Sec. 3.2: block size = TokensPerBlock x TokenSize + Quant.Params) and indexes
 * them through its own logical block table (Sec. 5.1 view mapping, Sec. 5.2 block-id
 * equation).  On top of that pool it runs the decode-phase attention read that Sec. 2.1
 * names as the memory-bound bottleneck, for KV stored as FP16, FP8-E4M3, INT8 or packed
 * INT4 (the KV formats of Sec. 2.2).
 *
 * Conventions
 *  - Every function returns FS_OK (0) or a negative fs_status; nothing throws or aborts.
 *    fs_last_error() gives a thread-local text for the last failure.
 *  - Arguments are validated on the host before any kernel is launched.  What lives in device memory (sequence
 *    lengths, block tables, chunk offsets) is range-checked by the kernels themselves: out-of-range values are
 *    clamped into the buffers and the pool and reported through fs_decode_status.
 *  - "device pointer" = HIP device memory of the current device; "host pointer" = ordinary
 *    process memory.  The library never frees caller memory.
 *  - Device calls are asynchronous on the given hipStream_t (passed as void*; NULL = the
 *    default stream).  The caller keeps every buffer alive until the stream has passed the call.
 *  - A pool is driven by one host thread at a time (one slab manager per GPU, Sec. 4).
 */
#ifndef FINESERVE_H_
#define FINESERVE_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fs_pool fs_pool; /* opaque, owned by the library, released by fs_pool_destroy */
typedef int32_t fs_model_t;     /* small index, valid until fs_model_unregister */

enum fs_kv_dtype { FS_KV_FP16 = 0, FS_KV_FP8_E4M3 = 1, FS_KV_INT8 = 2, FS_KV_INT4 = 3 };
enum fs_src_dtype { FS_SRC_FP16 = 0, FS_SRC_FP32 = 1 };
enum fs_status {
  FS_OK = 0,
  FS_ERR_INVALID = -1, /* bad argument */
  FS_ERR_NOMEM = -2,   /* pool exhausted / workspace too small */
  FS_ERR_STATE = -3,   /* double free, block of another model, model still holds blocks */
  FS_ERR_DEVICE = -4   /* a HIP call failed; see fs_last_error() */
};
enum fs_slab_state { FS_SLAB_FREE = 0, FS_SLAB_PARTIAL = 1, FS_SLAB_FULL = 2 };

/* Block layout of one model (all sizes in bytes).  A block holds tokens_per_block tokens of
 * every layer: layers consecutive, inside a layer the KV heads consecutive, inside a head
 * chunk  K tile | V tile | K params | V params,  a tile row being one token's head_dim
 * elements (INT4: element 2j in the low nibble of byte j).  Params per token: INT8 one fp16
 * scale; INT4 fp16 scale then fp16 zero-point; FP16/FP8 none.  (Sec. 3.2 fixes only the two
 * size equations; this byte layout is the library's own.) */
typedef struct {
  int32_t kv_dtype, n_kv_heads, head_dim, n_layers;
  int32_t tokens_per_block, param_bytes;
  int32_t blocks_per_slab, reserved;
  uint64_t block_budget; /* bytes reserved per block; block b starts at b * block_budget */
  uint64_t row_bytes, kv_tile, par_tile, head_chunk, layer_bytes, block_bytes;
} fs_geometry_t;

typedef struct {
  int64_t n_slabs, slabs_free, slabs_partial, slabs_full;
  int64_t live_blocks;   /* over all models */
  int64_t n_models;
  uint64_t stranded_bytes; /* bytes of live blocks not covered by their layout (budget - block_bytes) */
} fs_pool_stats_t;

/* ---- Pool (Sec. 5.1: one pre-allocated shared KV tensor per GPU, uniform slabs) -------------
 * slab_bytes: multiple of 256.  pool_bytes: multiple of slab_bytes, pool_bytes/slab_bytes < 2^31.
 * device_base: device pointer to pool_bytes bytes, 256-byte aligned, owned by the caller and
 * outliving the pool; or NULL, in which case the library allocates (and later frees) the memory.
 * The memory is not cleared.  *out receives the pool. */
int fs_pool_create(uint64_t slab_bytes, uint64_t pool_bytes, void* device_base, fs_pool** out);
int fs_pool_destroy(fs_pool* pool);
/* Device address of the pool's first byte (for tests that inspect slab bytes). */
void* fs_pool_base(fs_pool* pool);

/* ---- Models (Sec. 3.2 equations, inverted: the block byte budget is fixed, tokens derived) --
 * Registers a model whose blocks take one whole slab each (fs_model_register) or
 * block_budget_bytes each (fs_model_register_ex; must divide slab_bytes and be a multiple of
 * 256), and returns tokens_per_block (> 0) or a negative fs_status.  n_kv_heads is the per-GPU
 * (post tensor-parallel) count, as in the token-size equation.  head_dim must be a power of
 * two between 8 and 512.  *out receives the model index.  At most 64 models per pool. */
int fs_model_register(fs_pool* pool, int kv_dtype, int n_kv_heads, int head_dim, int n_layers, fs_model_t* out);
int fs_model_register_ex(fs_pool* pool, int kv_dtype, int n_kv_heads, int head_dim, int n_layers,
                         uint64_t block_budget_bytes, fs_model_t* out);
/* The paper's own direction of the same equations (Sec. 3.2: block size = TokensPerBlock x TokenSize +
 * Quant.Params; Sec. 5.2: all slabs of a GPU have one size, a multiple of the least common multiple of the
 * co-located models' block sizes, and a slab holds slab/block blocks of its key).  Host only.
 *   fs_block_bytes: bytes of the laid-out block that holds tokens_per_block tokens (a multiple of 256); 0 for
 *     an unsupported shape or tokens_per_block < 1.
 *   fs_slab_bytes_for_blocks: the smallest multiple of lcm(block_bytes[0..n-1]) that is >= min_slab_bytes; 0 if
 *     an entry is 0 or the result would exceed 2^40 (host pointer to n values).
 *   fs_model_register_tokens: registers a model whose blocks hold exactly tokens_per_block tokens (block budget =
 *     fs_block_bytes of it, which must divide the pool's slab_bytes); returns tokens_per_block or a negative
 *     fs_status, like fs_model_register_ex. */
uint64_t fs_block_bytes(int kv_dtype, int n_kv_heads, int head_dim, int n_layers, int tokens_per_block);
uint64_t fs_slab_bytes_for_blocks(const uint64_t* block_bytes, int n, uint64_t min_slab_bytes);
int fs_model_register_tokens(fs_pool* pool, int kv_dtype, int n_kv_heads, int head_dim, int n_layers,
                             int tokens_per_block, fs_model_t* out);
/* FP8 models: static fp32 scales per (layer, KV head), separate for K and V; host pointers to
 * [n_layers][n_kv_heads] floats, all > 0.  Copied to the device synchronously.  Must be called
 * before the first append/attention of an FP8 model. */
int fs_model_set_fp8_scales(fs_pool* pool, fs_model_t model, const float* k_scale, const float* v_scale);
int fs_model_unregister(fs_pool* pool, fs_model_t model); /* FS_ERR_STATE while it holds blocks */
int fs_model_geometry(fs_pool* pool, fs_model_t model, fs_geometry_t* out);

/* ---- Slab bookkeeping (Sec. 5.2), host only: no device work and no driver calls ------------
 * fs_block_alloc: takes a free block of a PARTIAL slab keyed to this model (lowest slab id,
 * lowest local id), else carves the most recently freed FREE slab (initially slab 0, 1, 2, ...);
 * returns Blk ID = slab ID x blocks_per_slab + local block ID.  FS_ERR_NOMEM leaves the pool
 * unchanged.  fs_block_free: FS_ERR_STATE for a block that is not live or not this model's;
 * a slab whose last block is freed returns to the shared tensor as FREE. */
int fs_block_alloc(fs_pool* pool, fs_model_t model, int32_t* blk_id_out);
int fs_block_free(fs_pool* pool, fs_model_t model, int32_t blk_id);
/* The blocks of a whole sequence (or prefill chunk) in one call, host pointers: fs_blocks_alloc writes the n ids that
 * n successive fs_block_alloc calls would return, in that order, or returns FS_ERR_NOMEM and takes none if fewer
 * than n are left for this model (its PARTIAL slabs' free blocks plus the FREE slabs).  fs_blocks_free frees ids[0],
 * ids[1], ... like successive fs_block_free calls and stops at the first one that fails (its error is returned, the
 * ids before it stay freed).  n == 0 is a no-op. */
int fs_blocks_alloc(fs_pool* pool, fs_model_t model, int32_t n, int32_t* blk_ids_out);
int fs_blocks_free(fs_pool* pool, fs_model_t model, const int32_t* blk_ids, int32_t n);
int fs_pool_stats(fs_pool* pool, fs_pool_stats_t* out);
/* Per-key view of the slab table (Sec. 5.2 keys every slab by the block size -- here the model -- it is formatted
 * for): the slabs this model holds, its live blocks, the free blocks left in its PARTIAL slabs (what the next
 * allocations of this key take before a FREE slab is carved), and its share of the pool's bytes. */
typedef struct {
  int64_t slabs_partial, slabs_full;
  int64_t live_blocks;
  int64_t free_blocks_in_partial_slabs;
  uint64_t live_bytes;     /* live_blocks * block_budget */
  uint64_t stranded_bytes; /* live_blocks * (block_budget - block_bytes) */
} fs_model_stats_t;
int fs_model_stats(fs_pool* pool, fs_model_t model, fs_model_stats_t* out);
/* Copies the slab table for bit-exact comparison: state/key(model or -1)/used per slab
 * ([n_slabs] each) and the free stack bottom-to-top ([n_slabs] capacity, *n_free entries). */
int fs_pool_dump(fs_pool* pool, int32_t* slab_state, int32_t* slab_key, int32_t* slab_used, int32_t* free_stack,
                 int64_t* n_free);
/* Occupancy of every block id of a model: live[n_slabs * blocks_per_slab] bytes, 0 or 1. */
int fs_model_dump_live(fs_pool* pool, fs_model_t model, uint8_t* live);

/* ---- fs_kv_append (Sec. 2.1: every new token appends its keys and values) -------------------
 * Quantizes the new K/V rows of n_tokens tokens of one layer and scatters them, with their
 * per-token parameters, into the slab blocks named by the block tables.
 *   k_new, v_new : device, [n_tokens][n_kv_heads][head_dim], fp16 or fp32 (src_dtype), 16-byte aligned
 *   seq_idx, pos : device int32 [n_tokens]; token i is position pos[i] of sequence seq_idx[i]
 *   block_tables : device int32 [n_seq][max_blocks]; entry [s][p / tokens_per_block] is the Blk ID
 * Quantizers (fp32, round-to-nearest-even, true division; finite inputs):
 *   FP16: nearest fp16.   FP8: nearest E4M3 of x / scale[layer][head], saturating at +-448.
 *   INT8: s = fp16(amax/127) per (token, head) (1 if that is 0), q = clamp(rne(x/s), -127, 127).
 *   INT4: lo = min(x, 0), hi = max(x, 0) over the row, s = fp16((hi-lo)/15) (1 if 0),
 *         z = clamp(rne(-lo/s), 0, 15), q = clamp(rne(x/s) + z, 0, 15); z stored as fp16.
 * Two tokens of one call must not name the same (sequence, position). */
int fs_kv_append(fs_pool* pool, fs_model_t model, int layer, const void* k_new, const void* v_new, int src_dtype,
                 const int32_t* seq_idx, const int32_t* pos, const int32_t* block_tables, int max_blocks,
                 int64_t n_tokens, void* stream);

/* The newest tokens of several models (Sec. 4: the co-located models decode side by side) in ONE launch: each entry
 * is one fs_kv_append call's arguments (host array of 1..8 entries; pointers inside are device pointers). */
typedef struct {
  fs_model_t model;
  int32_t layer;
  int32_t src_dtype;  /* fs_src_dtype */
  int32_t max_blocks;
  const void* k_new;
  const void* v_new;
  const int32_t* seq_idx;
  const int32_t* pos;
  const int32_t* block_tables;
  int64_t n_tokens;
} fs_append_t;
int fs_kv_append_multi(fs_pool* pool, const fs_append_t* appends, int n_appends, void* stream);

/* ---- Decode attention (Sec. 2.1 / 2.3: one query per sequence reads all its cached tokens
 * through the block table as if the KV were contiguous) ---------------------------------------
 * For sequence b (length n_b >= 1), query head h, KV head g = h / (n_q_heads / n_kv_heads):
 *   s_t = sm_scale * <q[b][h], K^[b][t][g]>,  p = softmax_t(s),  out[b][h] = sum_t p_t V^[b][t][g]
 * with K^, V^ the dequantized cache.  Long sequences are split along t over several
 * workgroups (split-K) and merged.
 *   q, out       : device fp16 [n_seq][n_q_heads][head_dim]
 *   block_tables : device int32 [n_seq][max_blocks]
 *   seq_lens     : device int32 [n_seq], 1 <= n_b <= max_blocks * tokens_per_block
 *   seq_lens_host: optional host copy of seq_lens, used only to size the workspace tightly
 *   lse          : optional device fp32 [n_seq][n_q_heads], receives max_t s_t + ln sum_t e^(s_t - max)
 * n_q_heads must be a multiple of n_kv_heads with ratio <= 16; q and out must be 16-byte aligned. */
typedef struct {
  fs_model_t model;
  int32_t layer;
  int32_t n_q_heads;
  float sm_scale;
  const void* q;
  const int32_t* block_tables;
  const int32_t* seq_lens;
  const int32_t* seq_lens_host;
  int32_t n_seq;
  int32_t max_blocks;
  void* out;
  float* lse;
} fs_batch_t;

/* Bytes of device workspace fs_decode_attention[_multi] needs for these batches (0 on invalid
 * arguments).  Without seq_lens_host the bound max_blocks * tokens_per_block is assumed for
 * every sequence. */
uint64_t fs_decode_workspace_bytes(fs_pool* pool, const fs_batch_t* batches, int n_batches);

/* One model's batch.  workspace: device memory of at least fs_decode_workspace_bytes bytes,
 * 256-byte aligned, private to this call until the stream has passed it. */
int fs_decode_attention(fs_pool* pool, fs_model_t model, int layer, int n_q_heads, float sm_scale, const void* q,
                        const int32_t* block_tables, const int32_t* seq_lens, int n_seq, int max_blocks, void* out,
                        float* lse, void* workspace, uint64_t workspace_bytes, void* stream);

/* Several models' batches (host array, at most 8) in one launch over one work queue. */
int fs_decode_attention_multi(fs_pool* pool, const fs_batch_t* batches, int n_batches, void* workspace,
                              uint64_t workspace_bytes, void* stream);

/* One decode step of one layer for all co-located models (Sec. 2.1: append the newest token's K/V, then attend over
 * the whole cache): fs_kv_append_multi(appends) followed by fs_decode_attention_multi(batches), in three launches
 * instead of n_appends + 3 -- the appends and the decode launch's work-list preparation do not depend on each other
 * and run in one kernel.  n_appends may be 0 (then `appends` may be NULL).  Arguments, workspace and status as for
 * the two calls it stands for. */
int fs_decode_step_multi(fs_pool* pool, const fs_append_t* appends, int n_appends, const fs_batch_t* batches,
                         int n_batches, void* workspace, uint64_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid it): fs_decode_attention_multi with its workspace in a 64 MiB array that the library holds in the
 * device's memory from load until the process ends (one copy per GPU).  Calls no hipMalloc / hipFree and no
 * allocating library routine; the caller still passes inputs and outputs.  The pool's device must be the current
 * device.  FS_ERR_NOMEM if the batches need more than 64 MiB (about 30 000 work items of 192 KiB of KV each for
 * four query heads per KV head: use fs_decode_attention_multi then), decided on the host before any launch.
 *   status_out: optional device uint32; receives the launch's fs_decode_status word (by a 4-byte device copy
 *   on `stream` behind the kernels).
 * Every call on one GPU uses the same array: two such calls that overlap on one GPU (different streams or
 * threads) race; calls on one stream are ordered and safe. */
int fs_decode_attention_multi_static(fs_pool* pool, const fs_batch_t* batches, int n_batches, uint32_t* status_out,
                                     void* stream);

/* After the stream has passed a decode call: 0 if every sequence length and block-table entry was in
 * range and the workspace sufficed, else a bit mask (1: length out of range, clamped; 2: workspace too
 * small, affected sequences left unwritten; 4: a block-table entry inside a sequence's length named no
 * block of the pool -- it was read as block 0, so no byte outside the pool is touched, and the outputs
 * of the affected sequences are meaningless).  Synchronizes the stream. */
int fs_decode_status(const void* workspace, void* stream);

/* ---- Prefill (chunked prefill) attention: FineServe Sec. 2.1 (the prefill phase processes the prompt's tokens),
 * Sec. 4.2 (it is scheduled in chunks), over the same slab pool (Sec. 5.1).
 * Sequence b holds seq_lens[b] tokens in the pool (device int32), the last n_b = q_offsets[b+1] - q_offsets[b]
 * of which are the chunk being prefilled -- append their keys and values with fs_kv_append first.  Query row r
 * of the chunk stands at position seq_lens[b] - n_b + r and attends to the cached tokens 0 .. that position,
 * dequantized exactly as fs_decode_attention sees them.
 *   q, out:  device fp16 [n_rows][n_q_heads][head_dim], 16-byte aligned, the sequences' chunks one after the
 *            other (n_rows = q_offsets[n_seq]); lse: device fp32 [n_rows][n_q_heads] or NULL
 *   q_offsets: device int32 [n_seq + 1], starting at 0, non-decreasing; q_offsets_host: the same values in
 *            host memory (sizes the launch; the kernels read the device copy, and clamp every row index into
 *            n_rows, so a mismatch cannot make them leave the buffers)
 *   workspace: device memory of fs_prefill_workspace_bytes(n_seq) bytes, 256-byte aligned, owned by the caller,
 *            in use until the stream has passed the call.  fs_decode_status(workspace, stream) afterwards: bit 0
 *            set if a length or a chunk size was out of range (clamped), bit 2 (value 4) if a block-table entry
 *            named no block of the pool (read as block 0; the affected rows are meaningless).
 * At most 16 query heads per KV head (FS_ERR_INVALID otherwise).  head_dim 128 with at least 8 tokens per block
 * runs on the MFMA kernels; head_dim 64 and 256 on the 16-column MFMA kernel (the other variants are built for 128;
 * FS_OPT_PREFILL_COLUMN_BLOCKS is not consulted); every other shape the pool accepts on a vector-ALU kernel (one
 * workgroup per query row and KV head: correct, far slower).  A softmax scale that is not positive and finite is
 * served by the 16-column kernel as well.
 * Asynchronous on `stream`; no allocation, no host synchronisation. */
uint64_t fs_prefill_workspace_bytes(int n_seq);
int fs_prefill_attention(fs_pool* pool, fs_model_t model, int layer, int n_q_heads, float sm_scale, const void* q,
                         const int32_t* block_tables, const int32_t* seq_lens, const int32_t* q_offsets,
                         const int32_t* q_offsets_host, int n_seq, int max_blocks, void* out, float* lse,
                         void* workspace, uint64_t workspace_bytes, void* stream);

/* ---- Two-level scheduler, host side (Sec. 6): no device work ---------------------------------------------------
 * fs_sched_select_batch: Algorithm 2 (Sec. 6.3), SLO-aware adaptive batching of ONE model's waiting queue at time
 * `now`.  Every request gets the deadline arrival_time + slo.  A request that would miss it even if prefilled
 * alone right away is dropped; the others are ordered earliest deadline first (queue order among equals); while
 * the predicted prefill time of the whole tentative batch ends after the FRONT request's deadline, the longest
 * request is removed (among equally long ones the latest in deadline order); the result is cut, in deadline order,
 * to at most n_max requests and t_max prompt tokens.  The chunked-prefill latency of a set R of requests is
 * predicted as  c0 + c1 * sum_R tokens + c2 * sum_R tokens^2  seconds (the algorithm takes TTFT(R) as a profiled
 * input; this three-coefficient form -- launch cost, linear layers, attention -- is the library's reading, fitted
 * from fs_prefill_attention timings).
 *   waiting[n_waiting]: host; selected / dropped: host int32 [n_waiting] each, receive indices into `waiting`
 *   (selected in deadline order, dropped in queue order); *n_selected, *n_dropped their counts.  Requests in neither
 *   list stay queued.
 * fs_sched_place_models: Algorithm 1 (Sec. 6.2).  Models are taken in descending order of their base footprint
 * F_M (input order among equals); each goes to the GPU G that maximises
 *   score(G | M) = (1 / |G'|) * sum_{m in G'} mu_m * K_rem(G'),   K_rem(G') = capacity_G - sum_{m in G'} F_m,
 * G' = G's residents plus M (the paper's approximation of the contested-memory score; GPUs with K_rem < 0 are no
 * candidates, equal scores go to the lowest index).  placement[i] receives model i's GPU, or -1 if none fits.
 *   footprint, mu: host double [n_models] (bytes, tokens per byte); capacity: host double [n_gpus]. */
typedef struct {
  double arrival_time; /* seconds */
  int32_t prompt_tokens;
  int32_t reserved;
} fs_request_t;
typedef struct {
  double slo;        /* TTFT SLO of the model, seconds */
  double c0, c1, c2; /* latency model of a prefill batch, see above */
  int32_t n_max;     /* cap on concurrent requests */
  int32_t t_max;     /* cap on batched prompt tokens */
} fs_sched_params_t;
int fs_sched_select_batch(const fs_request_t* waiting, int n_waiting, const fs_sched_params_t* params, double now,
                          int32_t* selected, int32_t* n_selected, int32_t* dropped, int32_t* n_dropped);
int fs_sched_place_models(const double* footprint, const double* mu, int n_models, const double* capacity, int n_gpus,
                          int32_t* placement);

/* ---- Per-pool options: kernel selection and measurement aids (no process-global state; a pool is driven by one
 * host thread at a time, and so are its options).  fs_pool_set_option returns FS_ERR_INVALID for an unknown option
 * or a value outside its range; fs_pool_get_option reads the current value. */
enum fs_option {
  /* decode kernel: 0 = automatic (default: the MFMA kernel for the batches with a head_dim of 64, 128 or 256 and at
   * least 8 tokens per block, one launch sequence per head_dim, and the generic kernel, in a launch sequence of its
   * own, for the other batches of the call), 1 = the generic vector-ALU kernel for all, 2 = the MFMA kernel (a call
   * with a shape it lacks then fails with FS_ERR_INVALID before anything is enqueued) */
  FS_OPT_DECODE_KERNEL = 0,
  /* target KV bytes per split-K work item, rounded to whole 32-token tiles; 0 (default) lets every launch choose
   * sizes in four tiers: 3/8 of a wave's share of the launch's KV bytes (judged from seq_lens_host where given,
   * otherwise from max_blocks * tokens_per_block), between 64 and 768 KiB, for the sequences that hold the first
   * 70 % of a batch's bytes, then half, a quarter and an eighth of it.  Otherwise 4096 .. 2^30: every item that size.
   * fs_decode_workspace_bytes answers for the pool's current setting. */
  FS_OPT_SPLIT_BYTES = 1,
  /* non-zero: every decode call brackets its attention kernel (not the work-list and combine kernels) with HIP
   * events on the call's stream; fs_pool_last_attention_kernel_ms waits for the latest pair.  (A call served by
   * several launch sequences, one per head_dim: from the first attention kernel's start to the last one's end.) */
  FS_OPT_KERNEL_TIMING = 2,
  /* prefill kernel: 0 = automatic (default: the workgroup kernel, or the 16-column kernel for launches with fewer
   * work items than compute units), 1 / 2 / 4 = the wave-level kernels with 16 / 32 / 64 logit columns per wave,
   * 16 = the workgroup kernel */
  FS_OPT_PREFILL_COLUMN_BLOCKS = 3,
  /* waves of the workgroup kernel: 0 or 8 = 8 x 32 columns (default), 4 = 4 x 64 columns */
  FS_OPT_PREFILL_WAVES = 4,
  /* non-zero: the 4-wave workgroup kernel in its software-pipelined form (one wave interleaves the MFMAs of the next
   * sub-tile's S^T with the current sub-tile's exponentials); default 0 */
  FS_OPT_PREFILL_PIPELINED = 5,
  /* INT8 / INT4 models on the 8-wave workgroup kernel: non-zero (default) = the waves that stage K and V in LDS leave
   * dequantized fp16 operands there, (code - zero point) * scale rounded to fp16, and every wave runs the FP16 tile
   * code: 15-26 % faster; 0 = the integer codes reach the MFMAs exactly and scales and zero points are applied in
   * fp32 around them, as in decode.  Both stay inside the prefill tolerance. */
  FS_OPT_PREFILL_STAGED_DEQUANT = 6,
  /* read-only: the kernel the pool's latest fs_prefill_attention call launched:
   * column blocks | waves << 8 | staged dequantization << 16 | pipelined << 17 (0: none yet; column blocks 0 with
   * bit 18 set: the vector-ALU kernel) */
  FS_OPT_LAST_PREFILL_KERNEL = 7
};
int fs_pool_set_option(fs_pool* pool, int option, int64_t value);
int fs_pool_get_option(fs_pool* pool, int option, int64_t* value);
/* Elapsed milliseconds of the latest attention kernel timed under FS_OPT_KERNEL_TIMING (negative if none). */
float fs_pool_last_attention_kernel_ms(fs_pool* pool);

const char* fs_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FINESERVE_H_ */
