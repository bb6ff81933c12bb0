// Device-side records of the split-K paged decode-attention launch (internal).
#pragma once

#include "fs_internal.h"

namespace fs {

constexpr int kTierSteps = 3;  // size tiers 0 .. kTierSteps of the work items (see DevBatch::tier_seq)

// One model's batch as the kernels see it.
struct DevBatch {
  DevGeom g;
  const uint8_t* layer_base;  // pool base + layer * layer_bytes
  const _Float16* q;
  const int32_t* tables;
  const int32_t* seq_lens;
  _Float16* out;
  float* lse;
  const float* k_scale;  // FP8: [H] of this layer; otherwise null
  const float* v_scale;
  int32_t n_seq, max_blocks, n_q, G;
  float sm_scale;
  int32_t chunk_tokens;  // generic kernel: tokens per split-K work item of size tier 0 (multiple of 32)
  int32_t seq_first;     // index of this batch's first sequence among all batches' sequences
  int32_t part_stride;   // floats per work item in the partial buffer: G * (D + 2)
  int32_t qrow_first;    // index of this batch's first (sequence, q head) row among all batches
  // MFMA kernel: a sequence is cut into runs of 8 token slots that never cross a block (R = ceil(T / 8) runs
  // per block, the last one of a block shifted back to end at slot T - 1); a work item is chunk_runs
  // consecutive runs.  chunk_runs == 0 selects the token-based splits of the generic kernel.
  int32_t chunk_runs;    // of size tier 0; multiple of 4
  // Size tiers: the sequences of a batch are queued in index order, so the last sequences' items are the last the
  // grid works on.  Sequence i belongs to tier (i >= tier_seq[0]) + ... + (i >= tier_seq[kTierSteps - 1]), and a
  // tier's work items are half the size of the tier before: large items while there is plenty of work (less set-up
  // per byte), small ones at the end (the waves finish within one small item of each other).  tier_seq[t] = n_seq
  // where a tier is unused.
  int32_t tier_seq[kTierSteps];
  // Runs one turn of the MFMA kernel's tile ring covers (4 per tile, 1 / 2 / 2 / 3 tiles for FP16 / FP8 / INT8 /
  // INT4): the kernel works in whole turns, so items are whole turns long (their surplus tiles would be computed
  // and masked, which the formats bound by the vector ALU cannot afford on small items).
  int32_t ring_runs;
  int32_t R;
  uint32_t r_magic;      // ceil(2^32 / R): run / R == umulhi(run, r_magic) while run * R < 2^32
  uint32_t n_blocks;     // blocks of this model's size the pool holds: valid table entries are 0 .. n_blocks - 1
};

// Workspace header words (uint32 unless noted).
enum : int {
  kHdrCounter = 0,     // generic kernel: work-queue ticket counter
  kHdrStatus = 1,      // bit 0: a sequence length was out of range; bit 1: partial buffer too small;
                       // bit 2: a block-table entry inside a sequence's length was outside the pool
  kHdrTotalItems = 2,  // number of work items
  kHdrBatchFirst = 8,  // [kMaxBatches] first work item of each batch (sequence-major numbering)
  kHdrPartOff = 32,    // [kMaxBatches] uint64: float offset of each batch's partials (word index of a uint64 array)
  kHdrPools = 64       // [kPools] ticket counters of the MFMA kernel's end-of-launch pools, kPoolStride words apart
};
constexpr int kPools = 64;
constexpr int kDecodePools = 64;  // the decode kernel's share of them (prefill uses all, eight per XCD)
static_assert(kDecodePools <= kPools, "the header holds kPools counters");
constexpr int kPoolStride = 16;  // one counter per 64 bytes: neighbours never share a cache line
constexpr uint32_t kHeaderBytes = 256 + kPools * kPoolStride * 4;

// Block id of a block-table entry.  The tables live in device memory and cannot be validated on the host: an entry
// outside the pool (a stale or -1 entry inside a sequence's length) is replaced by block 0 -- memory of the pool,
// so nothing outside it is ever read -- and reported through bit 2 of the status word.
__device__ __forceinline__ uint32_t checked_block(int32_t entry, uint32_t n_blocks, uint32_t* header) {
  if ((uint32_t)entry < n_blocks) return (uint32_t)entry;
  atomicOr(header + kHdrStatus, 4u);
  return 0u;
}

// A work item's record in the queue, two int4 (item_list[2 i] and item_list[2 i + 1]).  First: x = batch |
// KV head << 4, y = sequence, z = split, w = the item's index within its batch in sequence-major order (sequence,
// split, KV head) -- the order of the partial records.  Second: x = the sequence's length, already clamped into
// [1, max_blocks * tokens_per_block] (so that a kernel needs no look-up of its own before it can address the
// item's blocks); y, z, w = 0.
__device__ __host__ inline int4 make_rec(int batch, int seq, int split, int head, uint32_t local) {
  return int4{batch | (head << 4), seq, split, (int)local};
}
__device__ __host__ inline int rec_batch(const int4& r) { return r.x & 15; }
__device__ __host__ inline int rec_head(const int4& r) { return r.x >> 4; }

// Timeline build (-DFS_TIMELINE, bench_timeline.py; never the product library): the MFMA decode kernel leaves clock
// readings in a block at the end of the workspace, which fs_decode_workspace_bytes then includes.  Rows of eight
// 64-bit words: kTimelineWaves rows of waves (start, end, items, XCD), then kTimelineItems rows of work items, by
// queue index (draw resolved, address table ready, last tile done, output written, wave | batch << 32 | tier << 40,
// runs | sequence << 32).  Clock: the 100 MHz constant clock.
#ifdef FS_TIMELINE
constexpr uint64_t kTimelineWaves = 4096, kTimelineItems = 1ull << 17;
constexpr uint64_t kTimelineBytes = 64 * (kTimelineWaves + kTimelineItems);
#endif

struct MultiArgs {
  DevBatch b[kMaxBatches];
  uint32_t* header;
  uint32_t* item_base;  // [n_seq_total + 1] first work item of each sequence
  int4* item_list;      // [2 * item_capacity] record of every work item (two int4 each), queue order (see make_rec)
  float* partials;
  uint64_t part_capacity;  // floats
  uint32_t item_capacity;  // entries of item_list
  // MFMA kernel: waves of the grid.  Wave w's first item is item w of the queue without a draw (its home pool is
  // w % kDecodePools, its first ticket w / kDecodePools), so the pools' counters start past those tickets.
  uint32_t n_workers;
  int32_t n_batches;
  int32_t n_seq_total;
  int32_t n_qrows_total;
  int32_t pad;
#ifdef FS_TIMELINE
  uint64_t* timeline;
#endif
};

// Work item r of a sequence with n_chunks splits and H KV heads: chunk = r / H, head = r % H, so the heads
// of one (sequence, chunk) -- which lie in the same slabs -- are neighbours.  The queue merges the batches'
// sequence-major item lists proportionally (item i of n_b in batch b sorts by i / n_b), so that at any time
// the grid works on all batches -- all KV formats -- at once: formats bound by the vector ALU and formats
// bound by memory then share every compute unit instead of taking turns.

// Workgroups (of four waves) of the MFMA decode kernel per compute unit: two, or one at head_dim 256, whose 64
// accumulator registers per lane next to a 32 KiB tile need more than the 256 registers a wave gets at two.
constexpr int mfma_wgs_per_cu(int head_dim) { return head_dim == 256 ? 1 : 2; }

// 32-token tiles the MFMA decode kernel keeps in flight per wave: about 16 KiB of K/V rows (32 KiB at head_dim
// 256, where half as many waves run).  The host sizes work items in whole turns of this ring.
constexpr int ring_tiles(int kv_dtype, int head_dim) {
  const bool f16 = kv_dtype == FS_KV_FP16, i4 = kv_dtype == FS_KV_INT4;
  return head_dim <= 64 ? (f16 ? 2 : 4) : head_dim == 128 ? (f16 ? 1 : i4 ? 3 : 2) : (f16 ? 1 : i4 ? 4 : 2);
}

// Runs of 8 token slots that a sequence of `len` tokens occupies (MFMA kernel's unit of work).
__device__ __host__ inline int n_runs(int len, int T, int R) {
  const int nblk = (len + T - 1) / T;
  const int rem = len - (nblk - 1) * T;
  return (nblk - 1) * R + ((rem + 7) >> 3);
}

__device__ __host__ inline int tier_of(const DevBatch& B, int seq) {
  int t = 0;
#pragma unroll
  for (int i = 0; i < kTierSteps; ++i) t += seq >= B.tier_seq[i];
  return t;
}
// Runs (MFMA kernel) or tokens (generic kernel) per work item of sequence `seq`.
__device__ __host__ inline int chunk_runs_of(const DevBatch& B, int seq) {
  // whole turns of the tile ring, at least one (the host makes tier 0 a multiple of 8 turns when tiers are on, and
  // ring_runs = 4, one tile, when a size is forced)
  const int cr = B.chunk_runs >> tier_of(B, seq);
  return cr < B.ring_runs ? B.ring_runs : cr - cr % B.ring_runs;
}
__device__ __host__ inline int chunk_tokens_of(const DevBatch& B, int seq) {
  const int ct = (B.chunk_tokens >> tier_of(B, seq)) & ~31;
  return ct < 32 ? 32 : ct;
}

// Splits of sequence `seq`, `len` (already clamped) tokens long.
__device__ __host__ inline int n_splits(const DevBatch& B, int seq, int len) {
  if (B.chunk_runs) {
    const int cr = chunk_runs_of(B, seq);
    return (n_runs(len, B.g.T, B.R) + cr - 1) / cr;
  }
  const int ct = chunk_tokens_of(B, seq);
  return (len + ct - 1) / ct;
}

// Place in the queue of item `local` (of n[b]) of batch b: the batches' sequence-major item lists merged
// proportionally -- item i of batch b sorts by (i / n[b], b) -- so the place is i plus the number of items of the
// other batches that sort before it: those of a batch o < b with i' / n[o] <= i / n[b], of a batch o > b with
// i' / n[o] < i / n[b].  One-to-one onto 0 .. sum(n) - 1.
__device__ __host__ inline uint64_t queue_place(uint64_t local, int b, const uint32_t (&n)[kMaxBatches]) {
  const uint64_t n_b = n[b];
  uint64_t idx = local;
#pragma unroll
  for (int o = 0; o < kMaxBatches; ++o) {
    const uint64_t n_o = n[o];
    if (o == b || n_o == 0) continue;
    const uint64_t num = local * n_o;
    const uint64_t c = o < b ? num / n_b + 1 : (num + n_b - 1) / n_b;
    idx += c < n_o ? c : n_o;
  }
  return idx;
}

// ---- The MFMA kernels' walk over a sequence (plain integer arithmetic, host and device: the host-compiled check of
// tests/sanitize/fs_index_check.cpp runs exactly these functions over whole launches with every index asserted) ----
// A sequence is walked in runs of 8 token slots that never cross a block: block k holds runs k R .. k R + R - 1
// (R = ceil(T / 8)); run r of a block covers slots 8 r .. 8 r + 7, except that the last run of a block whose T
// is no multiple of 8 is shifted back to end at slot T - 1 and its first slots, which repeat tokens of the run
// before, are masked.  A tile is 4 consecutive runs.
struct ItemCtx {
  const uint64_t* chunk_ptr;  // LDS: head-chunk address of blocks k0 .. of this item's range
  int k0;                     // first block the item touches
  int v_end;                  // one past the item's last run
  int len;                    // tokens this lane's logit column may attend to (decode: the sequence length)
  int len_u;                  // tokens the sequence holds for any column (wave-uniform); decode: == len
  int T, R;
  uint32_t r_magic;           // ceil(2^32 / R)
};

// run / R  (r_magic = ceil(2^32 / R) does not fit 32 bits for R = 1; exact while run * R < 2^32)
__device__ __host__ inline int div_runs(int vr, int R, uint32_t r_magic) {
  return R == 1 ? vr : (int)(((uint64_t)(uint32_t)vr * (uint64_t)r_magic) >> 32);
}

// Run vr of an item: its block relative to the item's first (k_rel: the index into the item's address table), its
// first slot in the block, and the slots [lo, hi) of it that hold tokens this lane's column attends to (none for a
// run past the item's end, which is mapped onto the item's last run: valid memory); [lo, hi_u): the slots that hold
// tokens of the sequence at all (what V rows and per-token parameters, which all columns share, are judged by).
struct RunGeom {
  int k_rel, start, lo, hi, hi_u;
  int tok0;  // token index of the run's slot 0 (a huge value for a run past the item's end: no column reaches it)
};

__device__ __host__ inline RunGeom run_geom(const ItemCtx& X, int vr) {
  const int vc = vr < X.v_end - 1 ? vr : X.v_end - 1;
  const int k = div_runs(vc, X.R, X.r_magic);
  const int r8 = 8 * (vc - k * X.R);
  RunGeom L;
  L.start = r8 < X.T - 8 ? r8 : X.T - 8;
  L.lo = r8 - L.start;
  L.tok0 = vr < X.v_end ? k * X.T + L.start : 0x3fffffff;
  L.hi = 8 < X.len - L.tok0 ? 8 : X.len - L.tok0;
  L.hi_u = 8 < X.len_u - L.tok0 ? 8 : X.len_u - L.tok0;
  L.k_rel = k - X.k0;
  return L;
}

// Split `chunk` of a sequence of `len` (clamped) tokens as a decode work item: its runs [v0, v1) and the blocks
// k0 .. k0 + nb - 1 they lie in.
struct ItemRange {
  int v0, v1, k0, nb;
};

__device__ __host__ inline ItemRange item_range(const DevBatch& B, int seq, int chunk, int len) {
  ItemRange r;
  const int cr = chunk_runs_of(B, seq);
  const int all = n_runs(len, B.g.T, B.R);
  r.v0 = chunk * cr;
  r.v1 = all < r.v0 + cr ? all : r.v0 + cr;
  r.k0 = div_runs(r.v0, B.R, B.r_magic);
  r.nb = div_runs(r.v1 - 1, B.R, B.r_magic) - r.k0 + 1;
  return r;
}

// The device-side records of a decode call as the launch would build them (no workspace pointers, nothing
// enqueued): for checks that replay the kernels' index arithmetic on the host.  use_mfma: which kernel would run.
int debug_plan(fs_pool* p, const fs_batch_t* batches, int n_batches, MultiArgs* out, bool* use_mfma);

// Launchers implemented in the kernel translation units.
hipError_t launch_prep(const MultiArgs& A, hipStream_t s);
hipError_t launch_generic(const MultiArgs& A, int n_workgroups, hipStream_t s);
hipError_t launch_generic_prefill(const MultiArgs& A, const int32_t* q_offsets, int n_rows, int n_workgroups, hipStream_t s);
hipError_t launch_combine(const MultiArgs& A, hipStream_t s);
bool mfma_supports(const DevBatch& b);
hipError_t launch_mfma(const MultiArgs& A, int n_workgroups, hipStream_t s);

}  // namespace fs
