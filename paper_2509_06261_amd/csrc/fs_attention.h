// Device-side records of the split-K paged decode-attention launch (internal).
#pragma once

#include "fs_internal.h"

namespace fs {

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
  int32_t chunk_tokens;  // generic kernel: tokens per split-K work item (multiple of 32)
  int32_t seq_first;     // index of this batch's first sequence among all batches' sequences
  int32_t part_stride;   // floats per work item in the partial buffer: G * (D + 2)
  int32_t qrow_first;    // index of this batch's first (sequence, q head) row among all batches
  // MFMA kernel: a sequence is cut into runs of 8 token slots that never cross a block (R = ceil(T / 8) runs
  // per block, the last one of a block shifted back to end at slot T - 1); a work item is chunk_runs
  // consecutive runs.  chunk_runs == 0 selects the token-based splits of the generic kernel.
  int32_t chunk_runs;    // multiple of 4
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

// A work item's record in the queue: x = batch | KV head << 4, y = sequence, z = split, w = the item's index
// within its batch in sequence-major order (sequence, split, KV head) -- the order of the partial records.
__device__ __host__ inline int4 make_rec(int batch, int seq, int split, int head, uint32_t local) {
  return int4{batch | (head << 4), seq, split, (int)local};
}
__device__ __host__ inline int rec_batch(const int4& r) { return r.x & 15; }
__device__ __host__ inline int rec_head(const int4& r) { return r.x >> 4; }

struct MultiArgs {
  DevBatch b[kMaxBatches];
  uint32_t* header;
  uint32_t* item_base;  // [n_seq_total + 1] first work item of each sequence
  int4* item_list;      // [item_capacity] record of every work item, queue order (see make_rec)
  float* partials;
  uint64_t part_capacity;  // floats
  uint32_t item_capacity;  // entries of item_list
  uint32_t pad1;
  int32_t n_batches;
  int32_t n_seq_total;
  int32_t n_qrows_total;
  int32_t pad;
};

// Work item r of a sequence with n_chunks splits and H KV heads: chunk = r / H, head = r % H, so the heads
// of one (sequence, chunk) -- which lie in the same slabs -- are neighbours.  The queue merges the batches'
// sequence-major item lists proportionally (item i of n_b in batch b sorts by i / n_b), so that at any time
// the grid works on all batches -- all KV formats -- at once: formats bound by the vector ALU and formats
// bound by memory then share every compute unit instead of taking turns.

// Runs of 8 token slots that a sequence of `len` tokens occupies (MFMA kernel's unit of work).
__device__ __host__ inline int n_runs(int len, int T, int R) {
  const int nblk = (len + T - 1) / T;
  const int rem = len - (nblk - 1) * T;
  return (nblk - 1) * R + ((rem + 7) >> 3);
}

// Splits of a sequence of `len` (already clamped) tokens.
__device__ __host__ inline int n_splits(const DevBatch& B, int len) {
  if (B.chunk_runs) return (n_runs(len, B.g.T, B.R) + B.chunk_runs - 1) / B.chunk_runs;
  return (len + B.chunk_tokens - 1) / B.chunk_tokens;
}

// Launchers implemented in the kernel translation units.
hipError_t launch_prep(const MultiArgs& A, hipStream_t s);
hipError_t launch_generic(const MultiArgs& A, int n_workgroups, hipStream_t s);
hipError_t launch_generic_prefill(const MultiArgs& A, const int32_t* q_offsets, int n_rows, int n_workgroups, hipStream_t s);
hipError_t launch_combine(const MultiArgs& A, hipStream_t s);
bool mfma_supports(const DevBatch& b);
hipError_t launch_mfma(const MultiArgs& A, int n_workgroups, hipStream_t s);

}  // namespace fs
