// Index arithmetic of the prefill kernels' work queue (internal; plain integer functions for host and device: the
// host-compiled check of tests/sanitize/fs_index_check.cpp runs them over whole queues with every result asserted).
#pragma once

#include <cstdint>

#include "fs_attention.h"

namespace fs {

// Which item ticket `ticket` of pool `pool` stands for.  The item list is cut into chunks of 2^shift consecutive
// items, chunk k belongs to XCD k % 8, and the 8 pools of an XCD (pool = 8 s + xcd) take that XCD's items s, s + 8,
// ... in order.  Growing in the ticket for every pool, and every item belongs to exactly one (pool, ticket).
__device__ __host__ inline uint32_t pool_item(uint32_t pool, uint32_t ticket, uint32_t shift) {
  const uint32_t xcd = pool & 7, u = (pool >> 3) + 8 * ticket;  // u: index among the XCD's items
  return ((((u >> shift) << 3) + xcd) << shift) + (u & ((1u << shift) - 1));
}

// item -> (sequence, KV head, tile): sequence-major, then head, tiles of a head longest first.
// tf: [n_seq + 1] first query tile of each sequence; H: KV heads.  False for an item outside every sequence.
__device__ __host__ inline bool decode_item(const uint32_t* tf, int n_seq, uint32_t item, uint32_t H, int& seq, int& head,
                                            int& qt) {
  int lo = 0, hi = n_seq - 1;
  while (lo < hi) {  // last sequence whose first item is <= item
    const int mid = (lo + hi + 1) >> 1;
    if (tf[mid] * H <= item) lo = mid;
    else hi = mid - 1;
  }
  const uint32_t nt = tf[lo + 1] - tf[lo];
  if (nt == 0) return false;  // (cannot happen: an item lies in a sequence that has tiles)
  const uint32_t li = item - tf[lo] * H;
  seq = lo;
  head = (int)(li / nt);
  qt = (int)(nt - 1 - li % nt);
  return true;
}

// Runs of 8 token slots streamed per refill of a wave's block-address table (a multiple of 4, about 500 blocks),
// and the table's entries: the blocks such a segment can touch.
__device__ __host__ inline int32_t prefill_seg_runs(int R) {
  const int64_t want = (int64_t)500 * R / 4 * 4;
  return (int32_t)(want < 4 ? 4 : (want > 1024 ? 1024 : want));
}
__device__ __host__ inline int32_t prefill_table_entries(int seg_runs, int R) { return seg_runs / R + 4; }

}  // namespace fs
