// MFMA split-K paged decode-attention kernel for gfx950 (head_dim 128, all four KV formats).
//
// FineServe Sec. 2.1: the decode phase re-reads the whole KV cache for every generated token and is bound by
// memory bandwidth; Sec. 2.3 / 5.1: the cache is reached through each model's own block table over the
// shared slab pool.  The tile machinery (loads, dequantization around the MFMAs, online softmax) is in
// fs_mfma_tiles.h; this file holds the work decomposition:
//   a persistent grid of independent waves: each wave draws work items (sequence, split, KV head) from the
//   queue, streams the split's 32-token tiles with a private online-softmax state and writes the output (or
//   the split's partial record) straight from its accumulators.  No wave waits for another.
#include "fs_mfma_tiles.h"

namespace fs {
namespace {

// One work item, processed by ONE wave: all tiles of the split, then the output (or the split's partial
// record) straight from the accumulator registers.  Waves never synchronise with each other.
// s_ptr: this wave's LDS table of head-chunk addresses.
template <int DT, int GP>
__device__ void process_item(const MultiArgs& A, int b, int seq, int chunk, int head, uint32_t item, uint64_t* s_ptr) {  // item: index within the batch
  const DevBatch& B = A.b[b];
  const DevGeom& g = B.g;
  // The lane index is made opaque per item: otherwise the compiler hoists every variant's lane-dependent
  // constants out of the kernel's item loop, where they stay live across all other variants and push the
  // tile loops into spilling.
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int max_len = (int)min((int64_t)B.max_blocks * g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : (len > max_len ? max_len : len);
  const int n_chunks = n_splits(B, len);
  const int v0 = chunk * B.chunk_runs;
  const int v1 = min(n_runs(len, g.T, B.R), v0 + B.chunk_runs);

  const uint64_t* part_off = reinterpret_cast<const uint64_t*>(A.header + kHdrPartOff);
  const uint64_t part_base = part_off[b] + (uint64_t)item * (uint64_t)B.part_stride;  // item: index within the batch
  if (n_chunks > 1 && part_base + (uint64_t)B.part_stride > A.part_capacity) {  // wave-uniform
    if (lane == 0) atomicOr(A.header + kHdrStatus, 2u);
    return;
  }

  ItemCtx X;
  X.T = g.T;
  X.R = B.R;
  X.r_magic = B.r_magic;
  X.len = len;
  X.len_u = len;
  X.v_end = v1;
  X.k0 = div_runs(v0, B.R, B.r_magic);
  X.chunk_ptr = s_ptr;
  fill_table(s_ptr, B.tables + (int64_t)seq * B.max_blocks, B.layer_base + (uint64_t)head * g.head_chunk, g.block_budget, X.k0,
             div_runs(v1 - 1, B.R, B.r_magic) - X.k0 + 1, lane, B.n_blocks, A.header);

  // Q operand and per-head constants
  u32x4 qb[4];
  float qsum;
  load_q<DT>(B.q + ((int64_t)seq * B.n_q + head * G + c) * kD, c < G, j, qb, qsum);
  if constexpr (Fmt<DT>::kParBytes != 0) {
    qsum += __shfl_xor(qsum, 16, 64);
    qsum += __shfl_xor(qsum, 32, 64);
    if constexpr (GP == 4) qsum = __shfl(qsum, c & 3, 64);  // of the head this lane exponentiates
  }
  float alpha = B.sm_scale * kLog2e;
  if (DT == FS_KV_FP8_E4M3) alpha *= B.k_scale[head];

  State st;
#pragma unroll
  for (int e = 0; e < 8; ++e) st.acc[e] = float4v{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
  st.l = 0.f;
  st.zc = 0.f;

  stream_tiles<DT, GP>(X, g, v0, qb, qsum, alpha, st, j, c);

  // ---- output: per-head sums over the lanes of the head, then rows h < G straight from the accumulators ----
  if constexpr (GP == 4) {
    st.l += __shfl_xor(st.l, 4, 64);
    st.l += __shfl_xor(st.l, 8, 64);
  }
  st.l += __shfl_xor(st.l, 16, 64);
  st.l += __shfl_xor(st.l, 32, 64);
  if constexpr (Fmt<DT>::kParBytes != 0) {
    if constexpr (GP == 4) {
      st.zc += __shfl_xor(st.zc, 4, 64);
      st.zc += __shfl_xor(st.zc, 8, 64);
    }
    st.zc += __shfl_xor(st.zc, 16, 64);
    st.zc += __shfl_xor(st.zc, 32, 64);
  }
  const float v_static = DT == FS_KV_FP8_E4M3 ? B.v_scale[head] : 1.0f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int h = 4 * j + r;  // accumulator row r of this lane; its m, l, zc live in lane c = h
    const float L = __shfl(st.l, h, 64), M = __shfl(st.m, h, 64), Z = __shfl(st.zc, h, 64);
    if (h < G) {
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // integer formats: undo the 2^-24 of the subnormal encoding (and the 16 of INT4's odd code positions)
        const float f = DT == FS_KV_INT8 ? kTwo24 : (DT == FS_KV_INT4 ? ((e & 1) ? kTwo20 : kTwo24) : 1.0f);
        o[e] = st.acc[e][r] * f;
        if constexpr (Fmt<DT>::kParBytes != 0) o[e] += Z;
        o[e] *= v_static;
      }
      const int qh = head * G + h;
      if (n_chunks == 1) {
        const float inv = 1.0f / L;
        u32x4 w;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const half2v hv = {(_Float16)(o[2 * q] * inv), (_Float16)(o[2 * q + 1] * inv)};
          w[q] = h2u(hv);
        }
        *reinterpret_cast<u32x4*>(B.out + ((int64_t)seq * B.n_q + qh) * kD + 8 * c) = w;
        if (c == 0 && B.lse) B.lse[(int64_t)seq * B.n_q + qh] = (M + __builtin_amdgcn_logf(L)) * kLn2;
      } else {
        float* pr = A.partials + part_base + (uint64_t)h * (kD + 2);
#pragma unroll
        for (int e = 0; e < 8; ++e) pr[8 * c + e] = o[e];
        if (c == 0) {
          pr[kD] = M * kLn2;  // partial records keep the reference in natural-log units
          pr[kD + 1] = L;
        }
      }
    }
  }
}

template <int GP>
__device__ __forceinline__ void dispatch_dtype(const MultiArgs& A, int b, int4 rec, uint64_t* s_ptr) {
  const int head = rec_head(rec);
  const uint32_t local = (uint32_t)rec.w;  // the item's index within its batch: where its partial record goes
  switch (A.b[b].g.dtype) {
    case FS_KV_FP16: process_item<FS_KV_FP16, GP>(A, b, rec.y, rec.z, head, local, s_ptr); break;
    case FS_KV_FP8_E4M3: process_item<FS_KV_FP8_E4M3, GP>(A, b, rec.y, rec.z, head, local, s_ptr); break;
    case FS_KV_INT8: process_item<FS_KV_INT8, GP>(A, b, rec.y, rec.z, head, local, s_ptr); break;
    default: process_item<FS_KV_INT4, GP>(A, b, rec.y, rec.z, head, local, s_ptr); break;
  }
}

__device__ __forceinline__ void dispatch_item(const MultiArgs& A, uint32_t item, uint64_t* s_ptr) {
  const int4 rec = A.item_list[item];
  const int b = rec_batch(rec);
  if (A.b[b].G <= 4) dispatch_dtype<4>(A, b, rec, s_ptr);
  else dispatch_dtype<16>(A, b, rec, s_ptr);
}

__global__ __launch_bounds__(kThreads, 2) void mfma_attention_kernel(MultiArgs A, int table_entries) {
  extern __shared__ uint64_t smem64[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint64_t* s_ptr = smem64 + (size_t)wave * table_entries;
  const uint32_t total = A.header[kHdrTotalItems];
  // Every wave is its own worker and draws its items from kPools ticket counters: pool p holds the items
  // p, p + kPools, ... of the queue.  Waves that get short items, or sit on a faster compute unit, simply
  // draw more often; with a fixed deal (wave w takes items w, w + n_workers, ...) the slowest wave was
  // measured to finish a quarter later than the median one.  One counter for all items is no option: an
  // address serves an atomic every ~11 ns when idle and several times slower under streaming load, which
  // was measured to bound the kernel; kPools counters with about a thousand draws each do not.
  // A wave empties its home pool first, so every pool is emptied by its home waves whatever the others do;
  // after that it tries a few more pools and leaves.  The next ticket is drawn before the current item is
  // processed, so the atomic's latency is not waited for between items.
  const uint32_t worker = blockIdx.x * kWaves + wave;
  uint32_t pool = worker % kPools;
  uint32_t ticket = 0;
  if (lane == 0) ticket = atomicAdd(A.header + kHdrPools + pool * kPoolStride, 1u);
  for (int empty = 0;;) {
    uint32_t item = pool + kPools * __builtin_amdgcn_readfirstlane(ticket);
    while (item >= total && ++empty < 4) {  // this pool is empty: try another
      pool = (pool + 17) % kPools;
      if (lane == 0) ticket = atomicAdd(A.header + kHdrPools + pool * kPoolStride, 1u);
      item = pool + kPools * __builtin_amdgcn_readfirstlane(ticket);
    }
    if (item >= total) break;  // every wave leaves here after at most four empty pools
    if (lane == 0) ticket = atomicAdd(A.header + kHdrPools + pool * kPoolStride, 1u);
    dispatch_item(A, item, s_ptr);
  }
}

}  // namespace

// Shapes this kernel covers: head_dim 128, at least 8 tokens per block (a run of 8 slots fits a block), and
// run indices small enough for the multiply-high division by R.
bool mfma_supports(const DevBatch& b) {
  if (b.g.D != kD || b.g.T < 8 || b.G > 16) return false;
  const uint64_t max_tok = (uint64_t)b.max_blocks * (uint64_t)b.g.T;
  const uint64_t max_run = (uint64_t)b.max_blocks * (uint64_t)b.R + 8;
  return max_tok < (1ull << 31) && max_run * (uint64_t)b.R < (1ull << 32);
}

hipError_t launch_mfma(const MultiArgs& A, int n_workgroups, hipStream_t s) {
  // LDS: per wave one 8-byte address per block of the largest split (+ slack)
  int entries = 0;
  for (int i = 0; i < A.n_batches; ++i) entries = std::max(entries, A.b[i].chunk_runs / A.b[i].R + 4);
  const size_t smem = (size_t)kWaves * entries * sizeof(uint64_t);
  hipLaunchKernelGGL(mfma_attention_kernel, dim3(n_workgroups), dim3(kThreads), smem, s, A, entries);
  return hipGetLastError();
}

}  // namespace fs
