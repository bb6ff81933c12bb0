// MFMA split-K paged decode-attention kernel for gfx950 (head_dim 64, 128 or 256, all four KV formats).
//
// FineServe Sec. 2.1: the decode phase re-reads the whole KV cache for every generated token and is bound by
// memory bandwidth; Sec. 2.3 / 5.1: the cache is reached through each model's own block table over the
// shared slab pool.  The tile machinery (loads, dequantization around the MFMAs, online softmax) is in
// fs_mfma_tiles.h; this file holds the work decomposition:
//   a persistent grid of independent waves: each wave draws work items (sequence, split, KV head) from the
//   queue, streams the split's 32-token tiles with a private online-softmax state and writes the output (or
//   the split's partial record) straight from its accumulators.  No wave waits for another.
//   An item's record carries its sequence's length, so the only look-up between a queue ticket and the item's
//   first K/V requests is the record, then the block-table entries.
#include "fs_mfma_tiles.h"

namespace fs {
namespace {

// What the wave knows about an item before its tiles stream (all wave-uniform): the record's fields, the runs
// [v0, v1) it covers and the blocks k0 .. k0 + nb - 1 they lie in.
struct ItemPlan {
  int b, seq, chunk, head, len;
  uint32_t local;  // the item's index within its batch: where its partial record goes
  int v0, v1, k0, nb;
};

// rec: lane l < 8 holds dword l of the item's record (see make_rec).
__device__ __forceinline__ ItemPlan plan_item(const MultiArgs& A, uint32_t rec) {
  ItemPlan P;
  const int x = (int)__builtin_amdgcn_readlane(rec, 0);
  P.b = x & 15;
  P.head = x >> 4;
  P.seq = (int)__builtin_amdgcn_readlane(rec, 1);
  P.chunk = (int)__builtin_amdgcn_readlane(rec, 2);
  P.local = __builtin_amdgcn_readlane(rec, 3);
  P.len = (int)__builtin_amdgcn_readlane(rec, 4);
  const ItemRange r = item_range(A.b[P.b], P.seq, P.chunk, P.len);
  P.v0 = r.v0;
  P.v1 = r.v1;
  P.k0 = r.k0;
  P.nb = r.nb;
  return P;
}

constexpr int kTabRegs = 4;  // an item touches at most 64 * kTabRegs blocks (the host caps the item size accordingly)

// The item's block-table entries: entry i goes to register i / 64 of lane i % 64.
__device__ __forceinline__ void load_entries(const MultiArgs& A, const ItemPlan& P, int lane, int32_t (&tab)[kTabRegs]) {
  const DevBatch& B = A.b[P.b];
  const int32_t* t = B.tables + (int64_t)P.seq * B.max_blocks + P.k0;
#pragma unroll
  for (int q = 0; q < kTabRegs; ++q) tab[q] = lane + 64 * q < P.nb ? t[lane + 64 * q] : 0;
}

// Head-chunk addresses of the item's blocks into this wave's LDS table (see fill_table).
__device__ __forceinline__ void store_table(const MultiArgs& A, const ItemPlan& P, int lane, const int32_t (&tab)[kTabRegs],
                                            uint64_t* s_ptr) {
  const DevBatch& B = A.b[P.b];
  const uint8_t* head_base = B.layer_base + (uint64_t)P.head * B.g.head_chunk;
#pragma unroll
  for (int q = 0; q < kTabRegs; ++q)
    if (lane + 64 * q < P.nb)
      s_ptr[lane + 64 * q] = reinterpret_cast<uint64_t>(head_base + (uint64_t)checked_block(tab[q], B.n_blocks, A.header) * B.g.block_budget);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// One work item is processed by ONE wave in two steps: stream_item runs all tiles of the split through the wave's
// private online-softmax state; finish_item writes the output (or the split's partial record) straight from the
// accumulator registers.  Waves never synchronise with each other.  (Two steps, so that the tile loops of the
// eight format / group variants do not carry the output code's registers; the state has the same shape for all.)
// s_ptr: this wave's LDS table of head-chunk addresses, already holding the item's blocks.
template <int DT, int GP, int HD>
__device__ __forceinline__ void stream_item(const MultiArgs& A, const ItemPlan& P, uint64_t* s_ptr, StateT<HD>& st) {
  const int seq = P.seq, head = P.head;
  const DevBatch& B = A.b[P.b];
  const DevGeom& g = B.g;
  // The lane index is made opaque per item: otherwise the compiler hoists every variant's lane-dependent
  // constants out of the kernel's item loop, where they stay live across all other variants and push the
  // tile loops into spilling.
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;

  ItemCtx X;
  X.T = g.T;
  X.R = B.R;
  X.r_magic = B.r_magic;
  X.len = P.len;
  X.len_u = P.len;
  X.v_end = P.v1;
  X.k0 = P.k0;
  X.chunk_ptr = s_ptr;

  // Q operand and per-head constants
  u32x4 qb[HD / 32];
  float qsum;
  load_q<DT, true, HD>(B.q + ((int64_t)seq * B.n_q + head * G + c) * HD, c < G, j, qb, qsum);
  if constexpr (Fmt<DT, HD>::kParBytes != 0) {
    qsum += __shfl_xor(qsum, 16, 64);
    qsum += __shfl_xor(qsum, 32, 64);
    if constexpr (GP == 4) qsum = __shfl(qsum, c & 3, 64);  // of the head this lane exponentiates
  }
  float alpha = B.sm_scale * kLog2e;
  if (DT == FS_KV_FP8_E4M3) alpha *= B.k_scale[head];

#pragma unroll
  for (int e = 0; e < HD / 16; ++e) st.acc[e] = float4v{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
  st.l = 0.f;
  st.zc = 0.f;

  stream_tiles<DT, GP, HD, true>(X, g, P.v0, qb, qsum, alpha, st, j, c);
}

// part_off: the batches' offsets into the partial buffer (the workspace header's words, copied to LDS once per
// workgroup: read from memory here they would be one more round trip in front of every item's stores).
template <int DT, int GP, int HD>
__device__ __forceinline__ void finish_item(const MultiArgs& A, const ItemPlan& P, StateT<HD>& st, const uint64_t* part_off) {
  constexpr int NE = HD / 16;  // output columns NE c .. NE c + NE - 1 are this lane's
  const int b = P.b, seq = P.seq, head = P.head;
  const DevBatch& B = A.b[b];
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int n_chunks = n_splits(B, seq, P.len);
  const uint64_t part_base = part_off[b] + (uint64_t)P.local * (uint64_t)B.part_stride;  // local: index within the batch
  if (n_chunks > 1 && part_base + (uint64_t)B.part_stride > A.part_capacity) {  // wave-uniform
    // the workspace was sized for shorter sequences: reported, the item's record is not written
    if (lane == 0) atomicOr(A.header + kHdrStatus, 2u);
    return;
  }

  // ---- output: per-head sums over the lanes of the head, then rows h < G straight from the accumulators ----
  if constexpr (GP == 4) {
    st.l += __shfl_xor(st.l, 4, 64);
    st.l += __shfl_xor(st.l, 8, 64);
  }
  st.l += __shfl_xor(st.l, 16, 64);
  st.l += __shfl_xor(st.l, 32, 64);
  if constexpr (Fmt<DT, HD>::kParBytes != 0) {
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
      float o[NE];
#pragma unroll
      for (int e = 0; e < NE; ++e) {
        // integer formats: undo the 2^-24 of the subnormal encoding (and the 16 of INT4's odd code positions)
        const float f = DT == FS_KV_INT8 ? kTwo24 : (DT == FS_KV_INT4 ? ((e & 1) ? kTwo20 : kTwo24) : 1.0f);
        o[e] = st.acc[e][r] * f;
        if constexpr (Fmt<DT, HD>::kParBytes != 0) o[e] += Z;
        o[e] *= v_static;
      }
      const int qh = head * G + h;
      if (n_chunks == 1) {
        const float inv = 1.0f / L;
        uint32_t w[NE / 2];
#pragma unroll
        for (int q = 0; q < NE / 2; ++q) {
          const half2v hv = {(_Float16)(o[2 * q] * inv), (_Float16)(o[2 * q + 1] * inv)};
          w[q] = h2u(hv);
        }
        _Float16* orow = B.out + ((int64_t)seq * B.n_q + qh) * HD + NE * c;
        if constexpr (NE == 4) {
          *reinterpret_cast<u32x2*>(orow) = u32x2{w[0], w[1]};
        } else {
#pragma unroll
          for (int q = 0; q < NE / 8; ++q)
            reinterpret_cast<u32x4*>(orow)[q] = u32x4{w[4 * q], w[4 * q + 1], w[4 * q + 2], w[4 * q + 3]};
        }
        if (c == 0 && B.lse) B.lse[(int64_t)seq * B.n_q + qh] = (M + __builtin_amdgcn_logf(L)) * kLn2;
      } else {
        float* pr = A.partials + part_base + (uint64_t)h * (HD + 2);
        // (a row starts at a multiple of 8 bytes: part_stride and HD + 2 are even)
#pragma unroll
        for (int e = 0; e < NE; e += 2) *reinterpret_cast<float2*>(pr + NE * c + e) = float2{o[e], o[e + 1]};
        if (c == 0) {
          pr[HD] = M * kLn2;  // partial records keep the reference in natural-log units
          pr[HD + 1] = L;
        }
      }
    }
  }
}

// step 0: stream_item, step 1: finish_item
template <int STEP, int GP, int HD>
__device__ __forceinline__ void dispatch_dtype(const MultiArgs& A, const ItemPlan& P, uint64_t* s_ptr, StateT<HD>& st,
                                               const uint64_t* part_off) {
  switch (A.b[P.b].g.dtype) {
#define FS_STEP(DT)                                                  \
  if constexpr (STEP == 0) stream_item<DT, GP, HD>(A, P, s_ptr, st); \
  else finish_item<DT, GP, HD>(A, P, st, part_off);                  \
  break
    case FS_KV_FP16: FS_STEP(FS_KV_FP16);
    case FS_KV_FP8_E4M3: FS_STEP(FS_KV_FP8_E4M3);
    case FS_KV_INT8: FS_STEP(FS_KV_INT8);
    default: FS_STEP(FS_KV_INT4);
#undef FS_STEP
  }
}

template <int STEP, int HD>
__device__ __forceinline__ void dispatch_item(const MultiArgs& A, const ItemPlan& P, uint64_t* s_ptr, StateT<HD>& st,
                                              const uint64_t* part_off) {
  if (A.b[P.b].G <= 4) dispatch_dtype<STEP, 4, HD>(A, P, s_ptr, st, part_off);
  else dispatch_dtype<STEP, 16, HD>(A, P, s_ptr, st, part_off);
}

// One kernel per head_dim (every batch of a launch has the same one).
template <int HD>
__global__ __launch_bounds__(kThreads, mfma_wgs_per_cu(HD)) void mfma_attention_kernel(MultiArgs A, int table_entries) {
  extern __shared__ uint64_t smem64[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint64_t* s_ptr = smem64 + (size_t)wave * table_entries;
  __shared__ uint64_t s_part_off[kMaxBatches];
  if (threadIdx.x < kMaxBatches) s_part_off[threadIdx.x] = reinterpret_cast<const uint64_t*>(A.header + kHdrPartOff)[threadIdx.x];
  __syncthreads();
  const uint32_t total = A.header[kHdrTotalItems];
#ifdef FS_TIMELINE
  const uint64_t tl_start = wall_clock64();
  uint64_t tl_items = 0;
#endif
  // Every wave is its own worker and draws its items from kDecodePools ticket counters: pool p holds the items
  // p, p + kDecodePools, ... of the queue.  Waves that get short items, or sit on a faster compute unit, simply
  // draw more often; with a fixed deal (wave w takes items w, w + n_workers, ...) the slowest wave was
  // measured to finish a quarter later than the median one.  One counter for all items is no option: an
  // address serves an atomic every ~11 ns when idle and several times slower under streaming load, which
  // was measured to bound the kernel (and still to cost short launches a tenth with 8 counters); 64 do not.
  // A wave takes its tickets from the pools in turn (its k-th from pool w + k), so all counters advance at
  // about the same rate and the grid as a whole walks the queue roughly front to back: the large items of the
  // queue's front are all under way before its small last items are handed out.  (With a home pool per wave that
  // was emptied before the wave looked elsewhere, the pools drifted apart and the slowest pool's large items
  // started when the others were done: waves idled 5 % of the launch at its end, against 3.5 %.)
  // Once a wave meets an empty pool the launch is in its last few per cent.  From then on the wave looks at all
  // counters at once (lane p reads pool p's) and picks the pool of a random one of the items that are left, so
  // pools that lag get helpers in proportion to what they still hold, and stays there until that pool is
  // empty too.  It leaves only when every pool is past its last item.
  // The next ticket is drawn before the current item is processed, so the atomic's latency is not waited for
  // between items; a wave's first ticket needs no draw at all (the work-list kernel starts the counters past the
  // pools' first waves), which takes one round trip off the start of every launch.
  static_assert(kDecodePools <= 64, "one pool per lane in the look at all counters");
  const uint32_t worker = blockIdx.x * kWaves + wave;
  uint32_t pool = worker % kDecodePools;
  uint32_t ticket = worker / kDecodePools;
  bool in_turn = true;                            // false once an empty pool was met
  uint32_t rng = worker * 2654435761u + 0x9e3779b9u;  // wave-uniform
  constexpr uint32_t kNone = 0xffffffffu;
  auto draw = [&]() {
    if (lane == 0) ticket = atomicAdd(A.header + kHdrPools + pool * kPoolStride, 1u);
  };
  // the item the drawn ticket stands for, or kNone once every pool is empty (then no ticket is outstanding)
  auto resolve = [&]() -> uint32_t {
    for (;;) {
      const uint32_t item = pool + kDecodePools * __builtin_amdgcn_readfirstlane(ticket);
      if (item < total) return item;
      // this pool is empty: what do the others hold?  (the counters only grow)
      in_turn = false;
      const uint32_t cnt = lane < kDecodePools ? __hip_atomic_load(A.header + kHdrPools + lane * kPoolStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0u;
      const uint32_t held = lane < kDecodePools && (uint32_t)lane < total ? (total - lane + kDecodePools - 1) / kDecodePools : 0u;
      uint32_t incl = held > cnt ? held - cnt : 0u;  // items left in pool `lane`, then their inclusive sum over the lanes
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
      }
      const uint32_t left = __builtin_amdgcn_readlane(incl, 63);
      if (left == 0) return kNone;  // every pass finds fewer items left or takes one
      rng = rng * 1664525u + 1013904223u;
      const uint32_t k = (uint32_t)(((uint64_t)rng * (uint64_t)left) >> 32);  // one of the items left, uniformly
      pool = (uint32_t)__builtin_ctzll(__ballot(incl > k));                    // the pool it lies in (wave-uniform)
      draw();
    }
  };
  auto load_rec = [&](uint32_t item) -> uint32_t {
    return lane < 8 ? reinterpret_cast<const uint32_t*>(A.item_list + 2 * (size_t)item)[lane] : 0u;
  };
  for (;;) {
    const uint32_t item = resolve();
    if (item == kNone) break;  // every wave leaves here, once all pools are empty
#ifdef FS_TIMELINE
    const uint64_t tl_begin = wall_clock64();
#endif
    if (in_turn) pool = (pool + 1) % kDecodePools;
    draw();                    // the next ticket, answered while this item streams
    const ItemPlan P = plan_item(A, load_rec(item));
    int32_t tab[kTabRegs];
    load_entries(A, P, lane, tab);
    store_table(A, P, lane, tab, s_ptr);
#ifdef FS_TIMELINE
    const uint64_t tl_table = wall_clock64();
    ++tl_items;
#endif
    StateT<HD> st;
    dispatch_item<0, HD>(A, P, s_ptr, st, s_part_off);
#ifdef FS_TIMELINE
    const uint64_t tl_tiles = wall_clock64();
#endif
    dispatch_item<1, HD>(A, P, s_ptr, st, s_part_off);
#ifdef FS_TIMELINE
    if (lane == 0 && item < kTimelineItems) {
      uint64_t* row = A.timeline + 8 * (kTimelineWaves + item);
      row[0] = tl_begin;
      row[1] = tl_table;
      row[2] = tl_tiles;
      row[3] = wall_clock64();
      row[4] = (uint64_t)(blockIdx.x * kWaves + wave) | ((uint64_t)P.b << 32) | ((uint64_t)tier_of(A.b[P.b], P.seq) << 40);
      row[5] = (uint64_t)(P.v1 - P.v0) | ((uint64_t)P.seq << 32);
    }
#endif
  }
#ifdef FS_TIMELINE
  if (lane == 0 && blockIdx.x * kWaves + wave < kTimelineWaves) {
    uint64_t* row = A.timeline + 8 * (blockIdx.x * kWaves + wave);
    row[0] = tl_start;
    row[1] = wall_clock64();
    row[2] = tl_items;
    row[3] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7;  // hwreg(HW_REG_XCC_ID, 0, 4)
  }
#endif
}

}  // namespace

// Shapes this kernel covers: head_dim 64, 128 or 256, at least 8 tokens per block (a run of 8 slots fits a block),
// and run indices small enough for the multiply-high division by R.
bool mfma_supports(const DevBatch& b) {
  if ((b.g.D != 64 && b.g.D != 128 && b.g.D != 256) || b.g.T < 8 || b.G > 16) return false;
  const uint64_t max_tok = (uint64_t)b.max_blocks * (uint64_t)b.g.T;
  const uint64_t max_run = (uint64_t)b.max_blocks * (uint64_t)b.R + 8;
  return max_tok < (1ull << 31) && max_run * (uint64_t)b.R < (1ull << 32);
}

hipError_t launch_mfma(const MultiArgs& A, int n_workgroups, hipStream_t s) {
  // LDS: per wave one 8-byte address per block of the largest split (+ slack)
  int entries = 0;
  for (int i = 0; i < A.n_batches; ++i) entries = std::max(entries, A.b[i].chunk_runs / A.b[i].R + 4);
  const size_t smem = (size_t)kWaves * entries * sizeof(uint64_t);
  switch (A.b[0].g.D) {  // (the caller checked that all batches share it)
    case 64: hipLaunchKernelGGL(mfma_attention_kernel<64>, dim3(n_workgroups), dim3(kThreads), smem, s, A, entries); break;
    case 128: hipLaunchKernelGGL(mfma_attention_kernel<128>, dim3(n_workgroups), dim3(kThreads), smem, s, A, entries); break;
    default: hipLaunchKernelGGL(mfma_attention_kernel<256>, dim3(n_workgroups), dim3(kThreads), smem, s, A, entries); break;
  }
  return hipGetLastError();
}

}  // namespace fs
