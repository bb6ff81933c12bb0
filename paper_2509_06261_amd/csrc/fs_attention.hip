// Split-K paged decode attention over the slab pool: host entry points, work-list
// preparation and split combine.
//
// FineServe Sec. 2.1: in the decode phase every new token reads the whole KV cache of its
// sequence, which makes attention memory-bound; Sec. 2.3: the cache is read through a block
// table as if it were contiguous; Sec. 5.1: the same kernel serves every co-located model
// because each model only sees its own logical block ids.  Here several models' batches are
// flattened into one queue of work items (sequence, split, KV head) that a persistent grid
// drains, in place of the paper's separate per-engine launches.
#include <algorithm>
#include <cstdlib>

#include "fs_append_rows.h"
#include "fs_attention.h"

// Workspace of fs_decode_attention_multi_static, the entry point for callers that cannot allocate: one copy per
// GPU, held until the process ends.  In host code the name is only a stand-in for the symbol: the device address
// comes from hipGetSymbolAddress, once per device (g_scratch_ptr), and only that pointer is ever handed to a kernel
// or a copy.  The launch's preparation kernel resets every counter it uses, so nothing else needs clearing.
constexpr uint64_t kStaticScratchBytes = 64ull << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxScratchDevices = 64;
static uint8_t* g_scratch_ptr[kMaxScratchDevices] = {};

namespace fs {
namespace {

// Largest work items of a launch (size tier 0): at most 768 KiB of KV, at least 64 KiB.
constexpr uint64_t kSplitMax = 768u << 10, kSplitMin = 64u << 10;
// The last 30 %, 15 % and 5 % of a batch's KV bytes (in sequence order) go to work items of 1/2, 1/4 and 1/8 the size
// (never less than one turn of the kernel's tile ring).  Measured on the four-model pool with the queue handed out
// front to back: two more tiers (1/16 and 1/32 for the last 3 % and 1 %) cut the waves' idle time at the end of the
// launch from 63 to 25 us and still lost 1 % (a quarter more items); thresholds of 0.75 / 0.90 / 0.96 or 0.80 / 0.92 /
// 0.97 lost 1 - 1.5 %; a largest item of 1 MiB instead of 768 KiB lost 3 %.
constexpr double kTierFrom[kTierSteps] = {0.70, 0.85, 0.95};

// ---------------------------------------------------------------------------------------
// Work-list preparation: scans the sequences of all batches and writes, for every sequence,
// the index of its first work item in sequence-major numbering (items of a sequence = splits
// x KV heads) and, for every work item, its record at the item's place in the queue.  Every
// workgroup repeats the (small) scans and writes its own share of the records; workgroup 0
// also writes the per-sequence and per-batch words, validates the sequence lengths and resets
// the counters.
//
// Queue order: the batches' item lists merged proportionally -- item i of the n_b items of
// batch b sorts by (i / n_b, b).  Its place is i + the number of items of the other batches
// that sort before it, a closed form, so no sort is run.
// ---------------------------------------------------------------------------------------
constexpr int kPrepThreads = 1024;
constexpr int kPrepGroups = 64;

// Items of the sequence a thread looks at (0 past the batch's last sequence) and its clamped length; flags lengths
// out of range.
__device__ __forceinline__ uint32_t seq_items(const MultiArgs& A, const DevBatch& B, int i, bool report, int& len) {
  len = 1;
  if (i >= B.n_seq) return 0;
  const int max_len = (int)min((int64_t)B.max_blocks * B.g.T, (int64_t)0x7fffffff);
  len = B.seq_lens[i];
  if (len < 1 || len > max_len) {
    if (report) atomicOr(A.header + kHdrStatus, 1u);
    len = len < 1 ? 1 : max_len;
  }
  return (uint32_t)n_splits(B, i, len) * (uint32_t)B.g.H;
}

// group: this workgroup's index among the n_groups workgroups that prepare the list
__device__ __forceinline__ void prep_body(const MultiArgs& A, uint32_t group, uint32_t n_groups) {
  __shared__ uint32_t s_incl[kPrepThreads];  // inclusive scan of the item counts of this round's sequences
  __shared__ int32_t s_len[kPrepThreads];    // clamped lengths of this round's sequences
  __shared__ uint32_t s_wave[kPrepThreads / 64];
  __shared__ uint32_t s_count[kMaxBatches];  // items of each batch
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool leader = group == 0;
  uint64_t* part_off = reinterpret_cast<uint64_t*>(A.header + kHdrPartOff);
  if (leader && tid == 0) A.header[kHdrStatus] = 0;
  // (the tickets below a pool's number of home waves are taken: every wave starts with its own)
  if (leader && tid < kDecodePools) A.header[kHdrPools + tid * kPoolStride] = (A.n_workers + kDecodePools - 1 - tid) / kDecodePools;
  if (tid < kMaxBatches) s_count[tid] = 0;
  __syncthreads();  // workgroup 0: the reset precedes every flag its threads may raise below

  // pass 1: items per batch
  for (int b = 0; b < A.n_batches; ++b) {
    const DevBatch& B = A.b[b];
    uint32_t v = 0;
    int unused;
    for (int i = tid; i < B.n_seq; i += kPrepThreads) v += seq_items(A, B, i, leader, unused);
#pragma unroll
    for (int off = 32; off; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0 && v) atomicAdd(&s_count[b], v);
  }
  __syncthreads();
  uint32_t count[kMaxBatches];
#pragma unroll
  for (int b = 0; b < kMaxBatches; ++b) count[b] = b < A.n_batches ? s_count[b] : 0u;

  // pass 2: per-sequence first items and the records.  The batches are dealt to the workgroups (workgroup g walks
  // the batches g % n_batches, + n_groups, ...: with as many workgroups as batches or more, exactly one), so that
  // the batches' scans run side by side instead of one after the other in every workgroup; the first workgroup of a
  // batch writes the batch's and its sequences' words.
  uint32_t total_items = 0;
  uint64_t part_running = 0;
  for (int b = 0; b < A.n_batches; ++b) {
    const DevBatch& B = A.b[b];
    const uint32_t H = (uint32_t)B.g.H;
    const uint32_t batch_first = total_items;
    const uint64_t batch_part = part_running;
    total_items += count[b];
    part_running += (uint64_t)count[b] * (uint64_t)B.part_stride;
    // the workgroups of this batch: b, b + n_batches, ... (all of them if there are fewer workgroups than batches)
    const bool dealt = n_groups >= (uint32_t)A.n_batches;
    if (dealt && group % (uint32_t)A.n_batches != (uint32_t)b) continue;
    const uint32_t b_group = dealt ? group / (uint32_t)A.n_batches : group;
    const uint32_t b_groups = dealt ? (n_groups - (uint32_t)b + (uint32_t)A.n_batches - 1) / (uint32_t)A.n_batches : n_groups;
    const bool b_leader = b_group == 0;
    uint32_t running = batch_first;  // items before the current round, sequence-major (same value in every thread)
    if (b_leader && tid == 0) {
      A.header[kHdrBatchFirst + b] = batch_first;
      part_off[b] = batch_part;
    }
    for (int base = 0; base < B.n_seq; base += kPrepThreads) {
      const int i = base + tid;
      int len_i;
      const uint32_t v = seq_items(A, B, i, false, len_i);
      s_len[tid] = len_i;
      // inclusive scan: within each wave by shuffles, then over the waves' totals
      uint32_t incl = v;
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_up(incl, off, 64);
        if (lane >= off) incl += t;
      }
      if (lane == 63) s_wave[wave] = incl;
      __syncthreads();
      uint32_t before = 0;
      for (int w = 0; w < wave; ++w) before += s_wave[w];
      incl += before;
      s_incl[tid] = incl;
      __syncthreads();
      const uint32_t round_items = s_incl[kPrepThreads - 1];
      if (b_leader && i < B.n_seq) A.item_base[B.seq_first + i] = running + incl - v;
      // item r of the round (sequence-major: sequence, then split, KV heads innermost) belongs to the first
      // sequence k whose inclusive count exceeds r
      for (uint32_t r = b_group * kPrepThreads + tid; r < round_items; r += b_groups * kPrepThreads) {
        int lo = 0, hi = kPrepThreads - 1;
        while (lo < hi) {
          const int mid = (lo + hi) >> 1;
          if (s_incl[mid] > r) hi = mid;
          else lo = mid + 1;
        }
        const uint32_t rr = r - (lo ? s_incl[lo - 1] : 0u);
        const uint64_t local = running - batch_first + r;  // index within the batch
        const uint64_t idx = queue_place(local, b, count);
        if (idx < A.item_capacity) {
          A.item_list[2 * idx] = make_rec(b, base + lo, (int)(rr / H), (int)(rr % H), (uint32_t)local);
          A.item_list[2 * idx + 1] = int4{s_len[lo], 0, 0, 0};
        }
      }
      __syncthreads();  // s_incl, s_len and s_wave are rewritten by the next round
      running += round_items;
    }
  }
  if (leader && tid == 0) {
    A.item_base[A.n_seq_total] = total_items;
    if (total_items > A.item_capacity) atomicOr(A.header + kHdrStatus, 2u);  // lengths exceed what the workspace was sized for
    A.header[kHdrTotalItems] = min(total_items, A.item_capacity);
    A.header[kHdrCounter] = 0;
  }
}

__global__ __launch_bounds__(kPrepThreads) void prep_kernel(MultiArgs A) { prep_body(A, blockIdx.x, gridDim.x); }

// Front kernel of a decode step: the first kPrepGroups workgroups prepare the work list, the others append the
// step's new K/V rows.  Neither reads what the other writes, so they share one launch.
__global__ __launch_bounds__(kPrepThreads) void step_front_kernel(MultiArgs A, append::MultiAppendArgs P) {
  if (blockIdx.x < kPrepGroups) prep_body(A, blockIdx.x, kPrepGroups);
  else append::append_block(P, blockIdx.x - kPrepGroups, kPrepThreads / 64);
}
static_assert(sizeof(MultiArgs) + sizeof(append::MultiAppendArgs) <= 4096, "kernel arguments of the front kernel");

// ---------------------------------------------------------------------------------------
// Split combine: m = max m_i, l = sum l_i e^(m_i - m), out = sum acc_i e^(m_i - m) / l for the
// sequences that were split; sequences with a single split were finished by the attention
// kernel itself.  One wave per (sequence, query head).
// ---------------------------------------------------------------------------------------
constexpr int kCombineWaves = 4;

// NK = number of 64-wide column groups of the head dimension (lane handles d = lane + 64 k).
template <int NK>
__device__ __forceinline__ void combine_row(const float* P, uint64_t chunk_stride, int n_chunks, int D, int lane,
                                            _Float16* out, float* lse) {
  const int dl = min(lane, D - 1);  // head_dim < 64: the surplus lanes repeat the last column
  // the splits' references and sums, one split per lane (both loads of the first 64 splits in flight together)
  float m0 = -INFINITY, l0 = 0.f;
  if (lane < n_chunks) {
    m0 = P[lane * chunk_stride + D];
    l0 = P[lane * chunk_stride + D + 1];
  }
  // the first four splits' partial sums do not depend on the reference: requested before it is reduced (a row has
  // four to five splits on average, so this is most rows' whole read); splits past the row's last repeat it with
  // weight 0
  float x0[4][NK];
#pragma unroll
  for (int u = 0; u < 4; ++u)
#pragma unroll
    for (int k = 0; k < NK; ++k) x0[u][k] = P[min(u, n_chunks - 1) * chunk_stride + dl + 64 * k];
  float M = m0;
  for (int c = lane + 64; c < n_chunks; c += 64) M = fmaxf(M, P[c * chunk_stride + D]);
#pragma unroll
  for (int off = 32; off; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
  // out[d] = sum_c w_c acc_c[d] / sum_c w_c l_c with w_c = e^(m_c - M); lane c' of each group of 64 splits
  // prepares the weight of split c0 + c', the accumulation reads it from there
  float L = 0.f;
  float o[NK];
#pragma unroll
  for (int k = 0; k < NK; ++k) o[k] = 0.f;
  for (int c0 = 0; c0 < n_chunks; c0 += 64) {
    float w = 0.f;
    if (c0 == 0) {
      w = expf(m0 - M);  // lanes without a split: e^(-inf) = 0
      L = l0 * w;
    } else if (c0 + lane < n_chunks) {
      const float* pc = P + (c0 + lane) * chunk_stride;
      w = expf(pc[D] - M);
      L += pc[D + 1] * w;
    }
    const int n = min(64, n_chunks - c0);
    const float* pg = P + c0 * chunk_stride + dl;
    // weight of split c0 + i, 0 past the group's last split (i, n uniform)
    auto weight = [&](int i) {
      const float wi = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w), min(i, 63)));
      return i < n ? wi : 0.f;
    };
    int c = 0;
    if (c0 == 0) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float wc = weight(u);
#pragma unroll
        for (int k = 0; k < NK; ++k) o[k] += x0[u][k] * wc;
      }
      c = 4;
    }
    for (; c + 8 <= n; c += 8) {  // eight splits' loads in flight together
      float x[8][NK];
#pragma unroll
      for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int k = 0; k < NK; ++k) x[u][k] = pg[(c + u) * chunk_stride + 64 * k];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const float wc = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(w), c + u));
#pragma unroll
        for (int k = 0; k < NK; ++k) o[k] += x[u][k] * wc;
      }
    }
    for (; c < n; c += 4) {  // the rest in fours, again all in flight together; surplus splits repeat the last, weight 0
      float x[4][NK];
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int k = 0; k < NK; ++k) x[u][k] = pg[min(c + u, n - 1) * chunk_stride + 64 * k];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float wc = weight(c + u);
#pragma unroll
        for (int k = 0; k < NK; ++k) o[k] += x[u][k] * wc;
      }
    }
  }
#pragma unroll
  for (int off = 32; off; off >>= 1) L += __shfl_xor(L, off, 64);
  const float inv = 1.0f / L;
  if (lane < D) {
#pragma unroll
    for (int k = 0; k < NK; ++k) out[lane + 64 * k] = (_Float16)(o[k] * inv);
  }
  if (lse && lane == 0) *lse = M + logf(L);
}

// MAXNK: the largest head_dim / 64 among the launch's batches.  The wider rows' code is compiled out of the
// narrower kernels: with it the kernel needs 128 registers per lane, which halves the waves a compute unit holds,
// and this kernel lives on the number of waves that wait for memory at the same time.
template <int MAXNK>
__global__ __launch_bounds__(kCombineWaves * 64, MAXNK <= 2 ? 8 : 4) void combine_kernel(MultiArgs A) {
  const int lane = threadIdx.x & 63;
  // one wave per (sequence, query head); the wave index is made provably uniform so that everything derived
  // from the row stays in scalar registers
  const int row = blockIdx.x * kCombineWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (row >= A.n_qrows_total) return;
  int b = 0;
  while (b + 1 < A.n_batches && row >= A.b[b + 1].qrow_first) ++b;
  const DevBatch& B = A.b[b];
  const int local = row - B.qrow_first;
  const int seq = local / B.n_q, h = local % B.n_q;
  const int max_len = (int)min((int64_t)B.max_blocks * B.g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : (len > max_len ? max_len : len);
  const int n_chunks = n_splits(B, seq, len);
  if (n_chunks <= 1) return;
  const int D = B.g.D, H = B.g.H;
  const int kvh = h / B.G, gq = h % B.G;
  const uint32_t item0 = A.item_base[B.seq_first + seq];
  const uint64_t* part_off = reinterpret_cast<const uint64_t*>(A.header + kHdrPartOff);
  const uint64_t base = part_off[b] + (uint64_t)(item0 - A.header[kHdrBatchFirst + b]) * (uint64_t)B.part_stride;
  const uint64_t last = base + (uint64_t)((uint32_t)(n_chunks - 1) * H + kvh) * B.part_stride + (uint64_t)(gq + 1) * (D + 2);
  if (last > A.part_capacity) return;  // the attention kernel flagged this already
  const uint64_t chunk_stride = (uint64_t)H * B.part_stride;
  const float* P = A.partials + base + (uint64_t)kvh * B.part_stride + (uint64_t)gq * (D + 2);
  _Float16* out = B.out + ((int64_t)seq * B.n_q + h) * D;
  float* lse = B.lse ? B.lse + (int64_t)seq * B.n_q + h : nullptr;
  if (D <= 64) combine_row<1>(P, chunk_stride, n_chunks, D, lane, out, lse);
  else if (MAXNK >= 2 && D == 128) combine_row<2>(P, chunk_stride, n_chunks, D, lane, out, lse);
  else if (MAXNK >= 4 && D == 256) combine_row<4>(P, chunk_stride, n_chunks, D, lane, out, lse);
  else if (MAXNK >= 8) combine_row<8>(P, chunk_stride, n_chunks, D, lane, out, lse);
}

}  // namespace

hipError_t launch_prep(const MultiArgs& A, hipStream_t s) {
  hipLaunchKernelGGL(prep_kernel, dim3(kPrepGroups), dim3(kPrepThreads), 0, s, A);
  return hipGetLastError();
}

hipError_t launch_step_front(const fs_pool* p, const MultiArgs& A, append::MultiAppendArgs& P, hipStream_t s) {
  const uint32_t append_blocks = plan_append_blocks(p, P, kPrepThreads / 64);
  hipLaunchKernelGGL(step_front_kernel, dim3(kPrepGroups + append_blocks), dim3(kPrepThreads), 0, s, A, P);
  return hipGetLastError();
}

hipError_t launch_combine(const MultiArgs& A, hipStream_t s) {
  int max_d = 0;
  for (int i = 0; i < A.n_batches; ++i) max_d = std::max(max_d, (int)A.b[i].g.D);
  const dim3 grid((A.n_qrows_total + kCombineWaves - 1) / kCombineWaves), block(kCombineWaves * 64);
  if (max_d <= 64) hipLaunchKernelGGL(combine_kernel<1>, grid, block, 0, s, A);
  else if (max_d <= 128) hipLaunchKernelGGL(combine_kernel<2>, grid, block, 0, s, A);
  else if (max_d <= 256) hipLaunchKernelGGL(combine_kernel<4>, grid, block, 0, s, A);
  else hipLaunchKernelGGL(combine_kernel<8>, grid, block, 0, s, A);
  return hipGetLastError();
}

namespace {

struct Plan {
  MultiArgs args{};
  uint64_t workspace_bytes = 0;
  uint64_t ub_items = 0;
  bool all_mfma = true;
  bool use_mfma = false;
};

uint64_t align256(uint64_t x) { return (x + 255) & ~255ull; }

// Runs of 8 token slots per work item for a target of split_bytes per item (a multiple of 4, at most 250 blocks).
int32_t chunk_runs_for(const fs_geometry_t& g, uint64_t split_bytes) {
  const uint64_t token_bytes = 2 * (g.row_bytes + (uint64_t)g.param_bytes);  // K+V of one head
  const int64_t R = (g.tokens_per_block + 7) / 8;
  int64_t cr = (int64_t)(split_bytes / (8 * token_bytes)) / 4 * 4;
  cr = std::min<int64_t>(cr, 250 * R / 4 * 4);  // an item touches at most 256 blocks (the kernel's address table)
  return (int32_t)std::min<int64_t>(std::max<int64_t>(cr, 4), 1 << 17);
}

// KV bytes of one head that sequence s of a batch holds (lengths not known on the host count at their upper bound).
uint64_t head_bytes(const fs_batch_t& b, const fs_geometry_t& g, int s) {
  const uint64_t ub_len = (uint64_t)b.max_blocks * (uint64_t)g.tokens_per_block;
  const uint64_t len = b.seq_lens_host ? std::min<uint64_t>((uint64_t)std::max(b.seq_lens_host[s], 1), ub_len) : ub_len;
  return len * 2 * (g.row_bytes + (uint64_t)g.param_bytes);
}

// KV bytes per split-K work item of this launch (size tier 0).  A work item costs a few microseconds of set-up
// whatever its size (measured: about 3 us against 66 us of streaming for 192 KiB), and the launch ends when the
// last wave finishes its last item, on average 0.4 items after the others.  Large items for most of the launch and
// small ones at its end serve both: tier 0 is 3/8 of a wave's share of the launch (about two such items per wave
// before the smaller tiers begin), at most 768 KiB, and the later tiers halve it three times.  With
// FS_OPT_SPLIT_BYTES set every item has that size (no tiers).
uint64_t launch_split_bytes(const fs_pool* p, const fs_batch_t* batches, int n_batches) {
  if (p && p->opt.split_bytes) return p->opt.split_bytes;
  if (!p || !batches || p->n_cu == 0) return kSplitMax;
  uint64_t total = 0;
  for (int i = 0; i < n_batches; ++i) {
    const fs_batch_t& b = batches[i];
    if (b.model < 0 || b.model >= kMaxModels || !p->models[b.model].in_use || b.n_seq < 1 || b.max_blocks < 1) return kSplitMax;
    const fs_geometry_t& g = p->models[b.model].g;
    uint64_t bytes = 0;
    for (int s = 0; s < b.n_seq; ++s) bytes += head_bytes(b, g, s);
    total += bytes * (uint64_t)g.n_kv_heads;
  }
  const uint64_t waves = (uint64_t)p->n_cu * 4 * mfma_wgs_per_cu(p->models[batches[0].model].g.head_dim);
  return std::min(kSplitMax, std::max(kSplitMin, total / waves * 3 / 8 / 4096 * 4096));
}

// Validates the batches and lays the workspace out.  With workspace == nullptr only sizes are computed.
// need_scales: an FP8 model without its scales is refused (what every launch wants; the index check asks without).
int make_plan(fs_pool* p, const fs_batch_t* batches, int n_batches, void* workspace, Plan& plan, bool need_scales = true) {
  if (!p || !batches || n_batches < 1 || n_batches > kMaxBatches) {
    set_error("decode attention: need 1..8 batches");
    return FS_ERR_INVALID;
  }
  MultiArgs& A = plan.args;
  A.n_batches = n_batches;
  const uint64_t split_bytes = launch_split_bytes(p, batches, n_batches);
  int64_t seq_total = 0, qrows = 0;
  uint64_t part_floats = 0;
  for (int i = 0; i < n_batches; ++i) {
    const fs_batch_t& b = batches[i];
    if (b.model < 0 || b.model >= kMaxModels || !p->models[b.model].in_use) {
      set_error("decode attention: unknown model");
      return FS_ERR_INVALID;
    }
    const Model& M = p->models[b.model];
    const fs_geometry_t& g = M.g;
    if (b.layer < 0 || b.layer >= g.n_layers || b.n_seq < 1 || b.max_blocks < 1 || !b.q || !b.block_tables ||
        !b.seq_lens || !b.out || b.n_q_heads < g.n_kv_heads || b.n_q_heads % g.n_kv_heads ||
        b.n_q_heads / g.n_kv_heads > 16 || !(b.sm_scale == b.sm_scale)) {
      set_error("decode attention: invalid batch argument");
      return FS_ERR_INVALID;
    }
    if (((uintptr_t)b.q | (uintptr_t)b.out) & 15) {  // rows are moved as 16-byte vectors
      set_error("decode attention: q and out must be 16-byte aligned");
      return FS_ERR_INVALID;
    }
    if (need_scales && g.kv_dtype == FS_KV_FP8_E4M3 && !M.d_k_scale) {
      set_error("decode attention: FP8 model has no scales (fs_model_set_fp8_scales)");
      return FS_ERR_INVALID;
    }
    DevBatch& B = A.b[i];
    B.g = dev_geom(g);
    B.layer_base = p->base + (uint64_t)b.layer * g.layer_bytes;
    B.q = (const _Float16*)b.q;
    B.tables = b.block_tables;
    B.seq_lens = b.seq_lens;
    B.out = (_Float16*)b.out;
    B.lse = b.lse;
    B.k_scale = M.d_k_scale ? M.d_k_scale + (size_t)b.layer * g.n_kv_heads : nullptr;
    B.v_scale = M.d_v_scale ? M.d_v_scale + (size_t)b.layer * g.n_kv_heads : nullptr;
    B.n_seq = b.n_seq;
    B.max_blocks = b.max_blocks;
    B.n_q = b.n_q_heads;
    B.G = b.n_q_heads / g.n_kv_heads;
    B.sm_scale = b.sm_scale;
    const uint64_t token_bytes = 2 * (g.row_bytes + (uint64_t)g.param_bytes);  // K+V of one head
    const bool tiers = p->opt.split_bytes == 0;
    int64_t ct = (int64_t)(split_bytes / token_bytes) / 32 * 32;
    ct = std::min<int64_t>(ct, (int64_t)500 * g.tokens_per_block / 32 * 32);  // at most ~500 blocks per work item
    ct = std::min<int64_t>(std::max<int64_t>(ct, 32), 1 << 20);
    if (tiers && ct >= 256) ct = ct / 256 * 256;  // every tier's size stays a multiple of 32
    B.chunk_tokens = (int32_t)ct;
    B.R = (g.tokens_per_block + 7) / 8;
    B.r_magic = B.R == 1 ? 0u : (uint32_t)(((1ull << 32) + (uint64_t)B.R - 1) / (uint64_t)B.R);  // unused for R = 1
    B.chunk_runs = chunk_runs_for(g, split_bytes);
    B.ring_runs = 4 * ring_tiles(g.kv_dtype, g.head_dim);
    // with tiers every tier's size stays a whole number of ring turns; a forced size is rounded to whole tiles only
    if (tiers) B.chunk_runs = std::max(B.chunk_runs / (8 * B.ring_runs), 1) * 8 * B.ring_runs;
    else B.ring_runs = 4;
    B.n_blocks = (uint32_t)(p->pool_bytes / g.block_budget);
    // size tiers: first sequence of tiers 1.., by the share of the batch's KV bytes that lies in front of it
    for (int t = 0; t < kTierSteps; ++t) B.tier_seq[t] = b.n_seq;
    if (tiers) {
      uint64_t batch_bytes = 0;
      for (int s = 0; s < b.n_seq; ++s) batch_bytes += head_bytes(b, g, s);
      uint64_t before = 0;
      int t = 0;
      for (int s = 0; s < b.n_seq && t < kTierSteps; ++s) {
        while (t < kTierSteps && (double)before >= kTierFrom[t] * (double)batch_bytes) B.tier_seq[t++] = s;
        before += head_bytes(b, g, s);
      }
    }
    B.seq_first = (int32_t)seq_total;
    B.part_stride = B.G * (g.head_dim + 2);
    B.qrow_first = (int32_t)qrows;
    seq_total += b.n_seq;
    qrows += (int64_t)b.n_seq * b.n_q_heads;
    // upper bound on this batch's work items under either split rule (which kernel runs is decided below)
    uint64_t items_tok = 0, items_run = 0;
    const int64_t ub_len = std::min<int64_t>((int64_t)b.max_blocks * g.tokens_per_block, 0x7fffffff);
    for (int s = 0; s < b.n_seq; ++s) {
      const int64_t len = b.seq_lens_host ? std::min<int64_t>(std::max<int64_t>(b.seq_lens_host[s], 1), ub_len) : ub_len;
      const int64_t cts = chunk_tokens_of(B, s), crs = chunk_runs_of(B, s);
      items_tok += (uint64_t)((len + cts - 1) / cts);
      items_run += (uint64_t)((n_runs((int)len, g.tokens_per_block, B.R) + crs - 1) / crs);
    }
    const uint64_t items = std::max(items_tok, items_run) * (uint64_t)g.n_kv_heads;
    plan.ub_items += items;
    part_floats += items * (uint64_t)B.part_stride;
    // one launch of the MFMA kernel serves one head_dim
    if (!mfma_supports(B) || B.g.D != A.b[0].g.D) plan.all_mfma = false;
  }
  if (seq_total > 0x3fffffff || qrows > 0x7fffffff || plan.ub_items > 0xfffffff0ull) {
    set_error("decode attention: batch too large");
    return FS_ERR_INVALID;
  }
  // the generic kernel splits by tokens, the MFMA kernel by runs
  plan.use_mfma = plan.all_mfma && p->opt.decode_kernel != 1;
  if (!plan.use_mfma)
    for (int i = 0; i < n_batches; ++i) A.b[i].chunk_runs = 0;
  A.n_seq_total = (int32_t)seq_total;
  A.n_qrows_total = (int32_t)qrows;
  A.part_capacity = part_floats;
  const uint64_t off_items = kHeaderBytes;
  const uint64_t off_list = align256(off_items + 4ull * (uint64_t)(seq_total + 1));
  const uint64_t off_part = align256(off_list + 32ull * plan.ub_items);
  A.item_capacity = (uint32_t)plan.ub_items;
  plan.workspace_bytes = align256(off_part + 4ull * part_floats);
#ifdef FS_TIMELINE
  const uint64_t off_timeline = plan.workspace_bytes;
  plan.workspace_bytes += kTimelineBytes;
  if (workspace) A.timeline = (uint64_t*)((uint8_t*)workspace + off_timeline);
#endif
  if (workspace) {
    uint8_t* w = (uint8_t*)workspace;
    A.header = (uint32_t*)w;
    A.item_base = (uint32_t*)(w + off_items);
    A.item_list = (int4*)(w + off_list);
    A.partials = (float*)(w + off_part);
  }
  return FS_OK;
}

}  // namespace

int debug_plan(fs_pool* p, const fs_batch_t* batches, int n_batches, MultiArgs* out, bool* use_mfma) {
  Plan plan;
  const int rc = make_plan(p, batches, n_batches, nullptr, plan, false);
  if (rc != FS_OK) return rc;
  if (out) *out = plan.args;
  if (use_mfma) *use_mfma = plan.use_mfma;
  return FS_OK;
}

}  // namespace fs

using namespace fs;

namespace {
// Validates, lays the workspace out and enqueues work-list preparation, attention and split combine on `s`.
// Allocates nothing.
// time_begin / time_end: this launch holds the start / the end of what FS_OPT_KERNEL_TIMING brackets.
int decode_launch_one(fs_pool* p, const fs_batch_t* batches, int n_batches, void* workspace, uint64_t workspace_bytes,
                      const char* too_small, hipStream_t s, const fs_append_t* appends, int n_appends, bool time_begin,
                      bool time_end) {
  Plan plan;
  if (!workspace || ((uintptr_t)workspace & 255)) {
    set_error("decode attention: workspace must be a 256-byte aligned device pointer");
    return FS_ERR_INVALID;
  }
  int rc = make_plan(p, batches, n_batches, workspace, plan);
  if (rc != FS_OK) return rc;
  if (workspace_bytes < plan.workspace_bytes) {
    set_error(too_small);
    return FS_ERR_NOMEM;
  }
  if (p->n_cu == 0) {
    set_error("decode attention: pool has no HIP device");
    return FS_ERR_DEVICE;
  }
  const bool use_mfma = plan.use_mfma;
  if (p->opt.decode_kernel == 2 && !plan.all_mfma) {
    set_error("decode attention: MFMA kernel forced but a batch has a shape it does not support");
    return FS_ERR_INVALID;
  }
  append::MultiAppendArgs P{};
  for (int i = 0; i < n_appends; ++i) {
    rc = make_append_args(p, appends[i], P.a[P.n]);
    if (rc != FS_OK) return rc;
    if (appends[i].n_tokens > 0) ++P.n;
  }
  (void)hipGetLastError();  // drop any stale error of an earlier, unrelated runtime call
  // Persistent grid: as many workgroups as fit the compute units at once (two each, eight waves; one for the MFMA
  // kernel at head_dim 256) drain the queue (never more than the upper bound on work items, so tiny batches launch
  // tiny grids).
  const int wgs_per_cu = use_mfma ? mfma_wgs_per_cu(plan.args.b[0].g.D) : 2;
  // (the MFMA kernel's workers are waves, four to a workgroup; the generic kernel's are workgroups)
  const uint64_t workers_per_wg = use_mfma ? 4 : 1;
  const int n_wg = (int)std::min<uint64_t>((uint64_t)p->n_cu * wgs_per_cu,
                                           std::max<uint64_t>((plan.ub_items + workers_per_wg - 1) / workers_per_wg, 1));
  plan.args.n_workers = use_mfma ? (uint32_t)n_wg * (uint32_t)workers_per_wg : 0u;
  hipError_t e = P.n ? launch_step_front(p, plan.args, P, s) : launch_prep(plan.args, s);
  if (e != hipSuccess) return device_error(e, "prep launch");
  if (p->opt.timing && time_begin) (void)hipEventRecord(p->opt.ev0, s);
  e = use_mfma ? launch_mfma(plan.args, n_wg, s) : launch_generic(plan.args, n_wg, s);
  if (p->opt.timing && time_end) (void)hipEventRecord(p->opt.ev1, s);
  if (e != hipSuccess) return device_error(e, "attention launch");
  e = launch_combine(plan.args, s);
  if (e != hipSuccess) return device_error(e, "combine launch");
  return FS_OK;
}

// The MFMA kernel serves one head_dim per launch, and a launch with a batch it does not cover runs on the vector-ALU
// kernel as a whole.  A call whose batches differ in that respect is therefore run as one launch sequence (work list,
// attention, combine) per kind -- head_dim 64, 128, 256 on the MFMA kernel, everything else on the vector-ALU kernel --
// each in its own slice of the workspace.
constexpr int kMaxGroups = 4;
struct HeadDimGroups {
  int n = 1;                       // 1: the call is one launch
  int count[kMaxGroups] = {0, 0, 0, 0};
  fs_batch_t b[kMaxGroups][kMaxBatches];
};

void group_by_head_dim(const fs_pool* p, const fs_batch_t* batches, int n_batches, HeadDimGroups& G) {
  G.n = 1;
  if (!p || !batches || n_batches < 2 || n_batches > kMaxBatches || p->opt.decode_kernel == 1) return;
  int dims[kMaxGroups] = {0, 0, 0, 0}, n_dims = 0;  // a group's head_dim; 0: the batches the MFMA kernel does not cover
  for (int i = 0; i < n_batches; ++i) {
    const fs_batch_t& b = batches[i];
    if (b.model < 0 || b.model >= kMaxModels || !p->models[b.model].in_use) return;  // (make_plan reports it)
    const fs_geometry_t& g = p->models[b.model].g;
    if (g.n_kv_heads < 1 || b.n_q_heads < g.n_kv_heads || b.max_blocks < 1) return;
    DevBatch B{};
    B.g = dev_geom(g);
    B.G = b.n_q_heads / g.n_kv_heads;
    B.max_blocks = b.max_blocks;
    B.R = (g.tokens_per_block + 7) / 8;
    const int key = mfma_supports(B) ? g.head_dim : 0;
    int k = 0;
    while (k < n_dims && dims[k] != key) ++k;
    if (k == n_dims) dims[n_dims++] = key;  // (mfma_supports admits three head_dims: at most four kinds)
    G.b[k][G.count[k]++] = b;
  }
  if (n_dims < 2) {
    for (int k = 0; k < kMaxGroups; ++k) G.count[k] = 0;
    return;
  }
  G.n = n_dims;
}

__global__ void merge_status_kernel(uint32_t* first, const uint32_t* second, const uint32_t* third, const uint32_t* fourth) {
  if (threadIdx.x == 0)
    first[kHdrStatus] |= second[kHdrStatus] | (third ? third[kHdrStatus] : 0u) | (fourth ? fourth[kHdrStatus] : 0u);
}

int decode_launch(fs_pool* p, const fs_batch_t* batches, int n_batches, void* workspace, uint64_t workspace_bytes,
                  const char* too_small, hipStream_t s, const fs_append_t* appends = nullptr, int n_appends = 0) {
  HeadDimGroups G;
  group_by_head_dim(p, batches, n_batches, G);
  if (G.n == 1)
    return decode_launch_one(p, batches, n_batches, workspace, workspace_bytes, too_small, s, appends, n_appends, true, true);
  if (!workspace || ((uintptr_t)workspace & 255)) {
    set_error("decode attention: workspace must be a 256-byte aligned device pointer");
    return FS_ERR_INVALID;
  }
  // every launch's slice of the workspace; nothing is enqueued unless all of them fit
  uint8_t* slice[kMaxGroups] = {nullptr, nullptr, nullptr, nullptr};
  uint64_t bytes[kMaxGroups] = {0, 0, 0, 0}, used = 0;
  for (int k = 0; k < G.n; ++k) {
    Plan plan;
    const int rc = make_plan(p, G.b[k], G.count[k], nullptr, plan);
    if (rc != FS_OK) return rc;
    if (p->opt.decode_kernel == 2 && !plan.all_mfma) {
      set_error("decode attention: MFMA kernel forced but a batch has a shape it does not support");
      return FS_ERR_INVALID;
    }
    slice[k] = (uint8_t*)workspace + used;
    bytes[k] = plan.workspace_bytes;  // (a multiple of 256)
    used += plan.workspace_bytes;
  }
  if (used > workspace_bytes) {
    set_error(too_small);
    return FS_ERR_NOMEM;
  }
  for (int k = 0; k < G.n; ++k) {
    // the step's appends ride in the first launch's front kernel: they precede every attention launch of the call
    const int rc = decode_launch_one(p, G.b[k], G.count[k], slice[k], bytes[k], too_small, s, k == 0 ? appends : nullptr,
                                     k == 0 ? n_appends : 0, k == 0, k == G.n - 1);
    if (rc != FS_OK) return rc;
  }
  // fs_decode_status reads the first slice's header
  hipLaunchKernelGGL(merge_status_kernel, dim3(1), dim3(64), 0, s, (uint32_t*)slice[0], (const uint32_t*)slice[1],
                     (const uint32_t*)slice[2], (const uint32_t*)slice[3]);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return device_error(e, "status merge launch");
  return FS_OK;
}

}  // namespace

extern "C" {

int fs_pool_set_option(fs_pool* p, int option, int64_t value) {
  if (!p) return FS_ERR_INVALID;
  Options& o = p->opt;
  switch (option) {
    case FS_OPT_DECODE_KERNEL:
      if (value < 0 || value > 2) break;
      o.decode_kernel = (int)value;
      return FS_OK;
    case FS_OPT_SPLIT_BYTES:
      if (value != 0 && (value < 4096 || value > (1ll << 30))) break;
      o.split_bytes = (uint64_t)value;
      return FS_OK;
    case FS_OPT_KERNEL_TIMING:
      if (value && !o.ev0) {
        hipError_t e = hipEventCreate(&o.ev0);
        if (e == hipSuccess) e = hipEventCreate(&o.ev1);
        if (e != hipSuccess) return device_error(e, "hipEventCreate");
      }
      o.timing = value != 0;
      return FS_OK;
    case FS_OPT_PREFILL_COLUMN_BLOCKS:
      // (8 once selected a variant with two workgroups per compute unit, which is no longer built)
      if (value != 0 && value != 1 && value != 2 && value != 4 && value != 16) break;
      o.prefill_ncb = (int)value;
      return FS_OK;
    case FS_OPT_PREFILL_WAVES:
      if (value != 0 && value != 4 && value != 8) break;
      o.prefill_nw = (int)value;
      return FS_OK;
    case FS_OPT_PREFILL_PIPELINED:
      o.prefill_pipe = value != 0;
      return FS_OK;
    case FS_OPT_PREFILL_STAGED_DEQUANT:
      o.prefill_deq = value != 0;
      return FS_OK;
    default:
      break;
  }
  set_error("fs_pool_set_option: unknown option or value out of range");
  return FS_ERR_INVALID;
}

int fs_pool_get_option(fs_pool* p, int option, int64_t* value) {
  if (!p || !value) return FS_ERR_INVALID;
  const Options& o = p->opt;
  switch (option) {
    case FS_OPT_DECODE_KERNEL: *value = o.decode_kernel; return FS_OK;
    case FS_OPT_SPLIT_BYTES: *value = (int64_t)o.split_bytes; return FS_OK;
    case FS_OPT_KERNEL_TIMING: *value = o.timing; return FS_OK;
    case FS_OPT_PREFILL_COLUMN_BLOCKS: *value = o.prefill_ncb; return FS_OK;
    case FS_OPT_PREFILL_WAVES: *value = o.prefill_nw; return FS_OK;
    case FS_OPT_PREFILL_PIPELINED: *value = o.prefill_pipe; return FS_OK;
    case FS_OPT_PREFILL_STAGED_DEQUANT: *value = o.prefill_deq; return FS_OK;
    case FS_OPT_LAST_PREFILL_KERNEL: *value = o.last_prefill; return FS_OK;
    default: break;
  }
  set_error("fs_pool_get_option: unknown option");
  return FS_ERR_INVALID;
}

float fs_pool_last_attention_kernel_ms(fs_pool* p) {
  if (!p || !p->opt.ev0) return -1.0f;
  if (hipEventSynchronize(p->opt.ev1) != hipSuccess) return -1.0f;
  float ms = -1.0f;
  if (hipEventElapsedTime(&ms, p->opt.ev0, p->opt.ev1) != hipSuccess) return -1.0f;
  return ms;
}

#ifdef FS_TIMELINE
// (timeline build only) bytes of the clock readings at the end of a launch's workspace, and their layout
uint64_t fs_timeline_bytes(uint64_t* wave_rows, uint64_t* item_rows) {
  if (wave_rows) *wave_rows = kTimelineWaves;
  if (item_rows) *item_rows = kTimelineItems;
  return kTimelineBytes;
}
#endif

uint64_t fs_decode_workspace_bytes(fs_pool* p, const fs_batch_t* batches, int n_batches) {
  HeadDimGroups G;
  group_by_head_dim(p, batches, n_batches, G);
  uint64_t bytes = 0;
  for (int k = 0; k < G.n; ++k) {
    Plan plan;
    if (make_plan(p, G.n == 1 ? batches : G.b[k], G.n == 1 ? n_batches : G.count[k], nullptr, plan) != FS_OK) return 0;
    bytes += plan.workspace_bytes;
  }
  return bytes;
}

int fs_decode_attention_multi(fs_pool* p, const fs_batch_t* batches, int n_batches, void* workspace,
                              uint64_t workspace_bytes, void* stream) {
  return decode_launch(p, batches, n_batches, workspace, workspace_bytes, "decode attention: workspace too small (see fs_decode_workspace_bytes)",
                       (hipStream_t)stream);
}

int fs_decode_step_multi(fs_pool* p, const fs_append_t* appends, int n_appends, const fs_batch_t* batches, int n_batches,
                         void* workspace, uint64_t workspace_bytes, void* stream) {
  if (n_appends < 0 || n_appends > append::kMaxAppends || (n_appends > 0 && !appends)) {
    set_error("decode step: need 0..8 appends");
    return FS_ERR_INVALID;
  }
  return decode_launch(p, batches, n_batches, workspace, workspace_bytes,
                       "decode step: workspace too small (see fs_decode_workspace_bytes)", (hipStream_t)stream, appends, n_appends);
}

int fs_decode_attention_multi_static(fs_pool* p, const fs_batch_t* batches, int n_batches, uint32_t* status_out,
                                     void* stream) {
  if (!p) {
    set_error("decode attention: no pool");
    return FS_ERR_INVALID;
  }
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return device_error(e, "hipGetDevice");
  if (p->n_cu == 0 || dev != p->device || dev < 0 || dev >= kMaxScratchDevices) {
    set_error("decode attention (static scratch): the pool's device must be the current device");
    return FS_ERR_INVALID;
  }
  if (!g_scratch_ptr[dev]) {
    // once per device, with that device current: every GPU holds its own copy of the array at its own address
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return device_error(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = (uint8_t*)ptr;
  }
  uint8_t* ws = g_scratch_ptr[dev];
  const int rc = decode_launch(p, batches, n_batches, ws, kStaticScratchBytes,
                               "decode attention (static scratch): the batches need more than the 64 MiB static scratch; "
                               "use fs_decode_attention_multi with a caller workspace",
                               (hipStream_t)stream);
  if (rc != FS_OK) return rc;
  if (status_out) {
    e = hipMemcpyAsync(status_out, ws + 4 * kHdrStatus, 4, hipMemcpyDeviceToDevice, (hipStream_t)stream);
    if (e != hipSuccess) return device_error(e, "hipMemcpyAsync(status)");
  }
  return FS_OK;
}

int fs_decode_attention(fs_pool* p, fs_model_t model, int layer, int n_q_heads, float sm_scale, const void* q,
                        const int32_t* block_tables, const int32_t* seq_lens, int n_seq, int max_blocks, void* out,
                        float* lse, void* workspace, uint64_t workspace_bytes, void* stream) {
  fs_batch_t b{};
  b.model = model;
  b.layer = layer;
  b.n_q_heads = n_q_heads;
  b.sm_scale = sm_scale;
  b.q = q;
  b.block_tables = block_tables;
  b.seq_lens = seq_lens;
  b.seq_lens_host = nullptr;
  b.n_seq = n_seq;
  b.max_blocks = max_blocks;
  b.out = out;
  b.lse = lse;
  return fs_decode_attention_multi(p, &b, 1, workspace, workspace_bytes, stream);
}

int fs_decode_status(const void* workspace, void* stream) {
  if (!workspace) return FS_ERR_INVALID;
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return device_error(e, "hipStreamSynchronize");
  uint32_t hdr[4] = {0, 0, 0, 0};
  e = hipMemcpy(hdr, workspace, sizeof hdr, hipMemcpyDeviceToHost);
  if (e != hipSuccess) return device_error(e, "hipMemcpy(status)");
  return (int)hdr[kHdrStatus];
}

}  // extern "C"
