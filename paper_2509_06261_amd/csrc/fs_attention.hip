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

#include "fs_attention.h"

namespace fs {
namespace {

int g_kernel_mode = 0;
uint64_t g_split_bytes = 1u << 20;
bool g_timing = false;
hipEvent_t g_ev0 = nullptr, g_ev1 = nullptr;

// ---------------------------------------------------------------------------------------
// Work-list preparation: one workgroup scans the sequences of all batches and writes, for
// every sequence, the index of its first work item (items of a sequence = splits x KV heads).
// It also validates sequence lengths and resets the queue counter.
// ---------------------------------------------------------------------------------------
constexpr int kPrepThreads = 1024;

__device__ __forceinline__ int clamp_len(int len, int max_len, uint32_t* status) {
  if (len < 1 || len > max_len) {
    atomicOr(status, 1u);
    len = len < 1 ? 1 : max_len;
  }
  return len;
}

__global__ __launch_bounds__(kPrepThreads) void prep_kernel(MultiArgs A) {
  __shared__ uint32_t scan[kPrepThreads];
  __shared__ uint32_t s_running;
  const int tid = threadIdx.x;
  uint64_t* part_off = reinterpret_cast<uint64_t*>(A.header + kHdrPartOff);
  if (tid == 0) {
    s_running = 0;
    A.header[kHdrStatus] = 0;
  }
  __syncthreads();
  uint64_t part_running = 0;
  for (int b = 0; b < A.n_batches; ++b) {
    const DevBatch& B = A.b[b];
    const uint32_t batch_first = s_running;
    if (tid == 0) {
      A.header[kHdrBatchFirst + b] = batch_first;
      part_off[b] = part_running;
    }
    const int max_len = (int)min((int64_t)B.max_blocks * B.g.T, (int64_t)0x7fffffff);
    for (int base = 0; base < B.n_seq; base += kPrepThreads) {
      const int i = base + tid;
      uint32_t v = 0;
      if (i < B.n_seq) {
        const int len = clamp_len(B.seq_lens[i], max_len, A.header + kHdrStatus);
        v = (uint32_t)((len + B.chunk_tokens - 1) / B.chunk_tokens) * (uint32_t)B.g.H;
      }
      scan[tid] = v;
      __syncthreads();
      for (int off = 1; off < kPrepThreads; off <<= 1) {  // inclusive Hillis-Steele scan
        const uint32_t add = tid >= off ? scan[tid - off] : 0;
        __syncthreads();
        scan[tid] += add;
        __syncthreads();
      }
      const uint32_t running = s_running;
      if (i < B.n_seq) {
        const uint32_t first = running + scan[tid] - v;
        A.item_base[B.seq_first + i] = first;
        // the sequence's items in queue order: split-major, KV heads innermost
        const uint32_t H = (uint32_t)B.g.H;
        for (uint32_t r = 0; r < v && first + r < A.item_capacity; ++r)
          A.item_list[first + r] = make_int4(b, i, (int)(r / H), (int)(r % H));
      }
      __syncthreads();
      if (tid == kPrepThreads - 1) s_running = running + scan[tid];
      __syncthreads();
    }
    part_running += (uint64_t)(s_running - batch_first) * (uint64_t)B.part_stride;
  }
  if (tid == 0) {
    A.item_base[A.n_seq_total] = s_running;
    if (s_running > A.item_capacity) atomicOr(A.header + kHdrStatus, 2u);  // lengths exceed what the workspace was sized for
    A.header[kHdrTotalItems] = min(s_running, A.item_capacity);
    A.header[kHdrCounter] = 0;
  }
}

// ---------------------------------------------------------------------------------------
// Split combine: m = max m_i, l = sum l_i e^(m_i - m), out = sum acc_i e^(m_i - m) / l for the
// sequences that were split; sequences with a single split were finished by the attention
// kernel itself.  One workgroup per (sequence, query head).
// ---------------------------------------------------------------------------------------
constexpr int kCombineThreads = 128;

__global__ __launch_bounds__(kCombineThreads) void combine_kernel(MultiArgs A) {
  const int row = blockIdx.x;
  int b = 0;
  while (b + 1 < A.n_batches && row >= A.b[b + 1].qrow_first) ++b;
  const DevBatch& B = A.b[b];
  const int local = row - B.qrow_first;
  const int seq = local / B.n_q, h = local % B.n_q;
  const int max_len = (int)min((int64_t)B.max_blocks * B.g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : (len > max_len ? max_len : len);
  const int n_chunks = (len + B.chunk_tokens - 1) / B.chunk_tokens;
  if (n_chunks <= 1) return;
  const int D = B.g.D, H = B.g.H;
  const int kvh = h / B.G, gq = h % B.G;
  const uint32_t item0 = A.item_base[B.seq_first + seq];
  const uint64_t* part_off = reinterpret_cast<const uint64_t*>(A.header + kHdrPartOff);
  const uint64_t base = part_off[b] + (uint64_t)(item0 - A.header[kHdrBatchFirst + b]) * (uint64_t)B.part_stride;
  const uint64_t last = base + (uint64_t)((uint32_t)(n_chunks - 1) * H + kvh) * B.part_stride + (uint64_t)(gq + 1) * (D + 2);
  if (last > A.part_capacity) return;  // the attention kernel flagged this already
  const float* P = A.partials + base + (uint64_t)gq * (D + 2);
  const uint64_t chunk_stride = (uint64_t)H * B.part_stride;
  const uint64_t head_off = (uint64_t)kvh * B.part_stride;
  float M = -INFINITY;
  for (int c = 0; c < n_chunks; ++c) M = fmaxf(M, P[c * chunk_stride + head_off + D]);
  float L = 0.f;
  for (int c = 0; c < n_chunks; ++c) {
    const float* pc = P + c * chunk_stride + head_off;
    L += pc[D + 1] * expf(pc[D] - M);
  }
  const float inv = 1.0f / L;
  for (int d = threadIdx.x; d < D; d += kCombineThreads) {
    float o = 0.f;
    for (int c = 0; c < n_chunks; ++c) {
      const float* pc = P + c * chunk_stride + head_off;
      o += pc[d] * expf(pc[D] - M);
    }
    B.out[((int64_t)seq * B.n_q + h) * D + d] = (_Float16)(o * inv);
  }
  if (B.lse && threadIdx.x == 0) B.lse[(int64_t)seq * B.n_q + h] = M + logf(L);
}

}  // namespace

hipError_t launch_prep(const MultiArgs& A, hipStream_t s) {
  hipLaunchKernelGGL(prep_kernel, dim3(1), dim3(kPrepThreads), 0, s, A);
  return hipGetLastError();
}

hipError_t launch_combine(const MultiArgs& A, hipStream_t s) {
  hipLaunchKernelGGL(combine_kernel, dim3(A.n_qrows_total), dim3(kCombineThreads), 0, s, A);
  return hipGetLastError();
}

namespace {

struct Plan {
  MultiArgs args{};
  uint64_t workspace_bytes = 0;
  uint64_t ub_items = 0;
  bool all_mfma = true;
};

uint64_t align256(uint64_t x) { return (x + 255) & ~255ull; }

// Validates the batches and lays the workspace out.  With workspace == nullptr only sizes are computed.
int make_plan(fs_pool* p, const fs_batch_t* batches, int n_batches, void* workspace, Plan& plan) {
  if (!p || !batches || n_batches < 1 || n_batches > kMaxBatches) {
    set_error("decode attention: need 1..8 batches");
    return FS_ERR_INVALID;
  }
  MultiArgs& A = plan.args;
  A.n_batches = n_batches;
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
    if (g.kv_dtype == FS_KV_FP8_E4M3 && !M.d_k_scale) {
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
    int64_t ct = (int64_t)(g_split_bytes / token_bytes) / 32 * 32;
    ct = std::min<int64_t>(ct, (int64_t)2040 * g.tokens_per_block / 32 * 32);  // at most ~2K blocks per work item
    B.chunk_tokens = (int32_t)std::min<int64_t>(std::max<int64_t>(ct, 32), 1 << 20);
    B.seq_first = (int32_t)seq_total;
    B.part_stride = B.G * (g.head_dim + 2);
    B.qrow_first = (int32_t)qrows;
    B.t_magic = (uint32_t)(((1ull << 32) + (uint64_t)g.tokens_per_block - 1) / (uint64_t)g.tokens_per_block);
    seq_total += b.n_seq;
    qrows += (int64_t)b.n_seq * b.n_q_heads;
    // upper bound on this batch's work items
    uint64_t items = 0;
    const int64_t ub_len = std::min<int64_t>((int64_t)b.max_blocks * g.tokens_per_block, 0x7fffffff);
    if (b.seq_lens_host) {
      for (int s = 0; s < b.n_seq; ++s) {
        int64_t len = std::min<int64_t>(std::max<int64_t>(b.seq_lens_host[s], 1), ub_len);
        items += (uint64_t)((len + B.chunk_tokens - 1) / B.chunk_tokens);
      }
    } else {
      items = (uint64_t)b.n_seq * (uint64_t)((ub_len + B.chunk_tokens - 1) / B.chunk_tokens);
    }
    items *= (uint64_t)g.n_kv_heads;
    plan.ub_items += items;
    part_floats += items * (uint64_t)B.part_stride;
    if (!mfma_supports(B)) plan.all_mfma = false;
  }
  if (seq_total > 0x3fffffff || qrows > 0x7fffffff || plan.ub_items > 0xfffffff0ull) {
    set_error("decode attention: batch too large");
    return FS_ERR_INVALID;
  }
  A.n_seq_total = (int32_t)seq_total;
  A.n_qrows_total = (int32_t)qrows;
  A.part_capacity = part_floats;
  const uint64_t off_items = kHeaderBytes;
  const uint64_t off_list = align256(off_items + 4ull * (uint64_t)(seq_total + 1));
  const uint64_t off_part = align256(off_list + 16ull * plan.ub_items);
  A.item_capacity = (uint32_t)plan.ub_items;
  plan.workspace_bytes = align256(off_part + 4ull * part_floats);
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
}  // namespace fs

using namespace fs;

extern "C" {

int fs_set_kernel_mode(int mode) {
  if (mode < 0 || mode > 2) return FS_ERR_INVALID;
  g_kernel_mode = mode;
  return FS_OK;
}

int fs_set_kernel_timing(int enable) {
  if (enable && !g_ev0) {
    hipError_t e = hipEventCreate(&g_ev0);
    if (e == hipSuccess) e = hipEventCreate(&g_ev1);
    if (e != hipSuccess) return device_error(e, "hipEventCreate");
  }
  g_timing = enable != 0;
  return FS_OK;
}

float fs_last_attention_kernel_ms(void) {
  if (!g_ev0) return -1.0f;
  if (hipEventSynchronize(g_ev1) != hipSuccess) return -1.0f;
  float ms = -1.0f;
  if (hipEventElapsedTime(&ms, g_ev0, g_ev1) != hipSuccess) return -1.0f;
  return ms;
}

int fs_set_split_bytes(uint64_t bytes) {
  if (bytes < 4096 || bytes > (1ull << 30)) return FS_ERR_INVALID;
  g_split_bytes = bytes;
  return FS_OK;
}

uint64_t fs_decode_workspace_bytes(fs_pool* p, const fs_batch_t* batches, int n_batches) {
  Plan plan;
  if (make_plan(p, batches, n_batches, nullptr, plan) != FS_OK) return 0;
  return plan.workspace_bytes;
}

int fs_decode_attention_multi(fs_pool* p, const fs_batch_t* batches, int n_batches, void* workspace,
                              uint64_t workspace_bytes, void* stream) {
  Plan plan;
  if (!workspace || ((uintptr_t)workspace & 255)) {
    set_error("decode attention: workspace must be a 256-byte aligned device pointer");
    return FS_ERR_INVALID;
  }
  int rc = make_plan(p, batches, n_batches, workspace, plan);
  if (rc != FS_OK) return rc;
  if (workspace_bytes < plan.workspace_bytes) {
    set_error("decode attention: workspace too small (see fs_decode_workspace_bytes)");
    return FS_ERR_NOMEM;
  }
  if (p->n_cu == 0) {
    set_error("decode attention: pool has no HIP device");
    return FS_ERR_DEVICE;
  }
  bool use_mfma = plan.all_mfma;
  if (g_kernel_mode == 1) use_mfma = false;
  if (g_kernel_mode == 2 && !plan.all_mfma) {
    set_error("decode attention: MFMA kernel forced but a batch has a shape it does not support");
    return FS_ERR_INVALID;
  }
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();  // drop any stale error of an earlier, unrelated runtime call
  hipError_t e = launch_prep(plan.args, s);
  if (e != hipSuccess) return device_error(e, "prep launch");
  // Persistent grid: two workgroups per compute unit drain the queue (never more than the
  // upper bound on work items, so tiny batches launch tiny grids).
  static const int wgs_per_cu = [] {
    const char* e = getenv("FS_WGS_PER_CU");  // tuning knob for measurements
    const int v = e ? atoi(e) : 0;
    return v >= 1 && v <= 8 ? v : 2;
  }();
  const int n_wg = (int)std::min<uint64_t>((uint64_t)p->n_cu * wgs_per_cu, std::max<uint64_t>(plan.ub_items, 1));
  if (g_timing) (void)hipEventRecord(g_ev0, s);
  e = use_mfma ? launch_mfma(plan.args, n_wg, s) : launch_generic(plan.args, n_wg, s);
  if (g_timing) (void)hipEventRecord(g_ev1, s);
  if (e != hipSuccess) return device_error(e, "attention launch");
  e = launch_combine(plan.args, s);
  if (e != hipSuccess) return device_error(e, "combine launch");
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
