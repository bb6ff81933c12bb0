// Generic split-K paged decode-attention kernel (vector ALU only).
//
// Handles every supported shape (any head_dim that is a power of two multiple of 8 up to
// 512, any tokens_per_block, up to 16 query heads per KV head) and all four KV formats.
// It is the fallback for shapes the MFMA kernel does not cover and the second, independently
// structured GPU implementation that full-size runs are cross-checked against.
//
// FineServe Sec. 2.1 / 2.3: decode attention reads every cached token of a sequence through
// its block table; Sec. 5.1: block b of a model lives at pool + b * block_budget.
//
// Structure: a persistent grid pulls work items (sequence, split, KV head) from a ticket
// counter.  Inside a workgroup, groups of head_dim/8 lanes each own one token at a time
// (8 elements per lane), keep a private online-softmax state (m, l, acc) per query head of
// the KV head's group, and are merged through LDS at the end of the item.
#include "fs_attention.h"

namespace fs {
namespace {

constexpr int kThreads = 256;

// ---- 8-element row fragment loads, dequantized to fp32 (without per-token/static scale) ----
template <int DT>
__device__ __forceinline__ void load8(const uint8_t* p, float (&x)[8]);

template <>
__device__ __forceinline__ void load8<FS_KV_FP16>(const uint8_t* p, float (&x)[8]) {
  const uint4 v = *reinterpret_cast<const uint4*>(p);
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] & 0xFFFF));
    x[2 * i + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[i] >> 16));
  }
}

// Exact E4M3 -> fp32 by bit manipulation (normal codes: rebias the exponent; subnormal: m * 2^-9).
__device__ __forceinline__ float e4m3_to_f32(uint32_t b) {
  const uint32_t em = b & 0x7F;
  const float mag = (em >> 3) ? __uint_as_float((em << 20) + (120u << 23)) : (float)em * 0.001953125f;
  return (b & 0x80) ? -mag : mag;
}

template <>
__device__ __forceinline__ void load8<FS_KV_FP8_E4M3>(const uint8_t* p, float (&x)[8]) {
  const uint2 v = *reinterpret_cast<const uint2*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[i] = e4m3_to_f32((v.x >> (8 * i)) & 0xFF);
    x[4 + i] = e4m3_to_f32((v.y >> (8 * i)) & 0xFF);
  }
}

template <>
__device__ __forceinline__ void load8<FS_KV_INT8>(const uint8_t* p, float (&x)[8]) {
  const uint2 v = *reinterpret_cast<const uint2*>(p);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[i] = (float)(int8_t)((v.x >> (8 * i)) & 0xFF);
    x[4 + i] = (float)(int8_t)((v.y >> (8 * i)) & 0xFF);
  }
}

template <>
__device__ __forceinline__ void load8<FS_KV_INT4>(const uint8_t* p, float (&x)[8]) {
  const uint32_t v = *reinterpret_cast<const uint32_t*>(p);
#pragma unroll
  for (int i = 0; i < 8; ++i) x[i] = (float)((v >> (4 * i)) & 15u);
}

template <int DT>
struct Bits {
  static constexpr int value = DT == FS_KV_FP16 ? 16 : (DT == FS_KV_INT4 ? 4 : 8);
};

__device__ __forceinline__ float half_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }

// One work item for KV format DT, GP query heads at a time.  Decode: qrow == seq and len_override == 0.  Prefill
// (one query row of a chunk per item): q / out / lse are indexed by qrow, and the row attends to the first
// len_override tokens of sequence seq in one piece (no split).
template <int DT, int GP>
__device__ void process_item(const MultiArgs& A, int b, int seq, int chunk, int head, uint32_t item, float* smem,
                             int64_t qrow, int len_override) {
  const DevBatch& B = A.b[b];
  const DevGeom& g = B.g;
  const int D = g.D, T = g.T, G = B.G;
  const int lpt = D >> 3;               // lanes per token
  const int lig = threadIdx.x & (lpt - 1);
  const int grp = threadIdx.x / lpt;
  const int n_groups = kThreads / lpt;
  const int max_len = (int)min((int64_t)B.max_blocks * T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : (len > max_len ? max_len : len);
  if (len_override > 0) len = min(len, len_override);
  const int ct = chunk_tokens_of(B, seq);
  const int n_chunks = len_override > 0 ? 1 : (len + ct - 1) / ct;
  const int t0 = len_override > 0 ? 0 : chunk * ct;
  const int t1 = len_override > 0 ? len : min(len, t0 + ct);
  const int32_t* table = B.tables + (int64_t)seq * B.max_blocks;
  constexpr int kElemBytes8 = Bits<DT>::value;  // bytes of 8 elements
  const float k_static = DT == FS_KV_FP8_E4M3 ? B.k_scale[head] : 1.0f;
  const float v_static = DT == FS_KV_FP8_E4M3 ? B.v_scale[head] : 1.0f;
  const int red_stride = D + 2;

  // where this item's partial record goes (only used when the sequence is split)
  const uint64_t* part_off = reinterpret_cast<const uint64_t*>(A.header + kHdrPartOff);
  const uint64_t part_base =
      len_override > 0 ? 0 : part_off[b] + (uint64_t)item * (uint64_t)B.part_stride;  // item: index within the batch
  const bool part_ok = part_base + (uint64_t)B.part_stride <= A.part_capacity;
  if (n_chunks > 1 && !part_ok) {
    if (threadIdx.x == 0) atomicOr(A.header + kHdrStatus, 2u);
    return;
  }

  for (int g0 = 0; g0 < G; g0 += GP) {
    float qf[GP][8], acc[GP][8], m[GP], l[GP];
#pragma unroll
    for (int j = 0; j < GP; ++j) {
      m[j] = -INFINITY;
      l[j] = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        acc[j][i] = 0.f;
        qf[j][i] = 0.f;
      }
      if (g0 + j < G) {
        const _Float16* qp = B.q + (qrow * B.n_q + head * G + g0 + j) * D + lig * 8;
#pragma unroll
        for (int i = 0; i < 8; ++i) qf[j][i] = (float)qp[i];
      }
    }
    for (int t = t0 + grp; t < t1; t += n_groups) {
      const int bi = t / T;
      const int tib = t - bi * T;
      const uint8_t* chunkp = B.layer_base + (uint64_t)checked_block(table[bi], B.n_blocks, A.header) * g.block_budget + (uint64_t)head * g.head_chunk;
      float kf[8], vf[8];
      load8<DT>(chunkp + (uint64_t)tib * g.row_bytes + lig * kElemBytes8, kf);
      load8<DT>(chunkp + g.kv_tile + (uint64_t)tib * g.row_bytes + lig * kElemBytes8, vf);
      float ks = k_static, vs = v_static;
      if (DT == FS_KV_INT8) {
        const uint8_t* par = chunkp + 2u * g.kv_tile;
        ks = half_bits_to_f32(*reinterpret_cast<const uint16_t*>(par + 2 * tib));
        vs = half_bits_to_f32(*reinterpret_cast<const uint16_t*>(par + g.par_tile + 2 * tib));
      } else if (DT == FS_KV_INT4) {
        const uint8_t* par = chunkp + 2u * g.kv_tile;
        const uint32_t kp = *reinterpret_cast<const uint32_t*>(par + 4 * tib);
        const uint32_t vp = *reinterpret_cast<const uint32_t*>(par + g.par_tile + 4 * tib);
        ks = half_bits_to_f32((uint16_t)(kp & 0xFFFF));
        vs = half_bits_to_f32((uint16_t)(vp & 0xFFFF));
        const float kz = half_bits_to_f32((uint16_t)(kp >> 16)), vz = half_bits_to_f32((uint16_t)(vp >> 16));
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          kf[i] -= kz;
          vf[i] -= vz;
        }
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) vf[i] *= vs;
#pragma unroll
      for (int j = 0; j < GP; ++j) {
        float dot = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) dot = fmaf(qf[j][i], kf[i], dot);
        for (int o = lpt >> 1; o >= 1; o >>= 1) dot += __shfl_xor(dot, o, 64);
        const float s = dot * (B.sm_scale * ks);
        const float mn = fmaxf(m[j], s);
        const float corr = expf(m[j] - mn);
        const float pw = expf(s - mn);
        l[j] = l[j] * corr + pw;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[j][i] = fmaf(pw, vf[i], acc[j][i] * corr);
        m[j] = mn;
      }
    }
    // merge the groups of the workgroup through LDS
#pragma unroll
    for (int j = 0; j < GP; ++j) {
      float* r = smem + ((size_t)grp * GP + j) * red_stride;
#pragma unroll
      for (int i = 0; i < 8; ++i) r[lig * 8 + i] = acc[j][i];
      if (lig == 0) {
        r[D] = m[j];
        r[D + 1] = l[j];
      }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < GP * D; idx += kThreads) {
      const int j = idx / D, d = idx - j * D;
      if (g0 + j >= G) continue;
      float M = -INFINITY;
      for (int gi = 0; gi < n_groups; ++gi) M = fmaxf(M, smem[((size_t)gi * GP + j) * red_stride + D]);
      float L = 0.f, O = 0.f;
      for (int gi = 0; gi < n_groups; ++gi) {
        const float* r = smem + ((size_t)gi * GP + j) * red_stride;
        const float w = r[D] == -INFINITY ? 0.f : expf(r[D] - M);
        L += r[D + 1] * w;
        O += r[d] * w;
      }
      const int h = head * G + g0 + j;
      if (n_chunks == 1) {
        B.out[(qrow * B.n_q + h) * D + d] = (_Float16)(O / L);
        if (d == 0 && B.lse) B.lse[qrow * B.n_q + h] = M + logf(L);
      } else {
        float* pr = A.partials + part_base + (uint64_t)(g0 + j) * red_stride;
        pr[d] = O;
        if (d == 0) {
          pr[D] = M;
          pr[D + 1] = L;
        }
      }
    }
    __syncthreads();
  }
}

template <int DT>
__device__ __forceinline__ void dispatch_gp(const MultiArgs& A, int b, int seq, int chunk, int head, uint32_t item,
                                            float* smem, int64_t qrow, int len_override) {
  const int G = A.b[b].G;
  if (G == 1)
    process_item<DT, 1>(A, b, seq, chunk, head, item, smem, qrow, len_override);
  else if (G == 2)
    process_item<DT, 2>(A, b, seq, chunk, head, item, smem, qrow, len_override);
  else
    process_item<DT, 4>(A, b, seq, chunk, head, item, smem, qrow, len_override);
}

__device__ __forceinline__ void dispatch_dtype(const MultiArgs& A, int b, int seq, int chunk, int head, uint32_t item,
                                               float* smem, int64_t qrow, int len_override) {
  switch (A.b[b].g.dtype) {
    case FS_KV_FP16: dispatch_gp<FS_KV_FP16>(A, b, seq, chunk, head, item, smem, qrow, len_override); break;
    case FS_KV_FP8_E4M3: dispatch_gp<FS_KV_FP8_E4M3>(A, b, seq, chunk, head, item, smem, qrow, len_override); break;
    case FS_KV_INT8: dispatch_gp<FS_KV_INT8>(A, b, seq, chunk, head, item, smem, qrow, len_override); break;
    default: dispatch_gp<FS_KV_INT4>(A, b, seq, chunk, head, item, smem, qrow, len_override); break;
  }
}

__global__ __launch_bounds__(kThreads) void generic_attention_kernel(MultiArgs A) {
  extern __shared__ float smem[];
  __shared__ uint32_t s_item;
  const uint32_t total = A.header[kHdrTotalItems];
  for (;;) {
    if (threadIdx.x == 0) s_item = atomicAdd(A.header + kHdrCounter, 1u);
    __syncthreads();
    const uint32_t item = s_item;
    __syncthreads();
    if (item >= total) break;  // every wave of every workgroup reaches this once the queue is empty
    const int4 rec = A.item_list[2 * item];
    const int b = rec_batch(rec), seq = rec.y, chunk = rec.z, head = rec_head(rec);
    const uint32_t local = (uint32_t)rec.w;  // the item's index within its batch: where its partial record goes
    dispatch_dtype(A, b, seq, chunk, head, local, smem, seq, 0);
  }
}

// Prefill over any shape the library accepts (the MFMA prefill kernels cover head_dim 128 with at least 8 tokens
// per block): one workgroup per (query row, KV head), the decode work item with the row's causal length.  A.b[0]
// is the model's batch (q / out / lse hold the chunk rows), q_offsets the chunks' first rows.
__global__ __launch_bounds__(kThreads) void generic_prefill_kernel(MultiArgs A, const int32_t* q_offsets, int n_rows) {
  extern __shared__ float smem[];
  const DevBatch& B = A.b[0];
  const int H = B.g.H;
  const int max_len = (int)min((int64_t)B.max_blocks * B.g.T, (int64_t)0x7fffffff);
  for (int64_t work = blockIdx.x; work < (int64_t)n_rows * H; work += gridDim.x) {  // uniform over the workgroup
    const int row = (int)(work / H), head = (int)(work - (int64_t)row * H);
    int lo = 0, hi = B.n_seq - 1;
    while (lo < hi) {  // last sequence whose first row is <= row (sequences with empty chunks are passed over)
      const int mid = (lo + hi + 1) >> 1;
      if (q_offsets[mid] <= row) lo = mid;
      else hi = mid - 1;
    }
    int len = B.seq_lens[lo];
    len = len < 1 ? 1 : min(len, max_len);
    int n_new = q_offsets[lo + 1] - q_offsets[lo];
    n_new = n_new < 0 ? 0 : min(n_new, len);
    const int rr = row - q_offsets[lo];
    if (rr < 0 || rr >= n_new) continue;  // (inconsistent device offsets: the row is left unwritten, flagged by the prep kernel)
    dispatch_dtype(A, 0, lo, 0, head, 0u, smem, row, len - n_new + rr + 1);
  }
}

}  // namespace

hipError_t launch_generic_prefill(const MultiArgs& A, const int32_t* q_offsets, int n_rows, int n_workgroups, hipStream_t s) {
  const int D = A.b[0].g.D;
  if (D & (D - 1)) return hipErrorInvalidValue;
  const int gp = A.b[0].G == 1 ? 1 : (A.b[0].G == 2 ? 2 : 4);
  const size_t smem = (size_t)(kThreads / (D >> 3)) * gp * (D + 2) * sizeof(float);
  hipLaunchKernelGGL(generic_prefill_kernel, dim3(n_workgroups), dim3(kThreads), smem, s, A, q_offsets, n_rows);
  return hipGetLastError();
}

hipError_t launch_generic(const MultiArgs& A, int n_workgroups, hipStream_t s) {
  size_t smem = 0;
  for (int i = 0; i < A.n_batches; ++i) {
    const int D = A.b[i].g.D;
    if (D & (D - 1)) return hipErrorInvalidValue;  // lanes-per-token must be a power of two
    const int gp = A.b[i].G == 1 ? 1 : (A.b[i].G == 2 ? 2 : 4);
    const size_t need = (size_t)(kThreads / (D >> 3)) * gp * (D + 2) * sizeof(float);
    smem = need > smem ? need : smem;
  }
  hipLaunchKernelGGL(generic_attention_kernel, dim3(n_workgroups), dim3(kThreads), smem, s, A);
  return hipGetLastError();
}

}  // namespace fs
