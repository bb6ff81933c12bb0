// Device code of fs_kv_append: quantize new K/V rows and scatter them into slab blocks (shared by the append
// kernels and the decode step's front kernel, which appends and prepares the work list in one launch).
//
// FineServe Sec. 2.1: every new token appends its keys and values to the KV cache;
// Sec. 2.2 / 3.2: the cache may be FP16, FP8 or INT4 (here also INT8), with per-token
// quantization parameters stored inside the block.  The paper gives no quantizer
// arithmetic; the definitions implemented here are the ones stated in fineserve.h.
//
// A (token, KV head, K|V) row is handled by head_dim / 8 neighbouring lanes, eight elements each (a wave covers
// 4 rows at head_dim 128): 16-byte source loads, 16 / 8 / 8 / 4-byte stores for FP16 / FP8 / INT8 / INT4.  The
// row's extrema are reduced over its lanes with xor shuffles (max and min are exact in any order), and each lane
// stores its own bytes (INT4: a byte holds two codes of one lane, so no byte is shared between lanes or tokens).
// All arithmetic is IEEE fp32, round-to-nearest-even, correctly rounded division; every file that includes this
// header is compiled with floating-point contraction off so that the stored bytes are reproducible bit for bit.
#pragma once

#include "fs_internal.h"

namespace fs {
namespace append {


constexpr int kEpl = 8;    // elements per lane

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct AppendArgs {
  DevGeom g;
  uint8_t* pool;
  const void* k_new;
  const void* v_new;
  const int32_t* seq_idx;
  const int32_t* pos;
  const int32_t* tables;
  const float* k_scale;  // FP8: device [H] for this layer
  const float* v_scale;
  int64_t n_rows;        // rows of the launch: n_tokens rounded up to a multiple of 4, * H * 2
  int64_t n_tokens;
  int32_t lpr_shift;     // log2 of the lanes per row (head_dim / 8)
  int64_t n_blocks;      // valid block ids are [0, n_blocks)
  int32_t layer, max_blocks;
  int32_t src_f32;       // source rows are fp32 (else fp16)
  int32_t pad;
};

// Several appends in one launch: append i is worked on by the workgroups first_block[i] .. first_block[i + 1] - 1.
constexpr int kMaxAppends = 8;
struct MultiAppendArgs {
  AppendArgs a[kMaxAppends];
  uint32_t first_block[kMaxAppends + 1];
  int32_t n;
};

// max / min over the lanes of a row (lpr neighbouring lanes, lpr a power of two)
__device__ __forceinline__ float row_max(float v, int lpr) {
  for (int o = lpr >> 1; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float row_min(float v, int lpr) {
  for (int o = lpr >> 1; o >= 1; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
  return v;
}

__device__ __forceinline__ uint16_t f16_bits(float x) {
  _Float16 h = (_Float16)x;  // round-to-nearest-even
  return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float f16_value(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }

// fp16 scale of the integer quantizers: nearest fp16, saturating, 1.0 when it rounds to zero.
__device__ __forceinline__ uint16_t scale_bits(float s32) {
  uint16_t b = f16_bits(s32);
  if ((b & 0x7FFF) >= 0x7C00) b = 0x7BFF;
  if ((b & 0x7FFF) == 0) b = 0x3C00;
  return b;
}

// Nearest OCP E4M3 code, ties to even, saturating at +-448, sign of the input kept.
__device__ __forceinline__ uint32_t e4m3_bits(float y) {
  const uint32_t fb = __float_as_uint(y);
  const uint32_t sign = (fb >> 24) & 0x80u;
  const float a = fabsf(y);
  uint32_t code;
  if (!(a < 448.0f)) {
    code = 0x7E;
  } else if (a < 0.015625f) {  // below 2^-6: subnormal codes, spacing 2^-9
    code = (uint32_t)rintf(a * 512.0f);
  } else {
    const uint32_t ab = fb & 0x7FFFFFFFu;
    const uint32_t e = ab >> 23;           // biased fp32 exponent, >= 121 here
    uint32_t m3 = (ab >> 20) & 7u;
    const uint32_t rest = ab & 0xFFFFFu;
    code = ((e - 120u) << 3) + m3;         // E4M3 bias 7: exponent field = e - 127 + 7
    if (rest > 0x80000u || (rest == 0x80000u && (code & 1u))) code += 1;  // carry runs into the exponent
  }
  return sign | code;
}

// n / d for many n and one d.  The correctly rounded fp32 division is a reciprocal estimate, one Newton step on
// it, and a quotient with two residual corrections, all in fused multiply-adds; the first half depends on d
// alone and is done once per row here.  What is left out is the operand scaling of the general sequence, which
// only matters near the ends of the exponent range: d must be a normal number of moderate size (the fp16-valued
// scales of the integer formats: 2^-24 .. 65504) and n / d must stay finite (|n| <= the row's extremum, so the
// quotient is bounded by the format's range unless the scale saturated, and then by 2^128 / 65504).  Within that
// domain the result is the division's, bit for bit; a quotient in the subnormal range may differ in its last bits,
// where every value rounds to the integer 0 anyway.
struct Divisor {
  float d, r;
  __device__ __forceinline__ explicit Divisor(float d_) : d(d_) {
    const float r0 = __builtin_amdgcn_rcpf(d);
    const float e = __builtin_fmaf(-d, r0, 1.0f);
    r = __builtin_fmaf(e, r0, r0);
  }
  __device__ __forceinline__ float operator()(float n) const {
    float q = n * r;
    const float e1 = __builtin_fmaf(-d, q, n);
    q = __builtin_fmaf(e1, r, q);
    const float e2 = __builtin_fmaf(-d, q, n);
    return __builtin_fmaf(e2, r, q);
  }
};

// Source rows are read once and KV bytes written once per append: both carry the non-temporal hint.  Measured on the
// bulk append of a prefill chunk (kernel trace, one box, libraries alternating): FP16 rows 213-225 -> 205 us
// (1.15 GB), fp32 -> INT4 1.07-1.09 -> 1.06 ms (10.4 GB); the loads' hint gives most of it.
#ifndef FS_NT_APPEND_LOAD
#define FS_NT_APPEND_LOAD 1
#endif
#ifndef FS_NT_APPEND_STORE
#define FS_NT_APPEND_STORE 1
#endif
template <typename T>
__device__ __forceinline__ T src_load(const T* p) {
#if FS_NT_APPEND_LOAD
  return __builtin_nontemporal_load(p);
#else
  return *p;
#endif
}
template <typename T>
__device__ __forceinline__ void kv_store(T* p, T v) {
#if FS_NT_APPEND_STORE
  __builtin_nontemporal_store(v, p);
#else
  *p = v;
#endif
}

// the lane's eight source elements, widened exactly
template <bool kSrcF32>
__device__ __forceinline__ void load8(const void* src, int64_t idx, float (&x)[kEpl]) {
  if (kSrcF32) {
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 a = src_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(src) + idx));
    const f32x4 b = src_load(reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(src) + idx + 4));
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3];
    x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  } else {
    const u32x4 v = src_load(reinterpret_cast<const u32x4*>(reinterpret_cast<const uint16_t*>(src) + idx));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      x[2 * q] = f16_value((uint16_t)(v[q] & 0xFFFF));
      x[2 * q + 1] = f16_value((uint16_t)(v[q] >> 16));
    }
  }
}

// The rows of one append, dealt to n_workers waves; this wave is number `worker`.
template <bool kSrcF32>
__device__ __forceinline__ void append_rows(const AppendArgs& A, int64_t worker, int64_t n_workers) {
  const int lane = threadIdx.x & 63;
  const DevGeom& g = A.g;
  const int D = g.D;
  const int lpr = 1 << A.lpr_shift;           // lanes per row
  const int rpw = 64 >> A.lpr_shift;          // rows per wave
  const int lir = lane & (lpr - 1);           // lane within its row
  const int riw = lane >> A.lpr_shift;        // row within the wave
  const int64_t n_groups = (A.n_rows + rpw - 1) / rpw;
  for (int64_t grp = worker; grp < n_groups; grp += n_workers) {
    const int64_t r = grp * rpw + riw;
    // Lanes of a row agree on every test below; a row that is skipped computes on zeros and stores nothing, so
    // the shuffles stay unconditional.
    // Row order: four consecutive tokens of one (head, K|V) are neighbours, then K|V, the heads, the next four
    // tokens.  The rows a wave writes then lie side by side in the block whenever the tokens are consecutive
    // positions of one sequence (a prefill chunk): 256 contiguous bytes even for INT4's 64-byte rows, and the
    // source rows of a group of waves stay within four tokens.
    const int64_t rest = r >> 2;
    const int which = (int)(rest & 1);
    const int64_t th = rest >> 1;
    const int head = (int)(th % g.H);
    int64_t tok = (th / g.H) * 4 + (r & 3);
    bool ok = r < A.n_rows && tok < A.n_tokens;
    tok = ok ? tok : 0;
    const int p = ok ? A.pos[tok] : -1;
    const int s = ok ? A.seq_idx[tok] : -1;
    ok = ok && p >= 0 && s >= 0;
    const int bi = ok ? p / g.T : 0;
    ok = ok && bi < A.max_blocks;
    const int tib = p - bi * g.T;
    const int32_t blk = ok ? A.tables[(int64_t)s * A.max_blocks + bi] : -1;
    ok = ok && blk >= 0 && blk < A.n_blocks;  // never write outside the pool
    uint8_t* chunk = A.pool + (uint64_t)(ok ? blk : 0) * g.block_budget + (uint64_t)A.layer * g.layer_bytes +
                     (uint64_t)head * g.head_chunk;
    uint8_t* row = chunk + (which ? g.kv_tile : 0u) + (uint64_t)(ok ? tib : 0) * g.row_bytes;
    uint8_t* par = chunk + 2u * g.kv_tile + (which ? g.par_tile : 0u) + (uint64_t)(ok ? tib : 0) * (uint32_t)g.param_bytes;
    const void* src = which ? A.v_new : A.k_new;
    const int d0 = lir * kEpl;                // this lane's first element (head_dim >= 8: always inside the row)

    float x[kEpl];
#pragma unroll
    for (int q = 0; q < kEpl; ++q) x[q] = 0.f;
    if (ok) load8<kSrcF32>(src, (tok * g.H + head) * (int64_t)D + d0, x);

    if (g.dtype == FS_KV_FP16) {
      u32x4 w;
#pragma unroll
      for (int q = 0; q < 4; ++q) w[q] = (uint32_t)f16_bits(x[2 * q]) | ((uint32_t)f16_bits(x[2 * q + 1]) << 16);
      if (ok) kv_store(reinterpret_cast<u32x4*>(row + 2 * d0), w);
    } else if (g.dtype == FS_KV_FP8_E4M3) {
      const float sc = (which ? A.v_scale : A.k_scale)[head];
      u32x2 w = {0u, 0u};
#pragma unroll
      for (int q = 0; q < kEpl; ++q) w[q >> 2] |= e4m3_bits(__fdiv_rn(x[q], sc)) << (8 * (q & 3));
      if (ok) kv_store(reinterpret_cast<u32x2*>(row + d0), w);
    } else if (g.dtype == FS_KV_INT8) {
      float amax = 0.f;
#pragma unroll
      for (int q = 0; q < kEpl; ++q) amax = fmaxf(amax, fabsf(x[q]));
      amax = row_max(amax, lpr);
      const uint16_t sb = scale_bits(__fdiv_rn(amax, 127.0f));
      const float sf = f16_value(sb);
      const Divisor by_scale(sf);
      u32x2 w = {0u, 0u};
#pragma unroll
      for (int q = 0; q < kEpl; ++q) {
        const float c = fminf(fmaxf(rintf(by_scale(x[q])), -127.f), 127.f);
        w[q >> 2] |= ((uint32_t)(int)c & 0xFF) << (8 * (q & 3));
      }
      if (ok) {
        kv_store(reinterpret_cast<u32x2*>(row + d0), w);
        if (lir == 0) *reinterpret_cast<uint16_t*>(par) = sb;
      }
    } else {  // FS_KV_INT4
      float lo = 0.f, hi = 0.f;
#pragma unroll
      for (int q = 0; q < kEpl; ++q) {
        lo = fminf(lo, x[q]);
        hi = fmaxf(hi, x[q]);
      }
      lo = row_min(lo, lpr);
      hi = row_max(hi, lpr);
      const uint16_t sb = scale_bits(__fdiv_rn(hi - lo, 15.0f));
      const float sf = f16_value(sb);
      const Divisor by_scale(sf);
      const float z = fminf(fmaxf(rintf(by_scale(-lo)), 0.f), 15.f);
      uint32_t w = 0;
#pragma unroll
      for (int q = 0; q < kEpl; ++q) {
        const float c = fminf(fmaxf(rintf(by_scale(x[q])) + z, 0.f), 15.f);
        w |= (uint32_t)c << (4 * q);  // element 2j in the low nibble of byte j
      }
      if (ok) {
        kv_store(reinterpret_cast<uint32_t*>(row + (d0 >> 1)), w);
        if (lir == 0) *reinterpret_cast<uint32_t*>(par) = (uint32_t)sb | ((uint32_t)f16_bits(z) << 16);
      }
    }
  }
}

// The workgroup's share of a multi-append launch: `block` = its index among the launch's append workgroups,
// `waves` = waves per workgroup.
__device__ __forceinline__ void append_block(const MultiAppendArgs& P, uint32_t block, int waves) {
  int i = 0;
  while (i + 1 < P.n && block >= P.first_block[i + 1]) ++i;
  const AppendArgs& A = P.a[i];
  const int wave = threadIdx.x >> 6;
  const int64_t worker = (int64_t)(block - P.first_block[i]) * waves + wave;
  const int64_t n_workers = (int64_t)(P.first_block[i + 1] - P.first_block[i]) * waves;
  if (A.src_f32) append_rows<true>(A, worker, n_workers);
  else append_rows<false>(A, worker, n_workers);
}

}  // namespace append

// Host side (fs_append.hip): validates one append and fills its kernel arguments; sizes a multi-append launch for
// workgroups of `waves` waves (first_block, n; returns the number of workgroups).
int make_append_args(fs_pool* p, const fs_append_t& a, append::AppendArgs& out);
uint32_t plan_append_blocks(const fs_pool* p, append::MultiAppendArgs& P, int waves);

}  // namespace fs
