// MFMA tile machinery of the paged attention kernels for gfx950 (all four KV formats; head_dim HD = 64, 128 or 256,
// a template parameter that defaults to 128): shared by the split-K decode kernel and the prefill kernel.
//
// FineServe Sec. 2.1 / 2.3 / 5.1: attention reaches the KV cache through each model's own block table over
// the shared slab pool.  K/V rows stream straight from the slabs into registers (no LDS staging: every byte
// is used by exactly one lane), are dequantized in registers and feed v_mfma_f32_16x16x32_f16 for both
// contractions; the second matrix dimension is 16 logit columns: in decode the grouped query heads of a KV
// head (padded to 16), in prefill 16 (query token, query head) pairs.
//
// One 32-token tile (base token tb), lane l = 16*j + c:
//   S^T = K Q^T as two 16x16 MFMA tiles u = 0,1 (rows = tokens, columns = logit columns, "heads" below).  Row m of tile u
//   is token tb + 8*(m/4) + 4*u + (m%4), so that lane (j, c) ends up with the logits of head c for the
//   8 consecutive tokens tb + 8j .. tb + 8j + 7  (C layout: rows 4j..4j+3 of each tile).
//   Those 8 values, exponentiated and packed to fp16, are exactly the A operand (k index = token) of
//   out = P V; the B operand needs, per lane, the 8 tokens of its run for one d column, which is an
//   in-register 8x8 transpose (v_perm_b32) of the 8 row fragments the lane loaded.
//   K is loaded as the A operand of S^T: lane (j, c) reads 16 bytes of the row of token
//   tb + 8*(c/4) + 4u + (c%4); the d order inside a k-step is whatever the format's unpacking yields,
//   and the Q operand is pre-arranged once per item in the same order.
//   The head dimension decides the counts only: HD / 32 k-steps for S^T, HD / 16 output columns per lane (one
//   16x16 accumulator tile each), HD / 16 elements of every V row per lane.
//
// Dequantization is folded around the MFMAs: FP8 static scales and INT8/INT4 per-token K scales
// multiply the logits, per-token V scales multiply P; integer codes enter the MFMA unconverted, as fp16
// subnormals, and their offsets (128 for INT8, the zero-point for INT4) come back as rank-1
// corrections (z_k * sum(q) on the logits, sum_t p_t s_t z_t on the output).
#pragma once

#include <algorithm>
#include <utility>

#include "fs_attention.h"

namespace fs {
namespace {


typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#define FS_GLOBAL __attribute__((address_space(1)))
typedef const FS_GLOBAL uint8_t* gptr;  // global (not flat) address

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kD = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int DT, int HD = 128>
struct Fmt {
  static_assert(HD == 64 || HD == 128 || HD == 256, "head_dim of the MFMA kernels");
  static constexpr int kBits = DT == FS_KV_FP16 ? 16 : (DT == FS_KV_INT4 ? 4 : 8);
  static constexpr int kRowBytes = HD * kBits / 8;
  // K rows: the four lanes j of a row take kKLane bytes each per load (16, or 8 where the row has only 32 bytes)
  static constexpr int kKLane = kRowBytes / 4 < 16 ? kRowBytes / 4 : 16;
  static constexpr int kKLoads = kRowBytes / (4 * kKLane);
  static constexpr int kSteps = HD / 32;  // k-steps of S^T
  static constexpr int kNE = HD / 16;     // output columns (accumulator tiles) per lane
  // V rows: the sixteen lanes c of a row take kVBytes each (kNE elements)
  static constexpr int kVBytes = kRowBytes / 16;
  static constexpr int kVWords = kVBytes < 4 ? 1 : kVBytes / 4;
  // packed-fp16 registers one lane's share of a V row unpacks to (INT4: four per word, see int4x8)
  static constexpr int kVRegs = DT == FS_KV_INT4 ? 4 * kVWords : kNE / 2;
  static constexpr int kParBytes = DT == FS_KV_INT8 ? 2 : (DT == FS_KV_INT4 ? 4 : 0);
  static constexpr int kRing = ring_tiles(DT, HD);
};

template <int BYTES>
struct KVec {
  typedef u32x4 type;
};
template <>
struct KVec<8> {
  typedef u32x2 type;
};

// K/V bytes are read once per launch: FS_NT_K / FS_NT_V (0 or 1) select loads with the non-temporal hint.
// Measured on the four-model pool: the hint helps loads that cover whole 128-byte lines per instruction (the V
// rows: + 1.2 % on the kernel) and costs where an instruction takes half a line of each of 16 rows (the K operand
// pattern: - 0.3 %, and - 2.5 % with both), so V rows carry it and K rows do not.
#ifndef FS_NT_K
#define FS_NT_K 0
#endif
#ifndef FS_NT_V
#define FS_NT_V 1
#endif
template <bool NT, typename T>
__device__ __forceinline__ T stream_load(const FS_GLOBAL T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}

__device__ __forceinline__ uint32_t h2u(half2v h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ half2v u2h(uint32_t u) { return __builtin_bit_cast(half2v, u); }
__device__ __forceinline__ float f16lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFF)); }
__device__ __forceinline__ float f16hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }

// ---- 8 stored elements -> 4 registers of packed fp16 -----------------------------------------
// FP16 and FP8 convert to their exact fp16 values, register p holding elements (2p, 2p+1).
// The integer formats are not converted at all: a small integer n placed in the low mantissa bits of a
// zero-exponent half IS the fp16 subnormal n * 2^-24, which the MFMA consumes exactly; the common
// factor 2^24 is applied in fp32 afterwards.
//   INT8: byte b ^ 0x80 = b + 128 (unsigned) -> halves (u0, u1), (u2, u3) by v_perm_b32; the offset 128
//         comes back as a rank-1 correction (128 * sum(q) on the logits, 128 * sum(p') on the output).
//   INT4: w & 0x000F000F = codes (0, 4); w & 0x00F000F0 = 16 * codes (1, 5); the same on w >> 8 for
//         (2, 6) and 16 * (3, 7).  Register p thus holds codes (p, p + 4), odd p scaled by 16: the query
//         operand carries 1/16 at those positions, the output columns are rescaled at the end.

// two E4M3 bytes of a dword -> packed fp16 (exact)
__device__ __forceinline__ uint32_t fp8x2_lo(uint32_t w) { return h2u(__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false)); }
__device__ __forceinline__ uint32_t fp8x2_hi(uint32_t w) { return h2u(__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true)); }

__device__ __forceinline__ void int8x4(uint32_t w, uint32_t& r0, uint32_t& r1) {
  const uint32_t u = w ^ 0x80808080u;
  r0 = __builtin_amdgcn_perm(0u, u, 0x0C010C00u);  // selector 0x0C yields a zero byte
  r1 = __builtin_amdgcn_perm(0u, u, 0x0C030C02u);
}

__device__ __forceinline__ void int4x8(uint32_t w, uint32_t (&r)[4]) {
  const uint32_t w8 = w >> 8;
  r[0] = w & 0x000F000Fu;
  r[1] = w & 0x00F000F0u;
  r[2] = w8 & 0x000F000Fu;
  r[3] = w8 & 0x00F000F0u;
}

constexpr float kTwo24 = 16777216.0f;
constexpr float kTwo20 = 1048576.0f;
constexpr float kTau = 3.0f;  // log2 of the largest softmax weight tolerated before the reference is moved

// GP = padded group size: 4 when the KV head serves at most 4 query heads, else 16.  The MFMAs always work on 16
// head columns; GP decides how the softmax between them is spread over the lanes (see softmax_pv).
template <int DT, int GP, int HD = 128>
struct Tile {
  typename KVec<Fmt<DT, HD>::kKLane>::type k[2][Fmt<DT, HD>::kKLoads];
  uint32_t v[8][Fmt<DT, HD>::kVWords];
  // INT8/INT4 per-token parameters.  GP == 16: one register; lanes c < 8 hold the K parameters of token c of
  // the lane's run, lanes c >= 8 the V ones.  GP == 4: those of the lane's own two tokens, K K V V.
  uint32_t par[GP == 16 ? 1 : 4];
};

// Run vr of an item (run_geom, fs_attention.h) with the head-chunk address of its block.
struct RunLoc {
  gptr base;
  int start, lo, hi, hi_u;
  int tok0;  // token index of the run's slot 0 (a huge value for a run past the item's end: no column reaches it)
};

__device__ __forceinline__ RunLoc locate(const ItemCtx& X, int vr) {
  const RunGeom r = run_geom(X, vr);
  RunLoc L;
  L.start = r.start;
  L.lo = r.lo;
  L.tok0 = r.tok0;
  L.hi = r.hi;
  L.hi_u = r.hi_u;
  L.base = (gptr)X.chunk_ptr[r.k_rel];
  return L;
}

template <int DT, int GP, int HD>
__device__ __forceinline__ void issue_k(const ItemCtx& X, int vb, int j, int c, Tile<DT, GP, HD>& t) {
  using F = Fmt<DT, HD>;
  typedef typename KVec<F::kKLane>::type kvec;
  // row m = c of S^T tile u is slot 4u + (c & 3) of run c >> 2
  const RunLoc L = locate(X, vb + (c >> 2));
  const gptr p = L.base + (uint32_t)((L.start + (c & 3)) * F::kRowBytes) + F::kKLane * j;
#pragma unroll
  for (int u = 0; u < 2; ++u)
#pragma unroll
    for (int s = 0; s < F::kKLoads; ++s)
      t.k[u][s] = stream_load<FS_NT_K>(reinterpret_cast<const FS_GLOBAL kvec*>(p + u * 4 * F::kRowBytes + 4 * F::kKLane * s));
}

template <int DT, int HD>
__device__ __forceinline__ void load_v_row(gptr p, uint32_t (&v)[Fmt<DT, HD>::kVWords]) {
  constexpr int kVBytes = Fmt<DT, HD>::kVBytes;
  if constexpr (kVBytes == 32) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const u32x4 x = stream_load<FS_NT_V>(reinterpret_cast<const FS_GLOBAL u32x4*>(p) + h);
      v[4 * h + 0] = x[0];
      v[4 * h + 1] = x[1];
      v[4 * h + 2] = x[2];
      v[4 * h + 3] = x[3];
    }
  } else if constexpr (kVBytes == 16) {
    const u32x4 x = stream_load<FS_NT_V>(reinterpret_cast<const FS_GLOBAL u32x4*>(p));
    v[0] = x[0];
    v[1] = x[1];
    v[2] = x[2];
    v[3] = x[3];
  } else if constexpr (kVBytes == 8) {
    const u32x2 x = stream_load<FS_NT_V>(reinterpret_cast<const FS_GLOBAL u32x2*>(p));
    v[0] = x[0];
    v[1] = x[1];
  } else if constexpr (kVBytes == 4) {
    v[0] = stream_load<FS_NT_V>(reinterpret_cast<const FS_GLOBAL uint32_t*>(p));
  } else {
    v[0] = stream_load<FS_NT_V>(reinterpret_cast<const FS_GLOBAL uint16_t*>(p));
  }
}

template <int DT, int GP, int HD>
__device__ __forceinline__ void issue_v(const ItemCtx& X, const DevGeom& g, int vb, int j, int c, Tile<DT, GP, HD>& t) {
  using F = Fmt<DT, HD>;
  const RunLoc L = locate(X, vb + j);
  if constexpr (F::kParBytes != 0) {  // parameters first: the softmax needs them before the V rows
    const gptr pk = L.base + 2u * g.kv_tile;
    if constexpr (GP == 16) {
      const gptr p = pk + ((c >> 3) ? g.par_tile : 0u) + (uint32_t)((L.start + (c & 7)) * F::kParBytes);
      if constexpr (F::kParBytes == 2) t.par[0] = *reinterpret_cast<const FS_GLOBAL uint16_t*>(p);
      else t.par[0] = *reinterpret_cast<const FS_GLOBAL uint32_t*>(p);
    } else {
      const gptr p = pk + (uint32_t)((L.start + 2 * (c >> 2)) * F::kParBytes);  // slots 2 (c >> 2), + 1 of the run
      const gptr q = p + g.par_tile;
      if constexpr (F::kParBytes == 2) {
        t.par[0] = *reinterpret_cast<const FS_GLOBAL uint16_t*>(p);
        t.par[1] = *reinterpret_cast<const FS_GLOBAL uint16_t*>(p + 2);
        t.par[2] = *reinterpret_cast<const FS_GLOBAL uint16_t*>(q);
        t.par[3] = *reinterpret_cast<const FS_GLOBAL uint16_t*>(q + 2);
      } else {
        t.par[0] = *reinterpret_cast<const FS_GLOBAL uint32_t*>(p);
        t.par[1] = *reinterpret_cast<const FS_GLOBAL uint32_t*>(p + 4);
        t.par[2] = *reinterpret_cast<const FS_GLOBAL uint32_t*>(q);
        t.par[3] = *reinterpret_cast<const FS_GLOBAL uint32_t*>(q + 4);
      }
    }
  }
  const gptr p0 = L.base + g.kv_tile + (uint32_t)(L.start * F::kRowBytes) + c * F::kVBytes;
#pragma unroll
  for (int i = 0; i < 8; ++i) load_v_row<DT, HD>(p0 + i * F::kRowBytes, t.v[i]);
}

// The Q operand (B of S^T = K Q^T) of lane (j, c) for k-step ks: 8 halves of q[head c] in the d order
// (and with the per-position factors) that the format's K unpacking produces.  qsum = sum_d q[d].
// ODD16 (INT4): the K operand holds its odd code positions 16-fold, the query carries 1/16 there.  Without it the
// query keeps its values (a K operand that was dequantized on the way holds plain values at every position).
template <int DT, bool ODD16 = true, int HD = 128>
__device__ __forceinline__ void load_q(const _Float16* qrow, bool live, int j, u32x4 (&qb)[HD / 32], float& qsum) {
  qsum = 0.f;
  constexpr int W = Fmt<DT, HD>::kKLane / 4;  // dwords (k-steps, for INT4) one lane takes of a K row per load
#pragma unroll
  for (int ks = 0; ks < HD / 32; ++ks) {
    int d0;
    if (DT == FS_KV_FP16) d0 = 32 * ks + 8 * j;
    else if (DT == FS_KV_INT4) d0 = 32 * W * (ks / W) + 8 * W * j + 8 * (ks % W);
    else d0 = 64 * (ks >> 1) + 16 * j + 8 * (ks & 1);
    u32x4 x = {0u, 0u, 0u, 0u};
    if (live) x = *reinterpret_cast<const u32x4*>(qrow + d0);
#pragma unroll
    for (int p = 0; p < 4; ++p) qsum += f16lo(x[p]) + f16hi(x[p]);
    if (DT == FS_KV_INT4) {
      const half2v s16 = {(_Float16)0.0625f, (_Float16)0.0625f};
      u32x4 y;
      y[0] = __builtin_amdgcn_perm(x[2], x[0], 0x05040100u);  // q0, q4
      y[1] = __builtin_amdgcn_perm(x[2], x[0], 0x07060302u);  // q1, q5
      y[2] = __builtin_amdgcn_perm(x[3], x[1], 0x05040100u);  // q2, q6
      y[3] = __builtin_amdgcn_perm(x[3], x[1], 0x07060302u);  // q3, q7
      if (ODD16) {  // (q1, q5) / 16, (q3, q7) / 16
        y[1] = h2u(u2h(y[1]) * s16);
        y[3] = h2u(u2h(y[3]) * s16);
      }
      x = y;
    }
    qb[ks] = x;
  }
}

__device__ __forceinline__ float4v mfma(u32x4 a, u32x4 b, float4v acc) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), acc, 0, 0, 0);
}

// K fragments of one 16-token tile -> the A operands of S^T, one per k-step.
template <int DT, int HD = 128>
__device__ __forceinline__ void k_operands(const typename KVec<Fmt<DT, HD>::kKLane>::type (&k)[Fmt<DT, HD>::kKLoads],
                                           u32x4 (&a)[HD / 32]) {
  constexpr int KS = HD / 32;
  if constexpr (DT == FS_KV_FP16) {
#pragma unroll
    for (int s = 0; s < KS; ++s) a[s] = k[s];
  } else if constexpr (DT == FS_KV_FP8_E4M3) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const u32x4 x = k[ks >> 1];
      const uint32_t w0 = x[2 * (ks & 1)], w1 = x[2 * (ks & 1) + 1];
      a[ks][0] = fp8x2_lo(w0);
      a[ks][1] = fp8x2_hi(w0);
      a[ks][2] = fp8x2_lo(w1);
      a[ks][3] = fp8x2_hi(w1);
    }
  } else if constexpr (DT == FS_KV_INT8) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const u32x4 x = k[ks >> 1];
      uint32_t r0, r1, r2, r3;
      int8x4(x[2 * (ks & 1)], r0, r1);
      int8x4(x[2 * (ks & 1) + 1], r2, r3);
      a[ks][0] = r0;
      a[ks][1] = r1;
      a[ks][2] = r2;
      a[ks][3] = r3;
    }
  } else {
    constexpr int W = Fmt<DT, HD>::kKLane / 4;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint32_t r[4];
      int4x8(k[ks / W][ks % W], r);
      a[ks][0] = r[0];
      a[ks][1] = r[1];
      a[ks][2] = r[2];
      a[ks][3] = r[3];
    }
  }
}

// One lane's elements of a V row -> packed-fp16 registers (layout note above).
template <int DT, int HD = 128>
__device__ __forceinline__ void v_unpack(const uint32_t (&v)[Fmt<DT, HD>::kVWords], uint32_t (&x)[Fmt<DT, HD>::kVRegs]) {
  using F = Fmt<DT, HD>;
  if constexpr (DT == FS_KV_FP16) {
#pragma unroll
    for (int p = 0; p < F::kVRegs; ++p) x[p] = v[p];
  } else if constexpr (DT == FS_KV_FP8_E4M3) {
#pragma unroll
    for (int w = 0; w < F::kVWords; ++w) {
      x[2 * w] = fp8x2_lo(v[w]);
      x[2 * w + 1] = fp8x2_hi(v[w]);
    }
  } else if constexpr (DT == FS_KV_INT8) {
#pragma unroll
    for (int w = 0; w < F::kVWords; ++w) int8x4(v[w], x[2 * w], x[2 * w + 1]);
  } else {
#pragma unroll
    for (int w = 0; w < F::kVWords; ++w) {
      uint32_t r[4];
      int4x8(v[w], r);  // (a 16-bit share, head_dim 64: the high halves are zero and never selected)
#pragma unroll
      for (int q = 0; q < 4; ++q) x[4 * w + q] = r[q];
    }
  }
}

// value of lane I of the own 16-lane row, broadcast to the whole row (DPP row_newbcast)
template <int I>
__device__ __forceinline__ float row_bcast(float x) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(0u, __float_as_uint(x), 0x150 + I, 0xF, 0xF, false));
}

template <int... Is, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, Is...>, F&& f) {
  (f(std::integral_constant<int, Is>{}), ...);
}

// Per-wave online-softmax state.  acc[e] is the 16x16 output tile of d columns {kNE c' + e}: lane (j', c')
// holds rows (heads) 4j'..4j'+3.  m, l, zc belong to the head whose logits the lane exponentiates (see
// softmax_pv): m is the same in all lanes of a head, l and zc are the lane's share.
template <int HD>
struct StateT {
  float4v acc[HD / 16];
  float m;   // reference subtracted from the logits (base-2 domain): within kTau of the running max
  float l;   // this lane's share of the running sum
  float zc;  // INT8/INT4: this lane's share of the zero-point term  -sum_t p_t s_t z_t
};
typedef StateT<128> State;

// S^T = K Q^T for the 32 tokens of the tile: s[u][r] = raw logit of head c, slot 4u + r of run j.
template <int DT, int GP, int HD>
__device__ __forceinline__ void qk_tile(const Tile<DT, GP, HD>& t, const u32x4 (&qb)[HD / 32], float4v (&s)[2]) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    u32x4 a[HD / 32];
    k_operands<DT, HD>(t.k[u], a);
    float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < HD / 32; ++ks) acc = mfma(a[ks], qb[ks], acc);
    s[u] = acc;
  }
}

// lanes of the banks in BANKS take src from the lane SHIFT places to their right in the 16-lane row
// (DPP row_shr), the others keep old
template <int SHIFT, int BANKS>
__device__ __forceinline__ float take_shr(float old, float src) {
  return __uint_as_float(__builtin_amdgcn_update_dpp(__float_as_uint(old), __float_as_uint(src), 0x110 + SHIFT, 0xF, BANKS, false));
}
// value of the lane SHIFT places to the left in the row (DPP row_shl), 0 where the row ends
template <int SHIFT>
__device__ __forceinline__ uint32_t from_shl(uint32_t src) {
  return __builtin_amdgcn_update_dpp(0u, src, 0x100 + SHIFT, 0xF, 0xF, true);
}

// Moves the reference of the lazy online softmax: called when some logit of the tile exceeds its head's
// reference by more than kTau (always on the first tile, where m = -inf).  tmax = largest logit among this
// lane's tokens; the lanes of a head are those with equal c % GP.
template <int DT, int GP, int HD>
__device__ __forceinline__ void move_reference(StateT<HD>& st, float tmax, int j) {
  if constexpr (GP == 4) {
    tmax = fmaxf(tmax, __shfl_xor(tmax, 4, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 8, 64));
  }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
  const float m_new = fmaxf(st.m, tmax);  // finite: the tile's first run holds a token of the item
  const float corr = __builtin_amdgcn_exp2f(st.m - m_new);
  st.l *= corr;
  if constexpr (Fmt<DT>::kParBytes != 0) st.zc *= corr;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float cr = __shfl(corr, (4 * j + r) % GP, 64);  // head h keeps its factor in lane c = h
#pragma unroll
    for (int e = 0; e < HD / 16; ++e) st.acc[e][r] *= cr;
  }
  st.m = m_new;
}

// Online softmax over the tile and out += P V.
//
// The lazy running reference: the softmax is invariant to the value subtracted from the logits, so the
// reference m only has to stay within 2^kTau of the largest logit seen (P stays <= 2^kTau, far inside fp16).
//
// GP == 16: lane (j, c) exponentiates the 8 logits of head c it holds after S^T; its packed P is directly the A
// operand of P V.  Per-token parameters reach it by DPP broadcast from the lanes that loaded them.
// GP == 4: only head columns 0..3 are real, so 12 of 16 lanes would exponentiate padding.  Instead lane
// (j, c) takes head c % 4 and slots 2 (c / 4), + 1 of run j: it fetches those two logits from lane (j, c % 4)
// (DPP row shifts), loads the parameters of its own two tokens itself, and hands its packed pair of P back to
// lanes c < 4 (DPP again), which assemble the A operand.  A quarter of the exponentials, no broadcasts.
template <int DT, int GP, int HD>
__device__ __forceinline__ void softmax_pv(const ItemCtx& X, Tile<DT, GP, HD>& t, const float4v (&s)[2], int vb, int j, int c,
                                           float qsum, float alpha, StateT<HD>& st) {
  using F = Fmt<DT, HD>;
  const RunLoc L = locate(X, vb + j);
  const uint32_t n_ok = (uint32_t)max(L.hi - L.lo, 0);   // slot i of the run is live iff (unsigned)(i - lo) < n_ok
  const bool partial = !__all(L.lo == 0 && L.hi == 8);   // wave-uniform
  if (partial) {
    if constexpr (DT == FS_KV_FP16 || DT == FS_KV_FP8_E4M3) {
      // slots past the sequence's end may hold NaN/Inf bit patterns; 0 * NaN would poison the MFMA
      // (slots before lo repeat live tokens: finite, their weight is 0)
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int w = 0; w < F::kVWords; ++w) t.v[i][w] = i < L.hi_u ? t.v[i][w] : 0u;
    }
  }
  u32x4 pk;  // A operand of P V: halves (2q, 2q + 1) of pk[q] = weights of slots 2q, 2q + 1 of run j, head c
  if constexpr (GP == 16) {
    float x[8];
    // per-token dequantization factors, prepared by the lane that loaded the token's parameters
    float pa = 0.f, pb = 0.f;
    if constexpr (F::kParBytes != 0) {
      const float sc = f16lo(t.par[0]);
      const float zp = DT == FS_KV_INT4 ? f16hi(t.par[0]) : 128.0f;
      if (c < 8) {  // K: logit = alpha * sc * (2^24 * S_raw - zp * qsum)
        pa = alpha * kTwo24 * sc;
        pb = -alpha * sc * zp;
      } else {      // V: p' = p * sc, zero-point term -p * sc * zp
        const bool ok = (c & 7) >= L.lo && (c & 7) < L.hi_u;  // a slot past the sequence may hold any bit pattern
        pa = ok ? sc : 0.f;
        pb = ok ? -sc * zp : 0.f;
      }
    }
    float va[8], vb2[8];
    static_for(std::make_integer_sequence<int, 8>{}, [&](auto I) {
      constexpr int i = decltype(I)::value;
      const float v = s[i >> 2][i & 3];
      if constexpr (F::kParBytes != 0) {
        const float ka = row_bcast<i>(pa);
        const float kb = row_bcast<i>(pb);
        va[i] = row_bcast<8 + i>(pa);
        vb2[i] = row_bcast<8 + i>(pb);
        x[i] = fmaf(v, ka, kb * qsum);
      } else {
        x[i] = v * alpha;
      }
    });
    if (partial) {
#pragma unroll
      for (int i = 0; i < 8; ++i) x[i] = (uint32_t)(i - L.lo) < n_ok ? x[i] : -INFINITY;
    }
    float tmax = x[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) tmax = fmaxf(tmax, x[i]);
    if (__any(tmax - st.m > kTau)) move_reference<DT, GP, HD>(st, tmax, j);
    const float m = st.m;
    float p[8];
    float lsum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float e = __builtin_amdgcn_exp2f(x[i] - m);
      lsum += e;
      if constexpr (F::kParBytes != 0) {
        p[i] = e * va[i];
        st.zc = fmaf(e, vb2[i], st.zc);
      } else {
        p[i] = e;
      }
    }
    st.l += lsum;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const half2v h = {(_Float16)p[2 * q], (_Float16)p[2 * q + 1]};
      pk[q] = h2u(h);
    }
  } else {
    // the two logits of head c % 4 for slots 2 (c / 4), 2 (c / 4) + 1: registers 2 (c / 4), + 1 of lane (j, c % 4)
    float y0 = s[0][0], y1 = s[0][1];
    y0 = take_shr<4, 0x2>(y0, s[0][2]);
    y1 = take_shr<4, 0x2>(y1, s[0][3]);
    y0 = take_shr<8, 0x4>(y0, s[1][0]);
    y1 = take_shr<8, 0x4>(y1, s[1][1]);
    y0 = take_shr<12, 0x8>(y0, s[1][2]);
    y1 = take_shr<12, 0x8>(y1, s[1][3]);
    const int i0 = 2 * (c >> 2);
    bool ok0 = true, ok1 = true;
    if (partial) {
      ok0 = (uint32_t)(i0 - L.lo) < n_ok;
      ok1 = (uint32_t)(i0 + 1 - L.lo) < n_ok;
    }
    float x0, x1;
    if constexpr (F::kParBytes != 0) {
      // logit = alpha * sc * (2^24 * S_raw - zp * qsum)     (qsum: of this lane's head)
      const float a24 = alpha * kTwo24, aq = -alpha * qsum;
      const float s0 = f16lo(t.par[0]), s1 = f16lo(t.par[1]);
      const float z0 = DT == FS_KV_INT4 ? f16hi(t.par[0]) : 128.0f, z1 = DT == FS_KV_INT4 ? f16hi(t.par[1]) : 128.0f;
      x0 = fmaf(y0, s0 * a24, (s0 * z0) * aq);
      x1 = fmaf(y1, s1 * a24, (s1 * z1) * aq);
    } else {
      x0 = y0 * alpha;
      x1 = y1 * alpha;
    }
    if (partial) {
      x0 = ok0 ? x0 : -INFINITY;
      x1 = ok1 ? x1 : -INFINITY;
    }
    const float tmax = fmaxf(x0, x1);
    if (__any(tmax - st.m > kTau)) move_reference<DT, GP, HD>(st, tmax, j);
    const float m = st.m;
    const float e0 = __builtin_amdgcn_exp2f(x0 - m), e1 = __builtin_amdgcn_exp2f(x1 - m);
    st.l += e0 + e1;
    float p0 = e0, p1 = e1;
    if constexpr (F::kParBytes != 0) {
      // p' = p * sc, zero-point term -p' * zp
      float s0 = f16lo(t.par[2]), s1 = f16lo(t.par[3]);
      const float z0 = DT == FS_KV_INT4 ? f16hi(t.par[2]) : 128.0f, z1 = DT == FS_KV_INT4 ? f16hi(t.par[3]) : 128.0f;
      if (partial) {  // a dead slot's scale may be any bit pattern
        s0 = ok0 ? s0 : 0.f;
        s1 = ok1 ? s1 : 0.f;
      }
      p0 = e0 * s0;
      p1 = e1 * s1;
      st.zc = fmaf(-p0, z0, st.zc);
      st.zc = fmaf(-p1, z1, st.zc);
    }
    const half2v h = {(_Float16)p0, (_Float16)p1};
    const uint32_t pp = h2u(h);
    pk[0] = pp;  // rows c >= 4 of the operand are padding heads: whatever lands there is finite and unused
    pk[1] = from_shl<4>(pp);
    pk[2] = from_shl<8>(pp);
    pk[3] = from_shl<12>(pp);
  }
  // ---- V rows of the run -> B operands (8x8 in-register transpose) and out += P V ----
  uint32_t vx[8][F::kVRegs];
#pragma unroll
  for (int i = 0; i < 8; ++i) v_unpack<DT, HD>(t.v[i], vx[i]);
#pragma unroll
  for (int e = 0; e < F::kNE; ++e) {
    // element e of the lane's share: INT4 word e / 8 holds codes (p, p + 4) of its eight in register p
    const int reg = DT == FS_KV_INT4 ? 4 * (e >> 3) + (e & 3) : (e >> 1);
    const uint32_t sel = (DT == FS_KV_INT4 ? ((e >> 2) & 1) : (e & 1)) ? 0x07060302u : 0x05040100u;
    u32x4 b;
#pragma unroll
    for (int q = 0; q < 4; ++q) b[q] = __builtin_amdgcn_perm(vx[2 * q + 1][reg], vx[2 * q][reg], sel);
    st.acc[e] = mfma(pk, b, st.acc[e]);
  }
}

// Head-chunk addresses of blocks k0 .. k0 + nb - 1 of a sequence into this wave's LDS table: every lane of
// every tile looks its blocks up there instead of gathering them from the block table in memory.
__device__ __forceinline__ void fill_table(uint64_t* s_ptr, const int32_t* table, const uint8_t* head_base,
                                           uint64_t block_budget, int k0, int nb, int lane, uint32_t n_blocks,
                                           uint32_t* header) {
  for (int i = lane; i < nb; i += 64)
    s_ptr[i] = reinterpret_cast<uint64_t>(head_base + (uint64_t)checked_block(table[k0 + i], n_blocks, header) * block_budget);
  // the table is private to this wave; LDS operations of a wave complete in order, the fence only keeps the
  // compiler from moving the look-ups above the writes of other lanes
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Streams the runs [v0, X.v_end) of a sequence through the online softmax.
// Software pipeline over the tiles: a ring of NBUF register copies of a tile.  The K rows of the tile that
// will next occupy a slot are requested as soon as S^T of its current occupant is done, the V rows as soon
// as P V is done, so the narrower the format the more tiles are in flight (about 16 KiB per wave for every
// format).
// Every step of a turn refills its slot unconditionally: in the last refilling turn some refills may lie past the
// last tile, where the runs are mapped onto the last run (rows just read, so the refill hits in cache) and the data is
// never used.  With refills that depend on a condition the compiler cannot know how many loads are outstanding behind
// the one it needs and waits for all of them, the ones just issued included, which exposes the full memory latency on
// every tile.
// PEEL (decode): the last turn is a second copy of the step without any refill.  Then nothing is requested that no
// one will read (a ring of rows per item), and nothing is in flight when the caller goes on to write the item's
// result: that code reuses the tiles' registers and otherwise waits for those loads to land (a per-item timeline
// showed 4 us per item between the last tile and the end of the output, 4 % of the mixed launch and 14 % of a short
// one).  Without PEEL every turn refills, the last one past the item's end (runs mapped onto the last run, never used),
// and the tile count is rounded up to whole turns of masked tiles.
template <int DT, int GP, int HD = 128, bool PEEL = false>
__device__ __forceinline__ void stream_tiles(const ItemCtx& X, const DevGeom& g, int v0, const u32x4 (&qb)[HD / 32], float qsum,
                                             float alpha, StateT<HD>& st, int j, int c) {
  constexpr int NBUF = Fmt<DT, HD>::kRing;
  const int n_tiles = (X.v_end - v0 + 3) >> 2;
  Tile<DT, GP, HD> t[NBUF];
  static_for(std::make_integer_sequence<int, NBUF>{}, [&](auto Bi) {
    constexpr int bi = decltype(Bi)::value;
    issue_k<DT, GP, HD>(X, v0 + bi * 4, j, c, t[bi]);
    issue_v<DT, GP, HD>(X, g, v0 + bi * 4, j, c, t[bi]);
  });
  // One turn of the ring: every slot's tile is consumed and replaced by the tile NBUF further on.
  // (not for INT4, nor INT8 at head_dim 64: with the second copy of the step their tile loops spill registers)
  constexpr bool kPeel = PEEL && DT != FS_KV_INT4 && !(DT == FS_KV_INT8 && HD == 64);
  int k0 = 0;
  for (; k0 + (kPeel ? NBUF : 0) < n_tiles; k0 += NBUF) {
    static_for(std::make_integer_sequence<int, NBUF>{}, [&](auto Bi) {
      constexpr int bi = decltype(Bi)::value;
      const int vb = v0 + (k0 + bi) * 4;
      const int vb_next = vb + NBUF * 4;
      float4v s[2];
      qk_tile<DT, GP, HD>(t[bi], qb, s);
      issue_k<DT, GP, HD>(X, vb_next, j, c, t[bi]);
      softmax_pv<DT, GP, HD>(X, t[bi], s, vb, j, c, qsum, alpha, st);
      issue_v<DT, GP, HD>(X, g, vb_next, j, c, t[bi]);
    });
  }
  // the last turn: the 1 .. NBUF tiles that are left, no refills (slots past the last tile hold rows nobody needs)
  if constexpr (kPeel) {
    static_for(std::make_integer_sequence<int, NBUF>{}, [&](auto Bi) {
      constexpr int bi = decltype(Bi)::value;
      if (bi == 0 || k0 + bi < n_tiles) {  // wave-uniform
        float4v s[2];
        qk_tile<DT, GP, HD>(t[bi], qb, s);
        softmax_pv<DT, GP, HD>(X, t[bi], s, v0 + (k0 + bi) * 4, j, c, qsum, alpha, st);
      }
    });
  }
}

}  // namespace
}  // namespace fs
