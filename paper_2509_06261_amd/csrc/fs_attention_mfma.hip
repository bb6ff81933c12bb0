// MFMA split-K paged decode-attention kernel for gfx950 (head_dim 128, all four KV formats).
//
// FineServe Sec. 2.1: the decode phase re-reads the whole KV cache for every generated token and
// is bound by memory bandwidth; Sec. 2.3 / 5.1: the cache is reached through each model's own block
// table over the shared slab pool.  This kernel streams K/V rows straight from the slabs into
// registers (no LDS staging: every byte is used by exactly one lane), dequantizes in registers and
// feeds v_mfma_f32_16x16x32_f16 for both contractions; the grouped query heads of a KV head
// (padded to 16) form the second matrix dimension.
//
// Work decomposition
//   a persistent grid of independent waves: each wave takes every n-th work item (sequence, split, KV head)
//   of the queue, streams the split's 32-token tiles with a private online-softmax state and writes the
//   output (or the split's partial record) straight from its accumulators.  No wave waits for another.
//
// One 32-token tile (base token tb), lane l = 16*j + c:
//   S^T = K Q^T as two 16x16 MFMA tiles u = 0,1 (rows = tokens, columns = query heads).  Row m of tile u
//   is token tb + 8*(m/4) + 4*u + (m%4), so that lane (j, c) ends up with the logits of head c for the
//   8 consecutive tokens tb + 8j .. tb + 8j + 7  (C layout: rows 4j..4j+3 of each tile).
//   Those 8 values, exponentiated and packed to fp16, are exactly the A operand (k index = token) of
//   out = P V; the B operand needs, per lane, the 8 tokens of its run for one d column, which is an
//   in-register 8x8 transpose (v_perm_b32) of the 8 row fragments the lane loaded.
//   K is loaded as the A operand of S^T: lane (j, c) reads 16 bytes of the row of token
//   tb + 8*(c/4) + 4u + (c%4); the d order inside a k-step is whatever the format's unpacking yields,
//   and the Q operand is pre-arranged once per item in the same order.
//
// Dequantization is folded around the MFMAs: FP8 static scales and INT8/INT4 per-token K scales
// multiply the logits, per-token V scales multiply P; integer codes enter the MFMA unconverted, as fp16
// subnormals, and their offsets (128 for INT8, the zero-point for INT4) come back as rank-1
// corrections (z_k * sum(q) on the logits, sum_t p_t s_t z_t on the output).
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
constexpr int kTile = 32;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int DT>
struct Fmt;
template <>
struct Fmt<FS_KV_FP16> {
  static constexpr int kRowBytes = 256, kKLoads = 4, kVBytes = 16, kParBytes = 0, kRing = 1;
};
template <>
struct Fmt<FS_KV_FP8_E4M3> {
  static constexpr int kRowBytes = 128, kKLoads = 2, kVBytes = 8, kParBytes = 0, kRing = 2;
};
template <>
struct Fmt<FS_KV_INT8> {
  static constexpr int kRowBytes = 128, kKLoads = 2, kVBytes = 8, kParBytes = 2, kRing = 2;
};
template <>
struct Fmt<FS_KV_INT4> {
  static constexpr int kRowBytes = 64, kKLoads = 1, kVBytes = 4, kParBytes = 4, kRing = 3;
};

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

template <int DT>
struct Tile {
  u32x4 k[2][Fmt<DT>::kKLoads];
  uint32_t v[8][Fmt<DT>::kVBytes / 4];
  uint32_t par;  // INT8/INT4: lanes c < 8 hold the K parameters of token c of the lane's run, lanes c >= 8 the V ones
};

struct ItemCtx {
  const DevBatch* B;
  const uint64_t* chunk_ptr;  // LDS: head-chunk address of blocks b_first .. b_last + 1 of this item's range
  int b_first, b_last;        // first / last block the item's token range touches
  int t1;                     // end of this item's token range
  uint32_t t_magic;           // ceil(2^32 / T)
};

// Where an 8-token run starting at token `tok` lives: head-chunk addresses of its first block (c0) and of
// the block after it (c1), the slot r0 of its first token, and how many of its tokens stay in the first
// block (cross >= 8: no crossing).  Token i is slot r0 + i of c0 if i < cross, else slot i - cross of c1.
// A run wholly past the item's last block is mapped to slots 0..7 of a valid block (its data is masked).
struct Run {
  gptr c0;
  gptr c1;
  int r0, cross;
};

__device__ __forceinline__ Run locate_run(const ItemCtx& X, int tok) {
  const int T = X.B->g.T;
  const int bi = (int)__umulhi((uint32_t)tok, X.t_magic);
  Run r;
  r.r0 = tok - bi * T;
  r.cross = T - r.r0;
  int idx = bi - X.b_first;
  if (bi > X.b_last) {
    r.r0 = 0;
    r.cross = 8;
    idx = X.b_last + 1 - X.b_first;
  }
  r.c0 = (gptr)X.chunk_ptr[idx];
  r.c1 = (gptr)X.chunk_ptr[min(idx + 1, X.b_last + 1 - X.b_first)];
  return r;
}

template <int DT>
__device__ __forceinline__ void issue_k(const ItemCtx& X, int tb, int j, int c, Tile<DT>& t) {
  using F = Fmt<DT>;
  const Run r = locate_run(X, tb + 8 * (c >> 2));
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const int i = 4 * u + (c & 3);
    const bool first = i < r.cross;
    const gptr p = (first ? r.c0 : r.c1) + (uint32_t)((first ? r.r0 + i : i - r.cross) * F::kRowBytes) + 16 * j;
#pragma unroll
    for (int s = 0; s < F::kKLoads; ++s) t.k[u][s] = *reinterpret_cast<const FS_GLOBAL u32x4*>(p + 64 * s);
  }
}

template <int DT>
__device__ __forceinline__ void load_v_row(gptr p, uint32_t (&v)[Fmt<DT>::kVBytes / 4]) {
  if constexpr (Fmt<DT>::kVBytes == 16) {
    const u32x4 x = *reinterpret_cast<const FS_GLOBAL u32x4*>(p);
    v[0] = x[0];
    v[1] = x[1];
    v[2] = x[2];
    v[3] = x[3];
  } else if constexpr (Fmt<DT>::kVBytes == 8) {
    const u32x2 x = *reinterpret_cast<const FS_GLOBAL u32x2*>(p);
    v[0] = x[0];
    v[1] = x[1];
  } else {
    v[0] = *reinterpret_cast<const FS_GLOBAL uint32_t*>(p);
  }
}

template <int DT>
__device__ __forceinline__ void issue_v(const ItemCtx& X, int tb, int j, int c, Tile<DT>& t) {
  using F = Fmt<DT>;
  const DevGeom& g = X.B->g;
  const Run r = locate_run(X, tb + 8 * j);
  if constexpr (F::kParBytes != 0) {  // parameters first: the softmax needs them before the V rows
    const int i = c & 7;
    const bool first = i < r.cross;
    const gptr p = (first ? r.c0 : r.c1) + 2u * g.kv_tile + ((c >> 3) ? g.par_tile : 0u) +
                       (uint32_t)((first ? r.r0 + i : i - r.cross) * F::kParBytes);
    if constexpr (F::kParBytes == 2) t.par = *reinterpret_cast<const FS_GLOBAL uint16_t*>(p);
    else t.par = *reinterpret_cast<const FS_GLOBAL uint32_t*>(p);
  }
  const gptr p0 = r.c0 + g.kv_tile + (uint32_t)(r.r0 * F::kRowBytes) + c * F::kVBytes;
  if (__all(r.cross >= 8)) {  // no run of this wave crosses a block boundary: one base, constant offsets
#pragma unroll
    for (int i = 0; i < 8; ++i) load_v_row<DT>(p0 + i * F::kRowBytes, t.v[i]);
  } else {
    const gptr p1 = r.c1 + g.kv_tile + c * F::kVBytes - (int64_t)r.cross * F::kRowBytes;
#pragma unroll
    for (int i = 0; i < 8; ++i) load_v_row<DT>((i < r.cross ? p0 : p1) + i * F::kRowBytes, t.v[i]);
  }
}

// The Q operand (B of S^T = K Q^T) of lane (j, c) for k-step ks: 8 halves of q[head c] in the d order
// (and with the per-position factors) that the format's K unpacking produces.  qsum = sum_d q[d].
template <int DT>
__device__ __forceinline__ void load_q(const _Float16* qrow, bool live, int j, u32x4 (&qb)[4], float& qsum) {
  qsum = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    int d0;
    if (DT == FS_KV_FP16) d0 = 32 * ks + 8 * j;
    else if (DT == FS_KV_INT4) d0 = 32 * j + 8 * ks;
    else d0 = 64 * (ks >> 1) + 16 * j + 8 * (ks & 1);
    u32x4 x = {0u, 0u, 0u, 0u};
    if (live) x = *reinterpret_cast<const u32x4*>(qrow + d0);
#pragma unroll
    for (int p = 0; p < 4; ++p) qsum += f16lo(x[p]) + f16hi(x[p]);
    if (DT == FS_KV_INT4) {
      const half2v s16 = {(_Float16)0.0625f, (_Float16)0.0625f};
      u32x4 y;
      y[0] = __builtin_amdgcn_perm(x[2], x[0], 0x05040100u);             // q0, q4
      y[1] = h2u(u2h(__builtin_amdgcn_perm(x[2], x[0], 0x07060302u)) * s16);  // (q1, q5) / 16
      y[2] = __builtin_amdgcn_perm(x[3], x[1], 0x05040100u);             // q2, q6
      y[3] = h2u(u2h(__builtin_amdgcn_perm(x[3], x[1], 0x07060302u)) * s16);  // (q3, q7) / 16
      x = y;
    }
    qb[ks] = x;
  }
}

__device__ __forceinline__ float4v mfma(u32x4 a, u32x4 b, float4v acc) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, a), __builtin_bit_cast(half8, b), acc, 0, 0, 0);
}

// K fragments of one 16-token tile -> the four A operands of S^T.
template <int DT>
__device__ __forceinline__ void k_operands(const u32x4 (&k)[Fmt<DT>::kKLoads], u32x4 (&a)[4]) {
  if constexpr (DT == FS_KV_FP16) {
#pragma unroll
    for (int s = 0; s < 4; ++s) a[s] = k[s];
  } else if constexpr (DT == FS_KV_FP8_E4M3) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const u32x4 x = k[ks >> 1];
      const uint32_t w0 = x[2 * (ks & 1)], w1 = x[2 * (ks & 1) + 1];
      a[ks][0] = fp8x2_lo(w0);
      a[ks][1] = fp8x2_hi(w0);
      a[ks][2] = fp8x2_lo(w1);
      a[ks][3] = fp8x2_hi(w1);
    }
  } else if constexpr (DT == FS_KV_INT8) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
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
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      uint32_t r[4];
      int4x8(k[0][ks], r);
      a[ks][0] = r[0];
      a[ks][1] = r[1];
      a[ks][2] = r[2];
      a[ks][3] = r[3];
    }
  }
}

// 8 elements of one V row -> four packed-fp16 registers (layout note above).
template <int DT>
__device__ __forceinline__ void v_unpack(const uint32_t (&v)[Fmt<DT>::kVBytes / 4], uint32_t (&x)[4]) {
  if constexpr (DT == FS_KV_FP16) {
#pragma unroll
    for (int p = 0; p < 4; ++p) x[p] = v[p];
  } else if constexpr (DT == FS_KV_FP8_E4M3) {
    x[0] = fp8x2_lo(v[0]);
    x[1] = fp8x2_hi(v[0]);
    x[2] = fp8x2_lo(v[1]);
    x[3] = fp8x2_hi(v[1]);
  } else if constexpr (DT == FS_KV_INT8) {
    int8x4(v[0], x[0], x[1]);
    int8x4(v[1], x[2], x[3]);
  } else {
    int4x8(v[0], x);
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

// Per-wave online-softmax state.  acc[e] is the 16x16 output tile of d columns {8c' + e}: lane (j', c')
// holds rows (heads) 4j'..4j'+3.  m, l, zc are per head c in the S^T layout (lane (j, c), any j).
struct State {
  float4v acc[8];
  float m;   // reference subtracted from the logits (base-2 domain): within kTau of the running max
  float l;   // this lane's share of the running sum (its 8-token runs only)
  float zc;  // INT8/INT4: this lane's share of the zero-point term  -sum_t p_t s_t z_t
};

// S^T = K Q^T for the 32 tokens of the tile: s[u][r] = raw logit of head c, token tb + 8j + 4u + r.
template <int DT>
__device__ __forceinline__ void qk_tile(const Tile<DT>& t, const u32x4 (&qb)[4], float4v (&s)[2]) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    u32x4 a[4];
    k_operands<DT>(t.k[u], a);
    float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) acc = mfma(a[ks], qb[ks], acc);
    s[u] = acc;
  }
}

// Online softmax over the tile and out += P V.
template <int DT>
__device__ __forceinline__ void softmax_pv(const ItemCtx& X, Tile<DT>& t, const float4v (&s)[2], int tb, int j, int c,
                                           float qsum, float alpha, State& st) {
  const int n_valid = X.t1 - (tb + 8 * j);  // tokens of this lane's run inside the range
  const bool partial = tb + kTile > X.t1;    // wave-uniform
  float x[8];
  // per-token dequantization factors, prepared by the lane that loaded the token's parameters
  float pa = 0.f, pb = 0.f;
  if constexpr (Fmt<DT>::kParBytes != 0) {
    const float sc = f16lo(t.par);
    const float zp = DT == FS_KV_INT4 ? f16hi(t.par) : 128.0f;
    if (c < 8) {  // K: logit = alpha * sc * (2^24 * S_raw - zp * qsum)
      pa = alpha * kTwo24 * sc;
      pb = -alpha * sc * zp;
    } else {      // V: p' = p * sc, zero-point term -p * sc * zp
      const bool ok = (c & 7) < n_valid;
      pa = ok ? sc : 0.f;
      pb = ok ? -sc * zp : 0.f;
    }
  }
  float ka[8], kb[8], va[8], vb[8];
  static_for(std::make_integer_sequence<int, 8>{}, [&](auto I) {
    constexpr int i = decltype(I)::value;
    const float v = s[i >> 2][i & 3];
    if constexpr (Fmt<DT>::kParBytes != 0) {
      ka[i] = row_bcast<i>(pa);
      kb[i] = row_bcast<i>(pb);
      va[i] = row_bcast<8 + i>(pa);
      vb[i] = row_bcast<8 + i>(pb);
      x[i] = fmaf(v, ka[i], kb[i] * qsum);
    } else {
      x[i] = v * alpha;
    }
  });
  if (partial) {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = i < n_valid ? x[i] : -INFINITY;
    if constexpr (DT == FS_KV_FP16 || DT == FS_KV_FP8_E4M3) {
      // rows past the range may hold NaN/Inf bit patterns; 0 * NaN would poison the MFMA
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int w = 0; w < Fmt<DT>::kVBytes / 4; ++w) t.v[i][w] = i < n_valid ? t.v[i][w] : 0u;
    }
  }
  // ---- lazy running reference: the softmax is invariant to the value subtracted from the logits, so the
  // reference m only has to stay within 2^kTau of the largest logit seen (P stays <= 2^kTau, far inside fp16).
  // The exact cross-lane maximum and the rescale of the accumulators run only when some logit of the tile
  // exceeds its head's reference by more than kTau (always on a wave's first tile, where m = -inf).
  float tmax = x[0];
#pragma unroll
  for (int i = 1; i < 8; ++i) tmax = fmaxf(tmax, x[i]);
  if (__any(tmax - st.m > kTau)) {
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
    const float m_new = fmaxf(st.m, tmax);  // finite: token tb of every tile is inside the range
    const float corr = __builtin_amdgcn_exp2f(st.m - m_new);
    st.l *= corr;
    if constexpr (Fmt<DT>::kParBytes != 0) st.zc *= corr;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float cr = __shfl(corr, 4 * j + r, 64);  // head 4j + r keeps its factor in lane c = 4j + r
#pragma unroll
      for (int e = 0; e < 8; ++e) st.acc[e][r] *= cr;
    }
    st.m = m_new;
  }
  const float m_new = st.m;
  // ---- P (times the per-token V scale) ----
  float p[8];
  float lsum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float e = __builtin_amdgcn_exp2f(x[i] - m_new);
    lsum += e;
    if constexpr (Fmt<DT>::kParBytes != 0) {
      p[i] = e * va[i];
      st.zc = fmaf(e, vb[i], st.zc);
    } else {
      p[i] = e;
    }
  }
  st.l += lsum;
  u32x4 pk;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const half2v h = {(_Float16)p[2 * q], (_Float16)p[2 * q + 1]};
    pk[q] = h2u(h);
  }
  // ---- V rows of the run -> B operands (8x8 in-register transpose) and out += P V ----
  uint32_t vx[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i) v_unpack<DT>(t.v[i], vx[i]);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int reg = DT == FS_KV_INT4 ? (e & 3) : (e >> 1);
    const uint32_t sel = (DT == FS_KV_INT4 ? (e >> 2) : (e & 1)) ? 0x07060302u : 0x05040100u;
    u32x4 b;
#pragma unroll
    for (int q = 0; q < 4; ++q) b[q] = __builtin_amdgcn_perm(vx[2 * q + 1][reg], vx[2 * q][reg], sel);
    st.acc[e] = mfma(pk, b, st.acc[e]);
  }
}

// One work item, processed by ONE wave: all 32-token tiles of the split, then the output (or the split's
// partial record) straight from the accumulator registers.  Waves never synchronise with each other.
// s_ptr: this wave's LDS table of head-chunk addresses.
template <int DT>
__device__ void process_item(const MultiArgs& A, int b, int seq, int chunk, int head, uint32_t item, uint64_t* s_ptr) {
  const DevBatch& B = A.b[b];
  const DevGeom& g = B.g;
  const int lane = threadIdx.x & 63;
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int max_len = (int)min((int64_t)B.max_blocks * g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : (len > max_len ? max_len : len);
  const int n_chunks = (len + B.chunk_tokens - 1) / B.chunk_tokens;
  const int t0 = chunk * B.chunk_tokens;
  const int t1 = min(len, t0 + B.chunk_tokens);
  const int nblk = (len + g.T - 1) / g.T;

  const uint64_t* part_off = reinterpret_cast<const uint64_t*>(A.header + kHdrPartOff);
  const uint64_t part_base = part_off[b] + (uint64_t)(item - A.header[kHdrBatchFirst + b]) * (uint64_t)B.part_stride;
  if (n_chunks > 1 && part_base + (uint64_t)B.part_stride > A.part_capacity) {  // wave-uniform
    if (lane == 0) atomicOr(A.header + kHdrStatus, 2u);
    return;
  }

  ItemCtx X;
  X.B = &B;
  X.b_first = t0 / g.T;
  X.b_last = (t1 - 1) / g.T;
  X.t1 = t1;
  X.t_magic = B.t_magic;
  // head-chunk addresses of the blocks this item touches (plus one more), through LDS: every lane of
  // every tile looks its blocks up here instead of gathering them from the block table in memory
  X.chunk_ptr = s_ptr;
  {
    const int32_t* table = B.tables + (int64_t)seq * B.max_blocks;
    const uint8_t* head_base = B.layer_base + (uint64_t)head * g.head_chunk;
    const int nb = X.b_last - X.b_first + 2;
    for (int i = lane; i < nb; i += 64) {
      const int bi = min(X.b_first + i, nblk - 1);  // past the sequence's last block: alias it (valid memory)
      s_ptr[i] = reinterpret_cast<uint64_t>(head_base + (uint64_t)(uint32_t)table[bi] * g.block_budget);
    }
  }
  // the table is private to this wave; LDS operations of a wave complete in order, the fence only keeps the
  // compiler from moving the look-ups above the writes of other lanes
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

  // Q operand and per-head constants
  u32x4 qb[4];
  float qsum;
  load_q<DT>(B.q + ((int64_t)seq * B.n_q + head * G + c) * kD, c < G, j, qb, qsum);
  if constexpr (Fmt<DT>::kParBytes != 0) {
    qsum += __shfl_xor(qsum, 16, 64);
    qsum += __shfl_xor(qsum, 32, 64);
  }
  float alpha = B.sm_scale * kLog2e;
  if (DT == FS_KV_FP8_E4M3) alpha *= B.k_scale[head];

  State st;
#pragma unroll
  for (int e = 0; e < 8; ++e) st.acc[e] = float4v{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
  st.l = 0.f;
  st.zc = 0.f;

  // Software pipeline over the item's tiles: a ring of NBUF register copies of a tile.  The K rows of the
  // tile that will next occupy a slot are requested as soon as S^T of its current occupant is done, the V
  // rows as soon as P V is done, so the narrower the format the more tiles are in flight (about 16 KiB per
  // wave for every format).
  constexpr int NBUF = Fmt<DT>::kRing;
  const int n_tiles = (t1 - t0 + kTile - 1) / kTile;
  Tile<DT> t[NBUF];
  static_for(std::make_integer_sequence<int, NBUF>{}, [&](auto Bi) {
    constexpr int bi = decltype(Bi)::value;
    if (bi < n_tiles) {
      const int tb = t0 + bi * kTile;
      issue_k<DT>(X, tb, j, c, t[bi]);
      issue_v<DT>(X, tb, j, c, t[bi]);
    }
  });
  for (int k0 = 0; k0 < n_tiles; k0 += NBUF) {
    static_for(std::make_integer_sequence<int, NBUF>{}, [&](auto Bi) {
      constexpr int bi = decltype(Bi)::value;
      const int k = k0 + bi;
      if (k < n_tiles) {
        const int tb = t0 + k * kTile;
        const int tb_next = tb + NBUF * kTile;
        const bool more = k + NBUF < n_tiles;
        float4v s[2];
        qk_tile<DT>(t[bi], qb, s);
        if (more) issue_k<DT>(X, tb_next, j, c, t[bi]);
        softmax_pv<DT>(X, t[bi], s, tb, j, c, qsum, alpha, st);
        if (more) issue_v<DT>(X, tb_next, j, c, t[bi]);
      }
    });
  }

  // ---- output: per-head sums over the four lane groups, then rows h < G straight from the accumulators ----
  st.l += __shfl_xor(st.l, 16, 64);
  st.l += __shfl_xor(st.l, 32, 64);
  if constexpr (Fmt<DT>::kParBytes != 0) {
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

__device__ __forceinline__ void dispatch_item(const MultiArgs& A, uint32_t item, uint64_t* s_ptr) {
  const int4 rec = A.item_list[item];
  const int b = rec.x, seq = rec.y, chunk = rec.z, head = rec.w;
  switch (A.b[b].g.dtype) {
    case FS_KV_FP16: process_item<FS_KV_FP16>(A, b, seq, chunk, head, item, s_ptr); break;
    case FS_KV_FP8_E4M3: process_item<FS_KV_FP8_E4M3>(A, b, seq, chunk, head, item, s_ptr); break;
    case FS_KV_INT8: process_item<FS_KV_INT8>(A, b, seq, chunk, head, item, s_ptr); break;
    default: process_item<FS_KV_INT4>(A, b, seq, chunk, head, item, s_ptr); break;
  }
}

__global__ __launch_bounds__(kThreads, 2) void mfma_attention_kernel(MultiArgs A, int table_entries) {
  extern __shared__ uint64_t smem64[];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint64_t* s_ptr = smem64 + (size_t)wave * table_entries;
  const uint32_t total = A.header[kHdrTotalItems];
  // Every wave is its own worker and takes the items worker, worker + n_workers, ... of the queue.  Items
  // are splits of (nearly) equal bytes and every worker's stride walks through all batches alike, so this
  // fixed deal balances to within about one item per batch.  (Drawing the items from a shared ticket
  // counter instead was measured to bound the kernel: the memory system serves one atomic on a given
  // address every ~11 ns when idle and several times slower under streaming load.)
  const uint32_t n_workers = gridDim.x * kWaves, worker = blockIdx.x * kWaves + wave;
  for (uint32_t item = worker; item < total; item += n_workers) dispatch_item(A, item, s_ptr);
}

}  // namespace

// Shapes this kernel covers: head_dim 128, at least 8 tokens per block (an 8-token run then crosses at
// most one block boundary), and token indices small enough for the multiply-high division by T.
bool mfma_supports(const DevBatch& b) {
  if (b.g.D != kD || b.g.T < 8 || b.G > 16) return false;
  const uint64_t max_tok = (uint64_t)b.max_blocks * (uint64_t)b.g.T + 64;
  return max_tok <= (1ull << 32) / (uint64_t)b.g.T && max_tok < (1ull << 31);
}

hipError_t launch_mfma(const MultiArgs& A, int n_workgroups, hipStream_t s) {
  // LDS: per wave one 8-byte address per block of the largest split (+ slack)
  int entries = 0;
  for (int i = 0; i < A.n_batches; ++i) entries = std::max(entries, A.b[i].chunk_tokens / A.b[i].g.T + 4);
  const size_t smem = (size_t)kWaves * entries * sizeof(uint64_t);
  hipLaunchKernelGGL(mfma_attention_kernel, dim3(n_workgroups), dim3(kThreads), smem, s, A, entries);
  return hipGetLastError();
}

}  // namespace fs
