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
//   persistent workgroups (4 waves) pull work items (sequence, split, KV head) from a ticket counter;
//   inside an item wave w owns the 32-token tiles w, w+4, ... of the split and keeps a private
//   online-softmax state; the four waves are merged through LDS at the end of the item.
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
// multiply the logits, per-token V scales multiply P, INT4 codes are centred to n-8 exactly in fp16
// and the zero-points enter as rank-1 corrections ((8 - z_k) * sum(q) on the logits, sum_t p_t s_t
// (8 - z_v) on the output).
#include "fs_attention.h"

namespace fs {
namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

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
  static constexpr int kRowBytes = 256, kKLoads = 4, kVBytes = 16, kParBytes = 0;
};
template <>
struct Fmt<FS_KV_FP8_E4M3> {
  static constexpr int kRowBytes = 128, kKLoads = 2, kVBytes = 8, kParBytes = 0;
};
template <>
struct Fmt<FS_KV_INT8> {
  static constexpr int kRowBytes = 128, kKLoads = 2, kVBytes = 8, kParBytes = 2;
};
template <>
struct Fmt<FS_KV_INT4> {
  static constexpr int kRowBytes = 64, kKLoads = 1, kVBytes = 4, kParBytes = 4;
};

__device__ __forceinline__ uint32_t h2u(half2v h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ half2v u2h(uint32_t u) { return __builtin_bit_cast(half2v, u); }
__device__ __forceinline__ float f16lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFF)); }
__device__ __forceinline__ float f16hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)); }

// ---- 8 stored elements -> 4 registers of packed fp16 -----------------------------------------
// FP16 / FP8 / INT8: register p holds elements (2p, 2p+1).  INT4: register p holds codes (p, p+4).

// two E4M3 bytes of a dword -> packed fp16 (exact)
__device__ __forceinline__ uint32_t fp8x2_lo(uint32_t w) { return h2u(__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, false)); }
__device__ __forceinline__ uint32_t fp8x2_hi(uint32_t w) { return h2u(__builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w, 1.0f, true)); }

// four INT8 bytes -> two registers of packed fp16 (exact): x ^ 0x80 = x + 128 as an unsigned byte,
// 0x6400 | u is the fp16 number 1024 + u, and 1024 + u - 1152 = x.
__device__ __forceinline__ void int8x4(uint32_t w, uint32_t& r0, uint32_t& r1) {
  const uint32_t u = w ^ 0x80808080u;
  const half2v off = {(_Float16)-1152.0f, (_Float16)-1152.0f};
  r0 = h2u(u2h(__builtin_amdgcn_perm(0x64646464u, u, 0x04010400u)) + off);
  r1 = h2u(u2h(__builtin_amdgcn_perm(0x64646464u, u, 0x04030402u)) + off);
}

// eight INT4 codes of a dword -> four registers of packed fp16 holding code - 8 (exact):
// 0x6400 | n = 1024 + n;  0x6400 | (n << 4) = 1024 + 16 n, and (1024 + 16 n) / 16 - 72 = n - 8.
__device__ __forceinline__ void int4x8(uint32_t w, uint32_t (&r)[4]) {
  const half2v c1032 = {(_Float16)-1032.0f, (_Float16)-1032.0f};
  const half2v s16 = {(_Float16)0.0625f, (_Float16)0.0625f};
  const half2v c72 = {(_Float16)-72.0f, (_Float16)-72.0f};
  const uint32_t w8 = w >> 8;
  r[0] = h2u(u2h((w & 0x000F000Fu) | 0x64006400u) + c1032);                            // codes 0, 4
  r[1] = h2u(__builtin_elementwise_fma(u2h((w & 0x00F000F0u) | 0x64006400u), s16, c72));  // codes 1, 5
  r[2] = h2u(u2h((w8 & 0x000F000Fu) | 0x64006400u) + c1032);                           // codes 2, 6
  r[3] = h2u(__builtin_elementwise_fma(u2h((w8 & 0x00F000F0u) | 0x64006400u), s16, c72)); // codes 3, 7
}

// Address of the rows of one 8-token run: token i of the run lives at (i < cross ? p0 : p1) + i * stride.
struct Run {
  const uint8_t* c0;  // head chunk of the block holding the first token of the run
  const uint8_t* c1;  // head chunk of the next block (or c0 again when there is none)
  int r0;             // slot of the run's first token inside its block
  int cross;          // tokens of the run that stay in the first block (>= 8: no crossing)
};

template <int DT>
struct Tile {
  u32x4 k[2][Fmt<DT>::kKLoads];
  uint32_t v[8][Fmt<DT>::kVBytes / 4];
  uint32_t kpar[8], vpar[8];
};

struct ItemCtx {
  const DevBatch* B;
  const int32_t* table;
  const uint8_t* head_base;  // layer_base + head * head_chunk
  int nblk;                  // blocks of this sequence
  int t1;                    // end of this item's token range
  uint32_t t_magic;          // ceil(2^32 / T)
};

__device__ __forceinline__ Run make_run(const ItemCtx& X, int tok) {
  const DevGeom& g = X.B->g;
  const int bi = (int)__umulhi((uint32_t)tok, X.t_magic);
  Run r;
  r.r0 = tok - bi * g.T;
  r.cross = g.T - r.r0;
  const int b0 = min(bi, X.nblk - 1);  // tokens past the sequence end alias valid memory of its last block
  const uint32_t blk0 = (uint32_t)X.table[b0];
  r.c0 = X.head_base + (uint64_t)blk0 * g.block_budget;
  r.c1 = r.c0;
  if (r.cross < 8) {
    const uint32_t blk1 = bi + 1 < X.nblk ? (uint32_t)X.table[bi + 1] : blk0;
    r.c1 = X.head_base + (uint64_t)blk1 * g.block_budget;
  }
  if (bi >= X.nblk) {  // whole run is past the end: keep every address inside the last block
    r.r0 = 0;
    r.cross = 8;
  }
  return r;
}

// pointer to slot i of the run inside a tile that starts `tile_off` bytes into the head chunk
__device__ __forceinline__ const uint8_t* run_ptr(const Run& r, int i, uint32_t tile_off, int stride) {
  const bool first = i < r.cross;
  const uint8_t* c = first ? r.c0 : r.c1;
  const int slot = first ? r.r0 + i : i - r.cross;
  return c + tile_off + (uint32_t)(slot * stride);
}

template <int DT>
__device__ __forceinline__ void load_tile(const ItemCtx& X, int tb, int j, int c, Tile<DT>& t) {
  using F = Fmt<DT>;
  const DevGeom& g = X.B->g;
  // V role: the 8-token run tb + 8j .. +7, 8 elements (d = 8c .. 8c+7) of each row
  const Run rv = make_run(X, tb + 8 * j);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint8_t* p = run_ptr(rv, i, g.kv_tile, F::kRowBytes) + c * F::kVBytes;
    if constexpr (F::kVBytes == 16) {
      const u32x4 x = *reinterpret_cast<const u32x4*>(p);
      t.v[i][0] = x[0];
      t.v[i][1] = x[1];
      t.v[i][2] = x[2];
      t.v[i][3] = x[3];
    } else if constexpr (F::kVBytes == 8) {
      const u32x2 x = *reinterpret_cast<const u32x2*>(p);
      t.v[i][0] = x[0];
      t.v[i][1] = x[1];
    } else {
      t.v[i][0] = *reinterpret_cast<const uint32_t*>(p);
    }
    if constexpr (F::kParBytes == 2) {
      t.kpar[i] = *reinterpret_cast<const uint16_t*>(run_ptr(rv, i, 2u * g.kv_tile, 2));
      t.vpar[i] = *reinterpret_cast<const uint16_t*>(run_ptr(rv, i, 2u * g.kv_tile + g.par_tile, 2));
    } else if constexpr (F::kParBytes == 4) {
      t.kpar[i] = *reinterpret_cast<const uint32_t*>(run_ptr(rv, i, 2u * g.kv_tile, 4));
      t.vpar[i] = *reinterpret_cast<const uint32_t*>(run_ptr(rv, i, 2u * g.kv_tile + g.par_tile, 4));
    }
  }
  // K role: rows of tokens tb + 8*(c/4) + 4u + (c%4), 16 bytes at 64 s + 16 j of each
  const Run rk = make_run(X, tb + 8 * (c >> 2));
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    // slot index inside the run is 4u + (c & 3): not a compile-time constant, so select by value
    const int i = 4 * u + (c & 3);
    const bool first = i < rk.cross;
    const uint8_t* cb = first ? rk.c0 : rk.c1;
    const int slot = first ? rk.r0 + i : i - rk.cross;
    const uint8_t* p = cb + (uint32_t)(slot * F::kRowBytes) + 16 * j;
#pragma unroll
    for (int s = 0; s < F::kKLoads; ++s) t.k[u][s] = *reinterpret_cast<const u32x4*>(p + 64 * s);
  }
}

// The Q operand (B of S^T = K Q^T) of lane (j, c) for k-step ks: 8 halves of q[head c] in the d order
// that the format's K unpacking produces.
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
    if (DT == FS_KV_INT4) {
      // K registers hold codes (0,4), (1,5), (2,6), (3,7): bring q into the same order
      u32x4 y;
      y[0] = __builtin_amdgcn_perm(x[2], x[0], 0x05040100u);  // q0, q4
      y[1] = __builtin_amdgcn_perm(x[2], x[0], 0x07060302u);  // q1, q5
      y[2] = __builtin_amdgcn_perm(x[3], x[1], 0x05040100u);  // q2, q6
      y[3] = __builtin_amdgcn_perm(x[3], x[1], 0x07060302u);  // q3, q7
      x = y;
    }
#pragma unroll
    for (int p = 0; p < 4; ++p) qsum += f16lo(x[p]) + f16hi(x[p]);
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

// 8 elements of one V row -> four packed-fp16 registers (see the layout note above int8x4).
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

// Per-wave online-softmax state.  acc[e] is the 16x16 output tile of d columns {8c' + e}: lane (j', c')
// holds rows (heads) 4j'..4j'+3.  m, l, zc are per head c in the S^T layout (lane (j, c), any j).
struct State {
  float4v acc[8];
  float m;   // running max of the logits (base-2 domain)
  float l;   // this lane's share of the running sum (its 8-token runs only)
  float zc;  // INT4: this lane's share of sum_t p_t s_t (8 - z_t)
};

template <int DT>
__device__ __forceinline__ void compute_tile(const ItemCtx& X, const Tile<DT>& t, int tb, int j, int c,
                                             const u32x4 (&qb)[4], float qsum, float alpha, State& st) {
  // ---- S^T = K Q^T ----
  float4v s[2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    u32x4 a[4];
    k_operands<DT>(t.k[u], a);
    float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) acc = mfma(a[ks], qb[ks], acc);
    s[u] = acc;
  }
  // ---- logits of head c for tokens tb + 8j + i (i = 4u + r), base-2 domain ----
  const int n_valid = X.t1 - (tb + 8 * j);  // tokens of this lane's run inside the range
  float x[8], vs[8];
  float tmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    float v = s[i >> 2][i & 3];
    float sc = alpha;
    vs[i] = 1.0f;
    if (DT == FS_KV_INT8) {
      sc = alpha * f16lo(t.kpar[i]);
      vs[i] = f16lo(t.vpar[i]);
    } else if (DT == FS_KV_INT4) {
      sc = alpha * f16lo(t.kpar[i]);
      v = fmaf(8.0f - f16hi(t.kpar[i]), qsum, v);
      vs[i] = f16lo(t.vpar[i]);
    }
    x[i] = i < n_valid ? v * sc : -INFINITY;
    tmax = fmaxf(tmax, x[i]);
  }
  tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
  const float m_new = fmaxf(st.m, tmax);  // finite: every tile has at least one valid token (token tb)
  const float corr = __builtin_amdgcn_exp2f(st.m - m_new);
  // ---- rescale the running state when some head's max moved ----
  if (__any(m_new > st.m)) {
    st.l *= corr;
    if (DT == FS_KV_INT4) st.zc *= corr;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const float cr = __shfl(corr, 4 * j + r, 64);  // head 4j + r keeps its factor in lane c = 4j + r
#pragma unroll
      for (int e = 0; e < 8; ++e) st.acc[e][r] *= cr;
    }
  }
  st.m = m_new;
  // ---- P (and P scaled by the per-token V scale) ----
  float p[8];
  float lsum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float e = __builtin_amdgcn_exp2f(x[i] - m_new);
    lsum += e;
    p[i] = e;
    if (DT == FS_KV_INT8 || DT == FS_KV_INT4) p[i] = i < n_valid ? e * vs[i] : 0.f;
    if (DT == FS_KV_INT4) st.zc = fmaf(p[i], 8.0f - (i < n_valid ? f16hi(t.vpar[i]) : 8.0f), st.zc);
  }
  st.l += lsum;
  u32x4 pa;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const half2v h = {(_Float16)p[2 * q], (_Float16)p[2 * q + 1]};
    pa[q] = h2u(h);
  }
  // ---- V rows of the run -> B operands (8x8 in-register transpose) and out += P V ----
  uint32_t vx[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    v_unpack<DT>(t.v[i], vx[i]);
    if (DT == FS_KV_FP16 || DT == FS_KV_FP8_E4M3) {
      // rows past the range may hold NaN/Inf bit patterns; 0 * NaN would poison the MFMA
      if (i >= n_valid) vx[i][0] = vx[i][1] = vx[i][2] = vx[i][3] = 0u;
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int reg = DT == FS_KV_INT4 ? (e & 3) : (e >> 1);
    const uint32_t sel = (DT == FS_KV_INT4 ? (e >> 2) : (e & 1)) ? 0x07060302u : 0x05040100u;
    u32x4 b;
#pragma unroll
    for (int q = 0; q < 4; ++q) b[q] = __builtin_amdgcn_perm(vx[2 * q + 1][reg], vx[2 * q][reg], sel);
    st.acc[e] = mfma(pa, b, st.acc[e]);
  }
}

template <int DT>
__device__ void process_item(const MultiArgs& A, int b, int seq, int chunk, int head, uint32_t item, float* smem) {
  const DevBatch& B = A.b[b];
  const DevGeom& g = B.g;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int max_len = (int)min((int64_t)B.max_blocks * g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : (len > max_len ? max_len : len);
  const int n_chunks = (len + B.chunk_tokens - 1) / B.chunk_tokens;
  const int t0 = chunk * B.chunk_tokens;
  ItemCtx X;
  X.B = &B;
  X.table = B.tables + (int64_t)seq * B.max_blocks;
  X.head_base = B.layer_base + (uint64_t)head * g.head_chunk;
  X.nblk = (len + g.T - 1) / g.T;
  X.t1 = min(len, t0 + B.chunk_tokens);
  X.t_magic = B.t_magic;

  const uint64_t* part_off = reinterpret_cast<const uint64_t*>(A.header + kHdrPartOff);
  const uint64_t part_base = part_off[b] + (uint64_t)(item - A.header[kHdrBatchFirst + b]) * (uint64_t)B.part_stride;
  if (n_chunks > 1 && part_base + (uint64_t)B.part_stride > A.part_capacity) {
    if (threadIdx.x == 0) atomicOr(A.header + kHdrStatus, 2u);
    return;
  }

  // Q operand and per-head constants
  u32x4 qb[4];
  float qsum;
  load_q<DT>(B.q + ((int64_t)seq * B.n_q + head * G + c) * kD, c < G, j, qb, qsum);
  if (DT == FS_KV_INT4) {
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

  // software pipeline: the loads of tile n+1 are in flight while tile n is computed
  const int n_tiles = (X.t1 - t0 + kTile - 1) / kTile;
  int n = wave;
  Tile<DT> cur, nxt;
  if (n < n_tiles) load_tile<DT>(X, t0 + n * kTile, j, c, cur);
  for (; n < n_tiles; n += kWaves) {
    const bool more = n + kWaves < n_tiles;
    if (more) load_tile<DT>(X, t0 + (n + kWaves) * kTile, j, c, nxt);
    compute_tile<DT>(X, cur, t0 + n * kTile, j, c, qb, qsum, alpha, st);
    if (more) cur = nxt;
  }

  // ---- merge the four waves through LDS: [wave][head][D] accumulators, [wave][head] m, l, zc ----
  st.l += __shfl_xor(st.l, 16, 64);
  st.l += __shfl_xor(st.l, 32, 64);
  if (DT == FS_KV_INT4) {
    st.zc += __shfl_xor(st.zc, 16, 64);
    st.zc += __shfl_xor(st.zc, 32, 64);
  }
  float* s_acc = smem;                          // [kWaves][16][kD]
  float* s_m = smem + kWaves * 16 * kD;         // [kWaves][16]
  float* s_l = s_m + kWaves * 16;
  float* s_z = s_l + kWaves * 16;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int h = 4 * j + r;
    if (h < G) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s_acc[(wave * 16 + h) * kD + 8 * c + e] = st.acc[e][r];
    }
  }
  if (j == 0 && c < G) {
    s_m[wave * 16 + c] = st.m;
    s_l[wave * 16 + c] = st.l;
    s_z[wave * 16 + c] = st.zc;
  }
  __syncthreads();
  const float v_static = DT == FS_KV_FP8_E4M3 ? B.v_scale[head] : 1.0f;
  for (int idx = threadIdx.x; idx < G * kD; idx += kThreads) {
    const int h = idx >> 7, d = idx & (kD - 1);
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) M = fmaxf(M, s_m[w * 16 + h]);
    float L = 0.f, O = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float mw = s_m[w * 16 + h];
      const float wt = mw == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mw - M);
      L += s_l[w * 16 + h] * wt;
      float o = s_acc[(w * 16 + h) * kD + d];
      if (DT == FS_KV_INT4) o += s_z[w * 16 + h];
      O += o * wt;
    }
    O *= v_static;
    const int qh = head * G + h;
    if (n_chunks == 1) {
      B.out[((int64_t)seq * B.n_q + qh) * kD + d] = (_Float16)(O / L);
      if (d == 0 && B.lse) B.lse[(int64_t)seq * B.n_q + qh] = (M + __builtin_amdgcn_logf(L)) * kLn2;
    } else {
      float* pr = A.partials + part_base + (uint64_t)h * (kD + 2);
      pr[d] = O;
      if (d == 0) {
        pr[kD] = M * kLn2;  // partial records keep the max in natural-log units
        pr[kD + 1] = L;
      }
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(kThreads, 2) void mfma_attention_kernel(MultiArgs A) {
  extern __shared__ float smem[];
  __shared__ uint32_t s_item;
  const uint32_t total = A.header[kHdrTotalItems];
  for (;;) {
    if (threadIdx.x == 0) s_item = atomicAdd(A.header + kHdrCounter, 1u);
    __syncthreads();
    const uint32_t item = s_item;
    __syncthreads();
    if (item >= total) break;  // every wave of every workgroup leaves here once the queue is empty
    int lo = 0, hi = A.n_seq_total;
    while (hi - lo > 1) {  // sequence owning the item: last index with item_base[i] <= item
      const int mid = (lo + hi) >> 1;
      if (A.item_base[mid] <= item) lo = mid; else hi = mid;
    }
    int b = 0;
    while (b + 1 < A.n_batches && lo >= A.b[b + 1].seq_first) ++b;
    const int seq = lo - A.b[b].seq_first;
    const uint32_t r = item - A.item_base[lo];
    const int H = A.b[b].g.H;
    const int chunk = (int)(r / (uint32_t)H), head = (int)(r % (uint32_t)H);
    switch (A.b[b].g.dtype) {
      case FS_KV_FP16: process_item<FS_KV_FP16>(A, b, seq, chunk, head, item, smem); break;
      case FS_KV_FP8_E4M3: process_item<FS_KV_FP8_E4M3>(A, b, seq, chunk, head, item, smem); break;
      case FS_KV_INT8: process_item<FS_KV_INT8>(A, b, seq, chunk, head, item, smem); break;
      default: process_item<FS_KV_INT4>(A, b, seq, chunk, head, item, smem); break;
    }
  }
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
  const size_t smem = (size_t)(kWaves * 16 * kD + 3 * kWaves * 16) * sizeof(float);
  hipLaunchKernelGGL(mfma_attention_kernel, dim3(n_workgroups), dim3(kThreads), smem, s, A);
  return hipGetLastError();
}

}  // namespace fs
