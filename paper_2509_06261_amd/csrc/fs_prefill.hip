// MFMA paged prefill (chunked prefill) attention kernel for gfx950 (head_dim 128, all four KV formats).
//
// FineServe Sec. 2.1: the prefill phase processes the prompt's tokens, each attending to the tokens up to
// itself; Sec. 2.3: it is the compute-intensive phase; Sec. 4.2 schedules it in chunks.  Here a chunk's
// keys and values are first appended to the slab pool (fs_kv_append), then every query row of the chunk
// attends to the cached tokens 0..its own position, read from the pool exactly as decode attention reads
// them (same dequantization), through the sequence's block table (Sec. 5.1).
//
// Work decomposition: a work item is (sequence, KV head, tile of query tokens); the 16 logit columns of the
// MFMAs (see fs_mfma_tiles.h) are (query token, query head of the group) pairs, 16 / G tokens per block of 16
// columns.  One wave streams the cached tokens 0 .. last position of the tile once for all its columns;
// causality is a per-column sequence length, so only the tiles on the diagonal pay for masking.  Three kernels:
// prefill_kernel keeps one block of 16 columns per wave (two waves per SIMD); prefill_wide_kernel 2 or 4
// blocks (one wave per SIMD): a tile's K and V rows are then loaded, unpacked and transposed once for 32 or 64
// columns; prefill_wg_kernel (the default for launches with at least one item per compute unit) lets the waves
// of a workgroup share every unpacked K/V fragment through LDS.  Items of one (sequence, head) are neighbours in the queue, longest
// first, so that the waves streaming the same keys and values run side by side and share them through the
// L2.  Waves draw items from the same pooled ticket counters as the decode kernel.  A long context is
// streamed in segments, the wave's block-address table being refilled per segment.
#include <cstdlib>

// Prefill re-reads every K/V row once per query tile of its (sequence, head) -- from the L2 and the memory-side
// cache after the first time -- so its loads carry no non-temporal hint (decode, which reads every row once, hints
// its V loads; with the hint here config 2's prefill ran 6 % slower, 739 against 783 TFLOP/s on one box).
#define FS_NT_V 0
#include "fs_mfma_tiles.h"
#include "fs_prefill_index.h"

namespace fs {
namespace {

struct PrefillArgs {
  DevBatch b;                // geometry and the batch's pointers (q, tables, seq_lens, out, lse, FP8 scales)
  const int32_t* q_offsets;  // [n_seq + 1] first query row of each sequence's chunk
  uint32_t* header;          // workspace header: status word and the pools' ticket counters (layout of fs_attention.h)
  uint32_t* tile_first;      // [n_seq + 1] first query tile of each sequence
  int32_t tpt;               // query tokens per block of 16 logit columns: 16 / G
  int32_t ncb;               // column blocks per work item (1: prefill_kernel; 2, 4: prefill_wide_kernel)
  int32_t seg_runs;          // runs of 8 token slots streamed per refill of the block-address table (multiple of 4)
  int32_t table_entries;     // LDS table entries per wave
  int32_t n_rows;            // query rows in q / out (host value: every row index is clamped into it)
  int32_t tf_cache;          // workgroup kernels: 1 = tile_first is copied into LDS at kernel start
  int32_t whole_runs;        // 1 = tokens per block is a multiple of 8: run r starts at token 8 r, no run is shifted
  int32_t chunk_shift;       // workgroup kernels: log2 of the consecutive work items that go to one XCD
#ifdef FS_TIMELINE
  uint64_t* timeline;        // (timeline build) clock readings of the workgroup kernels, at the end of the workspace
#endif
};

// Timeline build (-DFS_TIMELINE, bench_timeline.py; never the product library): the workgroup kernels leave clock
// readings at the end of the workspace, which fs_prefill_workspace_bytes then includes.  Rows of eight 64-bit words:
// kPfTimelineGroups rows of workgroups (start, end, items, XCD, then the items' summed phases: entry -> address table
// in LDS, -> first sub-tiles staged, -> last step done, -> output written), then kPfTimelineItems rows of work items
// by item index (begin, end, sequence << 32 | KV head << 20 | query tile, workgroup | draw-and-barriers time << 32).
#ifdef FS_TIMELINE
constexpr uint64_t kPfTimelineGroups = 1024, kPfTimelineItems = 1ull << 18;
constexpr uint64_t kPfTimelineBytes = 64 * (kPfTimelineGroups + kPfTimelineItems);
#endif

constexpr int kPrepThreads = 1024;

// Query tiles per sequence -> tile_first (exclusive scan), validation flags, counter reset.  One workgroup.
__global__ __launch_bounds__(kPrepThreads) void prefill_prep_kernel(PrefillArgs P) {
  __shared__ uint32_t s_wave[kPrepThreads / 64];
  __shared__ uint32_t s_running;
  const DevBatch& B = P.b;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) {
    s_running = 0;
    P.header[kHdrStatus] = 0;
  }
  if (tid < kPools) P.header[kHdrPools + tid * kPoolStride] = 0;
  __syncthreads();
  const int max_len = (int)min((int64_t)B.max_blocks * B.g.T, (int64_t)0x7fffffff);
  for (int base = 0; base < B.n_seq; base += kPrepThreads) {
    const int i = base + tid;
    uint32_t v = 0;
    if (i < B.n_seq) {
      int len = B.seq_lens[i];
      int n_new = P.q_offsets[i + 1] - P.q_offsets[i];
      if (len < 1 || len > max_len || n_new < 0 || n_new > len) {
        atomicOr(P.header + kHdrStatus, 1u);
        len = len < 1 ? 1 : min(len, max_len);
        n_new = n_new < 0 ? 0 : min(n_new, len);
      }
      v = (uint32_t)((n_new + P.tpt * P.ncb - 1) / (P.tpt * P.ncb));
    }
    uint32_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t t = __shfl_up(incl, off, 64);
      if (lane >= off) incl += t;
    }
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    uint32_t before = s_running;
    for (int w = 0; w < wave; ++w) before += s_wave[w];
    if (i < B.n_seq) P.tile_first[i] = before + incl - v;
    __syncthreads();
    if (tid == kPrepThreads - 1) s_running = before + incl;
    __syncthreads();
  }
  if (tid == 0) P.tile_first[B.n_seq] = s_running;
}

template <int DT, int HD = kD>
__device__ void prefill_item(const PrefillArgs& P, int seq, int head, int qt, uint64_t* s_ptr) {
  constexpr int GP = 16;  // every logit column is live: one column per lane in the softmax
  const DevBatch& B = P.b;
  const DevGeom& g = B.g;
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));  // see the decode kernel: keeps lane constants out of the item loop
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int max_len = (int)min((int64_t)B.max_blocks * g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : min(len, max_len);
  int n_new = P.q_offsets[seq + 1] - P.q_offsets[seq];
  n_new = n_new < 0 ? 0 : min(n_new, len);
  const int r0 = qt * P.tpt;              // first query token of the tile within the chunk
  if (r0 >= n_new) return;                // (cannot happen with consistent inputs)
  const int first_pos = len - n_new + r0;  // its position in the sequence
  const int n_tok = min(P.tpt, n_new - r0);
  // column c = (query token c / G of the tile, query head c % G of the group)
  const int tok_c = c / G, hg_c = c - tok_c * G;
  const bool live = tok_c < n_tok;
  const int row_c = min(max(P.q_offsets[seq] + r0 + tok_c, 0), P.n_rows - 1);

  ItemCtx X;
  X.T = g.T;
  X.R = B.R;
  X.r_magic = B.r_magic;
  X.len_u = first_pos + n_tok;                  // the tile's last query sees this many tokens
  X.len = live ? first_pos + tok_c + 1 : 1;     // causality: a column sees the tokens up to its own position
  X.chunk_ptr = s_ptr;

  constexpr int NE = HD / 16;  // output columns NE c .. NE c + NE - 1 are this lane's
  u32x4 qb[HD / 32];
  float qsum;
  load_q<DT, true, HD>(B.q + ((int64_t)row_c * B.n_q + head * G + hg_c) * HD, live, j, qb, qsum);
  if constexpr (Fmt<DT>::kParBytes != 0) {
    qsum += __shfl_xor(qsum, 16, 64);
    qsum += __shfl_xor(qsum, 32, 64);
  }
  float alpha = B.sm_scale * kLog2e;
  if (DT == FS_KV_FP8_E4M3) alpha *= B.k_scale[head];

  StateT<HD> st;
#pragma unroll
  for (int e = 0; e < NE; ++e) st.acc[e] = float4v{0.f, 0.f, 0.f, 0.f};
  st.m = -INFINITY;
  st.l = 0.f;
  st.zc = 0.f;

  const int32_t* table = B.tables + (int64_t)seq * B.max_blocks;
  const uint8_t* head_base = B.layer_base + (uint64_t)head * g.head_chunk;
  const int n_run = n_runs(X.len_u, g.T, B.R);
  for (int v0 = 0; v0 < n_run; v0 += P.seg_runs) {
    X.v_end = min(n_run, v0 + P.seg_runs);
    X.k0 = div_runs(v0, B.R, B.r_magic);
    fill_table(s_ptr, table, head_base, g.block_budget, X.k0, div_runs(X.v_end - 1, B.R, B.r_magic) - X.k0 + 1, lane, B.n_blocks, P.header);
    stream_tiles<DT, GP, HD>(X, g, v0, qb, qsum, alpha, st, j, c);
  }

  // ---- output: per-column sums over the four lane groups, then the live rows straight from the accumulators ----
  st.l += __shfl_xor(st.l, 16, 64);
  st.l += __shfl_xor(st.l, 32, 64);
  if constexpr (Fmt<DT>::kParBytes != 0) {
    st.zc += __shfl_xor(st.zc, 16, 64);
    st.zc += __shfl_xor(st.zc, 32, 64);
  }
  const float v_static = DT == FS_KV_FP8_E4M3 ? B.v_scale[head] : 1.0f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int h = 4 * j + r;  // accumulator row r of this lane is logit column h; its m, l, zc live in lane c = h
    const float L = __shfl(st.l, h, 64), M = __shfl(st.m, h, 64), Z = __shfl(st.zc, h, 64);
    const int row_h = __shfl(row_c, h, 64);
    const int tok_h = h / G, hg_h = h - tok_h * G;
    if (tok_h < n_tok) {
      const float inv = 1.0f / L;
      uint32_t w[NE / 2];
#pragma unroll
      for (int q = 0; q < NE / 2; ++q) {
        float o[2];
#pragma unroll
        for (int z = 0; z < 2; ++z) {
          const int e = 2 * q + z;
          // integer formats: undo the 2^-24 of the subnormal encoding (and the 16 of INT4's odd code positions)
          const float f = DT == FS_KV_INT8 ? kTwo24 : (DT == FS_KV_INT4 ? ((e & 1) ? kTwo20 : kTwo24) : 1.0f);
          o[z] = st.acc[e][r] * f;
          if constexpr (Fmt<DT>::kParBytes != 0) o[z] += Z;
          o[z] *= v_static * inv;
        }
        const half2v hv = {(_Float16)o[0], (_Float16)o[1]};
        w[q] = h2u(hv);
      }
      const int64_t qrow = (int64_t)row_h * B.n_q + head * G + hg_h;
      _Float16* orow = B.out + qrow * HD + NE * c;
      if constexpr (NE == 4) {
        *reinterpret_cast<u32x2*>(orow) = u32x2{w[0], w[1]};
      } else {
#pragma unroll
        for (int q = 0; q < NE / 8; ++q)
          reinterpret_cast<u32x4*>(orow)[q] = u32x4{w[4 * q], w[4 * q + 1], w[4 * q + 2], w[4 * q + 3]};
      }
      if (c == 0 && B.lse) B.lse[qrow] = (M + __builtin_amdgcn_logf(L)) * kLn2;
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Wide variant: NCB blocks of 16 logit columns per wave.  A tile's K rows are unpacked once and multiplied
// with NCB query operands, its V rows are unpacked and transposed once and multiplied with NCB weight
// operands; per-token parameters are broadcast once.  Only the softmax itself is per block.  The accumulators
// (NCB x 32 registers) take the place of a second resident wave: the kernel runs one wave per SIMD.
// ---------------------------------------------------------------------------------------------------------
// Makes the query operand's loads complete here, once per item.  Their first real use is an MFMA inside the
// tile loop; left pending until there, the compiler's wait-count bookkeeping must assume at the loop head that
// they may still be in flight, and its wait for them also waits for the K/V loads issued just before -- the
// very loads the loop is arranged to keep in flight across a whole step.
__device__ __forceinline__ void settle_q(u32x4 (&q)[4]) {
  uint32_t any = 0;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) any |= q[ks][0] | q[ks][1] | q[ks][2] | q[ks][3];
  asm volatile("" ::"v"(any));
}

template <int NCB>
struct WideState {
  float4v acc[NCB][8];
  float m[NCB], l[NCB], zc[NCB];
};

// This file is compiled with VGPR-form MFMAs (-mllvm -amdgpu-mfma-vgpr-form, see build.py): accumulators, S^T
// results and operands all live in vector registers and the kernels use no AccVGPRs as MFMA operands.  With the
// default (accumulators in AccVGPRs, which the vector ALU cannot address) every S^T tile had to be read out with
// v_accvgpr_read before the softmax -- 16 of the ~100 vector instructions of a sub-tile -- and the rarely taken
// rescale of the accumulators needed explicit accvgpr moves in inline assembly to keep the register allocator
// from shuttling all of them between the register files on every tile.  256 vector registers per wave (two waves
// per SIMD) hold everything; measured against the AccVGPR build on one machine: + 10-14 % on every format.

// Moves the reference of column block cb (see the lazy online softmax of fs_mfma_tiles.h): tmax = this lane's
// largest logit of the tile for its column.
template <int DT, int NCB>
__device__ __forceinline__ void wide_move_reference(WideState<NCB>& st, int cb, float tmax, int j) {
  tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
  tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
  const float m_new = fmaxf(st.m[cb], tmax);  // finite: token 0 is seen by every column
  if (__all(st.m[cb] == -INFINITY)) {         // the item's first tile: nothing accumulated yet, nothing to rescale
    st.m[cb] = m_new;
    return;
  }
  const float corr = __builtin_amdgcn_exp2f(st.m[cb] - m_new);
  st.l[cb] *= corr;
  if constexpr (Fmt<DT>::kParBytes != 0) st.zc[cb] *= corr;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float cr = __shfl(corr, 4 * j + r, 64);  // column h keeps its factor in lane c = h
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[cb][e][r] *= cr;
  }
  st.m[cb] = m_new;
}

// One 32-token tile for NCB column blocks.  Order of work: all S^T MFMAs; the logits and, on the tiles that
// need it, their masks; the column maxima and one (rare) reference check for all column blocks; per column
// block the exponentials; the P V MFMAs.  A tile is interior when its four runs are whole (8 slots each, none
// repeated) and every column of the item sees all 32 tokens (the tile ends at or before the item's first query
// token): nothing is masked there, and the mask code is one skipped branch that touches no accumulator.
template <int DT, int NCB>
__device__ __forceinline__ void wide_tile(const ItemCtx& X, const DevGeom& g, Tile<DT, 16>& t, const u32x4 (&qb)[NCB][4],
                                          const float (&qsum)[NCB], const int (&len_cb)[NCB], float alpha, int first_pos,
                                          int vb, int vb_next, int j, int c, WideState<NCB>& st) {
  using F = Fmt<DT>;
  // ---- S^T = K Q^T for every column block ----
  float4v s[NCB][2];
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    u32x4 a[4];
    k_operands<DT>(t.k[u], a);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) acc = mfma(a[ks], qb[cb][ks], acc);
      s[cb][u] = acc;
    }
  }
  issue_k<DT, 16>(X, vb_next, j, c, t);

  const RunLoc L = locate(X, vb + j);  // X.len == X.len_u here: L.hi == L.hi_u
  const bool interior = __all(L.lo == 0 && L.tok0 + 8 <= first_pos + 1);  // wave-uniform
  // per-token dequantization factors, prepared by the lane that loaded the token's parameters, broadcast once
  float ka[8], kb[8], va[8], vb2[8];
  if constexpr (F::kParBytes != 0) {
    float pa, pb;
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
    static_for(std::make_integer_sequence<int, 8>{}, [&](auto I) {
      constexpr int i = decltype(I)::value;
      ka[i] = row_bcast<i>(pa);
      kb[i] = row_bcast<i>(pb);
      va[i] = row_bcast<8 + i>(pa);
      vb2[i] = row_bcast<8 + i>(pb);
    });
  }
  // logits in the base-2 domain (parameter formats) or raw products (FP16, FP8: their one common factor
  // alpha > 0 is applied inside the exponential's argument)
  float x[NCB][8];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = s[cb][i >> 2][i & 3];
      if constexpr (F::kParBytes != 0) x[cb][i] = fmaf(v, ka[i], kb[i] * qsum[cb]);
      else x[cb][i] = v;
    }
  if (!interior) {
    if constexpr (DT == FS_KV_FP16 || DT == FS_KV_FP8_E4M3) {
      // slots past the sequence's end may hold NaN/Inf bit patterns; 0 * NaN would poison the MFMA
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int w = 0; w < F::kVBytes / 4; ++w) t.v[i][w] = i < L.hi_u ? t.v[i][w] : 0u;
    }
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const int hi = min(L.hi_u, len_cb[cb] - L.tok0);  // causality: this lane's column sees tokens < len_cb
      const uint32_t n_ok = (uint32_t)max(hi - L.lo, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) x[cb][i] = (uint32_t)(i - L.lo) < n_ok ? x[cb][i] : -INFINITY;
    }
  }
  // ---- column maxima; the lazily moved reference (see fs_mfma_tiles.h) is checked once for all blocks ----
  float tmax[NCB];
  bool need = false;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    float mx = fmaxf(fmaxf(x[cb][0], x[cb][1]), x[cb][2]);
    mx = fmaxf(fmaxf(mx, x[cb][3]), x[cb][4]);
    mx = fmaxf(fmaxf(mx, x[cb][5]), x[cb][6]);
    mx = fmaxf(mx, x[cb][7]);
    if constexpr (F::kParBytes == 0) mx *= alpha;
    tmax[cb] = mx;
    need |= mx - st.m[cb] > kTau;
  }
  if (__any(need)) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) wide_move_reference<DT, NCB>(st, cb, tmax[cb], j);
  }
  // ---- weights ----
  u32x4 pk[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const float m = st.m[cb];
    if constexpr (F::kParBytes != 0) {
      float p[8], lsum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float e = __builtin_amdgcn_exp2f(x[cb][i] - m);
        lsum += e;
        p[i] = e * va[i];
        st.zc[cb] = fmaf(e, vb2[i], st.zc[cb]);
      }
      st.l[cb] += lsum;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const half2v h = {(_Float16)p[2 * q], (_Float16)p[2 * q + 1]};
        pk[cb][q] = h2u(h);
      }
    } else {
      // the running sum is taken over the weights as the MFMA sees them (rounded to fp16)
      const half2v one = {(_Float16)1.0f, (_Float16)1.0f};
      float l = st.l[cb];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float e0 = __builtin_amdgcn_exp2f(fmaf(x[cb][2 * q], alpha, -m));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(x[cb][2 * q + 1], alpha, -m));
        const half2v h = {(_Float16)e0, (_Float16)e1};
        pk[cb][q] = h2u(h);
        l = __builtin_amdgcn_fdot2(h, one, l, false);
      }
      st.l[cb] = l;
    }
  }
  // ---- V rows of the run -> B operands (8x8 in-register transpose), out += P V for every column block ----
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
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) st.acc[cb][e] = mfma(pk[cb], b, st.acc[cb][e]);
  }
  issue_v<DT, 16>(X, g, vb_next, j, c, t);
}

// One work item of the wide variant: (sequence, KV head, NCB consecutive 16-column query tiles).
template <int DT, int NCB>
__device__ void prefill_item_wide(const PrefillArgs& P, int seq, int head, int qt, uint64_t* s_ptr) {
  const DevBatch& B = P.b;
  const DevGeom& g = B.g;
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int max_len = (int)min((int64_t)B.max_blocks * g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : min(len, max_len);
  int n_new = P.q_offsets[seq + 1] - P.q_offsets[seq];
  n_new = n_new < 0 ? 0 : min(n_new, len);
  const int r0 = qt * P.tpt * NCB;  // first query token of the item within the chunk
  if (r0 >= n_new) return;
  const int first_pos = len - n_new + r0;
  const int n_tok = min(P.tpt * NCB, n_new - r0);
  const int tok_c = c / G, hg_c = c - tok_c * G;  // within a column block

  ItemCtx X;
  X.T = g.T;
  X.R = B.R;
  X.r_magic = B.r_magic;
  X.len_u = first_pos + n_tok;
  X.len = X.len_u;
  X.chunk_ptr = s_ptr;

  u32x4 qb[NCB][4];
  float qsum[NCB];
  int len_cb[NCB], row_cb[NCB];
  float alpha = B.sm_scale * kLog2e;
  if (DT == FS_KV_FP8_E4M3) alpha *= B.k_scale[head];
  WideState<NCB> st;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int tok = cb * P.tpt + tok_c;  // query token of this lane's column in block cb
    const bool live = tok_c < P.tpt && tok < n_tok;
    len_cb[cb] = live ? first_pos + tok + 1 : X.len_u;  // a dead column (q = 0, never written) sees everything
    row_cb[cb] = min(max(P.q_offsets[seq] + r0 + tok, 0), P.n_rows - 1);
    load_q<DT>(B.q + ((int64_t)row_cb[cb] * B.n_q + head * G + hg_c) * kD, live, j, qb[cb], qsum[cb]);
    settle_q(qb[cb]);
    if constexpr (Fmt<DT>::kParBytes != 0) {
      qsum[cb] += __shfl_xor(qsum[cb], 16, 64);
      qsum[cb] += __shfl_xor(qsum[cb], 32, 64);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[cb][e] = float4v{0.f, 0.f, 0.f, 0.f};
    st.m[cb] = -INFINITY;
    st.l[cb] = 0.f;
    st.zc[cb] = 0.f;
  }

  const int32_t* table = B.tables + (int64_t)seq * B.max_blocks;
  const uint8_t* head_base = B.layer_base + (uint64_t)head * g.head_chunk;
  const int n_run = n_runs(X.len_u, g.T, B.R);
  constexpr int NBUF = Fmt<DT>::kRing;
  for (int v0 = 0; v0 < n_run; v0 += P.seg_runs) {
    X.v_end = min(n_run, v0 + P.seg_runs);
    X.k0 = div_runs(v0, B.R, B.r_magic);
    fill_table(s_ptr, table, head_base, g.block_budget, X.k0, div_runs(X.v_end - 1, B.R, B.r_magic) - X.k0 + 1, lane, B.n_blocks, P.header);
    // the ring of stream_tiles (fs_mfma_tiles.h), with the wide tile step
    const int n_tiles = (X.v_end - v0 + 3) >> 2;
    Tile<DT, 16> t[NBUF];
    static_for(std::make_integer_sequence<int, NBUF>{}, [&](auto Bi) {
      constexpr int bi = decltype(Bi)::value;
      issue_k<DT, 16>(X, v0 + bi * 4, j, c, t[bi]);
      issue_v<DT, 16>(X, g, v0 + bi * 4, j, c, t[bi]);
    });
    for (int k0 = 0; k0 < n_tiles; k0 += NBUF) {
      static_for(std::make_integer_sequence<int, NBUF>{}, [&](auto Bi) {
        constexpr int bi = decltype(Bi)::value;
        const int vb = v0 + (k0 + bi) * 4;
        wide_tile<DT, NCB>(X, g, t[bi], qb, qsum, len_cb, alpha, first_pos, vb, vb + NBUF * 4, j, c, st);
      });
    }
  }

  const float v_static = DT == FS_KV_FP8_E4M3 ? B.v_scale[head] : 1.0f;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    float l = st.l[cb], zc = st.zc[cb];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if constexpr (Fmt<DT>::kParBytes != 0) {
      zc += __shfl_xor(zc, 16, 64);
      zc += __shfl_xor(zc, 32, 64);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int h = 4 * j + r;  // accumulator row r of this lane is logit column h of block cb
      const float L = __shfl(l, h, 64), M = __shfl(st.m[cb], h, 64), Z = __shfl(zc, h, 64);
      const int row_h = __shfl(row_cb[cb], h, 64);
      const int tok_h = h / G, hg_h = h - tok_h * G;
      if (tok_h < P.tpt && cb * P.tpt + tok_h < n_tok) {
        const float inv = 1.0f / L;
        u32x4 w;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float o[2];
#pragma unroll
          for (int z = 0; z < 2; ++z) {
            const int e = 2 * q + z;
            const float f = DT == FS_KV_INT8 ? kTwo24 : (DT == FS_KV_INT4 ? ((e & 1) ? kTwo20 : kTwo24) : 1.0f);
            o[z] = st.acc[cb][e][r] * f;
            if constexpr (Fmt<DT>::kParBytes != 0) o[z] += Z;
            o[z] *= v_static * inv;
          }
          const half2v hv = {(_Float16)o[0], (_Float16)o[1]};
          w[q] = h2u(hv);
        }
        const int64_t qrow = (int64_t)row_h * B.n_q + head * G + hg_h;
        *reinterpret_cast<u32x4*>(B.out + qrow * kD + 8 * c) = w;
        if (c == 0 && B.lse) B.lse[qrow] = (M + __builtin_amdgcn_logf(L)) * kLn2;
      }
    }
  }
}

// Which items a ticket pool holds.  The query tiles of one (sequence, KV head) stream the same keys and values,
// and each of the chip's eight XCDs has an L2 of its own: a pair's tiles must run on ONE XCD, side by side, for
// its K/V to be fetched from memory once instead of once per XCD (measured on a 0.58 GB cache: 36 GB fetched
// per launch with the tiles dealt round-robin over all XCDs).  The item list (sequence-major, then head, then
// tile) is therefore cut into chunks of consecutive items, chunk k belongs to XCD k % 8, and the 8
// pools of an XCD (pool = 8 s + xcd) take that XCD's items s, s + 8, ... in order.  A wave's home pool is one
// of its own XCD's (the XCC_ID hardware register says which); pools of other XCDs are only visited when the
// home pool has run dry, at the end of the launch.
static_assert(kPools == 64, "pool = 8 * sub-pool + XCD");
// chunk = 2^shift items = the workers resident per XCD (wave-level items: 128 waves, workgroup-level items: 32)
constexpr uint32_t kWaveChunkShift = 7, kWgChunkShift = 5;
__device__ __forceinline__ uint32_t home_pool(uint32_t worker) {  // worker: index among the workers of its XCD
  const uint32_t xcd = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7;  // hwreg(HW_REG_XCC_ID, 0, 4)
  return (worker & 7) * 8 + xcd;
}

// tf: tile_first, in global memory or its copy in LDS (ten dependent look-ups: a round trip to memory each otherwise)
__device__ __forceinline__ bool decode_item(const PrefillArgs& P, const uint32_t* tf, uint32_t item, uint32_t H, int& seq,
                                            int& head, int& qt) {
  return fs::decode_item(tf, P.b.n_seq, item, H, seq, head, qt);
}

// Drawing work items until none is left.  A wave first empties its home pool; after that it looks at all 64
// counters at once (lane p reads pool p's), moves to a pool that still holds items -- one of its own XCD's if
// there is one -- and goes on.  It leaves only when every pool is past its last item, so every item is taken
// whatever the grid size and wherever the workgroups landed.  The next ticket is drawn before the current item
// is processed.
struct ItemDraw {
  uint32_t pool, ticket;
};
__device__ __forceinline__ ItemDraw first_draw(uint32_t* header, uint32_t worker, int lane) {
  ItemDraw d{home_pool(worker), 0u};
  if (lane == 0) d.ticket = atomicAdd(header + kHdrPools + d.pool * kPoolStride, 1u);
  return d;
}
// The drawn item (and the next ticket drawn), or false when every pool is empty.
__device__ __forceinline__ bool next_item(ItemDraw& d, uint32_t* header, uint32_t total, uint32_t shift, int lane,
                                          uint32_t& item) {
  for (;;) {
    item = pool_item(d.pool, __builtin_amdgcn_readfirstlane(d.ticket), shift);
    if (item < total) break;
    const uint32_t cnt = __hip_atomic_load(header + kHdrPools + lane * kPoolStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint64_t left = __ballot(pool_item((uint32_t)lane, cnt, shift) < total);  // wave-uniform; counters only grow
    if (left == 0) return false;
    const uint64_t own = left & (0x0101010101010101ull << (d.pool & 7));
    if (own) left = own;
    const uint32_t r = (d.pool + 1) & 63;  // the first such pool after the current one, cyclically
    const uint64_t rot = r ? (left >> r) | (left << (64 - r)) : left;
    d.pool = (r + (uint32_t)__builtin_ctzll(rot)) & 63;
    if (lane == 0) d.ticket = atomicAdd(header + kHdrPools + d.pool * kPoolStride, 1u);
  }
  if (lane == 0) d.ticket = atomicAdd(header + kHdrPools + d.pool * kPoolStride, 1u);
  return true;
}

// One kernel per KV format: the model's format is known at launch, and a kernel that holds a single format's
// tile code leaves the register allocator a far smaller problem than a run-time switch over all four.
// WPS = waves per SIMD the kernel is built for (its register budget: 512 / WPS).  (Measured: a second wave of the
// 32-column kernel gains nothing; its loads already saturate the compute unit's vector memory pipeline.)
template <int DT, int NCB, int WPS>
__global__ __launch_bounds__(kThreads, WPS) void prefill_wide_kernel(PrefillArgs P) {
  extern __shared__ uint64_t smem64[];
  const DevBatch& B = P.b;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint64_t* s_ptr = smem64 + (size_t)wave * P.table_entries;
  const uint32_t H = (uint32_t)B.g.H;
  const uint32_t total = P.tile_first[B.n_seq] * H;
  ItemDraw d = first_draw(P.header, (blockIdx.x >> 3) * kWaves + wave, lane);
  for (uint32_t item; next_item(d, P.header, total, kWaveChunkShift, lane, item);) {
    int seq, head, qt;
    if (!decode_item(P, P.tile_first, item, H, seq, head, qt)) continue;
    prefill_item_wide<DT, NCB>(P, seq, head, qt, s_ptr);
  }
}

// ---------------------------------------------------------------------------------------------------------
// Workgroup variant.  Counters of the wave-level kernels show the compute unit's vector memory pipeline busy
// 92 % of the time: every wave fetches every K/V byte of its item itself, four times per compute unit.  Here
// the four waves of a workgroup take four neighbouring query tiles (64 logit columns each) of one (sequence,
// KV head) and walk the keys and values together, 128 tokens per step: wave w fetches sub-tile w (32 tokens) of
// the step, unpacks it, transposes its V rows, and leaves the finished MFMA operand fragments -- exactly what
// it would have fed its own MFMAs -- in LDS; after a barrier every wave multiplies all four sub-tiles from
// LDS.  Global loads, unpacking and transposes per wave drop to a quarter; the fragments are written and read
// lane-contiguously (16 bytes per lane), free of bank conflicts.  Two stages alternate, so one barrier per
// step suffices: a stage is rewritten only after the barrier that follows its last readers.
// Stage layout: K fragments [sub-tile][u][k-step][lane] 16 B, V fragments [sub-tile][e][lane] 16 B, per-token
// parameters [sub-tile][lane] 4 B.
constexpr uint32_t kFrag = 64 * 16;  // one operand fragment of a wave
// a stage of SUBS sub-tiles: K fragments, V fragments (8 KiB per sub-tile each), parameters
constexpr uint32_t stage_v(int subs) { return (uint32_t)subs * 8 * kFrag; }
constexpr uint32_t stage_par(int subs) { return 2 * (uint32_t)subs * 8 * kFrag; }
constexpr uint32_t stage_bytes(int subs) { return stage_par(subs) + (uint32_t)subs * 256; }
constexpr uint32_t kWgCtlBytes = 16;

template <int DT>
__device__ __forceinline__ void stage_k(uint8_t* stage, int sub, int lane, Tile<DT, 16>& t) {  // (K fragments lead the stage)
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    u32x4 a[4];
    k_operands<DT>(t.k[u], a);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      *reinterpret_cast<u32x4*>(stage + (uint32_t)((sub * 8 + u * 4 + ks) * kFrag) + lane * 16) = a[ks];
  }
}
template <int DT, int SUBS>
__device__ __forceinline__ void stage_v(uint8_t* stage, int sub, int lane, int j, Tile<DT, 16>& t, const ItemCtx& X, int vb) {
  using F = Fmt<DT>;
  if constexpr (DT == FS_KV_FP16 || DT == FS_KV_FP8_E4M3) {
    // slots past the sequence's end may hold NaN/Inf bit patterns; 0 * NaN would poison the MFMA
    const RunLoc L = locate(X, vb + j);
    if (!__all(L.hi_u >= 8)) {
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int q = 0; q < F::kVBytes / 4; ++q) t.v[i][q] = i < L.hi_u ? t.v[i][q] : 0u;
    }
  }
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
    *reinterpret_cast<u32x4*>(stage + stage_v(SUBS) + (uint32_t)((sub * 8 + e) * kFrag) + lane * 16) = b;
  }
  if constexpr (F::kParBytes != 0) *reinterpret_cast<uint32_t*>(stage + stage_par(SUBS) + sub * 256 + lane * 4) = t.par[0];
}

// ---- Staged dequantization (INT8 / INT4) ----------------------------------------------------------------------
// The staging wave may as well leave *dequantized* fp16 operands in LDS: (code - zero point) * scale, rounded to
// fp16 -- what an engine that dequantizes in front of its matrix cores feeds them.  Every consumer wave then runs
// the FP16 tile code (no per-logit scale, no zero-point terms: less than half the vector instructions per logit),
// and the conversion is paid once per workgroup instead of once per wave.  The codes are made exact fp16
// integers first (0x6400 | n = 1024 + n); the offset and the (integer) zero point are subtracted exactly, the
// multiplication by the scale rounds once (relative 2^-12).
__device__ __forceinline__ half2v splat_lo(uint32_t w) { return u2h(__builtin_amdgcn_perm(w, w, 0x01000100u)); }
__device__ __forceinline__ half2v splat_hi(uint32_t w) { return u2h(__builtin_amdgcn_perm(w, w, 0x03020302u)); }

// per-token constants of the dequantization: par = {scale, zero point} (INT4) or {scale} (INT8).  The INT4 zero
// point is an integer 0..15 (the quantizer rounds it), so 1024 + zp and 1024 + 16 zp are exact in fp16 and the
// offset of the integer encoding and the zero point leave in ONE exact subtraction.
template <int DT>
struct Deq {
  half2v sc, sc16, off, off16;
  __device__ __forceinline__ explicit Deq(uint32_t par) {
    const half2v c16 = {(_Float16)16.0f, (_Float16)16.0f}, r16 = {(_Float16)0.0625f, (_Float16)0.0625f};
    const half2v k1024 = {(_Float16)1024.0f, (_Float16)1024.0f}, k1152 = {(_Float16)1152.0f, (_Float16)1152.0f};
    sc = splat_lo(par);
    sc16 = sc * r16;
    if constexpr (DT == FS_KV_INT4) {
      const half2v zp = splat_hi(par);
      off = zp + k1024;
      off16 = zp * c16 + k1024;
    } else {
      off = k1152;  // 1024 + 128: the stored byte is the code + 128 after the sign flip
      off16 = k1152;
    }
  }
};

// Four registers of 8 stored codes -> (code - zp) * scale as packed fp16 (the subtraction exact, the product
// rounded once).  INT8: register p holds elements (2p, 2p + 1).  INT4: register p holds codes (p, p + 4); the odd
// registers hold them 16-fold (the nibble stays where it is stored), which the scale / 16 takes out again: every
// position ends up a plain value, with fp16's whole range.
template <int DT>
__device__ __forceinline__ void dequant8(const uint32_t* w, const Deq<DT>& q, uint32_t (&x)[4]) {
  if constexpr (DT == FS_KV_INT8) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t u = w[h] ^ 0x80808080u;  // code + 128, unsigned
      const uint32_t r0 = __builtin_amdgcn_perm(0x64646464u, u, 0x04010400u);  // halves 1024 + 128 + code
      const uint32_t r1 = __builtin_amdgcn_perm(0x64646464u, u, 0x04030402u);
      x[2 * h] = h2u((u2h(r0) - q.off) * q.sc);
      x[2 * h + 1] = h2u((u2h(r1) - q.off) * q.sc);
    }
  } else {
    const uint32_t w0 = w[0], w8 = w0 >> 8;
    const uint32_t r0 = (w0 & 0x000F000Fu) | 0x64006400u, r1 = (w0 & 0x00F000F0u) | 0x64006400u;  // 1024 + n, 1024 + 16 n
    const uint32_t r2 = (w8 & 0x000F000Fu) | 0x64006400u, r3 = (w8 & 0x00F000F0u) | 0x64006400u;
    x[0] = h2u((u2h(r0) - q.off) * q.sc);
    x[1] = h2u((u2h(r1) - q.off16) * q.sc16);
    x[2] = h2u((u2h(r2) - q.off) * q.sc);
    x[3] = h2u((u2h(r3) - q.off16) * q.sc16);
  }
}

// K parameters of the rows this lane stages: row c of half-tile u is slot 4u + (c & 3) of run c >> 2 (as issue_k)
template <int DT>
__device__ __forceinline__ void issue_kpar(const ItemCtx& X, const DevGeom& g, int vb, int c, uint32_t (&kpar)[2]) {
  using F = Fmt<DT>;
  const RunLoc L = locate(X, vb + (c >> 2));
  const gptr p = L.base + 2u * g.kv_tile + (uint32_t)((L.start + (c & 3)) * F::kParBytes);
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    if constexpr (F::kParBytes == 2) kpar[u] = *reinterpret_cast<const FS_GLOBAL uint16_t*>(p + u * 4 * F::kParBytes);
    else kpar[u] = *reinterpret_cast<const FS_GLOBAL uint32_t*>(p + u * 4 * F::kParBytes);
  }
}

template <int DT>
__device__ __forceinline__ void stage_k_deq(uint8_t* stage, int sub, int lane, Tile<DT, 16>& t, const uint32_t (&kpar)[2]) {
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    const Deq<DT> q(kpar[u]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      // the 8 codes of k-step ks: INT8 two dwords of load ks >> 1, INT4 dword ks of the one load
      uint32_t w[2];
      if constexpr (DT == FS_KV_INT8) {
        w[0] = t.k[u][ks >> 1][2 * (ks & 1)];
        w[1] = t.k[u][ks >> 1][2 * (ks & 1) + 1];
      } else {
        w[0] = t.k[u][0][ks];
        w[1] = 0u;
      }
      uint32_t x[4];
      dequant8<DT>(w, q, x);
      const u32x4 a = {x[0], x[1], x[2], x[3]};
      *reinterpret_cast<u32x4*>(stage + (uint32_t)((sub * 8 + u * 4 + ks) * kFrag) + lane * 16) = a;
    }
  }
}

template <int DT, int SUBS>
__device__ __forceinline__ void stage_v_deq(uint8_t* stage, int sub, int lane, int j, Tile<DT, 16>& t, const ItemCtx& X, int vb) {
  uint32_t vx[8][4];
  static_for(std::make_integer_sequence<int, 8>{}, [&](auto I) {
    constexpr int i = decltype(I)::value;
    // V parameters of slot i of the lane's run: held by lane 8 + i of the row
    const uint32_t par = __builtin_amdgcn_update_dpp(0u, t.par[0], 0x150 + 8 + i, 0xF, 0xF, false);
    const Deq<DT> q(par);
    dequant8<DT>(t.v[i], q, vx[i]);
  });
  // slots past the sequence's end may hold any codes and parameters (NaN / Inf after the conversion); 0 * NaN
  // would poison the MFMA
  const RunLoc L = locate(X, vb + j);
  if (!__all(L.hi_u >= 8)) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) vx[i][q] = i < L.hi_u ? vx[i][q] : 0u;
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int reg = DT == FS_KV_INT4 ? (e & 3) : (e >> 1);
    const uint32_t sel = (DT == FS_KV_INT4 ? (e >> 2) : (e & 1)) ? 0x07060302u : 0x05040100u;
    u32x4 b;
#pragma unroll
    for (int q = 0; q < 4; ++q) b[q] = __builtin_amdgcn_perm(vx[2 * q + 1][reg], vx[2 * q][reg], sel);
    *reinterpret_cast<u32x4*>(stage + stage_v(SUBS) + (uint32_t)((sub * 8 + e) * kFrag) + lane * 16) = b;
  }
}

// One staged 32-token sub-tile for the wave's column blocks: wide_tile with the operands read from LDS.
// VPRE: V fragments requested in front of the softmax (registers permitting)
template <int DT, int NCB, int SUBS, int VPRE = 0>
__device__ __forceinline__ void wg_tile(const uint8_t* stage, int sub, const ItemCtx& X, const u32x4 (&qb)[NCB][4],
                                        const float (&qsum)[NCB], const int (&len_cb)[NCB], float alpha, int first_pos,
                                        int vb, int lane, int j, int c, WideState<NCB>& st, bool whole_runs = false) {
  using F = Fmt<DT>;
  float4v s[NCB][2];
  // The wave raises its priority for its MFMA sections and drops it for the softmax: of the two waves of a SIMD
  // the one that feeds the matrix pipe goes first, the other's vector work fills in (+ 2.4-3.5 % measured).
  __builtin_amdgcn_s_setprio(1);
#pragma unroll
  for (int u = 0; u < 2; ++u) {
    u32x4 a[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      a[ks] = *reinterpret_cast<const u32x4*>(stage + (uint32_t)((sub * 8 + u * 4 + ks) * kFrag) + lane * 16);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      float4v acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) acc = mfma(a[ks], qb[cb][ks], acc);
      s[cb][u] = acc;
    }
  }
  __builtin_amdgcn_s_setprio(0);
  // the first V fragments are requested now, in front of the softmax's vector work, so that the P V MFMAs do not
  // start by waiting for LDS
  u32x4 vpre[VPRE > 0 ? VPRE : 1];
#pragma unroll
  for (int e = 0; e < VPRE; ++e)
    vpre[e] = *reinterpret_cast<const u32x4*>(stage + stage_v(SUBS) + (uint32_t)((sub * 8 + e) * kFrag) + lane * 16);
  // interior (wave-uniform): every token of the sub-tile lies at or before the wave's first query token and no run
  // is a shifted one -- nothing to mask.  With whole runs per block the test is scalar arithmetic and the run's
  // location is needed on the mask path only.
  RunLoc L;
  bool interior;
  if (F::kParBytes == 0 && whole_runs) {
    interior = vb + 4 <= X.v_end && 8 * (vb + 4) <= first_pos + 1;
    if (!interior) L = locate(X, vb + j);
  } else {
    L = locate(X, vb + j);
    interior = __all(L.lo == 0 && L.tok0 + 8 <= first_pos + 1);
  }
  float ka[8], kb[8], va[8], vb2[8];
  if constexpr (F::kParBytes != 0) {
    const uint32_t par = *reinterpret_cast<const uint32_t*>(stage + stage_par(SUBS) + sub * 256 + lane * 4);
    float pa, pb;
    const float sc = f16lo(par);
    const float zp = DT == FS_KV_INT4 ? f16hi(par) : 128.0f;
    if (c < 8) {  // K: logit = alpha * sc * (2^24 * S_raw - zp * qsum)
      pa = alpha * kTwo24 * sc;
      pb = -alpha * sc * zp;
    } else {      // V: p' = p * sc, zero-point term -p * sc * zp
      const bool ok = (c & 7) >= L.lo && (c & 7) < L.hi_u;  // a slot past the sequence may hold any bit pattern
      pa = ok ? sc : 0.f;
      pb = ok ? -sc * zp : 0.f;
    }
    static_for(std::make_integer_sequence<int, 8>{}, [&](auto I) {
      constexpr int i = decltype(I)::value;
      ka[i] = row_bcast<i>(pa);
      kb[i] = row_bcast<i>(pb);
      va[i] = row_bcast<8 + i>(pa);
      vb2[i] = row_bcast<8 + i>(pb);
    });
  }
  float x[NCB][8];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = s[cb][i >> 2][i & 3];
      if constexpr (F::kParBytes != 0) x[cb][i] = fmaf(v, ka[i], kb[i] * qsum[cb]);
      else x[cb][i] = v;
    }
  if (!interior) {
    // Blocks whose token count is no multiple of 8 end in a shifted run, whose first slots repeat tokens of the run
    // before: with 38 or 60 tokens per block most sub-tiles hold one.  Where every slot is a token that every
    // column sees, those repeats are all there is to mask.
    if (__all(L.tok0 + 8 <= first_pos + 1)) {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int i = 0; i < 8; ++i) x[cb][i] = i >= L.lo ? x[cb][i] : -INFINITY;
    } else {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        const int hi = min(L.hi_u, len_cb[cb] - L.tok0);  // causality: this lane's column sees tokens < len_cb
        const uint32_t n_ok = (uint32_t)max(hi - L.lo, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) x[cb][i] = (uint32_t)(i - L.lo) < n_ok ? x[cb][i] : -INFINITY;
      }
    }
  }
  float tmax[NCB];
  bool need = false;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    float mx = fmaxf(fmaxf(x[cb][0], x[cb][1]), x[cb][2]);
    mx = fmaxf(fmaxf(mx, x[cb][3]), x[cb][4]);
    mx = fmaxf(fmaxf(mx, x[cb][5]), x[cb][6]);
    mx = fmaxf(mx, x[cb][7]);
    if constexpr (F::kParBytes == 0) mx *= alpha;
    tmax[cb] = mx;
    need |= mx - st.m[cb] > kTau;
  }
  if (__any(need)) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) wide_move_reference<DT, NCB>(st, cb, tmax[cb], j);
  }
  u32x4 pk[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const float m = st.m[cb];
    if constexpr (F::kParBytes != 0) {
      float p[8], lsum = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const float e = __builtin_amdgcn_exp2f(x[cb][i] - m);
        lsum += e;
        p[i] = e * va[i];
        st.zc[cb] = fmaf(e, vb2[i], st.zc[cb]);
      }
      st.l[cb] += lsum;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const half2v h = {(_Float16)p[2 * q], (_Float16)p[2 * q + 1]};
        pk[cb][q] = h2u(h);
      }
    } else {
      const half2v one = {(_Float16)1.0f, (_Float16)1.0f};
      float l = st.l[cb];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float e0 = __builtin_amdgcn_exp2f(fmaf(x[cb][2 * q], alpha, -m));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(x[cb][2 * q + 1], alpha, -m));
        const half2v h = {(_Float16)e0, (_Float16)e1};
        pk[cb][q] = h2u(h);
        l = __builtin_amdgcn_fdot2(h, one, l, false);
      }
      st.l[cb] = l;
    }
  }
  __builtin_amdgcn_s_setprio(1);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    u32x4 b;
    if (e < VPRE) b = vpre[e];
    else b = *reinterpret_cast<const u32x4*>(stage + stage_v(SUBS) + (uint32_t)((sub * 8 + e) * kFrag) + lane * 16);
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) st.acc[cb][e] = mfma(pk[cb], b, st.acc[cb][e]);
  }
}

// One work item of the workgroup variant: (sequence, KV head, NW x NCB consecutive 16-column query tiles): NW waves
// of NCB column blocks each walk K/V in steps of SUBS sub-tiles (32 tokens each).  With NW == SUBS every wave fetches
// and stages K and V of sub-tile w; with NW == 2 SUBS waves 0..SUBS-1 stage the K fragments of sub-tile w and the
// others the V fragments and parameters of sub-tile w - SUBS.  Built variants: 8 waves x 2 blocks, 4 sub-tiles per
// step, one workgroup per compute unit (two waves per SIMD, so that one's softmax runs under the other's MFMAs);
// 4 x 4, 4 sub-tiles (one wave per SIMD).  (A third one -- 4 x 2 with 2 sub-tiles per step, two workgroups per
// compute unit -- passed its small cases but ended a full-size two-model run with the GPU faulted or hung; the
// cause was not found and the variant is no longer built.)
// smem: two stages, then the workgroup's block-address table.
// DEQ (INT8 / INT4 only): the staging waves dequantize, the tile code is the FP16 one.
template <int DT, int NW, int NCB, int SUBS, bool DEQ = false>
__device__ void prefill_item_wg(const PrefillArgs& P, int seq, int head, int qt, uint8_t* smem, uint64_t* s_tab, int w) {
  static_assert(NW == SUBS || NW == 2 * SUBS, "staging roles");
#ifdef FS_TIMELINE
  uint64_t tl_ph[5] = {(uint64_t)wall_clock64(), 0, 0, 0, 0};
#endif
  static_assert(!DEQ || Fmt<DT>::kParBytes != 0, "staged dequantization is for the formats with per-token parameters");
  constexpr int CDT = DEQ ? FS_KV_FP16 : DT;  // the format the consumer code sees
  // V fragments read ahead of the softmax: what the format's register budget leaves room for (two waves per SIMD)
  constexpr int kVPre = NW != 8 ? 0 : (DEQ && DT == FS_KV_INT4 ? 8 : 4);
  const bool whole_runs = P.whole_runs != 0;  // (uniform)
  const bool does_k = NW == SUBS || w < SUBS, does_v = NW == SUBS || w >= SUBS;  // wave-uniform staging roles
  const int sw = w % SUBS;                                                       // the sub-tile this wave stages
  const DevBatch& B = P.b;
  const DevGeom& g = B.g;
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int max_len = (int)min((int64_t)B.max_blocks * g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : min(len, max_len);
  int n_new = P.q_offsets[seq + 1] - P.q_offsets[seq];
  n_new = n_new < 0 ? 0 : min(n_new, len);
  const int qw = P.tpt * NCB;                 // query tokens per wave
  const int r0_wg = qt * qw * NW;             // first query token of the item within the chunk
  if (r0_wg >= n_new) return;                 // (cannot happen with consistent inputs; uniform over the workgroup)
  const int n_tok_wg = min(qw * NW, n_new - r0_wg);
  const int r0 = r0_wg + w * qw;              // this wave's share
  const int n_tok = max(0, min(qw, n_tok_wg - w * qw));
  const int first_pos = len - n_new + r0;
  const int tok_c = c / G, hg_c = c - tok_c * G;

  ItemCtx X;  // of the workgroup: everything its last query token sees
  X.T = g.T;
  X.R = B.R;
  X.r_magic = B.r_magic;
  X.len_u = len - n_new + r0_wg + n_tok_wg;
  X.len = X.len_u;
  X.chunk_ptr = s_tab;

  u32x4 qb[NCB][4];
  float qsum[NCB];
  int len_cb[NCB], row_cb[NCB];
  float alpha = B.sm_scale * kLog2e;
  if (DT == FS_KV_FP8_E4M3) alpha *= B.k_scale[head];
  WideState<NCB> st;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int tok = cb * P.tpt + tok_c;  // query token of this lane's column in block cb
    const bool live = tok_c < P.tpt && tok < n_tok;
    len_cb[cb] = live ? first_pos + tok + 1 : X.len_u;  // a dead column (q = 0, never written) sees everything
    row_cb[cb] = min(max(P.q_offsets[seq] + r0 + tok, 0), P.n_rows - 1);
    load_q<DT, !DEQ>(B.q + ((int64_t)row_cb[cb] * B.n_q + head * G + hg_c) * kD, live, j, qb[cb], qsum[cb]);
    if constexpr (Fmt<CDT>::kParBytes != 0) {
      qsum[cb] += __shfl_xor(qsum[cb], 16, 64);
      qsum[cb] += __shfl_xor(qsum[cb], 32, 64);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[cb][e] = float4v{0.f, 0.f, 0.f, 0.f};
    st.m[cb] = -INFINITY;
    st.l[cb] = 0.f;
    st.zc[cb] = 0.f;
  }

  const int32_t* table = B.tables + (int64_t)seq * B.max_blocks;
  const uint8_t* head_base = B.layer_base + (uint64_t)head * g.head_chunk;
  const int n_run = n_runs(X.len_u, g.T, B.R);
  for (int v0 = 0; v0 < n_run; v0 += P.seg_runs) {
    X.v_end = min(n_run, v0 + P.seg_runs);
    X.k0 = div_runs(v0, B.R, B.r_magic);
    {
      // the previous segment's (or item's) last barrier lies behind every use of the old table
      const int nb = div_runs(X.v_end - 1, B.R, B.r_magic) - X.k0 + 1;
      for (int i = threadIdx.x; i < nb; i += NW * 64)
        s_tab[i] = reinterpret_cast<uint64_t>(head_base + (uint64_t)checked_block(table[X.k0 + i], B.n_blocks, P.header) * g.block_budget);
      __syncthreads();
#ifdef FS_TIMELINE
      if (v0 == 0) tl_ph[1] = wall_clock64();
#endif
    }
    const int n_super = (X.v_end - v0 + 4 * SUBS - 1) / (4 * SUBS);
    Tile<DT, 16> t;
    uint32_t kpar[2] = {0u, 0u};  // (DEQ) K parameters of the rows this lane stages
    // fetch / stage this wave's share of the sub-tile that starts at run vb
    auto fetch = [&](int vb) {
      if (does_k) {
        issue_k<DT, 16>(X, vb, j, c, t);
        if constexpr (DEQ) issue_kpar<DT>(X, g, vb, c, kpar);
      }
      if (does_v) issue_v<DT, 16>(X, g, vb, j, c, t);
    };
    auto stage_to = [&](uint8_t* stage, int vb) {
      if constexpr (DEQ) {
        if (does_k) stage_k_deq<DT>(stage, sw, lane, t, kpar);
        if (does_v) stage_v_deq<DT, SUBS>(stage, sw, lane, j, t, X, vb);
      } else {
        if (does_k) stage_k<DT>(stage, sw, lane, t);
        if (does_v) stage_v<DT, SUBS>(stage, sw, lane, j, t, X, vb);
      }
    };
    fetch(v0 + 4 * sw);
    stage_to(smem, v0 + 4 * sw);
    __syncthreads();
#ifdef FS_TIMELINE
    if (v0 == 0) tl_ph[2] = wall_clock64();
#endif
    // the query operands' loads, issued before the table and the first K/V fetch, are collected here
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) settle_q(qb[cb]);
    for (int i = 0; i < n_super; ++i) {
      // next step's sub-tile of this wave; the segment's last step fetches and stages nothing (the wait in stage_to
      // is for this step's fetch alone, so the condition costs the compiler's wait counts nothing)
      const int vb_next = v0 + (i + 1) * 4 * SUBS + 4 * sw;
      const bool more = i + 1 < n_super;  // wave-uniform
      if (more) fetch(vb_next);
      const uint8_t* stage = smem + (uint32_t)(i & 1) * stage_bytes(SUBS);
      // A wave with query tokens multiplies every sub-tile of the step, also those past its own diagonal or past
      // the segment's end (fully masked there: weights 0 over finite operands; at most two per item).  A wave
      // WITHOUT query tokens (a ragged last item of a chunk; chunks shorter than the workgroup's 16 NW / G tokens)
      // only stages its share of K/V and leaves the SIMD to its sibling.
      if (n_tok > 0) {
#pragma unroll 1  // (unrolled by two: measured 0.5 % slower)
        for (int sub = 0; sub < SUBS; ++sub)
          wg_tile<CDT, NCB, SUBS, kVPre>(stage, sub, X, qb, qsum, len_cb, alpha, first_pos, v0 + (i * SUBS + sub) * 4, lane, j, c,
                                         st, whole_runs);
      }
      uint8_t* next = smem + (uint32_t)((i + 1) & 1) * stage_bytes(SUBS);
      if (more) stage_to(next, vb_next);
      __syncthreads();  // (also after the last step: the next staging overwrites what other waves may still read)
    }
  }
#ifdef FS_TIMELINE
  tl_ph[3] = wall_clock64();
#endif
  if (n_tok == 0) return;

  const float v_static = DT == FS_KV_FP8_E4M3 ? B.v_scale[head] : 1.0f;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    float l = st.l[cb], zc = st.zc[cb];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if constexpr (Fmt<CDT>::kParBytes != 0) {
      zc += __shfl_xor(zc, 16, 64);
      zc += __shfl_xor(zc, 32, 64);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int h = 4 * j + r;  // accumulator row r of this lane is logit column h of block cb
      const float L = __shfl(l, h, 64), M = __shfl(st.m[cb], h, 64), Z = __shfl(zc, h, 64);
      const int row_h = __shfl(row_cb[cb], h, 64);
      const int tok_h = h / G, hg_h = h - tok_h * G;
      if (tok_h < P.tpt && cb * P.tpt + tok_h < n_tok) {
        const float inv = 1.0f / L;
        u32x4 wv;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float o[2];
#pragma unroll
          for (int z = 0; z < 2; ++z) {
            const int e = 2 * q + z;
            const float f = CDT == FS_KV_INT8 ? kTwo24 : (CDT == FS_KV_INT4 ? ((e & 1) ? kTwo20 : kTwo24) : 1.0f);
            o[z] = st.acc[cb][e][r] * f;
            if constexpr (Fmt<CDT>::kParBytes != 0) o[z] += Z;
            o[z] *= v_static * inv;
          }
          const half2v hv = {(_Float16)o[0], (_Float16)o[1]};
          wv[q] = h2u(hv);
        }
        const int64_t qrow = (int64_t)row_h * B.n_q + head * G + hg_h;
        *reinterpret_cast<u32x4*>(B.out + qrow * kD + 8 * c) = wv;
        if (c == 0 && B.lse) B.lse[qrow] = (M + __builtin_amdgcn_logf(L)) * kLn2;
      }
    }
  }
#ifdef FS_TIMELINE
  if (threadIdx.x == 0 && blockIdx.x < kPfTimelineGroups) {
    uint64_t* row = P.timeline + 8 * blockIdx.x;
    tl_ph[4] = wall_clock64();
    for (int k = 0; k < 4; ++k) row[4 + k] += tl_ph[k + 1] - tl_ph[k];
  }
#endif
}

// ---------------------------------------------------------------------------------------------------------
// Software-pipelined workgroup variant (4 waves x 64 columns, one wave per SIMD).  The compiler emits a tile's
// MFMAs and its softmax as separate bursts, and the step barrier keeps the waves of a SIMD in phase, so in the
// variants above the matrix cores idle during every softmax.  Here one wave overlaps the two itself: while the
// vector ALU exponentiates sub-tile s, the MFMAs of S^T for sub-tile s + 1 are issued between its instructions
// (block 1); while the MFMAs of P V for sub-tile s run, the vector ALU turns the new S^T into logits and column
// maxima (block 2); scheduling-group barriers pin the interleave (one MFMA, then a few vector instructions).
// The pipeline is restarted at every step (S^T of the step's first sub-tile runs alone; block 1 of the last
// sub-tile multiplies the step's first sub-tile again and discards it): carrying it across the step barrier
// would let a fast wave overwrite a stage that a slow wave still reads.
// ---------------------------------------------------------------------------------------------------------
template <int DT, int NCB>
struct Logits {
  float x[NCB][8];   // logits (parameter formats) or raw products (FP16, FP8)
  float tmax[NCB];   // column maxima, base-2 domain
  float va[8], vb2[8];  // parameter formats: per-token V factors for the weights of this sub-tile
};

// S^T accumulators -> logits, masks, column maxima.  Returns whether some column's reference must move.
template <int DT, int NCB, int SUBS>
__device__ __forceinline__ bool make_logits(const float4v (&s)[NCB][2], const uint8_t* stage, int sub, const ItemCtx& X,
                                            const float (&qsum)[NCB], const int (&len_cb)[NCB], float alpha, int first_pos,
                                            int vb, int lane, int c, const WideState<NCB>& st, Logits<DT, NCB>& out) {
  using F = Fmt<DT>;
  const RunLoc L = locate(X, vb + (lane >> 4));
  const bool interior = __all(L.lo == 0 && L.tok0 + 8 <= first_pos + 1);  // wave-uniform
  float ka[8], kb[8];
  if constexpr (F::kParBytes != 0) {
    const uint32_t par = *reinterpret_cast<const uint32_t*>(stage + stage_par(SUBS) + sub * 256 + lane * 4);
    float pa, pb;
    const float sc = f16lo(par);
    const float zp = DT == FS_KV_INT4 ? f16hi(par) : 128.0f;
    if (c < 8) {
      pa = alpha * kTwo24 * sc;
      pb = -alpha * sc * zp;
    } else {
      const bool ok = (c & 7) >= L.lo && (c & 7) < L.hi_u;
      pa = ok ? sc : 0.f;
      pb = ok ? -sc * zp : 0.f;
    }
    static_for(std::make_integer_sequence<int, 8>{}, [&](auto I) {
      constexpr int i = decltype(I)::value;
      ka[i] = row_bcast<i>(pa);
      kb[i] = row_bcast<i>(pb);
      out.va[i] = row_bcast<8 + i>(pa);
      out.vb2[i] = row_bcast<8 + i>(pb);
    });
  }
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float v = s[cb][i >> 2][i & 3];
      if constexpr (F::kParBytes != 0) out.x[cb][i] = fmaf(v, ka[i], kb[i] * qsum[cb]);
      else out.x[cb][i] = v;
    }
  auto maxima = [&]() {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      float mx = fmaxf(fmaxf(out.x[cb][0], out.x[cb][1]), out.x[cb][2]);
      mx = fmaxf(fmaxf(mx, out.x[cb][3]), out.x[cb][4]);
      mx = fmaxf(fmaxf(mx, out.x[cb][5]), out.x[cb][6]);
      mx = fmaxf(mx, out.x[cb][7]);
      if constexpr (F::kParBytes == 0) mx *= alpha;
      out.tmax[cb] = mx;
    }
  };
  maxima();  // in the straight-line part, beside the caller's MFMAs; redone below on the rare masked tiles
  __builtin_amdgcn_sched_barrier(0);
  if (!interior) {
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) {
      const int hi = min(L.hi_u, len_cb[cb] - L.tok0);
      const uint32_t n_ok = (uint32_t)max(hi - L.lo, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) out.x[cb][i] = (uint32_t)(i - L.lo) < n_ok ? out.x[cb][i] : -INFINITY;
    }
    maxima();
  }
  bool need = false;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) need |= out.tmax[cb] - st.m[cb] > kTau;
  return need;
}

template <int DT>
__device__ void prefill_item_wgp(const PrefillArgs& P, int seq, int head, int qt, uint8_t* smem, uint64_t* s_tab, int w) {
  constexpr int NW = 4, NCB = 4, SUBS = 4;
  using F = Fmt<DT>;
  const DevBatch& B = P.b;
  const DevGeom& g = B.g;
  int lane = threadIdx.x & 63;
  asm volatile("" : "+v"(lane));
  const int j = lane >> 4, c = lane & 15;
  const int G = B.G;
  const int max_len = (int)min((int64_t)B.max_blocks * g.T, (int64_t)0x7fffffff);
  int len = B.seq_lens[seq];
  len = len < 1 ? 1 : min(len, max_len);
  int n_new = P.q_offsets[seq + 1] - P.q_offsets[seq];
  n_new = n_new < 0 ? 0 : min(n_new, len);
  const int qw = P.tpt * NCB;
  const int r0_wg = qt * qw * NW;
  if (r0_wg >= n_new) return;
  const int n_tok_wg = min(qw * NW, n_new - r0_wg);
  const int r0 = r0_wg + w * qw;
  const int n_tok = max(0, min(qw, n_tok_wg - w * qw));
  const int first_pos = len - n_new + r0;
  const int tok_c = c / G, hg_c = c - tok_c * G;

  ItemCtx X;
  X.T = g.T;
  X.R = B.R;
  X.r_magic = B.r_magic;
  X.len_u = len - n_new + r0_wg + n_tok_wg;
  X.len = X.len_u;
  X.chunk_ptr = s_tab;

  u32x4 qb[NCB][4];
  float qsum[NCB];
  int len_cb[NCB], row_cb[NCB];
  float alpha = B.sm_scale * kLog2e;
  if (DT == FS_KV_FP8_E4M3) alpha *= B.k_scale[head];
  WideState<NCB> st;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int tok = cb * P.tpt + tok_c;
    const bool live = tok_c < P.tpt && tok < n_tok;
    len_cb[cb] = live ? first_pos + tok + 1 : X.len_u;
    row_cb[cb] = min(max(P.q_offsets[seq] + r0 + tok, 0), P.n_rows - 1);
    load_q<DT>(B.q + ((int64_t)row_cb[cb] * B.n_q + head * G + hg_c) * kD, live, j, qb[cb], qsum[cb]);
    if constexpr (F::kParBytes != 0) {
      qsum[cb] += __shfl_xor(qsum[cb], 16, 64);
      qsum[cb] += __shfl_xor(qsum[cb], 32, 64);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) st.acc[cb][e] = float4v{0.f, 0.f, 0.f, 0.f};
    st.m[cb] = -INFINITY;
    st.l[cb] = 0.f;
    st.zc[cb] = 0.f;
  }

  const int32_t* table = B.tables + (int64_t)seq * B.max_blocks;
  const uint8_t* head_base = B.layer_base + (uint64_t)head * g.head_chunk;
  const int n_run = n_runs(X.len_u, g.T, B.R);
  for (int v0 = 0; v0 < n_run; v0 += P.seg_runs) {
    X.v_end = min(n_run, v0 + P.seg_runs);
    X.k0 = div_runs(v0, B.R, B.r_magic);
    {
      const int nb = div_runs(X.v_end - 1, B.R, B.r_magic) - X.k0 + 1;
      for (int i = threadIdx.x; i < nb; i += NW * 64)
        s_tab[i] = reinterpret_cast<uint64_t>(head_base + (uint64_t)checked_block(table[X.k0 + i], B.n_blocks, P.header) * g.block_budget);
      __syncthreads();
    }
    const int n_super = (X.v_end - v0 + 4 * SUBS - 1) / (4 * SUBS);
    Tile<DT, 16> t;
    issue_k<DT, 16>(X, v0 + 4 * w, j, c, t);
    issue_v<DT, 16>(X, g, v0 + 4 * w, j, c, t);
    stage_k<DT>(smem, w, lane, t);
    stage_v<DT, SUBS>(smem, w, lane, j, t, X, v0 + 4 * w);
    __syncthreads();
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) settle_q(qb[cb]);  // (issued before the table and the first K/V fetch)
    for (int i = 0; i < n_super; ++i) {
      const int vb_next = v0 + (i + 1) * 4 * SUBS + 4 * w;
      issue_k<DT, 16>(X, vb_next, j, c, t);
      issue_v<DT, 16>(X, g, vb_next, j, c, t);
      const uint8_t* stage = smem + (uint32_t)(i & 1) * stage_bytes(SUBS);
      const uint8_t* lane_base = stage + lane * 16;
      // ---- pipeline start: S^T and logits of the step's first sub-tile ----
      u32x4 kf[2][4];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) kf[u][ks] = *reinterpret_cast<const u32x4*>(lane_base + (uint32_t)((u * 4 + ks) * kFrag));
      float4v sn[NCB][2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
          float4v a4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) a4 = mfma(kf[u][ks], qb[cb][ks], a4);
          sn[cb][u] = a4;
        }
      Logits<DT, NCB> cur;
      if (__any(make_logits<DT, NCB, SUBS>(sn, stage, 0, X, qsum, len_cb, alpha, first_pos, v0 + i * 4 * SUBS, lane, c, st, cur))) {
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) wide_move_reference<DT, NCB>(st, cb, cur.tmax[cb], j);
      }
#pragma unroll 1  // (unrolled by two: measured 0.5 % slower)
      for (int sub = 0; sub < SUBS; ++sub) {
        const int nsub = (sub + 1) & (SUBS - 1);  // after the last sub-tile: the first again, its result unused
        // ---- block 1: S^T of sub-tile nsub (MFMA) beside the exponentials of sub-tile sub (vector ALU) ----
        u32x4 vf[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vf[e] = *reinterpret_cast<const u32x4*>(lane_base + stage_v(SUBS) + (uint32_t)((sub * 8 + e) * kFrag));
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks)
            kf[u][ks] = *reinterpret_cast<const u32x4*>(lane_base + (uint32_t)((nsub * 8 + u * 4 + ks) * kFrag));
#pragma unroll
        for (int u = 0; u < 2; ++u)
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb) {
            float4v a4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) a4 = mfma(kf[u][ks], qb[cb][ks], a4);
            sn[cb][u] = a4;
          }
        u32x4 pk[NCB];
#pragma unroll
        for (int cb = 0; cb < NCB; ++cb) {
          const float m = st.m[cb];
          if constexpr (F::kParBytes != 0) {
            float pw[8], lsum = 0.f;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              const float ex = __builtin_amdgcn_exp2f(cur.x[cb][q] - m);
              lsum += ex;
              pw[q] = ex * cur.va[q];
              st.zc[cb] = fmaf(ex, cur.vb2[q], st.zc[cb]);
            }
            st.l[cb] += lsum;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const half2v h = {(_Float16)pw[2 * q], (_Float16)pw[2 * q + 1]};
              pk[cb][q] = h2u(h);
            }
          } else {
            const half2v one = {(_Float16)1.0f, (_Float16)1.0f};
            float l = st.l[cb];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float e0 = __builtin_amdgcn_exp2f(fmaf(cur.x[cb][2 * q], alpha, -m));
              const float e1 = __builtin_amdgcn_exp2f(fmaf(cur.x[cb][2 * q + 1], alpha, -m));
              const half2v h = {(_Float16)e0, (_Float16)e1};
              pk[cb][q] = h2u(h);
              l = __builtin_amdgcn_fdot2(h, one, l, false);
            }
            st.l[cb] = l;
          }
        }
        // one MFMA, then a few vector instructions, 32 times
#pragma unroll
        for (int r = 0; r < 2 * NCB * 4; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);  // VALU
          __builtin_amdgcn_sched_group_barrier(0x400, 1, 0);  // transcendental
        }
        __builtin_amdgcn_sched_barrier(0);
        // ---- block 2: P V of sub-tile sub (MFMA) beside the logits of sub-tile nsub (vector ALU) ----
#pragma unroll
        for (int e = 0; e < 8; ++e)
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb) st.acc[cb][e] = mfma(pk[cb], vf[e], st.acc[cb][e]);
#pragma unroll
        for (int r = 0; r < 8 * NCB; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);  // MFMA
          __builtin_amdgcn_sched_group_barrier(0x002, 2, 1);  // VALU
        }
        const bool need = make_logits<DT, NCB, SUBS>(sn, stage, nsub, X, qsum, len_cb, alpha, first_pos,
                                                     v0 + (i * SUBS + nsub) * 4, lane, c, st, cur);
        if (sub + 1 < SUBS && __any(need)) {  // (the wrapped-around sub-tile's logits are discarded)
#pragma unroll
          for (int cb = 0; cb < NCB; ++cb) wide_move_reference<DT, NCB>(st, cb, cur.tmax[cb], j);
        }
      }
      uint8_t* next = smem + (uint32_t)((i + 1) & 1) * stage_bytes(SUBS);
      stage_k<DT>(next, w, lane, t);
      stage_v<DT, SUBS>(next, w, lane, j, t, X, vb_next);
      __syncthreads();
    }
  }
  if (n_tok == 0) return;

  const float v_static = DT == FS_KV_FP8_E4M3 ? B.v_scale[head] : 1.0f;
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    float l = st.l[cb], zc = st.zc[cb];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if constexpr (F::kParBytes != 0) {
      zc += __shfl_xor(zc, 16, 64);
      zc += __shfl_xor(zc, 32, 64);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int h = 4 * j + r;
      const float Lh = __shfl(l, h, 64), M = __shfl(st.m[cb], h, 64), Z = __shfl(zc, h, 64);
      const int row_h = __shfl(row_cb[cb], h, 64);
      const int tok_h = h / G, hg_h = h - tok_h * G;
      if (tok_h < P.tpt && cb * P.tpt + tok_h < n_tok) {
        const float inv = 1.0f / Lh;
        u32x4 wv;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float o[2];
#pragma unroll
          for (int z = 0; z < 2; ++z) {
            const int e = 2 * q + z;
            const float f = DT == FS_KV_INT8 ? kTwo24 : (DT == FS_KV_INT4 ? ((e & 1) ? kTwo20 : kTwo24) : 1.0f);
            o[z] = st.acc[cb][e][r] * f;
            if constexpr (F::kParBytes != 0) o[z] += Z;
            o[z] *= v_static * inv;
          }
          const half2v hv = {(_Float16)o[0], (_Float16)o[1]};
          wv[q] = h2u(hv);
        }
        const int64_t qrow = (int64_t)row_h * B.n_q + head * G + hg_h;
        *reinterpret_cast<u32x4*>(B.out + qrow * kD + 8 * c) = wv;
        if (c == 0 && B.lse) B.lse[qrow] = (M + __builtin_amdgcn_logf(Lh)) * kLn2;
      }
    }
  }
}

// WPC = workgroups per compute unit the kernel is built for
template <int DT, int NW, int NCB, int SUBS, int WPC, bool PIPE = false, bool DEQ = false>
__global__ __launch_bounds__(NW * 64, WPC) void prefill_wg_kernel(PrefillArgs P) {
  extern __shared__ uint64_t smem64[];
  uint8_t* smem = reinterpret_cast<uint8_t*>(smem64);
  uint64_t* s_tab = reinterpret_cast<uint64_t*>(smem + 2 * stage_bytes(SUBS));
  volatile uint32_t* s_ctl = reinterpret_cast<volatile uint32_t*>(smem + 2 * stage_bytes(SUBS) + (size_t)P.table_entries * 8);
  const DevBatch& B = P.b;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t H = (uint32_t)B.g.H;
  const uint32_t total = P.tile_first[B.n_seq] * H;
  const uint32_t* tf = P.tile_first;
  if (P.tf_cache) {  // (uniform)
    uint32_t* s_tf = reinterpret_cast<uint32_t*>(smem + 2 * stage_bytes(SUBS) + (size_t)P.table_entries * 8 + kWgCtlBytes);
    for (int i = threadIdx.x; i <= B.n_seq; i += NW * 64) s_tf[i] = P.tile_first[i];
    __syncthreads();
    tf = s_tf;
  }
#ifdef FS_TIMELINE
  const uint64_t tl_start = wall_clock64();
  uint64_t tl_items = 0;
#endif
  ItemDraw d{0u, 0u};
  if (wave == 0) d = first_draw(P.header, blockIdx.x >> 3, lane);
  for (;;) {
#ifdef FS_TIMELINE
    const uint64_t tl_top = wall_clock64();
#endif
    if (wave == 0) {  // one wave draws for the workgroup
      uint32_t item;
      const bool ok = next_item(d, P.header, total, (uint32_t)P.chunk_shift, lane, item);
      if (lane == 0) s_ctl[0] = ok ? item : 0xffffffffu;
    }
    __syncthreads();
    const uint32_t item = __builtin_amdgcn_readfirstlane(s_ctl[0]);  // (an LDS load is not uniform to the compiler)
    __syncthreads();  // everyone holds the item before the next draw may overwrite it
    if (item == 0xffffffffu) break;
    int seq, head, qt;
    if (!decode_item(P, tf, item, H, seq, head, qt)) continue;
#ifdef FS_TIMELINE
    const uint64_t tl_begin = wall_clock64();
#endif
    if constexpr (PIPE) prefill_item_wgp<DT>(P, seq, head, qt, smem, s_tab, wave);
    else prefill_item_wg<DT, NW, NCB, SUBS, DEQ>(P, seq, head, qt, smem, s_tab, wave);
#ifdef FS_TIMELINE
    ++tl_items;
    if (threadIdx.x == 0 && item < kPfTimelineItems) {
      uint64_t* row = P.timeline + 8 * (kPfTimelineGroups + item);
      row[0] = tl_begin;
      row[1] = wall_clock64();
      row[2] = ((uint64_t)seq << 32) | ((uint64_t)head << 20) | (uint64_t)qt;
      row[3] = (uint64_t)blockIdx.x | ((tl_begin - tl_top) << 32);
    }
#endif
  }
#ifdef FS_TIMELINE
  if (threadIdx.x == 0 && blockIdx.x < kPfTimelineGroups) {
    uint64_t* row = P.timeline + 8 * blockIdx.x;
    row[0] = tl_start;
    row[1] = wall_clock64();
    row[2] = tl_items;
    row[3] = __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7;  // hwreg(HW_REG_XCC_ID, 0, 4)
  }
#endif
}

// The 16-column kernel; the only MFMA prefill kernel for head_dim 64 and 256 (HD: its tile code takes any of the three).
template <int HD>
__global__ __launch_bounds__(kThreads, mfma_wgs_per_cu(HD)) void prefill_kernel(PrefillArgs P) {
  extern __shared__ uint64_t smem64[];
  const DevBatch& B = P.b;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint64_t* s_ptr = smem64 + (size_t)wave * P.table_entries;
  const uint32_t H = (uint32_t)B.g.H;
  const uint32_t total = P.tile_first[B.n_seq] * H;
  ItemDraw d = first_draw(P.header, (blockIdx.x >> 3) * kWaves + wave, lane);
  for (uint32_t item; next_item(d, P.header, total, kWaveChunkShift, lane, item);) {
    int seq, head, qt;
    if (!decode_item(P, P.tile_first, item, H, seq, head, qt)) continue;
    switch (B.g.dtype) {
      case FS_KV_FP16: prefill_item<FS_KV_FP16, HD>(P, seq, head, qt, s_ptr); break;
      case FS_KV_FP8_E4M3: prefill_item<FS_KV_FP8_E4M3, HD>(P, seq, head, qt, s_ptr); break;
      case FS_KV_INT8: prefill_item<FS_KV_INT8, HD>(P, seq, head, qt, s_ptr); break;
      default: prefill_item<FS_KV_INT4, HD>(P, seq, head, qt, s_ptr); break;
    }
  }
}

uint64_t align256(uint64_t x) { return (x + 255) & ~255ull; }

}  // namespace
}  // namespace fs

using namespace fs;

#ifdef FS_TIMELINE
// (timeline build only) bytes of the clock readings at the end of a prefill workspace, and their layout
extern "C" uint64_t fs_prefill_timeline_bytes(uint64_t* group_rows, uint64_t* item_rows) {
  if (group_rows) *group_rows = kPfTimelineGroups;
  if (item_rows) *item_rows = kPfTimelineItems;
  return kPfTimelineBytes;
}
#endif

uint64_t fs_prefill_workspace_bytes(int n_seq) {
  if (n_seq < 1) return 0;
#ifdef FS_TIMELINE
  return align256(kHeaderBytes + 4ull * ((uint64_t)n_seq + 1)) + kPfTimelineBytes;
#else
  return align256(kHeaderBytes + 4ull * ((uint64_t)n_seq + 1));
#endif
}

int fs_prefill_attention(fs_pool* p, fs_model_t model, int layer, int n_q_heads, float sm_scale, const void* q,
                         const int32_t* block_tables, const int32_t* seq_lens, const int32_t* q_offsets,
                         const int32_t* q_offsets_host, int n_seq, int max_blocks, void* out, float* lse, void* workspace,
                         uint64_t workspace_bytes, void* stream) {
  if (!p || model < 0 || model >= kMaxModels || !p->models[model].in_use) {
    set_error("prefill attention: unknown pool or model");
    return FS_ERR_INVALID;
  }
  const Model& M = p->models[model];
  const fs_geometry_t& g = M.g;
  if (layer < 0 || layer >= g.n_layers || n_seq < 1 || max_blocks < 1 || !q || !block_tables || !seq_lens || !q_offsets ||
      !q_offsets_host || !out || n_q_heads < g.n_kv_heads || n_q_heads % g.n_kv_heads || !(sm_scale == sm_scale)) {
    set_error("prefill attention: invalid argument");
    return FS_ERR_INVALID;
  }
  if (((uintptr_t)q | (uintptr_t)out) & 15) {
    set_error("prefill attention: q and out must be 16-byte aligned");
    return FS_ERR_INVALID;
  }
  if (q_offsets_host[0] != 0) {
    set_error("prefill attention: q_offsets must start at 0");
    return FS_ERR_INVALID;
  }
  const int G = n_q_heads / g.n_kv_heads;
  if (G > 16) {
    set_error("prefill attention: more than 16 query heads per KV head");
    return FS_ERR_INVALID;
  }
  const int tpt = 16 / G;
  const int ncb_env = p->opt.prefill_ncb;  // FS_OPT_PREFILL_COLUMN_BLOCKS
  // Default: the workgroup kernel (measured fastest for every format once a launch has a work item per
  // compute unit); the 16-column wave-level kernel, whose items are sixteen times finer, for smaller launches.
  const int ncb_default = 16;
  // the wide kernels fold the (positive) softmax scale into the exponential's argument; any other scale takes
  // the 16-column kernel, which does not
  const bool scale_ok = sm_scale > 0.f && sm_scale < INFINITY;
  // (head_dim 64 and 256: the 16-column kernel is the one whose tile code is built for them)
  int ncb = !scale_ok || g.head_dim != kD ? 1 : (ncb_env ? ncb_env : ncb_default);
  uint64_t tiles = 0;
  for (int pass = 0; pass < 2; ++pass) {
    tiles = 0;
    for (int b = 0; b < n_seq; ++b) {
      const int64_t n_new = (int64_t)q_offsets_host[b + 1] - q_offsets_host[b];
      if (n_new < 0) {
        set_error("prefill attention: q_offsets must not decrease");
        return FS_ERR_INVALID;
      }
      tiles += (uint64_t)((n_new + tpt * ncb - 1) / (tpt * ncb));
    }
    // a launch with fewer workgroup-level items than compute units: the finest items instead
    if (pass == 0 && ncb == 16 && !ncb_env && tiles * (uint64_t)g.n_kv_heads < (uint64_t)p->n_cu) ncb = 1;
    else break;
  }
  const int64_t n_rows = q_offsets_host[n_seq];
  if (tiles * (uint64_t)g.n_kv_heads > 0xfffffff0ull || n_rows > 0x7fffffff) {
    set_error("prefill attention: batch too large");
    return FS_ERR_INVALID;
  }
  if (g.kv_dtype == FS_KV_FP8_E4M3 && !M.d_k_scale) {
    set_error("prefill attention: FP8 model has no scales (fs_model_set_fp8_scales)");
    return FS_ERR_INVALID;
  }
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < fs_prefill_workspace_bytes(n_seq)) {
    set_error("prefill attention: workspace missing, not 256-byte aligned or too small (see fs_prefill_workspace_bytes)");
    return workspace && !((uintptr_t)workspace & 255) ? FS_ERR_NOMEM : FS_ERR_INVALID;
  }
  if (p->n_cu == 0) {
    set_error("prefill attention: pool has no HIP device");
    return FS_ERR_DEVICE;
  }
  PrefillArgs P{};
  DevBatch& B = P.b;
  B.g = dev_geom(g);
  B.layer_base = p->base + (uint64_t)layer * g.layer_bytes;
  B.q = (const _Float16*)q;
  B.tables = block_tables;
  B.seq_lens = seq_lens;
  B.out = (_Float16*)out;
  B.lse = lse;
  B.k_scale = M.d_k_scale ? M.d_k_scale + (size_t)layer * g.n_kv_heads : nullptr;
  B.v_scale = M.d_v_scale ? M.d_v_scale + (size_t)layer * g.n_kv_heads : nullptr;
  B.n_seq = n_seq;
  B.max_blocks = max_blocks;
  B.n_q = n_q_heads;
  B.G = G;
  B.sm_scale = sm_scale;
  B.R = (g.tokens_per_block + 7) / 8;
  B.r_magic = B.R == 1 ? 0u : (uint32_t)(((1ull << 32) + (uint64_t)B.R - 1) / (uint64_t)B.R);
  B.n_blocks = (uint32_t)(p->pool_bytes / g.block_budget);
  for (int t = 0; t < kTierSteps; ++t) B.tier_seq[t] = 0x7fffffff;  // (decode's split sizes: not used by prefill)
  B.ring_runs = 4;
  const bool generic = !mfma_supports(B);  // head_dim other than 64, 128 or 256, or blocks of fewer than 8 tokens
  if (generic && (g.head_dim & (g.head_dim - 1))) {
    set_error("prefill attention: head_dim must be a power of two");
    return FS_ERR_INVALID;
  }
  P.q_offsets = q_offsets;
  P.header = (uint32_t*)workspace;
  P.tile_first = (uint32_t*)((uint8_t*)workspace + kHeaderBytes);
#ifdef FS_TIMELINE
  P.timeline = (uint64_t*)((uint8_t*)workspace + align256(kHeaderBytes + 4ull * ((uint64_t)n_seq + 1)));
#endif
  P.tpt = tpt;
  P.ncb = ncb;
  P.seg_runs = prefill_seg_runs(B.R);
  P.table_entries = prefill_table_entries(P.seg_runs, B.R);
  P.n_rows = (int32_t)n_rows;
  P.whole_runs = (g.tokens_per_block & 7) == 0;
  if (n_rows == 0) return FS_OK;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();
  hipLaunchKernelGGL(prefill_prep_kernel, dim3(1), dim3(kPrepThreads), 0, s, P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return device_error(e, "prefill prep launch");
  if (generic) {
    // one workgroup per (query row, KV head) on the vector ALU: every shape the pool can hold
    MultiArgs A{};
    A.b[0] = B;
    A.header = P.header;
    A.n_batches = 1;
    const uint64_t work = (uint64_t)n_rows * (uint64_t)g.n_kv_heads;
    p->opt.last_prefill = 1 << 18;
    e = launch_generic_prefill(A, q_offsets, (int)n_rows, (int)std::min<uint64_t>(work, (uint64_t)p->n_cu * 8), s);
    if (e != hipSuccess) return device_error(e, "prefill launch (generic kernel)");
    return FS_OK;
  }
  const uint64_t items = tiles * (uint64_t)g.n_kv_heads;
  // waves per SIMD: the 16-column kernel runs two, the wider wave-level ones one
  const int wps = ncb == 1 ? mfma_wgs_per_cu(g.head_dim) : 1;
  // workgroup kernels: 16 blocks = 8 waves x 2 (default) or 4 x 4, 4 sub-tiles per step, one workgroup per compute unit
  const bool wg = ncb == 16;
  const int nw = p->opt.prefill_nw == 4 ? 4 : 8;
  const int subs = 4, wpc = 1;
  const int n_wg = wg ? (int)std::min<uint64_t>((uint64_t)p->n_cu * wpc, std::max<uint64_t>(items, 1))
                      : (int)std::min<uint64_t>((uint64_t)p->n_cu * wps, std::max<uint64_t>((items + kWaves - 1) / kWaves, 1));
  // Consecutive items -- the query tiles of one (sequence, head), which stream the same K/V -- go to one XCD in
  // chunks of 128 (a head of 8192 tokens in one piece: measured + 1.4 % over chunks of 32 on long prompts), of
  // fewer while that leaves an XCD less than eight chunks to balance with.
  P.chunk_shift = 7;
  while (P.chunk_shift > (int32_t)kWgChunkShift && (items >> P.chunk_shift) < 64) --P.chunk_shift;
  // the per-sequence tile counts go to LDS while they fit beside the stages (16 KiB: 4095 sequences)
  P.tf_cache = wg && (uint64_t)n_seq + 1 <= 4096;
  const size_t smem = wg ? 2 * (size_t)stage_bytes(subs) + (size_t)P.table_entries * 8 + kWgCtlBytes +
                               (P.tf_cache ? (((size_t)n_seq + 1) * 4 + 15) / 16 * 16 : 0)
                         : (size_t)kWaves * P.table_entries * sizeof(uint64_t);
  if (wg) {
    void (*kern)(PrefillArgs) = nullptr;
#define FS_WG(DT)                                  \
  (nw == 8 ? prefill_wg_kernel<DT, 8, 2, 4, 1> \
           : (p->opt.prefill_pipe ? prefill_wg_kernel<DT, 4, 4, 4, 1, true> : prefill_wg_kernel<DT, 4, 4, 4, 1>))
    const bool deq = p->opt.prefill_deq && nw == 8;  // (the 8-wave kernel only)
    switch (g.kv_dtype) {
      case FS_KV_FP16: kern = FS_WG(FS_KV_FP16); break;
      case FS_KV_FP8_E4M3: kern = FS_WG(FS_KV_FP8_E4M3); break;
      case FS_KV_INT8: kern = deq ? prefill_wg_kernel<FS_KV_INT8, 8, 2, 4, 1, false, true> : FS_WG(FS_KV_INT8); break;
      default: kern = deq ? prefill_wg_kernel<FS_KV_INT4, 8, 2, 4, 1, false, true> : FS_WG(FS_KV_INT4); break;
    }
#undef FS_WG
    // more than 64 KiB of dynamic LDS has to be granted per kernel
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return device_error(e, "prefill LDS attribute");
    const bool deq_used = deq && (g.kv_dtype == FS_KV_INT8 || g.kv_dtype == FS_KV_INT4);
    p->opt.last_prefill = 16 | (nw << 8) | ((int64_t)deq_used << 16) | ((int64_t)(nw == 4 && p->opt.prefill_pipe) << 17);
    hipLaunchKernelGGL(kern, dim3(n_wg), dim3(nw * 64), smem, s, P);
  } else if (ncb == 1) {
    p->opt.last_prefill = 1;
    if (g.head_dim == 64) hipLaunchKernelGGL(prefill_kernel<64>, dim3(n_wg), dim3(kThreads), smem, s, P);
    else if (g.head_dim == 256) hipLaunchKernelGGL(prefill_kernel<256>, dim3(n_wg), dim3(kThreads), smem, s, P);
    else hipLaunchKernelGGL(prefill_kernel<kD>, dim3(n_wg), dim3(kThreads), smem, s, P);
  } else {
    void (*kern)(PrefillArgs) = nullptr;
#define FS_WIDE(DT) (ncb == 4 ? prefill_wide_kernel<DT, 4, 1> : prefill_wide_kernel<DT, 2, 1>)
    switch (g.kv_dtype) {
      case FS_KV_FP16: kern = FS_WIDE(FS_KV_FP16); break;
      case FS_KV_FP8_E4M3: kern = FS_WIDE(FS_KV_FP8_E4M3); break;
      case FS_KV_INT8: kern = FS_WIDE(FS_KV_INT8); break;
      default: kern = FS_WIDE(FS_KV_INT4); break;
    }
#undef FS_WIDE
    p->opt.last_prefill = ncb;
    hipLaunchKernelGGL(kern, dim3(n_wg), dim3(kThreads), smem, s, P);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return device_error(e, "prefill launch");
  return FS_OK;
}
