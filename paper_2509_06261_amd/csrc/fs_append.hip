// fs_kv_append: quantize new K/V rows and scatter them into slab blocks.
//
// FineServe Sec. 2.1: every new token appends its keys and values to the KV cache;
// Sec. 2.2 / 3.2: the cache may be FP16, FP8 or INT4 (here also INT8), with per-token
// quantization parameters stored inside the block.  The paper gives no quantizer
// arithmetic; the definitions implemented here are the ones stated in fineserve.h.
//
// One wavefront handles one (token, KV head, K|V) row: lanes hold element pairs, the row's
// extrema are reduced across the wave with DPP shuffles, and each lane stores its own bytes
// (INT4: one byte = the lane's two codes, so no byte is shared between lanes or tokens).
// All arithmetic is IEEE fp32, round-to-nearest-even, correctly rounded division, and this
// file is compiled with floating-point contraction off so that the stored bytes are
// reproducible bit for bit.
#include "fs_internal.h"

namespace fs {
namespace {

constexpr int kWaves = 4;        // waves per workgroup
constexpr int kMaxPairIters = 4; // head_dim <= 512 -> at most 4 element pairs per lane

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
  int64_t n_rows;        // n_tokens * H * 2
  int64_t n_blocks;      // valid block ids are [0, n_blocks)
  int32_t layer, max_blocks;
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) v = fminf(v, __shfl_xor(v, o, 64));
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

template <bool kSrcF32>
__device__ __forceinline__ void load_pair(const void* src, int64_t idx, float& a, float& b) {
  if (kSrcF32) {
    const float2 v = *reinterpret_cast<const float2*>(reinterpret_cast<const float*>(src) + idx);
    a = v.x;
    b = v.y;
  } else {
    const uint32_t v = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint16_t*>(src) + idx);
    a = f16_value((uint16_t)(v & 0xFFFF));
    b = f16_value((uint16_t)(v >> 16));
  }
}

template <bool kSrcF32>
__global__ __launch_bounds__(kWaves * 64) void kv_append_kernel(AppendArgs A) {
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const DevGeom& g = A.g;
  const int D = g.D;
  const int n_iter = (D + 127) >> 7;
  for (int64_t r = (int64_t)blockIdx.x * kWaves + wave; r < A.n_rows; r += (int64_t)gridDim.x * kWaves) {
    const int which = (int)(r & 1);
    const int64_t th = r >> 1;
    const int head = (int)(th % g.H);
    const int64_t tok = th / g.H;
    const int p = A.pos[tok];
    const int s = A.seq_idx[tok];
    if (p < 0 || s < 0) continue;
    const int bi = p / g.T;
    if (bi >= A.max_blocks) continue;
    const int tib = p - bi * g.T;
    const int32_t blk = A.tables[(int64_t)s * A.max_blocks + bi];
    if (blk < 0 || blk >= A.n_blocks) continue;  // never write outside the pool
    uint8_t* chunk = A.pool + (uint64_t)blk * g.block_budget + (uint64_t)A.layer * g.layer_bytes +
                     (uint64_t)head * g.head_chunk;
    uint8_t* row = chunk + (which ? g.kv_tile : 0u) + (uint64_t)tib * g.row_bytes;
    uint8_t* par = chunk + 2u * g.kv_tile + (which ? g.par_tile : 0u) + (uint64_t)tib * (uint32_t)g.param_bytes;
    const void* src = which ? A.v_new : A.k_new;
    const int64_t src_row = (tok * g.H + head) * (int64_t)D;

    float xa[kMaxPairIters], xb[kMaxPairIters];
#pragma unroll
    for (int it = 0; it < kMaxPairIters; ++it) {
      xa[it] = 0.f;
      xb[it] = 0.f;
      const int d = it * 128 + lane * 2;
      if (it < n_iter && d < D) load_pair<kSrcF32>(src, src_row + d, xa[it], xb[it]);
    }

    if (g.dtype == FS_KV_FP16) {
#pragma unroll
      for (int it = 0; it < kMaxPairIters; ++it) {
        const int d = it * 128 + lane * 2;
        if (it < n_iter && d < D)
          *reinterpret_cast<uint32_t*>(row + 2 * d) = (uint32_t)f16_bits(xa[it]) | ((uint32_t)f16_bits(xb[it]) << 16);
      }
    } else if (g.dtype == FS_KV_FP8_E4M3) {
      const float sc = (which ? A.v_scale : A.k_scale)[head];
#pragma unroll
      for (int it = 0; it < kMaxPairIters; ++it) {
        const int d = it * 128 + lane * 2;
        if (it < n_iter && d < D) {
          const uint32_t c0 = e4m3_bits(__fdiv_rn(xa[it], sc)), c1 = e4m3_bits(__fdiv_rn(xb[it], sc));
          *reinterpret_cast<uint16_t*>(row + d) = (uint16_t)(c0 | (c1 << 8));
        }
      }
    } else if (g.dtype == FS_KV_INT8) {
      float amax = 0.f;
#pragma unroll
      for (int it = 0; it < kMaxPairIters; ++it) amax = fmaxf(amax, fmaxf(fabsf(xa[it]), fabsf(xb[it])));
      amax = wave_max(amax);
      const uint16_t sb = scale_bits(__fdiv_rn(amax, 127.0f));
      const float sf = f16_value(sb);
#pragma unroll
      for (int it = 0; it < kMaxPairIters; ++it) {
        const int d = it * 128 + lane * 2;
        if (it < n_iter && d < D) {
          const float q0 = fminf(fmaxf(rintf(__fdiv_rn(xa[it], sf)), -127.f), 127.f);
          const float q1 = fminf(fmaxf(rintf(__fdiv_rn(xb[it], sf)), -127.f), 127.f);
          *reinterpret_cast<uint16_t*>(row + d) = (uint16_t)(((uint32_t)(int)q0 & 0xFF) | (((uint32_t)(int)q1 & 0xFF) << 8));
        }
      }
      if (lane == 0) *reinterpret_cast<uint16_t*>(par) = sb;
    } else {  // FS_KV_INT4
      float lo = 0.f, hi = 0.f;
#pragma unroll
      for (int it = 0; it < kMaxPairIters; ++it) {
        lo = fminf(lo, fminf(xa[it], xb[it]));
        hi = fmaxf(hi, fmaxf(xa[it], xb[it]));
      }
      lo = wave_min(lo);
      hi = wave_max(hi);
      const uint16_t sb = scale_bits(__fdiv_rn(hi - lo, 15.0f));
      const float sf = f16_value(sb);
      const float z = fminf(fmaxf(rintf(__fdiv_rn(-lo, sf)), 0.f), 15.f);
#pragma unroll
      for (int it = 0; it < kMaxPairIters; ++it) {
        const int d = it * 128 + lane * 2;
        if (it < n_iter && d < D) {
          const float q0 = fminf(fmaxf(rintf(__fdiv_rn(xa[it], sf)) + z, 0.f), 15.f);
          const float q1 = fminf(fmaxf(rintf(__fdiv_rn(xb[it], sf)) + z, 0.f), 15.f);
          row[d >> 1] = (uint8_t)((uint32_t)q0 | ((uint32_t)q1 << 4));
        }
      }
      if (lane == 0) *reinterpret_cast<uint32_t*>(par) = (uint32_t)sb | ((uint32_t)f16_bits(z) << 16);
    }
  }
}

}  // namespace
}  // namespace fs

using namespace fs;

extern "C" int fs_kv_append(fs_pool* p, fs_model_t model, int layer, const void* k_new, const void* v_new,
                            int src_dtype, const int32_t* seq_idx, const int32_t* pos, const int32_t* block_tables,
                            int max_blocks, int64_t n_tokens, void* stream) {
  if (!p || model < 0 || model >= kMaxModels || !p->models[model].in_use) {
    set_error("fs_kv_append: unknown model");
    return FS_ERR_INVALID;
  }
  const Model& M = p->models[model];
  if (n_tokens == 0) return FS_OK;
  if (n_tokens < 0 || layer < 0 || layer >= M.g.n_layers || !k_new || !v_new || !seq_idx || !pos || !block_tables ||
      max_blocks < 1 || (src_dtype != FS_SRC_FP16 && src_dtype != FS_SRC_FP32)) {
    set_error("fs_kv_append: invalid argument");
    return FS_ERR_INVALID;
  }
  if (M.g.kv_dtype == FS_KV_FP8_E4M3 && !M.d_k_scale) {
    set_error("fs_kv_append: FP8 model has no scales (fs_model_set_fp8_scales)");
    return FS_ERR_INVALID;
  }
  if (p->n_cu == 0) {
    set_error("fs_kv_append: pool has no HIP device");
    return FS_ERR_DEVICE;
  }
  AppendArgs A{};
  A.g = dev_geom(M.g);
  A.pool = p->base;
  A.k_new = k_new;
  A.v_new = v_new;
  A.seq_idx = seq_idx;
  A.pos = pos;
  A.tables = block_tables;
  A.k_scale = M.d_k_scale ? M.d_k_scale + (size_t)layer * M.g.n_kv_heads : nullptr;
  A.v_scale = M.d_v_scale ? M.d_v_scale + (size_t)layer * M.g.n_kv_heads : nullptr;
  A.n_rows = n_tokens * M.g.n_kv_heads * 2;
  A.n_blocks = (int64_t)(p->pool_bytes / M.g.block_budget);
  A.layer = layer;
  A.max_blocks = max_blocks;
  int64_t blocks = (A.n_rows + kWaves - 1) / kWaves;
  const int64_t cap = (int64_t)p->n_cu * 64;
  if (blocks > cap) blocks = cap;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();  // drop any stale error of an earlier, unrelated runtime call
  if (src_dtype == FS_SRC_FP32)
    hipLaunchKernelGGL(kv_append_kernel<true>, dim3((unsigned)blocks), dim3(kWaves * 64), 0, s, A);
  else
    hipLaunchKernelGGL(kv_append_kernel<false>, dim3((unsigned)blocks), dim3(kWaves * 64), 0, s, A);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return device_error(e, "fs_kv_append launch");
  return FS_OK;
}
