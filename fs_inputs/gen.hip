// Device-side twin of gen.py: the same counter-based generator, evaluated in HBM.
//
// This file produces synthetic *inputs* only (source K/V rows in fp16 or fp32).
// It holds none of the decode-attention method's arithmetic and is linked into a
// library of its own (libfs_inputs.so); neither the product library nor the CPU
// oracle shares code with it.
//
// Generator (all arithmetic modulo 2^64), identical to gen.py:
//   mix64 = splitmix64 finalizer
//   key   = mix64(mix64(seed ^ GOLD*(model+1)) + (layer<<34) + (which<<32) + seq)
//   word(w) = mix64(key + GOLD*(w+1));  element e = (pos*H + head)*D + dim
//   u = (word(e>>2) >> 16*(e&3)) & 0xFFFF;  x = table[u]
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint64_t kGold = 0x9E3779B97F4A7C15ull;

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}

// One thread per 4 consecutive elements (one 64-bit word of the generator).
// row_elems = H*D must be a multiple of 4.
template <typename OutT>
__global__ void fill_rows_kernel(OutT* __restrict__ out, const float* __restrict__ table,
                                 uint64_t key_base, uint64_t layer_which,
                                 const int32_t* __restrict__ seq_id, const int32_t* __restrict__ pos,
                                 uint32_t row_elems, uint64_t n_words_total) {
  const uint32_t words_per_row = row_elems >> 2;
  for (uint64_t w = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x; w < n_words_total;
       w += (uint64_t)gridDim.x * blockDim.x) {
    const uint64_t tok = w / words_per_row;
    const uint32_t wr = (uint32_t)(w - tok * words_per_row);
    const uint64_t key = mix64(key_base + layer_which + (uint64_t)(uint32_t)seq_id[tok]);
    const uint64_t e = (uint64_t)(uint32_t)pos[tok] * row_elems + (uint64_t)wr * 4u;
    const uint64_t word = mix64(key + kGold * ((e >> 2) + 1ull));
    OutT* o = out + tok * (uint64_t)row_elems + (uint64_t)wr * 4u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const uint32_t u = (uint32_t)(word >> (16 * i)) & 0xFFFFu;
      o[i] = (OutT)table[u];  // fp16: round-to-nearest-even, same as numpy astype(float16)
    }
  }
}

}  // namespace

extern "C" {

// Fills out[n_tokens][row_elems] (row_elems = n_heads*head_dim) with the generator's
// values for tokens (seq_id[i], pos[i]).  All pointers are device pointers; table is the
// 65536-entry float32 table of gen.py uploaded by the caller.  out_is_f32: 0 -> fp16,
// 1 -> fp32.  Asynchronous on `stream`.  Returns 0, or the hipError_t of the launch.
int fsi_fill_rows(void* out, int out_is_f32, const float* table, uint64_t seed, int model, int layer,
                  int which, const int32_t* seq_id, const int32_t* pos, int row_elems, int64_t n_tokens,
                  void* stream) {
  if (n_tokens <= 0) return 0;
  if (row_elems <= 0 || (row_elems & 3)) return -1;
  // host-side part of the key: mix64(seed ^ GOLD*(model+1)); the kernel adds layer/which/seq.
  uint64_t a = seed ^ (kGold * (uint64_t)(model + 1));
  a ^= a >> 30; a *= 0xBF58476D1CE4E5B9ull; a ^= a >> 27; a *= 0x94D049BB133111EBull; a ^= a >> 31;
  const uint64_t lw = ((uint64_t)layer << 34) + ((uint64_t)which << 32);
  const uint64_t n_words = (uint64_t)n_tokens * (uint64_t)(row_elems >> 2);
  const int threads = 256;
  uint64_t blocks = (n_words + threads - 1) / threads;
  if (blocks > 65536) blocks = 65536;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();  // drop any stale error of an earlier, unrelated runtime call
  if (out_is_f32)
    hipLaunchKernelGGL(fill_rows_kernel<float>, dim3((unsigned)blocks), dim3(threads), 0, s, (float*)out, table, a,
                       lw, seq_id, pos, (uint32_t)row_elems, n_words);
  else
    hipLaunchKernelGGL(fill_rows_kernel<_Float16>, dim3((unsigned)blocks), dim3(threads), 0, s, (_Float16*)out,
                       table, a, lw, seq_id, pos, (uint32_t)row_elems, n_words);
  return (int)hipGetLastError();
}

}  // extern "C"
