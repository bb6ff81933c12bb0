// fs_kv_append / fs_kv_append_multi: host entry points and kernels (the device code is in fs_append_rows.h).
//
// FineServe Sec. 2.1: every new token appends its keys and values to the KV cache; Sec. 4: co-located models share
// the GPU, so one launch serves the newest tokens of all of them.
#include <algorithm>

#include "fs_append_rows.h"

namespace fs {
namespace {

using namespace append;
constexpr int kWaves = 4;  // waves per workgroup

template <bool kSrcF32>
__global__ __launch_bounds__(kWaves * 64) void kv_append_kernel(AppendArgs A) {
  append_rows<kSrcF32>(A, (int64_t)blockIdx.x * kWaves + (threadIdx.x >> 6), (int64_t)gridDim.x * kWaves);
}

__global__ __launch_bounds__(kWaves * 64) void kv_append_multi_kernel(MultiAppendArgs P) { append_block(P, blockIdx.x, kWaves); }

}  // namespace

int make_append_args(fs_pool* p, const fs_append_t& a, append::AppendArgs& A) {
  if (!p || a.model < 0 || a.model >= kMaxModels || !p->models[a.model].in_use) {
    set_error("fs_kv_append: unknown model");
    return FS_ERR_INVALID;
  }
  const Model& M = p->models[a.model];
  if (a.n_tokens < 0 || a.layer < 0 || a.layer >= M.g.n_layers || a.max_blocks < 1 ||
      (a.src_dtype != FS_SRC_FP16 && a.src_dtype != FS_SRC_FP32) ||
      (a.n_tokens > 0 && (!a.k_new || !a.v_new || !a.seq_idx || !a.pos || !a.block_tables))) {
    set_error("fs_kv_append: invalid argument");
    return FS_ERR_INVALID;
  }
  if (((uintptr_t)a.k_new | (uintptr_t)a.v_new) & 15) {
    set_error("fs_kv_append: k_new and v_new must be 16-byte aligned");
    return FS_ERR_INVALID;
  }
  if (M.g.kv_dtype == FS_KV_FP8_E4M3 && !M.d_k_scale) {
    set_error("fs_kv_append: FP8 model has no scales (fs_model_set_fp8_scales)");
    return FS_ERR_INVALID;
  }
  A = append::AppendArgs{};
  A.g = dev_geom(M.g);
  A.pool = p->base;
  A.k_new = a.k_new;
  A.v_new = a.v_new;
  A.seq_idx = a.seq_idx;
  A.pos = a.pos;
  A.tables = a.block_tables;
  A.k_scale = M.d_k_scale ? M.d_k_scale + (size_t)a.layer * M.g.n_kv_heads : nullptr;
  A.v_scale = M.d_v_scale ? M.d_v_scale + (size_t)a.layer * M.g.n_kv_heads : nullptr;
  A.n_tokens = a.n_tokens;
  A.n_rows = (a.n_tokens + 3) / 4 * 4 * M.g.n_kv_heads * 2;
  A.n_blocks = (int64_t)(p->pool_bytes / M.g.block_budget);
  A.layer = a.layer;
  A.max_blocks = a.max_blocks;
  A.src_f32 = a.src_dtype == FS_SRC_FP32;
  int lpr_shift = 0;
  while ((append::kEpl << lpr_shift) < M.g.head_dim) ++lpr_shift;  // head_dim is a power of two >= 8
  A.lpr_shift = lpr_shift;
  return FS_OK;
}

uint32_t plan_append_blocks(const fs_pool* p, append::MultiAppendArgs& P, int waves) {
  const int64_t cap = std::max<int64_t>((int64_t)p->n_cu * 64 * 4 / waves, 1);  // per append: as the single-append launch
  uint32_t next = 0;
  for (int i = 0; i < P.n; ++i) {
    const int64_t rows_per_wg = (int64_t)waves * (64 >> P.a[i].lpr_shift);
    P.first_block[i] = next;
    next += (uint32_t)std::min<int64_t>((P.a[i].n_rows + rows_per_wg - 1) / rows_per_wg, cap);
  }
  for (int i = P.n; i <= append::kMaxAppends; ++i) P.first_block[i] = next;
  return next;
}

}  // namespace fs

using namespace fs;

extern "C" int fs_kv_append(fs_pool* p, fs_model_t model, int layer, const void* k_new, const void* v_new,
                            int src_dtype, const int32_t* seq_idx, const int32_t* pos, const int32_t* block_tables,
                            int max_blocks, int64_t n_tokens, void* stream) {
  fs_append_t a{};
  a.model = model;
  a.layer = layer;
  a.src_dtype = src_dtype;
  a.max_blocks = max_blocks;
  a.k_new = k_new;
  a.v_new = v_new;
  a.seq_idx = seq_idx;
  a.pos = pos;
  a.block_tables = block_tables;
  a.n_tokens = n_tokens;
  if (p && model >= 0 && model < kMaxModels && p->models[model].in_use && n_tokens == 0) return FS_OK;
  append::AppendArgs A;
  const int rc = make_append_args(p, a, A);
  if (rc != FS_OK) return rc;
  if (p->n_cu == 0) {
    set_error("fs_kv_append: pool has no HIP device");
    return FS_ERR_DEVICE;
  }
  const int64_t rows_per_wg = (int64_t)kWaves * (64 >> A.lpr_shift);
  int64_t blocks = (A.n_rows + rows_per_wg - 1) / rows_per_wg;
  const int64_t cap = (int64_t)p->n_cu * 64;
  if (blocks > cap) blocks = cap;
  hipStream_t s = (hipStream_t)stream;
  (void)hipGetLastError();  // drop any stale error of an earlier, unrelated runtime call
  if (A.src_f32)
    hipLaunchKernelGGL(kv_append_kernel<true>, dim3((unsigned)blocks), dim3(kWaves * 64), 0, s, A);
  else
    hipLaunchKernelGGL(kv_append_kernel<false>, dim3((unsigned)blocks), dim3(kWaves * 64), 0, s, A);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return device_error(e, "fs_kv_append launch");
  return FS_OK;
}

extern "C" int fs_kv_append_multi(fs_pool* p, const fs_append_t* appends, int n_appends, void* stream) {
  if (!p || !appends || n_appends < 1 || n_appends > append::kMaxAppends) {
    set_error("fs_kv_append_multi: need 1..8 appends");
    return FS_ERR_INVALID;
  }
  append::MultiAppendArgs P{};
  for (int i = 0; i < n_appends; ++i) {
    const int rc = make_append_args(p, appends[i], P.a[P.n]);
    if (rc != FS_OK) return rc;
    if (appends[i].n_tokens > 0) ++P.n;  // an empty append takes no workgroup
  }
  if (P.n == 0) return FS_OK;
  if (p->n_cu == 0) {
    set_error("fs_kv_append_multi: pool has no HIP device");
    return FS_ERR_DEVICE;
  }
  const uint32_t blocks = plan_append_blocks(p, P, kWaves);
  (void)hipGetLastError();
  hipLaunchKernelGGL(kv_append_multi_kernel, dim3(blocks), dim3(kWaves * 64), 0, (hipStream_t)stream, P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return device_error(e, "fs_kv_append_multi launch");
  return FS_OK;
}
