// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <set>
#include <string>
#include <vector>

#include "fineserve.h"

namespace fs {

constexpr int kMaxModels = 64;
constexpr int kMaxBatches = 8;  // batches per multi-model launch

// Host-side record of one registered model.
struct Model {
  bool in_use = false;
  fs_geometry_t g{};
  int64_t live_blocks = 0;
  std::vector<uint8_t> live;        // [n_slabs * blocks_per_slab]
  std::set<int32_t> partial_slabs;  // slabs of this key in PARTIAL state, ordered by id
  float* d_k_scale = nullptr;       // FP8: device [L][H]
  float* d_v_scale = nullptr;
};

}  // namespace fs

namespace fs {
// Per-pool settings (fs_pool_set_option): kernel selection and measurement aids.  Nothing here is process-global.
struct Options {
  int decode_kernel = 0;        // FS_OPT_DECODE_KERNEL
  uint64_t split_bytes = 0;     // FS_OPT_SPLIT_BYTES (0: chosen per launch)
  bool timing = false;          // FS_OPT_KERNEL_TIMING
  int prefill_ncb = 0;          // FS_OPT_PREFILL_COLUMN_BLOCKS
  int prefill_nw = 0;           // FS_OPT_PREFILL_WAVES
  bool prefill_pipe = false;    // FS_OPT_PREFILL_PIPELINED
  bool prefill_deq = true;      // FS_OPT_PREFILL_STAGED_DEQUANT
  int64_t last_prefill = 0;     // FS_OPT_LAST_PREFILL_KERNEL (read-only)
  hipEvent_t ev0 = nullptr, ev1 = nullptr;  // around the latest timed attention kernel
};
}  // namespace fs

struct fs_pool {
  fs::Options opt;
  uint64_t slab_bytes = 0, pool_bytes = 0;
  int64_t n_slabs = 0;
  uint8_t* base = nullptr;  // device
  bool owns_base = false;
  int device = 0;
  int n_cu = 0;
  std::vector<int32_t> state, key, used, free_stack;
  fs::Model models[fs::kMaxModels];
};

namespace fs {

void set_error(const std::string& msg);
int device_error(hipError_t e, const char* what);

// Geometry record handed to kernels (by value inside kernel arguments).
struct DevGeom {
  uint64_t block_budget;
  uint64_t layer_bytes;
  uint32_t head_chunk, kv_tile, par_tile, row_bytes;
  int32_t dtype, T, H, D;
  int32_t param_bytes, L;
  uint32_t pad0, pad1;
};
static_assert(sizeof(DevGeom) == 64, "device geometry record is 64 bytes");

inline DevGeom dev_geom(const fs_geometry_t& g) {
  DevGeom d{};
  d.block_budget = g.block_budget;
  d.layer_bytes = g.layer_bytes;
  d.head_chunk = (uint32_t)g.head_chunk;
  d.kv_tile = (uint32_t)g.kv_tile;
  d.par_tile = (uint32_t)g.par_tile;
  d.row_bytes = (uint32_t)g.row_bytes;
  d.dtype = g.kv_dtype;
  d.T = g.tokens_per_block;
  d.H = g.n_kv_heads;
  d.D = g.head_dim;
  d.param_bytes = g.param_bytes;
  d.L = g.n_layers;
  return d;
}

}  // namespace fs
