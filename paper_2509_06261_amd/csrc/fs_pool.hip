// Host side of the KV slab manager: pool, model geometry, slab table and block allocator.
//
// FineServe Sec. 5.1: one shared KV tensor is pre-allocated and carved into uniform slabs;
// a slab is viewed as an array of blocks of whichever model formats it, without any driver
// call at run time.  Sec. 5.2: Blk ID = slab ID x (#blocks per slab) + local block ID; the
// slab table records FREE / PARTIAL / FULL and which key owns a slab; a block is taken from
// a matching slab or a new slab is carved; an emptied slab returns to the shared tensor.
// Sec. 3.2: block size = TokensPerBlock x TokenSize + Quant.Params -- inverted here: the
// byte budget of a block is fixed and the token count derived.
#include <algorithm>
#include <cstring>

#include "fs_internal.h"

namespace fs {

static thread_local std::string g_last_error;

void set_error(const std::string& msg) { g_last_error = msg; }

int device_error(hipError_t e, const char* what) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
  return FS_ERR_DEVICE;
}

static uint64_t align_up(uint64_t x, uint64_t a) { return (x + a - 1) & ~(a - 1); }

// Lays out a block of `tokens` tokens; returns its defined byte count.
static uint64_t layout(fs_geometry_t& g, int64_t tokens) {
  const int bits = g.kv_dtype == FS_KV_FP16 ? 16 : (g.kv_dtype == FS_KV_INT4 ? 4 : 8);
  g.param_bytes = g.kv_dtype == FS_KV_INT8 ? 2 : (g.kv_dtype == FS_KV_INT4 ? 4 : 0);
  g.row_bytes = (uint64_t)g.head_dim * bits / 8;
  g.kv_tile = align_up((uint64_t)tokens * g.row_bytes, 16);
  g.par_tile = align_up((uint64_t)tokens * (uint64_t)g.param_bytes, 16);
  g.head_chunk = 2 * (g.kv_tile + g.par_tile);
  g.layer_bytes = align_up((uint64_t)g.n_kv_heads * g.head_chunk, 256);
  g.block_bytes = (uint64_t)g.n_layers * g.layer_bytes;
  g.tokens_per_block = (int32_t)tokens;
  return g.block_bytes;
}

// Largest token count that fits the budget: start from the padding-free estimate
// budget / (L * H * 2 * (row + params)), which can only over-estimate, and step down.
static int solve_tokens(fs_geometry_t& g) {
  fs_geometry_t probe = g;
  layout(probe, 1);
  const uint64_t per_token = (uint64_t)g.n_layers * g.n_kv_heads * 2 * (probe.row_bytes + probe.param_bytes);
  int64_t t = (int64_t)(g.block_budget / per_token);
  if (t > 0x7fffffff) t = 0x7fffffff;
  while (t >= 1 && layout(probe, t) > g.block_budget) --t;
  if (t < 1) return FS_ERR_INVALID;
  layout(g, t);
  return FS_OK;
}

}  // namespace fs

using namespace fs;

extern "C" {

const char* fs_last_error(void) { return g_last_error.c_str(); }

int fs_pool_create(uint64_t slab_bytes, uint64_t pool_bytes, void* device_base, fs_pool** out) {
  if (!out) return FS_ERR_INVALID;
  *out = nullptr;
  if (slab_bytes == 0 || (slab_bytes & 255) || pool_bytes == 0 || pool_bytes % slab_bytes) {
    set_error("fs_pool_create: slab_bytes must be a non-zero multiple of 256 and divide pool_bytes");
    return FS_ERR_INVALID;
  }
  const uint64_t n = pool_bytes / slab_bytes;
  if (n >= (1ull << 31)) {
    set_error("fs_pool_create: too many slabs");
    return FS_ERR_INVALID;
  }
  if (device_base && ((uintptr_t)device_base & 255)) {
    set_error("fs_pool_create: device_base must be 256-byte aligned");
    return FS_ERR_INVALID;
  }
  fs_pool* p = new fs_pool();
  p->slab_bytes = slab_bytes;
  p->pool_bytes = pool_bytes;
  p->n_slabs = (int64_t)n;
  // Without a HIP device the pool can still do its bookkeeping (slab table, block ids) when the
  // caller supplies the base address; every device entry point then fails with FS_ERR_DEVICE.
  hipError_t e = hipGetDevice(&p->device);
  if (e == hipSuccess) e = hipDeviceGetAttribute(&p->n_cu, hipDeviceAttributeMultiprocessorCount, p->device);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    p->n_cu = 0;
    if (!device_base) {
      delete p;
      return device_error(e, "fs_pool_create: no usable HIP device");
    }
  }
  if (device_base) {
    p->base = (uint8_t*)device_base;
  } else {
    void* mem = nullptr;
    e = hipMalloc(&mem, pool_bytes);
    if (e != hipSuccess) {
      delete p;
      return device_error(e, "hipMalloc(pool)");
    }
    p->base = (uint8_t*)mem;
    p->owns_base = true;
  }
  p->state.assign(n, FS_SLAB_FREE);
  p->key.assign(n, -1);
  p->used.assign(n, 0);
  p->free_stack.resize(n);
  for (uint64_t i = 0; i < n; ++i) p->free_stack[i] = (int32_t)(n - 1 - i);  // back() == slab 0
  *out = p;
  return FS_OK;
}

int fs_pool_destroy(fs_pool* p) {
  if (!p) return FS_ERR_INVALID;
  for (auto& m : p->models) {
    if (m.d_k_scale) (void)hipFree(m.d_k_scale);
    if (m.d_v_scale) (void)hipFree(m.d_v_scale);
  }
  if (p->owns_base) (void)hipFree(p->base);
  if (p->opt.ev0) (void)hipEventDestroy(p->opt.ev0);
  if (p->opt.ev1) (void)hipEventDestroy(p->opt.ev1);
  delete p;
  return FS_OK;
}

void* fs_pool_base(fs_pool* p) { return p ? p->base : nullptr; }

// forced_tokens > 0: exactly that many tokens per block (they must fit the budget); 0: as many as fit
static int register_model(fs_pool* p, int kv_dtype, int n_kv_heads, int head_dim, int n_layers, uint64_t block_budget_bytes,
                          int forced_tokens, fs_model_t* out) {
  if (!p || !out) return FS_ERR_INVALID;
  if (kv_dtype < FS_KV_FP16 || kv_dtype > FS_KV_INT4 || n_kv_heads < 1 || n_kv_heads > 1024 || n_layers < 1 ||
      n_layers > 4096 || head_dim < 8 || head_dim > 512 || (head_dim & (head_dim - 1))) {
    set_error("fs_model_register: unsupported model shape");
    return FS_ERR_INVALID;
  }
  if (block_budget_bytes == 0 || (block_budget_bytes & 255) || p->slab_bytes % block_budget_bytes ||
      p->pool_bytes / block_budget_bytes >= (1ull << 31)) {
    set_error("fs_model_register: block budget must be a multiple of 256 that divides slab_bytes");
    return FS_ERR_INVALID;
  }
  fs_geometry_t g{};
  g.kv_dtype = kv_dtype;
  g.n_kv_heads = n_kv_heads;
  g.head_dim = head_dim;
  g.n_layers = n_layers;
  g.block_budget = block_budget_bytes;
  g.blocks_per_slab = (int32_t)(p->slab_bytes / block_budget_bytes);
  if (forced_tokens > 0) {
    if (layout(g, forced_tokens) > g.block_budget) {
      set_error("fs_model_register: the requested tokens do not fit the block budget");
      return FS_ERR_INVALID;
    }
  } else if (solve_tokens(g) != FS_OK) {
    set_error("fs_model_register: not even one token fits the block budget");
    return FS_ERR_INVALID;
  }
  for (int m = 0; m < kMaxModels; ++m) {
    if (p->models[m].in_use) continue;
    Model& M = p->models[m];
    M = Model();
    M.in_use = true;
    M.g = g;
    M.live.assign((size_t)p->n_slabs * g.blocks_per_slab, 0);
    *out = m;
    return g.tokens_per_block;
  }
  set_error("fs_model_register: too many models");
  return FS_ERR_NOMEM;
}

int fs_model_register_ex(fs_pool* p, int kv_dtype, int n_kv_heads, int head_dim, int n_layers,
                         uint64_t block_budget_bytes, fs_model_t* out) {
  return register_model(p, kv_dtype, n_kv_heads, head_dim, n_layers, block_budget_bytes, 0, out);
}

static bool shape_ok(int kv_dtype, int n_kv_heads, int head_dim, int n_layers) {
  return kv_dtype >= FS_KV_FP16 && kv_dtype <= FS_KV_INT4 && n_kv_heads >= 1 && n_kv_heads <= 1024 && n_layers >= 1 &&
         n_layers <= 4096 && head_dim >= 8 && head_dim <= 512 && !(head_dim & (head_dim - 1));
}

uint64_t fs_block_bytes(int kv_dtype, int n_kv_heads, int head_dim, int n_layers, int tokens_per_block) {
  if (!shape_ok(kv_dtype, n_kv_heads, head_dim, n_layers) || tokens_per_block < 1) return 0;
  fs_geometry_t g{};
  g.kv_dtype = kv_dtype;
  g.n_kv_heads = n_kv_heads;
  g.head_dim = head_dim;
  g.n_layers = n_layers;
  return layout(g, tokens_per_block);
}

uint64_t fs_slab_bytes_for_blocks(const uint64_t* block_bytes, int n, uint64_t min_slab_bytes) {
  if (!block_bytes || n < 1) return 0;
  const uint64_t limit = 1ull << 40;  // a slab beyond 1 TiB is no slab
  uint64_t l = 1;
  for (int i = 0; i < n; ++i) {
    const uint64_t b = block_bytes[i];
    if (b == 0 || b > limit) return 0;
    uint64_t x = l, y = b;
    while (y) {  // gcd
      const uint64_t t = x % y;
      x = y;
      y = t;
    }
    const uint64_t f = b / x;
    if (l > limit / f) return 0;
    l *= f;
  }
  const uint64_t k = min_slab_bytes <= l ? 1 : (min_slab_bytes + l - 1) / l;
  if (k > limit / l) return 0;
  return k * l;
}

int fs_model_register_tokens(fs_pool* p, int kv_dtype, int n_kv_heads, int head_dim, int n_layers, int tokens_per_block,
                             fs_model_t* out) {
  if (!p || !out) return FS_ERR_INVALID;
  const uint64_t b = fs_block_bytes(kv_dtype, n_kv_heads, head_dim, n_layers, tokens_per_block);
  if (b == 0) {
    set_error("fs_model_register_tokens: unsupported model shape or token count");
    return FS_ERR_INVALID;
  }
  // the block's own size is its budget; the token count is imposed (alignment padding may leave room for more)
  return register_model(p, kv_dtype, n_kv_heads, head_dim, n_layers, b, tokens_per_block, out);
}

int fs_model_register(fs_pool* p, int kv_dtype, int n_kv_heads, int head_dim, int n_layers, fs_model_t* out) {
  if (!p) return FS_ERR_INVALID;
  return fs_model_register_ex(p, kv_dtype, n_kv_heads, head_dim, n_layers, p->slab_bytes, out);
}

static Model* get_model(fs_pool* p, fs_model_t m) {
  if (!p || m < 0 || m >= kMaxModels || !p->models[m].in_use) return nullptr;
  return &p->models[m];
}

int fs_model_set_fp8_scales(fs_pool* p, fs_model_t model, const float* k_scale, const float* v_scale) {
  Model* M = get_model(p, model);
  if (!M || !k_scale || !v_scale || M->g.kv_dtype != FS_KV_FP8_E4M3) return FS_ERR_INVALID;
  const size_t n = (size_t)M->g.n_layers * M->g.n_kv_heads;
  for (size_t i = 0; i < n; ++i)
    if (!(k_scale[i] > 0.f) || !(v_scale[i] > 0.f) || k_scale[i] > 3e38f || v_scale[i] > 3e38f) {
      set_error("fs_model_set_fp8_scales: scales must be positive and finite");
      return FS_ERR_INVALID;
    }
  hipError_t e;
  if (!M->d_k_scale) {
    if ((e = hipMalloc((void**)&M->d_k_scale, n * sizeof(float))) != hipSuccess) return device_error(e, "hipMalloc");
    if ((e = hipMalloc((void**)&M->d_v_scale, n * sizeof(float))) != hipSuccess) return device_error(e, "hipMalloc");
  }
  if ((e = hipMemcpy(M->d_k_scale, k_scale, n * sizeof(float), hipMemcpyHostToDevice)) != hipSuccess)
    return device_error(e, "hipMemcpy(k_scale)");
  if ((e = hipMemcpy(M->d_v_scale, v_scale, n * sizeof(float), hipMemcpyHostToDevice)) != hipSuccess)
    return device_error(e, "hipMemcpy(v_scale)");
  return FS_OK;
}

int fs_model_unregister(fs_pool* p, fs_model_t model) {
  Model* M = get_model(p, model);
  if (!M) return FS_ERR_INVALID;
  if (M->live_blocks) {
    set_error("fs_model_unregister: model still holds blocks");
    return FS_ERR_STATE;
  }
  if (M->d_k_scale) (void)hipFree(M->d_k_scale);
  if (M->d_v_scale) (void)hipFree(M->d_v_scale);
  *M = Model();
  return FS_OK;
}

int fs_model_geometry(fs_pool* p, fs_model_t model, fs_geometry_t* out) {
  Model* M = get_model(p, model);
  if (!M || !out) return FS_ERR_INVALID;
  *out = M->g;
  return FS_OK;
}

int fs_block_alloc(fs_pool* p, fs_model_t model, int32_t* blk_id_out) {
  Model* M = get_model(p, model);
  if (!M || !blk_id_out) return FS_ERR_INVALID;
  const int32_t bps = M->g.blocks_per_slab;
  int32_t slab;
  if (!M->partial_slabs.empty()) {
    slab = *M->partial_slabs.begin();
  } else {
    if (p->free_stack.empty()) return FS_ERR_NOMEM;
    slab = p->free_stack.back();
    p->free_stack.pop_back();
    p->key[slab] = model;
    p->used[slab] = 0;
    p->state[slab] = FS_SLAB_PARTIAL;
    if (bps > 1) M->partial_slabs.insert(slab);
  }
  uint8_t* row = &M->live[(size_t)slab * bps];
  const int32_t local = (int32_t)(std::find(row, row + bps, (uint8_t)0) - row);
  row[local] = 1;
  M->live_blocks += 1;
  if (++p->used[slab] == bps) {
    p->state[slab] = FS_SLAB_FULL;
    if (bps > 1) M->partial_slabs.erase(slab);
  }
  *blk_id_out = slab * bps + local;
  return FS_OK;
}

int fs_block_free(fs_pool* p, fs_model_t model, int32_t blk_id) {
  Model* M = get_model(p, model);
  if (!M) return FS_ERR_INVALID;
  const int32_t bps = M->g.blocks_per_slab;
  if (blk_id < 0 || (int64_t)blk_id >= p->n_slabs * bps) return FS_ERR_INVALID;
  const int32_t slab = blk_id / bps, local = blk_id % bps;
  if (p->key[slab] != model || !M->live[(size_t)slab * bps + local]) {
    set_error("fs_block_free: block is not live or belongs to another model");
    return FS_ERR_STATE;
  }
  M->live[(size_t)slab * bps + local] = 0;
  M->live_blocks -= 1;
  if (--p->used[slab] == 0) {
    if (bps > 1) M->partial_slabs.erase(slab);
    p->state[slab] = FS_SLAB_FREE;
    p->key[slab] = -1;
    p->free_stack.push_back(slab);
  } else {
    p->state[slab] = FS_SLAB_PARTIAL;
    M->partial_slabs.insert(slab);
  }
  return FS_OK;
}

int fs_blocks_alloc(fs_pool* p, fs_model_t model, int32_t n, int32_t* blk_ids_out) {
  Model* M = get_model(p, model);
  if (!M || n < 0 || (n > 0 && !blk_ids_out)) return FS_ERR_INVALID;
  // all or none: what this model can still get
  const int64_t bps = M->g.blocks_per_slab;
  int64_t avail = (int64_t)p->free_stack.size() * bps;
  for (auto it = M->partial_slabs.begin(); it != M->partial_slabs.end() && avail < n; ++it) avail += bps - p->used[*it];
  if (avail < n) return FS_ERR_NOMEM;
  for (int32_t i = 0; i < n; ++i) {
    const int rc = fs_block_alloc(p, model, blk_ids_out + i);
    if (rc != FS_OK) return rc;  // (cannot happen: counted above)
  }
  return FS_OK;
}

int fs_blocks_free(fs_pool* p, fs_model_t model, const int32_t* blk_ids, int32_t n) {
  if (!get_model(p, model) || n < 0 || (n > 0 && !blk_ids)) return FS_ERR_INVALID;
  for (int32_t i = 0; i < n; ++i) {
    const int rc = fs_block_free(p, model, blk_ids[i]);
    if (rc != FS_OK) return rc;
  }
  return FS_OK;
}

int fs_pool_stats(fs_pool* p, fs_pool_stats_t* out) {
  if (!p || !out) return FS_ERR_INVALID;
  fs_pool_stats_t s{};
  s.n_slabs = p->n_slabs;
  for (int64_t i = 0; i < p->n_slabs; ++i) {
    if (p->state[i] == FS_SLAB_FREE) ++s.slabs_free;
    else if (p->state[i] == FS_SLAB_PARTIAL) ++s.slabs_partial;
    else ++s.slabs_full;
  }
  for (const auto& m : p->models) {
    if (!m.in_use) continue;
    ++s.n_models;
    s.live_blocks += m.live_blocks;
    s.stranded_bytes += (uint64_t)m.live_blocks * (m.g.block_budget - m.g.block_bytes);
  }
  *out = s;
  return FS_OK;
}

int fs_model_stats(fs_pool* p, fs_model_t model, fs_model_stats_t* out) {
  if (!p || !out || model < 0 || model >= kMaxModels || !p->models[model].in_use) {
    set_error("fs_model_stats: unknown pool or model");
    return FS_ERR_INVALID;
  }
  const Model& M = p->models[model];
  fs_model_stats_t s{};
  for (int64_t i = 0; i < p->n_slabs; ++i) {
    if (p->key[i] != model) continue;
    if (p->state[i] == FS_SLAB_PARTIAL) ++s.slabs_partial;
    else if (p->state[i] == FS_SLAB_FULL) ++s.slabs_full;
    s.free_blocks_in_partial_slabs += M.g.blocks_per_slab - p->used[i];
  }
  s.live_blocks = M.live_blocks;
  s.live_bytes = (uint64_t)M.live_blocks * M.g.block_budget;
  s.stranded_bytes = (uint64_t)M.live_blocks * (M.g.block_budget - M.g.block_bytes);
  *out = s;
  return FS_OK;
}

int fs_pool_dump(fs_pool* p, int32_t* slab_state, int32_t* slab_key, int32_t* slab_used, int32_t* free_stack,
                 int64_t* n_free) {
  if (!p || !slab_state || !slab_key || !slab_used || !free_stack || !n_free) return FS_ERR_INVALID;
  const size_t n = (size_t)p->n_slabs;
  memcpy(slab_state, p->state.data(), n * sizeof(int32_t));
  memcpy(slab_key, p->key.data(), n * sizeof(int32_t));
  memcpy(slab_used, p->used.data(), n * sizeof(int32_t));
  memcpy(free_stack, p->free_stack.data(), p->free_stack.size() * sizeof(int32_t));
  *n_free = (int64_t)p->free_stack.size();
  return FS_OK;
}

int fs_model_dump_live(fs_pool* p, fs_model_t model, uint8_t* live) {
  Model* M = get_model(p, model);
  if (!M || !live) return FS_ERR_INVALID;
  memcpy(live, M->live.data(), M->live.size());
  return FS_OK;
}

}  // extern "C"
