/*
 * CPU oracle for decode attention over a shared, precision-aware KV slab pool.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct
 * implementation used only to check the HIP library and to be timed as the CPU
 * baseline.  The product path never links, loads or calls it, and it shares no
 * code, header, table or constant generator with the HIP path.
 *
 * What it follows (FineServe, arXiv 2509.06261):
 *   - Sec. 3.2 (C1): KV block size = TokensPerBlock x TokenSize + Quant.Params,
 *     TokenSize = (#Heads/TP) x HeadDim x 2 x bytes(precision); per-token
 *     quantization parameters live inside the block.
 *   - Sec. 5.1: one pre-allocated shared KV tensor is carved into uniform slabs;
 *     each engine views the same bytes as an array of blocks of its own size.
 *   - Sec. 5.2: Blk ID = slab ID x (#blocks per slab) + local block ID; slab table
 *     with FREE / PARTIAL / FULL states; allocate from a matching slab or carve a
 *     new one; an emptied slab returns to the shared tensor.
 *   - Sec. 2.1 / 2.3: decode attention reads every cached token of a sequence
 *     through its block table as if the KV were contiguous; the prefill phase
 *     processes the prompt's tokens, each attending to the tokens up to itself
 *     (Sec. 4.2's chunked prefill: a chunk of the prompt at a time, against the
 *     cache that the earlier chunks and the chunk itself have filled).
 * The paper fixes no byte layout, no quantizer arithmetic and no allocator
 * tie-breaks; the readings used here are listed where each function is defined.
 *
 * Parity pins (tests/ with -m "not gpu"): the paper's worked block-id example
 * (Fig. "kv_slab_detail"), closed-form geometry, allocator invariants on random
 * traces, exhaustive E4M3 / fp16 tables against independent definitions, the
 * quantizer error bounds and idempotence, dense fp64 softmax(qK^T)V from numpy,
 * placement invariance and the degenerate attention cases; prefill attention
 * against decode attention of the truncated sequence, a dense masked numpy
 * softmax, causality under perturbation of later tokens and chunk invariance.
 * The allocator
 * tie-break policy itself (which free slab is taken first) is fixed by this
 * repository's own reading, not by the paper: "parity unpinned" beyond the
 * invariants.
 *
 * Plain C11, no dependencies beyond libm and pthreads.  All floating-point
 * quantizer arithmetic is IEEE binary32 with round-to-nearest-even and no FMA
 * contraction (build with -ffp-contract=off); attention is binary64.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { FSO_FP16 = 0, FSO_FP8 = 1, FSO_INT8 = 2, FSO_INT4 = 3 };
enum { FSO_OK = 0, FSO_ERR_INVALID = -1, FSO_ERR_NOMEM = -2, FSO_ERR_STATE = -3 };
enum { FSO_FREE = 0, FSO_PARTIAL = 1, FSO_FULL = 2 };

/* ------------------------------------------------------------------------- */
/* Geometry (Sec. 3.2 block-size and token-size equations, inverted: the byte  */
/* budget of a block is given and the token count is derived).                 */
/* ------------------------------------------------------------------------- */

typedef struct {
  int32_t dtype, n_kv_heads, head_dim, n_layers;
  int32_t tokens_per_block; /* T */
  int32_t param_bytes;      /* per token, per head, per K or V: 0, 0, 2, 4 */
  uint64_t block_budget;    /* bytes reserved per block (divides slab_bytes) */
  uint64_t row_bytes;       /* head_dim * bits / 8 */
  uint64_t kv_tile;         /* bytes of the K (or V) tile of one head */
  uint64_t par_tile;        /* bytes of the K (or V) parameter tile of one head */
  uint64_t head_chunk;      /* K tile | V tile | K params | V params */
  uint64_t layer_bytes;     /* all heads, rounded up to 256 */
  uint64_t block_bytes;     /* all layers: the defined bytes of a block */
} fso_geom;

static uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

static int dtype_bits(int dtype) {
  switch (dtype) {
    case FSO_FP16: return 16;
    case FSO_FP8: return 8;
    case FSO_INT8: return 8;
    case FSO_INT4: return 4;
    default: return 0;
  }
}

/* Fills every size field of g for a candidate token count T. */
static void geom_for_tokens(fso_geom* g, int T) {
  int bits = dtype_bits(g->dtype);
  g->param_bytes = g->dtype == FSO_INT8 ? 2 : (g->dtype == FSO_INT4 ? 4 : 0);
  g->row_bytes = (uint64_t)g->head_dim * (uint64_t)bits / 8;
  g->kv_tile = round_up((uint64_t)T * g->row_bytes, 16);
  g->par_tile = g->param_bytes ? round_up((uint64_t)T * (uint64_t)g->param_bytes, 16) : 0;
  g->head_chunk = 2 * g->kv_tile + 2 * g->par_tile;
  g->layer_bytes = round_up((uint64_t)g->n_kv_heads * g->head_chunk, 256);
  g->block_bytes = (uint64_t)g->n_layers * g->layer_bytes;
  g->tokens_per_block = T;
}

/* T = the largest token count whose laid-out block fits block_budget.  The block
 * size grows monotonically with T, so a linear search upward is exact. */
int fso_geometry(int dtype, int n_kv_heads, int head_dim, int n_layers, uint64_t block_budget, fso_geom* out) {
  if (dtype_bits(dtype) == 0 || n_kv_heads < 1 || head_dim < 2 || (head_dim & 1) || n_layers < 1 ||
      block_budget == 0)
    return FSO_ERR_INVALID;
  fso_geom g;
  memset(&g, 0, sizeof g);
  g.dtype = dtype;
  g.n_kv_heads = n_kv_heads;
  g.head_dim = head_dim;
  g.n_layers = n_layers;
  g.block_budget = block_budget;
  geom_for_tokens(&g, 1);
  if (g.block_bytes > block_budget) return FSO_ERR_INVALID;
  int T = 1;
  for (;;) {
    fso_geom n = g;
    geom_for_tokens(&n, T + 1);
    if (n.block_bytes > block_budget) break;
    g = n;
    ++T;
  }
  *out = g;
  return FSO_OK;
}

/* Sec. 3.2, forward: bytes of the laid-out block that holds T tokens (0: invalid arguments). */
uint64_t fso_block_bytes(int dtype, int n_kv_heads, int head_dim, int n_layers, int T) {
  if (dtype_bits(dtype) == 0 || n_kv_heads < 1 || head_dim < 2 || (head_dim & 1) || n_layers < 1 || T < 1) return 0;
  fso_geom g;
  memset(&g, 0, sizeof g);
  g.dtype = dtype;
  g.n_kv_heads = n_kv_heads;
  g.head_dim = head_dim;
  g.n_layers = n_layers;
  geom_for_tokens(&g, T);
  return g.block_bytes;
}

/* Sec. 5.2: the slab size is a multiple of the least common multiple of the co-located block sizes; here the
 * smallest such multiple that is at least min_slab (0: an entry is 0, or the result exceeds 2^40).  The lcm is
 * found as the first multiple of the largest block size that every block size divides. */
uint64_t fso_lcm_slab_bytes(const uint64_t* block_bytes, int n, uint64_t min_slab) {
  if (!block_bytes || n < 1) return 0;
  uint64_t big = 0;
  for (int i = 0; i < n; ++i) {
    if (block_bytes[i] == 0) return 0;
    if (block_bytes[i] > big) big = block_bytes[i];
  }
  const uint64_t limit = 1ull << 40;
  for (uint64_t cand = big; cand <= limit; cand += big) {
    int all = 1;
    for (int i = 0; i < n; ++i)
      if (cand % block_bytes[i]) all = 0;
    if (all) {
      uint64_t slab = cand;
      while (slab < min_slab) slab += cand;
      return slab <= limit ? slab : 0;
    }
  }
  return 0;
}

/* View mapping of Sec. 5.1: block blk_id of a model starts at blk_id * block_budget
 * from the pool base (= slab * slab_bytes + local * block_budget). */
uint64_t fso_block_offset(const fso_geom* g, int32_t blk_id) { return (uint64_t)blk_id * g->block_budget; }

/* Byte offset (from the pool base) of the K (which=0) or V (which=1) row of token slot
 * tok of head `head`, layer `layer`, in block blk_id. */
uint64_t fso_row_offset(const fso_geom* g, int32_t blk_id, int layer, int head, int which, int tok) {
  return fso_block_offset(g, blk_id) + (uint64_t)layer * g->layer_bytes + (uint64_t)head * g->head_chunk +
         (which ? g->kv_tile : 0) + (uint64_t)tok * g->row_bytes;
}

/* Byte offset of the per-token parameters (INT8: fp16 scale; INT4: fp16 scale, fp16 zero-point). */
uint64_t fso_param_offset(const fso_geom* g, int32_t blk_id, int layer, int head, int which, int tok) {
  return fso_block_offset(g, blk_id) + (uint64_t)layer * g->layer_bytes + (uint64_t)head * g->head_chunk +
         2 * g->kv_tile + (which ? g->par_tile : 0) + (uint64_t)tok * (uint64_t)g->param_bytes;
}

/* ------------------------------------------------------------------------- */
/* Slab allocator (Sec. 5.2).  Tie-breaks, which the paper leaves open:        */
/*  - free slabs form a LIFO stack that initially pops 0, 1, 2, ...; a slab     */
/*    that becomes empty is pushed on top;                                      */
/*  - the slab key is the model (all models share one block byte size per pool  */
/*    configuration, so size alone cannot tell their token layouts apart);      */
/*  - allocation takes the PARTIAL slab of that key with the lowest slab id and  */
/*    in it the lowest free local id; otherwise it carves the top free slab.     */
/* ------------------------------------------------------------------------- */

#define FSO_MAX_MODELS 64

typedef struct {
  int in_use;
  fso_geom geom;
  int64_t bps;         /* blocks per slab */
  int64_t live_blocks; /* blocks currently held */
  int64_t n_partial;   /* slabs of this key in PARTIAL state */
  uint8_t* live;       /* [n_slabs * bps] occupancy */
} fso_model;

typedef struct {
  uint64_t slab_bytes, pool_bytes;
  int64_t n_slabs;
  int32_t* state; /* FSO_FREE / PARTIAL / FULL */
  int32_t* key;   /* owning model or -1 */
  int32_t* used;  /* live blocks in the slab */
  int32_t* free_stack;
  int64_t n_free;
  fso_model models[FSO_MAX_MODELS];
} fso_pool;

fso_pool* fso_pool_new(uint64_t slab_bytes, uint64_t pool_bytes) {
  if (slab_bytes == 0 || pool_bytes == 0 || pool_bytes % slab_bytes) return NULL;
  uint64_t n = pool_bytes / slab_bytes;
  if (n >= (1ull << 31)) return NULL;
  fso_pool* p = (fso_pool*)calloc(1, sizeof *p);
  p->slab_bytes = slab_bytes;
  p->pool_bytes = pool_bytes;
  p->n_slabs = (int64_t)n;
  p->state = (int32_t*)calloc(n, sizeof(int32_t));
  p->key = (int32_t*)malloc(n * sizeof(int32_t));
  p->used = (int32_t*)calloc(n, sizeof(int32_t));
  p->free_stack = (int32_t*)malloc(n * sizeof(int32_t));
  for (uint64_t i = 0; i < n; ++i) {
    p->key[i] = -1;
    p->free_stack[i] = (int32_t)(n - 1 - i); /* top of the stack is slab 0 */
  }
  p->n_free = (int64_t)n;
  return p;
}

void fso_pool_delete(fso_pool* p) {
  if (!p) return;
  for (int m = 0; m < FSO_MAX_MODELS; ++m) free(p->models[m].live);
  free(p->state);
  free(p->key);
  free(p->used);
  free(p->free_stack);
  free(p);
}

/* Registers a model; returns its id (>= 0) or an error.  block_budget must divide slab_bytes. */
int fso_model_add(fso_pool* p, int dtype, int n_kv_heads, int head_dim, int n_layers, uint64_t block_budget) {
  if (!p || block_budget == 0 || p->slab_bytes % block_budget) return FSO_ERR_INVALID;
  if (p->pool_bytes / block_budget >= (1ull << 31)) return FSO_ERR_INVALID;
  fso_geom g;
  int rc = fso_geometry(dtype, n_kv_heads, head_dim, n_layers, block_budget, &g);
  if (rc != FSO_OK) return rc;
  for (int m = 0; m < FSO_MAX_MODELS; ++m) {
    if (!p->models[m].in_use) {
      fso_model* M = &p->models[m];
      memset(M, 0, sizeof *M);
      M->in_use = 1;
      M->geom = g;
      M->bps = (int64_t)(p->slab_bytes / block_budget);
      M->live = (uint8_t*)calloc((size_t)(p->n_slabs * M->bps), 1);
      return m;
    }
  }
  return FSO_ERR_NOMEM;
}

/* Sec. 3.2 / 5.2, the paper's direction: a model whose blocks hold exactly T tokens; the block's own size is its
 * budget and must divide slab_bytes. */
int fso_model_add_tokens(fso_pool* p, int dtype, int n_kv_heads, int head_dim, int n_layers, int T) {
  uint64_t b = fso_block_bytes(dtype, n_kv_heads, head_dim, n_layers, T);
  if (!p || b == 0 || p->slab_bytes % b) return FSO_ERR_INVALID;
  if (p->pool_bytes / b >= (1ull << 31)) return FSO_ERR_INVALID;
  for (int m = 0; m < FSO_MAX_MODELS; ++m) {
    if (!p->models[m].in_use) {
      fso_model* M = &p->models[m];
      memset(M, 0, sizeof *M);
      M->in_use = 1;
      M->geom.dtype = dtype;
      M->geom.n_kv_heads = n_kv_heads;
      M->geom.head_dim = head_dim;
      M->geom.n_layers = n_layers;
      M->geom.block_budget = b;
      geom_for_tokens(&M->geom, T);
      M->bps = (int64_t)(p->slab_bytes / b);
      M->live = (uint8_t*)calloc((size_t)(p->n_slabs * M->bps), 1);
      return m;
    }
  }
  return FSO_ERR_NOMEM;
}

int fso_model_remove(fso_pool* p, int model) {
  if (!p || model < 0 || model >= FSO_MAX_MODELS || !p->models[model].in_use) return FSO_ERR_INVALID;
  if (p->models[model].live_blocks) return FSO_ERR_STATE;
  free(p->models[model].live);
  memset(&p->models[model], 0, sizeof p->models[model]);
  return FSO_OK;
}

int fso_model_geometry(const fso_pool* p, int model, fso_geom* out) {
  if (!p || model < 0 || model >= FSO_MAX_MODELS || !p->models[model].in_use) return FSO_ERR_INVALID;
  *out = p->models[model].geom;
  return FSO_OK;
}

int fso_block_alloc(fso_pool* p, int model, int32_t* blk_id_out) {
  if (!p || model < 0 || model >= FSO_MAX_MODELS || !p->models[model].in_use || !blk_id_out) return FSO_ERR_INVALID;
  fso_model* M = &p->models[model];
  int64_t slab = -1;
  if (M->n_partial > 0) {
    for (int64_t s = 0; s < p->n_slabs; ++s)
      if (p->state[s] == FSO_PARTIAL && p->key[s] == model) {
        slab = s;
        break;
      }
  }
  if (slab < 0) {
    if (p->n_free == 0) return FSO_ERR_NOMEM;
    slab = p->free_stack[--p->n_free];
    p->key[slab] = model;
    p->state[slab] = FSO_PARTIAL;
    p->used[slab] = 0;
    M->n_partial += 1;
  }
  int64_t local = 0;
  while (M->live[slab * M->bps + local]) ++local; /* a PARTIAL slab always has a free slot */
  M->live[slab * M->bps + local] = 1;
  p->used[slab] += 1;
  M->live_blocks += 1;
  if (p->used[slab] == M->bps) {
    p->state[slab] = FSO_FULL;
    M->n_partial -= 1;
  }
  *blk_id_out = (int32_t)(slab * M->bps + local); /* Sec. 5.2 block-id equation */
  return FSO_OK;
}

int fso_block_free(fso_pool* p, int model, int32_t blk_id) {
  if (!p || model < 0 || model >= FSO_MAX_MODELS || !p->models[model].in_use) return FSO_ERR_INVALID;
  fso_model* M = &p->models[model];
  if (blk_id < 0 || (int64_t)blk_id >= p->n_slabs * M->bps) return FSO_ERR_INVALID;
  int64_t slab = blk_id / M->bps, local = blk_id % M->bps;
  if (p->state[slab] == FSO_FREE || p->key[slab] != model || !M->live[slab * M->bps + local]) return FSO_ERR_STATE;
  M->live[slab * M->bps + local] = 0;
  if (p->state[slab] == FSO_FULL) M->n_partial += 1; /* FULL -> PARTIAL (or straight on to FREE) */
  p->used[slab] -= 1;
  M->live_blocks -= 1;
  if (p->used[slab] == 0) {
    p->state[slab] = FSO_FREE;
    p->key[slab] = -1;
    M->n_partial -= 1;
    p->free_stack[p->n_free++] = (int32_t)slab;
  } else {
    p->state[slab] = FSO_PARTIAL;
  }
  return FSO_OK;
}

int64_t fso_pool_n_slabs(const fso_pool* p) { return p->n_slabs; }
int64_t fso_pool_n_free(const fso_pool* p) { return p->n_free; }
int64_t fso_model_live_blocks(const fso_pool* p, int model) { return p->models[model].live_blocks; }
int64_t fso_model_blocks_per_slab(const fso_pool* p, int model) { return p->models[model].bps; }

/* Copies the slab table: state/key/used per slab and the free stack bottom-to-top. */
void fso_pool_dump(const fso_pool* p, int32_t* state, int32_t* key, int32_t* used, int32_t* free_stack) {
  memcpy(state, p->state, (size_t)p->n_slabs * sizeof(int32_t));
  memcpy(key, p->key, (size_t)p->n_slabs * sizeof(int32_t));
  memcpy(used, p->used, (size_t)p->n_slabs * sizeof(int32_t));
  memcpy(free_stack, p->free_stack, (size_t)p->n_free * sizeof(int32_t));
}

/* Occupancy of every block id of a model: live[n_slabs * bps]. */
void fso_model_dump_live(const fso_pool* p, int model, uint8_t* live) {
  const fso_model* M = &p->models[model];
  memcpy(live, M->live, (size_t)(p->n_slabs * M->bps));
}

/* ------------------------------------------------------------------------- */
/* Number formats.                                                             */
/* ------------------------------------------------------------------------- */

/* IEEE binary16 -> binary32, exact. */
float fso_f16_to_f32(uint16_t h) {
  int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  float v;
  if (e == 0)
    v = ldexpf((float)m, -24);
  else if (e == 31)
    v = m ? NAN : INFINITY;
  else
    v = ldexpf(1.0f + (float)m / 1024.0f, e - 15);
  return sign ? -v : v;
}

/* binary32 -> binary16, round-to-nearest-even; overflow gives infinity. */
uint16_t fso_f32_to_f16(float x) {
  uint16_t sign = signbit(x) ? 0x8000 : 0;
  if (isnan(x)) return (uint16_t)(sign | 0x7E00);
  float a = fabsf(x);
  if (a >= 65520.0f) return (uint16_t)(sign | 0x7C00); /* 65520 is the midpoint above the largest finite value */
  if (a < ldexpf(1.0f, -14)) {
    /* subnormal range: spacing 2^-24; a * 2^24 is exact, rintf rounds half to even */
    int q = (int)rintf(ldexpf(a, 24));
    return (uint16_t)(sign | q); /* q == 1024 is exactly the smallest normal */
  }
  int e;
  float m = frexpf(a, &e); /* a = m * 2^e, m in [0.5, 1) */
  int mant = (int)rintf((2.0f * m - 1.0f) * 1024.0f);
  int bits = ((e - 1 + 15) << 10) + mant; /* mant == 1024 carries into the exponent */
  return (uint16_t)(sign | bits);
}

/* fp16 scale used by the INT8 / INT4 quantizers: nearest fp16, saturating at the largest
 * finite value, and 1.0 when the scale rounds to zero (all-zero row, or underflow). */
static uint16_t scale_to_f16(float s32) {
  uint16_t s = fso_f32_to_f16(s32);
  if ((s & 0x7FFF) >= 0x7C00) s = 0x7BFF;
  if ((s & 0x7FFF) == 0) s = 0x3C00;
  return s;
}

/* OCP FP8 E4M3 ("FN": bias 7, no infinity, 0x7F/0xFF NaN, largest finite 448). */
float fso_e4m3_decode(uint8_t b) {
  int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
  float v;
  if (e == 15 && m == 7)
    v = NAN;
  else if (e == 0)
    v = ldexpf((float)m / 8.0f, -6);
  else
    v = ldexpf(1.0f + (float)m / 8.0f, e - 7);
  return sign ? -v : v;
}

/* Nearest E4M3 value, ties to the even code, magnitudes above 448 saturate to 448; the
 * sign of the input (including -0 and values that round to zero) is kept. */
uint8_t fso_e4m3_encode(float y) {
  uint8_t sign = signbit(y) ? 0x80 : 0;
  if (isnan(y)) return (uint8_t)(sign | 0x7F);
  double a = fabs((double)y);
  if (a >= 448.0) return (uint8_t)(sign | 0x7E);
  /* codes 0x00..0x7E are increasing in value: find the largest code whose value is <= a */
  int lo = 0, hi = 0x7E;
  while (hi - lo > 1) {
    int mid = (lo + hi) / 2;
    if ((double)fso_e4m3_decode((uint8_t)mid) <= a)
      lo = mid;
    else
      hi = mid;
  }
  double dl = a - (double)fso_e4m3_decode((uint8_t)lo), dh = (double)fso_e4m3_decode((uint8_t)hi) - a;
  int code;
  if (dl < dh)
    code = lo;
  else if (dh < dl)
    code = hi;
  else
    code = (lo & 1) ? hi : lo;
  return (uint8_t)(sign | code);
}

/* INT8, symmetric, one fp16 scale per (token, KV head) row. */
void fso_quant_row_int8(const float* x, int D, int8_t* q, uint16_t* scale_out) {
  float amax = 0.0f;
  for (int d = 0; d < D; ++d) amax = fmaxf(amax, fabsf(x[d]));
  float s32 = amax / 127.0f;
  uint16_t s = scale_to_f16(s32);
  float sf = fso_f16_to_f32(s);
  for (int d = 0; d < D; ++d) {
    float r = rintf(x[d] / sf);
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    q[d] = (int8_t)r;
  }
  *scale_out = s;
}

/* INT4, asymmetric, fp16 scale and integer-valued fp16 zero-point per (token, KV head) row;
 * the range is widened to contain 0; two codes per byte, element 2j in the low nibble. */
void fso_quant_row_int4(const float* x, int D, uint8_t* packed, uint16_t* scale_out, uint16_t* zp_out) {
  float lo = 0.0f, hi = 0.0f;
  for (int d = 0; d < D; ++d) {
    lo = fminf(lo, x[d]);
    hi = fmaxf(hi, x[d]);
  }
  float s32 = (hi - lo) / 15.0f;
  uint16_t s = scale_to_f16(s32);
  float sf = fso_f16_to_f32(s);
  float z = rintf(-lo / sf);
  z = fminf(fmaxf(z, 0.0f), 15.0f);
  for (int d = 0; d < D; d += 2) {
    float a = rintf(x[d] / sf) + z, b = rintf(x[d + 1] / sf) + z;
    a = fminf(fmaxf(a, 0.0f), 15.0f);
    b = fminf(fmaxf(b, 0.0f), 15.0f);
    packed[d / 2] = (uint8_t)((unsigned)a | ((unsigned)b << 4));
  }
  *scale_out = s;
  *zp_out = fso_f32_to_f16(z);
}

/* ------------------------------------------------------------------------- */
/* KV append: quantize the new K/V rows of tokens (seq_idx[i], pos[i]) and     */
/* write them, with their parameters, into the slab blocks the block table     */
/* names (Sec. 2.1 "appends its keys and values"; formats of Sec. 2.2).        */
/* ------------------------------------------------------------------------- */

static float src_elem(const void* src, int src_is_f32, uint64_t i) {
  return src_is_f32 ? ((const float*)src)[i] : fso_f16_to_f32(((const uint16_t*)src)[i]);
}

/* pool_mem: host mirror of the pool (base of the shared KV tensor).
 * k_new/v_new: [n_tokens][H][D] fp16 (src_is_f32=0) or fp32 (1).
 * k_scale/v_scale: FP8 only, [n_layers][H] fp32 static scales. */
int fso_kv_append(uint8_t* pool_mem, const fso_geom* g, int layer, const void* k_new, const void* v_new,
                  int src_is_f32, const int32_t* seq_idx, const int32_t* pos, const int32_t* block_tables,
                  int max_blocks, int64_t n_tokens, const float* k_scale, const float* v_scale) {
  const int H = g->n_kv_heads, D = g->head_dim, T = g->tokens_per_block;
  if (layer < 0 || layer >= g->n_layers) return FSO_ERR_INVALID;
  if (g->dtype == FSO_FP8 && (!k_scale || !v_scale)) return FSO_ERR_INVALID;
  float* row = (float*)malloc((size_t)D * sizeof(float));
  for (int64_t i = 0; i < n_tokens; ++i) {
    int p = pos[i];
    if (p < 0 || p / T >= max_blocks) {
      free(row);
      return FSO_ERR_INVALID;
    }
    int32_t blk = block_tables[(int64_t)seq_idx[i] * max_blocks + p / T];
    int tok = p % T;
    for (int which = 0; which < 2; ++which) {
      const void* src = which ? v_new : k_new;
      for (int h = 0; h < H; ++h) {
        for (int d = 0; d < D; ++d) row[d] = src_elem(src, src_is_f32, ((uint64_t)i * H + h) * D + d);
        uint8_t* dst = pool_mem + fso_row_offset(g, blk, layer, h, which, tok);
        uint8_t* par = pool_mem + fso_param_offset(g, blk, layer, h, which, tok);
        switch (g->dtype) {
          case FSO_FP16:
            for (int d = 0; d < D; ++d) {
              uint16_t b = fso_f32_to_f16(row[d]);
              memcpy(dst + 2 * d, &b, 2);
            }
            break;
          case FSO_FP8: {
            float sc = (which ? v_scale : k_scale)[layer * H + h];
            for (int d = 0; d < D; ++d) dst[d] = fso_e4m3_encode(row[d] / sc);
            break;
          }
          case FSO_INT8: {
            uint16_t s;
            fso_quant_row_int8(row, D, (int8_t*)dst, &s);
            memcpy(par, &s, 2);
            break;
          }
          case FSO_INT4: {
            uint16_t s, z;
            fso_quant_row_int4(row, D, dst, &s, &z);
            memcpy(par, &s, 2);
            memcpy(par + 2, &z, 2);
            break;
          }
        }
      }
    }
  }
  free(row);
  return FSO_OK;
}

/* ------------------------------------------------------------------------- */
/* Decode attention: for sequence b and query head h (KV head g = h / (n_q /   */
/* n_kv)), s_t = sm_scale * <q, K^_t>, p = softmax_t(s), out = sum_t p_t V^_t   */
/* over the n_b cached tokens, K^/V^ read from the pool bytes through the block  */
/* table and dequantized exactly; every sum in binary64.                        */
/* ------------------------------------------------------------------------- */

/* Dequantizes one stored row into D doubles. */
static void load_row(const uint8_t* pool_mem, const fso_geom* g, int32_t blk, int layer, int head, int which,
                     int tok, double static_scale, double* out) {
  const int D = g->head_dim;
  const uint8_t* src = pool_mem + fso_row_offset(g, blk, layer, head, which, tok);
  const uint8_t* par = pool_mem + fso_param_offset(g, blk, layer, head, which, tok);
  switch (g->dtype) {
    case FSO_FP16:
      for (int d = 0; d < D; ++d) {
        uint16_t b;
        memcpy(&b, src + 2 * d, 2);
        out[d] = (double)fso_f16_to_f32(b);
      }
      break;
    case FSO_FP8:
      for (int d = 0; d < D; ++d) out[d] = (double)fso_e4m3_decode(src[d]) * static_scale;
      break;
    case FSO_INT8: {
      uint16_t s;
      memcpy(&s, par, 2);
      double sc = (double)fso_f16_to_f32(s);
      for (int d = 0; d < D; ++d) out[d] = (double)(int8_t)src[d] * sc;
      break;
    }
    case FSO_INT4: {
      uint16_t s, z;
      memcpy(&s, par, 2);
      memcpy(&z, par + 2, 2);
      double sc = (double)fso_f16_to_f32(s), zp = (double)fso_f16_to_f32(z);
      for (int d = 0; d < D; ++d) {
        int code = (src[d / 2] >> ((d & 1) * 4)) & 15;
        out[d] = ((double)code - zp) * sc;
      }
      break;
    }
  }
}

/* Dense dequantized view of one sequence: k_out/v_out [n_tokens][H][D] doubles. */
int fso_dequant_sequence(const uint8_t* pool_mem, const fso_geom* g, int layer, const int32_t* block_table,
                         int n_tokens, const float* k_scale, const float* v_scale, double* k_out, double* v_out) {
  const int H = g->n_kv_heads, D = g->head_dim, T = g->tokens_per_block;
  for (int t = 0; t < n_tokens; ++t)
    for (int h = 0; h < H; ++h) {
      double ks = g->dtype == FSO_FP8 ? (double)k_scale[layer * H + h] : 1.0;
      double vs = g->dtype == FSO_FP8 ? (double)v_scale[layer * H + h] : 1.0;
      load_row(pool_mem, g, block_table[t / T], layer, h, 0, t % T, ks, k_out + ((size_t)t * H + h) * D);
      load_row(pool_mem, g, block_table[t / T], layer, h, 1, t % T, vs, v_out + ((size_t)t * H + h) * D);
    }
  return FSO_OK;
}

typedef struct {
  const uint8_t* pool_mem;
  const fso_geom* g;
  int layer, n_q_heads;
  double sm_scale;
  const uint16_t* q;
  const int32_t* block_tables;
  const int32_t* seq_lens;
  int n_seq, max_blocks;
  const float *k_scale, *v_scale;
  double *out, *lse;
  int first, stride;
} attn_job;

static void attend_sequence(const attn_job* J, int b) {
  const fso_geom* g = J->g;
  const int H = g->n_kv_heads, D = g->head_dim, T = g->tokens_per_block, nq = J->n_q_heads;
  const int group = nq / H;
  const int n = J->seq_lens[b];
  const int32_t* table = J->block_tables + (int64_t)b * J->max_blocks;
  double* row = (double*)malloc((size_t)D * sizeof(double));
  double* s = (double*)malloc((size_t)n * sizeof(double));
  double* acc = (double*)malloc((size_t)D * sizeof(double));
  for (int h = 0; h < nq; ++h) {
    const int kvh = h / group;
    const uint16_t* qh = J->q + ((int64_t)b * nq + h) * D;
    double ks = g->dtype == FSO_FP8 ? (double)J->k_scale[J->layer * H + kvh] : 1.0;
    double vs = g->dtype == FSO_FP8 ? (double)J->v_scale[J->layer * H + kvh] : 1.0;
    double m = -INFINITY;
    for (int t = 0; t < n; ++t) {
      load_row(J->pool_mem, g, table[t / T], J->layer, kvh, 0, t % T, ks, row);
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += (double)fso_f16_to_f32(qh[d]) * row[d];
      s[t] = J->sm_scale * dot;
      if (s[t] > m) m = s[t];
    }
    double l = 0.0;
    for (int d = 0; d < D; ++d) acc[d] = 0.0;
    for (int t = 0; t < n; ++t) {
      double p = exp(s[t] - m);
      l += p;
      load_row(J->pool_mem, g, table[t / T], J->layer, kvh, 1, t % T, vs, row);
      for (int d = 0; d < D; ++d) acc[d] += p * row[d];
    }
    double* o = J->out + ((int64_t)b * nq + h) * D;
    for (int d = 0; d < D; ++d) o[d] = acc[d] / l;
    if (J->lse) J->lse[(int64_t)b * nq + h] = m + log(l);
  }
  free(row);
  free(s);
  free(acc);
}

static void* attn_worker(void* arg) {
  const attn_job* J = (const attn_job*)arg;
  for (int b = J->first; b < J->n_seq; b += J->stride) attend_sequence(J, b);
  return NULL;
}

/* q: [n_seq][n_q_heads][D] fp16 bits; out: [n_seq][n_q_heads][D] doubles; lse (may be NULL):
 * [n_seq][n_q_heads].  Sequences are dealt round-robin to n_threads threads (results do not
 * depend on the thread count: each sequence is computed by exactly one thread).  seq_lens >= 1. */
int fso_decode_attention(const uint8_t* pool_mem, const fso_geom* g, int layer, int n_q_heads, double sm_scale,
                         const uint16_t* q, const int32_t* block_tables, const int32_t* seq_lens, int n_seq,
                         int max_blocks, const float* k_scale, const float* v_scale, double* out, double* lse,
                         int n_threads) {
  if (layer < 0 || layer >= g->n_layers || n_q_heads < g->n_kv_heads || n_q_heads % g->n_kv_heads)
    return FSO_ERR_INVALID;
  if (g->dtype == FSO_FP8 && (!k_scale || !v_scale)) return FSO_ERR_INVALID;
  for (int b = 0; b < n_seq; ++b)
    if (seq_lens[b] < 1 || (seq_lens[b] + g->tokens_per_block - 1) / g->tokens_per_block > max_blocks)
      return FSO_ERR_INVALID;
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 256) n_threads = 256;
  if (n_threads > n_seq) n_threads = n_seq;
  attn_job jobs[256];
  pthread_t th[256];
  for (int i = 0; i < n_threads; ++i) {
    attn_job J = {pool_mem, g, layer, n_q_heads, sm_scale, q, block_tables, seq_lens, n_seq, max_blocks,
                  k_scale, v_scale, out, lse, i, n_threads};
    jobs[i] = J;
  }
  for (int i = 1; i < n_threads; ++i) pthread_create(&th[i], NULL, attn_worker, &jobs[i]);
  if (n_threads > 0) attn_worker(&jobs[0]);
  for (int i = 1; i < n_threads; ++i) pthread_join(th[i], NULL);
  return FSO_OK;
}

/* ---------------------------------------------------------------------------------------------
 * Prefill (chunked prefill) attention over the pool: Sec. 2.1.  Sequence b has seq_lens[b] tokens
 * in the pool, the last n_b = q_offsets[b+1] - q_offsets[b] of which are the chunk being prefilled;
 * query row r of the chunk stands at position p = seq_lens[b] - n_b + r and attends to the cached
 * tokens 0..p (itself included), dequantized exactly as decode attention sees them.
 * q: [n_rows][n_q_heads][D] fp16 bits, sequences' chunks one after the other; out: same shape,
 * doubles; lse (may be NULL): [n_rows][n_q_heads].  Rows are dealt round-robin to the threads.
 * --------------------------------------------------------------------------------------------- */
typedef struct {
  const uint8_t* pool_mem;
  const fso_geom* g;
  int layer, n_q_heads;
  double sm_scale;
  const uint16_t* q;
  const int32_t* block_tables;
  const int32_t* seq_lens;
  const int32_t* q_offsets;
  int n_seq, max_blocks;
  const float *k_scale, *v_scale;
  double *out, *lse;
  int first, stride;
} prefill_job;

static void prefill_row(const prefill_job* J, int b, int row) {
  const fso_geom* g = J->g;
  const int H = g->n_kv_heads, D = g->head_dim, T = g->tokens_per_block, nq = J->n_q_heads;
  const int group = nq / H;
  const int n_new = J->q_offsets[b + 1] - J->q_offsets[b];
  const int pos = J->seq_lens[b] - n_new + (row - J->q_offsets[b]);
  const int n = pos + 1; /* tokens this row attends to */
  const int32_t* table = J->block_tables + (int64_t)b * J->max_blocks;
  double* kv = (double*)malloc((size_t)D * sizeof(double));
  double* s = (double*)malloc((size_t)n * sizeof(double));
  double* acc = (double*)malloc((size_t)D * sizeof(double));
  for (int h = 0; h < nq; ++h) {
    const int kvh = h / group;
    const uint16_t* qh = J->q + ((int64_t)row * nq + h) * D;
    double ks = g->dtype == FSO_FP8 ? (double)J->k_scale[J->layer * H + kvh] : 1.0;
    double vs = g->dtype == FSO_FP8 ? (double)J->v_scale[J->layer * H + kvh] : 1.0;
    double m = -INFINITY;
    for (int t = 0; t < n; ++t) {
      load_row(J->pool_mem, g, table[t / T], J->layer, kvh, 0, t % T, ks, kv);
      double dot = 0.0;
      for (int d = 0; d < D; ++d) dot += (double)fso_f16_to_f32(qh[d]) * kv[d];
      s[t] = J->sm_scale * dot;
      if (s[t] > m) m = s[t];
    }
    double l = 0.0;
    for (int d = 0; d < D; ++d) acc[d] = 0.0;
    for (int t = 0; t < n; ++t) {
      double p = exp(s[t] - m);
      l += p;
      load_row(J->pool_mem, g, table[t / T], J->layer, kvh, 1, t % T, vs, kv);
      for (int d = 0; d < D; ++d) acc[d] += p * kv[d];
    }
    double* o = J->out + ((int64_t)row * nq + h) * D;
    for (int d = 0; d < D; ++d) o[d] = acc[d] / l;
    if (J->lse) J->lse[(int64_t)row * nq + h] = m + log(l);
  }
  free(kv);
  free(s);
  free(acc);
}

static void* prefill_worker(void* arg) {
  const prefill_job* J = (const prefill_job*)arg;
  const int n_rows = J->q_offsets[J->n_seq];
  int b = 0;
  for (int row = 0; row < n_rows; ++row) {
    while (row >= J->q_offsets[b + 1]) ++b;
    if (row % J->stride == J->first) prefill_row(J, b, row);
  }
  return NULL;
}

int fso_prefill_attention(const uint8_t* pool_mem, const fso_geom* g, int layer, int n_q_heads, double sm_scale,
                          const uint16_t* q, const int32_t* block_tables, const int32_t* seq_lens,
                          const int32_t* q_offsets, int n_seq, int max_blocks, const float* k_scale,
                          const float* v_scale, double* out, double* lse, int n_threads) {
  if (layer < 0 || layer >= g->n_layers || n_q_heads < g->n_kv_heads || n_q_heads % g->n_kv_heads)
    return FSO_ERR_INVALID;
  if (g->dtype == FSO_FP8 && (!k_scale || !v_scale)) return FSO_ERR_INVALID;
  if (n_seq < 1 || q_offsets[0] != 0) return FSO_ERR_INVALID;
  for (int b = 0; b < n_seq; ++b) {
    const int n_new = q_offsets[b + 1] - q_offsets[b];
    if (n_new < 0 || seq_lens[b] < 1 || n_new > seq_lens[b] ||
        (seq_lens[b] + g->tokens_per_block - 1) / g->tokens_per_block > max_blocks)
      return FSO_ERR_INVALID;
  }
  if (n_threads < 1) n_threads = 1;
  if (n_threads > 256) n_threads = 256;
  prefill_job jobs[256];
  pthread_t th[256];
  for (int i = 0; i < n_threads; ++i) {
    prefill_job J = {pool_mem, g, layer, n_q_heads, sm_scale, q, block_tables, seq_lens, q_offsets, n_seq,
                     max_blocks, k_scale, v_scale, out, lse, i, n_threads};
    jobs[i] = J;
  }
  for (int i = 1; i < n_threads; ++i) pthread_create(&th[i], NULL, prefill_worker, &jobs[i]);
  prefill_worker(&jobs[0]);
  for (int i = 1; i < n_threads; ++i) pthread_join(th[i], NULL);
  return FSO_OK;
}
