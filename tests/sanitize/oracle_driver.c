/* Exerciser of the CPU oracle (oracle/fs_oracle.c) for AddressSanitizer / UBSan builds.
 *
 * Built by tests/test_host_sanitizers.py with gcc -fsanitize=address,undefined.  The oracle's source is included as
 * is (one translation unit, nothing of it is changed); the driver runs every entry point on small seeded inputs --
 * geometry search, allocator traces with the error paths, both source types through the four quantizers, decode and
 * prefill attention over shuffled block tables on several threads -- and checks return codes and that the results
 * are finite; the sanitizers check the memory accesses and the arithmetic. */
#include <stdio.h>

#include "../../oracle/fs_oracle.c"

static uint64_t g_state = 0x2545F4914F6CDD1DULL;
static uint64_t rnd(void) {
  g_state ^= g_state >> 12;
  g_state ^= g_state << 25;
  g_state ^= g_state >> 27;
  return g_state * 0x2545F4914F6CDD1DULL;
}
static int rnd_int(int n) { return (int)(rnd() % (uint64_t)n); }
static float rnd_normalish(void) { return ((float)rnd_int(20001) - 10000.0f) / 2500.0f; }

static int g_failures = 0;
#define CHECK(cond)                                                    \
  do {                                                                 \
    if (!(cond)) {                                                     \
      printf("CHECK failed at line %d: %s\n", __LINE__, #cond);        \
      ++g_failures;                                                    \
    }                                                                  \
  } while (0)

static void allocator_trace(void) {
  const uint64_t slab = 64 << 10;
  fso_pool* p = fso_pool_new(slab, 128 * slab);
  CHECK(p != NULL);
  int m0 = fso_model_add(p, FSO_FP16, 2, 64, 1, slab);
  int m1 = fso_model_add(p, FSO_INT4, 2, 64, 2, slab / 4);
  int m2 = fso_model_add_tokens(p, FSO_FP8, 2, 64, 1, 16);
  CHECK(m0 >= 0 && m1 >= 0);
  (void)m2;
  int32_t held[2][600];
  int n_held[2] = {0, 0};
  const int mm[2] = {m0, m1};
  for (int op = 0; op < 30000; ++op) {
    const int k = rnd_int(2);
    if (rnd_int(2) && n_held[k] < 600) {
      int32_t b = -1;
      const int rc = fso_block_alloc(p, mm[k], &b);
      if (rc == FSO_OK) held[k][n_held[k]++] = b;
      else CHECK(rc == FSO_ERR_NOMEM);
    } else if (n_held[k]) {
      const int i = rnd_int(n_held[k]);
      CHECK(fso_block_free(p, mm[k], held[k][i]) == FSO_OK);
      CHECK(fso_block_free(p, mm[k], held[k][i]) == FSO_ERR_STATE);
      held[k][i] = held[k][--n_held[k]];
    } else {
      CHECK(fso_block_free(p, mm[k], -3) != FSO_OK);
      CHECK(fso_block_free(p, mm[k], 1 << 28) != FSO_OK);
    }
  }
  int32_t st[128], key[128], used[128], fstack[128];
  fso_pool_dump(p, st, key, used, fstack);
  uint8_t live[128 * 4];
  fso_model_dump_live(p, m1, live);
  int n_live = 0;
  for (int i = 0; i < 128 * 4; ++i) n_live += live[i];
  CHECK(n_live == n_held[1] && fso_model_live_blocks(p, m1) == n_held[1]);
  CHECK(fso_model_remove(p, m0) == (n_held[0] ? FSO_ERR_STATE : FSO_OK));
  fso_pool_delete(p);
}

static void formats_and_attention(int dtype, int src_is_f32, int H, int D, int n_q, int L) {
  const uint64_t slab = 32 << 10;
  const int n_blocks = 64;
  fso_geom g;
  CHECK(fso_geometry(dtype, H, D, L, slab, &g) == FSO_OK);
  const int T = g.tokens_per_block;
  CHECK(T >= 1 && g.block_bytes <= slab);
  uint8_t* mem = (uint8_t*)malloc((size_t)n_blocks * slab);
  memset(mem, 0xA5, (size_t)n_blocks * slab);
  enum { NSEQ = 5 };
  const int lens[NSEQ] = {1, T, T + 1, 3 * T - 1, 5 * T + 2};
  int max_blocks = 6, next = 0;
  int32_t perm[64];
  for (int i = 0; i < n_blocks; ++i) perm[i] = i;
  for (int i = n_blocks - 1; i > 0; --i) {
    const int j = rnd_int(i + 1);
    const int32_t t = perm[i];
    perm[i] = perm[j];
    perm[j] = t;
  }
  int32_t tables[NSEQ * 6];
  int total = 0;
  for (int s = 0; s < NSEQ; ++s) {
    for (int b = 0; b < max_blocks; ++b) tables[s * max_blocks + b] = b < (lens[s] + T - 1) / T ? perm[next++] : -1;
    total += lens[s];
  }
  CHECK(next <= n_blocks);
  const size_t row = (size_t)H * D;
  void* k = malloc((size_t)total * row * (src_is_f32 ? 4 : 2));
  void* v = malloc((size_t)total * row * (src_is_f32 ? 4 : 2));
  int32_t* seq_idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)total);
  int32_t* pos = (int32_t*)malloc(sizeof(int32_t) * (size_t)total);
  int t = 0;
  for (int s = 0; s < NSEQ; ++s)
    for (int i = 0; i < lens[s]; ++i, ++t) {
      seq_idx[t] = s;
      pos[t] = i;
    }
  for (size_t i = 0; i < (size_t)total * row; ++i) {
    const float a = rnd_normalish(), b = rnd_normalish();
    if (src_is_f32) {
      ((float*)k)[i] = a;
      ((float*)v)[i] = b;
    } else {
      ((uint16_t*)k)[i] = fso_f32_to_f16(a);
      ((uint16_t*)v)[i] = fso_f32_to_f16(b);
    }
  }
  float* ks = (float*)malloc(sizeof(float) * (size_t)L * H);
  float* vs = (float*)malloc(sizeof(float) * (size_t)L * H);
  for (int i = 0; i < L * H; ++i) {
    ks[i] = 0.01f + (float)i * 0.001f;
    vs[i] = 0.02f;
  }
  const int layer = L - 1;
  CHECK(fso_kv_append(mem, &g, layer, k, v, src_is_f32, seq_idx, pos, tables, max_blocks, total, ks, vs) == FSO_OK);
  CHECK(fso_kv_append(mem, &g, L, k, v, src_is_f32, seq_idx, pos, tables, max_blocks, total, ks, vs) == FSO_ERR_INVALID);
  uint16_t* q = (uint16_t*)malloc(sizeof(uint16_t) * (size_t)total * n_q * D);
  for (size_t i = 0; i < (size_t)total * n_q * D; ++i) q[i] = fso_f32_to_f16(rnd_normalish());
  double* out = (double*)malloc(sizeof(double) * (size_t)total * n_q * D);
  double* lse = (double*)malloc(sizeof(double) * (size_t)total * n_q);
  CHECK(fso_decode_attention(mem, &g, layer, n_q, 0.125, q, tables, lens, NSEQ, max_blocks, ks, vs, out, lse, 3) == FSO_OK);
  for (size_t i = 0; i < (size_t)NSEQ * n_q * D; ++i) CHECK(isfinite(out[i]));
  for (size_t i = 0; i < (size_t)NSEQ * n_q; ++i) CHECK(isfinite(lse[i]));
  CHECK(fso_decode_attention(mem, &g, layer, n_q, 0.125, q, tables, lens, NSEQ, max_blocks, ks, vs, out, NULL, 1) == FSO_OK);
  /* whole prompts as prefill chunks, then short trailing chunks (one of them empty) */
  int32_t q_off[NSEQ + 1] = {0};
  for (int s = 0; s < NSEQ; ++s) q_off[s + 1] = q_off[s] + lens[s];
  CHECK(fso_prefill_attention(mem, &g, layer, n_q, 0.125, q, tables, lens, q_off, NSEQ, max_blocks, ks, vs, out, lse, 4) ==
        FSO_OK);
  for (size_t i = 0; i < (size_t)total * n_q * D; ++i) CHECK(isfinite(out[i]));
  for (int s = 0; s < NSEQ; ++s) q_off[s + 1] = q_off[s] + (s == 2 ? 0 : (lens[s] < 3 ? lens[s] : 3));
  CHECK(fso_prefill_attention(mem, &g, layer, n_q, 0.125, q, tables, lens, q_off, NSEQ, max_blocks, ks, vs, out, NULL, 2) ==
        FSO_OK);
  double* kd = (double*)malloc(sizeof(double) * (size_t)lens[4] * row);
  double* vd = (double*)malloc(sizeof(double) * (size_t)lens[4] * row);
  CHECK(fso_dequant_sequence(mem, &g, layer, tables + 4 * max_blocks, lens[4], ks, vs, kd, vd) == FSO_OK);
  for (size_t i = 0; i < (size_t)lens[4] * row; ++i) CHECK(isfinite(kd[i]) && isfinite(vd[i]));
  /* addressing helpers stay inside the block */
  CHECK(fso_row_offset(&g, 3, layer, H - 1, 1, T - 1) + g.row_bytes <= 4 * slab);
  if (g.param_bytes) CHECK(fso_param_offset(&g, 3, layer, H - 1, 1, T - 1) + (uint64_t)g.param_bytes <= 3 * slab + g.block_bytes);
  free(kd); free(vd); free(out); free(lse); free(q); free(ks); free(vs); free(seq_idx); free(pos); free(k); free(v); free(mem);
}

int main(void) {
  allocator_trace();
  for (int dtype = 0; dtype < 4; ++dtype)
    for (int f32 = 0; f32 < 2; ++f32) {
      formats_and_attention(dtype, f32, 2, 64, 4, 2);
      formats_and_attention(dtype, f32, 1, 128, 3, 1);
      formats_and_attention(dtype, f32, 3, 8, 3, 3);
    }
  uint64_t bb[3] = {fso_block_bytes(FSO_FP16, 8, 128, 32, 16), fso_block_bytes(FSO_FP8, 8, 128, 32, 16), 0};
  CHECK(bb[0] == 2u << 20 && bb[1] == 1u << 20);
  CHECK(fso_lcm_slab_bytes(bb, 2, 1) == 2u << 20);
  CHECK(fso_lcm_slab_bytes(bb, 3, 1) == 0);
  printf("oracle_driver: %d failed checks\n", g_failures);
  return g_failures ? 1 : 0;
}
