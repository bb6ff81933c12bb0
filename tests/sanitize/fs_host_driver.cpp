// Host-side exerciser of libfineserve's C ABI for AddressSanitizer / UBSan builds (no GPU needed).
//
// Compiled together with the library's sources by tests/test_host_sanitizers.py with the host sanitizers on
// (device code is compiled as usual and never runs: the pool is created over a caller-supplied base address that is
// never dereferenced, so every device entry point stops after its host-side validation and planning).  It drives the
// slab allocator through long seeded traces with the error paths mixed in, the size helpers, the statistics and
// dump calls, the per-pool options, the decode planner (workspace sizing over many batch shapes) and the two
// scheduler calls, and checks return codes and a few invariants; the sanitizers check the memory accesses.
#include <cinttypes>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "fineserve.h"

namespace {

uint64_t g_state = 0x9E3779B97F4A7C15ull;
uint64_t rnd() {
  g_state ^= g_state >> 12;
  g_state ^= g_state << 25;
  g_state ^= g_state >> 27;
  return g_state * 0x2545F4914F6CDD1Dull;
}
int rnd_int(int n) { return (int)(rnd() % (uint64_t)n); }

int g_failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::printf("CHECK failed at line %d: %s\n", __LINE__, #cond);       \
      ++g_failures;                                                        \
    }                                                                      \
  } while (0)

void* const kFakeBase = (void*)0x10000000;

void allocator_traces() {
  const uint64_t slab = 64 << 10;
  for (int round = 0; round < 4; ++round) {
    fs_pool* p = nullptr;
    CHECK(fs_pool_create(slab, 256 * slab, kFakeBase, &p) == FS_OK);
    fs_model_t m[3];
    CHECK(fs_model_register(p, FS_KV_FP16, 2, 64, 1, &m[0]) > 0);
    CHECK(fs_model_register_ex(p, FS_KV_INT4, 2, 64, 2, slab / 4, &m[1]) > 0);
    CHECK(fs_model_register_ex(p, FS_KV_INT8, 1, 128, 1, slab / 2, &m[2]) > 0);
    std::vector<int32_t> held[3];
    for (int op = 0; op < 40000; ++op) {
      const int k = rnd_int(3);
      const int what = rnd_int(10);
      if (what < 5) {
        int32_t b = -1;
        const int rc = fs_block_alloc(p, m[k], &b);
        if (rc == FS_OK) held[k].push_back(b);
        else CHECK(rc == FS_ERR_NOMEM);
      } else if (what < 9 && !held[k].empty()) {
        const size_t i = (size_t)rnd_int((int)held[k].size());
        CHECK(fs_block_free(p, m[k], held[k][i]) == FS_OK);
        CHECK(fs_block_free(p, m[k], held[k][i]) == FS_ERR_STATE);  // double free
        held[k][i] = held[k].back();
        held[k].pop_back();
      } else {
        // foreign, negative and out-of-range block ids
        CHECK(fs_block_free(p, m[k], -1 - rnd_int(5)) != FS_OK);
        CHECK(fs_block_free(p, m[k], 1 << 28) != FS_OK);
        if (!held[(k + 1) % 3].empty()) {
          const int32_t other = held[(k + 1) % 3][0];
          const int rc = fs_block_free(p, m[k], other);  // another model's block (ids of different block sizes may coincide)
          if (rc == FS_OK) {  // it named a live block of model k as well: take it out of the books
            bool found = false;
            for (size_t i = 0; i < held[k].size() && !found; ++i)
              if (held[k][i] == other) {
                held[k][i] = held[k].back();
                held[k].pop_back();
                found = true;
              }
            CHECK(found);
          }
        }
      }
      if (op % 5000 == 0) {
        fs_pool_stats_t st;
        CHECK(fs_pool_stats(p, &st) == FS_OK);
        CHECK(st.live_blocks == (int64_t)(held[0].size() + held[1].size() + held[2].size()));
        CHECK(st.slabs_free + st.slabs_partial + st.slabs_full == st.n_slabs);
        int64_t full = 0, partial = 0;
        for (int j = 0; j < 3; ++j) {
          fs_model_stats_t ms;
          CHECK(fs_model_stats(p, m[j], &ms) == FS_OK);
          CHECK(ms.live_blocks == (int64_t)held[j].size());
          full += ms.slabs_full;
          partial += ms.slabs_partial;
        }
        CHECK(full == st.slabs_full && partial == st.slabs_partial);
        std::vector<int32_t> a(256), b(256), c(256), d(256);
        int64_t nf = -1;
        CHECK(fs_pool_dump(p, a.data(), b.data(), c.data(), d.data(), &nf) == FS_OK);
        CHECK(nf == st.slabs_free);
        fs_geometry_t g;
        CHECK(fs_model_geometry(p, m[1], &g) == FS_OK);
        std::vector<uint8_t> live((size_t)256 * (size_t)g.blocks_per_slab);
        CHECK(fs_model_dump_live(p, m[1], live.data()) == FS_OK);
        int64_t n_live = 0;
        for (uint8_t x : live) n_live += x;
        CHECK(n_live == (int64_t)held[1].size());
      }
    }
    CHECK(fs_model_unregister(p, m[0]) == (held[0].empty() ? FS_OK : FS_ERR_STATE));
    for (int k = 0; k < 3; ++k)
      for (int32_t b : held[k]) CHECK(fs_block_free(p, m[k], b) == FS_OK);
    // the batched calls: a whole sequence's blocks at once, more than the pool holds, none, bad arguments
    {
      std::vector<int32_t> ids(33);
      CHECK(fs_blocks_alloc(p, m[1], 33, ids.data()) == FS_OK);
      CHECK(fs_blocks_alloc(p, m[1], 1 << 30, ids.data()) == FS_ERR_NOMEM);
      CHECK(fs_blocks_alloc(p, m[1], 0, nullptr) == FS_OK);
      CHECK(fs_blocks_alloc(p, m[1], -3, ids.data()) == FS_ERR_INVALID);
      CHECK(fs_blocks_alloc(p, m[1], 2, nullptr) == FS_ERR_INVALID);
      CHECK(fs_blocks_free(p, m[1], ids.data(), 33) == FS_OK);
      CHECK(fs_blocks_free(p, m[1], ids.data(), 1) == FS_ERR_STATE);
      CHECK(fs_blocks_free(p, m[1], nullptr, 0) == FS_OK);
    }
    fs_pool_stats_t st;
    CHECK(fs_pool_stats(p, &st) == FS_OK);
    CHECK(st.slabs_free == st.n_slabs && st.live_blocks == 0);
    CHECK(fs_model_unregister(p, m[1]) == FS_OK);
    CHECK(fs_model_unregister(p, m[1]) != FS_OK);
    CHECK(fs_pool_destroy(p) == FS_OK);
  }
}

void sizes_and_registration() {
  for (int dt = 0; dt < 4; ++dt)
    for (int i = 0; i < 200; ++i) {
      const int H = 1 + rnd_int(40), D = 8 << rnd_int(7), L = 1 + rnd_int(48), T = 1 + rnd_int(200);
      const uint64_t bb = fs_block_bytes(dt, H, D, L, T);
      CHECK(bb > 0 && bb % 256 == 0);
      const uint64_t list[2] = {bb, fs_block_bytes(dt, H, D, L, 2 * T)};
      const uint64_t sl = fs_slab_bytes_for_blocks(list, 2, 1 << 20);
      CHECK(sl == 0 || (sl % list[0] == 0 && sl % list[1] == 0 && sl >= (1u << 20)));
    }
  CHECK(fs_block_bytes(0, 8, 100, 1, 1) == 0);  // head_dim not a power of two
  CHECK(fs_block_bytes(9, 8, 128, 1, 1) == 0);
  CHECK(fs_slab_bytes_for_blocks(nullptr, 0, 0) == 0);
  fs_pool* p = nullptr;
  CHECK(fs_pool_create(100, 1000, kFakeBase, &p) != FS_OK);
  CHECK(fs_pool_create(2 << 20, (uint64_t)64 << 20, kFakeBase, &p) == FS_OK);
  fs_model_t m;
  CHECK(fs_model_register(p, 7, 8, 128, 32, &m) < 0);
  CHECK(fs_model_register(p, FS_KV_FP16, 8, 96, 32, &m) < 0);
  CHECK(fs_model_register_ex(p, FS_KV_FP16, 8, 128, 32, 3 << 19, &m) < 0);  // budget does not divide the slab
  CHECK(fs_model_register(p, FS_KV_FP16, 1024, 512, 4096, &m) < 0);         // not a single token fits
  for (int i = 0; i < 64; ++i) CHECK(fs_model_register(p, i & 3, 8, 128, 8, &m) > 0);
  CHECK(fs_model_register(p, FS_KV_FP16, 8, 128, 8, &m) < 0);  // the model table is full
  CHECK(fs_pool_destroy(p) == FS_OK);
}

void options_and_planner() {
  fs_pool* p = nullptr;
  CHECK(fs_pool_create(2 << 20, (uint64_t)1 << 30, kFakeBase, &p) == FS_OK);
  int64_t v = -1;
  for (int opt = -2; opt < 12; ++opt)
    for (int64_t val : {(int64_t)-5, (int64_t)0, (int64_t)1, (int64_t)2, (int64_t)4, (int64_t)8, (int64_t)16, (int64_t)65536,
                        (int64_t)1 << 40}) {
      if (opt == FS_OPT_KERNEL_TIMING && val != 0) continue;  // would create HIP events: there is no device here
      const int rc = fs_pool_set_option(p, opt, val);
      CHECK(rc == FS_OK || rc == FS_ERR_INVALID);
      (void)fs_pool_get_option(p, opt, &v);
    }
  CHECK(fs_pool_set_option(p, FS_OPT_SPLIT_BYTES, 0) == FS_OK && fs_pool_set_option(p, FS_OPT_DECODE_KERNEL, 0) == FS_OK);
  CHECK(fs_pool_last_attention_kernel_ms(p) < 0.f);
  fs_model_t m[4];
  CHECK(fs_model_register(p, FS_KV_FP16, 8, 128, 8, &m[0]) > 0);
  CHECK(fs_model_register(p, FS_KV_INT4, 40, 128, 10, &m[1]) > 0);
  CHECK(fs_model_register(p, FS_KV_INT8, 4, 64, 1, &m[2]) > 0);
  CHECK(fs_model_register(p, FS_KV_FP8_E4M3, 8, 128, 8, &m[3]) > 0);
  // planner: many batch shapes, with and without host lengths; nothing is launched (no device): FS_ERR_DEVICE at most
  alignas(16) static char dummy[64];
  for (int it = 0; it < 300; ++it) {
    fs_batch_t b[8];
    const int nb = 1 + rnd_int(8);
    std::vector<std::vector<int32_t>> lens(nb);
    for (int i = 0; i < nb; ++i) {
      const int k = rnd_int(3);  // (the FP8 model has no scales: that error path is taken separately)
      b[i] = fs_batch_t{};
      b[i].model = m[k];
      b[i].layer = 0;
      const int heads[3] = {8, 40, 4};
      b[i].n_q_heads = heads[k] * (1 + rnd_int(4));
      b[i].sm_scale = 0.1f;
      b[i].q = dummy;
      b[i].out = dummy;
      b[i].block_tables = (const int32_t*)dummy;
      b[i].seq_lens = (const int32_t*)dummy;
      b[i].n_seq = 1 + rnd_int(300);
      b[i].max_blocks = 1 + rnd_int(900);
      if (rnd_int(2)) {
        lens[i].resize((size_t)b[i].n_seq);
        for (auto& l : lens[i]) l = rnd_int(70000) - 100;  // includes lengths out of range (clamped by the planner)
        b[i].seq_lens_host = lens[i].data();
      }
    }
    if (it % 3 == 0) CHECK(fs_pool_set_option(p, FS_OPT_SPLIT_BYTES, 4096 << rnd_int(10)) == FS_OK);
    const uint64_t need = fs_decode_workspace_bytes(p, b, nb);
    CHECK(need > 0 && need % 256 == 0);
    const int rc = fs_decode_attention_multi(p, b, nb, (void*)0x20000000, need, nullptr);
    CHECK(rc == FS_ERR_DEVICE);
    CHECK(fs_decode_attention_multi(p, b, nb, (void*)0x20000000, need - 256, nullptr) == FS_ERR_NOMEM);
    CHECK(fs_decode_attention_multi_static(p, b, nb, nullptr, nullptr) != FS_OK);  // no device: refused
  }
  fs_batch_t bad{};
  bad.model = m[3];
  bad.n_q_heads = 32;
  bad.q = bad.out = dummy;
  bad.block_tables = bad.seq_lens = (const int32_t*)dummy;
  bad.n_seq = 4;
  bad.max_blocks = 4;
  CHECK(fs_decode_workspace_bytes(p, &bad, 1) == 0);  // FP8 model without scales
  CHECK(fs_decode_workspace_bytes(p, &bad, 0) == 0 && fs_decode_workspace_bytes(p, &bad, 9) == 0);
  CHECK(fs_kv_append(p, m[0], 0, dummy, dummy, FS_SRC_FP16, (const int32_t*)dummy, (const int32_t*)dummy,
                     (const int32_t*)dummy, 4, 16, nullptr) == FS_ERR_DEVICE);
  CHECK(fs_kv_append(p, m[0], 9, dummy, dummy, FS_SRC_FP16, (const int32_t*)dummy, (const int32_t*)dummy,
                     (const int32_t*)dummy, 4, 16, nullptr) == FS_ERR_INVALID);
  CHECK(fs_kv_append(p, 63, 0, dummy, dummy, FS_SRC_FP16, (const int32_t*)dummy, (const int32_t*)dummy,
                     (const int32_t*)dummy, 4, 16, nullptr) == FS_ERR_INVALID);
  CHECK(fs_last_error() != nullptr);
  CHECK(fs_pool_destroy(p) == FS_OK);
}

void scheduler_calls() {
  for (int it = 0; it < 2000; ++it) {
    const int n = rnd_int(40);
    std::vector<fs_request_t> w((size_t)n);
    for (auto& r : w) {
      r.arrival_time = (double)rnd_int(1000) / 100.0;
      r.prompt_tokens = 1 + rnd_int(8000);
      r.reserved = 0;
    }
    fs_sched_params_t par{0.5 + rnd_int(100) / 50.0, 1e-3, 2e-5, 1e-9, 1 + rnd_int(64), 1 + rnd_int(100000)};
    std::vector<int32_t> sel((size_t)n + 1), drp((size_t)n + 1);
    int32_t ns = -1, nd = -1;
    CHECK(fs_sched_select_batch(w.data(), n, &par, 5.0 + rnd_int(500) / 100.0, sel.data(), &ns, drp.data(), &nd) == FS_OK);
    CHECK(ns >= 0 && nd >= 0 && ns + nd <= n && ns <= par.n_max);
    int64_t tok = 0;
    for (int i = 0; i < ns; ++i) {
      CHECK(sel[(size_t)i] >= 0 && sel[(size_t)i] < n);
      tok += w[(size_t)sel[(size_t)i]].prompt_tokens;
    }
    CHECK(tok <= par.t_max);
    const int ng = 1 + rnd_int(6), nm = rnd_int(12);
    std::vector<double> f((size_t)nm), mu((size_t)nm), cap((size_t)ng);
    for (auto& x : f) x = 1.0 + rnd_int(70);
    for (auto& x : mu) x = 0.1 + rnd_int(100) / 10.0;
    for (auto& x : cap) x = 40.0 + rnd_int(100);
    std::vector<int32_t> place((size_t)nm + 1, -7);
    CHECK(fs_sched_place_models(f.data(), mu.data(), nm, cap.data(), ng, place.data()) == FS_OK);
    std::vector<double> used((size_t)ng, 0.0);
    for (int i = 0; i < nm; ++i) {
      CHECK(place[(size_t)i] >= -1 && place[(size_t)i] < ng);
      if (place[(size_t)i] >= 0) used[(size_t)place[(size_t)i]] += f[(size_t)i];
    }
    for (int g = 0; g < ng; ++g) CHECK(used[(size_t)g] <= cap[(size_t)g] + 1e-9);
  }
  CHECK(fs_sched_select_batch(nullptr, 3, nullptr, 0.0, nullptr, nullptr, nullptr, nullptr) == FS_ERR_INVALID);
}

}  // namespace

int main() {
  allocator_traces();
  sizes_and_registration();
  options_and_planner();
  scheduler_calls();
  std::printf("fs_host_driver: %d failed checks\n", g_failures);
  return g_failures ? 1 : 0;
}
