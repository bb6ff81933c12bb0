// Host-compiled replay of the MFMA decode kernel's index arithmetic, every index asserted (no GPU needed).
//
// Compiled together with the library's sources by tests/test_host_sanitizers.py (host sanitizers on).  For seeded
// pools, models and batches it asks the library for the device-side records of a decode call (fs::debug_plan: what
// the launch would hand its kernels) and then walks every work item the work-list kernel would queue -- sequence,
// split, KV head -- with the very functions the kernels use (n_splits, item_range, run_geom, ring_tiles): for every
// tile of the item's ring turns, refills past the item's end included, and every lane of the wave it computes the
// addresses the K, V and parameter loads would form and checks that
//   * the block index stays inside the item's address table (0 <= k_rel < nb <= 256 entries),
//   * every K row, V row and parameter word lies inside its tile of the block's head chunk,
//   * the runs of a sequence's items cover every token exactly once with the slots [lo, hi) the softmax keeps,
//     and no kept slot lies at or past the sequence's length,
//   * the items of a sequence tile its runs without gap or overlap, and their number is what n_splits says.
// The prefill kernels' queue arithmetic (fs_prefill_index.h) is replayed the same way: every item of a queue belongs
// to exactly one (pool, ticket) and a pool's items grow with the ticket (what lets a wave call a pool empty at its
// first ticket past the end); item -> (sequence, KV head, query tile) is one-to-one onto the tiles the sequences
// have; and a table segment of a context never touches more blocks than the wave's address table holds.
// The decode work queue's closed-form placement (queue_place: the batches' item lists merged proportionally) is
// checked to be one-to-one onto the queue and order-preserving within a batch.
// The vector-ALU kernel's launch is replayed where the device's lengths are not the ones the host sized the workspace
// for: what is queued, every queued item's tokens and table entries, the partial records and the combine's rows stay
// inside the plan's capacities or are the ones the kernels skip and report.
#include <algorithm>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "fs_attention.h"
#include "fs_prefill_index.h"

namespace {

uint64_t g_state = 0xD1B54A32D192ED03ull;
uint64_t rnd() {
  g_state ^= g_state >> 12;
  g_state ^= g_state << 25;
  g_state ^= g_state >> 27;
  return g_state * 0x2545F4914F6CDD1Dull;
}
int rnd_int(int n) { return (int)(rnd() % (uint64_t)n); }

long g_failures = 0, g_items = 0, g_tiles = 0;
#define CHECK(cond)                                                                  \
  do {                                                                               \
    if (!(cond)) {                                                                   \
      if (g_failures < 20) std::printf("CHECK failed at line %d: %s\n", __LINE__, #cond); \
      ++g_failures;                                                                  \
    }                                                                                \
  } while (0)

void* const kFakeBase = (void*)0x10000000;

// Bytes per lane of the K and V loads of a tile, as the tile code derives them from the format and the head_dim.
struct LoadShape {
  int row_bytes, k_lane, k_loads, v_bytes, par_bytes;
};
LoadShape load_shape(int dtype, int D) {
  LoadShape s;
  const int bits = dtype == FS_KV_FP16 ? 16 : (dtype == FS_KV_INT4 ? 4 : 8);
  s.row_bytes = D * bits / 8;
  s.k_lane = s.row_bytes / 4 < 16 ? s.row_bytes / 4 : 16;
  s.k_loads = s.row_bytes / (4 * s.k_lane);
  s.v_bytes = s.row_bytes / 16;
  s.par_bytes = dtype == FS_KV_INT8 ? 2 : (dtype == FS_KV_INT4 ? 4 : 0);
  return s;
}

void check_batch(const fs::DevBatch& B, const std::vector<int32_t>& lens) {
  const fs::DevGeom& g = B.g;
  const LoadShape S = load_shape(g.dtype, g.D);
  CHECK((uint32_t)S.row_bytes == g.row_bytes);
  CHECK((uint64_t)g.T * g.row_bytes <= g.kv_tile);
  CHECK(2ull * g.kv_tile + 2ull * g.par_tile <= g.head_chunk);
  const int ring = fs::ring_tiles(g.dtype, g.D);
  std::vector<int> seen;
  for (int seq = 0; seq < B.n_seq; ++seq) {
    const int64_t max_len = (int64_t)B.max_blocks * g.T;
    const int len = (int)std::min<int64_t>(std::max(lens[seq], 1), max_len);
    const int n_items = fs::n_splits(B, seq, len);
    const int all_runs = fs::n_runs(len, g.T, B.R);
    seen.assign(len, 0);
    int next_run = 0;
    for (int chunk = 0; chunk < n_items; ++chunk) {
      ++g_items;
      const fs::ItemRange r = fs::item_range(B, seq, chunk, len);
      CHECK(r.v0 == next_run && r.v1 > r.v0 && r.v1 <= all_runs);
      next_run = r.v1;
      CHECK(r.nb >= 1 && r.nb <= 256);  // the kernel's address table: four registers of 64 lanes
      CHECK(r.k0 >= 0 && r.k0 + r.nb <= B.max_blocks);
      fs::ItemCtx X;
      X.chunk_ptr = nullptr;
      X.T = g.T;
      X.R = B.R;
      X.r_magic = B.r_magic;
      X.len = len;
      X.len_u = len;
      X.v_end = r.v1;
      X.k0 = r.k0;
      const int n_tiles = (r.v1 - r.v0 + 3) >> 2;
      const int turns = (n_tiles + ring - 1) / ring;
      // tiles consumed: at most turns * ring (the surplus ones of the last turn keep nothing); tiles requested: at
      // most one ring more (the last turn's refills, which the formats with a refill-free last turn leave out)
      for (int tile = 0; tile < (turns + 1) * ring; ++tile) {
        ++g_tiles;
        const int vb = r.v0 + 4 * tile;
        const bool consumed = tile < turns * ring;
        for (int lane = 0; lane < 64; ++lane) {
          const int j = lane >> 4, c = lane & 15;
          // K operand rows: run c / 4 of the tile, slots 4 u + c % 4
          const fs::RunGeom Lk = fs::run_geom(X, vb + (c >> 2));
          CHECK(Lk.k_rel >= 0 && Lk.k_rel < r.nb);
          CHECK(Lk.start >= 0 && Lk.start + 8 <= g.T);
          for (int u = 0; u < 2; ++u)
            for (int s = 0; s < S.k_loads; ++s) {
              const int64_t off = (int64_t)(Lk.start + (c & 3) + 4 * u) * S.row_bytes + S.k_lane * j + 4 * S.k_lane * s;
              CHECK(off >= 0 && off + S.k_lane <= (int64_t)g.T * S.row_bytes);
            }
          // V rows and parameters: run j of the tile
          const fs::RunGeom Lv = fs::run_geom(X, vb + j);
          CHECK(Lv.k_rel >= 0 && Lv.k_rel < r.nb);
          for (int i = 0; i < 8; ++i) {
            const int64_t off = (int64_t)(Lv.start + i) * S.row_bytes + c * S.v_bytes;
            CHECK(off >= 0 && off + S.v_bytes <= (int64_t)g.T * S.row_bytes);
          }
          if (S.par_bytes) {
            const int64_t off16 = (int64_t)(Lv.start + (c & 7)) * S.par_bytes;           // one column per lane
            const int64_t off4 = (int64_t)(Lv.start + 2 * (c >> 2) + 1) * S.par_bytes;   // four lanes per column
            CHECK(off16 + S.par_bytes <= (int64_t)g.par_tile && off4 + S.par_bytes <= (int64_t)g.par_tile);
          }
          // what the softmax keeps of run j: counted once per run (by the lane c == 0 of its lane group)
          if (consumed && c == 0) {
            CHECK(Lv.lo >= 0 && Lv.lo <= 8 && Lv.hi <= 8);
            for (int i = std::max(Lv.lo, 0); i < Lv.hi; ++i) {
              const int tok = Lv.tok0 + i;
              CHECK(tok >= 0 && tok < len);
              if (tok >= 0 && tok < len) ++seen[tok];
            }
            if (vb + j >= r.v1) CHECK(Lv.hi <= Lv.lo || Lv.hi <= 0);  // a run past the item's end keeps nothing
          }
        }
      }
    }
    CHECK(next_run == all_runs);
    for (int t = 0; t < len; ++t) CHECK(seen[t] == 1);
  }
}

void run(int rounds) {
  const int dtypes[4] = {FS_KV_FP16, FS_KV_FP8_E4M3, FS_KV_INT8, FS_KV_INT4};
  const int dims[3] = {64, 128, 256};
  const int want_T[12] = {8, 9, 13, 16, 23, 38, 60, 64, 126, 128, 200, 333};
  for (int round = 0; round < rounds; ++round) {
    const int dtype = dtypes[round % 4], D = dims[(round / 4) % 3];
    const int H = 1 + rnd_int(3), L = 1 + rnd_int(2);
    const int bits = dtype == FS_KV_FP16 ? 16 : (dtype == FS_KV_INT4 ? 4 : 8);
    const int par = dtype == FS_KV_INT8 ? 2 : (dtype == FS_KV_INT4 ? 4 : 0);
    const uint64_t tok_bytes = 2ull * H * L * (uint64_t)(D * bits / 8 + par);
    const uint64_t slab = std::max<uint64_t>(4096, (want_T[rnd_int(12)] * tok_bytes + 255) / 256 * 256 + 256 * (uint64_t)rnd_int(3));
    fs_pool* p = nullptr;
    CHECK(fs_pool_create(slab, 4096 * slab, kFakeBase, &p) == FS_OK);
    if (!p) continue;
    fs_model_t m;
    const int T = fs_model_register(p, dtype, H, D, L, &m);
    CHECK(T > 0);
    if (T < 8) {  // the vector-ALU kernel's shape
      fs_pool_destroy(p);
      continue;
    }
    const int n_seq = 1 + rnd_int(6);
    std::vector<int32_t> lens(n_seq);
    const int special[12] = {1, 2, 7, 8, 9, T - 1, T, T + 1, 2 * T, 4 * T + 3, 31, 33};
    int max_len = 1;
    for (int i = 0; i < n_seq; ++i) {
      lens[i] = rnd_int(3) ? std::max(1, special[rnd_int(12)]) : 1 + rnd_int(6000);
      max_len = std::max(max_len, (int)lens[i]);
    }
    const int G[8] = {1, 2, 3, 4, 5, 8, 12, 16};
    fs_batch_t b{};
    b.model = m;
    b.layer = rnd_int(L);
    b.n_q_heads = H * G[rnd_int(8)];
    b.sm_scale = 0.1f;
    b.q = (const void*)0x20000000;
    b.block_tables = (const int32_t*)0x30000000;
    b.seq_lens = (const int32_t*)0x40000000;
    b.seq_lens_host = rnd_int(4) ? lens.data() : nullptr;
    b.n_seq = n_seq;
    b.max_blocks = (max_len + T - 1) / T + rnd_int(2);
    b.out = (void*)0x50000000;
    const int64_t split[5] = {0, 0, 8 << 10, 24 << 10, 100 << 10};
    CHECK(fs_pool_set_option(p, FS_OPT_SPLIT_BYTES, split[rnd_int(5)]) == FS_OK);
    fs::MultiArgs A{};
    bool use_mfma = false;
    CHECK(fs::debug_plan(p, &b, 1, &A, &use_mfma) == FS_OK);
    CHECK(use_mfma);
    if (use_mfma) check_batch(A.b[0], lens);
    fs_pool_destroy(p);
  }
}

void prefill_queues(int rounds) {
  for (int round = 0; round < rounds; ++round) {
    const int n_seq = 1 + rnd_int(round % 7 == 0 ? 3000 : 40);
    const uint32_t H = 1 + (uint32_t)rnd_int(40);
    std::vector<uint32_t> tf(n_seq + 1, 0);
    for (int i = 0; i < n_seq; ++i) tf[i + 1] = tf[i] + (rnd_int(5) ? 1 + (uint32_t)rnd_int(rnd_int(4) ? 6 : 200) : 0u);
    const uint32_t total = tf[n_seq] * H;
    if (total == 0 || total > 3000000) continue;
    // item -> (sequence, head, tile)
    std::vector<uint8_t> hit(total, 0);
    for (uint32_t item = 0; item < total; ++item) {
      int seq = -1, head = -1, qt = -1;
      const bool ok = fs::decode_item(tf.data(), n_seq, item, H, seq, head, qt);
      CHECK(ok);
      if (!ok) continue;
      CHECK(seq >= 0 && seq < n_seq && head >= 0 && (uint32_t)head < H);
      const uint32_t nt = tf[seq + 1] - tf[seq];
      CHECK(qt >= 0 && (uint32_t)qt < nt);
      const uint64_t back = (uint64_t)tf[seq] * H + (uint64_t)head * nt + (nt - 1 - (uint32_t)qt);
      CHECK(back == item);
      ++g_items;
    }
    // (pool, ticket) -> item
    for (uint32_t shift = 5; shift <= 7; ++shift) {
      std::fill(hit.begin(), hit.end(), 0);
      for (uint32_t pool = 0; pool < 64; ++pool) {
        uint32_t prev = 0;
        for (uint32_t ticket = 0;; ++ticket) {
          const uint32_t item = fs::pool_item(pool, ticket, shift);
          CHECK(ticket == 0 || item > prev);
          prev = item;
          if (item >= total) break;
          CHECK(hit[item] == 0);
          hit[item] = 1;
        }
      }
      for (uint32_t item = 0; item < total; ++item) CHECK(hit[item] == 1);
    }
  }
  // table segments: tokens per block 8 .. 340, contexts up to 40000 tokens
  for (int T = 8; T <= 340; ++T) {
    const int R = (T + 7) / 8;
    const uint32_t r_magic = R == 1 ? 0u : (uint32_t)(((1ull << 32) + (uint64_t)R - 1) / (uint64_t)R);
    const int seg = fs::prefill_seg_runs(R), entries = fs::prefill_table_entries(seg, R);
    CHECK(seg >= 4 && seg % 4 == 0 && entries <= 1024 / 1 + 4);
    const int lens[6] = {1, T, T + 1, 1000, 8191, 40000};
    for (int li = 0; li < 6; ++li) {
      const int n_run = fs::n_runs(lens[li], T, R);
      for (int v0 = 0; v0 < n_run; v0 += seg) {
        const int v_end = std::min(n_run, v0 + seg);
        const int k0 = fs::div_runs(v0, R, r_magic);
        const int nb = fs::div_runs(v_end - 1, R, r_magic) - k0 + 1;
        CHECK(k0 == v0 / R && nb >= 1 && nb <= entries);
        CHECK((int64_t)(k0 + nb - 1) * T < (int64_t)lens[li] + T);  // the last block touched holds a token of the context
      }
    }
  }
}

// The decode work queue: every item of every batch gets one place, the places are 0 .. total - 1, and each batch's
// items keep their order (so a sequence's size tiers stay in queue order).
void decode_queue_places(int rounds) {
  for (int round = 0; round < rounds; ++round) {
    uint32_t n[fs::kMaxBatches] = {0, 0, 0, 0, 0, 0, 0, 0};
    const int nb = 1 + rnd_int(fs::kMaxBatches);
    uint64_t total = 0;
    for (int b = 0; b < nb; ++b) {
      n[b] = rnd_int(6) == 0 ? 1u : 1u + (uint32_t)rnd_int(round % 5 == 0 ? 70000 : 3000);
      total += n[b];
    }
    std::vector<uint8_t> hit(total, 0);
    for (int b = 0; b < nb; ++b) {
      uint64_t prev = 0;
      for (uint32_t i = 0; i < n[b]; ++i) {
        const uint64_t at = fs::queue_place(i, b, n);
        CHECK(at < total);
        CHECK(i == 0 || at > prev);
        prev = at;
        if (at < total) {
          CHECK(hit[at] == 0);
          hit[at] = 1;
        }
        ++g_items;
      }
    }
    for (uint64_t at = 0; at < total; ++at) CHECK(hit[at] == 1);
  }
}


// The vector-ALU kernel's launch when the lengths on the device are not the ones the host sized the workspace for
// (longer, far out of range, zero): the work list, the kernel's item loop and the combine are replayed with the plan's
// own capacities -- what the work-list kernel would count, where every queued item's tokens, table entries and partial
// record lie, and which rows the combine reads.  Everything stays inside its buffer, or the item / row is one of
// those the kernels skip and report.
void token_split_overflow(int rounds) {
  const int dtypes[4] = {FS_KV_FP16, FS_KV_FP8_E4M3, FS_KV_INT8, FS_KV_INT4};
  const int dims[5] = {32, 64, 128, 256, 512};
  for (int round = 0; round < rounds; ++round) {
    const uint64_t slab = 64 << 10;
    fs_pool* p = nullptr;
    CHECK(fs_pool_create(slab, 2048 * slab, kFakeBase, &p) == FS_OK);
    if (!p) continue;
    const int nb = 1 + rnd_int(4);
    fs_batch_t b[4] = {};
    std::vector<int32_t> host[4], dev[4];
    bool ok = true;
    for (int k = 0; k < nb; ++k) {
      const int dtype = dtypes[rnd_int(4)], D = dims[rnd_int(5)], H = 1 + rnd_int(2);
      fs_model_t m;
      const int T = fs_model_register(p, dtype, H, D, 1 + rnd_int(2), &m);
      ok = ok && T > 0;
      if (!ok) break;
      const int n_seq = 1 + rnd_int(5);
      int max_len = 1;
      for (int i = 0; i < n_seq; ++i) {
        host[k].push_back(1 + rnd_int(rnd_int(3) ? 300 : 2000));
        max_len = std::max(max_len, (int)host[k].back());
      }
      dev[k] = host[k];
      if (round % 3)  // the device disagrees on some sequences
        for (int i = 0; i < n_seq; ++i)
          if (rnd_int(2)) dev[k][i] = rnd_int(4) == 0 ? 1000000 : (rnd_int(4) == 0 ? -rnd_int(2) : 1 + rnd_int(3 * max_len));
      const int G[5] = {1, 2, 4, 8, 16};
      b[k].model = m;
      b[k].layer = 0;
      b[k].n_q_heads = H * G[rnd_int(5)];
      b[k].sm_scale = 0.1f;
      b[k].q = (const void*)0x20000000;
      b[k].block_tables = (const int32_t*)0x30000000;
      b[k].seq_lens = (const int32_t*)0x40000000;
      b[k].seq_lens_host = rnd_int(3) ? host[k].data() : nullptr;
      b[k].n_seq = n_seq;
      b[k].max_blocks = (max_len + T - 1) / T + rnd_int(2);
      b[k].out = (void*)0x50000000;
    }
    if (ok) {
      CHECK(fs_pool_set_option(p, FS_OPT_DECODE_KERNEL, 1) == FS_OK);
      const int64_t split[3] = {0, 8 << 10, 24 << 10};
      CHECK(fs_pool_set_option(p, FS_OPT_SPLIT_BYTES, split[rnd_int(3)]) == FS_OK);
      fs::MultiArgs A{};
      bool use_mfma = true;
      CHECK(fs::debug_plan(p, b, nb, &A, &use_mfma) == FS_OK);
      CHECK(!use_mfma);
      // the work-list kernel: items per batch from the device's (clamped) lengths
      uint32_t count[fs::kMaxBatches] = {0, 0, 0, 0, 0, 0, 0, 0};
      std::vector<int> clen[4];
      for (int k = 0; k < nb; ++k) {
        const fs::DevBatch& B = A.b[k];
        CHECK(B.chunk_runs == 0);
        const int max_len = (int)std::min<int64_t>((int64_t)B.max_blocks * B.g.T, 0x7fffffff);
        for (int i = 0; i < B.n_seq; ++i) {
          const int l = dev[k][i] < 1 ? 1 : std::min((int)dev[k][i], max_len);
          clen[k].push_back(l);
          count[k] += (uint32_t)fs::n_splits(B, i, l) * (uint32_t)B.g.H;
        }
      }
      uint64_t total = 0, part_off[4] = {0, 0, 0, 0}, running = 0;
      for (int k = 0; k < nb; ++k) {
        part_off[k] = running;
        running += (uint64_t)count[k] * (uint64_t)A.b[k].part_stride;
        total += count[k];
      }
      const bool same = [&] { for (int k = 0; k < nb; ++k) if (!b[k].seq_lens_host || dev[k] != host[k]) return false; return true; }();
      // (the workspace is sized for the larger of the two kernels' split rules)
      if (same) CHECK(total <= A.item_capacity && running <= A.part_capacity);
      const uint64_t queued = std::min<uint64_t>(total, A.item_capacity);
      std::vector<uint8_t> hit(total, 0);
      for (int k = 0; k < nb; ++k) {
        const fs::DevBatch& B = A.b[k];
        uint64_t local = 0;
        for (int i = 0; i < B.n_seq; ++i) {
          const int len = clen[k][i], ct = fs::chunk_tokens_of(B, i), n_chunks = fs::n_splits(B, i, len);
          const uint64_t first_local = local;
          for (int chunk = 0; chunk < n_chunks; ++chunk)
            for (int head = 0; head < B.g.H; ++head, ++local) {
              ++g_items;
              const uint64_t at = fs::queue_place(local, k, count);
              CHECK(at < total && hit[at] == 0);
              if (at < total) hit[at] = 1;
              if (at >= queued) continue;  // not queued: the launch reports the overflow
              // the item as the vector-ALU kernel walks it
              const int t0 = chunk * ct, t1 = std::min(len, t0 + ct);
              CHECK(t0 < t1);
              CHECK((t1 - 1) / B.g.T < B.max_blocks);
              const uint64_t part_base = part_off[k] + local * (uint64_t)B.part_stride;
              if (same) CHECK(n_chunks == 1 || part_base + (uint64_t)B.part_stride <= A.part_capacity);
            }
          // the combine's rows of this sequence
          if (n_chunks > 1)
            for (int h = 0; h < B.n_q; ++h) {
              const int kvh = h / B.G, gq = h % B.G;
              const uint64_t base = part_off[k] + first_local * (uint64_t)B.part_stride;
              const uint64_t last = base + (uint64_t)((uint32_t)(n_chunks - 1) * B.g.H + kvh) * B.part_stride + (uint64_t)(gq + 1) * (B.g.D + 2);
              if (same) CHECK(last <= A.part_capacity);  // (otherwise: read only if it lies inside, the kernel's own test)
              CHECK(base <= last);
            }
        }
        CHECK(local == count[k]);
      }
      for (uint64_t at = 0; at < total; ++at) CHECK(hit[at] == 1);
    }
    fs_pool_destroy(p);
  }
}

}  // namespace

int main() {
  run(600);
  prefill_queues(60);
  decode_queue_places(200);
  token_split_overflow(400);
  std::printf("fs_index_check: %ld items, %ld tiles, %ld failed checks\n", g_items, g_tiles, g_failures);
  return g_failures ? 1 : 0;
}
