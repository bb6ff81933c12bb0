// Host side of FineServe's two-level scheduler (Sec. 6): the decisions that feed the attention path its batches.
//   fs_sched_select_batch -- Algorithm 2 (Sec. 6.3), SLO-aware adaptive batching of one model's waiting queue
//   fs_sched_place_models -- Algorithm 1 (Sec. 6.2), model-to-GPU placement by the averaged-mu score proxy
// No device work.  Both run in O(n log n) / O(models x GPUs); the decisions are defined by integer sums and one
// fixed fp64 expression, so that they can be compared with a plain re-statement of the algorithms bit for bit.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <queue>
#include <vector>

#include "fs_internal.h"

using namespace fs;

namespace {

// Predicted chunked-prefill latency of a request set from its two token sums (Sec. 6.3's TTFT(R); the
// three-coefficient form is this library's reading: launch cost, linear layers, attention).
inline double ttft(const fs_sched_params_t& m, int64_t s1, int64_t s2) { return m.c0 + m.c1 * (double)s1 + m.c2 * (double)s2; }

}  // namespace

int fs_sched_select_batch(const fs_request_t* waiting, int n_waiting, const fs_sched_params_t* params, double now,
                          int32_t* selected, int32_t* n_selected, int32_t* dropped, int32_t* n_dropped) {
  if (n_waiting < 0 || (n_waiting > 0 && !waiting) || !params || !selected || !n_selected || !dropped || !n_dropped ||
      !(params->slo == params->slo) || !(now == now) || params->n_max < 0 || params->t_max < 0) {
    set_error("fs_sched_select_batch: invalid argument");
    return FS_ERR_INVALID;
  }
  const fs_sched_params_t& M = *params;
  for (int i = 0; i < n_waiting; ++i)
    if (waiting[i].prompt_tokens < 0 || !(waiting[i].arrival_time == waiting[i].arrival_time)) {
      set_error("fs_sched_select_batch: a request has a negative length or a NaN arrival time");
      return FS_ERR_INVALID;
    }
  // Algorithm 2 (Sec. 6.3), first step: a request that misses its deadline even alone, served now, is dropped
  std::vector<int32_t> S;
  S.reserve(n_waiting);
  int nd = 0;
  for (int i = 0; i < n_waiting; ++i) {
    const int64_t n = waiting[i].prompt_tokens;
    const double d = waiting[i].arrival_time + M.slo;
    if (now + ttft(M, n, n * n) < d) S.push_back(i);
    else dropped[nd++] = i;
  }
  // Algorithm 2 (Sec. 6.3): earliest deadline first (queue order among equal deadlines)
  std::stable_sort(S.begin(), S.end(), [&](int32_t a, int32_t b) {
    return waiting[a].arrival_time + M.slo < waiting[b].arrival_time + M.slo;
  });
  // Algorithm 2 (Sec. 6.3), removal loop: while the whole batch's prefill would finish after the front request's deadline, remove the
  // longest request (the latest in deadline order among equally long ones).  Running integer sums, a max-heap over
  // (length, position) and a front pointer over removed flags replace the rescans.
  const int ns = (int)S.size();
  int64_t s1 = 0, s2 = 0;
  std::priority_queue<std::pair<int64_t, int32_t>> longest;  // (tokens, position in S)
  for (int k = 0; k < ns; ++k) {
    const int64_t n = waiting[S[k]].prompt_tokens;
    s1 += n;
    s2 += n * n;
    longest.emplace(n, k);
  }
  std::vector<char> gone(ns, 0);
  int front = 0, left = ns;
  while (left > 0) {
    while (gone[front]) ++front;
    const double d0 = waiting[S[front]].arrival_time + M.slo;
    if (now + ttft(M, s1, s2) < d0) break;
    const int k = longest.top().second;  // never a removed one: each entry is popped when its request goes
    longest.pop();
    gone[k] = 1;
    const int64_t n = waiting[S[k]].prompt_tokens;
    s1 -= n;
    s2 -= n * n;
    --left;
  }
  // Algorithm 2 (Sec. 6.3), last step: trim to the caps, in deadline order
  int nsel = 0;
  int64_t total = 0;
  for (int k = 0; k < ns; ++k) {
    if (gone[k]) continue;
    const int64_t n = waiting[S[k]].prompt_tokens;
    if (nsel + 1 > M.n_max || total + n > M.t_max) break;
    selected[nsel++] = S[k];
    total += n;
  }
  *n_selected = nsel;
  *n_dropped = nd;
  return FS_OK;
}

int fs_sched_place_models(const double* footprint, const double* mu, int n_models, const double* capacity, int n_gpus,
                          int32_t* placement) {
  if (n_models < 0 || n_gpus < 0 || (n_models > 0 && (!footprint || !mu || !placement)) || (n_gpus > 0 && !capacity)) {
    set_error("fs_sched_place_models: invalid argument");
    return FS_ERR_INVALID;
  }
  std::vector<int32_t> order(n_models);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return footprint[a] > footprint[b]; });
  std::vector<std::vector<int32_t>> resident(n_gpus);
  for (int i = 0; i < n_models; ++i) placement[i] = -1;
  for (int32_t m : order) {
    int best = -1;
    double best_score = 0.0;
    for (int g = 0; g < n_gpus; ++g) {
      // K_rem(G') and the group's mu sum, added in residence order then the candidate (the order of the plain
      // re-statement, so the two agree to the last bit)
      double used = 0.0, mus = 0.0;
      for (int32_t r : resident[g]) {
        used += footprint[r];
        mus += mu[r];
      }
      used += footprint[m];
      mus += mu[m];
      const double k_rem = capacity[g] - used;
      if (k_rem < 0) continue;
      const double score = (mus / (double)(resident[g].size() + 1)) * k_rem;
      if (best < 0 || score > best_score) {
        best = g;
        best_score = score;
      }
    }
    if (best >= 0) {
      resident[best].push_back(m);
      placement[m] = best;
    }
  }
  return FS_OK;
}
