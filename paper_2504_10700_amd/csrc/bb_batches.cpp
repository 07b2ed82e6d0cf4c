// Load balancer: Algorithm CREATE-BALANCED-BATCHES of arXiv 2504.10700 (Section 3), host code.
// See include/bb.h for the operation and the readings taken.
//
// Cost: one stable sort of the graphs, then per sweep one stable sort of the active bins and
// one pass over them; every sweep but the last of a call places at least one graph per
// surviving bin, so the total is O(N log N + N log M) as the paper states.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <string>
#include <vector>

#include "../../include/bb.h"
#include "sc_internal.h"

extern "C" sc_status bb_create_balanced_batches(const int32_t* sizes, int64_t n_graphs, int64_t capacity,
                                                int32_t n_gpus, int32_t* bin_of_graph, int32_t* slot_of_graph,
                                                int64_t* n_bins) {
  using sc::set_error;
  if (!n_bins) return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: n_bins is NULL");
  *n_bins = 0;
  if (n_graphs < 0 || capacity < 1 || n_gpus < 1)
    return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: n_graphs < 0, capacity < 1 or n_gpus < 1");
  if (n_graphs == 0) return SC_OK;
  if (!sizes || !bin_of_graph) return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: NULL array");
  if (n_graphs > (int64_t(1) << 31) - 1)
    return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: more than 2^31-1 graphs");
  for (int64_t i = 0; i < n_graphs; ++i)
    if (sizes[i] < 0 || sizes[i] > capacity)
      return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: graph " + std::to_string(i) +
                                               " is larger than the capacity (or negative)");
  const int64_t N = n_graphs;
  // (L, I) <- StableSort(L, descending)
  std::vector<int32_t> order(N);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return sizes[a] > sizes[b]; });

  std::vector<int64_t> cap;         // remaining capacity of every bin created so far
  std::vector<int32_t> fill;        // graphs placed in every bin so far
  std::vector<int64_t> active, still, full;
  int64_t p = 0;                    // pointer into the sorted list
  while (p < N) {                   // one round = one (recursive) call of the algorithm on the rest
    int64_t S = 0;
    for (int64_t q = p; q < N; ++q) S += sizes[order[q]];
    int64_t M = (S + capacity - 1) / capacity;
    if (M < 1) M = 1;
    M = (M + n_gpus - 1) / n_gpus * n_gpus;
    const int64_t first = static_cast<int64_t>(cap.size());
    if (first + M > (int64_t(1) << 31) - 1)
      return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: more than 2^31-1 bins");
    cap.resize(first + M, capacity);
    fill.resize(first + M, 0);
    active.resize(M);
    std::iota(active.begin(), active.end(), first);
    while (p < N && !active.empty()) {
      std::stable_sort(active.begin(), active.end(), [&](int64_t a, int64_t b) { return cap[a] > cap[b]; });
      still.clear();
      full.clear();
      for (const int64_t j : active) {
        if (p < N && cap[j] >= sizes[order[p]]) {
          const int32_t g = order[p];
          bin_of_graph[g] = static_cast<int32_t>(j);
          if (slot_of_graph) slot_of_graph[g] = fill[j];
          ++fill[j];
          cap[j] -= sizes[g];
          ++p;
          still.push_back(j);
        } else if (p < N) {
          full.push_back(j);        // cannot take the current graph: marked full
        } else {
          still.push_back(j);       // the sweep ended with the last graph: untouched bins stay
        }
      }
      active.swap(still);
      if (!full.empty() && !active.empty()) {
        int64_t min_active = cap[active[0]], max_full = cap[full[0]];
        for (const int64_t j : active) min_active = std::min(min_active, cap[j]);
        for (const int64_t j : full) max_full = std::max(max_full, cap[j]);
        if (min_active < max_full) active.insert(active.end(), full.begin(), full.end());  // second chance
      }
    }
  }
  *n_bins = static_cast<int64_t>(cap.size());
  return SC_OK;
}
