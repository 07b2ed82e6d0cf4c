// Load balancer: Algorithm CREATE-BALANCED-BATCHES of arXiv 2504.10700 (Section 3), host code.
// See include/bb.h for the operation and the readings taken.
//
// Graphs wait in one queue, largest first.  A round opens its bins and runs passes over the bins
// that still accept graphs, kept as records (room left, bin number) in one array that is
// stable-sorted by room before every pass; bins given up in a pass are moved to a side array and
// come back only if a bin that is still accepting has ended the pass with less room than one of
// them.  Every pass but the last of a round places at least one graph per surviving bin, so the
// total cost is O(N log N + N log M), as the paper states.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <string>
#include <vector>

#include "../../include/bb.h"
#include "sc_internal.h"

namespace {

struct OpenBin {
  int64_t room;    // capacity not yet used
  int32_t number;  // position in the output numbering
};

}  // namespace

extern "C" sc_status bb_create_balanced_batches(const int32_t* sizes, int64_t n_graphs, int64_t capacity,
                                                int32_t n_gpus, int32_t* bin_of_graph, int32_t* slot_of_graph,
                                                int64_t* n_bins) {
  using sc::set_error;
  constexpr int64_t kMost = (int64_t(1) << 31) - 1;
  if (!n_bins) return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: n_bins is NULL");
  *n_bins = 0;
  if (n_graphs < 0 || capacity < 1 || n_gpus < 1)
    return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: n_graphs < 0, capacity < 1 or n_gpus < 1");
  if (n_graphs == 0) return SC_OK;
  if (!sizes || !bin_of_graph) return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: NULL array");
  if (n_graphs > kMost) return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: more than 2^31-1 graphs");
  for (int64_t i = 0; i < n_graphs; ++i)
    if (sizes[i] < 0 || sizes[i] > capacity)
      return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: graph " + std::to_string(i) +
                                               " is larger than the capacity (or negative)");

  // the queue: graph indices, largest graph first, equal graphs in input order
  std::vector<int32_t> queue(n_graphs);
  std::iota(queue.begin(), queue.end(), 0);
  std::stable_sort(queue.begin(), queue.end(), [&](int32_t a, int32_t b) { return sizes[a] > sizes[b]; });
  int64_t unplaced = 0;  // vertices of the graphs still in the queue
  for (int64_t i = 0; i < n_graphs; ++i) unplaced += sizes[i];

  std::vector<int32_t> filled;  // graphs in every bin opened so far (the next slot number)
  std::vector<OpenBin> accepting, given_up;
  int64_t head = 0;             // next graph of the queue
  while (head < n_graphs) {     // one round per iteration
    int64_t opened = std::max<int64_t>((unplaced + capacity - 1) / capacity, 1);
    opened = (opened + n_gpus - 1) / n_gpus * n_gpus;
    const int64_t first = static_cast<int64_t>(filled.size());
    if (first + opened > kMost) return set_error(SC_ERR_INVALID_ARG, "bb_create_balanced_batches: more than 2^31-1 bins");
    filled.resize(first + opened, 0);
    accepting.clear();
    for (int64_t k = 0; k < opened; ++k) accepting.push_back(OpenBin{capacity, static_cast<int32_t>(first + k)});

    while (head < n_graphs && !accepting.empty()) {  // one pass per iteration
      std::stable_sort(accepting.begin(), accepting.end(),
                       [](const OpenBin& a, const OpenBin& b) { return a.room > b.room; });
      given_up.clear();
      size_t keep = 0;  // accepting[0..keep) survive the pass, in order
      for (size_t k = 0; k < accepting.size(); ++k) {
        OpenBin bin = accepting[k];
        if (head < n_graphs) {
          const int32_t g = queue[head];
          if (bin.room < sizes[g]) {  // no room for the graph on offer: out for this round, the graph stays next
            given_up.push_back(bin);
            continue;
          }
          bin_of_graph[g] = bin.number;
          if (slot_of_graph) slot_of_graph[g] = filled[bin.number];
          ++filled[bin.number];
          bin.room -= sizes[g];
          unplaced -= sizes[g];
          ++head;
        }
        accepting[keep++] = bin;  // also the bins the pass did not reach once the queue was empty
      }
      accepting.resize(keep);
      if (accepting.empty() || given_up.empty()) continue;
      const auto by_room = [](const OpenBin& a, const OpenBin& b) { return a.room < b.room; };
      const int64_t least_accepting = std::min_element(accepting.begin(), accepting.end(), by_room)->room;
      const int64_t most_given_up = std::max_element(given_up.begin(), given_up.end(), by_room)->room;
      if (least_accepting < most_given_up) accepting.insert(accepting.end(), given_up.begin(), given_up.end());
    }
  }
  *n_bins = static_cast<int64_t>(filled.size());
  return SC_OK;
}
