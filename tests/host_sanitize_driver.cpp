// Driver for the host-side code of the library under AddressSanitizer and
// UndefinedBehaviorSanitizer (built and run by tests/test_host_sanitizers.py; CPU only):
// the coupling-table builder (sc_tables.cpp) over every supported configuration family and
// the load balancer (bb_batches.cpp) on seeded size lists, including its error paths.
#include <cstdint>
#include <cstdio>
#include <random>
#include <string>
#include <vector>

#include "../include/bb.h"
#include "../paper_2504_10700_amd/csrc/sc_tables.h"

namespace sc {
// what sc_api.hip provides in the library
sc_status set_error(sc_status code, const std::string&) { return code; }
}  // namespace sc

int main() {
  long checksum = 0;
  for (int l_max = 0; l_max <= 3; ++l_max)
    for (int nu_max = 1; nu_max <= 3; ++nu_max) {
      std::vector<int> out_l, out_p;
      for (int L = 0; L <= 3; ++L) {
        out_l.push_back(L);
        out_p.push_back(L % 2 ? -1 : 1);
      }
      for (size_t n_out = 1; n_out <= out_l.size(); ++n_out) {
        sc::PathTable t;
        const char* msg = nullptr;
        const std::vector<int> ol(out_l.begin(), out_l.begin() + n_out), op(out_p.begin(), out_p.begin() + n_out);
        if (!sc::build_path_table(l_max, nu_max, ol, op, &t, &msg)) continue;   // an irrep no path reaches
        for (const auto& terms : t.terms) checksum += static_cast<long>(terms.size());
      }
    }
  for (int l1 = 0; l1 <= 6; ++l1)
    for (int l2 = 0; l2 <= 6; ++l2)
      for (int l3 = 0; l3 <= 6; ++l3) checksum += static_cast<long>(sc::coupling_tensor(l1, l2, l3).size());

  std::mt19937 rng(17);
  for (int rep = 0; rep < 20; ++rep) {
    const int n = 1 + static_cast<int>(rng() % 3000);
    const int64_t cap = 64 + rng() % 3000;
    std::vector<int32_t> sizes(n), bins(n), slots(n);
    for (auto& s : sizes) s = static_cast<int32_t>(rng() % (cap + 1));
    int64_t n_bins = 0;
    if (bb_create_balanced_batches(sizes.data(), n, cap, 1 + rep % 8, bins.data(), slots.data(), &n_bins) != SC_OK) return 2;
    for (int i = 0; i < n; ++i)
      if (bins[i] < 0 || bins[i] >= n_bins) return 3;
    checksum += n_bins;
  }
  {  // error paths
    int32_t one = 5, bin = 0;
    int64_t nb = 0;
    if (bb_create_balanced_batches(&one, 1, 4, 1, &bin, nullptr, &nb) != SC_ERR_INVALID_ARG) return 4;
    if (bb_create_balanced_batches(nullptr, 0, 4, 1, nullptr, nullptr, &nb) != SC_OK) return 5;
    if (bb_create_balanced_batches(&one, 1, 0, 1, &bin, nullptr, &nb) != SC_ERR_INVALID_ARG) return 6;
  }
  std::printf("host sanitizer driver done, checksum %ld\n", checksum);
  return 0;
}
