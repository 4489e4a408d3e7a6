#include "plan.h"

#include <algorithm>
#include <numeric>

namespace dit {

int plan_validate(const int32_t* cu, int32_t n_seqs) {
  if (n_seqs < 0) return 1;
  if (cu[0] != 0) return 1;
  for (int32_t i = 0; i < n_seqs; ++i)
    if (cu[i + 1] < cu[i]) return 1;
  return 0;
}

void plan_build(const int32_t* cu, int32_t n_seqs, int32_t n_heads, int32_t block_m,
                std::vector<WorkItem>& items) {
  items.clear();
  // Sequence order: by length, longest first; ties keep pack order (stable).
  std::vector<int32_t> order(static_cast<size_t>(n_seqs));
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    return (cu[a + 1] - cu[a]) > (cu[b + 1] - cu[b]);
  });
  size_t total = 0;
  for (int32_t i = 0; i < n_seqs; ++i) {
    const int64_t len = cu[i + 1] - cu[i];
    total += static_cast<size_t>((len + block_m - 1) / block_m) * static_cast<size_t>(n_heads);
  }
  items.reserve(total);
  for (int32_t s : order) {
    const int32_t start = cu[s];
    const int32_t len = cu[s + 1] - cu[s];
    if (len == 0) continue;
    for (int32_t h = 0; h < n_heads; ++h) {
      for (int32_t m0 = 0; m0 < len; m0 += block_m) {
        const int32_t rows = std::min(block_m, len - m0);
        items.push_back(WorkItem{start + m0, start, len, (rows << 16) | h});
      }
    }
  }
}

}  // namespace dit
