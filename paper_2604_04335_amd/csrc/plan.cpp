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
  plan_build_cross(cu, cu, n_seqs, n_heads, block_m, items);
}

void plan_build_cross(const int32_t* cu_q, const int32_t* cu_k, int32_t n_seqs, int32_t n_heads, int32_t block_m,
                      std::vector<WorkItem>& items, int32_t n_splits, int32_t block_n) {
  items.clear();
  // Sequence order: by number of keys (the cost of one item), most first; ties keep pack order (stable).
  std::vector<int32_t> order(static_cast<size_t>(n_seqs));
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
    return (cu_k[a + 1] - cu_k[a]) > (cu_k[b + 1] - cu_k[b]);
  });
  size_t total = 0;
  for (int32_t i = 0; i < n_seqs; ++i) {
    const int64_t len = cu_q[i + 1] - cu_q[i];
    if (cu_k[i + 1] > cu_k[i])
      total += static_cast<size_t>((len + block_m - 1) / block_m) * static_cast<size_t>(n_heads) * static_cast<size_t>(n_splits);
  }
  items.reserve(total);
  for (int32_t s : order) {
    const int32_t q0 = cu_q[s], q_len = cu_q[s + 1] - cu_q[s];
    const int32_t k0 = cu_k[s], k_len = cu_k[s + 1] - cu_k[s];
    if (q_len == 0 || k_len == 0) continue;
    const int32_t tiles = (k_len + block_n - 1) / block_n;
    const int32_t tiles_per_part = (tiles + n_splits - 1) / n_splits;
    const int32_t chunk = tiles_per_part * block_n;
    auto push_tile = [&](int32_t h, int32_t m0) {
      const int32_t rows = std::min(block_m, q_len - m0);
      for (int32_t part = 0, kb = 0; kb < k_len; ++part, kb += chunk)
        items.push_back(WorkItem{q0 + m0, k0 + kb, std::min(chunk, k_len - kb), (part << 28) | (rows << 16) | h});
    };
    // Whole query tiles of all heads first, then the ragged last tile of every head: a ragged tile is quicker (its
    // wavefronts without rows compute nothing), and a workgroup that gets ahead of the others in the middle of a
    // sequence streams K and V on its own from then on instead of sharing them in L2 with the workgroups beside it.
    const int32_t whole = q_len / block_m * block_m;
    for (int32_t h = 0; h < n_heads; ++h)
      for (int32_t m0 = 0; m0 < whole; m0 += block_m) push_tile(h, m0);
    if (whole < q_len)
      for (int32_t h = 0; h < n_heads; ++h) push_tile(h, whole);
  }
}

int plan_cache_victim(const uint64_t* last_use, const uint8_t* pinned, int n) {
  int victim = -1;
  for (int i = 0; i < n; ++i)
    if (!pinned[i] && (victim < 0 || last_use[i] < last_use[victim])) victim = i;
  return victim;
}

}  // namespace dit
