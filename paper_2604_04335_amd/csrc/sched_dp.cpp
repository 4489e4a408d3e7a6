// Round scheduler: Algorithm 1 of the paper (Section 4.4) with Eq. 1, 4, 5, 6.  Host code; see include/dit_sched.h for
// the interface and the readings.  O(N * (n_images + G * K)) per call, no heap use beyond a few small vectors.
#include "../../include/dit_sched.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

namespace {

struct Value {  // lexicographic (recoverable count, utility)
  int32_t rec;
  double f;
  bool valid;
};
inline bool better(const Value& a, const Value& b) {  // a > b; an invalid value is below every valid one
  if (!a.valid) return false;
  if (!b.valid) return true;
  return a.rec != b.rec ? a.rec > b.rec : a.f > b.f;
}

struct ImagePlan {
  Value value{0, 0.0, true};
  std::vector<int32_t> batch_of;  // per image, -1 = not served
  int32_t n_batches = 0;
};

// Stage 1, images: earliest-deadline-first batching on g GPUs and its Eq. 4 score.
ImagePlan edf_batch(const std::vector<int32_t>& order, const double* deadline, int32_t n_images, double t, int32_t g,
                    const double* t_img, int32_t b_max) {
  ImagePlan plan;
  plan.batch_of.assign(static_cast<size_t>(n_images), -1);
  std::vector<int32_t> sizes;
  double open_min_deadline = 0.0;  // earliest deadline in the open batch (its first member, by the order)
  for (int32_t i : order) {
    bool placed = false;
    if (!sizes.empty()) {
      const int32_t b = sizes.back() + 1;
      // members were added in deadline order, so the first member has the earliest deadline and the newcomer the latest
      if (b <= b_max && t + t_img[b - 1] <= open_min_deadline && t + t_img[b - 1] <= deadline[i]) {
        sizes.back() = b;
        placed = true;
      }
    }
    if (!placed && static_cast<int32_t>(sizes.size()) < g && t + t_img[0] <= deadline[i]) {
      sizes.push_back(1);
      open_min_deadline = deadline[i];
      placed = true;
    }
    if (placed) plan.batch_of[static_cast<size_t>(i)] = static_cast<int32_t>(sizes.size()) - 1;
  }
  plan.n_batches = static_cast<int32_t>(sizes.size());
  for (int32_t i = 0; i < n_images; ++i) {
    const int32_t k = plan.batch_of[static_cast<size_t>(i)];
    if (k < 0) continue;
    const double slack = deadline[i] - (t + t_img[sizes[static_cast<size_t>(k)] - 1]);
    plan.value.rec += 1;
    plan.value.f += 1.0 / (1.0 + std::max(0.0, slack));
  }
  return plan;
}

}  // namespace

extern "C" {

double dit_sched_laxity(double deadline, double t_now, int32_t steps_remaining, double t_step) {
  return deadline - t_now - static_cast<double>(steps_remaining) * t_step;
}

int dit_sched_plan_round(int32_t n_gpus, const dit_sched_candidate* candidates, const int32_t* cand_offsets, int32_t n_videos,
                         const double* image_deadlines, int32_t n_images, double t_now, const double* t_img, int32_t b_max,
                         int32_t* choice, int32_t* image_batch, int32_t* image_gpu, int32_t* n_batches, int32_t* video_gpus,
                         int32_t* recoverable, double* utility) {
  if (n_gpus < 1 || n_gpus > 32 || n_videos < 0 || n_images < 0 || b_max < 1) return DIT_SCHED_ERR_ARG;
  if (!cand_offsets || !t_img || (n_images > 0 && !image_deadlines)) return DIT_SCHED_ERR_NULL;
  if (cand_offsets[0] != 0) return DIT_SCHED_ERR_ARG;
  for (int32_t j = 0; j < n_videos; ++j)
    if (cand_offsets[j + 1] < cand_offsets[j]) return DIT_SCHED_ERR_ARG;
  const int32_t n_cand = cand_offsets[n_videos];
  if (n_cand > 0 && !candidates) return DIT_SCHED_ERR_NULL;
  const uint32_t all = n_gpus == 32 ? 0xFFFFFFFFu : ((1u << n_gpus) - 1u);
  for (int32_t c = 0; c < n_cand; ++c) {
    const dit_sched_candidate& cd = candidates[c];
    if (cd.gpus < 0 || cd.gpus > n_gpus || (cd.gpu_mask & ~all) || cd.reserved != 0) return DIT_SCHED_ERR_ARG;
    // An anchored candidate names exactly the GPUs it counts: the GPU assignment of the image batches relies on it.
    if (cd.gpu_mask != 0 && __builtin_popcount(cd.gpu_mask) != cd.gpus) return DIT_SCHED_ERR_ARG;
  }

  try {
    const int32_t N = n_gpus, G = n_videos;
    // Stage 1: image plans for every budget (deadline order computed once).
    std::vector<int32_t> order(static_cast<size_t>(n_images));
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return image_deadlines[a] < image_deadlines[b]; });
    std::vector<ImagePlan> img(static_cast<size_t>(N) + 1);
    for (int32_t g = 0; g <= N; ++g) img[static_cast<size_t>(g)] = edf_batch(order, image_deadlines, n_images, t_now, g, t_img, b_max);

    // Stage 2: dp[j][b], back-pointers and the GPU set behind each state.
    const size_t W = static_cast<size_t>(N) + 1;
    std::vector<Value> dp((static_cast<size_t>(G) + 1) * W, Value{0, 0.0, false});
    std::vector<uint32_t> used((static_cast<size_t>(G) + 1) * W, 0u);
    std::vector<int32_t> back((static_cast<size_t>(G) + 1) * W, -1);
    dp[0] = Value{0, 0.0, true};
    for (int32_t j = 1; j <= G; ++j) {
      for (int32_t b = 0; b <= N; ++b) {
        Value best{0, 0.0, false};
        int32_t best_c = -1;
        uint32_t best_used = 0;
        for (int32_t c = cand_offsets[j - 1]; c < cand_offsets[j]; ++c) {
          const dit_sched_candidate& cd = candidates[c];
          if (cd.gpus > b) continue;
          const size_t prev = static_cast<size_t>(j - 1) * W + static_cast<size_t>(b - cd.gpus);
          if (!dp[prev].valid || (cd.gpu_mask & used[prev])) continue;
          Value s = dp[prev];
          if (!cd.hold) {  // Eq. 5
            s.rec += cd.laxity >= 0.0 ? 1 : 0;
            s.f += 1.0 / (1.0 + std::fabs(cd.laxity));
          }
          if (better(s, best)) {
            best = s;
            best_c = c - cand_offsets[j - 1];
            best_used = used[prev] | cd.gpu_mask;
          }
        }
        const size_t cur = static_cast<size_t>(j) * W + static_cast<size_t>(b);
        dp[cur] = best;
        back[cur] = best_c;
        used[cur] = best_used;
      }
    }

    // Stage 3: terminal states with the image plan for the GPUs left.
    Value best{0, 0.0, false};
    int32_t best_b = -1;
    for (int32_t b = 0; b <= N; ++b) {
      const Value& v = dp[static_cast<size_t>(G) * W + static_cast<size_t>(b)];
      if (!v.valid) continue;
      const Value& im = img[static_cast<size_t>(N - b)].value;
      const Value total{v.rec + im.rec, v.f + im.f, true};
      if (better(total, best)) {
        best = total;
        best_b = b;
      }
    }
    if (best_b < 0) return DIT_SCHED_ERR_INFEASIBLE;

    // Back-tracking and materialisation.
    const uint32_t video_mask = used[static_cast<size_t>(G) * W + static_cast<size_t>(best_b)];
    if (choice) {
      int32_t b = best_b;
      for (int32_t j = G; j >= 1; --j) {
        const int32_t ci = back[static_cast<size_t>(j) * W + static_cast<size_t>(b)];
        choice[j - 1] = ci;
        b -= candidates[cand_offsets[j - 1] + ci].gpus;
      }
    }
    const ImagePlan& plan = img[static_cast<size_t>(N - best_b)];
    if (image_batch) std::copy(plan.batch_of.begin(), plan.batch_of.end(), image_batch);
    if (image_gpu) {
      int32_t k = 0;
      for (int32_t gidx = 0; gidx < N; ++gidx) {
        image_gpu[gidx] = -1;
      }
      for (int32_t gidx = 0; gidx < N && k < plan.n_batches; ++gidx)
        if (!((video_mask >> gidx) & 1u)) image_gpu[k++] = gidx;
    }
    if (n_batches) *n_batches = plan.n_batches;
    if (video_gpus) *video_gpus = best_b;
    if (recoverable) *recoverable = best.rec;
    if (utility) *utility = best.f;
    return DIT_SCHED_OK;
  } catch (...) {
    return DIT_SCHED_ERR_ARG;
  }
}

}  // extern "C"
