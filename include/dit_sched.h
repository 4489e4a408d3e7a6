/*
 * dit_sched.h - C ABI of the round scheduler that decides which packs the attention kernels see
 * (paper Section 4.4 "SLO-aware Online Scheduler", Algorithm 1; deadline slack Eq. 1, image score Eq. 4, video
 * candidate score Eq. 5, DP transition Eq. 6).  Host-only: no GPU, no context, no allocation visible to the caller;
 * all pointers are HOST pointers; thread-safe (no global state).
 *
 * One call plans one round at time t for a cluster of n_gpus GPUs:
 *   Stage 1  for every GPU budget g = 0..n_gpus an earliest-deadline-first batching of the pending images
 *            (B*(g,t), scored by Eq. 4); every video candidate scored by Eq. 5 from its projected laxity;
 *   Stage 2  knapsack DP over the video groups, lexicographic objective (recoverable count, utility), Eq. 6,
 *            candidates anchored to GPU sets may not share a GPU with the selections behind the predecessor state;
 *   Stage 3  every terminal state combined with the image plan for the GPUs it leaves free; back-tracking.
 *
 * Readings where the paper is silent:
 *   - EdfBatch: images in deadline order (ties: input order); an image joins the open batch if with the batch one
 *     larger (at most b_max) every member still finishes by its deadline, completion being t + t_img[b-1]; otherwise
 *     it opens the next batch if a GPU is left and it can meet its deadline alone; otherwise it is not served this
 *     round.  One batch per GPU.
 *   - among equal scores the first candidate in list order wins; among equal terminal values the smallest number of
 *     video GPUs wins.
 *   - one image class per call (one latency table).
 */
#ifndef DIT_SCHED_H_
#define DIT_SCHED_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DIT_SCHED_OK             0
#define DIT_SCHED_ERR_NULL      (-1)  /* a required pointer is NULL */
#define DIT_SCHED_ERR_ARG       (-2)  /* n_gpus outside 1..32, negative counts, b_max < 1, a candidate with gpus < 0 or
                                         > n_gpus, a mask with bits at or above n_gpus, a non-zero mask whose bit count
                                         is not `gpus`, a non-zero `reserved`, offsets not increasing */
#define DIT_SCHED_ERR_INFEASIBLE (-3) /* some video has no candidate that fits (give every video a hold candidate) */

/* One candidate of one video (Section 4.4: hold, continue, scale up / down, resume on a pool). */
typedef struct {
  int32_t gpus;      /* w(c): GPUs the candidate occupies; 0 for hold */
  uint32_t gpu_mask; /* the GPU set it is anchored to (bit i = GPU i), 0 if not anchored */
  double laxity;     /* l_v(c,t) = D_v - (t + S_rem_v * T_step(config of c)), see dit_sched_laxity; unused for hold */
  int32_t hold;      /* non-zero: hold candidate, value (0, 0) */
  int32_t reserved;  /* must be 0 */
} dit_sched_candidate;

/* Eq. 1 evaluated for a configuration: deadline - t_now - steps_remaining * t_step. */
double dit_sched_laxity(double deadline, double t_now, int32_t steps_remaining, double t_step);

/*
 * Plans one round.
 *   n_gpus           N, 1..32
 *   candidates       all videos' candidates, video j's are candidates[cand_offsets[j] .. cand_offsets[j+1])
 *   cand_offsets     n_videos + 1 increasing offsets starting at 0
 *   image_deadlines  n_images deadlines D_i (same clock as t_now); may be NULL when n_images == 0
 *   t_img            b_max latencies: t_img[b-1] = profiled latency of a batch of b images
 * Outputs (caller-allocated, may be NULL if not wanted):
 *   choice[n_videos]          index (within the video's own list) of the chosen candidate
 *   image_batch[n_images]     batch index 0..n_batches-1 of each image, -1 if not served this round
 *   image_gpu[n_gpus]         image_gpu[k] = GPU id given to image batch k (the free GPUs in increasing order; valid for
 *                             k < *n_batches; anchored video candidates' GPUs are excluded, unanchored ones are assumed to
 *                             be placed by the caller)
 *   n_batches, video_gpus     number of image batches; GPUs occupied by the chosen video candidates (b*)
 *   recoverable, utility      the plan's value: requests that meet their deadline, sum of f
 * Returns DIT_SCHED_OK or an error code; outputs are untouched on error.
 */
int dit_sched_plan_round(int32_t n_gpus,
                         const dit_sched_candidate* candidates, const int32_t* cand_offsets, int32_t n_videos,
                         const double* image_deadlines, int32_t n_images, double t_now,
                         const double* t_img, int32_t b_max,
                         int32_t* choice, int32_t* image_batch, int32_t* image_gpu, int32_t* n_batches,
                         int32_t* video_gpus, int32_t* recoverable, double* utility);

#ifdef __cplusplus
}
#endif
#endif /* DIT_SCHED_H_ */
