"""CPU oracle for the round scheduler (paper Section 4.4, Algorithm 1).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file; it shares no code with the C++
implementation in the library.

The algorithm's steps, in the paper's order and notation.

Stage 1.  Image candidates: for every GPU budget g in 0..N, EdfBatch(I(t), g) gives a plan B*(g, t); its score is the
pair (|B*(g,t)|, f_img_g) with  f_img_g = sum_{i in B*} 1 / (1 + max(0, slack_i(g,t)))  (Eq. 4), slack_i being the time
between the predicted completion of i's batch and i's deadline.  Video candidates: every video v has a list C_v(t);
candidate c has a GPU cost w(c), a GPU set, and a projected laxity l_v(c,t) = D_v - (t + S_rem_v * T_step(p(c)))
(the deadline slack of Eq. 1 evaluated for the candidate's configuration); its score is
(recoverable(c), f(c)) = (1[l >= 0], 1 / (1 + |l|))  (Eq. 5); a hold candidate costs no GPU and scores (0, 0).

Stage 2.  dp[0][0] = (0, 0), every other dp[0][b] = -inf.  For j = 1..G, b = 0..N:
    dp[j][b] = max over c in C_{v_j} with w(c) <= b and no GPU shared with the selections behind dp[j-1][b-w(c)]
               of dp[j-1][b-w(c)] + (recoverable(c), f(c))                                                   (Eq. 6)
compared lexicographically, with a back-pointer.

Stage 3.  For every terminal b with dp[G][b] finite, g_free = N - b and the plan's value is
dp[G][b] + (|B*(g_free)|, f_img_{g_free}), again lexicographic; the best one is back-tracked.

Readings where the paper is silent (also listed in the design notes):
  * EdfBatch: images sorted by deadline (ties: input order); the next image joins the open batch if, with the batch one
    larger, every member still finishes by its deadline (completion t + T_img(b)) and b <= b_max; otherwise, if it can
    meet its deadline alone and a GPU is left, it opens the next batch; otherwise it is left out of B*.  One batch per GPU.
  * the first candidate (in list order) among equal scores wins; among equal terminal values the smallest b wins.
  * "no GPU overlap" is checked against the selections on the back-pointer path of the predecessor state (a state keeps
    one path, so with anchored GPU sets the DP is a heuristic; with unanchored candidates - empty sets - it is exact).

Pins (tests/test_sched_dp.py): hand-worked rounds; an exhaustive enumeration of all candidate combinations on small
instances with unanchored candidates (the DP must reach the enumerated optimum); EdfBatch against hand cases and its
invariants; Eq. 1/4/5 values computed by hand.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

__all__ = ["VideoCandidate", "edf_batch", "image_score", "video_score", "laxity", "solve_round", "enumerate_best"]

NEG = (-math.inf, -math.inf)


@dataclass
class VideoCandidate:
    gpus: int                 # w(c)
    gpu_mask: int = 0         # bit i set: GPU i; 0 = not anchored (or hold)
    laxity: float = 0.0       # l_v(c, t)
    hold: bool = False


def laxity(deadline: float, t: float, steps_remaining: int, t_step: float) -> float:
    """Eq. 1 for a candidate configuration: D_v - t - S_rem * T_step."""
    return deadline - t - steps_remaining * t_step


def video_score(c: VideoCandidate):
    """Eq. 5: (recoverable, f)."""
    if c.hold:
        return (0, 0.0)
    return (1 if c.laxity >= 0 else 0, 1.0 / (1.0 + abs(c.laxity)))


def edf_batch(deadlines, t: float, g: int, t_img, b_max: int):
    """B*(g, t).  deadlines: list of D_i; t_img[b-1]: latency of a batch of b images.  Returns (batch_of_image, sizes):
    batch_of_image[i] = index of i's batch (0..g-1) or -1; sizes[k] = images in batch k."""
    order = sorted(range(len(deadlines)), key=lambda i: (deadlines[i], i))
    batch_of = [-1] * len(deadlines)
    batches = []  # lists of image indices
    for i in order:
        placed = False
        if batches:
            cur = batches[-1]
            b = len(cur) + 1
            if b <= b_max and all(t + t_img[b - 1] <= deadlines[m] for m in cur + [i]):
                cur.append(i)
                placed = True
        if not placed and len(batches) < g and t + t_img[0] <= deadlines[i]:
            batches.append([i])
            placed = True
        if placed:
            batch_of[i] = len(batches) - 1
    return batch_of, [len(b) for b in batches]


def image_score(deadlines, t: float, batch_of, sizes, t_img):
    """(|B*|, f_img) of a plan, Eq. 4."""
    n, f = 0, 0.0
    for i, k in enumerate(batch_of):
        if k < 0:
            continue
        slack = deadlines[i] - (t + t_img[sizes[k] - 1])
        n += 1
        f += 1.0 / (1.0 + max(0.0, slack))
    return (n, f)


def _add(a, b):
    return (a[0] + b[0], a[1] + b[1])


def solve_round(n_gpus: int, videos, image_deadlines, t: float, t_img, b_max: int):
    """videos: list (one per video) of lists of VideoCandidate.  Returns a dict with the chosen candidate index per video,
    the GPUs used by videos (b*), the image plan for the free GPUs and the value (recoverable count, f sum)."""
    N, G = n_gpus, len(videos)
    img = []
    for g in range(N + 1):                                                   # Stage 1
        batch_of, sizes = edf_batch(image_deadlines, t, g, t_img, b_max)
        img.append((image_score(image_deadlines, t, batch_of, sizes, t_img), batch_of, sizes))
    dp = [[NEG] * (N + 1) for _ in range(G + 1)]                            # Stage 2
    used = [[0] * (N + 1) for _ in range(G + 1)]
    back = [[None] * (N + 1) for _ in range(G + 1)]
    dp[0][0] = (0, 0.0)
    for j in range(1, G + 1):
        for b in range(N + 1):
            for ci, c in enumerate(videos[j - 1]):
                w = c.gpus
                if w > b or dp[j - 1][b - w] == NEG:
                    continue
                if c.gpu_mask & used[j - 1][b - w]:
                    continue
                s = _add(dp[j - 1][b - w], video_score(c))
                if s > dp[j][b]:
                    dp[j][b], back[j][b], used[j][b] = s, ci, used[j - 1][b - w] | c.gpu_mask
    best, best_b = NEG, -1                                                   # Stage 3
    for b in range(N + 1):
        if dp[G][b] == NEG:
            continue
        total = _add(dp[G][b], img[N - b][0])
        if total > best:
            best, best_b = total, b
    if best_b < 0:
        return {"feasible": False}
    choice, b = [0] * G, best_b
    for j in range(G, 0, -1):
        ci = back[j][b]
        choice[j - 1] = ci
        b -= videos[j - 1][ci].gpus
    return {"feasible": True, "choice": choice, "video_gpus": best_b, "value": best,
            "image_batch_of": img[N - best_b][1], "image_batch_sizes": img[N - best_b][2], "used_mask": used[G][best_b]}


def enumerate_best(n_gpus: int, videos, image_deadlines, t: float, t_img, b_max: int):
    """Exhaustive search over one candidate per video (capacity and GPU-set disjointness enforced exactly); the value of
    the best combination including the image plan for the GPUs left.  For pinning solve_round on small instances."""
    import itertools
    best = NEG
    for combo in itertools.product(*[range(len(c)) for c in videos]):
        cs = [videos[j][ci] for j, ci in enumerate(combo)]
        b = sum(c.gpus for c in cs)
        if b > n_gpus:
            continue
        mask, ok = 0, True
        for c in cs:
            if c.gpu_mask & mask:
                ok = False
                break
            mask |= c.gpu_mask
        if not ok:
            continue
        val = (0, 0.0)
        for c in cs:
            val = _add(val, video_score(c))
        batch_of, sizes = edf_batch(image_deadlines, t, n_gpus - b, t_img, b_max)
        val = _add(val, image_score(image_deadlines, t, batch_of, sizes, t_img))
        if val > best:
            best = val
    return best
