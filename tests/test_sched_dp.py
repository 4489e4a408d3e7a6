"""Pins for the round-scheduler oracle, and parity of the C++ implementation (host code, no GPU needed) with it."""
import math
import os

import numpy as np
import pytest

from oracle import sched_dp_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "sched_cases.txt")
T_IMG = [1.0, 1.5, 2.0, 2.5]


def _parse_cases():
    cases = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, vids, imgs, exp = [p.strip() for p in line.split("|")]
        videos = []
        for v in vids.split(";"):
            cands = []
            for c in v.split(","):
                c = c.strip()
                if c == "H":
                    cands.append(orc.VideoCandidate(gpus=0, hold=True))
                else:
                    g, l = c.split(":")
                    cands.append(orc.VideoCandidate(gpus=int(g), laxity=float(l)))
            videos.append(cands)
        deadlines = [float(x) for x in imgs.split(";")] if imgs else []
        ch, b, rec, f = [p.strip() for p in exp.split(";")]
        cases.append((name, videos, deadlines, [int(x) for x in ch.split(",")], int(b), int(rec), float(f)))
    return cases


@pytest.mark.parametrize("case", _parse_cases(), ids=lambda c: c[0])
def test_hand_worked_rounds(case):
    name, videos, deadlines, choice, b, rec, f = case
    r = orc.solve_round(4, videos, deadlines, 0.0, T_IMG, 4)
    assert r["feasible"] and r["choice"] == choice and r["video_gpus"] == b
    assert r["value"][0] == rec and abs(r["value"][1] - f) < 1e-12


def test_equations_by_hand():
    # Eq. 1: deadline 100, now 40, 20 steps of 2.5 s left -> slack 10
    assert orc.laxity(100.0, 40.0, 20, 2.5) == 10.0
    # Eq. 5: laxity 3 -> (1, 1/4); laxity -1 -> (0, 1/2); hold -> (0, 0)
    assert orc.video_score(orc.VideoCandidate(2, 0, 3.0)) == (1, 0.25)
    assert orc.video_score(orc.VideoCandidate(2, 0, -1.0)) == (0, 0.5)
    assert orc.video_score(orc.VideoCandidate(0, 0, 9.0, hold=True)) == (0, 0.0)
    # Eq. 4: two images in one batch of 2 (finishes at 1.5) with deadlines 2 and 4.5: slacks 0.5 and 3 -> 1/1.5 + 1/4
    assert orc.image_score([2.0, 4.5], 0.0, [0, 0], [2], T_IMG) == (2, 1 / 1.5 + 0.25)


def test_edf_batch_hand_cases_and_invariants():
    # deadlines 3, 1, 2.6, 0.5 (the last cannot be met even alone), one GPU: EDF order 0.5(skip), 1, 2.6, 3.
    # {1} alone; adding 2.6 makes b = 2 finish at 1.5 > 1 -> no second GPU, left out; same for 3.
    assert orc.edf_batch([3.0, 1.0, 2.6, 0.5], 0.0, 1, T_IMG, 4) == ([-1, 0, -1, -1], [1])
    # two GPUs: {1}, then {2.6} opens batch 2 and 3 joins it (b = 2 finishes at 1.5)
    assert orc.edf_batch([3.0, 1.0, 2.6, 0.5], 0.0, 2, T_IMG, 4) == ([1, 0, 1, -1], [1, 2])
    # b_max caps a batch even when deadlines are loose; no GPU, no plan
    assert orc.edf_batch([9.0] * 5, 0.0, 1, T_IMG, 4)[1] == [4]
    assert orc.edf_batch([9.0] * 5, 0.0, 0, T_IMG, 4) == ([-1] * 5, [])
    g = np.random.Generator(np.random.PCG64(501))
    for _ in range(200):
        n, gpus = int(g.integers(0, 12)), int(g.integers(0, 5))
        d = list(g.uniform(0.5, 4.0, size=n))
        batch_of, sizes = orc.edf_batch(d, 0.0, gpus, T_IMG, 4)
        assert len(sizes) <= gpus and all(1 <= s <= 4 for s in sizes)
        for i, k in enumerate(batch_of):
            assert k == -1 or T_IMG[sizes[k] - 1] <= d[i]
        assert sorted(k for k in batch_of if k >= 0) == sorted(sum(([k] * s for k, s in enumerate(sizes)), []))


def _random_instance(g, anchored):
    N = int(g.choice([2, 4, 8]))
    G = int(g.integers(0, 5))
    videos = []
    for _ in range(G):
        cands = [orc.VideoCandidate(gpus=0, hold=True)]
        for p in (1, 2, 4, 8):
            if p <= N and g.random() < 0.7:
                mask = 0
                if anchored:
                    start = int(g.integers(0, N // p)) * p
                    mask = ((1 << p) - 1) << start
                cands.append(orc.VideoCandidate(gpus=p, gpu_mask=mask, laxity=float(np.round(g.normal(1.0, 3.0), 3))))
        order = g.permutation(len(cands))
        videos.append([cands[i] for i in order])
    deadlines = list(np.round(g.uniform(0.5, 4.0, size=int(g.integers(0, 7))), 3))
    return N, videos, deadlines


def test_dp_reaches_the_enumerated_optimum_without_anchoring():
    g = np.random.Generator(np.random.PCG64(502))
    for _ in range(300):
        N, videos, deadlines = _random_instance(g, anchored=False)
        r = orc.solve_round(N, videos, deadlines, 0.0, T_IMG, 4)
        best = orc.enumerate_best(N, videos, deadlines, 0.0, T_IMG, 4)
        assert r["feasible"] and r["value"][0] == best[0] and abs(r["value"][1] - best[1]) < 1e-9


def test_dp_plans_are_valid_with_anchoring_and_never_beat_the_optimum():
    g = np.random.Generator(np.random.PCG64(503))
    for _ in range(300):
        N, videos, deadlines = _random_instance(g, anchored=True)
        r = orc.solve_round(N, videos, deadlines, 0.0, T_IMG, 4)
        assert r["feasible"]                                # hold is always there
        mask = 0
        for j, ci in enumerate(r["choice"]):
            c = videos[j][ci]
            assert not (c.gpu_mask & mask)
            mask |= c.gpu_mask
        assert sum(videos[j][ci].gpus for j, ci in enumerate(r["choice"])) == r["video_gpus"] <= N
        assert len(r["image_batch_sizes"]) <= N - r["video_gpus"]
        assert r["value"] <= orc.enumerate_best(N, videos, deadlines, 0.0, T_IMG, 4)


# ---------------------------------------------------------------- the C++ implementation against the oracle (host code)

def _solve_cpp(N, videos, deadlines, t=0.0):
    import paper_2604_04335_amd as da
    return da.dit_sched_plan_round(N, [[(c.gpus, c.gpu_mask, c.laxity, c.hold) for c in v] for v in videos], deadlines, t, T_IMG)


@pytest.mark.parametrize("case", _parse_cases(), ids=lambda c: c[0])
def test_cpp_hand_worked_rounds(case):
    name, videos, deadlines, choice, b, rec, f = case
    r = _solve_cpp(4, videos, deadlines)
    assert r["choice"] == choice and r["video_gpus"] == b and r["recoverable"] == rec and abs(r["utility"] - f) < 1e-12


@pytest.mark.parametrize("anchored", [False, True])
def test_cpp_matches_oracle_on_random_rounds(anchored):
    """Same plan (choice per video, image batches) and same value, bit for bit in the integer parts; the tie rules are the
    same on both sides, so the selections are compared directly."""
    g = np.random.Generator(np.random.PCG64(504 + anchored))
    for _ in range(500):
        N, videos, deadlines = _random_instance(g, anchored)
        t = float(np.round(g.uniform(0.0, 0.5), 3))
        want = orc.solve_round(N, videos, deadlines, t, T_IMG, 4)
        got = _solve_cpp(N, videos, deadlines, t)
        assert got["choice"] == want["choice"] and got["video_gpus"] == want["video_gpus"]
        assert got["recoverable"] == want["value"][0] and abs(got["utility"] - want["value"][1]) < 1e-12
        assert got["image_batch"] == want["image_batch_of"] and got["n_batches"] == len(want["image_batch_sizes"])
        # image batches sit on free GPUs, one each, none of them a video's anchored GPU
        assert len(set(got["image_gpu"])) == got["n_batches"]
        assert all(0 <= x < N and not ((want["used_mask"] >> x) & 1) for x in got["image_gpu"])


def test_cpp_laxity_and_errors():
    import paper_2604_04335_amd as da
    assert da.dit_sched_laxity(100.0, 40.0, 20, 2.5) == 10.0
    with pytest.raises(da.DitAttnError) as e:
        da.dit_sched_plan_round(0, [], [], 0.0, T_IMG)
    assert e.value.code == -2
    with pytest.raises(da.DitAttnError) as e:
        da.dit_sched_plan_round(4, [[(5, 0, 1.0, False)]], [], 0.0, T_IMG)      # more GPUs than the cluster has
    assert e.value.code == -2
    with pytest.raises(da.DitAttnError) as e:
        da.dit_sched_plan_round(2, [[(2, 0, 1.0, False)], [(1, 0, 1.0, False)]], [], 0.0, T_IMG)  # no hold, does not fit
    assert e.value.code == -3
    with pytest.raises(da.DitAttnError) as e:
        da.dit_sched_plan_round(4, [[(0, 0, 0.0, True), (2, 0b0111, 1.0, False)]], [], 0.0, T_IMG)  # mask names 3 GPUs, gpus says 2
    assert e.value.code == -2
    with pytest.raises(da.DitAttnError) as e:
        da.dit_sched_plan_round(4, [[da.SchedCandidate(1, 0, 1.0, 0, 7)]], [], 0.0, T_IMG)          # reserved must be 0
    assert e.value.code == -2
    r = da.dit_sched_plan_round(8, [], [], 0.0, T_IMG)                           # nothing to do
    assert r["recoverable"] == 0 and r["video_gpus"] == 0 and r["n_batches"] == 0


def test_cpp_large_round_is_fast():
    """N = 8 GPUs (the paper's cluster), 16 videos with 5 candidates each, 64 pending images: far below the 0.24-0.41 ms
    mean the paper reports for its solver (Table 6)."""
    import time
    g = np.random.Generator(np.random.PCG64(506))
    videos = [[orc.VideoCandidate(0, hold=True)] + [orc.VideoCandidate(p, 0, float(g.normal(1, 3))) for p in (1, 2, 4, 8)] for _ in range(16)]
    deadlines = list(g.uniform(0.5, 6.0, size=64))
    t0 = time.perf_counter()
    for _ in range(200):
        r = _solve_cpp(8, videos, deadlines)
    dt = (time.perf_counter() - t0) / 200
    want = orc.solve_round(8, videos, deadlines, 0.0, T_IMG, 4)
    assert r["choice"] == want["choice"] and r["recoverable"] == want["value"][0]
    assert dt < 2e-3, dt   # includes the Python marshalling of 80 candidates; the C++ part is a few microseconds
