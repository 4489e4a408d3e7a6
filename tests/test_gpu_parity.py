"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same seeded inputs.

Bar (from the benchmark definition): max-abs error <= 2e-2 and relative L2 error <= 1e-2
(bf16 inputs, fp32 accumulation); which rows are written, and which keys feed them, bit-exact.
"""
import os
import sys

import numpy as np
import pytest
import torch

import paper_2604_04335_amd as da
from dit_workloads import bf16_bits_to_f32, f32_to_bf16_bits, make_custom, make_workload, sample_rows
from oracle import dit_attn_oracle as orc

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from gpu_util import MAX_ABS_TOL, REL_L2_TOL, Runner, assert_parity, errors, to_bits, to_dev, widen  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def runner():
    r = Runner()
    yield r
    r.close()


def _say(msg):
    print(msg, flush=True)


# ------------------------------------------------------------------ element-by-element on small packs

SMALL = [
    # (lens, H, D, seed)  -- several tiles (128-row query tiles, 64-key tiles) and ragged tails
    ([300, 77, 129, 1, 0, 64, 200], 3, 128, 1),
    ([1, 2, 3, 31, 32, 33, 63, 64, 65, 127, 128, 129], 2, 128, 2),
    ([513], 5, 64, 3),
    ([96, 640, 0, 17], 4, 64, 4),
    ([1000], 1, 128, 5),
    ([255, 257], 40, 128, 6),
]


@pytest.mark.parametrize("lens,H,D,seed", SMALL, ids=[f"case{i}" for i in range(len(SMALL))])
def test_small_packs_full_oracle(runner, lens, H, D, seed):
    _say(f"small pack lens={lens} H={H} D={D} seed={seed}")
    w = make_custom(lens, H, D, seed)
    got = runner.run(w)
    ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert_parity(got, ref, f"lens={lens}")
    # per sequence as well, so that one short sequence cannot hide behind a long one
    cu = w.cu_seqlens
    for i in range(len(lens)):
        s, e = int(cu[i]), int(cu[i + 1])
        if e > s:
            assert_parity(got[s:e], ref[s:e], f"seq {i} of lens={lens}")


def test_tiny_image_full_oracle(runner):
    _say("config tiny_image, full oracle")
    w = make_workload("tiny_image")
    got = runner.run(w)
    ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    max_abs, rel = assert_parity(got, ref, "tiny_image")
    _say(f"tiny_image max_abs={max_abs:.3e} rel_l2={rel:.3e}")


# ------------------------------------------------------------------ the four large configurations, sampled rows

# (name, kernel): None = the kernel the library picks for the pack (the benchmark's launch configuration); the second
# sp_shard entry forces the 128-row kernel, so that its tail path (76112 = 1189 * 64 + 16) is checked at full length too.
LARGE = [("t2i_batch", None), ("t2v_single", None), ("mixed_varlen", None), ("sp_shard", None), ("sp_shard", "KERNEL_128")]


@pytest.mark.parametrize("name,kernel", LARGE, ids=[n + ("" if k is None else "-" + k) for n, k in LARGE])
def test_full_size_configs_sampled_rows(runner, name, kernel):
    """Full-size call in the benchmark's launch configuration; the oracle checks a stratified row sample: one row in
    every 64-row block of every sequence (so every wavefront of every query tile is hit) plus the rows around the
    sequence ends and tile boundaries, on all heads.  Every sampled row uses all keys of its sequence, so each checked
    row is exact."""
    _say(f"config {name}: generating")
    w = make_workload(name)
    rows = sample_rows(w.cu_seqlens, seed=w.seed, block=64)
    _say(f"config {name}: T={w.total_tokens} H={w.n_heads} rows checked={len(rows)}; running GPU")
    got = runner.run(w, kernel=None if kernel is None else getattr(da, kernel))
    _say(f"config {name}: running oracle on {len(rows)} rows")
    ref = orc.attention_varlen_rows(w.q, w.k, w.v, w.cu_seqlens, w.scale, rows)
    max_abs, rel = assert_parity(got[rows], ref, name)
    _say(f"config {name}: max_abs={max_abs:.3e} rel_l2={rel:.3e} max|ref|={np.max(np.abs(ref)):.3e}")
    # per sequence
    cu = w.cu_seqlens
    for i in range(len(cu) - 1):
        sel = np.nonzero((rows >= cu[i]) & (rows < cu[i + 1]))[0]
        if len(sel):
            assert_parity(got[rows[sel]], ref[sel], f"{name} seq {i}")
    # property that holds at any size: every output lies in the convex hull of its sequence's values
    vf = bf16_bits_to_f32(w.v)
    gf = bf16_bits_to_f32(got)
    for i in range(len(cu) - 1):
        s, e = int(cu[i]), int(cu[i + 1])
        if e > s:
            lo, hi = vf[s:e].min(axis=0), vf[s:e].max(axis=0)
            assert np.all(gf[s:e] >= lo[None] - 1e-6) and np.all(gf[s:e] <= hi[None] + 1e-6)


def _bf16_ulp(x):
    """Spacing of bf16 values at |x| (8 significant bits): 2^(floor(log2 |x|) - 7)."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def test_t2i_batch_every_output_against_the_oracle(runner):
    """Configuration 2 (four batched 1024x1024 image requests, per-head value scale) against the oracle on EVERY
    output.  Its outputs reach |O| = 4..10, where half a bf16 output ulp is already 1.6e-2 (|O| >= 4) and 3.1e-2
    (|O| >= 8), so the max-abs bar of 2e-2 cannot hold for a bf16 result with |O| >= 8 however it is computed.
    Asserted: relative L2 <= 1e-2 over everything and per sequence; max-abs <= 2e-2 on every element with |ref| < 8;
    for the remaining elements (counted, a handful) the error is within output rounding, half a bf16 ulp of the
    reference plus the 2e-3 that the fp32 arithmetic before the rounding may contribute."""
    w = make_workload("t2i_batch")
    _say(f"t2i_batch: T={w.total_tokens} H={w.n_heads}; running GPU")
    got = widen(runner.run(w))
    _say("t2i_batch: full oracle (0.93 TFLOP fp64)")
    ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert np.all(np.isfinite(got))
    err = np.abs(got - ref)
    max_abs, rel = errors(got, ref)
    big = np.abs(ref) >= 8.0
    _say(f"t2i_batch: rel_l2={rel:.3e} max_abs={max_abs:.3e} max|ref|={np.max(np.abs(ref)):.2f} "
         f"elements with |ref|>=8: {int(big.sum())}, of them over 2e-2: {int((err[big] > MAX_ABS_TOL).sum())}, "
         f"elements over 1.8e-2: {int((err > 1.8e-2).sum())}")
    assert rel <= REL_L2_TOL
    cu = w.cu_seqlens
    for i in range(len(cu) - 1):
        s, e = int(cu[i]), int(cu[i + 1])
        assert errors(got[s:e], ref[s:e])[1] <= REL_L2_TOL, f"sequence {i}"
    assert np.max(err[~big], initial=0.0) <= MAX_ABS_TOL
    assert int(big.sum()) <= 64, "the exception must stay a handful of elements"
    assert np.all(err[big] <= 0.5 * _bf16_ulp(ref[big]) + 2e-3)


def test_tensors_beyond_four_gib(runner):
    """Maximum sizes: 2.3e9 elements and 4.6 GB per tensor, so element indices pass 2^31 and byte offsets pass 2^32
    inside the pack.  Three heads (first, middle, last) hold the seeded generator's data and are checked against the
    oracle on sampled rows of every sequence, the last of which lies wholly above 4 GiB; the other heads hold
    device-side seeded noise and are checked for the convex-hull property on a stretch of rows."""
    lens, H, D = [9000, 6700, 800], 1100, 128
    heads = [0, 547, H - 1]
    w = make_custom(lens, len(heads), D, seed=77)
    cu, T = w.cu_seqlens, int(w.cu_seqlens[-1])
    assert T * H * D > 2 ** 31 and int(cu[2]) * H * D * 2 > 2 ** 32
    _say(f"large tensors: T={T} H={H} D={D}, {T * H * D * 2 / 2**30:.2f} GiB each; filling")
    gen = torch.Generator(device="cuda").manual_seed(77)
    dev = []
    for bits in (w.q, w.k, w.v):
        t = torch.empty((T, H, D), dtype=torch.bfloat16, device="cuda")
        t.normal_(generator=gen)
        t[:, heads, :] = to_dev(bits)
        dev.append(t)
    _say("large tensors: running GPU")
    out = runner.run_dev(dev[0], dev[1], dev[2], cu, H, D, w.scale)
    rows = sample_rows(cu, seed=77, block=64, max_rows=240)
    got = to_bits(out[torch.from_numpy(rows).cuda()][:, heads, :])
    _say(f"large tensors: oracle on {len(rows)} rows x {len(heads)} heads")
    ref = orc.attention_varlen_rows(w.q, w.k, w.v, cu, w.scale, rows)
    max_abs, rel = assert_parity(got, ref, "large tensors")
    _say(f"large tensors: max_abs={max_abs:.3e} rel_l2={rel:.3e}")
    for i in range(len(lens)):
        sel = np.nonzero((rows >= cu[i]) & (rows < cu[i + 1]))[0]
        assert_parity(got[sel], ref[sel], f"large tensors seq {i}")
    # every head of the last sequence (all of it above 4 GiB): outputs inside the hull of that sequence's values
    s, e = int(cu[2]), int(cu[3])
    vf, of = dev[2][s:e].float(), out[s:e].float()
    assert bool(torch.isfinite(of).all())
    lo, hi = vf.amin(dim=0, keepdim=True), vf.amax(dim=0, keepdim=True)
    assert bool(((of >= lo - 1e-6) & (of <= hi + 1e-6)).all())


def test_largest_head_count(runner):
    """65535 heads, the most the work-list's 16-bit head field and the argument check allow: first, middle and last
    head against the oracle (seeded generator data there, device-side seeded noise elsewhere)."""
    lens, H, D = [70, 3, 130], 65535, 64
    heads = [0, 32768, H - 1]
    w = make_custom(lens, len(heads), D, seed=78)
    cu, T = w.cu_seqlens, int(w.cu_seqlens[-1])
    _say(f"largest head count: T={T} H={H} D={D}")
    gen = torch.Generator(device="cuda").manual_seed(78)
    dev = []
    for bits in (w.q, w.k, w.v):
        t = torch.empty((T, H, D), dtype=torch.bfloat16, device="cuda").normal_(generator=gen)
        t[:, heads, :] = to_dev(bits)
        dev.append(t)
    out = runner.run_dev(dev[0], dev[1], dev[2], cu, H, D, w.scale)
    ref = orc.attention_varlen(w.q, w.k, w.v, cu, w.scale)
    assert_parity(to_bits(out[:, heads, :]), ref, "largest head count")
    assert bool(torch.isfinite(out.float()).all())


# ------------------------------------------------------------------ invariants, on the GPU

def test_one_token_sequences_return_v_bits(runner):
    w = make_custom([1, 130, 1, 1], 3, 128, seed=20)
    got = runner.run(w)
    for r in (0, 131, 132):
        assert np.array_equal(got[r], w.v[r])


def test_pack_isolation_bitwise(runner):
    """A sequence's output bits do not depend on what it is packed with."""
    w = make_custom([200, 333, 64], 2, 128, seed=21)
    full = runner.run(w)
    cu = w.cu_seqlens
    for i in range(3):
        s, e = int(cu[i]), int(cu[i + 1])
        alone = make_custom([e - s], 2, 128, seed=0)
        alone.q, alone.k, alone.v = w.q[s:e].copy(), w.k[s:e].copy(), w.v[s:e].copy()
        assert np.array_equal(runner.run(alone), full[s:e]), f"sequence {i}"
    # perturb the middle sequence: neighbours unchanged bit for bit
    w2 = make_custom([200, 333, 64], 2, 128, seed=21)
    w2.k[200:533] = f32_to_bf16_bits(bf16_bits_to_f32(w2.k[200:533]) + 1.0)
    w2.v[200:533] = f32_to_bf16_bits(bf16_bits_to_f32(w2.v[200:533]) * 2.0)
    pert = runner.run(w2)
    assert np.array_equal(pert[:200], full[:200]) and np.array_equal(pert[533:], full[533:])
    assert not np.array_equal(pert[200:533], full[200:533])


def test_both_kernels_give_the_same_bits(runner):
    """A large pack runs the 256-row ping-pong kernel, a small one the 128-row kernel: same bits per sequence.
    (35 query tiles x 12 heads = 420 items of 256 rows: 1.64 per compute unit, so the ping-pong kernel is chosen.)"""
    w = make_custom([8192, 300, 77], 12, 64, seed=28)
    items, bm = da.dit_attn_plan(w.cu_seqlens, 12, 64)
    assert bm == 256
    full = runner.run(w)
    assert da.dit_attn_last_launch_kernel(runner.ctx) == da.KERNEL_PINGPONG
    for s, e in ((8192, 8492), (8492, 8569)):
        alone = make_custom([e - s], 12, 64, seed=0)
        alone.q, alone.k, alone.v = w.q[s:e].copy(), w.k[s:e].copy(), w.v[s:e].copy()
        assert da.dit_attn_plan(alone.cu_seqlens, 12, 64)[1] == 128
        assert np.array_equal(runner.run(alone), full[s:e])
    rows = sample_rows(w.cu_seqlens, seed=3, block=256)
    ref = orc.attention_varlen_rows(w.q, w.k, w.v, w.cu_seqlens, w.scale, rows)
    assert_parity(full[rows], ref, "ping-pong kernel, head_dim 64")


def test_launch_clock_sample(runner):
    """The clock sample of the last launch: a plausible shader clock (MI355X runs at 2.4 GHz at most) and a duration."""
    w = make_custom([2048], 8, 128, seed=33)
    runner.run(w)
    mhz, ms = da.dit_attn_last_launch_clock(runner.ctx)
    assert 300.0 < mhz < 2600.0, mhz
    assert 0.0 < ms < 1000.0, ms
    # 8 x 8 = 64 items of 256 rows: fewer than compute units, so the 128-row kernel ran; a forced kernel is reported too
    assert da.dit_attn_last_launch_kernel(runner.ctx) == da.KERNEL_128
    runner.run(w, kernel=da.KERNEL_PINGPONG)
    assert da.dit_attn_last_launch_kernel(runner.ctx) == da.KERNEL_PINGPONG


def test_head_subset_equals_heads_of_wider_run(runner):
    """The head-split shard view: running heads [10, 20) alone equals those heads of a 40-head run."""
    w = make_custom([700], 40, 128, seed=22)
    full = runner.run(w)
    sub = make_custom([700], 10, 128, seed=0)
    sub.q, sub.k, sub.v = (np.ascontiguousarray(x[:, 10:20]) for x in (w.q, w.k, w.v))
    assert np.array_equal(runner.run(sub), full[:, 10:20])


def test_scale_zero_and_negative_scale(runner):
    w = make_custom([150, 70], 2, 64, seed=23)
    got0 = widen(runner.run(w, scale=0.0))
    vf = widen(w.v)
    for s, e in ((0, 150), (150, 220)):
        mean = vf[s:e].mean(axis=0)
        assert np.max(np.abs(got0[s:e] - mean[None])) <= 4e-3  # bf16 rounding of the output
    neg = runner.run(w, scale=-0.2)
    ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, -0.2)
    assert_parity(neg, ref, "negative scale")


def test_identical_keys_give_mean_of_v(runner):
    w = make_custom([257], 2, 128, seed=24)
    w.k[:] = w.k[0:1]
    got = widen(runner.run(w))
    mean = widen(w.v).mean(axis=0)
    assert np.max(np.abs(got - mean[None])) <= 4e-3


def test_key_permutation_invariance(runner):
    w = make_custom([389], 2, 128, seed=25)
    base = widen(runner.run(w))
    perm = np.random.Generator(np.random.PCG64(7)).permutation(389)
    w.k, w.v = np.ascontiguousarray(w.k[perm]), np.ascontiguousarray(w.v[perm])
    got = widen(runner.run(w))
    max_abs, rel = errors(got, base)
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL


def test_peaky_softmax_large_logits(runner):
    """Logit standard deviation ~16: exercises the running-maximum path."""
    w = make_custom([300], 2, 128, seed=26, scale=16.0 / np.sqrt(128.0))
    got = runner.run(w)
    ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert_parity(got, ref, "peaky")


def test_increasing_logits_force_rescaling(runner):
    """Keys ordered so that the row maximum grows tile after tile."""
    w = make_custom([640], 1, 128, seed=27, scale=1.0)
    qf = np.ones((640, 1, 128), dtype=np.float32) * 0.25
    kf = np.zeros((640, 1, 128), dtype=np.float32)
    kf[:, 0, :] = (np.arange(640, dtype=np.float32) / 640.0)[:, None]  # logit j = 32 * j / 640
    w.q, w.k = f32_to_bf16_bits(qf), f32_to_bf16_bits(kf)
    got = runner.run(w)
    ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert_parity(got, ref, "increasing logits")


def test_lazy_reference_staircase(runner):
    """Logits that are constant per 64-key tile and step from tile to tile by just under the rescale threshold (2^8 in
    the base-2 exponent: the reference stays), just over it (it moves), by a huge amount, and down again; every
    kernel, against the oracle and against each other bit for bit."""
    steps_log2 = [0.0, 7.5, 7.9, 8.5, 0.3, 200.0, -150.0, 7.99, 8.01, -30.0]  # increments per tile
    level = np.cumsum(steps_log2) * np.log(2.0)  # natural-log logit of each tile
    n = 64 * len(level)
    for heads, reps in ((1, 1), (3, 3)):
        w = make_custom([n] * reps, heads, 128, seed=29, scale=1.0)
        qf = np.zeros((n * reps, heads, 128), dtype=np.float32)
        qf[:, :, 0] = 1.0  # logit of (query, key) = K[key, 0]
        kf = np.zeros((n * reps, heads, 128), dtype=np.float32)
        kf[:, :, 0] = np.tile(np.repeat(level, 64), reps)[:, None]
        w.q, w.k = f32_to_bf16_bits(qf), f32_to_bf16_bits(kf)
        ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
        outs = [runner.run(w, kernel=kern) for kern in (da.KERNEL_128, da.KERNEL_PINGPONG)]
        for got in outs:
            assert_parity(got, ref, "staircase logits")
        assert np.array_equal(outs[0], outs[1])


# ------------------------------------------------------------------ call mechanics

def test_deterministic_and_plan_cache(runner):
    a = make_custom([300, 200], 2, 128, seed=30)
    b = make_custom([123], 2, 128, seed=31)
    ra1 = runner.run(a)
    rb1 = runner.run(b)
    ra2 = runner.run(a)
    rb2 = runner.run(b)
    assert np.array_equal(ra1, ra2) and np.array_equal(rb1, rb2)


def test_many_packs_evict_cached_plans(runner):
    ref = None
    for i in range(40):  # more distinct packs than the cache holds
        w = make_custom([64 + i, 10], 1, 64, seed=32)
        got = runner.run(w)
        if i == 0:
            ref = got
    w = make_custom([64, 10], 1, 64, seed=32)
    assert np.array_equal(runner.run(w), ref)


def test_non_default_stream(runner):
    w = make_custom([400], 2, 128, seed=33)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    torch.cuda.synchronize()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        out = runner.run_dev(q, k, v, w.cu_seqlens, 2, 128, w.scale, stream=st.cuda_stream)
    ref = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert_parity(to_bits(out), ref, "stream")


@pytest.mark.parametrize("lens,heads", [([300, 70], 3), ([4096], 16)], ids=["128-row kernel", "ping-pong kernel"])
def test_graph_capture_and_replay(runner, lens, heads):
    """A forward call captured into a HIP graph (after one eager call has cached the pack's work-list: the first call
    allocates and copies, which a capture cannot record) and replayed several times, with eager work and
    synchronisations between the replays: every replay reproduces the eager bits.  The work counters that the kernel
    uses are cleared by its last workgroup, not by the host, so a replay finds them as a launch leaves them."""
    w = make_custom(lens, heads, 128, seed=35)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    eager = torch.empty_like(q)
    da.dit_attn_varlen_fwd(runner.ctx, q, k, v, w.cu_seqlens, heads, 128, w.scale, eager, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    out = torch.zeros_like(q)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        da.dit_attn_varlen_fwd(runner.ctx, q, k, v, w.cu_seqlens, heads, 128, w.scale, out, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for i in range(4):
        out.zero_()
        # the program's own eager work between replays: another pack through the same context, and a reduction
        other = runner.run(make_custom([200 + 17 * i], 2, 128, seed=36 + i))
        assert other.shape[0] == 200 + 17 * i
        _ = float(q.float().sum().item())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), f"replay {i}"
    rows = sample_rows(w.cu_seqlens, seed=5, block=16, max_rows=64)
    ref = orc.attention_varlen_rows(w.q, w.k, w.v, w.cu_seqlens, w.scale, rows)
    assert_parity(to_bits(out)[rows], ref, "graph replay")


def test_captured_pack_survives_plan_cache_eviction(runner):
    """A captured launch keeps reading its pack's device work-list on every replay, so that pack is pinned in the plan
    cache: after more distinct packs than the cache holds have gone through the context, a replay still reproduces the
    eager bits.  A call under capture for a pack the context has never seen is refused (it would have to allocate and
    copy), and the capture can go on without it."""
    w = make_custom([500, 130], 2, 128, seed=40)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    stream = lambda: torch.cuda.current_stream().cuda_stream
    eager = torch.empty_like(q)
    da.dit_attn_varlen_fwd(runner.ctx, q, k, v, w.cu_seqlens, 2, 128, w.scale, eager, stream())
    torch.cuda.synchronize()
    out = torch.zeros_like(q)
    unseen = np.array([0, 499, 630], dtype=np.int32)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        with pytest.raises(da.DitAttnError) as ei:
            da.dit_attn_varlen_fwd(runner.ctx, q, k, v, unseen, 2, 128, w.scale, out, stream())
        assert ei.value.code == -12
        da.dit_attn_varlen_fwd(runner.ctx, q, k, v, w.cu_seqlens, 2, 128, w.scale, out, stream())
    torch.cuda.synchronize()
    for i in range(40):  # more distinct packs than the cache holds: every unpinned plan is evicted at least once
        runner.run(make_custom([70 + i, 9], 1, 64, seed=41))
    out.zero_()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), eager.view(torch.int16))


def test_empty_inputs_launch_nothing(runner):
    da.dit_attn_varlen_fwd(runner.ctx, 0, 0, 0, np.array([0], dtype=np.int32), 2, 128, 1.0, 0, None)
    da.dit_attn_varlen_fwd(runner.ctx, 0, 0, 0, np.array([0, 0, 0], dtype=np.int32), 2, 128, 1.0, 0, None)


def test_argument_errors_leave_out_untouched(runner):
    w = make_custom([100], 2, 128, seed=34)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    out = torch.full((100, 2, 128), 0x7FC1, dtype=torch.int16, device="cuda")
    cu = w.cu_seqlens

    def expect(code, **kw):
        args = dict(q=q, k=k, v=v, cu=cu, H=2, D=128, scale=1.0, out=out)
        args.update(kw)
        with pytest.raises(da.DitAttnError) as ei:
            da.dit_attn_varlen_fwd(runner.ctx, args["q"], args["k"], args["v"], args["cu"], args["H"], args["D"],
                                   args["scale"], args["out"], None)
        assert ei.value.code == code, (code, ei.value)

    expect(-2, D=96)
    expect(-6, H=0)
    expect(-3, cu=np.array([1, 100], dtype=np.int32))
    expect(-3, cu=np.array([0, 100, 50], dtype=np.int32))
    expect(-5, scale=float("nan"))
    expect(-5, scale=float("inf"))
    expect(-1, q=0)
    expect(-1, out=0)
    expect(-7, k=k.data_ptr() + 2)
    torch.cuda.synchronize()
    assert bool((out == 0x7FC1).all())
    assert "aligned" in da.dit_attn_last_error(runner.ctx)
    # and the context still works afterwards
    got = runner.run(w)
    assert_parity(got, orc.attention_varlen(w.q, w.k, w.v, cu, w.scale), "after errors")
