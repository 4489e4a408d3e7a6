"""GPU parity of the log-sum-exp output, the merge of partial results and cross-attention against the CPU oracle.

Tolerances.  O: the attention bars of tests/gpu_util.py (max-abs 2e-2 and relative L2 1e-2).  lse: computed in fp32 as
ln 2 * (c*m + log2 l), where m is the row's lazily updated reference value and l the fp32 sum of the probabilities as
rounded to bf16 for the second contraction.  Every rounded term is within 2^-8 relative of its exact value and all are
positive, so lse is within ln(1 + 2^-8) = 3.9e-3 of the exact value (LSE_TOL below, which is also the contract stated
in include/dit_attn.h); the fp32 arithmetic around it adds ~1e-5.
Merged O: the parts are bf16 (2^-9 relative each) and the result is rounded once more, so the same attention bars apply.
"""
import os
import sys

import numpy as np
import pytest
import torch

import paper_2604_04335_amd as da
from dit_workloads import bf16_bits_to_f32, make_cross, make_custom, make_workload, sample_rows
from oracle import dit_attn_oracle as orc

sys.path.insert(0, os.path.dirname(__file__))
from gpu_util import MAX_ABS_TOL, REL_L2_TOL, assert_parity, to_bits, to_dev, widen  # noqa: E402

pytestmark = pytest.mark.gpu
# The row sum l is taken over the probabilities as rounded to bf16 for the second contraction (so that O / l is a convex
# combination whatever the rounding did).  bf16 keeps 8 significant bits, so each term is off by at most 2^-8 relative
# (half an ulp just above a power of two); all terms are positive, so l is off by at most 2^-8 relative and lse by at
# most ln(1 + 2^-8) = 3.9e-3 (reached only by a row that one key dominates; typical rows average it down to < 1e-3).
# The fp32 arithmetic around it adds ~1e-5.
LSE_TOL = 4.0e-3


@pytest.fixture(scope="module")
def ctx():
    da.load_library()
    c = da.dit_attn_create(0)
    yield c
    da.dit_attn_destroy(c)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _fwd_lse(ctx, w, kernel=None):
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    out = torch.empty_like(q)
    lse = torch.full((q.shape[0], w.n_heads), float("nan"), dtype=torch.float32, device="cuda")
    if kernel is not None:
        da.dit_attn_set_kernel(ctx, kernel)
    try:
        da.dit_attn_varlen_fwd_lse(ctx, q, k, v, w.cu_seqlens, w.n_heads, w.head_dim, w.scale, out, lse, _stream())
    finally:
        da.dit_attn_set_kernel(ctx, da.KERNEL_AUTO)
    torch.cuda.synchronize()
    return out, lse


@pytest.mark.parametrize("head_dim,kernel", [(64, None), (128, None), (128, da.KERNEL_PINGPONG), (64, da.KERNEL_PINGPONG)])
def test_lse_matches_oracle(ctx, head_dim, kernel):
    w = make_custom([300, 1, 129, 64, 777], 3, head_dim, seed=41)
    out, lse = _fwd_lse(ctx, w, kernel)
    ref_o, ref_l = orc.attention_varlen_lse(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert_parity(to_bits(out), ref_o, "O with lse requested")
    got = lse.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - ref_l)) <= LSE_TOL, np.max(np.abs(got - ref_l))
    # O does not depend on whether lse is asked for
    out2 = torch.empty_like(out)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    if kernel is not None:
        da.dit_attn_set_kernel(ctx, kernel)
    da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, w.n_heads, w.head_dim, w.scale, out2, _stream())
    da.dit_attn_set_kernel(ctx, da.KERNEL_AUTO)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))


def test_lse_negative_and_zero_scale_and_large_logits(ctx):
    w = make_custom([150, 70], 2, 64, seed=42)
    for scale in (-0.4, 0.0, 3.0):
        w.scale = scale
        _, lse = _fwd_lse(ctx, w)
        _, ref = orc.attention_varlen_lse(w.q, w.k, w.v, w.cu_seqlens, scale)
        tol = LSE_TOL * max(1.0, float(np.max(np.abs(ref))) / 60.0)
        assert np.max(np.abs(lse.cpu().numpy() - ref)) <= tol


def test_lse_full_size_sampled_rows(ctx):
    """mixed_varlen at full size, in the bench's launch configuration: one head of a stratified row sample."""
    w = make_workload("mixed_varlen")
    _, lse = _fwd_lse(ctx, w)
    got = lse.cpu().numpy()
    cu, h = w.cu_seqlens, 3
    for r in sample_rows(cu, seed=5, block=2048):
        i = int(np.searchsorted(cu, r, side="right") - 1)
        ref = orc.logsumexp_scores(orc.widen_bf16(w.q[r:r + 1, h]), orc.widen_bf16(w.k[cu[i]:cu[i + 1], h]), w.scale)
        assert abs(got[r, h] - ref[0]) <= LSE_TOL


@pytest.mark.parametrize("bounds", [(0, 700, 1300), (0, 64, 65, 1000, 1300), (0, 1300)])
def test_split_keys_then_merge_equals_full_attention(ctx, bounds):
    """What a ring step does: the same queries against blocks of keys, one call each, then one merge."""
    L, H, D = 1300, 3, 128
    w = make_custom([L], H, D, seed=43)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    outs, lses = [], []
    for a, b in zip(bounds[:-1], bounds[1:]):
        o = torch.empty_like(q)
        l = torch.empty((L, H), dtype=torch.float32, device="cuda")
        da.dit_attn_cross_varlen_fwd(ctx, q, k[a:b].contiguous(), v[a:b].contiguous(), [0, L], [0, b - a], H, D, w.scale, o, l, _stream())
        outs.append(o); lses.append(l)
    merged = torch.empty_like(q)
    lse = torch.empty((L, H), dtype=torch.float32, device="cuda")
    da.dit_attn_merge(ctx, outs, lses, L, H, D, merged, lse, _stream())
    torch.cuda.synchronize()
    ref_o, ref_l = orc.attention_varlen_lse(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert_parity(to_bits(merged), ref_o, f"merge of {len(outs)} key blocks")
    assert np.max(np.abs(lse.cpu().numpy() - ref_l)) <= LSE_TOL
    # merging into one of the parts gives the same bits
    da.dit_attn_merge(ctx, outs, lses, L, H, D, outs[0], None, _stream())
    torch.cuda.synchronize()
    assert torch.equal(outs[0].view(torch.int16), merged.view(torch.int16))


@pytest.mark.parametrize("n_parts,head_dim", [(1, 64), (2, 128), (5, 64), (8, 128)])
def test_merge_kernel_against_oracle_on_random_parts(ctx, n_parts, head_dim):
    T, H = 517, 3
    g = np.random.Generator(np.random.PCG64(44 + n_parts))
    from dit_workloads import f32_to_bf16_bits
    o_bits = [f32_to_bf16_bits(g.standard_normal((T, H, head_dim)).astype(np.float32)) for _ in range(n_parts)]
    lse = [(4.0 * g.standard_normal((T, H))).astype(np.float32) for _ in range(n_parts)]
    if n_parts >= 2:
        lse[1][5] = -np.inf                      # a part without keys in one row
        o_bits[1][5] = 0x7FC0                    # ... whose O is NaN: must not leak
        for p in range(n_parts):
            lse[p][9, 1] = -np.inf               # a (row, head) with no keys at all
    outs = [to_dev(x) for x in o_bits]
    lses = [torch.from_numpy(x).cuda() for x in lse]
    out = torch.empty_like(outs[0])
    lo = torch.empty((T, H), dtype=torch.float32, device="cuda")
    da.dit_attn_merge(ctx, outs, lses, T, H, head_dim, out, lo, _stream())
    torch.cuda.synchronize()
    o64 = np.stack([np.where(np.isfinite(widen(b)), widen(b), 0.0) for b in o_bits])
    ref_o, ref_l = orc.merge_partials(o64, np.stack(lse).astype(np.float64))
    got = widen(to_bits(out))
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - ref_o)) <= MAX_ABS_TOL and np.sqrt(np.sum((got - ref_o) ** 2) / np.sum(ref_o ** 2)) <= REL_L2_TOL
    gl = lo.cpu().numpy().astype(np.float64)
    fin = np.isfinite(ref_l)
    assert np.array_equal(np.isfinite(gl), fin) and np.all(gl[~fin] == -np.inf)
    assert np.max(np.abs(gl[fin] - ref_l[fin])) <= LSE_TOL
    if n_parts >= 2:
        assert np.all(got[9, 1] == 0.0)


def test_merge_beyond_four_gib(ctx):
    """Two parts of 2.3e9 elements (4.6 GB) each: the merge kernel's chunk and byte offsets pass 2^32.  Device-side
    seeded parts; the oracle merges sampled rows, among them the rows on either side of the 4 GiB line and the last."""
    T, H, D = 16500, 1100, 128
    assert T * H * D * 2 > 2 ** 32
    print(f"merge beyond 4 GiB: T={T} H={H} D={D}", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(505)
    outs = [torch.empty((T, H, D), dtype=torch.bfloat16, device="cuda").normal_(generator=gen) for _ in range(2)]
    lses = [torch.empty((T, H), dtype=torch.float32, device="cuda").normal_(std=3.0, generator=gen) for _ in range(2)]
    out = torch.empty_like(outs[0])
    lo = torch.empty((T, H), dtype=torch.float32, device="cuda")
    da.dit_attn_merge(ctx, outs, lses, T, H, D, out, lo, _stream())
    torch.cuda.synchronize()
    line = 2 ** 32 // (H * D * 2)
    rows = np.unique(np.concatenate([np.linspace(0, T - 1, 24).astype(int), [line - 1, line, line + 1, T - 2]]))
    rt = torch.from_numpy(rows).cuda()
    o64 = np.stack([widen(to_bits(o[rt])) for o in outs])
    l64 = np.stack([l[rt].cpu().numpy().astype(np.float64) for l in lses])
    ref_o, ref_l = orc.merge_partials(o64, l64)
    got = widen(to_bits(out[rt]))
    assert np.all(np.isfinite(got))
    assert np.max(np.abs(got - ref_o)) <= MAX_ABS_TOL and np.sqrt(np.sum((got - ref_o) ** 2) / np.sum(ref_o ** 2)) <= REL_L2_TOL
    assert np.max(np.abs(lo[rt].cpu().numpy().astype(np.float64) - ref_l)) <= LSE_TOL


@pytest.mark.parametrize("q_lens,k_lens,H,D", [
    ([300, 5, 129], [77, 226, 1], 3, 128),          # ragged, keys shorter than one tile
    ([1000, 0, 64, 200], [226, 50, 0, 512], 2, 64),  # a sequence without queries, one without keys
    ([4352, 4352], [226, 512], 4, 128),              # latent queries against text keys at the image-step length
])
def test_cross_attention_matches_oracle(ctx, q_lens, k_lens, H, D):
    w = make_cross(q_lens, k_lens, H, D, seed=45)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    SENT = 0x7FC1
    out = torch.full(q.shape, SENT, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    lse = torch.full((q.shape[0], H), float("nan"), dtype=torch.float32, device="cuda")
    da.dit_attn_cross_varlen_fwd(ctx, q, k, v, w.cu_seqlens_q, w.cu_seqlens_k, H, D, w.scale, out, lse, _stream())
    torch.cuda.synchronize()
    ref_o, ref_l = orc.attention_cross_varlen(w.q, w.k, w.v, w.cu_seqlens_q, w.cu_seqlens_k, w.scale)
    assert_parity(to_bits(out), ref_o, "cross-attention")
    gl = lse.cpu().numpy().astype(np.float64)
    fin = np.isfinite(ref_l)
    assert np.array_equal(np.isfinite(gl), fin) and np.all(gl[~fin] == -np.inf)
    assert np.max(np.abs(gl[fin] - ref_l[fin])) <= LSE_TOL
    # rows of a sequence without keys are exactly zero
    got = to_bits(out)
    for i in range(len(q_lens)):
        if k_lens[i] == 0:
            assert np.all(got[w.cu_seqlens_q[i]:w.cu_seqlens_q[i + 1]] == 0)
    # lse is optional, and the same boundaries for q and k reproduce self-attention bit for bit
    out2 = torch.empty_like(out)
    da.dit_attn_cross_varlen_fwd(ctx, q, k, v, w.cu_seqlens_q, w.cu_seqlens_k, H, D, w.scale, out2, None, _stream())
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))


def test_cross_with_equal_boundaries_is_self_attention(ctx):
    w = make_custom([500, 33], 2, 128, seed=46)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    a, b = torch.empty_like(q), torch.empty_like(q)
    da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, 2, 128, w.scale, a, _stream())
    da.dit_attn_cross_varlen_fwd(ctx, q, k, v, w.cu_seqlens, w.cu_seqlens, 2, 128, w.scale, b, None, _stream())
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_new_entry_points_reject_bad_arguments(ctx):
    w = make_custom([100], 2, 64, seed=47)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    out = torch.empty_like(q)
    lse = torch.empty((100, 2), dtype=torch.float32, device="cuda")
    with pytest.raises(da.DitAttnError) as e:
        da.dit_attn_varlen_fwd_lse(ctx, q, k, v, w.cu_seqlens, 2, 64, w.scale, out, None, _stream())
    assert e.value.code == -1
    with pytest.raises(da.DitAttnError) as e:
        da.dit_attn_cross_varlen_fwd(ctx, q, k, v, w.cu_seqlens, None, 2, 64, w.scale, out, None, _stream())
    assert e.value.code == -1
    with pytest.raises(da.DitAttnError) as e:
        da.dit_attn_cross_varlen_fwd(ctx, q, k, v, w.cu_seqlens, [5, 100], 2, 64, w.scale, out, None, _stream())
    assert e.value.code == -3
    with pytest.raises(da.DitAttnError) as e:
        da.dit_attn_merge(ctx, [out] * 9, [lse] * 9, 100, 2, 64, out, None, _stream())
    assert e.value.code == -10
    with pytest.raises(da.DitAttnError) as e:
        da.dit_attn_merge(ctx, [out], [lse], 100, 2, 96, out, None, _stream())
    assert e.value.code == -2
    da.dit_attn_merge(ctx, [out], [lse], 0, 2, 64, out, None, _stream())  # nothing to do
    torch.cuda.synchronize()


# ---------------------------------------------------------------- split-KV

@pytest.mark.parametrize("lens,H,D,max_splits", [
    ([4096], 4, 64, 8),             # 128 items of 128 rows -> 4 chunks of 1024 keys
    ([6200, 6147, 10000], 1, 128, 8),  # ragged: chunks of whole tiles, short last chunks, sequences with different chunk counts
    ([6145], 1, 128, 3),
    ([16000], 1, 64, 2),            # two chunks pay only for long sequences
])
def test_split_kv_matches_oracle_and_unsplit_result(ctx, lens, H, D, max_splits):
    w = make_custom(lens, H, D, seed=48)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    base = torch.empty_like(q)
    da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, H, D, w.scale, base, _stream())
    SENT = 0x7FC1
    buf = torch.full((q.shape[0] + 128, H, D), SENT, dtype=torch.int16, device="cuda")
    out = buf[64:64 + q.shape[0]].view(torch.bfloat16)
    lse = torch.full((q.shape[0], H), float("nan"), dtype=torch.float32, device="cuda")
    da.dit_attn_set_split_kv(ctx, max_splits)
    try:
        da.dit_attn_varlen_fwd_lse(ctx, q, k, v, w.cu_seqlens, H, D, w.scale, out, lse, _stream())
        out2 = torch.empty_like(q)
        da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, H, D, w.scale, out2, _stream())   # same plan from the cache, no lse
    finally:
        da.dit_attn_set_split_kv(ctx, 1)
    torch.cuda.synchronize()
    assert bool((buf[:64] == SENT).all()) and bool((buf[64 + q.shape[0]:] == SENT).all())
    ref_o, ref_l = orc.attention_varlen_lse(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert_parity(to_bits(out), ref_o, "split-KV")
    assert np.max(np.abs(lse.cpu().numpy() - ref_l)) <= LSE_TOL
    assert torch.equal(out.view(torch.int16), out2.view(torch.int16))
    # against the unsplit kernel: the same result up to the rounding of different summation orders
    d = widen(to_bits(out)) - widen(to_bits(base))
    assert np.max(np.abs(d)) <= MAX_ABS_TOL
    assert not torch.equal(out.view(torch.int16), base.view(torch.int16))   # the split path did run
    # after switching it off again the unsplit bits are back
    again = torch.empty_like(q)
    da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, H, D, w.scale, again, _stream())
    torch.cuda.synchronize()
    assert torch.equal(again.view(torch.int16), base.view(torch.int16))


def test_split_kv_leaves_large_packs_alone_and_rejects_bad_counts(ctx):
    w = make_custom([8192, 300], 8, 64, seed=49)   # enough items: no split, bits unchanged
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    a, b = torch.empty_like(q), torch.empty_like(q)
    da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, 8, 64, w.scale, a, _stream())
    da.dit_attn_set_split_kv(ctx, 8)
    try:
        da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, 8, 64, w.scale, b, _stream())
    finally:
        da.dit_attn_set_split_kv(ctx, 1)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    for bad in (0, 9):
        with pytest.raises(da.DitAttnError) as e:
            da.dit_attn_set_split_kv(ctx, bad)
        assert e.value.code == -10


def test_split_kv_cross_attention(ctx):
    w = make_cross([600, 100], [5000, 3300], 2, 128, seed=50)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    out = torch.empty_like(q)
    da.dit_attn_set_split_kv(ctx, 4)
    try:
        da.dit_attn_cross_varlen_fwd(ctx, q, k, v, w.cu_seqlens_q, w.cu_seqlens_k, 2, 128, w.scale, out, None, _stream())
    finally:
        da.dit_attn_set_split_kv(ctx, 1)
    torch.cuda.synchronize()
    ref_o, _ = orc.attention_cross_varlen(w.q, w.k, w.v, w.cu_seqlens_q, w.cu_seqlens_k, w.scale)
    assert_parity(to_bits(out), ref_o, "split-KV cross-attention")
