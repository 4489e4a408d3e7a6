"""Pins for the CPU oracle: it is checked against things other than itself.

Each test is chosen so that a plausible slip in the oracle (dropped scale,
missing max-subtraction, normalising over the wrong axis, transposed operand,
keys leaking across sequences or heads) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch

from dit_workloads import bf16_bits_to_f32, f32_to_bf16_bits, make_custom, make_workload, sample_rows
from oracle import dit_attn_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_cases.txt")


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def _pack1(q, k, v):
    """[L, D] float64 arrays -> [L, 1, D] with a one-sequence cu_seqlens."""
    L = q.shape[0]
    return q[:, None, :], k[:, None, :], v[:, None, :], np.array([0, L], dtype=np.int32)


# ---------------------------------------------------------------- P1: hand cases and brute force

def _parse_rows(txt):
    env = {"ln2": math.log(2), "ln3": math.log(3), "ln4": math.log(4), "ln5": math.log(5)}
    return np.array([[eval(e, {"__builtins__": {}}, env) for e in row.split(",")]
                     for row in txt.strip().split(";")], dtype=np.float64)


def _golden_cases():
    cases = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, scale, q, k, v, o = [p.strip() for p in line.split("|")]
            cases.append((name, float(scale), _parse_rows(q), _parse_rows(k), _parse_rows(v), _parse_rows(o)))
    return cases


@pytest.mark.parametrize("case", _golden_cases(), ids=lambda c: c[0])
def test_hand_computed_cases(case):
    _, scale, q, k, v, o = case
    # queries and keys may have different counts in these cases: use the single-head primitive
    got = orc.attention_single(q, k, v, scale)
    np.testing.assert_allclose(got, o, rtol=0, atol=1e-12)


def _brute(q, k, v, cu, scale):
    """Independent pure-Python triple loop with math.exp (no numpy arithmetic)."""
    T, H, D = q.shape
    out = [[[0.0] * D for _ in range(H)] for _ in range(T)]
    for i in range(len(cu) - 1):
        s, e = int(cu[i]), int(cu[i + 1])
        for h in range(H):
            for r in range(s, e):
                logits = []
                for j in range(s, e):
                    acc = 0.0
                    for d in range(D):
                        acc += float(q[r, h, d]) * float(k[j, h, d])
                    logits.append(scale * acc)
                mx = max(logits)
                w = [math.exp(x - mx) for x in logits]
                z = sum(w)
                for d in range(D):
                    out[r][h][d] = sum(w[jj] * float(v[s + jj, h, d]) for jj in range(e - s)) / z
    return np.array(out)


@pytest.mark.parametrize("lens,H,D", [([1], 1, 1), ([2], 1, 1), ([4], 1, 2), ([3, 1, 4], 2, 2), ([2, 0, 3], 3, 4)])
def test_brute_force_tiny(lens, H, D):
    T = sum(lens)
    q, k, v = _rand((T, H, D), 1), _rand((T, H, D), 2), _rand((T, H, D), 3)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    got = orc.attention_varlen(q, k, v, cu, 0.7)
    np.testing.assert_allclose(got, _brute(q, k, v, cu, 0.7), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P2: two-key closed form

def test_two_key_logistic():
    D = 8
    q = _rand((1, D), 10)
    k = _rand((2, D), 11)
    v = _rand((2, D), 12)
    scale = 0.37
    z = scale * float(q[0] @ (k[0] - k[1]))
    sig = 1.0 / (1.0 + math.exp(-z))
    want = sig * v[0] + (1 - sig) * v[1]
    got = orc.attention_single(q, k, v, scale)[0]
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P3: rows of P sum to one, over keys

def test_probs_rows_sum_to_one():
    q, k = _rand((7, 16), 20), _rand((11, 16), 21)
    P = orc.softmax_probs(q, k, 0.25)
    assert P.shape == (7, 11)
    np.testing.assert_allclose(P.sum(axis=1), np.ones(7), rtol=0, atol=1e-12)
    assert np.all(P > 0)
    # normalising over the wrong axis would make columns, not rows, sum to one
    assert np.max(np.abs(P.sum(axis=0) - 1.0)) > 1e-3


# ---------------------------------------------------------------- P4: identical keys -> mean of V

def test_identical_keys_give_mean_of_v():
    L, D = 13, 8
    q, v = _rand((L, D), 30), _rand((L, D), 31)
    k = np.tile(_rand((1, D), 32), (L, 1))
    got = orc.attention_varlen(*_pack1(q, k, v), 0.5)[:, 0, :]
    np.testing.assert_allclose(got, np.tile(v.mean(axis=0), (L, 1)), rtol=0, atol=1e-12)


# ---------------------------------------------------------------- P5: a one-token sequence returns V

def test_one_token_sequence_returns_v_bits():
    w = make_custom([1, 5, 1], 3, 16, seed=40)
    out = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    vf = orc.widen_bf16(w.v)
    assert np.array_equal(out[0], vf[0])
    assert np.array_equal(out[6], vf[6])


# ---------------------------------------------------------------- P6: permutations

def test_key_permutation_invariance_and_query_equivariance():
    L, D = 17, 8
    q, k, v = _rand((L, D), 50), _rand((L, D), 51), _rand((L, D), 52)
    base = orc.attention_single(q, k, v, 0.3)
    perm = np.random.Generator(np.random.PCG64(53)).permutation(L)
    np.testing.assert_allclose(orc.attention_single(q, k[perm], v[perm], 0.3), base, rtol=0, atol=1e-12)
    np.testing.assert_allclose(orc.attention_single(q[perm], k, v, 0.3), base[perm], rtol=0, atol=1e-12)
    # permuting keys without values must change the result (K and V are paired by row)
    assert np.max(np.abs(orc.attention_single(q, k[perm], v, 0.3) - base)) > 1e-3


# ---------------------------------------------------------------- P7: key shift (pins the max subtraction)

def test_key_shift_invariance_and_large_logits():
    L, D = 9, 4
    q, k, v = _rand((L, D), 60), _rand((L, D), 61), _rand((L, D), 62)
    base = orc.attention_single(q, k, v, 1.0)
    c = _rand((1, D), 63) * 3
    np.testing.assert_allclose(orc.attention_single(q, k + c, v, 1.0), base, rtol=0, atol=1e-10)
    # logits around 1e4 overflow exp() unless the row maximum is subtracted first
    big = orc.attention_single(q * 100, k * 100, v, 1.0)
    assert np.all(np.isfinite(big))


# ---------------------------------------------------------------- P8: scale = 0 -> mean of V; scale matters

def test_scale_zero_gives_mean_and_scale_is_used():
    L, D = 6, 4
    q, k, v = _rand((L, D), 70), _rand((L, D), 71), _rand((L, D), 72)
    got = orc.attention_single(q, k, v, 0.0)
    np.testing.assert_allclose(got, np.tile(v.mean(axis=0), (L, 1)), rtol=0, atol=1e-12)
    # scale * (q k^T) == (scale q) k^T: a dropped scale would break this equality
    np.testing.assert_allclose(orc.attention_single(q, k, v, 0.4), orc.attention_single(0.4 * q, k, v, 1.0),
                               rtol=0, atol=1e-12)
    assert np.max(np.abs(orc.attention_single(q, k, v, 0.4) - orc.attention_single(q, k, v, 1.0))) > 1e-3


# ---------------------------------------------------------------- P9: convex hull

def test_output_inside_convex_hull_of_values():
    w = make_custom([33, 7], 2, 16, seed=80)
    out = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    vf = orc.widen_bf16(w.v)
    for i in range(2):
        s, e = int(w.cu_seqlens[i]), int(w.cu_seqlens[i + 1])
        for h in range(2):
            lo, hi = vf[s:e, h].min(axis=0), vf[s:e, h].max(axis=0)
            assert np.all(out[s:e, h] >= lo - 1e-15) and np.all(out[s:e, h] <= hi + 1e-15)


# ---------------------------------------------------------------- P10: hard-max limit

def test_hard_max_limit():
    L, D = 8, 4
    q = _rand((1, D), 90)
    k = np.zeros((L, D))
    k[5] = 50.0 * q[0] / np.linalg.norm(q[0])
    v = _rand((L, D), 91)
    got = orc.attention_single(q, k, v, 1.0)[0]
    # weight of every other key is exp(-50 |q|)
    bound = (L - 1) * math.exp(-50.0 * np.linalg.norm(q[0])) * 2 * np.max(np.abs(v))
    assert np.max(np.abs(got - v[5])) <= max(bound, 1e-9)


# ---------------------------------------------------------------- P11: pack isolation

def test_pack_isolation():
    w = make_custom([5, 12, 0, 3], 2, 8, seed=100)
    full = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    cu = w.cu_seqlens
    for i in range(4):
        s, e = int(cu[i]), int(cu[i + 1])
        if e == s:
            continue
        alone = orc.attention_varlen(w.q[s:e], w.k[s:e], w.v[s:e], np.array([0, e - s]), w.scale)
        assert np.array_equal(full[s:e], alone)
    # perturbing sequence 1 leaves sequences 0 and 3 bit-identical, and changes sequence 1
    k2, v2 = w.k.copy(), w.v.copy()
    k2[5:17] = f32_to_bf16_bits(bf16_bits_to_f32(k2[5:17]) + 1.0)
    v2[5:17] = f32_to_bf16_bits(bf16_bits_to_f32(v2[5:17]) * 2.0)
    pert = orc.attention_varlen(w.q, k2, v2, cu, w.scale)
    assert np.array_equal(pert[0:5], full[0:5]) and np.array_equal(pert[17:20], full[17:20])
    assert np.max(np.abs(pert[5:17] - full[5:17])) > 1e-3


# ---------------------------------------------------------------- P12: head independence

def test_head_independence():
    w = make_custom([9, 4], 5, 8, seed=110)
    full = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    for h in range(5):
        one = orc.attention_varlen(w.q[:, h:h + 1], w.k[:, h:h + 1], w.v[:, h:h + 1], w.cu_seqlens, w.scale)
        assert np.array_equal(full[:, h:h + 1], one)
    # a head subset of a wider run equals a narrower run on those heads (the head-split shard view)
    sub = orc.attention_varlen(w.q[:, 2:4], w.k[:, 2:4], w.v[:, 2:4], w.cu_seqlens, w.scale)
    assert np.array_equal(full[:, 2:4], sub)


# ---------------------------------------------------------------- P13: a library routine on the equal-length case

@pytest.mark.parametrize("B,L,H,D", [(3, 37, 4, 16), (2, 130, 2, 64)])
def test_against_torch_sdpa_fp64(B, L, H, D):
    w = make_custom([L] * B, H, D, seed=120 + L)
    got = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)

    def to_t(bits):
        x = torch.from_numpy(bf16_bits_to_f32(bits).astype(np.float64))
        return x.reshape(B, L, H, D).permute(0, 2, 1, 3)  # [B, H, L, D]

    ref = torch.nn.functional.scaled_dot_product_attention(to_t(w.q), to_t(w.k), to_t(w.v), scale=w.scale)
    ref = ref.permute(0, 2, 1, 3).reshape(B * L, H, D).numpy()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-10)


# ---------------------------------------------------------------- row-subset variant equals the full definition

def test_rows_variant_matches_full():
    w = make_custom([70, 0, 131, 1], 3, 16, seed=130)
    full = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    rows = sample_rows(w.cu_seqlens, seed=5, block=16)
    part = orc.attention_varlen_rows(w.q, w.k, w.v, w.cu_seqlens, w.scale, rows)
    np.testing.assert_allclose(part, full[rows], rtol=0, atol=1e-13)
    # chunking of query rows changes nothing
    chunked = orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale, row_chunk=7)
    np.testing.assert_allclose(chunked, full, rtol=0, atol=1e-13)


def test_widen_bf16_exact():
    bits = np.array([0x0000, 0x3F80, 0xBF80, 0x4000, 0x3F00, 0x4049, 0x0080, 0x7F7F], dtype=np.uint16)
    want = np.array([0.0, 1.0, -1.0, 2.0, 0.5, 3.140625, 2.0 ** -126, (2 - 2 ** -7) * 2.0 ** 127])
    assert np.array_equal(orc.widen_bf16(bits), want)


# ---------------------------------------------------------------- workload generator sanity (no arithmetic of the method)

def test_bf16_rounding_rne():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -2.5], dtype=np.float32)
    bits = f32_to_bf16_bits(x)
    back = bf16_bits_to_f32(bits)
    # ties go to even mantissa: 1+2^-8 -> 1.0, 1+3*2^-8 -> 1+2^-6
    assert back.tolist() == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7, -2.5]


def test_named_workload_shapes():
    w = make_workload("tiny_image")
    assert w.q.shape == (1024, 8, 64) and w.cu_seqlens.tolist() == [0, 1024] and w.scale == 0.125
    w2 = make_workload("tiny_image")
    assert np.array_equal(w.q, w2.q) and np.array_equal(w.v, w2.v)
    assert not np.array_equal(w.q, w.k)
    # statistics of the draw: N(0,1)
    qf = bf16_bits_to_f32(w.q)
    assert abs(float(qf.mean())) < 0.01 and abs(float(qf.std()) - 1.0) < 0.01


def test_mixed_varlen_layout():
    from dit_workloads import _CONFIGS  # lengths only; no tensors drawn here
    lens = sorted(_CONFIGS["mixed_varlen"]["lens"])
    assert lens == [1280] * 2 + [4352] * 6 + [20506] and sum(lens) == 49178
    assert _CONFIGS["sp_shard"]["lens"] == [76112] and _CONFIGS["t2v_single"]["lens"] == [20506]


def test_sample_rows_properties():
    cu = np.array([0, 300, 300, 1000, 1001], dtype=np.int32)
    rows = sample_rows(cu, seed=1, block=64)
    assert np.all(np.diff(rows) > 0) and rows[0] == 0 and rows[-1] == 1000
    for r in (298, 299, 300, 301, 998, 999):
        assert r in rows
    # one pick in every 64-row block of every sequence
    for s, e in ((0, 300), (300, 1000)):
        for b in range(s, e, 64):
            assert np.any((rows >= b) & (rows < min(e, b + 64)))
    few = sample_rows(cu, seed=1, block=64, max_rows=30)
    assert len(few) <= 30 and 999 in few


# ---------------------------------------------------------------- log-sum-exp, merge of partial results, cross-attention

GOLDEN_LSE = os.path.join(os.path.dirname(__file__), "golden", "lse_merge_cases.txt")


def _lse_merge_cases(kind):
    env = {"ln2": math.log(2), "ln3": math.log(3), "ln4": math.log(4), "ln5": math.log(5), "ln8": math.log(8)}
    ev = lambda e: eval(e, {"__builtins__": {}}, env)  # noqa: E731
    vec = lambda t: np.array([ev(x) for x in t.split(";")], dtype=np.float64)  # noqa: E731
    cases = []
    with open(GOLDEN_LSE) as f:
        for line in f:
            parts = [p.strip() for p in line.strip().split("|")]
            if not line.strip() or line.startswith("#") or parts[0] != kind:
                continue
            cases.append(parts[1:] if kind == "lse" else parts[1:])
    return cases, ev, vec


def test_lse_hand_cases():
    cases, ev, vec = _lse_merge_cases("lse")
    assert len(cases) >= 2
    for name, scale, q, k, want in cases:
        qa = np.array([[ev(q)]]); ka = vec(k)[:, None]
        got = orc.logsumexp_scores(qa, ka, float(scale))
        assert abs(got[0] - ev(want)) < 1e-14, name


def test_merge_hand_cases():
    cases, ev, vec = _lse_merge_cases("merge")
    assert len(cases) >= 2
    for name, lses, os_, want_lse, want_o in cases:
        l = vec(lses)[:, None, None]
        o = vec(os_)[:, None, None, None]
        got_o, got_l = orc.merge_partials(o, l)
        assert abs(got_l[0, 0] - ev(want_lse)) < 1e-14 and abs(got_o[0, 0, 0] - ev(want_o)) < 1e-14, name


def test_lse_against_scipy_and_closed_forms():
    from scipy.special import logsumexp
    q, k = _rand((7, 16), 301), _rand((13, 16), 302)
    for scale in (0.25, -0.7, 0.0):
        want = logsumexp(scale * np.einsum("rd,jd->rj", q, k), axis=1)
        assert np.allclose(orc.logsumexp_scores(q, k, scale), want, rtol=0, atol=1e-13)
    # identical keys: lse = scale <q, k> + ln L; one key: lse = scale <q, k>; huge logits do not overflow
    k1 = np.repeat(_rand((1, 16), 303), 9, axis=0)
    assert np.allclose(orc.logsumexp_scores(q, k1, 0.3), 0.3 * (q @ k1[0]) + math.log(9), atol=1e-13)
    assert np.allclose(orc.logsumexp_scores(q, k1[:1], 0.3), 0.3 * (q @ k1[0]), atol=1e-13)
    big = orc.logsumexp_scores(1e3 * q, 1e3 * k, 1.0)
    assert np.all(np.isfinite(big)) and np.allclose(big, (1e6 * (q @ k.T)).max(axis=1), rtol=1e-12)
    assert np.all(orc.logsumexp_scores(q, k[:0], 1.0) == -np.inf)


def test_varlen_lse_layout_and_o_unchanged():
    w = make_custom([5, 1, 9], 2, 8, seed=304)
    o, lse = orc.attention_varlen_lse(w.q, w.k, w.v, w.cu_seqlens, w.scale)
    assert np.array_equal(o, orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale))
    qf, kf = orc.widen_bf16(w.q), orc.widen_bf16(w.k)
    for (s, e) in ((0, 5), (5, 6), (6, 15)):
        for h in range(2):
            for r in range(s, e):
                want = math.log(sum(math.exp(w.scale * float(qf[r, h] @ kf[j, h])) for j in range(s, e)))
                assert abs(lse[r, h] - want) < 1e-12


@pytest.mark.parametrize("splits", [(4, 9), (1, 2, 12), (13,)])
def test_merge_of_disjoint_key_sets_is_attention_over_the_union(splits):
    """The identity the merge rests on, against the (separately pinned) attention definition."""
    L, D, scale = 13, 8, 0.4
    q, k, v = _rand((6, D), 305), _rand((L, D), 306), _rand((L, D), 307)
    perm = np.random.Generator(np.random.PCG64(308)).permutation(L)   # parts need not be contiguous ranges
    bounds = [0] + list(splits) + ([L] if splits[-1] != L else [])
    o_parts, l_parts = [], []
    for a, b in zip(bounds[:-1], bounds[1:]):
        idx = perm[a:b]
        o_parts.append(orc.attention_single(q, k[idx], v[idx], scale)[:, None, :])
        l_parts.append(orc.logsumexp_scores(q, k[idx], scale)[:, None])
    o, lse = orc.merge_partials(np.stack(o_parts), np.stack(l_parts))
    assert np.allclose(o[:, 0], orc.attention_single(q, k, v, scale), rtol=0, atol=1e-13)
    assert np.allclose(lse[:, 0], orc.logsumexp_scores(q, k, scale), rtol=0, atol=1e-13)
    # order of the parts does not matter; a part without keys changes nothing
    o2, lse2 = orc.merge_partials(np.stack(o_parts[::-1] + [np.full_like(o_parts[0], 7.0)]),
                                  np.stack(l_parts[::-1] + [np.full_like(l_parts[0], -np.inf)]))
    assert np.allclose(o2, o, atol=1e-13) and np.allclose(lse2, lse, atol=1e-13)


def test_merge_brute_force_and_degenerate_rows():
    g = np.random.Generator(np.random.PCG64(309))
    P, T, H, D = 3, 4, 2, 3
    o, l = g.standard_normal((P, T, H, D)), 3.0 * g.standard_normal((P, T, H))
    got_o, got_l = orc.merge_partials(o, l)
    for t in range(T):
        for h in range(H):
            z = sum(math.exp(l[p, t, h]) for p in range(P))
            assert abs(got_l[t, h] - math.log(z)) < 1e-12
            for d in range(D):
                assert abs(got_o[t, h, d] - sum(math.exp(l[p, t, h]) * o[p, t, h, d] for p in range(P)) / z) < 1e-12
    # identical parts give that part (weights sum to one); a row whose parts are all empty is zero with lse -inf
    same, ls = np.repeat(o[:1], 3, axis=0), l.copy()
    assert np.allclose(orc.merge_partials(same, ls)[0], o[0], atol=1e-13)
    ls[:, 1, 0] = -np.inf
    zo, zl = orc.merge_partials(o, ls)
    assert np.all(zo[1, 0] == 0.0) and zl[1, 0] == -np.inf and np.all(np.isfinite(zo))


def test_cross_attention_equals_self_attention_on_equal_boundaries_and_brute_force():
    w = make_custom([6, 3, 10], 2, 8, seed=310)
    o, _ = orc.attention_cross_varlen(w.q, w.k, w.v, w.cu_seqlens, w.cu_seqlens, w.scale)
    assert np.array_equal(o, orc.attention_varlen(w.q, w.k, w.v, w.cu_seqlens, w.scale))
    # different query and key lengths, a sequence without keys, one without queries
    cq, ck = np.array([0, 4, 6, 6, 9]), np.array([0, 7, 7, 9, 14])
    q, k, v = _rand((9, 2, 4), 311), _rand((14, 2, 4), 312), _rand((14, 2, 4), 313)
    o, lse = orc.attention_cross_varlen(q, k, v, cq, ck, 0.6)
    for i in range(4):
        for r in range(cq[i], cq[i + 1]):
            for h in range(2):
                keys = range(ck[i], ck[i + 1])
                if len(keys) == 0:
                    assert np.all(o[r, h] == 0.0) and lse[r, h] == -np.inf
                    continue
                wts = [math.exp(0.6 * float(q[r, h] @ k[j, h])) for j in keys]
                z = sum(wts)
                want = sum(wj * v[j, h] for wj, j in zip(wts, keys)) / z
                assert np.allclose(o[r, h], want, atol=1e-13) and abs(lse[r, h] - math.log(z)) < 1e-12


def test_cross_attention_against_torch_and_invariances():
    Lq, Lk, H, D = 5, 11, 3, 16
    q, k, v = _rand((Lq, H, D), 314), _rand((Lk, H, D), 315), _rand((Lk, H, D), 316)
    o, _ = orc.attention_cross_varlen(q, k, v, [0, Lq], [0, Lk], 0.37)
    tq, tk, tv = (torch.from_numpy(x).permute(1, 0, 2)[None] for x in (q, k, v))
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.37)[0].permute(1, 0, 2).numpy()
    assert np.allclose(o, want, atol=1e-12)
    perm = np.random.Generator(np.random.PCG64(317)).permutation(Lk)
    assert np.allclose(orc.attention_cross_varlen(q, k[perm], v[perm], [0, Lq], [0, Lk], 0.37)[0], o, atol=1e-13)
    assert not np.allclose(orc.attention_cross_varlen(q, k[perm], v, [0, Lq], [0, Lk], 0.37)[0], o, atol=1e-3)
    # pack isolation: a second sequence's keys do not reach the first sequence's queries
    q2, k2, v2 = np.concatenate([q, q[:2]]), np.concatenate([k, _rand((4, H, D), 318)]), np.concatenate([v, _rand((4, H, D), 319)])
    o2, _ = orc.attention_cross_varlen(q2, k2, v2, [0, Lq, Lq + 2], [0, Lk, Lk + 4], 0.37)
    assert np.array_equal(o2[:Lq], o)
