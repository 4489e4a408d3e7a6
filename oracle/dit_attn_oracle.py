"""CPU oracle for the DiT denoising-step self-attention.  TEST INFRASTRUCTURE ONLY.

This file is the slow, plain definition that the HIP path is checked against.
Only tests, the smoke check and the benchmark's CPU-baseline leg may import it;
the product path never does.  It shares no code with the HIP path.

What it computes.  A denoising step runs the DiT blocks over a batch of
requests (paper Section 2.1: DiT blocks dominate the step; Section 4.3: same
resolution image requests are batched into one step call; Section 5: with
sequence parallelism each GPU holds a head subset over the full sequence).
Inside a block the quadratic term (Section 7.1) is softmax attention.  The
paper states no kernel and no variant of the math, so the oracle is the
textbook definition, per sequence i with token rows R_i = [cu[i], cu[i+1]),
per head h, per query row r in R_i, all in float64:

    s_j      = scale * sum_d Q[r,h,d] * K[j,h,d]        for j in R_i
    p_j      = exp(s_j - max_j s_j) / sum_j exp(s_j - max_j s_j)
    O[r,h,:] = sum_j p_j * V[j,h,:]

Readings where the paper is silent: no mask inside a sequence (denoising is
bidirectional); a row attends only to keys of its own sequence (requests in a
batch are independent); text and latent tokens are ordinary rows of one joint
sequence; q, k and v have the same number of heads; no dropout; `scale`
multiplies the float64 dot product; nothing is rounded anywhere.

Inputs are bf16 bit patterns (uint16) widened exactly to float64; the output
is float64.  Query rows may be processed in chunks to bound memory: rows are
independent, so this changes no arithmetic of any row.

Pins (tests/test_oracle.py): a hand-computed two-key case, an independent
pure-Python triple loop on tiny inputs, the two-key logistic closed form, rows
of P summing to one, identical keys giving the mean of V, a one-token sequence
returning V, key-permutation invariance and query-permutation equivariance,
key-shift invariance, scale = 0 giving the mean of V, the convex-hull bound,
the hard-max limit, pack isolation, head independence, and agreement with
torch's CPU scaled_dot_product_attention in float64.

Further definitions (same status: test infrastructure), each pinned in the same file:

  * the row-wise log-sum-exp  lse[r,h] = log sum_j exp(s_j)  (natural log) that goes with O.  It is what makes
    partial results over disjoint key sets combinable, which sequence parallelism along the sequence (the ring half
    of the unified sequence parallelism of Section 5) needs.  Pins: scipy's logsumexp on explicit logits, the
    identical-keys and one-key closed forms, a hand case with logits ln 2 and ln 3.
  * merge_partials: given P results (O_p, lse_p) of the same queries over disjoint key sets,
        lse = log sum_p exp(lse_p),   O = sum_p exp(lse_p - lse) O_p,
    which is the attention over the union (a softmax over a union of sets is the lse-weighted mixture of the softmaxes
    over the sets).  Pins: attention over the union computed directly, a pure-Python loop, order invariance, a part
    with no keys, identical parts.
  * attention_cross_varlen: queries and keys with separate sequence boundaries (Section 2.1: DiT blocks also
    cross-attend to the text tokens; sequence i's queries cu_q[i]:cu_q[i+1] see keys cu_k[i]:cu_k[i+1]).  Reading:
    a sequence without keys gives O = 0 and lse = -inf (an empty sum).  Pins: equals the self-attention oracle when the
    boundaries coincide, a pure-Python loop with Lq != Lk, torch's CPU attention in float64 with Lq != Lk, key
    permutation invariance, pack isolation.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "widen_bf16",
    "softmax_probs",
    "attention_single",
    "attention_varlen",
    "attention_varlen_rows",
    "logsumexp_scores",
    "attention_varlen_lse",
    "attention_cross_varlen",
    "merge_partials",
]


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly (bf16 is the top half of an fp32)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    f32 = (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return f32.astype(np.float64)


def softmax_probs(q: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """P[r, j] for one sequence and one head.  q: [Lq, D], k: [Lk, D], float64."""
    s = scale * (q @ k.T)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def attention_single(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float) -> np.ndarray:
    """O = softmax(scale * q k^T) v for one sequence and one head, float64."""
    return softmax_probs(q, k, scale) @ v


def _as_f64(x: np.ndarray) -> np.ndarray:
    if x.dtype == np.uint16:
        return widen_bf16(x)
    return np.asarray(x, dtype=np.float64)


def attention_varlen(q, k, v, cu_seqlens, scale: float, row_chunk: int = 2048) -> np.ndarray:
    """Attention over a packed batch.

    q, k, v: [T, H, D], uint16 bf16 bit patterns (or any float array, used as
    float64).  cu_seqlens: [n_seqs + 1] with cu_seqlens[0] == 0, non-decreasing.
    Returns float64 [T, H, D].  Zero-length sequences contribute no rows.
    """
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    T, H, D = q.shape
    assert int(cu[0]) == 0 and int(cu[-1]) == T and np.all(np.diff(cu) >= 0)
    out = np.zeros((T, H, D), dtype=np.float64)
    for i in range(len(cu) - 1):
        s, e = int(cu[i]), int(cu[i + 1])
        if e == s:
            continue
        for h in range(H):
            qh = _as_f64(q[s:e, h, :])
            kh = _as_f64(k[s:e, h, :])
            vh = _as_f64(v[s:e, h, :])
            for r0 in range(0, e - s, row_chunk):
                r1 = min(e - s, r0 + row_chunk)
                out[s + r0:s + r1, h, :] = attention_single(qh[r0:r1], kh, vh, scale)
    return out


def attention_varlen_rows(q, k, v, cu_seqlens, scale: float, rows) -> np.ndarray:
    """The same definition, evaluated only for the given global query rows.

    Every selected row still uses all keys of its own sequence, so each returned
    row equals the corresponding row of attention_varlen.  rows: increasing
    int array of global token indices.  Returns float64 [len(rows), H, D].
    """
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    rows = np.asarray(rows, dtype=np.int64)
    T, H, D = q.shape
    assert int(cu[0]) == 0 and int(cu[-1]) == T
    assert np.all(rows >= 0) and np.all(rows < T) and np.all(np.diff(rows) > 0)
    out = np.zeros((len(rows), H, D), dtype=np.float64)
    for i in range(len(cu) - 1):
        s, e = int(cu[i]), int(cu[i + 1])
        lo, hi = np.searchsorted(rows, s), np.searchsorted(rows, e)
        if hi == lo:
            continue
        sel = rows[lo:hi]
        for h in range(H):
            qh = _as_f64(q[sel, h, :])
            kh = _as_f64(k[s:e, h, :])
            vh = _as_f64(v[s:e, h, :])
            out[lo:hi, h, :] = attention_single(qh, kh, vh, scale)
    return out


def logsumexp_scores(q: np.ndarray, k: np.ndarray, scale: float) -> np.ndarray:
    """lse[r] = log sum_j exp(scale * <q_r, k_j>) for one sequence and one head, float64; -inf where k has no rows."""
    if k.shape[0] == 0:
        return np.full(q.shape[0], -np.inf)
    s = scale * (q @ k.T)
    m = s.max(axis=1)
    return m + np.log(np.exp(s - m[:, None]).sum(axis=1))


def attention_cross_varlen(q, k, v, cu_seqlens_q, cu_seqlens_k, scale: float, row_chunk: int = 2048):
    """Attention with separate query and key boundaries.  q: [Tq, H, D]; k, v: [Tk, H, D].

    Sequence i: query rows cu_seqlens_q[i]:cu_seqlens_q[i+1] attend to key rows cu_seqlens_k[i]:cu_seqlens_k[i+1].
    Returns (O float64 [Tq, H, D], lse float64 [Tq, H]).  A sequence without keys: O = 0, lse = -inf.
    """
    cq = np.asarray(cu_seqlens_q, dtype=np.int64)
    ck = np.asarray(cu_seqlens_k, dtype=np.int64)
    Tq, H, D = q.shape
    assert len(cq) == len(ck) and int(cq[0]) == 0 and int(ck[0]) == 0
    assert int(cq[-1]) == Tq and int(ck[-1]) == k.shape[0] == v.shape[0]
    assert np.all(np.diff(cq) >= 0) and np.all(np.diff(ck) >= 0)
    out = np.zeros((Tq, H, D), dtype=np.float64)
    lse = np.full((Tq, H), -np.inf, dtype=np.float64)
    for i in range(len(cq) - 1):
        qs, qe, ks, ke = int(cq[i]), int(cq[i + 1]), int(ck[i]), int(ck[i + 1])
        if qe == qs or ke == ks:
            continue
        for h in range(H):
            qh = _as_f64(q[qs:qe, h, :])
            kh = _as_f64(k[ks:ke, h, :])
            vh = _as_f64(v[ks:ke, h, :])
            for r0 in range(0, qe - qs, row_chunk):
                r1 = min(qe - qs, r0 + row_chunk)
                out[qs + r0:qs + r1, h, :] = attention_single(qh[r0:r1], kh, vh, scale)
                lse[qs + r0:qs + r1, h] = logsumexp_scores(qh[r0:r1], kh, scale)
    return out, lse


def attention_varlen_lse(q, k, v, cu_seqlens, scale: float, row_chunk: int = 2048):
    """(O, lse) of the self-attention over a packed batch: attention_varlen plus the row-wise log-sum-exp [T, H]."""
    return attention_cross_varlen(q, k, v, cu_seqlens, cu_seqlens, scale, row_chunk)


def merge_partials(o_parts, lse_parts):
    """Combine P partial results over disjoint key sets.  o_parts: [P, T, H, D]; lse_parts: [P, T, H]; float64.

    Returns (O [T, H, D], lse [T, H]).  A part whose lse is -inf (no keys) has weight 0; if every part of a row is
    -inf the row is 0 with lse -inf.
    """
    o = np.asarray(o_parts, dtype=np.float64)
    l = np.asarray(lse_parts, dtype=np.float64)
    assert o.ndim == 4 and l.shape == o.shape[:3]
    m = l.max(axis=0)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    e = np.exp(l - m_safe[None])          # exp(-inf) = 0
    tot = e.sum(axis=0)
    with np.errstate(divide="ignore"):
        lse = m_safe + np.log(tot)        # log(0) = -inf
    w = np.divide(e, tot[None], out=np.zeros_like(e), where=tot[None] > 0)
    return (w[..., None] * o).sum(axis=0), lse
