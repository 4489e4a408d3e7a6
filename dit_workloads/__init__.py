"""Seeded synthetic inputs for the DiT denoising-step attention workloads.

This module is the only code shared by the CPU oracle's tests and the GPU
path's tests / benchmark.  It holds *no* attention arithmetic: it only draws
random numbers, rounds them to bf16 bit patterns and lays out packs of
variable-length sequences.

Workload shapes follow the paper's batched denoising step: same-resolution
image requests are coalesced into one step call (Section 4.3, "SLO-aware
Dynamic Batching"), one video runs per sequence-parallel group (Section 4.4,
Eq. 2-3), and a Ulysses-style head split leaves each GPU with a head subset
over the full sequence (Section 5).  The five named configurations are the
benchmark's own; the paper's prompts, weights and traces are not used, only
token counts and a Gaussian value distribution.

Everything is produced on the host with numpy's PCG64 so that the oracle and
the GPU see the same bits.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "Workload",
    "CrossWorkload",
    "make_cross",
    "CONFIG_NAMES",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "make_workload",
    "make_custom",
    "sample_rows",
    "attention_flops",
]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 -> bf16 (round-to-nearest-even), returned as uint16 bit patterns.

    Done with integer arithmetic on the fp32 bits so the result does not depend
    on any library's bf16 support.  NaN payloads are not preserved (inputs here
    are finite).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float32 exactly."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Workload:
    """One packed denoising-step attention call.

    q, k, v: uint16 arrays of bf16 bit patterns, shape [T, n_heads, head_dim],
    C-contiguous.  cu_seqlens: int32 [n_seqs + 1], cu_seqlens[0] == 0.
    """

    name: str
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    cu_seqlens: np.ndarray
    n_heads: int
    head_dim: int
    scale: float
    seed: int
    meta: dict = field(default_factory=dict)

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def seq_lens(self) -> list:
        return [int(x) for x in np.diff(self.cu_seqlens)]


# name -> (sequence lengths before shuffling, heads, head_dim, per-head value scale?, shuffle?, metadata)
_CONFIGS = {
    # Tiny image step: 64 text + 960 latent tokens.
    "tiny_image": dict(lens=[1024], H=8, D=64, head_scale=False, shuffle=False,
                       meta={"text": 64, "latent": 960}),
    # T2I batch: 4 x (256 text + 4096 latent) (1024x1024, 8x VAE, 2x2 patch).
    "t2i_batch": dict(lens=[4352] * 4, H=24, D=128, head_scale=True, shuffle=False,
                      meta={"text": 256, "latent": 4096}),
    # T2V single request: 226 text + 13*30*52 latent tokens.
    "t2v_single": dict(lens=[226 + 13 * 30 * 52], H=24, D=128, head_scale=False, shuffle=False,
                       meta={"text": 226, "latent": 13 * 30 * 52}),
    # Mixed dynamic batch: 6 images of 4352 + 1 video of 20506 + 2 images of 1280, order shuffled.
    "mixed_varlen": dict(lens=[4352] * 6 + [20506] + [1280] * 2, H=24, D=128, head_scale=False,
                         shuffle=True, meta={}),
    # One GPU's share of a head-split (degree 4) long video: 512 text + 21*45*80 latent, 10 of 40 heads.
    "sp_shard": dict(lens=[512 + 21 * 45 * 80], H=10, D=128, head_scale=False, shuffle=False,
                     meta={"text": 512, "latent": 21 * 45 * 80, "heads_total": 40, "sp_degree": 4}),
}

CONFIG_NAMES = list(_CONFIGS.keys())


def _draw_bf16(rng: np.random.Generator, shape, head_scale: np.ndarray | None) -> np.ndarray:
    x = rng.standard_normal(shape, dtype=np.float32)
    if head_scale is not None:
        x *= head_scale.astype(np.float32)[None, :, None]
    return f32_to_bf16_bits(x)


def make_custom(seq_lens, n_heads: int, head_dim: int, seed: int, *, scale: float | None = None,
                head_scale: bool = False, name: str = "custom") -> Workload:
    """A pack with the given sequence lengths (zeros allowed), N(0,1) values rounded to bf16."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = np.asarray(list(seq_lens), dtype=np.int64)
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lens)
    T = int(cu[-1])
    hs = rng.uniform(0.5, 2.0, size=n_heads) if head_scale else None
    shape = (T, n_heads, head_dim)
    q = _draw_bf16(rng, shape, hs)
    k = _draw_bf16(rng, shape, hs)
    v = _draw_bf16(rng, shape, hs)
    if scale is None:
        scale = 1.0 / math.sqrt(head_dim)
    return Workload(name=name, q=q, k=k, v=v, cu_seqlens=cu, n_heads=n_heads, head_dim=head_dim,
                    scale=float(scale), seed=seed,
                    meta={"head_scale": None if hs is None else hs.tolist()})


@dataclass
class CrossWorkload:
    """Cross-attention pack: q [Tq, H, D]; k, v [Tk, H, D] (uint16 bf16 bits); separate boundaries."""
    q: np.ndarray
    k: np.ndarray
    v: np.ndarray
    cu_seqlens_q: np.ndarray
    cu_seqlens_k: np.ndarray
    n_heads: int
    head_dim: int
    scale: float
    seed: int


def make_cross(q_lens, k_lens, n_heads: int, head_dim: int, seed: int, *, scale: float | None = None) -> CrossWorkload:
    """Queries of the given lengths against keys of the given lengths (same number of sequences, zeros allowed), N(0,1)
    values rounded to bf16.  The DiT models of the paper's evaluation condition on text (Section 2.1): latent queries
    (thousands of tokens) against a few hundred text keys is the typical shape."""
    rng = np.random.Generator(np.random.PCG64(seed))
    ql, kl = np.asarray(list(q_lens), dtype=np.int64), np.asarray(list(k_lens), dtype=np.int64)
    assert len(ql) == len(kl)
    cq, ck = np.zeros(len(ql) + 1, dtype=np.int32), np.zeros(len(kl) + 1, dtype=np.int32)
    cq[1:], ck[1:] = np.cumsum(ql), np.cumsum(kl)
    q = _draw_bf16(rng, (int(cq[-1]), n_heads, head_dim), None)
    k = _draw_bf16(rng, (int(ck[-1]), n_heads, head_dim), None)
    v = _draw_bf16(rng, (int(ck[-1]), n_heads, head_dim), None)
    if scale is None:
        scale = 1.0 / math.sqrt(head_dim)
    return CrossWorkload(q=q, k=k, v=v, cu_seqlens_q=cq, cu_seqlens_k=ck, n_heads=n_heads, head_dim=head_dim,
                         scale=float(scale), seed=seed)


def make_workload(name: str, seed: int | None = None) -> Workload:
    """One of the five named benchmark configurations.

    The default seed is 1000 + (1-based index of the configuration).  For
    "t2i_batch" a per-head factor s_h ~ U[0.5, 2] multiplies that head's Q, K
    and V before rounding (a data-distribution knob that makes logits of some
    heads peaky; the softmax scale argument stays 1/sqrt(head_dim)).  For
    "mixed_varlen" the sequence order is a seeded permutation.
    """
    cfg = _CONFIGS[name]
    if seed is None:
        seed = 1000 + CONFIG_NAMES.index(name) + 1
    lens = list(cfg["lens"])
    if cfg["shuffle"]:
        order_rng = np.random.Generator(np.random.PCG64(seed ^ 0x5EED))
        lens = [lens[i] for i in order_rng.permutation(len(lens))]
    w = make_custom(lens, cfg["H"], cfg["D"], seed, head_scale=cfg["head_scale"], name=name)
    w.meta.update(cfg["meta"])
    return w


def sample_rows(cu_seqlens: np.ndarray, seed: int, block: int = 64, max_rows: int | None = None) -> np.ndarray:
    """A stratified sample of global query-row indices.

    For every sequence: one seeded-random row in every `block`-row stretch, the
    first and last two rows, and the rows next to multiples of 64/128/256 closest
    to the sequence end (where tile tails live).  Sorted, unique, int64.
    If `max_rows` is given the per-block picks are thinned evenly to fit while
    the boundary rows are kept.
    """
    rng = np.random.Generator(np.random.PCG64(seed ^ 0xA77E))
    cu = np.asarray(cu_seqlens, dtype=np.int64)
    picks = []
    edges = []
    for i in range(len(cu) - 1):
        s, e = int(cu[i]), int(cu[i + 1])
        L = e - s
        if L <= 0:
            continue
        nblk = (L + block - 1) // block
        for b in range(nblk):
            lo = b * block
            hi = min(L, lo + block)
            picks.append(s + lo + int(rng.integers(0, hi - lo)))
        local = {0, 1, L - 2, L - 1}
        for m in (64, 128, 256):
            t = (L // m) * m
            local.update({t - 1, t, t + 1})
        edges.extend(s + r for r in local if 0 <= r < L)
    picks = np.asarray(picks, dtype=np.int64)
    edges = np.asarray(sorted(set(edges)), dtype=np.int64)
    if max_rows is not None and len(picks) + len(edges) > max_rows:
        keep = max(1, max_rows - len(edges))
        idx = np.linspace(0, len(picks) - 1, keep).round().astype(np.int64)
        picks = picks[idx]
    return np.unique(np.concatenate([picks, edges]))


def attention_flops(cu_seqlens, n_heads: int, head_dim: int) -> float:
    """4 * H * D * sum(L_i^2): two contractions, multiply-add = 2, non-causal, softmax not counted."""
    lens = np.diff(np.asarray(cu_seqlens, dtype=np.int64)).astype(np.float64)
    return 4.0 * n_heads * head_dim * float(np.sum(lens * lens))
