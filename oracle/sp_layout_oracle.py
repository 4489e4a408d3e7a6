"""CPU oracle for the head-split sequence-parallel layout change.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this file; the product path never does, and
it shares no code with the HIP path.

What it defines.  With sequence parallelism of degree p over a long video (paper Section 4.3, elastic sequence
parallelism; Section 5: the head-split half of the unified sequence parallelism), rank s holds rows
[s*n, (s+1)*n) of a sequence of L = p*n tokens with all H heads, X_s of shape [n, H, D].  Attention needs, on rank g,
the whole sequence for head group g: Y_g = X[:, g*H/p:(g+1)*H/p, :] of shape [L, H/p, D].  The all-to-all between the
two moves, from rank s to rank g, the block X_s[:, g*H/p:(g+1)*H/p, :].  Its single-GPU halves are pure index maps:

    pack    [n, H, D] -> [p, n, H/p, D]     send[g, r, h, :] = x[r, g*H/p + h, :]     (block g goes to rank g)
    unpack  [p, n, H/p, D] -> [n, H, D]     y[r, g*H/p + h, :] = recv[g, r, h, :]     (block g came from rank g)

Before attention only pack is needed (the blocks received from ranks 0..p-1 are already rows 0..L-1 in order); after
attention only unpack is needed (rank g's [L, H/p, D] result is already p row blocks, one per destination).

Both are written as explicit loops over (g, r, h).  Pins (tests/test_sp_layout.py): a simulated exchange between p
ranks built from pack delivers exactly X[:, head group g] on rank g (the defining property, checked against plain
slicing of the full tensor); the reverse path with unpack restores every rank's X_s; unpack is the inverse of pack; a
hand case with recognisable numbers; p = 1 is the identity.
"""
from __future__ import annotations

import numpy as np

__all__ = ["pack_heads", "unpack_heads"]


def pack_heads(x: np.ndarray, p: int) -> np.ndarray:
    """x: [n, H, D] (any dtype) -> [p, n, H/p, D]."""
    n, H, D = x.shape
    assert p >= 1 and H % p == 0
    hp = H // p
    out = np.empty((p, n, hp, D), dtype=x.dtype)
    for g in range(p):
        for r in range(n):
            for h in range(hp):
                out[g, r, h, :] = x[r, g * hp + h, :]
    return out


def unpack_heads(y: np.ndarray) -> np.ndarray:
    """y: [p, n, H/p, D] -> [n, H, D]."""
    p, n, hp, D = y.shape
    out = np.empty((n, p * hp, D), dtype=y.dtype)
    for g in range(p):
        for r in range(n):
            for h in range(hp):
                out[r, g * hp + h, :] = y[g, r, h, :]
    return out
