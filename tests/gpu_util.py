"""Helpers for the GPU parity tests: move bf16 bit patterns to the device, run the C-ABI call, compare."""
import numpy as np
import torch

import paper_2604_04335_amd as da
from dit_workloads import bf16_bits_to_f32

# Parity bar of the benchmark definition: bf16 inputs, fp32 accumulation.
MAX_ABS_TOL = 2e-2
REL_L2_TOL = 1e-2

SENTINEL = 0x7FC1  # a NaN bit pattern the kernel never produces from finite inputs
GUARD_ROWS = 64


def to_dev(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to("cuda").view(torch.bfloat16)


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def widen(bits: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(bits).astype(np.float64)


class Runner:
    """One context; runs a workload through dit_attn_varlen_fwd with guard rows around `out`."""

    def __init__(self):
        self.ctx = da.dit_attn_create(0)

    def close(self):
        da.dit_attn_destroy(self.ctx)
        self.ctx = 0

    def run_dev(self, q, k, v, cu, H, D, scale, stream=None):
        """q, k, v: device bf16 tensors [T, H, D].  Returns device bf16 [T, H, D]; checks the guard rows."""
        T = int(cu[-1])
        buf = torch.full((T + 2 * GUARD_ROWS, H, D), SENTINEL, dtype=torch.int16, device="cuda")
        out = buf[GUARD_ROWS:GUARD_ROWS + T].view(torch.bfloat16)
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        da.dit_attn_varlen_fwd(self.ctx, q, k, v, cu, H, D, scale, out, stream)
        torch.cuda.synchronize()
        assert bool((buf[:GUARD_ROWS] == SENTINEL).all()), "rows before out[0] were written"
        assert bool((buf[GUARD_ROWS + T:] == SENTINEL).all()), "rows after out[T-1] were written"
        return out

    def run(self, w, scale=None, kernel=None):
        """w: dit_workloads.Workload.  Returns uint16 bits [T, H, D].  kernel: one of da.KERNEL_* for this call only."""
        q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
        if kernel is not None:
            da.dit_attn_set_kernel(self.ctx, kernel)
        try:
            out = self.run_dev(q, k, v, w.cu_seqlens, w.n_heads, w.head_dim, w.scale if scale is None else scale)
        finally:
            if kernel is not None:
                da.dit_attn_set_kernel(self.ctx, da.KERNEL_AUTO)
        return to_bits(out)


def errors(got: np.ndarray, ref: np.ndarray):
    """got, ref float64 arrays of the same shape -> (max_abs, rel_l2)."""
    diff = got - ref
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    denom = float(np.sqrt(np.sum(ref * ref)))
    rel = float(np.sqrt(np.sum(diff * diff)) / denom) if denom > 0 else 0.0
    return max_abs, rel


def assert_parity(got_bits: np.ndarray, ref: np.ndarray, what: str = ""):
    got = widen(got_bits)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    max_abs, rel = errors(got, ref)
    assert max_abs <= MAX_ABS_TOL and rel <= REL_L2_TOL, f"{what}: max_abs={max_abs:.3e} rel_l2={rel:.3e}"
    return max_abs, rel
