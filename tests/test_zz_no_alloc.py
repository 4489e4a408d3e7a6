"""The entry point that allocates nothing (dit_attn_varlen_fwd_noalloc) against dit_attn_varlen_fwd: same bits, on two
calls in a row, the second with a smaller input (the device scratch keeps the first call's work-list); both kernels;
the limits are refused with `out` untouched."""
import os
import sys

import numpy as np
import pytest
import torch

import paper_2604_04335_amd as da
from dit_workloads import make_custom

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from gpu_util import GUARD_ROWS, SENTINEL, to_dev  # noqa: E402

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = da.dit_attn_create(0)
    yield c
    da.dit_attn_destroy(c)


def _both(ctx, w):
    """(bits of the allocating entry point, bits of the non-allocating one) for workload w, guard rows checked."""
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    T, H, D = q.shape
    stream = torch.cuda.current_stream().cuda_stream
    ref = torch.empty_like(q)
    da.dit_attn_varlen_fwd(ctx, q, k, v, w.cu_seqlens, H, D, w.scale, ref, stream)
    kernel = da.dit_attn_last_launch_kernel(ctx)
    buf = torch.full((T + 2 * GUARD_ROWS, H, D), SENTINEL, dtype=torch.int16, device="cuda")
    out = buf[GUARD_ROWS:GUARD_ROWS + T].view(torch.bfloat16)
    da.dit_attn_varlen_fwd_noalloc(ctx, q, k, v, w.cu_seqlens, H, D, w.scale, out, stream)
    torch.cuda.synchronize()
    assert da.dit_attn_last_launch_kernel(ctx) == kernel
    assert bool((buf[:GUARD_ROWS] == SENTINEL).all()) and bool((buf[GUARD_ROWS + T:] == SENTINEL).all())
    return ref.view(torch.int16), out.view(torch.int16)


def test_two_calls_in_a_row_second_smaller(ctx):
    # 24 query tiles of 256 rows x 40 heads = 960 items (3.75 per compute unit), ragged sequences and an empty one: the
    # ping-pong kernel
    big = make_custom([4352, 130, 0, 1000, 65, 1], 40, 128, seed=51)
    print("noalloc: first call", big.seq_lens, flush=True)
    a, b = _both(ctx, big)
    assert da.dit_attn_last_launch_kernel(ctx) == da.KERNEL_PINGPONG
    assert torch.equal(a, b)
    # a smaller pack right after it (fewer items, other boundaries): the 128-row kernel
    small = make_custom([300, 77, 129], 3, 128, seed=52)
    print("noalloc: second call", small.seq_lens, flush=True)
    a, b = _both(ctx, small)
    assert da.dit_attn_last_launch_kernel(ctx) == da.KERNEL_128
    assert torch.equal(a, b)
    # and the first again, head dimension 64 this time
    again = make_custom([4352, 130, 0, 1000, 65, 1], 40, 64, seed=53)
    a, b = _both(ctx, again)
    assert da.dit_attn_last_launch_kernel(ctx) == da.KERNEL_PINGPONG
    assert torch.equal(a, b)


def test_sequence_order_ties_and_negative_scale(ctx):
    w = make_custom([640, 1280, 640, 1280, 64], 6, 128, seed=54, scale=-0.11)
    a, b = _both(ctx, w)
    assert torch.equal(a, b)


def test_limits_are_refused(ctx):
    w = make_custom([8] * 65, 1, 64, seed=55)
    q, k, v = to_dev(w.q), to_dev(w.k), to_dev(w.v)
    out = torch.full(q.shape, SENTINEL, dtype=torch.int16, device="cuda")
    with pytest.raises(da.DitAttnError) as e:
        da.dit_attn_varlen_fwd_noalloc(ctx, q, k, v, w.cu_seqlens, 1, 64, w.scale, out, None)
    assert e.value.code == -11 and "64 sequences" in str(e.value)
    # 16385 items: 16385 heads of one 256-row tile would be 8 GB; use the argument check alone with a fake shape
    cu = np.array([0, 200], dtype=np.int32)
    with pytest.raises(da.DitAttnError) as e:
        da.dit_attn_varlen_fwd_noalloc(ctx, q, k, v, cu, 16385, 64, w.scale, out, None)
    assert e.value.code == -11 and "work items" in str(e.value)
    torch.cuda.synchronize()
    assert bool((out == SENTINEL).all())
    # the same pack at the limit of 64 sequences runs
    w = make_custom([8] * 64, 1, 64, seed=56)
    a, b = _both(ctx, w)
    assert torch.equal(a, b)
