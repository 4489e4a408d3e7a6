"""Pins for the sequence-parallel layout oracle, and GPU parity (bit-exact) of the pack / unpack kernels."""
import os
import sys

import numpy as np
import pytest

from oracle import sp_layout_oracle as lay


def _x(n, H, D, seed):
    return np.random.Generator(np.random.PCG64(seed)).integers(0, 65536, size=(n, H, D), dtype=np.uint16)


def test_hand_case():
    # n = 2 rows, H = 4 heads, D = 1, value = 10*row + head; p = 2: block g holds heads 2g, 2g+1
    x = np.array([[[0], [1], [2], [3]], [[10], [11], [12], [13]]], dtype=np.uint16)
    want = np.array([[[[0], [1]], [[10], [11]]], [[[2], [3]], [[12], [13]]]], dtype=np.uint16)
    assert np.array_equal(lay.pack_heads(x, 2), want)
    assert np.array_equal(lay.unpack_heads(want), x)


@pytest.mark.parametrize("p,n,H,D", [(1, 5, 4, 8), (2, 7, 6, 8), (4, 3, 8, 16), (8, 2, 40, 8)])
def test_simulated_exchange_delivers_head_groups_and_returns_shards(p, n, H, D):
    """The defining property: after every rank packs and block g of rank s is handed to rank g, rank g holds the full
    sequence for head group g; after the way back every rank holds its rows with all heads."""
    full = _x(p * n, H, D, 100 + p)
    shards = [full[s * n:(s + 1) * n] for s in range(p)]
    send = [lay.pack_heads(xs, p) for xs in shards]
    hp = H // p
    for g in range(p):
        recv = np.concatenate([send[s][g] for s in range(p)], axis=0)          # blocks in source-rank order
        assert np.array_equal(recv, full[:, g * hp:(g + 1) * hp, :])
    # way back: rank g owns y_g = [L, hp, D]; its row block s goes to rank s, which stacks them by source rank g
    ys = [full[:, g * hp:(g + 1) * hp, :] for g in range(p)]
    for s in range(p):
        recv = np.stack([ys[g][s * n:(s + 1) * n] for g in range(p)])           # [p, n, hp, D]
        assert np.array_equal(lay.unpack_heads(recv), shards[s])


def test_unpack_inverts_pack_and_p1_is_identity():
    x = _x(9, 12, 4, 7)
    for p in (1, 2, 3, 4, 6, 12):
        assert np.array_equal(lay.unpack_heads(lay.pack_heads(x, p)), x)
    assert np.array_equal(lay.pack_heads(x, 1)[0], x)
    # a transposed map (heads split the other way round) is not the same thing
    assert not np.array_equal(lay.pack_heads(x, 3).reshape(9, 12, 4), x)


# ---------------------------------------------------------------- GPU

@pytest.mark.gpu
@pytest.mark.parametrize("p,n,H,D", [(1, 33, 8, 64), (2, 1000, 24, 128), (4, 19028, 40, 128), (8, 257, 40, 64), (3, 0, 6, 128)])
def test_gpu_pack_unpack_bit_exact(p, n, H, D):
    import torch
    import paper_2604_04335_amd as da
    sys.path.insert(0, os.path.dirname(__file__))
    from gpu_util import to_bits, to_dev
    ctx = da.dit_attn_create(0)
    try:
        x = _x(n, H, D, 200 + p)
        xd = to_dev(x) if n else torch.empty((0, H, D), dtype=torch.bfloat16, device="cuda")
        GUARD = 64
        buf = torch.full((p * n * (H // p) * D + 2 * GUARD,), 0x7FC1, dtype=torch.int16, device="cuda")
        packed = buf[GUARD:GUARD + p * n * (H // p) * D].view(torch.bfloat16).view(p, n, H // p, D)
        st = torch.cuda.current_stream().cuda_stream
        da.dit_attn_sp_pack_heads(ctx, xd, packed, n, H, D, p, st)
        back = torch.empty_like(xd)
        da.dit_attn_sp_unpack_heads(ctx, packed, back, n, H, D, p, st)
        torch.cuda.synchronize()
        assert bool((buf[:GUARD] == 0x7FC1).all()) and bool((buf[-GUARD:] == 0x7FC1).all())
        if n:
            # sampled rows against the loop oracle (the big case would take minutes in pure Python), every row by numpy
            rows = np.unique(np.linspace(0, n - 1, 50).astype(int))
            want = lay.pack_heads(x[rows], p)
            got = packed.view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(got[:, rows], want)
            assert np.array_equal(got, x.reshape(n, p, H // p, D).transpose(1, 0, 2, 3))
            assert np.array_equal(to_bits(back), x)
    finally:
        da.dit_attn_destroy(ctx)


@pytest.mark.gpu
def test_gpu_pack_unpack_beyond_four_gib():
    """2.3e9 elements, 4.6 GB: chunk indices pass 2^28 and byte offsets 2^32.  Device-side seeded bit patterns; the
    oracle checks sampled rows (the first, the last, and rows on either side of the 4 GiB line), the round trip every bit."""
    import torch
    import paper_2604_04335_amd as da
    p, n, H, D = 4, 16500, 1100, 128
    assert n * H * D * 2 > 2 ** 32
    print(f"layout beyond 4 GiB: n={n} H={H} D={D} p={p}", flush=True)
    ctx = da.dit_attn_create(0)
    try:
        gen = torch.Generator(device="cuda").manual_seed(404)
        xd = torch.randint(-32768, 32767, (n, H, D), dtype=torch.int16, device="cuda", generator=gen)
        packed = torch.full((p, n, H // p, D), 0x7FC1, dtype=torch.int16, device="cuda")
        back = torch.full_like(xd, 0x7FC1)
        st = torch.cuda.current_stream().cuda_stream
        da.dit_attn_sp_pack_heads(ctx, xd, packed, n, H, D, p, st)
        da.dit_attn_sp_unpack_heads(ctx, packed, back, n, H, D, p, st)
        torch.cuda.synchronize()
        line = 2 ** 32 // (H * D * 2)
        rows = np.unique(np.concatenate([np.linspace(0, n - 1, 40).astype(int), [line - 1, line, line + 1, n - 2]]))
        rt = torch.from_numpy(rows).cuda()
        want = lay.pack_heads(xd[rt].cpu().numpy(), p)
        assert np.array_equal(packed[:, rt].cpu().numpy(), want)
        assert torch.equal(back, xd)
    finally:
        da.dit_attn_destroy(ctx)


@pytest.mark.gpu
def test_gpu_layout_errors():
    import torch
    import paper_2604_04335_amd as da
    ctx = da.dit_attn_create(0)
    try:
        x = torch.zeros((4, 6, 64), dtype=torch.bfloat16, device="cuda")
        y = torch.zeros_like(x)
        with pytest.raises(da.DitAttnError) as e:
            da.dit_attn_sp_pack_heads(ctx, x, y, 4, 6, 64, 4, None)   # 6 heads do not split 4 ways
        assert e.value.code == -6
        with pytest.raises(da.DitAttnError) as e:
            da.dit_attn_sp_pack_heads(ctx, x, None, 4, 6, 64, 2, None)
        assert e.value.code == -1
    finally:
        da.dit_attn_destroy(ctx)
