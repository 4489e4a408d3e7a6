"""Host-side checks that need no GPU: the library loads, exports what the header declares,
and the work-list covers every (sequence, head, query row) exactly once."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2604_04335_amd as da

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    """Every function that any header under include/ declares."""
    import glob
    names = set()
    for path in sorted(glob.glob(os.path.join(ROOT, "include", "*.h"))):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names |= set(re.findall(r"\b(dit_(?:attn|sched)_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_loads_and_exports_every_declared_symbol():
    lib = da.load_library()
    names = _declared_symbols()
    assert {"dit_attn_create", "dit_attn_varlen_fwd", "dit_attn_destroy", "dit_attn_last_error",
            "dit_attn_plan", "dit_attn_version", "dit_attn_varlen_fwd_lse", "dit_attn_cross_varlen_fwd", "dit_attn_merge",
            "dit_attn_sp_pack_heads", "dit_attn_sp_unpack_heads", "dit_attn_set_kernel", "dit_attn_last_launch_clock", "dit_attn_last_launch_kernel",
            "dit_sched_plan_round", "dit_sched_laxity"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert "gfx950" in da.dit_attn_version()


def test_no_cpu_fallback_when_no_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(da.DitAttnError) as ei:
        da.dit_attn_create(0)
    assert ei.value.code == -4


def _check_plan(lens, H, D):
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    items, bm = da.dit_attn_plan(cu, H, D)
    assert bm in (64, 128, 256)
    T = int(cu[-1])
    cover = np.zeros((T, H), dtype=np.int32)
    seq_of = np.repeat(np.arange(len(lens)), lens)
    for q_start, kv_start, kv_len, rh in items.tolist():
        rows, head = rh >> 16, rh & 0xFFFF
        assert 1 <= rows <= bm and 0 <= head < H
        s = seq_of[q_start]
        assert kv_start == cu[s] and kv_len == cu[s + 1] - cu[s]
        assert q_start + rows <= cu[s + 1]
        # tiles start at the sequence start, in steps of block_m
        assert (q_start - kv_start) % bm == 0
        cover[q_start:q_start + rows, head] += 1
    assert np.all(cover == 1)
    # longest first
    kv = items[:, 2]
    assert np.all(np.diff(kv) <= 0)
    return items, bm


@pytest.mark.parametrize("lens,H,D", [
    ([1024], 8, 64),
    ([4352] * 4, 24, 128),
    ([5, 0, 300, 1, 129, 128, 127], 3, 128),
    ([0, 0], 2, 64),
    ([4352, 1280, 20506, 4352, 1280], 2, 128),
])
def test_plan_covers_every_row_once(lens, H, D):
    items, bm = _check_plan(lens, H, D)
    expect = sum(-(-l // bm) for l in lens) * H
    assert len(items) == expect


def test_plan_puts_ragged_tiles_behind_the_whole_tiles_of_their_sequence():
    """Inside a sequence: heads slow and whole query tiles fast (neighbouring workgroups stream the same K/V rows), then
    the ragged last tile of every head (a quicker item, which would take its workgroup out of step with its
    neighbours in the middle of the sequence)."""
    lens, H = [1000, 600], 3
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    items, bm = da.dit_attn_plan(cu, H, 128)
    for s, L in enumerate(lens):
        mine = items[items[:, 1] == cu[s]]
        whole, rows = L // bm, mine[:, 3] >> 16
        assert np.all(rows[:whole * H] == bm) and np.all(rows[whole * H:] == L - whole * bm)
        assert list(mine[:whole * H, 3] & 0xFFFF) == [h for h in range(H) for _ in range(whole)]
        assert list(mine[:whole * H, 0] - cu[s]) == [t * bm for _ in range(H) for t in range(whole)]
        assert list(mine[whole * H:, 3] & 0xFFFF) == list(range(H))
        assert np.all(mine[whole * H:, 0] - cu[s] == whole * bm)


def test_plan_is_independent_of_packing():
    # a sequence's tiles (relative to its start) do not depend on its neighbours
    a, bm = da.dit_attn_plan(np.array([0, 300], dtype=np.int32), 2, 128)
    b, _ = da.dit_attn_plan(np.array([0, 77, 377], dtype=np.int32), 2, 128)
    b = b[b[:, 2] == 300]
    assert np.array_equal(a[:, 0] - a[:, 1], b[:, 0] - b[:, 1]) and np.array_equal(a[:, 3], b[:, 3])


def test_plan_rejects_bad_arguments():
    lib = da.load_library()
    i32p = ctypes.POINTER(ctypes.c_int32)

    def call(cu, n_seqs, H, D):
        arr = np.asarray(cu, dtype=np.int32)
        return lib.dit_attn_plan(arr.ctypes.data_as(i32p), n_seqs, H, D, None, 0, None)

    assert call([0, 4], 1, 2, 128) == 2 * 1
    assert call([1, 4], 1, 2, 128) == -3      # does not start at 0
    assert call([0, 4, 3], 2, 2, 128) == -3   # decreasing
    assert call([0, 4], -1, 2, 128) == -3
    assert call([0, 4], 1, 2, 96) == -2
    assert call([0, 4], 1, 0, 128) == -6
    assert call([0, 4], 1, 70000, 128) == -6
    assert lib.dit_attn_plan(None, 1, 2, 128, None, 0, None) == -1
    # capacity too small
    buf = np.zeros(4, dtype=np.int32)
    arr = np.array([0, 1000], dtype=np.int32)
    assert lib.dit_attn_plan(arr.ctypes.data_as(i32p), 1, 2, 128, buf.ctypes.data_as(i32p), 1, None) == -8


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: `bench.py --gpus N` with N > 1 exits with a message and a non-zero status, before touching a GPU."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


def test_kernel_choice_by_items_per_compute_unit():
    """dit_attn_plan's block_m shows which kernel family a pack gets on a 256-CU device: the 128-row kernel for under
    0.45 256-row items per compute unit and for packs whose second round of such items would be at most 40 % full,
    the 256-row (ping-pong) kernel otherwise.  4096 tokens are 16 items of 256 rows per head."""
    def block_m(lens, heads):
        cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        return da.dit_attn_plan(cu, heads, 128)[1]
    expect = {6: 128, 7: 128, 8: 256, 9: 256, 10: 256, 12: 256, 16: 256, 17: 128, 20: 128, 22: 128, 23: 256, 24: 256, 25: 256,
              32: 256, 40: 256, 41: 256, 48: 256, 49: 256, 64: 256}
    for heads, bm in expect.items():
        assert block_m([4096], heads) == bm, heads
    assert block_m([20506], 24) == 256
    assert block_m([4352] * 4, 24) == 256
    assert block_m([1024], 8) == 128


def test_plan_cache_evicts_least_recently_used_unpinned_pack():
    """A pack whose launch was recorded into a HIP graph is pinned and never evicted; among the others the least
    recently used one goes; when all are pinned nothing is evicted (the cache grows)."""
    v = da.dit_attn_plan_cache_victim
    assert v([5, 3, 9, 4], [0, 0, 0, 0]) == 1
    assert v([5, 3, 9, 4], [0, 1, 0, 0]) == 3
    assert v([5, 3, 9, 4], [0, 1, 0, 1]) == 0
    assert v([5, 3, 9, 4], [1, 1, 0, 1]) == 2
    assert v([5, 3, 9, 4], [1, 1, 1, 1]) == -1
    assert v([], []) == -1
    assert v([7], [0]) == 0
    # ties: the first of equal use counts
    assert v([2, 2, 2], [1, 0, 0]) == 1
