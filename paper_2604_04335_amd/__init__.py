"""Python binding of the MI355X DiT denoising-step attention library.

Argument marshalling only: every step of the computation runs in the HIP
kernels behind the C ABI declared in include/dit_attn.h.  PyTorch is used by
callers for device memory and streams; this module itself only needs ctypes
and numpy, and accepts anything with `data_ptr()` (torch tensors) or a raw
integer device address.

There is no CPU fallback: if the shared library has not been built
(`python -m paper_2604_04335_amd.build`) importing the symbols raises.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

__all__ = [
    "DitAttnError",
    "lib_path",
    "load_library",
    "dit_attn_version",
    "dit_attn_create",
    "dit_attn_varlen_fwd",
    "dit_attn_varlen_fwd_noalloc",
    "dit_attn_varlen_fwd_lse",
    "dit_attn_cross_varlen_fwd",
    "dit_attn_merge",
    "dit_attn_sp_pack_heads",
    "dit_attn_sp_unpack_heads",
    "dit_sched_laxity",
    "dit_sched_plan_round",
    "SchedCandidate",
    "dit_attn_destroy",
    "dit_attn_last_error",
    "dit_attn_plan",
    "dit_attn_plan_cache_victim",
    "dit_attn_set_kernel",
    "dit_attn_set_split_kv",
    "dit_attn_last_launch_clock",
    "dit_attn_last_launch_kernel",
    "KERNEL_AUTO",
    "KERNEL_128",
    "KERNEL_PINGPONG",
    "DitAttention",
]

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
_LIB = None

ERROR_NAMES = {
    0: "DIT_ATTN_OK",
    -1: "DIT_ATTN_ERR_NULL",
    -2: "DIT_ATTN_ERR_HEAD_DIM",
    -3: "DIT_ATTN_ERR_CU_SEQLENS",
    -4: "DIT_ATTN_ERR_HIP",
    -5: "DIT_ATTN_ERR_SCALE",
    -6: "DIT_ATTN_ERR_N_HEADS",
    -7: "DIT_ATTN_ERR_ALIGN",
    -8: "DIT_ATTN_ERR_CAPACITY",
    -9: "DIT_ATTN_ERR_KERNEL",
    -10: "DIT_ATTN_ERR_PARTS",
    -11: "DIT_ATTN_ERR_LIMIT",
    -12: "DIT_ATTN_ERR_CAPTURE",
}


class SchedCandidate(ctypes.Structure):
    """dit_sched_candidate of include/dit_sched.h."""
    _fields_ = [("gpus", ctypes.c_int32), ("gpu_mask", ctypes.c_uint32), ("laxity", ctypes.c_double),
                ("hold", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class DitAttnError(RuntimeError):
    def __init__(self, code: int, message: str = ""):
        self.code = code
        super().__init__(f"{ERROR_NAMES.get(code, code)}: {message}")


def lib_path() -> str:
    return os.path.join(_PKG_DIR, "libdit_attn.so")


def load_library() -> ctypes.CDLL:
    """Load libdit_attn.so (built in-tree).  Raises if it is missing: there is no fallback."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing; build it with `python -m paper_2604_04335_amd.build`")
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.dit_attn_version.restype = ctypes.c_char_p
    lib.dit_attn_version.argtypes = []
    lib.dit_attn_create.restype = ctypes.c_int
    lib.dit_attn_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int]
    lib.dit_attn_varlen_fwd.restype = ctypes.c_int
    lib.dit_attn_varlen_fwd.argtypes = [vp, vp, vp, vp, i32p, i32, i32, i32, ctypes.c_float, vp, vp]
    lib.dit_attn_varlen_fwd_noalloc.restype = ctypes.c_int
    lib.dit_attn_varlen_fwd_noalloc.argtypes = [vp, vp, vp, vp, i32p, i32, i32, i32, ctypes.c_float, vp, vp]
    lib.dit_attn_destroy.restype = None
    lib.dit_attn_destroy.argtypes = [vp]
    lib.dit_attn_varlen_fwd_lse.restype = ctypes.c_int
    lib.dit_attn_varlen_fwd_lse.argtypes = [vp, vp, vp, vp, i32p, i32, i32, i32, ctypes.c_float, vp, vp, vp]
    lib.dit_attn_cross_varlen_fwd.restype = ctypes.c_int
    lib.dit_attn_cross_varlen_fwd.argtypes = [vp, vp, vp, vp, i32p, i32p, i32, i32, i32, ctypes.c_float, vp, vp, vp]
    for fn in (lib.dit_attn_sp_pack_heads, lib.dit_attn_sp_unpack_heads):
        fn.restype = ctypes.c_int
        fn.argtypes = [vp, vp, vp, i64, i32, i32, i32, vp]
    lib.dit_sched_laxity.restype = ctypes.c_double
    lib.dit_sched_laxity.argtypes = [ctypes.c_double, ctypes.c_double, i32, ctypes.c_double]
    f64p = ctypes.POINTER(ctypes.c_double)
    lib.dit_sched_plan_round.restype = ctypes.c_int
    lib.dit_sched_plan_round.argtypes = [i32, ctypes.POINTER(SchedCandidate), i32p, i32, f64p, i32, ctypes.c_double, f64p, i32,
                                         i32p, i32p, i32p, i32p, i32p, i32p, f64p]
    lib.dit_attn_merge.restype = ctypes.c_int
    lib.dit_attn_merge.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), i32, i64, i32, i32, vp, vp, vp]
    lib.dit_attn_last_error.restype = ctypes.c_char_p
    lib.dit_attn_last_error.argtypes = [vp]
    lib.dit_attn_set_split_kv.restype = ctypes.c_int
    lib.dit_attn_set_split_kv.argtypes = [vp, ctypes.c_int]
    lib.dit_attn_set_kernel.restype = ctypes.c_int
    lib.dit_attn_set_kernel.argtypes = [vp, ctypes.c_int]
    lib.dit_attn_last_launch_kernel.restype = ctypes.c_int
    lib.dit_attn_last_launch_kernel.argtypes = [vp]
    lib.dit_attn_last_launch_clock.restype = ctypes.c_int
    lib.dit_attn_last_launch_clock.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    lib.dit_attn_plan_cache_victim.restype = i32
    lib.dit_attn_plan_cache_victim.argtypes = [ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint8), i32]
    lib.dit_attn_plan.restype = i64
    lib.dit_attn_plan.argtypes = [i32p, i32, i32, i32, i32p, i64, i32p]
    _LIB = lib
    return lib


def _ptr(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def _cu_array(cu_seqlens) -> np.ndarray:
    if hasattr(cu_seqlens, "detach"):  # torch tensor: must live on the host
        if cu_seqlens.device.type != "cpu":
            raise ValueError("cu_seqlens must be a host array")
        cu_seqlens = cu_seqlens.detach().numpy()
    return np.ascontiguousarray(cu_seqlens, dtype=np.int32)


def dit_attn_version() -> str:
    return load_library().dit_attn_version().decode()


def dit_attn_last_error(ctx) -> str:
    return load_library().dit_attn_last_error(ctypes.c_void_p(ctx or 0)).decode()


def dit_attn_create(device_id: int = 0) -> int:
    """Returns an opaque context handle (an integer address)."""
    lib = load_library()
    h = ctypes.c_void_p()
    rc = lib.dit_attn_create(ctypes.byref(h), int(device_id))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(None))
    return int(h.value)


KERNEL_AUTO, KERNEL_128, KERNEL_PINGPONG = -1, 0, 1


def dit_attn_set_kernel(ctx, kernel: int) -> None:
    """Force one of the library's kernels for later calls on `ctx` (KERNEL_AUTO: chosen per pack)."""
    rc = load_library().dit_attn_set_kernel(ctypes.c_void_p(ctx), int(kernel))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def dit_attn_set_split_kv(ctx, max_splits: int) -> None:
    """Allow small packs to split every sequence's keys into up to max_splits chunks (1 = off); see include/dit_attn.h."""
    rc = load_library().dit_attn_set_split_kv(ctypes.c_void_p(ctx), int(max_splits))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def dit_attn_last_launch_clock(ctx):
    """(shader clock in MHz, milliseconds) sampled by the first workgroup of the last launch; synchronises the device."""
    mhz, ms = ctypes.c_double(0.0), ctypes.c_double(0.0)
    rc = load_library().dit_attn_last_launch_clock(ctypes.c_void_p(ctx), ctypes.byref(mhz), ctypes.byref(ms))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))
    return mhz.value, ms.value


def dit_attn_last_launch_kernel(ctx) -> int:
    """KERNEL_128 / KERNEL_PINGPONG: the kernel the last forward call launched; KERNEL_AUTO before any."""
    return int(load_library().dit_attn_last_launch_kernel(ctypes.c_void_p(ctx)))


def dit_attn_destroy(ctx) -> None:
    if ctx:
        load_library().dit_attn_destroy(ctypes.c_void_p(ctx))


def dit_attn_varlen_fwd(ctx, q, k, v, cu_seqlens, n_heads: int, head_dim: int, scale: float, out, stream=None,
                        n_seqs: int | None = None) -> None:
    """One denoising-step attention call; see include/dit_attn.h.

    q, k, v, out: device buffers (torch tensors or integer addresses), bf16 [T, n_heads, head_dim].
    cu_seqlens: host int32 sequence of n_seqs + 1 offsets.  stream: integer hipStream_t or None.
    Raises DitAttnError on a non-zero return code.
    """
    lib = load_library()
    cu = _cu_array(cu_seqlens)
    if n_seqs is None:
        n_seqs = len(cu) - 1
    rc = lib.dit_attn_varlen_fwd(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(q)), ctypes.c_void_p(_ptr(k)),
                                 ctypes.c_void_p(_ptr(v)), cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                 int(n_seqs), int(n_heads), int(head_dim), float(scale),
                                 ctypes.c_void_p(_ptr(out)), ctypes.c_void_p(_ptr(stream)))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def dit_attn_varlen_fwd_noalloc(ctx, q, k, v, cu_seqlens, n_heads: int, head_dim: int, scale: float, out, stream=None,
                                n_seqs: int | None = None) -> None:
    """dit_attn_varlen_fwd for callers that cannot allocate: same arguments and result, fixed limits; see include/dit_attn.h."""
    lib = load_library()
    cu = _cu_array(cu_seqlens)
    if n_seqs is None:
        n_seqs = len(cu) - 1
    rc = lib.dit_attn_varlen_fwd_noalloc(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(q)), ctypes.c_void_p(_ptr(k)),
                                         ctypes.c_void_p(_ptr(v)), cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                         int(n_seqs), int(n_heads), int(head_dim), float(scale),
                                         ctypes.c_void_p(_ptr(out)), ctypes.c_void_p(_ptr(stream)))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def dit_attn_varlen_fwd_lse(ctx, q, k, v, cu_seqlens, n_heads: int, head_dim: int, scale: float, out, lse, stream=None,
                            n_seqs: int | None = None) -> None:
    """dit_attn_varlen_fwd that also writes lse (device fp32 [T, n_heads], natural log); see include/dit_attn.h."""
    lib = load_library()
    cu = _cu_array(cu_seqlens)
    if n_seqs is None:
        n_seqs = len(cu) - 1
    rc = lib.dit_attn_varlen_fwd_lse(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(q)), ctypes.c_void_p(_ptr(k)),
                                     ctypes.c_void_p(_ptr(v)), cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                     int(n_seqs), int(n_heads), int(head_dim), float(scale),
                                     ctypes.c_void_p(_ptr(out)), ctypes.c_void_p(_ptr(lse)), ctypes.c_void_p(_ptr(stream)))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def dit_attn_cross_varlen_fwd(ctx, q, k, v, cu_seqlens_q, cu_seqlens_k, n_heads: int, head_dim: int, scale: float, out,
                              lse=None, stream=None, n_seqs: int | None = None) -> None:
    """Cross-attention with separate query and key boundaries; lse may be None.  See include/dit_attn.h."""
    lib = load_library()
    cq = _cu_array(cu_seqlens_q)
    ck = None if cu_seqlens_k is None else _cu_array(cu_seqlens_k)
    if n_seqs is None:
        n_seqs = len(cq) - 1
    i32p = ctypes.POINTER(ctypes.c_int32)
    rc = lib.dit_attn_cross_varlen_fwd(ctypes.c_void_p(ctx), ctypes.c_void_p(_ptr(q)), ctypes.c_void_p(_ptr(k)),
                                       ctypes.c_void_p(_ptr(v)), cq.ctypes.data_as(i32p),
                                       None if ck is None else ck.ctypes.data_as(i32p),
                                       int(n_seqs), int(n_heads), int(head_dim), float(scale),
                                       ctypes.c_void_p(_ptr(out)), ctypes.c_void_p(_ptr(lse)), ctypes.c_void_p(_ptr(stream)))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def dit_attn_merge(ctx, o_parts, lse_parts, total_rows: int, n_heads: int, head_dim: int, out, lse_out=None,
                   stream=None) -> None:
    """Merge partial results over disjoint key sets; o_parts / lse_parts: sequences of device buffers.  See the header."""
    lib = load_library()
    n = len(o_parts)
    vp = ctypes.c_void_p
    o_arr = (vp * max(n, 1))(*[vp(_ptr(x)) for x in o_parts])
    l_arr = (vp * max(n, 1))(*[vp(_ptr(x)) for x in lse_parts]) if len(lse_parts) == n else None
    if l_arr is None:
        raise ValueError("o_parts and lse_parts must have the same length")
    rc = lib.dit_attn_merge(vp(ctx), o_arr, l_arr, int(n), int(total_rows), int(n_heads), int(head_dim), vp(_ptr(out)),
                            vp(_ptr(lse_out)), vp(_ptr(stream)))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def _sp_layout(name, ctx, src, dst, n_rows, n_heads, head_dim, sp_degree, stream):
    vp = ctypes.c_void_p
    rc = getattr(load_library(), name)(vp(ctx), vp(_ptr(src)), vp(_ptr(dst)), int(n_rows), int(n_heads), int(head_dim),
                                       int(sp_degree), vp(_ptr(stream)))
    if rc != 0:
        raise DitAttnError(rc, dit_attn_last_error(ctx))


def dit_attn_sp_pack_heads(ctx, src, dst, n_rows: int, n_heads: int, head_dim: int, sp_degree: int, stream=None) -> None:
    """[n_rows, H, D] -> [p, n_rows, H/p, D] (block g goes to rank g); see include/dit_attn.h."""
    _sp_layout("dit_attn_sp_pack_heads", ctx, src, dst, n_rows, n_heads, head_dim, sp_degree, stream)


def dit_attn_sp_unpack_heads(ctx, src, dst, n_rows: int, n_heads: int, head_dim: int, sp_degree: int, stream=None) -> None:
    """[p, n_rows, H/p, D] -> [n_rows, H, D] (block g came from rank g); see include/dit_attn.h."""
    _sp_layout("dit_attn_sp_unpack_heads", ctx, src, dst, n_rows, n_heads, head_dim, sp_degree, stream)


def dit_attn_plan(cu_seqlens, n_heads: int, head_dim: int):
    """Host-only: the ordered work-list as an int32 array [n_items, 4] and the tile height block_m."""
    lib = load_library()
    cu = _cu_array(cu_seqlens)
    n_seqs = len(cu) - 1
    cu_p = cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    bm = ctypes.c_int32(0)
    n = lib.dit_attn_plan(cu_p, n_seqs, int(n_heads), int(head_dim), None, 0, ctypes.byref(bm))
    if n < 0:
        raise DitAttnError(int(n), "dit_attn_plan")
    items = np.zeros((max(int(n), 1), 4), dtype=np.int32)
    n2 = lib.dit_attn_plan(cu_p, n_seqs, int(n_heads), int(head_dim),
                           items.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), int(items.shape[0]), ctypes.byref(bm))
    if n2 < 0:
        raise DitAttnError(int(n2), "dit_attn_plan")
    return items[:int(n2)], int(bm.value)


def dit_attn_plan_cache_victim(last_use, pinned) -> int:
    """Host-only: which of the cached packs (use counters, pin flags) the plan cache evicts next; -1 if all are pinned."""
    lu = np.ascontiguousarray(last_use, dtype=np.uint64)
    pn = np.ascontiguousarray(pinned, dtype=np.uint8)
    assert lu.size == pn.size
    return int(load_library().dit_attn_plan_cache_victim(lu.ctypes.data_as(ctypes.POINTER(ctypes.c_uint64)),
                                                         pn.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), int(lu.size)))


class DitAttention:
    """Owns one context; `forward` takes torch tensors and uses torch's current stream."""

    def __init__(self, device_id: int = 0):
        self.device_id = int(device_id)
        self.ctx = dit_attn_create(self.device_id)

    def forward(self, q, k, v, cu_seqlens, scale: float | None = None, out=None, stream=None):
        import torch  # device memory and streams only

        T, H, D = q.shape
        assert q.dtype == torch.bfloat16 and q.is_contiguous() and k.is_contiguous() and v.is_contiguous()
        assert k.shape == q.shape and v.shape == q.shape
        if out is None:
            out = torch.empty_like(q)
        if scale is None:
            scale = float(D) ** -0.5
        if stream is None:
            stream = torch.cuda.current_stream(q.device).cuda_stream
        dit_attn_varlen_fwd(self.ctx, q, k, v, cu_seqlens, H, D, scale, out, stream)
        return out

    __call__ = forward

    def close(self):
        if self.ctx:
            dit_attn_destroy(self.ctx)
            self.ctx = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def dit_sched_laxity(deadline: float, t_now: float, steps_remaining: int, t_step: float) -> float:
    """Eq. 1 of the paper for a configuration; see include/dit_sched.h."""
    return float(load_library().dit_sched_laxity(float(deadline), float(t_now), int(steps_remaining), float(t_step)))


def dit_sched_plan_round(n_gpus: int, videos, image_deadlines, t_now: float, t_img):
    """One round of the paper's Algorithm 1 (include/dit_sched.h).  videos: per video a sequence of candidates, each a
    SchedCandidate or a tuple (gpus, gpu_mask, laxity, hold).  Returns a dict with choice, video_gpus, image_batch,
    image_gpu (one GPU id per image batch), recoverable, utility.  Raises DitAttnError on an error code."""
    lib = load_library()
    flat, offs = [], [0]
    for cands in videos:
        for c in cands:
            flat.append(c if isinstance(c, SchedCandidate) else SchedCandidate(int(c[0]), int(c[1]), float(c[2]), int(bool(c[3])), 0))
        offs.append(len(flat))
    arr = (SchedCandidate * max(len(flat), 1))(*flat)
    offs_a = np.asarray(offs, dtype=np.int32)
    dl = np.ascontiguousarray(image_deadlines, dtype=np.float64)
    timg = np.ascontiguousarray(t_img, dtype=np.float64)
    G, n_img = len(videos), int(dl.size)
    choice = np.zeros(max(G, 1), dtype=np.int32)
    batch = np.zeros(max(n_img, 1), dtype=np.int32)
    gpu = np.zeros(max(int(n_gpus), 1), dtype=np.int32)
    nb, vg, rec = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    util = ctypes.c_double(0.0)
    i32p, f64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_double)
    rc = lib.dit_sched_plan_round(int(n_gpus), arr, offs_a.ctypes.data_as(i32p), G,
                                  dl.ctypes.data_as(f64p) if n_img else None, n_img, float(t_now),
                                  timg.ctypes.data_as(f64p), int(timg.size), choice.ctypes.data_as(i32p),
                                  batch.ctypes.data_as(i32p), gpu.ctypes.data_as(i32p), ctypes.byref(nb), ctypes.byref(vg),
                                  ctypes.byref(rec), ctypes.byref(util))
    if rc != 0:
        raise DitAttnError(rc, "dit_sched_plan_round")
    return {"choice": choice[:G].tolist(), "video_gpus": int(vg.value), "image_batch": batch[:n_img].tolist(),
            "image_gpu": gpu[:int(nb.value)].tolist(), "n_batches": int(nb.value), "recoverable": int(rec.value),
            "utility": float(util.value)}
