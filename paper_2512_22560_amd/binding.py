"""ctypes binding of librollattn's C ABI for torch tensors.

Argument marshalling only: every step of the attention path (planning, paged loads,
softmax, the split-K merge) runs in the library's HIP kernels.  torch supplies device
memory and the current stream.  There is no fallback: if the shared library has not been
built, `lib()` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librollattn.so")

F32, BF16, FP8_E4M3 = 0, 1, 2
EXPORTS = (
    "attn_decode", "attn_decode_static", "rollattn_static_scratch_bytes", "rollattn_static_init", "attn_append", "attn_decode_lse", "attn_append_lse", "attn_merge", "attn_step", "attn_decode_shared",
    "kv_write", "rollattn_workspace_bytes",
    "rollattn_step_workspace_bytes", "rollattn_shared_workspace_bytes", "rollattn_debug_gather",
    "rollattn_debug_check_inputs",
    "rollattn_debug_plan", "rollattn_plan_capacity", "rollattn_plan_workers", "rollattn_debug_read_plan", "rollattn_debug_set_decode_workers", "rollattn_debug_read_append_plan", "rollattn_append_plan_capacity", "rollattn_step_append_offset",
    "rollattn_profile_enable", "rollattn_profile_read", "rollattn_profile_append_clock", "rollattn_status_string",
    "rollattn_last_hip_error", "rollattn_version",
)


class Desc(ctypes.Structure):
    _fields_ = [
        ("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
        ("num_pages", ctypes.c_int64), ("q_dtype", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
        ("sm_scale", ctypes.c_float), ("k_scale", ctypes.c_void_p), ("v_scale", ctypes.c_void_p),
    ]


class RollattnError(RuntimeError):
    def __init__(self, status: int, where: str):
        l = lib()
        msg = l.rollattn_status_string(status).decode()
        if status == -6:
            msg += ": " + l.rollattn_last_hip_error().decode()
        super().__init__(f"{where}: {msg} (status {status})")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2512_22560_amd.build` "
                               "(or __graft_entry__.build())")
        l = ctypes.CDLL(LIB_PATH)
        vp, i32, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)
        dp = ctypes.POINTER(Desc)
        l.attn_decode.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        l.attn_decode.restype = ctypes.c_int
        l.attn_decode_static.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp]
        l.attn_decode_static.restype = ctypes.c_int
        l.rollattn_static_scratch_bytes.argtypes = []
        l.rollattn_static_scratch_bytes.restype = ctypes.c_size_t
        l.rollattn_static_init.argtypes = []
        l.rollattn_static_init.restype = ctypes.c_int
        l.attn_append.argtypes = [dp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        l.attn_append.restype = ctypes.c_int
        l.attn_decode_lse.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        l.attn_decode_lse.restype = ctypes.c_int
        l.attn_append_lse.argtypes = [dp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        l.attn_append_lse.restype = ctypes.c_int
        l.attn_merge.argtypes = [dp, ctypes.c_int64, vp, vp, vp, vp, vp, vp, vp]
        l.attn_merge.restype = ctypes.c_int
        l.attn_step.argtypes = [dp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        l.attn_step.restype = ctypes.c_int
        l.rollattn_step_workspace_bytes.argtypes = [dp, i32]
        l.rollattn_step_workspace_bytes.restype = ctypes.c_size_t
        l.attn_decode_shared.argtypes = [dp, vp, vp, vp, vp, vp, i32, vp, vp, vp, ctypes.c_size_t, vp]
        l.attn_decode_shared.restype = ctypes.c_int
        l.rollattn_shared_workspace_bytes.argtypes = [dp, i32]
        l.rollattn_shared_workspace_bytes.restype = ctypes.c_size_t
        l.kv_write.argtypes = [dp, vp, vp, vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        l.kv_write.restype = ctypes.c_int
        l.rollattn_workspace_bytes.argtypes = [dp, i32]
        l.rollattn_workspace_bytes.restype = ctypes.c_size_t
        l.rollattn_debug_gather.argtypes = [dp, vp, vp, vp, i32, i32, vp, vp]
        l.rollattn_debug_gather.restype = ctypes.c_int
        l.rollattn_debug_check_inputs.argtypes = [dp, vp, vp, vp, vp, vp, i32p, vp]
        l.rollattn_debug_check_inputs.restype = ctypes.c_int
        l.rollattn_debug_plan.argtypes = [dp, i32p, i32p, i32p, i32p, i32p]
        l.rollattn_debug_plan.restype = ctypes.c_int
        l.rollattn_plan_capacity.argtypes = [dp]
        l.rollattn_plan_capacity.restype = ctypes.c_int32
        l.rollattn_plan_workers.argtypes = [dp]
        l.rollattn_plan_workers.restype = ctypes.c_int32
        l.rollattn_debug_read_plan.argtypes = [dp, vp, i32p, i32p, i32p, vp]
        l.rollattn_debug_read_plan.restype = ctypes.c_int
        l.rollattn_debug_read_append_plan.argtypes = [dp, vp, i32, i32p, i32p, vp]
        l.rollattn_debug_read_append_plan.restype = ctypes.c_int
        l.rollattn_append_plan_capacity.argtypes = [dp, i32]
        l.rollattn_append_plan_capacity.restype = ctypes.c_int32
        l.rollattn_step_append_offset.argtypes = [dp]
        l.rollattn_step_append_offset.restype = ctypes.c_size_t
        l.rollattn_debug_set_decode_workers.argtypes = [ctypes.c_int32]
        l.rollattn_debug_set_decode_workers.restype = ctypes.c_int32
        l.rollattn_profile_enable.argtypes = [ctypes.c_int]
        l.rollattn_profile_enable.restype = ctypes.c_int
        l.rollattn_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_int]
        l.rollattn_profile_read.restype = ctypes.c_int
        l.rollattn_profile_append_clock.argtypes = [ctypes.POINTER(ctypes.c_double)]
        l.rollattn_profile_append_clock.restype = ctypes.c_int
        l.rollattn_status_string.argtypes = [ctypes.c_int]
        l.rollattn_status_string.restype = ctypes.c_char_p
        l.rollattn_last_hip_error.argtypes = []
        l.rollattn_last_hip_error.restype = ctypes.c_char_p
        l.rollattn_version.argtypes = []
        l.rollattn_version.restype = ctypes.c_int
        _lib = l
    return _lib


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype in (torch.uint8, torch.float8_e4m3fn):
        return FP8_E4M3
    raise TypeError(f"unsupported element type {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def make_desc(q, k_pages, page_table, *, sm_scale, k_scale=None, v_scale=None, batch=None) -> Desc:
    num_pages, hkv, page_size, d = k_pages.shape
    return Desc(
        batch=int(page_table.shape[0] if batch is None else batch), num_q_heads=int(q.shape[1]),
        num_kv_heads=int(hkv), head_dim=int(d), page_size=int(page_size),
        max_pages_per_seq=int(page_table.shape[1]), num_pages=int(num_pages), q_dtype=_dtype_code(q),
        kv_dtype=_dtype_code(k_pages), sm_scale=float(sm_scale),
        k_scale=None if k_scale is None else k_scale.data_ptr(),
        v_scale=None if v_scale is None else v_scale.data_ptr(),
    )


def workspace_bytes(desc: Desc, total_q: int) -> int:
    return int(lib().rollattn_workspace_bytes(ctypes.byref(desc), int(total_q)))


def alloc_workspace(desc: Desc, total_q: int, device) -> torch.Tensor:
    n = workspace_bytes(desc, total_q)
    if n == 0:
        raise RollattnError(-2, "rollattn_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _check_contig(*ts):
    for t in ts:
        if t is not None and not t.is_contiguous():
            raise ValueError("librollattn takes dense row-major arrays")


def attn_decode(q, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, k_scale=None, v_scale=None,
                out=None, workspace=None, stream=None) -> torch.Tensor:
    """out[b, h, :] = attention of q[b, h, :] over trajectory b's cached tokens."""
    _check_contig(q, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale, out)
    desc = make_desc(q, k_pages, page_table, sm_scale=sm_scale, k_scale=k_scale, v_scale=v_scale)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        workspace = alloc_workspace(desc, q.shape[0], q.device)
    rc = lib().attn_decode(ctypes.byref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(page_table),
                           _ptr(ctx_lens), _ptr(out), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_decode")
    return out


def attn_decode_static(q, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, k_scale=None, v_scale=None,
                       out, stream=None) -> torch.Tensor:
    """attn_decode without a workspace: the library's built-in scratch array takes its place.  `out` is the
    caller's (this call allocates nothing)."""
    _check_contig(q, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale, out)
    desc = make_desc(q, k_pages, page_table, sm_scale=sm_scale, k_scale=k_scale, v_scale=v_scale)
    rc = lib().attn_decode_static(ctypes.byref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(page_table),
                                  _ptr(ctx_lens), _ptr(out), _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_decode_static")
    return out


def attn_append(q_chunk, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, max_q_len,
                k_scale=None, v_scale=None, out=None, workspace=None, stream=None) -> torch.Tensor:
    """Rows of q_chunk (packed by trajectory) attend causally inside their chunk and fully to the prefix."""
    _check_contig(q_chunk, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale, out)
    desc = make_desc(q_chunk, k_pages, page_table, sm_scale=sm_scale, k_scale=k_scale, v_scale=v_scale)
    total_q = int(q_chunk.shape[0])
    if out is None:
        out = torch.empty_like(q_chunk)
    if workspace is None:
        workspace = alloc_workspace(desc, total_q, q_chunk.device)
    rc = lib().attn_append(ctypes.byref(desc), _ptr(q_chunk), _ptr(q_lens), _ptr(q_offsets), total_q,
                           int(max_q_len), _ptr(k_pages), _ptr(v_pages), _ptr(page_table), _ptr(ctx_lens),
                           _ptr(out), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_append")
    return out


def attn_decode_lse(q, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, k_scale=None, v_scale=None,
                    out=None, lse=None, workspace=None, stream=None):
    """attn_decode plus lse [B, Hq] float32: log2 of every row's softmax denominator (-inf for an empty context)."""
    _check_contig(q, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale, out, lse)
    desc = make_desc(q, k_pages, page_table, sm_scale=sm_scale, k_scale=k_scale, v_scale=v_scale)
    if out is None:
        out = torch.empty_like(q)
    if lse is None:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(desc, q.shape[0], q.device)
    rc = lib().attn_decode_lse(ctypes.byref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(page_table), _ptr(ctx_lens),
                               _ptr(out), _ptr(lse), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_decode_lse")
    return out, lse


def attn_append_lse(q_chunk, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, max_q_len,
                    k_scale=None, v_scale=None, out=None, lse=None, workspace=None, stream=None):
    """attn_append plus lse [total_q, Hq] float32."""
    _check_contig(q_chunk, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale, out, lse)
    desc = make_desc(q_chunk, k_pages, page_table, sm_scale=sm_scale, k_scale=k_scale, v_scale=v_scale)
    total_q = int(q_chunk.shape[0])
    if out is None:
        out = torch.empty_like(q_chunk)
    if lse is None:
        lse = torch.empty(q_chunk.shape[:2], dtype=torch.float32, device=q_chunk.device)
    if workspace is None:
        workspace = alloc_workspace(desc, total_q, q_chunk.device)
    rc = lib().attn_append_lse(ctypes.byref(desc), _ptr(q_chunk), _ptr(q_lens), _ptr(q_offsets), total_q, int(max_q_len),
                               _ptr(k_pages), _ptr(v_pages), _ptr(page_table), _ptr(ctx_lens), _ptr(out), _ptr(lse),
                               _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_append_lse")
    return out, lse


def attn_merge(o1, lse1, o2, lse2, *, out=None, lse_out=None, stream=None):
    """Attention over the union of two disjoint token ranges from (o, lse) over each; returns (out, lse_out)."""
    _check_contig(o1, lse1, o2, lse2, out, lse_out)
    rows, hq, d = o1.shape
    desc = Desc(batch=0, num_q_heads=int(hq), num_kv_heads=int(hq), head_dim=int(d), page_size=16, max_pages_per_seq=1,
                num_pages=0, q_dtype=_dtype_code(o1), kv_dtype=_dtype_code(o1), sm_scale=1.0, k_scale=None, v_scale=None)
    if out is None:
        out = torch.empty_like(o1)
    if lse_out is None:
        lse_out = torch.empty_like(lse1)
    rc = lib().attn_merge(ctypes.byref(desc), int(rows), _ptr(o1), _ptr(lse1), _ptr(o2), _ptr(lse2), _ptr(out), _ptr(lse_out),
                          _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_merge")
    return out, lse_out


def attn_step(q, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, max_q_len,
              k_scale=None, v_scale=None, out=None, workspace=None, stream=None) -> torch.Tensor:
    """One engine step on a mixed batch: trajectories with one row take the decode path, those with a chunk the
    append path, decided on the device from q_lens."""
    _check_contig(q, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale, out)
    desc = make_desc(q, k_pages, page_table, sm_scale=sm_scale, k_scale=k_scale, v_scale=v_scale)
    total_q = int(q.shape[0])
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        n = int(lib().rollattn_step_workspace_bytes(ctypes.byref(desc), total_q))
        workspace = torch.empty(max(n, 256), dtype=torch.uint8, device=q.device)
    rc = lib().attn_step(ctypes.byref(desc), _ptr(q), _ptr(q_lens), _ptr(q_offsets), total_q, int(max_q_len),
                         _ptr(k_pages), _ptr(v_pages), _ptr(page_table), _ptr(ctx_lens), _ptr(out), _ptr(workspace),
                         workspace.numel(), _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_step")
    return out


def attn_decode_shared(q, k_pages, v_pages, page_table, ctx_lens, *, group_size, shared_lens, sm_scale, k_scale=None,
                       v_scale=None, out=None, workspace=None, stream=None) -> torch.Tensor:
    """attn_decode for groups of group_size consecutive trajectories whose tables alias the pages of their first
    shared_lens[group] tokens; those pages are read once per group."""
    _check_contig(q, k_pages, v_pages, page_table, ctx_lens, shared_lens, k_scale, v_scale, out)
    desc = make_desc(q, k_pages, page_table, sm_scale=sm_scale, k_scale=k_scale, v_scale=v_scale)
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        n = int(lib().rollattn_shared_workspace_bytes(ctypes.byref(desc), int(group_size)))
        if n == 0:
            raise RollattnError(-2, "rollattn_shared_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=q.device)
    rc = lib().attn_decode_shared(ctypes.byref(desc), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(page_table), _ptr(ctx_lens),
                                  int(group_size), _ptr(shared_lens), _ptr(out), _ptr(workspace), workspace.numel(), _stream(stream))
    if rc:
        raise RollattnError(rc, "attn_decode_shared")
    return out


def kv_write(k_new, v_new, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, *, max_q_len,
             k_scale=None, v_scale=None, stream=None) -> None:
    """Puts the new tokens' K / V rows (packed by trajectory, [total_q, Hkv, D]) into the pools in place;
    FP8 pools also get their page scales updated in place."""
    _check_contig(k_new, v_new, q_lens, q_offsets, k_pages, v_pages, page_table, ctx_lens, k_scale, v_scale)
    desc = make_desc(k_new, k_pages, page_table, sm_scale=1.0)
    rc = lib().kv_write(ctypes.byref(desc), _ptr(k_new), _ptr(v_new), _ptr(q_lens), _ptr(q_offsets), int(k_new.shape[0]),
                        int(max_q_len), _ptr(k_pages), _ptr(v_pages), _ptr(page_table), _ptr(ctx_lens), _ptr(k_scale),
                        _ptr(v_scale), _stream(stream))
    if rc:
        raise RollattnError(rc, "kv_write")


def debug_gather(pages, page_table, ctx_lens, b, kv_head, length, stream=None) -> torch.Tensor:
    """Logical tokens [0, length) of (trajectory b, KV head) copied out of a pool, unconverted."""
    kv = _dtype_code(pages)
    desc = Desc(batch=int(page_table.shape[0]), num_q_heads=int(pages.shape[1]), num_kv_heads=int(pages.shape[1]),
                head_dim=int(pages.shape[3]), page_size=int(pages.shape[2]), max_pages_per_seq=int(page_table.shape[1]),
                num_pages=int(pages.shape[0]), q_dtype=F32 if kv == F32 else BF16, kv_dtype=kv, sm_scale=1.0,
                k_scale=None, v_scale=None)
    dst = torch.empty((int(length), pages.shape[3]), dtype=pages.dtype, device=pages.device)
    rc = lib().rollattn_debug_gather(ctypes.byref(desc), _ptr(pages), _ptr(page_table), _ptr(ctx_lens), int(b),
                                     int(kv_head), _ptr(dst), _stream(stream))
    if rc:
        raise RollattnError(rc, "rollattn_debug_gather")
    return dst


def check_inputs(desc: Desc, page_table, ctx_lens, q_lens=None, q_offsets=None, stream=None) -> np.ndarray:
    """Device-side check of lengths, page ids and the chunk description: int32[4] counts of violations (all zero
    for inputs the attention calls may be given).  Synchronises."""
    counts_dev = torch.empty(4, dtype=torch.int32, device=page_table.device)
    out = np.zeros(4, dtype=np.int32)
    rc = lib().rollattn_debug_check_inputs(ctypes.byref(desc), _ptr(page_table), _ptr(ctx_lens), _ptr(q_lens), _ptr(q_offsets),
                                           _ptr(counts_dev), out.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), _stream(stream))
    if rc:
        raise RollattnError(rc, "rollattn_debug_check_inputs")
    return out


def debug_plan(desc: Desc, ctx_lens_host: np.ndarray):
    """Host twin of the decode partition: (per, total, segments [n, 6] int32)."""
    l = lib()
    cap = int(l.rollattn_plan_capacity(ctypes.byref(desc)))
    lens = np.ascontiguousarray(ctx_lens_host, dtype=np.int32)
    segs = np.zeros((max(cap, 1), 6), dtype=np.int32)
    per, total, n = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    i32p = ctypes.POINTER(ctypes.c_int32)
    rc = l.rollattn_debug_plan(ctypes.byref(desc), lens.ctypes.data_as(i32p), ctypes.byref(per), ctypes.byref(total),
                               segs.ctypes.data_as(i32p), ctypes.byref(n))
    if rc:
        raise RollattnError(rc, "rollattn_debug_plan")
    return int(per.value), int(total.value), segs[: n.value].copy()


def plan_workers(desc: Desc) -> int:
    return int(lib().rollattn_plan_workers(ctypes.byref(desc)))


def read_plan(desc: Desc, workspace: torch.Tensor, stream=None):
    """The plan the last attn_decode call left in `workspace`: (per, total, starts [W, 4] int32)."""
    l = lib()
    workers = plan_workers(desc)
    starts = np.zeros((max(workers, 1), 4), dtype=np.int32)
    per, total = ctypes.c_int32(0), ctypes.c_int32(0)
    i32p = ctypes.POINTER(ctypes.c_int32)
    rc = l.rollattn_debug_read_plan(ctypes.byref(desc), _ptr(workspace), ctypes.byref(per), ctypes.byref(total),
                                    starts.ctypes.data_as(i32p), _stream(stream))
    if rc:
        raise RollattnError(rc, "rollattn_debug_read_plan")
    return int(per.value), int(total.value), starts


def read_append_plan(desc: Desc, workspace: torch.Tensor, total_q: int, stream=None) -> np.ndarray:
    """The tile list the last attn_append call left in `workspace`: int32 [n_tiles, 2] of (b, first row in the chunk)."""
    l = lib()
    cap = int(l.rollattn_append_plan_capacity(ctypes.byref(desc), int(total_q)))
    tiles = np.zeros((max(cap, 1), 2), dtype=np.int32)
    n = ctypes.c_int32(0)
    i32p = ctypes.POINTER(ctypes.c_int32)
    rc = l.rollattn_debug_read_append_plan(ctypes.byref(desc), _ptr(workspace), int(total_q), ctypes.byref(n),
                                           tiles.ctypes.data_as(i32p), _stream(stream))
    if rc:
        raise RollattnError(rc, "rollattn_debug_read_append_plan")
    return tiles[: n.value].copy()


def profile_enable(on: bool) -> None:
    lib().rollattn_profile_enable(1 if on else 0)


def profile_read(cap: int = 1024) -> np.ndarray:
    buf = (ctypes.c_float * cap)()
    n = lib().rollattn_profile_read(buf, cap)
    return np.frombuffer(buf, dtype=np.float32, count=n).copy()


def profile_append_clock() -> float:
    """Shader clock (MHz) the MFMA append kernel ran at over the profiled launches since the last call; 0.0 if none."""
    mhz = ctypes.c_double(0.0)
    rc = lib().rollattn_profile_append_clock(ctypes.byref(mhz))
    if rc != 0:
        raise RollattnError(rc, "rollattn_profile_append_clock")
    return float(mhz.value)


def set_decode_workers(workers: int) -> int:
    """Testing aid: cut every decode partition for this many workers (0: the default, all of them); returns the previous setting."""
    return int(lib().rollattn_debug_set_decode_workers(int(workers)))
