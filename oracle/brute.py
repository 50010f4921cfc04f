"""ctypes loader for the scalar C twin (brute_attn.c).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "brute_attn.c")
_LIB = os.path.join(_HERE, "libbrute_attn.so")
_DTYPE_CODE = {"f32": 0, "bf16": 1, "fp8_e4m3": 2}


def build(force: bool = False) -> str:
    """Compile the C twin with gcc (plain -O2, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def paged_attention(q, q_lens, k_pages, v_pages, page_table, ctx_lens, *, sm_scale, q_dtype,
                    kv_dtype, k_scale=None, v_scale=None) -> np.ndarray:
    """Decode (q_lens None) or append attention by scalar loops; float64 [rows, Hq, D]."""
    lib = ctypes.CDLL(build())
    fn = lib.brute_paged_attention
    fn.restype = ctypes.c_int
    q = np.ascontiguousarray(q)
    k_pages = np.ascontiguousarray(k_pages)
    v_pages = np.ascontiguousarray(v_pages)
    page_table = np.ascontiguousarray(page_table, dtype=np.int32)
    ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    ql = None if q_lens is None else np.ascontiguousarray(q_lens, dtype=np.int32)
    ks = None if k_scale is None else np.ascontiguousarray(k_scale, dtype=np.float32)
    vs = None if v_scale is None else np.ascontiguousarray(v_scale, dtype=np.float32)
    rows, hq, d = q.shape
    num_pages, hkv, page_size, _ = k_pages.shape
    out = np.empty((rows, hq, d), dtype=np.float64)
    rc = fn(_ptr(q), ctypes.c_int(_DTYPE_CODE[q_dtype]), _ptr(ql), _ptr(k_pages), _ptr(v_pages),
            ctypes.c_int(_DTYPE_CODE[kv_dtype]), _ptr(ks), _ptr(vs), _ptr(page_table), _ptr(ctx_lens),
            ctypes.c_int(len(ctx_lens)), ctypes.c_int(hq), ctypes.c_int(hkv), ctypes.c_int(d),
            ctypes.c_int(page_size), ctypes.c_int64(page_table.shape[1]), ctypes.c_int64(num_pages),
            ctypes.c_float(sm_scale), _ptr(out))
    if rc:
        raise IndexError("page table entry outside the pool")
    return out
