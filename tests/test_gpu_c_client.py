"""The C ABI called from C code (tests/c_abi_client.c: dlopen, hipMalloc, plain pointers): no torch tensor, no
Python marshalling between the caller and the library.  The batch goes to the C code as raw files, the oracle
sees the very same bytes, and the output file is compared with the oracle like any other parity case."""
from __future__ import annotations

import ctypes
import os

import numpy as np
import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check, oracle_append, oracle_decode

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
CLIENT = os.path.join(HERE, "libc_abi_client.so")
CODE = {"f32": B.F32, "bf16": B.BF16, "fp8_e4m3": B.FP8_E4M3}


def _dump(d, name, t):
    if t is not None:
        W.raw_numpy(t).tofile(os.path.join(d, name + ".bin"))


@pytest.mark.parametrize("mode,qd,kvd", [("decode", "bf16", "bf16"), ("decode", "f32", "f32"), ("append", "bf16", "fp8_e4m3")])
def test_c_code_calling_the_abi_gets_the_oracles_result(tmp_path, mode, qd, kvd):
    if not os.path.exists(CLIENT):
        pytest.fail(f"{CLIENT} has not been built (__graft_entry__.build() compiles it)")
    qlen = ("const", 1) if mode == "decode" else ("uniform", 1, 90)
    w = W.Workload(f"c_{mode}", 7, 8, 2, 128 if qd == "bf16" else 64, qd, kvd, ("uniform", 1, 700), qlen=qlen, seed=91,
                   ctx_is_prefix=(mode == "append"))
    b = W.build(w, "cpu")                                   # host tensors only: device memory is the C code's business
    d = str(tmp_path)
    for name in ("q", "k_pages", "v_pages", "page_table", "ctx_lens", "q_lens", "q_offsets", "k_scale", "v_scale"):
        _dump(d, name, getattr(b, name))
    args = ["c_abi_client", B.LIB_PATH, d, mode, w.batch, w.num_q_heads, w.num_kv_heads, w.head_dim, CODE[qd], CODE[kvd],
            b.page_table.shape[1], b.num_pages, b.total_q, int(b.q_lens_host.max()), repr(float(w.sm_scale))]
    client = ctypes.CDLL(CLIENT)
    client.c_abi_client_run.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_char_p)]
    client.c_abi_client_error.restype = ctypes.c_char_p
    argv = (ctypes.c_char_p * len(args))(*[str(a).encode() for a in args])
    rc = client.c_abi_client_run(len(args), argv)
    assert rc == 0, client.c_abi_client_error().decode()
    dt = np.float32 if qd == "f32" else np.uint16
    raw = np.fromfile(os.path.join(d, "out.bin"), dtype=dt).reshape(tuple(b.q.shape))
    got = torch.from_numpy(raw) if qd == "f32" else torch.from_numpy(raw.view(np.int16)).view(torch.bfloat16)
    ref = oracle_decode(b) if mode == "decode" else oracle_append(b)
    check(got, ref, qd, f"C client, {mode} {qd}/{kvd}")
