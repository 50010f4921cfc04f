"""attn_decode_static: the decode call whose plan and split partials live in the library's built-in scratch array.
It must give what attn_decode gives on the same arguments (same kernels, so bit for bit; the parity bar against
the oracle is checked as well), on two calls in a row that share the array, the second on a smaller batch, and
it must not change the amount of free device memory."""
from __future__ import annotations

import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check, gpu_decode, oracle_decode

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _static(batch, out):
    w = batch.workload
    return B.attn_decode_static(batch.q, batch.k_pages, batch.v_pages, batch.page_table, batch.ctx_lens,
                                sm_scale=w.sm_scale, k_scale=batch.k_scale, v_scale=batch.v_scale, out=out)


@pytest.mark.parametrize("name,hq,hkv,d,qd,kvd", [
    ("static_bf16", 32, 8, 128, "bf16", "bf16"), ("static_fp8", 64, 4, 128, "bf16", "fp8_e4m3"),
    ("static_f32", 8, 2, 64, "f32", "f32"),
])
def test_two_calls_in_a_row_match_attn_decode(name, hq, hkv, d, qd, kvd):
    assert B.lib().rollattn_static_init() == 0
    assert B.lib().rollattn_static_scratch_bytes() == 36 << 20
    # long-tailed lengths: many rows are split over several workers, so the partials in the array are used
    big = W.build(W.Workload(name, 48, hq, hkv, d, qd, kvd, ("lognormal", 1500, 0.9, 1, 9000), seed=W.BASE_SEED + 71), DEV)
    small = W.build(W.Workload(name + "_small", 5, hq, hkv, d, qd, kvd, ("uniform", 1, 400), seed=W.BASE_SEED + 72), DEV)
    want_big, want_small = gpu_decode(big), gpu_decode(small)
    out_big, out_small = torch.full_like(big.q, 7.0), torch.full_like(small.q, 7.0)
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    _static(big, out_big)
    _static(small, out_small)      # the array still holds the larger call's plan and partials
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0, "the call changed the amount of free device memory"
    bits = torch.int32 if qd == "f32" else torch.int16
    assert torch.equal(out_big.view(bits), want_big.view(bits))
    assert torch.equal(out_small.view(bits), want_small.view(bits))
    check(out_big, oracle_decode(big), qd, name)
    check(out_small, oracle_decode(small), qd, name + " (second, smaller call)")
    # and once more the other way round
    out_big.fill_(7.0)
    _static(big, out_big)
    torch.cuda.synchronize()
    assert torch.equal(out_big.view(bits), want_big.view(bits))


def test_a_batch_beyond_the_array_is_refused():
    import ctypes
    d = B.Desc(batch=1 << 20, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, max_pages_per_seq=4,
               num_pages=1 << 20, q_dtype=B.BF16, kv_dtype=B.BF16, sm_scale=0.1, k_scale=None, v_scale=None)
    fake = ctypes.c_void_p(0x1000)   # never dereferenced: the size check comes first
    assert B.lib().attn_decode_static(ctypes.byref(d), fake, fake, fake, fake, fake, fake, None) == -7
