"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments before touching the device, and its host twin of the
decode partition rule agrees integer for integer with the oracle's statement of the rule."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import attention as O
from paper_2512_22560_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _desc(**kw):
    base = dict(batch=4, num_q_heads=8, num_kv_heads=2, head_dim=64, page_size=16, max_pages_per_seq=16,
                num_pages=43, q_dtype=B.F32, kv_dtype=B.F32, sm_scale=0.125, k_scale=None, v_scale=None)
    base.update(kw)
    return B.Desc(**base)


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "rollattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(attn_\w+|kv_\w+|rollattn_\w+)\s*\(", text))
    declared -= {"rollattn_desc", "rollattn_status", "rollattn_dtype"}
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name
    assert lib.rollattn_version() >= 100


def test_descriptor_errors_are_reported_before_any_launch():
    lib = B.lib()
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    def decode(d, q=fake, ws=fake, ws_bytes=1 << 40):
        return lib.attn_decode(ctypes.byref(d), q, fake, fake, fake, fake, fake, ws, ws_bytes, None)
    assert decode(_desc(num_q_heads=7)) == -2                      # Hq % Hkv
    assert decode(_desc(head_dim=96)) == -2
    assert decode(_desc(page_size=32)) == -2
    assert decode(_desc(q_dtype=B.F32, kv_dtype=B.BF16)) == -3
    assert decode(_desc(q_dtype=B.BF16, kv_dtype=B.FP8_E4M3, head_dim=128)) == -3   # no scales
    assert decode(_desc(batch=-1)) == -1
    assert decode(_desc(), q=None) == -1
    assert decode(_desc(), q=ctypes.c_void_p(0x1008)) == -4
    assert decode(_desc(), ws_bytes=16) == -5
    assert decode(_desc(batch=0)) == 0                             # empty batch: success, no launch
    assert lib.attn_decode(None, fake, fake, fake, fake, fake, fake, fake, 0, None) == -1
    assert lib.attn_append(ctypes.byref(_desc()), fake, fake, fake, 0, 0, fake, fake, fake, fake, fake, fake, 0, None) == 0
    assert lib.attn_append(ctypes.byref(_desc()), fake, fake, fake, -1, 0, fake, fake, fake, fake, fake, fake, 0, None) == -1
    assert lib.attn_append(ctypes.byref(_desc()), fake, fake, fake, 8, 2, fake, fake, fake, fake, fake, fake, 16, None) == -5
    # the workspace-free decode call checks its descriptor, then its size limit, before it touches the device
    assert lib.attn_decode_static(ctypes.byref(_desc(head_dim=96)), fake, fake, fake, fake, fake, fake, None) == -2
    assert lib.attn_decode_static(ctypes.byref(_desc(batch=0)), fake, fake, fake, fake, fake, fake, None) == 0
    assert lib.attn_decode_static(ctypes.byref(_desc(batch=12_000_000)), fake, fake, fake, fake, fake, fake, None) == -7
    assert lib.rollattn_static_scratch_bytes() == 36 << 20
    def write(d, total_q=4, k_new=fake, ks=fake, max_q=1):
        return lib.kv_write(ctypes.byref(d), k_new, fake, fake, fake, total_q, max_q, fake, fake, fake, fake, ks, fake, None)
    assert write(_desc(), total_q=0) == 0                          # nothing to write: success, no launch
    assert write(_desc(), total_q=-1) == -1
    assert write(_desc(head_dim=96)) == -2
    assert write(_desc(), k_new=None) == -1
    assert write(_desc(), k_new=ctypes.c_void_p(0x1004)) == -4
    assert write(_desc(q_dtype=B.BF16, kv_dtype=B.FP8_E4M3, head_dim=128), ks=None) == -3   # FP8 pools need scale arrays
    assert write(_desc(q_dtype=B.F32, kv_dtype=B.FP8_E4M3)) == -3
    assert write(_desc(batch=70000)) == -2
    def shared(d, group_size=2, sl=fake, ws_bytes=1 << 40):
        return lib.attn_decode_shared(ctypes.byref(d), fake, fake, fake, fake, fake, group_size, sl, fake, fake, ws_bytes, None)
    bf = dict(q_dtype=B.BF16, kv_dtype=B.BF16, head_dim=128)
    assert shared(_desc(batch=4, **bf), group_size=3) == -1        # batch is not a whole number of groups
    assert shared(_desc(batch=4, **bf), group_size=0) == -1
    assert shared(_desc(batch=4)) == -3                            # float32 queries: not on this path
    assert shared(_desc(batch=4, **bf), sl=None) == -1
    assert shared(_desc(batch=4, **bf), ws_bytes=64) == -5
    assert shared(_desc(batch=0, **bf)) == 0
    assert lib.rollattn_shared_workspace_bytes(ctypes.byref(_desc(batch=4, **bf)), 2) > lib.rollattn_workspace_bytes(ctypes.byref(_desc(batch=4, **bf)), 4)
    assert lib.rollattn_shared_workspace_bytes(ctypes.byref(_desc(batch=4, **bf)), 3) == 0
    def step(d, total_q=8, ql=fake, ws=fake, ws_bytes=1 << 40):
        return lib.attn_step(ctypes.byref(d), fake, ql, fake, total_q, 2, fake, fake, fake, fake, fake, ws, ws_bytes, None)
    assert step(_desc(**bf), total_q=0) == 0                       # nothing to do: success, no launch
    assert step(_desc(**bf), total_q=-1) == -1
    assert step(_desc(head_dim=96)) == -2
    assert step(_desc(**bf), ql=None) == -1
    assert step(_desc(**bf), ws=None) == -1
    assert step(_desc(**bf), ws=ctypes.c_void_p(0x1008)) == -4
    assert step(_desc(**bf), ws_bytes=1024) == -5
    d = _desc(**bf)
    assert lib.rollattn_step_workspace_bytes(ctypes.byref(d), 8) >= (lib.rollattn_workspace_bytes(ctypes.byref(d), 8) + 256)
    assert lib.rollattn_step_workspace_bytes(ctypes.byref(_desc(head_dim=96)), 8) == 0
    assert lib.attn_decode_lse(ctypes.byref(_desc()), fake, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == -1   # no lse buffer
    assert lib.attn_decode_lse(ctypes.byref(_desc()), fake, fake, fake, fake, fake, fake, ctypes.c_void_p(0x1004), fake, 1 << 40, None) == -4
    assert lib.attn_decode_lse(ctypes.byref(_desc(batch=0)), fake, fake, fake, fake, fake, fake, None, fake, 0, None) == 0
    assert lib.attn_append_lse(ctypes.byref(_desc()), fake, fake, fake, 8, 2, fake, fake, fake, fake, fake, None, fake, 1 << 40, None) == -1
    assert lib.attn_append_lse(ctypes.byref(_desc()), fake, fake, fake, 0, 0, fake, fake, fake, fake, fake, None, fake, 0, None) == 0
    def merge(d, rows=5, o1=fake, l2=fake, lo=fake):
        return lib.attn_merge(ctypes.byref(d), rows, o1, fake, fake, l2, fake, lo, None)
    assert merge(_desc(), rows=0) == 0
    assert merge(_desc(), rows=-1) == -1
    assert merge(_desc(), o1=None) == -1
    assert merge(_desc(), l2=ctypes.c_void_p(0x1008)) == -4
    assert merge(_desc(), lo=ctypes.c_void_p(0x1008)) == -4
    assert merge(_desc(head_dim=96)) == -2
    counts = (ctypes.c_int32 * 4)(7, 7, 7, 7)
    def check(d, table=fake, scratch=fake):
        return lib.rollattn_debug_check_inputs(ctypes.byref(d), table, fake, None, None, scratch, counts, None)
    assert check(_desc(batch=0)) == 0 and list(counts) == [0, 0, 0, 0]     # nothing to check
    assert check(_desc(), table=None) == -1
    assert check(_desc(), scratch=None) == -1
    assert check(_desc(), scratch=ctypes.c_void_p(0x1004)) == -4
    assert check(_desc(head_dim=96)) == -2
    for code in range(-6, 1):
        assert lib.rollattn_status_string(code)
    assert lib.rollattn_workspace_bytes(ctypes.byref(_desc(head_dim=96)), 4) == 0
    assert lib.rollattn_workspace_bytes(ctypes.byref(_desc()), 4) > 0
    assert lib.rollattn_profile_read(None, 0) == 0
    # the testing knob of the decode partition: fewer workers than the launch has, reported by rollattn_plan_workers
    every = lib.rollattn_plan_workers(ctypes.byref(_desc()))
    assert every > 7 and lib.rollattn_debug_set_decode_workers(7) == 0
    assert lib.rollattn_plan_workers(ctypes.byref(_desc())) == 7
    assert lib.rollattn_debug_set_decode_workers(10 ** 9) == 7 and lib.rollattn_plan_workers(ctypes.byref(_desc())) == every
    assert lib.rollattn_debug_set_decode_workers(0) == 10 ** 9 and lib.rollattn_plan_workers(ctypes.byref(_desc())) == every
    assert lib.rollattn_profile_append_clock(None) == -1
    mhz = ctypes.c_double(-1.0)
    assert lib.rollattn_profile_append_clock(ctypes.byref(mhz)) == 0 and mhz.value == 0.0     # profiling never switched on


@pytest.mark.parametrize("seed", range(8))
def test_host_plan_twin_matches_the_oracle_rule(seed):
    rng = np.random.default_rng(seed)
    hkv = int(rng.choice([1, 2, 4, 8]))
    group = int(rng.choice([1, 4, 5, 16, 20]))
    f32 = bool(seed % 2)
    batch = int(rng.choice([1, 3, 64, 700]))
    hi = int(rng.choice([40, 3000, 20000]))
    lens = rng.integers(0, hi, batch).astype(np.int32)
    d = _desc(batch=batch, num_kv_heads=hkv, num_q_heads=hkv * group, max_pages_per_seq=hi // 16 + 1,
              head_dim=128, q_dtype=B.F32 if f32 else B.BF16, kv_dtype=B.F32 if f32 else B.BF16)
    tile = 4 if f32 else 16
    rows_per_b = hkv * -(-group // tile)
    workers = B.plan_workers(d)
    assert workers == (1024 if f32 else 2048)
    per, total, segs = B.debug_plan(d, lens)
    o_per, o_total, _, o_segs = O.split_plan(lens, rows_per_b, workers)
    assert (per, total) == (o_per, o_total)
    assert np.array_equal(segs, o_segs)


def test_plan_on_the_benchmark_length_draws():
    from paper_2512_22560_amd import workloads as W
    for c in (2, 3):
        w = W.CONFIGS[c]
        lens, _, table, npages = W.draw_structure(w)
        d = _desc(batch=w.batch, num_kv_heads=w.num_kv_heads, num_q_heads=w.num_q_heads, head_dim=128,
                  max_pages_per_seq=table.shape[1], num_pages=npages, q_dtype=B.BF16, kv_dtype=B.BF16)
        per, total, segs = B.debug_plan(d, lens)
        o_per, o_total, _, o_segs = O.split_plan(lens, w.num_kv_heads, 2048)
        assert (per, total) == (o_per, o_total) and np.array_equal(segs, o_segs)
        assert segs[:, 4].sum() == total == w.num_kv_heads * ((lens + 31) // 32).sum()
