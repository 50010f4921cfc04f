"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the host twin of the decode
partition rule (csrc/host_plan.h, the code behind rollattn_debug_plan) and the scalar C twin of the oracle
(oracle/brute_attn.c) are built as small programs with -fsanitize=address,undefined, every input array in a heap
block of exactly its size, and run on plan and attention cases; their answers must also equal the oracle's."""
from __future__ import annotations

import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import attention as O
from paper_2512_22560_amd import workloads as W
from tests.helpers import oracle_args, tiny

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-O1", "-g"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def _build(tmp_path, compiler, src, extra):
    exe = str(tmp_path / (os.path.basename(src) + ".san"))
    r = subprocess.run([compiler, *SAN, *extra, os.path.join(ROOT, "tests", src), "-o", exe, "-lm"], capture_output=True, text=True)
    if r.returncode and ("asan" in r.stderr.lower() or "sanitize" in r.stderr.lower()):
        pytest.skip("no sanitizer runtime for the host compiler here: " + r.stderr.strip().splitlines()[-1])
    assert r.returncode == 0, r.stderr
    return exe


def test_host_plan_twin_under_the_sanitizers(tmp_path):
    exe = _build(tmp_path, "g++", "sanitize_plan_main.cpp", ["-std=c++17", "-I", os.path.join(ROOT, "paper_2512_22560_amd", "csrc")])
    rng = np.random.default_rng(11)
    cases = [(8, 2048, rng.integers(0, 9000, 64)), (2, 7, rng.integers(0, 90, 50)), (1, 5, np.array([0, 33, 0, 0, 1, 64, 0])),
             (8, 16, np.array([0, 0])), (4, 2048, rng.integers(1, 300, 10)), (16, 1024, rng.integers(0, 40, 3000)),
             (3, 1, rng.integers(0, 500, 9)), (8, 2048, np.zeros(0, dtype=np.int64)), (1, 2048, np.array([1_000_003]))]
    for rows_per_b, workers, lens in cases:
        text = f"{rows_per_b} {workers} {len(lens)}\n" + " ".join(str(int(x)) for x in lens) + "\n"
        r = subprocess.run([exe], input=text, capture_output=True, text=True, env=ENV)
        assert r.returncode == 0 and not r.stderr, (rows_per_b, workers, r.stderr[-2000:])
        nums = np.array(r.stdout.split(), dtype=np.int64)
        per, total, n = nums[:3]
        segs = nums[3:].reshape(-1, 6)
        o_per, o_total, _, o_segs = O.split_plan(lens, rows_per_b, workers)
        assert (per, total, n) == (o_per, o_total, len(o_segs))
        assert np.array_equal(segs, o_segs)


_CODE = {"f32": 0, "bf16": 1, "fp8_e4m3": 2}


def _run_brute(exe, tmp_path, b, append):
    w = b.workload
    a = oracle_args(b)
    q = W.raw_numpy(b.q)
    rows, hq, d = q.shape
    num_pages, hkv, ps, _ = a["k_pages"].shape
    has_scales = a["k_scale"] is not None
    head = [rows, len(b.ctx_lens_host), hq, hkv, d, ps, a["page_table"].shape[1], num_pages, _CODE[w.q_dtype], _CODE[w.kv_dtype],
            1 if append else 0, 1 if has_scales else 0]
    blob = struct.pack("<12q", *head) + struct.pack("<f", w.sm_scale) + np.ascontiguousarray(q).tobytes()
    if append:
        blob += b.q_lens_host.astype(np.int32).tobytes()
    blob += np.ascontiguousarray(a["k_pages"]).tobytes() + np.ascontiguousarray(a["v_pages"]).tobytes()
    if has_scales:
        blob += a["k_scale"].astype(np.float32).tobytes() + a["v_scale"].astype(np.float32).tobytes()
    # dead table entries are -1 in the generator: the twin must never follow them
    blob += np.ascontiguousarray(a["page_table"], dtype=np.int32).tobytes() + b.ctx_lens_host.astype(np.int32).tobytes()
    fin, fout = tmp_path / "in.bin", tmp_path / "out.bin"
    fin.write_bytes(blob)
    r = subprocess.run([exe, str(fin), str(fout)], capture_output=True, text=True, env=ENV)
    assert r.returncode == 0 and not r.stderr, r.stderr[-2000:]
    return np.frombuffer(fout.read_bytes(), dtype=np.float64).reshape(rows, hq, d)


def test_scalar_twin_of_the_oracle_under_the_sanitizers(tmp_path):
    exe = _build(tmp_path, "gcc", "sanitize_brute_main.c", ["-std=c99"])
    for qd, kvd, d in (("f32", "f32", 16), ("bf16", "bf16", 32), ("bf16", "fp8_e4m3", 32)):
        # ragged lengths around the page edges, decode and append
        b = tiny(f"san_dec_{kvd}", batch=7, hq=4, hkv=2, d=d, q_dtype=qd, kv_dtype=kvd, ctx=("uniform", 1, 70), seed=31)
        got = _run_brute(exe, tmp_path, b, append=False)
        np.testing.assert_allclose(got, O.attn_decode(W.raw_numpy(b.q), **oracle_args(b)), rtol=0, atol=1e-12)
        b = tiny(f"san_app_{kvd}", batch=5, hq=4, hkv=2, d=d, q_dtype=qd, kv_dtype=kvd, ctx=("uniform", 0, 40), qlen=("uniform", 0, 20),
                 ctx_is_prefix=True, seed=32)
        got = _run_brute(exe, tmp_path, b, append=True)
        np.testing.assert_allclose(got, O.attn_append(W.raw_numpy(b.q), b.q_lens_host, **oracle_args(b)), rtol=0, atol=1e-12)
