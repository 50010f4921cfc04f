"""Seeded sweep over shapes that no hand-picked case names: head counts, group sizes, head dimensions, storage
types, batch sizes and length mixes are drawn together, and every entry point of the attention path is compared
with the oracle on each draw.  The draws are small (the oracle takes well under a second each) but reach
several query tiles, several 64-token blocks, rows without work and ragged tails on both axes."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check, gpu_append, gpu_decode, oracle_append, oracle_decode

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

TYPES = [("f32", "f32"), ("bf16", "bf16"), ("bf16", "fp8_e4m3")]


def _draw(seed):
    r = np.random.default_rng(1000 + seed)
    hkv = int(r.choice([1, 2, 3, 4, 8]))
    group = int(r.choice([1, 2, 3, 4, 5, 8, 16]))
    d = int(r.choice([64, 128]))
    qd, kvd = TYPES[int(r.integers(0, 3))]
    batch = int(r.integers(1, 13))
    hi = int(r.choice([40, 300, 1500]))
    kind = str(r.choice(["uniform", "loguniform"]))
    qhi = int(r.choice([1, 17, 130, 400]))
    return dict(hkv=hkv, hq=hkv * group, d=d, qd=qd, kvd=kvd, batch=batch, ctx=(kind, 1, hi), qhi=qhi)


@pytest.mark.parametrize("seed", range(24))
def test_decode_on_drawn_shapes(seed):
    p = _draw(seed)
    b = W.build(W.Workload(f"sweep_d{seed}", p["batch"], p["hq"], p["hkv"], p["d"], p["qd"], p["kvd"], p["ctx"],
                           seed=3000 + seed), DEV)
    check(gpu_decode(b), oracle_decode(b), p["qd"], f"decode {p}")


@pytest.mark.parametrize("seed", range(24))
def test_append_on_drawn_shapes(seed):
    p = _draw(100 + seed)
    b = W.build(W.Workload(f"sweep_a{seed}", p["batch"], p["hq"], p["hkv"], p["d"], p["qd"], p["kvd"], p["ctx"],
                           qlen=("uniform", 0, p["qhi"]), seed=4000 + seed, ctx_is_prefix=True), DEV)
    ref = oracle_append(b)
    got = gpu_append(b)
    assert got.shape[0] == int(b.q_lens_host.sum())
    check(got, ref, p["qd"], f"append {p}")


@pytest.mark.parametrize("seed", range(12))
def test_shared_prefix_decode_on_drawn_shapes(seed):
    p = _draw(200 + seed)
    r = np.random.default_rng(5000 + seed)
    group_size = int(r.choice([1, 2, 3, 4, 8]))
    n_groups = int(r.integers(1, 5))
    kvd = "bf16" if p["kvd"] == "f32" else p["kvd"]            # the shared-prefix entry point has no float32 path
    lo = int(r.choice([1, 70, 400]))
    b = W.build(W.Workload(f"sweep_s{seed}", n_groups * group_size, p["hq"], p["hkv"], p["d"], "bf16", kvd,
                           ("uniform", lo, lo + p["ctx"][2]), seed=6000 + seed), DEV)
    shared = r.integers(0, lo + p["ctx"][2], n_groups)          # some longer than the shortest member
    b = W.alias_shared_prefix(b, group_size, shared)
    sl = torch.from_numpy(shared.astype(np.int32)).to(DEV)
    out = B.attn_decode_shared(b.q, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, group_size=group_size,
                               shared_lens=sl, sm_scale=b.workload.sm_scale, k_scale=b.k_scale, v_scale=b.v_scale)
    torch.cuda.synchronize()
    check(out, oracle_decode(b), "bf16", f"shared {p} groups of {group_size}, shared {shared.tolist()}")
