"""Shared-prompt decode against the attention oracle.  The definition is that of attn_decode: the oracle
reads every trajectory through its own (aliased) page-table row, so nothing about sharing enters it."""
import numpy as np
import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check, gpu_decode, oracle_decode

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _grouped(name, batch, hq, hkv, d, kvd, ctx, group_size, shared, seed):
    b = W.build(W.Workload(name, batch, hq, hkv, d, "bf16", kvd, ctx, seed=seed), DEV)
    shared = np.asarray(shared, dtype=np.int64)
    return W.alias_shared_prefix(b, group_size, shared), torch.from_numpy(shared.astype(np.int32)).to(DEV)


def _shared(b, group_size, shared_lens, **kw):
    w = b.workload
    return B.attn_decode_shared(b.q, b.k_pages, b.v_pages, b.page_table, b.ctx_lens, group_size=group_size,
                                shared_lens=shared_lens, sm_scale=w.sm_scale, k_scale=b.k_scale, v_scale=b.v_scale, **kw)


@pytest.mark.parametrize("name,hq,hkv,d,kvd", [
    ("sp_g4", 32, 8, 128, "bf16"), ("sp_g16_fp8", 64, 4, 128, "fp8_e4m3"), ("sp_g1", 4, 4, 128, "bf16"),
    ("sp_g8_d64", 16, 2, 64, "bf16"), ("sp_g40", 40, 1, 128, "fp8_e4m3"),
])
def test_groups_of_eight_with_shared_prompts(name, hq, hkv, d, kvd):
    # prompts of 0 .. 900 tokens shared by 8 trajectories that continue for 1 .. 700 tokens each: shared lengths
    # that are not multiples of the block, a group without a shared part, one whose prompt is longer than its
    # shortest member (the library must lower it), several 64-token blocks in both halves
    rng = np.random.default_rng(17)
    shared = np.array([0, 33, 900, 257, 5000])
    b, sl = _grouped(name, 40, hq, hkv, d, kvd, ("uniform", 300, 1600), 8, shared, 401)
    out = _shared(b, 8, sl)
    torch.cuda.synchronize()
    check(out, oracle_decode(b), "bf16", name)


@pytest.mark.parametrize("group_size", [1, 2, 4, 16])
def test_other_group_sizes(group_size):
    n_groups = 48 // group_size
    shared = np.random.default_rng(5).integers(0, 400, n_groups)
    b, sl = _grouped("sp_sizes", 48, 16, 4, 128, "bf16", ("uniform", 64, 500), group_size, shared, 402)
    out = _shared(b, group_size, sl)
    torch.cuda.synchronize()
    check(out, oracle_decode(b), "bf16", f"group size {group_size}")


def test_agrees_with_plain_decode_and_with_no_sharing_at_all():
    shared = np.array([512, 96, 0, 2048])
    b, sl = _grouped("sp_same", 32, 32, 8, 128, "bf16", ("uniform", 600, 2500), 8, shared, 403)
    plain = gpu_decode(b).float()
    both = _shared(b, 8, sl).float()
    none = _shared(b, 8, torch.zeros_like(sl)).float()
    torch.cuda.synchronize()
    ref = oracle_decode(b)
    check(both, ref, "bf16", "shared"); check(none, ref, "bf16", "zero shared lengths")
    # the three routes round differently (the halves are rounded to bf16 before the merge) but stay close
    assert (plain - both).abs().max().item() <= 1e-2 and (plain - none).abs().max().item() <= 1e-2


def test_mixed_config_shape_full_size():
    # the decode rows of the mixed FP8 configuration regrouped as 48 groups of 8 whose prompts cover half of
    # the group's shortest context: the launch configuration the bench times, sampled rows against the oracle
    b = W.build(W.CONFIGS[5], DEV)
    dec = b.select(b.decode_rows())
    shared = np.array([dec.ctx_lens_host[j * 8:(j + 1) * 8].min() // 2 for j in range(48)])
    dec = W.alias_shared_prefix(dec, 8, shared)
    sl = torch.from_numpy(shared.astype(np.int32)).to(DEV)
    out = _shared(dec, 8, sl)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    rows = np.array(sorted({0, 7, 8, 100, 201, 383, int(np.argmax(dec.ctx_lens_host)), int(np.argmin(dec.ctx_lens_host))}))
    sub = dec.select(rows)
    check(out[torch.from_numpy(rows).to(DEV)], oracle_decode(sub), "bf16", "mixed config, shared prompts")
