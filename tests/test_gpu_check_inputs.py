"""rollattn_debug_check_inputs: the device-side check of what the attention calls take on trust.  The planted
violations go to the checker only (it reads nothing it has not bounded itself), never to an attention call."""
from __future__ import annotations

import numpy as np
import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _batch():
    w = W.Workload("check", 37, 8, 2, 64, "bf16", "bf16", ("uniform", 1, 900), qlen=("uniform", 0, 40), seed=W.BASE_SEED + 61,
                   ctx_is_prefix=True)
    b = W.build(w, DEV)
    desc = B.make_desc(b.q, b.k_pages, b.page_table, sm_scale=1.0)
    return b, desc


def test_valid_inputs_count_nothing():
    b, desc = _batch()
    assert B.check_inputs(desc, b.page_table, b.ctx_lens).tolist() == [0, 0, 0, 0]
    assert B.check_inputs(desc, b.page_table, b.ctx_lens, b.q_lens, b.q_offsets).tolist() == [0, 0, 0, 0]
    # the table's unused tail holds -1: entries past the last live page are nobody's business
    assert int((b.page_table < 0).sum()) > 0


def test_every_kind_of_violation_is_counted():
    b, desc = _batch()
    table = b.page_table.clone()
    ctx = b.ctx_lens.clone()
    q_lens = b.q_lens.clone()
    q_offs = b.q_offsets.clone()
    max_pages = table.shape[1]
    lens = b.ctx_lens_host
    # two lengths out of range (their tables are then not looked at)
    ctx[3] = -5
    ctx[11] = 16 * max_pages + 1
    # three bad ids on live pages of healthy trajectories, one of them the last live page; one in a dead entry
    table[0, 0] = b.num_pages
    table[5, (int(lens[5]) + 15) // 16 - 1] = -1
    table[20, 0] = 2 ** 31 - 1
    if (int(lens[7]) + 15) // 16 < max_pages:
        table[7, max_pages - 1] = -77                      # past the live pages: not counted
    # chunk lengths: one negative, one longer than its context
    q_lens[9] = -1
    q_lens[14] = int(lens[14]) + 1
    got = B.check_inputs(desc, table, ctx, q_lens, q_offs).tolist()
    # q_offsets was the scan of the original q_lens: rows 9 and 14 no longer agree with it
    assert got == [2, 3, 2, 2], got
    # a shifted scan disagrees at its first entry only (differences are unchanged elsewhere)
    assert B.check_inputs(desc, b.page_table, b.ctx_lens, b.q_lens, b.q_offsets + 1).tolist() == [0, 0, 0, 1]
