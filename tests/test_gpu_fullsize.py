"""Full-size parity: the four benchmark workloads exactly as bench.py launches them (same batches,
same entry points, same workspace sizing), checked against the oracle on what it can afford one by one:
for decode sampled trajectories (the shortest, the longest and a few seeded random ones), for append
sampled rows of the shortest, the median and the longest trajectory and of a few random ones."""
import numpy as np
import pytest
import torch

from paper_2512_22560_amd import binding as B
from paper_2512_22560_amd import workloads as W
from tests.gpu_common import check, gpu_append, gpu_decode, oracle_append, oracle_decode

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _sample(batch, n_random, seed):
    lens = batch.ctx_lens_host
    rows = {int(np.argmin(lens)), int(np.argmax(lens))}
    rng = np.random.default_rng(seed)
    for r in rng.permutation(len(lens)):
        if len(rows) >= n_random + 2:
            break
        rows.add(int(r))
    return np.asarray(sorted(rows))


def _check_sampled_chunk_rows(batch, out, seed, what):
    """Append parity at full size on sampled rows.  Row i of a chunk equals a decode step at context
    L - n + i + 1, which is what the oracle computes, one row at a time: the first and last rows, the rows
    on either side of every kind of tile edge and seeded random rows of the trajectories with the shortest, the
    median and the longest context (the longest is the one with the most blocks, tiles and ring wraps in the
    launch that the bench times) and of a few seeded random trajectories."""
    from oracle import attention as O
    from tests.helpers import oracle_args
    w = batch.workload
    tile_tokens = max(1, 256 // (w.num_q_heads // w.num_kv_heads))
    rng = np.random.default_rng(seed)
    offs = np.concatenate([[0], np.cumsum(batch.q_lens_host)])
    order = np.argsort(batch.ctx_lens_host, kind="stable")
    trajs = [int(order[0]), int(order[len(order) // 2]), int(order[-1])] + rng.choice(len(order), 3, replace=False).tolist()
    args = oracle_args(batch)
    q, pt = W.raw_numpy(batch.q), args["page_table"]
    qs, tables, lens, idx = [], [], [], []
    for traj in dict.fromkeys(trajs):
        n, L = int(batch.q_lens_host[traj]), int(batch.ctx_lens_host[traj])
        picks = [0, 1, tile_tokens - 1, tile_tokens, 2 * tile_tokens - 1, n // 2, n - tile_tokens, n - 2, n - 1] + rng.integers(0, n, 5).tolist()
        for i in sorted(set(i for i in picks if 0 <= i < n)):
            qs.append(q[offs[traj] + i]); tables.append(pt[traj]); lens.append(L - n + i + 1); idx.append(int(offs[traj] + i))
    ref = O.attn_decode(np.stack(qs), args["k_pages"], args["v_pages"], np.stack(tables), np.asarray(lens), sm_scale=args["sm_scale"],
                        q_dtype=args["q_dtype"], kv_dtype=args["kv_dtype"], k_scale=args["k_scale"], v_scale=args["v_scale"])
    check(out[torch.tensor(idx, device=DEV)], ref, "bf16", f"{what}: {len(idx)} rows of trajectories {list(dict.fromkeys(trajs))}")


@pytest.mark.parametrize("c", [2, 3])
def test_decode_workloads_full_size(c):
    b = W.build(W.CONFIGS[c], DEV)
    out = gpu_decode(b)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    rows = _sample(b, 8, seed=c)
    sub = b.select(rows)
    ref = oracle_decode(sub)
    check(out[torch.from_numpy(rows).to(DEV)], ref, "bf16", f"config {c} rows {rows.tolist()}")


def test_append_workload_full_size():
    b = W.build(W.CONFIGS[4], DEV)
    out = gpu_append(b)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    _check_sampled_chunk_rows(b, out, seed=4, what="config 4")


def test_mixed_step_full_size():
    b = W.build(W.CONFIGS[5], DEV)
    dec, app = b.select(b.decode_rows()), b.select(b.append_rows())
    out_d = gpu_decode(dec)
    out_a = gpu_append(app)
    torch.cuda.synchronize()
    assert torch.isfinite(out_d.float()).all() and torch.isfinite(out_a.float()).all()
    rows = _sample(dec, 6, seed=5)
    check(out_d[torch.from_numpy(rows).to(DEV)], oracle_decode(dec.select(rows)), "bf16",
          f"config 5 decode rows {rows.tolist()}")
    _check_sampled_chunk_rows(app, out_a, seed=6, what="config 5 append")


def test_workspace_is_sized_from_the_descriptor_alone():
    # the same workspace serves any lengths the descriptor admits, e.g. every row at the maximum
    w = W.Workload("maxlen", 16, 32, 8, 128, "bf16", "bf16", ("const", 4096), seed=9)
    b = W.build(w, DEV)
    desc = B.make_desc(b.q, b.k_pages, b.page_table, sm_scale=w.sm_scale)
    ws = B.alloc_workspace(desc, b.total_q, DEV)
    check(gpu_decode(b, workspace=ws), oracle_decode(b), "bf16", "all rows at max length")
    short = np.full(16, 5)
    b.ctx_lens_host = short
    b.ctx_lens = torch.from_numpy(short.astype(np.int32)).to(DEV)
    check(gpu_decode(b, workspace=ws), oracle_decode(b), "bf16", "same workspace, short rows")


def test_recompute_prefill_full_size():
    # KV recomputation after a weight update (Section 6.2, protocol step 5): append with an empty
    # prefix over whole histories, in the launch configuration the bench times.  Row i of a chunk
    # equals a decode step at context i + 1: that is what the oracle computes for the sampled rows
    # (tile edges, block edges, first and last rows of the shortest, the median and the longest
    # history, and seeded random ones).
    from oracle import attention as O
    w = W.RECOMPUTE
    b = W.build(w, DEV)
    out = gpu_append(b)
    torch.cuda.synchronize()
    assert torch.isfinite(out.float()).all()
    rng = np.random.default_rng(7)
    offs = np.concatenate([[0], np.cumsum(b.q_lens_host)])
    order = np.argsort(b.ctx_lens_host)
    q, kp, vp, pt = (W.raw_numpy(t) for t in (b.q, b.k_pages, b.v_pages, b.page_table))
    qs, tables, lens, idx = [], [], [], []
    for traj in (int(order[0]), int(order[len(order) // 2]), int(order[-1])):
        n = int(b.q_lens_host[traj])
        for i in sorted(set([0, 1, 63, 64, 255, 256, n // 2, n - 2, n - 1] + rng.integers(0, n, 6).tolist())):
            if 0 <= i < n:
                qs.append(q[offs[traj] + i]); tables.append(pt[traj]); lens.append(i + 1); idx.append(int(offs[traj] + i))
    ref = O.attn_decode(np.stack(qs), kp, vp, np.stack(tables), np.asarray(lens), sm_scale=w.sm_scale, q_dtype="bf16", kv_dtype="bf16")
    check(out[torch.tensor(idx, device=DEV)], ref, "bf16", "recompute prefill, sampled rows")


@pytest.mark.parametrize("c", [4, 5])
def test_append_is_bit_identical_from_run_to_run(c):
    # the append kernel moves tiles HBM -> LDS asynchronously and hands them between the two halves of the
    # workgroup with bare barriers and counted waits: a race there would show up as run-to-run differences
    b = W.build(W.CONFIGS[c], DEV)
    sub = b.select(b.append_rows())
    first = gpu_append(sub).clone()
    for _ in range(4):
        # other work in between, so that the runs do not meet the machine in the same state
        torch.randn(1 << 22, device=DEV).sum().item()
        again = gpu_append(sub)
        torch.cuda.synchronize()
        assert torch.equal(first.view(torch.int16), again.view(torch.int16))


def test_one_very_long_trajectory_next_to_short_ones():
    # a million-token context (62 501 pages, 31 251 decode blocks, 15 626 append blocks per tile) beside a chunk
    # with no history and a mid-size one: block and page indices far beyond anything the benchmark configs reach,
    # the decode partition cutting one row into ~2000 pieces, the append ring wrapping thousands of times
    import dataclasses
    long_len = 1_000_003
    w = W.Workload("very_long", 3, 8, 2, 128, "bf16", "fp8_e4m3", ("const", long_len), qlen=("const", 24), seed=77)
    b = W.build(w, DEV)
    lens = np.array([long_len, 24, 40_001], dtype=np.int64)
    b = dataclasses.replace(b, ctx_lens=torch.from_numpy(lens.astype(np.int32)).to(DEV), ctx_lens_host=lens)
    assert np.array_equal(b.q_lens_host, [24, 24, 24])
    out = gpu_append(b)
    torch.cuda.synchronize()
    check(out, oracle_append(b), "bf16", "append on a million-token context")
    # decode on the same pools: one query row per trajectory (the first row of each chunk stands in for it)
    offs = np.concatenate([[0], np.cumsum(b.q_lens_host)])[:-1]
    dec = dataclasses.replace(b, q=b.q[torch.from_numpy(offs).to(DEV)].contiguous(),
                              q_lens=torch.ones(3, dtype=torch.int32, device=DEV),
                              q_offsets=torch.arange(4, dtype=torch.int32, device=DEV), q_lens_host=np.ones(3, dtype=np.int64))
    out = gpu_decode(dec)
    torch.cuda.synchronize()
    check(out, oracle_decode(dec), "bf16", "decode on a million-token context")
