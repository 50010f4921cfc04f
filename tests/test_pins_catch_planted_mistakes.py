"""The pins are only worth what they catch.  Each case below plants one plausible mistake in a private copy of
the oracle's source (a dropped softmax scale, an off-by-one causal boundary, a wrong slot or page index, swapped
K/V scales, a rounding rule, ...) and runs the pin tests against that copy in a child process: every planted
mistake must make at least one pin fail, and the untouched copy must pass.  Nothing here touches the files under
oracle/ themselves, and nothing runs on a GPU."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

ATTENTION = ("attention.py", "tests/test_oracle_pins.py", [
    ("decode: softmax scale dropped", "z = scale * (k @ qf[b, h, :])", "z = (k @ qf[b, h, :])"),
    ("append: softmax scale dropped", "z = scale * (q[row0:row0 + n, h, :] @ k.T)", "z = (q[row0:row0 + n, h, :] @ k.T)"),
    ("append: rows one position early", "pos = length - n + np.arange(n)", "pos = length - n + np.arange(n) - 1"),
    ("append: rows one position late", "pos = length - n + np.arange(n)", "pos = length - n + np.arange(n) + 1"),
    ("append: a row does not see itself", "visible = np.arange(length)[None, :] <= pos[:, None]",
     "visible = np.arange(length)[None, :] < pos[:, None]"),
    ("decode: every head its own KV head", "group = hq // hkv\n    out = np.zeros((bsz", "group = 1\n    out = np.zeros((bsz"),
    ("gather: slot off by one", "slot = t % page_size", "slot = (t + 1) % page_size"),
    ("gather: next page's id", "phys = np.asarray(page_table)[b, t // page_size]",
     "phys = np.asarray(page_table)[b, np.minimum(t // page_size + 1, (length - 1) // page_size)]"),
    ("decode: V read with the K scales",
     "v = gather_tokens(v_pages, page_table, b, g, length, kv_dtype, v_scale)\n            for h in range(g * group, (g + 1) * group):\n                z = scale * (k @",
     "v = gather_tokens(v_pages, page_table, b, g, length, kv_dtype, k_scale)\n            for h in range(g * group, (g + 1) * group):\n                z = scale * (k @"),
    ("E4M3: subnormal exponent", "subnormal = (m / 8.0) * 2.0 ** (-6)", "subnormal = (m / 8.0) * 2.0 ** (-7)"),
    ("decode: sign of the exponent", "w = np.exp(z - z.max())", "w = np.exp(z.max() - z)"),
    ("merge: partial sums not weighted", "a = np.exp(ms - ms.max()) * ls", "a = np.exp(ms - ms.max())"),
    ("lse: natural logarithm", "lse[row0 + i, h] = (top + np.log(np.exp(z - top).sum())) / np.log(2.0)",
     "lse[row0 + i, h] = (top + np.log(np.exp(z - top).sum()))"),
    ("lse: chunk row sees one token too many", "seen = length - n + i + 1 ", "seen = min(length, length - n + i + 2) "),
    ("lse: maximum left out", "lse[row0 + i, h] = (top + np.log(np.exp(z - top).sum())) / np.log(2.0)",
     "lse[row0 + i, h] = (np.log(np.exp(z - top).sum())) / np.log(2.0)"),
    ("merge of ranges: weights e^lse", "w1, w2 = np.exp2(l1 - safe), np.exp2(l2 - safe)", "w1, w2 = np.exp(l1 - safe), np.exp(l2 - safe)"),
    ("merge of ranges: denominator without the reference", "lse = np.where(tot > 0, safe + np.log2(tot), -np.inf)",
     "lse = np.where(tot > 0, np.log2(tot), -np.inf)"),
    ("merge of ranges: plain average", "(w1[..., None] * o1 + w2[..., None] * o2) / tot[..., None]", "(o1 + o2) / 2"),
    ("tile list: shortest context first", "order.sort(key=lambda b: (-ctx[b], b))", "order.sort(key=lambda b: (ctx[b], b))"),
    ("tile list: a chunk's first tile first", "for start in reversed(starts):", "for start in starts:"),
    ("tile list: last tile takes a full tile's rows", "tiles.append((b, start, min(tile_tokens, q[b] - start)))",
     "tiles.append((b, start, tile_tokens))"),
    ("tile list: one-token chunks kept in a mixed step", "if skip_unit_chunks and q[b] == 1:", "if False:"),
    ("tile list: ties by higher index", "order.sort(key=lambda b: (-ctx[b], b))", "order.sort(key=lambda b: (-ctx[b], -b))"),
    ("partition: runs one block short", "per = max(1, -(-total // workers))", "per = max(1, total // workers)"),
])

KV_WRITE = ("kv_write.py", "tests/test_kv_write_pins.py", [
    ("encoder: ties away from zero", "np.rint(a / step)", "np.floor(a / step + 0.5)"),
    ("encoder: no clamp at 448", "np.minimum(a, 448.0)", "a"),
    ("encoder: one binade too many below", "np.maximum(ex - 1, -6)", "np.maximum(ex - 1, -7)"),
    ("encoder: sign in the wrong bit", "sign = (np.signbit(x)).astype(np.uint8) << 7", "sign = (np.signbit(x)).astype(np.uint8) << 6"),
    ("write: previous page's id", "phys = int(page_table[b, page_i])", "phys = int(page_table[b, max(page_i - 1, 0)])"),
    ("write: scale never grows", "if need > s_old:", "if False:"),
    ("write: all-zero fresh page gets scale 0.5", "s_new = need if amax > 0 else np.float32(1.0)",
     "s_new = need if amax > 0 else np.float32(0.5)"),
    ("write: old codes decoded with the new scale", "old = (old * s_old).astype(np.float32)", "old = (old * s_new).astype(np.float32)"),
    ("write: multiplied by the scale", "(x / s_new).astype(np.float32)", "(x * s_new).astype(np.float32)"),
    ("write: heads reversed", "pool[phys, :, s0:s1, :] = np.swapaxes(src, 0, 1)", "pool[phys, :, s0:s1, :] = np.swapaxes(src, 0, 1)[::-1]"),
    ("write: rows of later trajectories from their chunk's start",
     "rows = slice(offs[b] + lo - first, offs[b] + hi - first)",
     "rows = slice(offs[b] + lo - first, offs[b] + hi - first) if b == 0 else slice(offs[b], offs[b] + hi - lo)"),
])

CONTROL = "control: untouched copy"
SENTINEL = "control: the copy is the one that runs"


def _run(work, fname, pins, name, old, new):
    """Pin tests against a copy of oracle/ with `old` replaced by `new` in fname; returns (name, exit code, output)."""
    d = os.path.join(work, "".join(c if c.isalnum() else "_" for c in name))
    shutil.copytree(os.path.join(ROOT, "oracle"), os.path.join(d, "oracle"), ignore=shutil.ignore_patterns("__pycache__"))
    path = os.path.join(d, "oracle", fname)
    text = open(path).read()
    if old is not None:
        assert text.count(old) >= 1, f"{name}: the text to replace is not in {fname} any more"
        text = text.replace(old, new, 1)
        open(path, "w").write(text)
    env = dict(os.environ, PYTHONPATH=d + os.pathsep + ROOT, PYTHONDONTWRITEBYTECODE="1")
    r = subprocess.run([sys.executable, "-m", "pytest", os.path.join(ROOT, pins), "-x", "-q", "-p", "no:cacheprovider"],
                       cwd=d, env=env, capture_output=True, text=True, timeout=900)
    return name, r.returncode, (r.stdout + r.stderr)[-1500:]


@pytest.mark.parametrize("fname,pins,cases", [ATTENTION, KV_WRITE], ids=["attention", "kv_write"])
def test_every_planted_mistake_fails_a_pin(tmp_path, fname, pins, cases):
    first_def = "def gather_tokens(" if fname == "attention.py" else "def float32_to_e4m3fn("
    jobs = [(CONTROL, None, None), (SENTINEL, first_def, "raise RuntimeError('planted sentinel')\n" + first_def)] + list(cases)
    with ThreadPoolExecutor(max_workers=6) as pool:
        results = list(pool.map(lambda c: _run(str(tmp_path), fname, pins, *c), jobs))
    by_name = {n: (rc, out) for n, rc, out in results}
    assert by_name[CONTROL][0] == 0, by_name[CONTROL][1]
    assert by_name[SENTINEL][0] != 0 and "planted sentinel" in by_name[SENTINEL][1], by_name[SENTINEL][1]
    missed = [n for n, rc, _ in results if n not in (CONTROL, SENTINEL) and rc != 1]     # 1 = some test failed
    assert not missed, f"no pin fails for: {missed}"
