"""Do the pins bite?  Plants one mistake at a time in a COPY of the oracle's source (on the CPU, in a
scratch directory) and requires that the pin suite fails on every copy, and passes on the unchanged
copy.  The oracle in the tree is never touched.

Each mutation is a text replacement that must apply exactly once, so the list cannot silently go
stale when the oracle's source changes.
"""
import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE = os.path.join(ROOT, "oracle", "stem_oracle.py")

# (name, text in the oracle, what a plausible mistake would have written instead)
MUTATIONS = [
    ("magnitude term not clamped at zero",
     "magnitude = np.maximum(0.0, m_v)", "magnitude = np.where(np.isfinite(m_v), m_v, 0.0)"),
    ("wrong GQA map in the metric", "            g = h // G\n", "            g = h % Hkv\n"),
    ("wrong GQA map in the attention",
     "block_size, i, h, h // G, blocks, scale", "block_size, i, h, h % Hkv, blocks, scale"),
    ("Eq. 3 evaluated at the 0-based index",
     "slope * (i + 1) + FLOOR_GUARD", "slope * i + FLOOR_GUARD"),
    ("strict causal mask", "visible = key_tok[None, :] <= ", "visible = key_tok[None, :] < "),
    ("lowest scores selected",
     'np.argsort(-scores[h, r, free], kind="stable")', 'np.argsort(scores[h, r, free], kind="stable")'),
    ("log base 2", "np.log(norms).max(axis=0)", "np.log2(norms).max(axis=0)"),
    ("mean instead of max pooling of the value magnitude",
     "np.log(norms).max(axis=0)", "np.log(norms).mean(axis=0)"),
    ("sum pooling of Q",
     "q_bar[:, row0 + b, a, :] = qb[a::S].mean(axis=0)", "q_bar[:, row0 + b, a, :] = qb[a::S].sum(axis=0)"),
    ("K pooled over the full class size, padding counted",
     "k_bar[:, row0 + b, a, :] = kb[a::S].mean(axis=0)",
     "k_bar[:, row0 + b, a, :] = kb[a::S].sum(axis=0) / (block_size // S)"),
    ("local window one block too long",
     "tail = set(range(max(0, i - n_local + 1), i + 1))", "tail = set(range(max(0, i - n_local), i + 1))"),
    ("softmax scale dropped", "s = scale * (qt @ ks.T)", "s = (qt @ ks.T)"),
    ("residue classes paired a with a", "[:, ::-1, :]  # residue", "[:, ::1, :]  # residue"),
    ("1/S of the strided routing term dropped", ".reshape(nb, S * d).T) / S", ".reshape(nb, S * d).T)"),
    ("minimum budget ignored", "int(k_min), len(forced_blocks", "0, len(forced_blocks"),
    ("ties go to the higher index",
     'free[np.argsort(-scores[h, r, free], kind="stable")]',
     'free[::-1][np.argsort(-scores[h, r, free[::-1]], kind="stable")]'),
    ("forced windows on top of the budget",
     "need = k - len(forced)", "need = min(k, len(free))"),
    ("budget not clamped to the causal range", "out[i] = min(i + 1, k)", "out[i] = k"),
    ("group mean divides by the KV head count", "return grouped.sum(axis=1) / G", "return grouped.sum(axis=1) / num_kv_heads"),
    ("beta applied to the routing term",
     "m = route_scale * route + beta * magnitude", "m = beta * route_scale * route + magnitude"),
    ("softmax not normalised", "out = (p / z) @ vs", "out = p @ vs"),
    ("lse without the maximum", "lse = (m + np.log(z))[:, 0]", "lse = np.log(z)[:, 0]"),
    ("empty list returns NaN-free garbage",
     "return np.zeros((t1 - t0, q.shape[2])), np.full(t1 - t0, NEG_INF)",
     "return np.zeros((t1 - t0, q.shape[2])), np.zeros(t1 - t0)"),
    ("packed budget does not restart per sequence",
     "parts = [tpd_budget(nb, k_start_blocks[s], mu, k_min, n_sink, n_local)",
     "parts = [tpd_budget(nb, k_start_blocks[0], mu, k_min, n_sink, n_local)"),
]


def _scratch_tree(tmp, name, source):
    """A directory that looks like the repository to the pin suite, with `source` as the oracle."""
    root = os.path.join(tmp, name)
    os.makedirs(os.path.join(root, "oracle"))
    os.makedirs(os.path.join(root, "tests"))
    open(os.path.join(root, "oracle", "__init__.py"), "w").close()
    with open(os.path.join(root, "oracle", "stem_oracle.py"), "w") as f:
        f.write(source)
    for item in ("conftest.py", "test_oracle_pins.py"):
        shutil.copy(os.path.join(ROOT, "tests", item), os.path.join(root, "tests", item))
    shutil.copytree(os.path.join(ROOT, "tests", "golden"), os.path.join(root, "tests", "golden"))
    # the pins read the benchmark configurations (no arithmetic of the method lives there)
    os.makedirs(os.path.join(root, "paper_2603_06274_amd"))
    for item in ("__init__.py", "workloads.py"):
        shutil.copy(os.path.join(ROOT, "paper_2603_06274_amd", item), os.path.join(root, "paper_2603_06274_amd", item))
    return root


def _pins_pass(root):
    env = dict(os.environ, PYTHONPATH=root, PYTHONDONTWRITEBYTECODE="1")
    res = subprocess.run([sys.executable, "-m", "pytest", "tests/test_oracle_pins.py", "-x", "-q",
                          "-p", "no:cacheprovider"], cwd=root, env=env, capture_output=True, text=True)
    return res.returncode == 0, res.stdout[-2000:]


def test_every_planted_mistake_fails_a_pin(tmp_path):
    source = open(ORACLE).read()
    trees = [("unchanged", _scratch_tree(str(tmp_path), "m_unchanged", source))]
    for n, (name, old, new) in enumerate(MUTATIONS):
        assert source.count(old) == 1, "mutation %r no longer applies exactly once" % name
        trees.append((name, _scratch_tree(str(tmp_path), "m%02d" % n, source.replace(old, new))))
    with ThreadPoolExecutor(max_workers=4) as ex:
        results = list(ex.map(lambda t: _pins_pass(t[1]), trees))
    ok, tail = results[0]
    assert ok, "the pins fail on the unchanged oracle copy:\n" + tail
    survivors = [name for (name, _), (passed, _) in zip(trees[1:], results[1:]) if passed]
    assert not survivors, "planted mistakes no pin caught: %s" % survivors
