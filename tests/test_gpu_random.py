"""Seeded random small workloads through the whole path against the oracle: shapes, packings,
budgets and windows the hand-picked cases do not cover."""
import numpy as np
import pytest

from paper_2603_06274_amd import workloads as wl

from test_gpu_parity import run_both

pytestmark = pytest.mark.gpu


def random_workload(seed: int) -> wl.Workload:
    r = np.random.default_rng(1000 + seed)
    B = int(r.choice([64, 128]))
    hkv = int(r.choice([1, 2, 3]))
    g = int(r.choice([1, 2, 4]))
    batch = int(r.integers(1, 6))
    lens = [int(r.integers(2, 14 * B)) if r.random() < 0.6 else int(r.choice([0, 1, B - 1, B, B + 1]))
            for _ in range(batch)]
    if sum(lens) == 0:
        lens[0] = 3 * B + 5
    n_local = int(r.integers(1, 4))                      # the diagonal is always kept
    return wl.small("random_%d" % seed, seed=seed, num_q_heads=hkv * g, num_kv_heads=hkv, seq_lens=tuple(lens),
                    block_size=B, k_start=tuple(float(r.integers(0, 9)) + float(r.choice([0.0, 0.4])) for _ in lens),
                    n_sink=int(r.integers(0, 4)), n_local=n_local, outliers=tuple(int(r.integers(0, 3)) for _ in lens),
                    mu=float(r.choice([0.5, 0.7, 1.0])), k_min=int(r.integers(0, 6)),
                    beta=float(r.choice([0.0, 0.2, 1.0])), route_scale=float(r.choice([1.0, 128 ** -0.5])))


@pytest.mark.parametrize("seed", range(24))
def test_random_workload_whole_path(seed):
    run_both(random_workload(seed))
