"""Seeded random small workloads through the whole path against the oracle: shapes, packings,
budgets and windows the hand-picked cases do not cover."""
import numpy as np
import pytest

from paper_2603_06274_amd import workloads as wl

from test_gpu_parity import run_both

pytestmark = pytest.mark.gpu


def random_workload(seed: int, head_dim: int = 128) -> wl.Workload:
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
                    beta=float(r.choice([0.0, 0.2, 1.0])), route_scale=float(r.choice([1.0, 128 ** -0.5])),
                    head_dim=head_dim)


@pytest.mark.parametrize("seed", range(24))
def test_random_workload_whole_path(seed):
    run_both(random_workload(seed))


@pytest.mark.parametrize("seed", range(24, 40))
def test_random_workload_with_options(seed):
    """The same with a random anti-diagonal stride, the fused stage 1-2 or group-shared lists."""
    run_with_options(random_workload(seed), seed)


@pytest.mark.parametrize("head_dim", [64, 256])
@pytest.mark.parametrize("seed", range(40, 52))
def test_random_workload_other_head_sizes(seed, head_dim):
    """Head sizes 64 and 256: plain on even seeds, with random options on odd ones."""
    w = random_workload(seed, head_dim)
    if seed % 2:
        run_with_options(w, seed)
    else:
        run_both(w)


def run_with_options(w, seed):
    import torch
    from oracle import stem_oracle as so
    from paper_2603_06274_amd.prefill import StemPrefill
    import parity_util as pu

    r = np.random.default_rng(5000 + seed)
    S = int(r.choice([1, 2, 4, 8]))
    group = [None, "max", "mean"][int(r.integers(0, 3))]
    fused = group is None and bool(r.integers(0, 2))
    print("case", w.name, "lens", w.seq_lens, "B", w.block_size, "S", S, "group", group, "fused", fused, flush=True)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    dev = torch.device("cuda:0")
    q, k, v = (data[x].to(dev) for x in "qkv")
    pf = StemPrefill(q, k, v, w.cu_seqlens, w.block_size, w.k_start_blocks, w.mu, w.k_min, w.n_sink, w.n_local,
                     w.beta, w.route_scale, w.softmax_scale, want_lse=True, ad_stride=S, group_share=group)
    pf.run(fused=fused)
    torch.cuda.synchronize()
    scores = pu.oracle_estimate(w, qkv, S)[3]
    G = w.num_q_heads // w.num_kv_heads
    if group:
        scores = so.group_scores(scores, w.num_kv_heads, group)
    _, counts, indices = pu.oracle_select(w, scores)
    same = pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, scores, print)
    rep = G if group else 1
    o_out, o_lse = so.sparse_attention(*qkv, w.cu_seqlens, w.block_size, np.repeat(counts, rep, axis=0),
                                       np.repeat(indices, rep, axis=0), w.softmax_scale)
    B = w.block_size
    for (lo, hi, nb, row0) in so.sequence_table(w.cu_seqlens, B):
        for i in range(nb):
            for h in range(w.num_q_heads):
                if not same[h // rep, row0 + i]:
                    o_out[lo + i * B:min(lo + (i + 1) * B, hi), h] = np.nan
                    o_lse[h, lo + i * B:min(lo + (i + 1) * B, hi)] = np.nan
    pu.check_output(pf.out, o_out, w.name, print,
                    pu.ListedKeys(qkv, w.cu_seqlens, B, np.repeat(counts, rep, axis=0), np.repeat(indices, rep, axis=0),
                                  w.softmax_scale))
    if (~np.isnan(o_lse)).any():
        pu.check_lse(pf.lse, o_lse, w.name)
