"""Parity at the benchmark's full sizes, in the launch configuration bench.py times.

Stages 1 and 2 are compared in full (every pooled vector, every score, every list).  Stage 3 is
compared on sampled (head, query-block row) pairs the oracle computes one by one: the first and last
rows of every sequence, the rows around the end of the causal ramp, and random rows.  Invariants that
hold at any size are checked on the whole output: no NaN, and the first token of every sequence
returns its own value row.
"""
import numpy as np
import pytest
import torch

from oracle import stem_oracle as so
from paper_2603_06274_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu

_cache = {}


def say(*a):
    print(*a, flush=True)


def tensors_for(w):
    """The sweep configurations share one set of tensors (same seed and shape)."""
    key = (w.seed, w.seq_lens, w.num_q_heads, w.num_kv_heads, w.block_size, w.head_dim)
    if key not in _cache:
        _cache.clear()
        data = wl.generate(w)
        _cache[key] = (data, pu.host_arrays(data))
    return _cache[key]


def uniform_control(w):
    """Uniform top-k with the total block count closest to the decay schedule's (ties: smaller k)."""
    def total(ks, mu):
        return int(so.packed_budget(w.cu_seqlens, w.block_size, [ks], mu, w.k_min, w.n_sink, w.n_local).sum())
    target = total(w.k_start_blocks[0], w.mu)
    k_uni = min(range(1, int(w.k_start_blocks[0]) + 1), key=lambda k: (abs(total(k, 1.0) - target), k))
    return wl.with_budget(w, [k_uni], 1.0, "_uniform"), target, total(k_uni, 1.0)


def full_size_case(w, n_random_rows, heads):
    say("case", w.name, "seed", w.seed, "T", w.total_tokens, "ks", w.k_start_blocks, "mu", w.mu)
    data, qkv = tensors_for(w)
    pf = pu.device_prefill(w, data)
    pf.run()
    torch.cuda.synchronize()
    q_bar, k_bar, m_v, scores = pu.oracle_estimate(w, qkv)
    budget, counts, indices = pu.oracle_select(w, scores)
    assert pf.budget_host.numpy().tolist() == budget.tolist()
    density = counts.sum() / (w.admissible_blocks * w.num_q_heads)
    assert density >= w.target_density
    pu.check_pooled(pf, q_bar, k_bar, m_v)
    err = pu.check_scores(pf.scores.cpu().numpy(), scores)
    same = pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, scores, say)
    assert same.mean() > 0.99

    rows = pu.sample_rows(w, n_random_rows, seed=w.seed + 100)
    o_out, o_lse = so.sparse_attention(*qkv, w.cu_seqlens, w.block_size, counts, indices, w.softmax_scale,
                                       heads=heads, rows=rows)
    B = w.block_size
    for (lo, hi, nb, row0) in so.sequence_table(w.cu_seqlens, B):
        for i in range(nb):
            for h in heads:
                if not same[h, row0 + i]:
                    o_out[lo + i * B:min(lo + (i + 1) * B, hi), h] = np.nan
    max_abs, rel_l2 = pu.check_output(pf.out, o_out, w.name)
    m = ~np.isnan(o_lse)
    assert np.abs(pf.lse.cpu().numpy()[m] - o_lse[m]).max() <= 5e-3
    # whole-output invariants
    assert not torch.isnan(pf.out).any().item()
    G = w.num_q_heads // w.num_kv_heads
    for s in range(len(w.seq_lens)):
        if w.seq_lens[s]:
            t0 = w.cu_seqlens[s]
            assert torch.equal(pf.out[t0].cpu(), data["v"][t0].repeat_interleave(G, dim=0))
    say("%s: density %.4f, score err %.3g, %d sampled rows x %d heads: max-abs %.4g rel-L2 %.4g"
        % (w.name, density, err, len(rows), len(heads), max_abs, rel_l2))
    del pf
    torch.cuda.empty_cache()


def test_llama_32k():
    full_size_case(wl.LLAMA_32K, 24, heads=[0, 5, 14, 31])


def test_llama_128k_headline():
    full_size_case(wl.LLAMA_128K, 16, heads=[0, 9, 22, 31])


@pytest.mark.parametrize("d", [64, 256])
def test_llama_128k_other_head_sizes(d):
    """The headline layer's shape and schedule at the two other head sizes."""
    full_size_case(wl.EXTRA_CONFIGS["llama8b_128k_d%d" % d], 8, heads=[0, 22])


@pytest.mark.parametrize("point", ["d100", "d50", "d20", "d10", "d5"])
def test_budget_sweep_64k(point):
    n_rows = {"d100": 2, "d50": 4, "d20": 10, "d10": 16, "d5": 16}[point]
    full_size_case(wl.SWEEP_64K[point], n_rows, heads=[0, 13, 27])


def test_budget_sweep_64k_uniform_control():
    w, decay_total, uni_total = uniform_control(wl.SWEEP_64K["d10"])
    say("uniform control: k_uni", w.k_start_blocks, "blocks", uni_total, "vs decay", decay_total)
    assert abs(uni_total - decay_total) <= 512
    assert w.k_start_blocks[0] / wl.SWEEP_64K["d10"].k_start_blocks[0] == pytest.approx(0.85, abs=0.05)
    full_size_case(wl.with_budget(w, w.k_start_blocks, 1.0, ""), 12, heads=[3, 20])


def test_packed_varlen_128k():
    full_size_case(wl.PACKED_128K, 16, heads=[2, 17, 28])


def test_fused_estimate_select_128k_and_most_blocks():
    """The fused stage 1-2 at the headline size (16-row bands) and at 4096 key blocks (4-row bands):
    lists against the oracle, and the whole chained output against the unfused path's."""
    big = wl.small("max_blocks_b64", seed=51, num_q_heads=2, num_kv_heads=1, seq_lens=(4096 * 64 - 17,),
                   block_size=64, k_start=(40,), n_sink=2, n_local=2, outliers=(32,))
    for w in (wl.LLAMA_128K, big):
        say("case", w.name, "fused")
        data, qkv = tensors_for(w)
        pf = pu.device_prefill(w, data)
        pf.run(fused=True)
        torch.cuda.synchronize()
        scores = pu.oracle_estimate(w, qkv)[3]
        _, counts, indices = pu.oracle_select(w, scores)
        same = pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, scores, say)
        assert same.mean() > 0.99
        fused_out, fused_counts, fused_idx = pf.out.clone(), pf.counts.clone(), pf.indices.clone()
        pf.run(fused=False)
        torch.cuda.synchronize()
        agree = (fused_idx == pf.indices).all(dim=2) & (fused_counts == pf.counts)      # [Hq, R]
        assert agree.float().mean().item() > 0.99
        B = w.block_size
        for (lo, hi, nb, row0) in so.sequence_table(w.cu_seqlens, B):
            rows_ok = agree[:, row0:row0 + nb].all(dim=0).cpu().numpy()
            for i in np.nonzero(rows_ok)[0]:
                t0, t1 = lo + i * B, min(lo + (i + 1) * B, hi)
                assert torch.equal(fused_out[t0:t1], pf.out[t0:t1])
        del pf
        torch.cuda.empty_cache()


def test_most_blocks_per_sequence_b64_ragged():
    """STEM_MAX_BLOCKS key blocks in one sequence (B = 64, 262 127 tokens, partial last block): the
    widest selection rows (64 keys per lane), the most score tiles, the longest causal ramp."""
    w = wl.small("max_blocks_b64", seed=51, num_q_heads=2, num_kv_heads=1, seq_lens=(4096 * 64 - 17,),
                 block_size=64, k_start=(40,), n_sink=2, n_local=2, outliers=(32,))
    assert so.total_rows(w.cu_seqlens, w.block_size) == (4096, 4096)
    full_size_case(w, 10, heads=[0, 1])
