"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded tensors.
Needs a real MI355X: every test here is marked gpu."""
import numpy as np
import pytest
import torch

from oracle import stem_oracle as so
from paper_2603_06274_amd import binding as sb
from paper_2603_06274_amd import workloads as wl

from paper_2603_06274_amd.prefill import StemPrefill

import parity_util as pu

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


SMALL = {
    # ragged single sequence, GQA 2:1, B = 64
    "ragged_b64": wl.small("ragged_b64", seed=21, num_q_heads=4, num_kv_heads=2, seq_lens=(1000,),
                           block_size=64, k_start=(6,), n_sink=1, n_local=1, outliers=(2,)),
    # packed batch with an empty and a sub-block sequence, GQA 4:1, B = 128
    "packed_b128": wl.small("packed_b128", seed=22, num_q_heads=8, num_kv_heads=2,
                            seq_lens=(700, 0, 1536, 130, 50), block_size=128, k_start=(3, 1, 5, 2, 1),
                            n_sink=1, n_local=2, outliers=(1, 0, 2, 1, 1)),
    # more than 64 blocks: several score tiles per row, B = 128, MHA
    "long_b128": wl.small("long_b128", seed=23, num_q_heads=2, num_kv_heads=2, seq_lens=(9000,),
                          block_size=128, k_start=(12,), n_sink=2, n_local=2, outliers=(6,)),
    # paper preset windows (4 initial + 4 local, minimum budget) on a short sequence
    "preset_b128": wl.small("preset_b128", seed=24, num_q_heads=4, num_kv_heads=1, seq_lens=(4096,),
                            block_size=128, k_start=(6.4,), n_sink=4, n_local=4, outliers=(3,), k_min=10),
    # the largest batch: 64 sequences of 0..300 tokens (empty ones and single tokens included)
    "batch64_b64": wl.small("batch64_b64", seed=26, num_q_heads=4, num_kv_heads=2,
                            seq_lens=tuple([0, 1, 64, 65, 300, 2] + [(37 * x) % 301 for x in range(58)]),
                            block_size=64, k_start=tuple([2] * 64), n_sink=1, n_local=1, outliers=tuple([1] * 64)),
    # a start budget of zero: every row keeps exactly its forced windows
    "forced_only_b128": wl.small("forced_only_b128", seed=28, num_q_heads=2, num_kv_heads=1, seq_lens=(2000, 300),
                                 block_size=128, k_start=(0, 0), n_sink=2, n_local=3, outliers=(1, 1)),
    # 8 and 4 KV heads at a size the oracle does whole: the two workgroup -> XCD mappings of stage 3
    # that the benchmark layers use (one XCD per KV head; two XCDs per KV head taking alternate rows)
    "kv8_b128": wl.small("kv8_b128", seed=61, num_q_heads=16, num_kv_heads=8, seq_lens=(2900, 1300),
                         block_size=128, k_start=(6, 4), n_sink=2, n_local=2, outliers=(3, 2)),
    "kv4_gqa7_b128": wl.small("kv4_gqa7_b128", seed=62, num_q_heads=28, num_kv_heads=4, seq_lens=(3333,),
                              block_size=128, k_start=(7,), n_sink=2, n_local=2, outliers=(4,)),
    "kv4_b64": wl.small("kv4_b64", seed=63, num_q_heads=8, num_kv_heads=4, seq_lens=(1500, 700, 64),
                        block_size=64, k_start=(6, 4, 1), n_sink=1, n_local=2, outliers=(3, 2, 1)),
    # no forced windows at all, uniform budget
    "noforce_b64": wl.small("noforce_b64", seed=25, num_q_heads=2, num_kv_heads=1, seq_lens=(2048, 1024),
                            block_size=64, k_start=(5, 3), n_sink=0, n_local=1, outliers=(2, 2), mu=1.0),
}


def run_both(w, rows=None, heads=None):
    say("case", w.name, "seed", w.seed, "T", w.total_tokens, "Hq/Hkv", w.num_q_heads, w.num_kv_heads,
        "B", w.block_size)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    pf = pu.device_prefill(w, data)
    pf.out.fill_(float("nan"))
    pf.lse.fill_(float("nan"))
    pf.run()
    torch.cuda.synchronize()
    q_bar, k_bar, m_v, scores = pu.oracle_estimate(w, qkv)
    budget, counts, indices = pu.oracle_select(w, scores)
    assert pf.budget_host.numpy().tolist() == budget.tolist()
    pu.check_pooled(pf, q_bar, k_bar, m_v)
    err = pu.check_scores(pf.scores.cpu().numpy(), scores)
    same = pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, scores, say)
    o_out, o_lse = so.sparse_attention(*qkv, w.cu_seqlens, w.block_size, counts, indices,
                                       w.softmax_scale, heads=heads, rows=rows)
    # compare the chained output on rows whose lists agree
    B = w.block_size
    for (lo, hi, nb, row0) in so.sequence_table(w.cu_seqlens, B):
        for i in range(nb):
            for h in range(w.num_q_heads):
                if not same[h, row0 + i]:
                    o_out[lo + i * B:min(lo + (i + 1) * B, hi), h] = np.nan
                    o_lse[h, lo + i * B:min(lo + (i + 1) * B, hi)] = np.nan
    keys = pu.ListedKeys(qkv, w.cu_seqlens, w.block_size, counts, indices, w.softmax_scale)
    max_abs, rel_l2 = pu.check_output(pf.out, o_out, w.name, say, keys)
    lse_err = pu.check_lse(pf.lse, o_lse, w.name)
    # out and lse were NaN before the run: every row of every head has been written
    assert not torch.isnan(pf.out).any().item() and not torch.isnan(pf.lse).any().item()
    say("%s: score err %.3g, out max-abs %.4g rel-L2 %.4g, lse err %.3g" % (w.name, err, max_abs, rel_l2, lse_err))
    return pf, data, qkv, (counts, indices)


@pytest.mark.parametrize("name", sorted(SMALL))
def test_small_cases_whole_path(name):
    run_both(SMALL[name])


def test_tiny_4k_whole_path():
    run_both(wl.TINY_4K)


STRIDED = {
    # tails of 40 and 3 tokens: with S >= 4 the last block of the second sequence has empty classes
    "tails_b64": wl.small("tails_b64", seed=31, num_q_heads=4, num_kv_heads=2, seq_lens=(1000, 67),
                          block_size=64, k_start=(6, 2), n_sink=1, n_local=1, outliers=(2, 1)),
    "packed_b128": SMALL["packed_b128"],
    "long_b128": SMALL["long_b128"],
}


@pytest.mark.parametrize("ad_stride", [2, 4, 8, 16])
@pytest.mark.parametrize("name", sorted(STRIDED))
def test_anti_diagonal_strides_estimate_and_select(name, ad_stride):
    """Stages 1-2 with S partial means per block (the strided anti-diagonal sample of the block's
    logits); stage 3 does not depend on S."""
    w = STRIDED[name]
    say("case", w.name, "seed", w.seed, "ad_stride", ad_stride)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    pf = pu.device_prefill(w, data, ad_stride=ad_stride)
    pf.estimate()
    pf.select()
    torch.cuda.synchronize()
    q_bar, k_bar, m_v, scores = pu.oracle_estimate(w, qkv, ad_stride)
    assert q_bar.shape[2] == ad_stride
    pu.check_pooled(pf, q_bar, k_bar, m_v)
    err = pu.check_scores(pf.scores.cpu().numpy(), scores)
    budget, counts, indices = pu.oracle_select(w, scores)
    pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, scores, say)
    # the strided sample is a different estimate from the block mean, not a relabelling of it
    mean_scores = pu.oracle_estimate(w, qkv, 1)[3]
    fin = np.isfinite(scores)
    assert np.abs(scores[fin] - mean_scores[fin]).max() > 1e-3
    say("%s S=%d: score err %.3g" % (w.name, ad_stride, err))


@pytest.mark.parametrize("ad_stride,fused,head_dim", [(1, False, 128), (4, True, 128), (2, False, 64), (1, True, 256)])
def test_chunked_prefill_gives_the_rows_of_the_one_piece_call(ad_stride, fused, head_dim):
    """A prompt processed in three chunks against its growing KV, with one workspace kept between
    the calls (each call pools only its own blocks): every chunk's scores, lists, outputs and lse
    are bit-identical to the matching rows of the one-piece call, whose parity with the oracle is
    then checked on the assembled output."""
    w = wl.small("chunks_b128", seed=41, num_q_heads=4, num_kv_heads=2, seq_lens=(1536, 700),
                 block_size=128, k_start=(6, 4), n_sink=1, n_local=2, outliers=(3, 2), head_dim=head_dim)
    B, cu = w.block_size, list(w.cu_seqlens)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    full = pu.device_prefill(w, data, ad_stride=ad_stride)
    dump = torch.empty_like(full.scores) if fused else None
    if fused:
        full.estimate_select(dump)
        full.scores.copy_(dump)
        full.attend()
    else:
        full.run()
    torch.cuda.synchronize()
    dev = torch.device("cuda:0")
    q, k, v = (data[x].to(dev) for x in "qkv")
    calls = [([0, 0], [512, 256]), ([512, 256], [1024, 700]), ([1024, 700], [1536, 700])]
    need = 0
    for starts, ends in calls:
        shape = sb.Shape.from_tensors(q, k, B, cu, (starts, ends))
        need = max(need, sb.stem_workspace_bytes(shape, ad_stride))
    ws = torch.full((need,), 0xFF, dtype=torch.uint8, device=dev)     # NaN patterns where nothing was pooled
    out = torch.zeros_like(full.out)
    full_row0 = [0, -(-(cu[1] - cu[0]) // B)]
    for starts, ends in calls:
        say("chunk", starts, ends)
        qc = torch.cat([q[cu[s] + starts[s]:cu[s] + ends[s]] for s in range(2)]).contiguous()
        pf = StemPrefill(qc, k, v, cu, B, w.k_start_blocks, w.mu, w.k_min, w.n_sink, w.n_local, w.beta,
                         w.route_scale, w.softmax_scale, want_lse=True, chunk=(starts, ends), workspace=ws,
                         ad_stride=ad_stride, fill_scores=True)
        if fused:
            chunk_dump = torch.empty_like(pf.scores)
            pf.estimate_select(chunk_dump)
            pf.scores.copy_(chunk_dump)
            pf.attend()
        else:
            pf.run()
        torch.cuda.synchronize()
        r = t = 0
        for s in range(2):
            first, rows = starts[s] // B, -(-ends[s] // B) - starts[s] // B if ends[s] > starts[s] else 0
            fr = full_row0[s] + first
            n_tok = ends[s] - starts[s]
            nb = pf.nbmax
            assert torch.equal(pf.scores[:, r:r + rows, :nb], full.scores[:, fr:fr + rows, :nb])
            assert torch.isinf(full.scores[:, fr:fr + rows, nb:]).all()
            assert torch.equal(pf.counts[:, r:r + rows], full.counts[:, fr:fr + rows])
            kk = min(pf.kmax, full.kmax)
            assert torch.equal(pf.indices[:, r:r + rows, :kk], full.indices[:, fr:fr + rows, :kk])
            assert (pf.indices[:, r:r + rows, kk:] == -1).all() and (full.indices[:, fr:fr + rows, kk:] == -1).all()
            lo = cu[s] + starts[s]
            assert torch.equal(pf.out[t:t + n_tok], full.out[lo:lo + n_tok])
            assert torch.equal(pf.lse[:, t:t + n_tok], full.lse[:, lo:lo + n_tok])
            out[lo:lo + n_tok] = pf.out[t:t + n_tok]
            r += rows
            t += n_tok
        assert r == pf.rows and t == qc.shape[0]
    # and the assembled chunks against the oracle's one-piece result
    scores = pu.oracle_estimate(w, qkv, ad_stride)[3]
    _, counts, indices = pu.oracle_select(w, scores)
    same = pu.check_lists(w, full.counts.cpu().numpy(), full.indices.cpu().numpy(), counts, indices, scores, say)
    assert same.all()
    o_out, _ = so.sparse_attention(*qkv, cu, B, counts, indices, w.softmax_scale)
    pu.check_output(out, o_out, w.name, say, pu.ListedKeys(qkv, cu, B, counts, indices, w.softmax_scale))


@pytest.mark.parametrize("ad_stride", [1, 4])
@pytest.mark.parametrize("name", ["ragged_b64", "packed_b128", "long_b128", "batch64_b64", "noforce_b64"])
def test_fused_estimate_select(name, ad_stride):
    """Stages 1-2 without the score tensor: the scores the fused kernel saw (debug dump) and its
    lists against the oracle; the same lists with and without the dump."""
    w = SMALL[name]
    say("case", w.name, "seed", w.seed, "fused, ad_stride", ad_stride)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    pf = pu.device_prefill(w, data, ad_stride=ad_stride)
    dump = torch.full_like(pf.scores, float("nan"))
    pf.estimate_select(dump)
    torch.cuda.synchronize()
    counts_dbg, idx_dbg = pf.counts.clone(), pf.indices.clone()
    q_bar, k_bar, m_v, scores = pu.oracle_estimate(w, qkv, ad_stride)
    pu.check_pooled(pf, q_bar, k_bar, m_v)
    pu.check_scores(dump.cpu().numpy(), scores)
    _, counts, indices = pu.oracle_select(w, scores)
    pu.check_lists(w, counts_dbg.cpu().numpy(), idx_dbg.cpu().numpy(), counts, indices, scores, say)
    pf.counts.fill_(-7)
    pf.indices.fill_(-7)
    pf.estimate_select(None)
    torch.cuda.synchronize()
    assert torch.equal(pf.counts, counts_dbg) and torch.equal(pf.indices, idx_dbg)


@pytest.mark.parametrize("how", ["max", "mean"])
@pytest.mark.parametrize("name", ["packed_b128", "ragged_b64", "odd_b64"])
def test_group_shared_selection(name, how):
    """One list per (KV head, row) from the group-reduced metric, used by all heads of the group.
    odd_b64 has 15 x 15 scores per head, which the reduction cannot take four at a time."""
    w = SMALL[name] if name in SMALL else wl.small("odd_b64", seed=27, num_q_heads=6, num_kv_heads=2,
                                                    seq_lens=(15 * 64 - 3,), block_size=64, k_start=(5,),
                                                    n_sink=1, n_local=1, outliers=(2,))
    G = w.num_q_heads // w.num_kv_heads
    say("case", w.name, "seed", w.seed, "group", how, "G", G)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    dev = torch.device("cuda:0")
    q, k, v = (data[x].to(dev) for x in "qkv")
    pf = StemPrefill(q, k, v, w.cu_seqlens, w.block_size, w.k_start_blocks, w.mu, w.k_min, w.n_sink,
                     w.n_local, w.beta, w.route_scale, w.softmax_scale, want_lse=True, group_share=how,
                     fill_scores=True)
    pf.run()
    torch.cuda.synchronize()
    scores = pu.oracle_estimate(w, qkv)[3]
    grouped = so.group_scores(scores, w.num_kv_heads, how)
    assert pf.counts.shape[0] == w.num_kv_heads
    pu.check_scores(pf.group_scores.cpu().numpy(), grouped)
    _, counts, indices = pu.oracle_select(w, grouped)
    same = pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, grouped, say)
    # every query head attends over its KV head's list
    o_out, o_lse = so.sparse_attention(*qkv, w.cu_seqlens, w.block_size, np.repeat(counts, G, axis=0),
                                       np.repeat(indices, G, axis=0), w.softmax_scale)
    B = w.block_size
    for (lo, hi, nb, row0) in so.sequence_table(w.cu_seqlens, B):
        for i in range(nb):
            for h in range(w.num_q_heads):
                if not same[h // G, row0 + i]:
                    o_out[lo + i * B:min(lo + (i + 1) * B, hi), h] = np.nan
                    o_lse[h, lo + i * B:min(lo + (i + 1) * B, hi)] = np.nan
    pu.check_output(pf.out, o_out, w.name, say,
                    pu.ListedKeys(qkv, w.cu_seqlens, B, np.repeat(counts, G, axis=0), np.repeat(indices, G, axis=0),
                                  w.softmax_scale))
    pu.check_lse(pf.lse, o_lse, w.name)
    # the shared lists differ from the per-head ones (the reduction does something)
    _, c_h, i_h = pu.oracle_select(w, scores)
    assert not np.array_equal(np.repeat(indices, G, axis=0)[:, :, :min(indices.shape[2], i_h.shape[2])],
                              i_h[:, :, :min(indices.shape[2], i_h.shape[2])])


def test_zero_blocks_in_the_inputs():
    """A key block of zeros (scores reduce to the magnitude term), a value block of zeros (its
    magnitude is ln 0 = -inf, clamped to 0 in the metric) and a query block of zeros (uniform
    attention over what it selects)."""
    w = wl.small("zeros_b64", seed=29, num_q_heads=4, num_kv_heads=2, seq_lens=(1024,), block_size=64,
                 k_start=(5,), n_sink=1, n_local=1, outliers=(2,))
    data = wl.generate(w)
    data["k"][3 * 64:4 * 64] = 0
    data["v"][5 * 64:6 * 64] = 0
    data["q"][9 * 64:10 * 64] = 0
    qkv = pu.host_arrays(data)
    pf = pu.device_prefill(w, data)
    pf.run()
    torch.cuda.synchronize()
    q_bar, k_bar, m_v, scores = pu.oracle_estimate(w, qkv)
    assert np.isneginf(m_v[:, 5]).all()
    pu.check_pooled(pf, q_bar, k_bar, m_v)
    pu.check_scores(pf.scores.cpu().numpy(), scores)
    _, counts, indices = pu.oracle_select(w, scores)
    same = pu.check_lists(w, pf.counts.cpu().numpy(), pf.indices.cpu().numpy(), counts, indices, scores, say)
    o_out, _ = so.sparse_attention(*qkv, w.cu_seqlens, w.block_size, counts, indices, w.softmax_scale)
    for h, r in np.argwhere(~same):
        o_out[r * 64:(r + 1) * 64, h] = np.nan
    pu.check_output(pf.out, o_out, w.name, say,
                    pu.ListedKeys(qkv, w.cu_seqlens, w.block_size, counts, indices, w.softmax_scale))


@pytest.mark.parametrize("name", ["long_b128", "packed_b128", "kv8_b128"])
def test_scores_without_the_non_causal_fill(name):
    """fill_non_causal = 0: tiles (64 rows x 64 key blocks) without a causal pair are not touched, the
    others are written exactly as with the fill, and the selection and the output do not change."""
    w = SMALL[name] if name != "long_b128" else wl.small("long_b128", seed=23, num_q_heads=2, num_kv_heads=2,
                                                          seq_lens=(20000,), block_size=128, k_start=(12,),
                                                          n_sink=2, n_local=2, outliers=(6,))
    data = wl.generate(w)
    full = pu.device_prefill(w, data)                  # fill_scores = True
    full.run()
    lean = pu.device_prefill(w, data)
    lean.fill_scores = False
    lean.scores.fill_(float("nan"))
    lean.run()
    torch.cuda.synchronize()
    a, b = full.scores.cpu().numpy(), lean.scores.cpu().numpy()
    touched = ~np.isnan(b)
    assert np.array_equal(a[touched].view(np.int32), b[touched].view(np.int32))     # bit-identical where written
    causal = np.isfinite(a)
    assert touched[causal].all()                       # every causal entry is written
    untouched = int((~touched).sum())
    R, nbmax = full.rows, full.nbmax
    say("%s: %d of %d score entries left untouched" % (w.name, untouched, a.size))
    if max(w.blocks_per_seq) > 128:
        assert untouched > a.size // 8                 # whole tiles above the diagonal were skipped
    # an untouched entry lies in a 64 x 64 tile that holds no causal pair
    for (lo, hi, nb, row0) in so.sequence_table(w.cu_seqlens, w.block_size):
        for i in range(nb):
            first_skipped = 64 * (i // 64) + 64        # first key block of the first tile above the row's tile row
            assert touched[:, row0 + i, :min(first_skipped, nbmax)].all()
            assert not touched[:, row0 + i, first_skipped:].any()
    assert torch.equal(full.counts, lean.counts) and torch.equal(full.indices, lean.indices)
    assert torch.equal(full.out, lean.out) and torch.equal(full.lse, lean.lse)


def test_select_is_bit_exact_on_shared_fp32_scores():
    """Stage 2 alone, on one fp32 score tensor given to both sides (exactly representable in fp64, so
    no near-tie allowance), with planted exact ties, +-0, and equal rows."""
    r = np.random.default_rng(31)
    for (nb, B, Hq, n_sink, n_local, ks) in [(40, 64, 3, 2, 1, 9), (300, 128, 2, 3, 2, 40), (70, 64, 2, 0, 1, 7),
                                              (1100, 128, 1, 2, 2, 60)]:
        say("select case nb", nb, "Hq", Hq)
        cu = [0, nb * B - 5]
        sc = r.standard_normal((Hq, nb, nb)).astype(np.float32)
        sc = np.round(sc * 4) / 4                          # many exact ties
        sc[:, :, 3] = 0.0
        sc[:, ::2, 5] = -0.0
        sc[0, nb // 2] = 1.0                               # a fully tied row
        sc = np.where(np.tril(np.ones((nb, nb), bool))[None], sc, -np.inf).astype(np.float32)
        budget = so.packed_budget(cu, B, [ks], 0.7, 0, n_sink, n_local)
        want_c, want_i = so.select_blocks(sc.astype(np.float64), budget, cu, B, n_sink, n_local)
        shape = sb.Shape(Hq, 1, 128, B, cu, (Hq * 128, 128), (128, 128))
        kmax = int(budget.max())
        dev = torch.device("cuda:0")
        counts = torch.zeros((Hq, nb), dtype=torch.int32, device=dev)
        idx = torch.zeros((Hq, nb, kmax), dtype=torch.int32, device=dev)
        sb.stem_select(shape, torch.from_numpy(sc).to(dev), torch.from_numpy(budget).to(dev), n_sink, n_local,
                       counts, idx, kmax)
        torch.cuda.synchronize()
        assert np.array_equal(counts.cpu().numpy(), want_c)
        assert np.array_equal(idx.cpu().numpy(), want_i[:, :, :kmax])
        # a list pitch below the largest budget cuts the rows to it: the same as a clipped budget
        cut = max(n_sink + n_local, kmax // 2)
        want_c, want_i = so.select_blocks(sc.astype(np.float64), np.minimum(budget, cut), cu, B, n_sink, n_local)
        idx_cut = torch.zeros((Hq, nb, cut), dtype=torch.int32, device=dev)
        sb.stem_select(shape, torch.from_numpy(sc).to(dev), torch.from_numpy(budget).to(dev), n_sink, n_local,
                       counts, idx_cut, cut)
        torch.cuda.synchronize()
        assert np.array_equal(counts.cpu().numpy(), want_c)
        assert np.array_equal(idx_cut.cpu().numpy(), want_i[:, :, :cut])


def test_attention_on_given_lists_full_budget_and_random():
    """Stage 3 alone on caller-made lists: the full causal budget (dense attention) and random
    ascending lists that hold the diagonal; packed, ragged, GQA 4:1."""
    w = wl.small("attn_lists", seed=41, num_q_heads=8, num_kv_heads=2, seq_lens=(1300, 640, 77), block_size=128,
                 k_start=(1, 1, 1), outliers=(1, 1, 1))
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    cu, B, Hq = w.cu_seqlens, w.block_size, w.num_q_heads
    R, nbmax = so.total_rows(cu, B)
    r = np.random.default_rng(42)
    for mode in ("full", "random"):
        counts = np.zeros((Hq, R), np.int32)
        idx = np.full((Hq, R, nbmax), -1, np.int32)
        for (_, _, nb, row0) in so.sequence_table(cu, B):
            for i in range(nb):
                for h in range(Hq):
                    if mode == "full":
                        pick = list(range(i + 1))
                    else:
                        pick = sorted(set(r.choice(i + 1, size=min(3, i + 1), replace=False).tolist()) | {i})
                    counts[h, row0 + i] = len(pick)
                    idx[h, row0 + i, :len(pick)] = pick
        say("attention lists mode", mode)
        dev = torch.device("cuda:0")
        q, k, v = (data[x].to(dev) for x in "qkv")
        shape = sb.Shape.from_tensors(q, k, B, cu)
        out = torch.zeros_like(q)
        lse = torch.zeros((Hq, q.shape[0]), dtype=torch.float32, device=dev)
        sb.stem_sparse_attn(shape, q, k, v, torch.from_numpy(counts).to(dev), torch.from_numpy(idx).to(dev),
                            nbmax, w.softmax_scale, out, lse)
        torch.cuda.synchronize()
        o_out, o_lse = so.sparse_attention(*qkv, cu, B, counts, idx, w.softmax_scale)
        pu.check_output(out, o_out, mode, say, pu.ListedKeys(qkv, cu, B, counts, idx, w.softmax_scale))
        pu.check_lse(lse, o_lse, mode)


@pytest.mark.parametrize("B,d", [(128, 128), (64, 128), (128, 64), (64, 256)])
def test_rows_without_a_usable_entry_give_zeros_and_minus_infinity(B, d):
    """Rows whose list is empty (count 0) or holds only entries outside 0..i: the sums over an empty
    key set, out = 0 and lse = -inf (the oracle states the same for an empty list; junk-only lists
    cannot be expressed there, so their expectation is written here).  The other rows of the same
    launch, some sharing a KV head with the empty ones, still match the oracle."""
    w = wl.small("empty_rows", seed=71, num_q_heads=4, num_kv_heads=2, seq_lens=(5 * B + 9, 2 * B), block_size=B,
                 k_start=(3, 2), outliers=(1, 1), head_dim=d)
    data = wl.generate(w)
    qkv = pu.host_arrays(data)
    cu, Hq = w.cu_seqlens, w.num_q_heads
    R, nbmax = so.total_rows(cu, B)
    kmax = nbmax + 2
    counts = np.zeros((Hq, R), np.int32)
    idx = np.full((Hq, R, kmax), -1, np.int32)
    o_counts, o_idx = counts.copy(), idx.copy()
    kind = {}                                              # (h, r) -> "empty" / "junk"
    r_ = np.random.default_rng(3)
    for (_, _, nb, row0) in so.sequence_table(cu, B):
        for i in range(nb):
            for h in range(Hq):
                r = row0 + i
                what = ["full", "empty", "junk"][int(r_.integers(0, 3))] if (h, i) != (0, 0) else "empty"
                if what == "full":
                    pick = list(range(i + 1))
                    counts[h, r] = o_counts[h, r] = len(pick)
                    idx[h, r, :len(pick)] = o_idx[h, r, :len(pick)] = pick
                elif what == "junk":
                    junk = [-7, i + 1, 2 ** 30][:int(r_.integers(1, 4))]
                    counts[h, r] = len(junk)
                    idx[h, r, :len(junk)] = junk
                    kind[(h, r)] = what
                else:
                    idx[h, r, :2] = [0, i]                 # beyond the count: must not be read as entries
                    kind[(h, r)] = what
    assert {"empty", "junk"} <= set(kind.values())
    dev = torch.device("cuda:0")
    qd, kd, vd = (data[x].to(dev) for x in "qkv")
    shape = sb.Shape.from_tensors(qd, kd, B, cu)
    out = torch.full_like(qd, float("nan"))
    lse = torch.full((Hq, qd.shape[0]), float("nan"), dtype=torch.float32, device=dev)
    sb.stem_sparse_attn(shape, qd, kd, vd, torch.from_numpy(counts).to(dev), torch.from_numpy(idx).to(dev), kmax,
                        w.softmax_scale, out, lse)
    torch.cuda.synchronize()
    o_out, o_lse = so.sparse_attention(*qkv, cu, B, o_counts, o_idx, w.softmax_scale)
    for (lo, hi, nb, row0) in so.sequence_table(cu, B):
        for i in range(nb):
            for h in range(Hq):
                if (h, row0 + i) in kind:
                    t0, t1 = lo + i * B, min(lo + (i + 1) * B, hi)
                    assert not o_out[t0:t1, h].any() and np.isneginf(o_lse[h, t0:t1]).all()    # the oracle's empty list
                    assert (out[t0:t1, h] == 0).all().item(), (kind[(h, row0 + i)], h, i)
                    assert torch.isneginf(lse[h, t0:t1]).all().item(), (kind[(h, row0 + i)], h, i)
                    o_out[t0:t1, h] = np.nan
                    o_lse[h, t0:t1] = np.nan
    pu.check_output(out, o_out, w.name, say, pu.ListedKeys(qkv, cu, B, o_counts, o_idx, w.softmax_scale))
    pu.check_lse(lse, o_lse, w.name)
    assert not torch.isnan(out).any().item() and not torch.isnan(lse).any().item()


@pytest.mark.parametrize("sign", [1.0, -1.0])
@pytest.mark.parametrize("B,d", [(128, 128), (64, 128), (128, 64), (64, 64), (128, 256), (64, 256)])
def test_attention_reference_moves_and_unusable_entries(B, d, sign):
    """Two things ordinary data does not reach.  (1) Logits far outside the exponent range of a
    fixed reference, growing along the keys and jumping inside blocks, so that the softmax reference
    has to move at every check point of a block (and O is rescaled) - against the oracle's
    max-subtracted fp64 softmax; with sign = -1 every logit is hugely negative instead, so a
    reference of zero would lose the row.  (2) List entries outside 0..i, also at the head of a
    list: they must contribute nothing."""
    torch.manual_seed(7)
    Hq, Hkv, T = 4, 2, 1536
    cu = [0, 1000, T]
    q = torch.randn(T, Hq, d) * 3.0
    k = torch.randn(T, Hkv, d)
    v = torch.randn(T, Hkv, d)
    ramp = 1.0 + 6.0 * torch.arange(T).float() / T                     # later keys score higher
    ramp[40::97] *= 3.0                                                # spikes inside blocks
    k = sign * (k * ramp[:, None, None] + 0.5 * q.view(T, Hkv, 2, d).mean(2) * ramp[:, None, None])
    q, k, v = (x.to(torch.bfloat16) for x in (q, k, v))
    qkv = tuple(x.float().numpy() for x in (q, k, v))
    scale = d ** -0.5
    logits = np.einsum("td,sd->ts", qkv[0][:, 0], qkv[1][:, 0]) * scale
    assert np.abs(logits).max() > 200.0                                # e^200 overflows fp32
    R, nbmax = so.total_rows(cu, B)
    counts = np.zeros((Hq, R), np.int32)
    idx = np.full((Hq, R, nbmax + 3), -1, np.int32)
    clean_c, clean_i = counts.copy(), idx.copy()
    r = np.random.default_rng(5)
    for (_, _, nb, row0) in so.sequence_table(cu, B):
        for i in range(nb):
            for h in range(Hq):
                pick = list(range(i + 1))
                clean_c[h, row0 + i] = len(pick)
                clean_i[h, row0 + i, :len(pick)] = pick
                junk = [-3, i + 1 + int(r.integers(0, 50)), 2 ** 30][:int(r.integers(0, 4))]
                dirty = junk[2:] + pick[:len(pick) // 2] + junk[:1] + pick[len(pick) // 2:] + junk[1:2]
                counts[h, row0 + i] = len(dirty)
                idx[h, row0 + i, :len(dirty)] = dirty
    dev = torch.device("cuda:0")
    qd, kd, vd = (x.to(dev) for x in (q, k, v))
    shape = sb.Shape.from_tensors(qd, kd, B, cu)
    o_out, o_lse = so.sparse_attention(*qkv, cu, B, clean_c, clean_i, scale)
    for name, c, ix in (("clean", clean_c, clean_i), ("with unusable entries", counts, idx)):
        out = torch.full_like(qd, float("nan"))
        lse = torch.zeros((Hq, T), dtype=torch.float32, device=dev)
        sb.stem_sparse_attn(shape, qd, kd, vd, torch.from_numpy(c).to(dev), torch.from_numpy(ix).to(dev),
                            ix.shape[2], scale, out, lse)
        torch.cuda.synchronize()
        max_abs, rel_l2 = pu.check_output(out, o_out, name, say, pu.ListedKeys(qkv, cu, B, clean_c, clean_i, scale))
        if name == "clean":                                           # lse is optional: same output without it
            out2 = torch.full_like(qd, float("nan"))
            sb.stem_sparse_attn(shape, qd, kd, vd, torch.from_numpy(c).to(dev), torch.from_numpy(ix).to(dev),
                                ix.shape[2], scale, out2, None)
            torch.cuda.synchronize()
            assert torch.equal(out, out2)
        err = np.abs(lse.cpu().numpy() - o_lse) / np.maximum(1.0, np.abs(o_lse))
        say("%s: max-abs %.4g rel-L2 %.4g, lse rel err %.3g" % (name, max_abs, rel_l2, err.max()))
        assert err.max() <= 5e-3


def test_side_stream_and_graph_replay():
    """The library enqueues on the caller's stream and neither allocates nor synchronises: the
    three calls run on a side stream, and captured into a HIP graph they replay to the same bits,
    with eager work and synchronisations between the replays."""
    w = SMALL["packed_b128"]
    data = wl.generate(w)
    pf = pu.device_prefill(w, data)
    want = pf.run().clone()
    want_idx, want_lse = pf.indices.clone(), pf.lse.clone()
    torch.cuda.synchronize()

    def wipe():
        pf.out.fill_(float("nan")); pf.indices.fill_(-5); pf.counts.fill_(-5); pf.scores.fill_(0); pf.lse.fill_(0)

    side = torch.cuda.Stream()
    wipe()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        pf.run()
    side.synchronize()
    assert torch.equal(pf.out, want) and torch.equal(pf.indices, want_idx) and torch.equal(pf.lse, want_lse)

    graph = torch.cuda.CUDAGraph()
    wipe()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        pf.run()
    for rep in range(3):
        wipe()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(pf.out, want) and torch.equal(pf.indices, want_idx) and torch.equal(pf.lse, want_lse), rep
        pf.run(fused=True)                               # eager work between the replays
        torch.cuda.synchronize()


def test_outputs_are_deterministic_and_strided_views_work():
    """Same inputs twice give bit-identical results; Q/K/V given as views of a fused [T, H, d] QKV
    buffer (non-trivial token stride) give the same result as contiguous tensors."""
    w = SMALL["packed_b128"]
    data = wl.generate(w)
    pf = pu.device_prefill(w, data)
    a = pf.run().clone()
    ia = pf.indices.clone()
    torch.cuda.synchronize()
    b = pf.run()
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(ia, pf.indices)
    dev = a.device
    Hq, Hkv = w.num_q_heads, w.num_kv_heads
    fused = torch.zeros((w.total_tokens, Hq + 2 * Hkv, 128), dtype=torch.bfloat16, device=dev)
    fused[:, :Hq] = data["q"].to(dev)
    fused[:, Hq:Hq + Hkv] = data["k"].to(dev)
    fused[:, Hq + Hkv:] = data["v"].to(dev)
    from paper_2603_06274_amd.prefill import StemPrefill
    pf2 = StemPrefill(fused[:, :Hq], fused[:, Hq:Hq + Hkv], fused[:, Hq + Hkv:], w.cu_seqlens, w.block_size,
                      w.k_start_blocks, w.mu, w.k_min, w.n_sink, w.n_local, w.beta, w.route_scale,
                      w.softmax_scale)
    c = pf2.run()
    torch.cuda.synchronize()
    assert torch.equal(pf2.indices, ia) and torch.equal(c, a)
