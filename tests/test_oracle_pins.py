"""Pins of the CPU oracle against things other than itself (no GPU needed).

The paper prints no worked numerical example, so each oracle function is held to what the paper
and the mathematics fix: brute force at token level, closed forms, textbook definitions, the
appendix's rank-equivalence argument, and invariants.  Each test names the mistake it would catch.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest

from oracle import stem_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
PAPER = json.load(open(os.path.join(GOLDEN, "paper_constants.json")))


def rng_qkv(seed, T, Hq, Hkv, d):
    r = np.random.default_rng(seed)
    return (r.standard_normal((T, Hq, d)), r.standard_normal((T, Hkv, d)),
            r.standard_normal((T, Hkv, d)))


# ------------------------------------------------------------------------------------------------
# stage 1
# ------------------------------------------------------------------------------------------------

def brute_route(q, k, cu, B, S, h, g, seq, i, j):
    """Mean of the token-level logits <Q_r, K_c> over the sampled cells of block (i, j): all B*B
    cells for S = 1, else the cells on the anti-diagonals (r + c) mod S == S - 1."""
    lo = cu[seq]
    acc, cnt = 0.0, 0
    for r in range(B):
        for c in range(B):
            if (r + c) % S != S - 1:
                continue
            acc += float(np.dot(q[lo + i * B + r, h], k[lo + j * B + c, g]))
            cnt += 1
    return acc / cnt


@pytest.mark.parametrize("S", [1, 2, 4])
def test_routing_term_is_mean_of_block_logits(S):
    # catches: sum-vs-mean pooling, Q/K transposed, wrong GQA map, residue pairing a<->S-1-a wrong,
    # packed sequences leaking into each other
    B, Hq, Hkv, d = 4, 4, 2, 8
    cu = [0, 12, 20]
    q, k, v = rng_qkv(1, 20, Hq, Hkv, d)
    qb, kb, mv = so.pool_blocks(q, k, v, cu, B, ad_stride=S)
    sc = so.oam_scores(qb, kb, mv, cu, B, beta=0.0, route_scale=1.0)
    assert sc.shape == (Hq, 5, 3)
    rows = [(0, 0, 0), (0, 1, 1), (0, 2, 2), (1, 0, 3), (1, 1, 4)]
    for h in range(Hq):
        g = h // 2
        for seq, i, r in rows:
            for j in range(3):
                nb = 3 if seq == 0 else 2
                if j <= i and j < nb:
                    want = brute_route(q, k, cu, B, S, h, g, seq, i, j)
                    assert sc[h, r, j] == pytest.approx(want, rel=1e-12, abs=1e-12)
                else:
                    assert sc[h, r, j] == -np.inf


def test_route_scale_multiplies_routing_only():
    B = 4
    q, k, v = rng_qkv(2, 16, 2, 1, 8)
    v *= 3.0
    qb, kb, mv = so.pool_blocks(q, k, v, [0, 16], B)
    s1 = so.oam_scores(qb, kb, mv, [0, 16], B, beta=0.3, route_scale=1.0)
    s0 = so.oam_scores(qb, kb, mv, [0, 16], B, beta=0.3, route_scale=0.0)
    sr = so.oam_scores(qb, kb, mv, [0, 16], B, beta=0.0, route_scale=1.0)
    fin = np.isfinite(s1)
    assert np.allclose(s1[fin], (s0 + sr)[fin], rtol=0, atol=1e-12)
    assert np.allclose(so.oam_scores(qb, kb, mv, [0, 16], B, beta=0.0, route_scale=0.25)[fin],
                       0.25 * sr[fin], atol=1e-12)


def test_magnitude_term_closed_forms():
    # catches: wrong log base, mean instead of max pooling, missing clamp, beta misplaced,
    # norm^2 instead of norm
    B, d = 4, 8
    cu = [0, 16]
    q, k, v = rng_qkv(3, 16, 2, 2, d)
    beta = PAPER["beta"]["value"]
    # unit-norm values: ln 1 = 0, the metric is pure routing (the SAM special case, beta-ablation)
    v1 = v / np.linalg.norm(v, axis=2, keepdims=True)
    qb, kb, mv = so.pool_blocks(q, k, v1, cu, B)
    assert np.allclose(mv, 0.0, atol=1e-12)
    sam = so.oam_scores(qb, kb, mv, cu, B, beta=0.0)
    oam = so.oam_scores(qb, kb, mv, cu, B, beta=beta)
    fin = np.isfinite(sam)
    assert np.allclose(sam[fin], oam[fin], atol=1e-12)
    # scale one key block of KV head 1 by 4: its column rises by beta*ln 4 for that head's group only
    v4 = v1.copy()
    v4[8:12, 1] *= 4.0
    _, _, mv4 = so.pool_blocks(q, k, v4, cu, B)
    oam4 = so.oam_scores(qb, kb, mv4, cu, B, beta=beta)
    delta = np.where(fin, oam4, 0.0) - np.where(fin, oam, 0.0)
    want = np.zeros_like(delta)
    want[1, 2:, 2] = beta * math.log(4.0)            # head 1 <-> kv head 1; rows >= 2 see block 2
    assert np.allclose(delta, want, atol=1e-12)
    assert beta * math.log(4.0) == pytest.approx(0.277259, abs=1e-6)
    # max pooling: a single large token decides the block's magnitude
    v5 = v1 * 0.5
    v5[5, 0] *= 2.0 * math.e ** 2                     # norm e^2 -> ln = 2
    _, _, mv5 = so.pool_blocks(q, k, v5, cu, B)
    assert mv5[0, 1] == pytest.approx(2.0, abs=1e-12)
    # norms below one are clamped away; all-zero values give no contribution and no NaN
    assert np.all(mv5[1] < 0)
    s5 = so.oam_scores(qb, kb, mv5, cu, B, beta=1.0)
    assert np.allclose(s5[1][fin[1]] - sam[1][fin[1]], 0.0, atol=1e-12)
    _, _, mv0 = so.pool_blocks(q, k, np.zeros_like(v), cu, B)
    s0 = so.oam_scores(qb, kb, mv0, cu, B, beta=1.0)
    assert np.allclose(s0[fin], sam[fin], atol=1e-12) and not np.isnan(s0).any()


def test_ragged_tail_pools_valid_tokens_only():
    B = 4
    q, k, v = rng_qkv(4, 10, 1, 1, 8)
    qb, kb, mv = so.pool_blocks(q, k, v, [0, 10], B)
    assert qb.shape[1] == 3
    assert np.allclose(qb[0, 2, 0], q[8:10, 0].mean(axis=0))
    assert np.allclose(kb[0, 2, 0], k[8:10, 0].mean(axis=0))
    assert mv[0, 2] == pytest.approx(np.log(np.linalg.norm(v[8:10, 0], axis=1)).max())


def brute_route_ragged(q, k, lo, hi, B, S, h, g, i, j):
    """Token-level statement of the routing term when blocks may be partial: the average over the S
    anti-diagonal classes a of the mean logit over the valid cells (r, c) of block pair (i, j) with
    r = a and c = S-1-a (mod S); a class with no valid cell contributes 0.  Also returns the plain
    mean over all sampled valid cells, which is a different number when the classes are uneven."""
    per_class, all_cells = [], []
    for a in range(S):
        cells = []
        for r in range(B):
            for c in range(B):
                tq, tk = lo + i * B + r, lo + j * B + c
                if tq < hi and tk < hi and r % S == a and c % S == S - 1 - a:
                    cells.append(float(np.dot(q[tq, h], k[tk, g])))
        per_class.append(sum(cells) / len(cells) if cells else 0.0)
        all_cells += cells
    return sum(per_class) / S, (sum(all_cells) / len(all_cells) if all_cells else None)


@pytest.mark.parametrize("S", [2, 4, 8])
def test_strided_routing_term_on_partial_blocks(S):
    # The reading taken for ad_stride > 1 on a partial last block: Algorithm 1 pools first and
    # multiplies afterwards, so each residue class is normalised by its own number of valid tokens
    # when it is pooled; the score is the mean over classes of the class-mean logits (an empty class
    # counts as 0), NOT the mean over all sampled valid cells.  On full blocks the two coincide.
    # catches: dividing a class by B/S instead of its valid count, dropping the 1/S, pairing a with a,
    # skipping empty classes in the average, pooling padding rows
    B, Hq, Hkv, d = 8, 2, 1, 6
    cu = [0, 19, 33]            # tails of 3 tokens (classes 3.. empty for S >= 4) and of 6 tokens (uneven classes)
    q, k, v = rng_qkv(17, 33, Hq, Hkv, d)
    qb, kb, mv = so.pool_blocks(q, k, v, cu, B, ad_stride=S)
    sc = so.oam_scores(qb, kb, mv, cu, B, beta=0.0, route_scale=1.0)
    differs = 0
    row0 = 0
    for s_ in range(2):
        lo, hi = cu[s_], cu[s_ + 1]
        nb = -(-(hi - lo) // B)
        for i in range(nb):
            for j in range(i + 1):
                for h in range(Hq):
                    want, cell_mean = brute_route_ragged(q, k, lo, hi, B, S, h, 0, i, j)
                    assert sc[h, row0 + i, j] == pytest.approx(want, rel=1e-12, abs=1e-12)
                    if i < nb - 1:          # both blocks full: the reading is the mean over the sampled cells
                        assert want == pytest.approx(cell_mean, rel=1e-12, abs=1e-12)
                    elif cell_mean is None:   # no sampled cell is valid: the routing term is 0
                        assert want == 0.0
                    elif abs(want - cell_mean) > 1e-6:
                        differs += 1
        row0 += nb
    assert differs > 0          # on the partial blocks it is a reading, not an identity
    # a class without valid tokens is pooled to zeros
    if S >= 4:
        assert not qb[:, 2, 3:].any() and not kb[:, 2, 3:].any()


def test_empty_list_gives_empty_sums():
    # a row without any listed block (the selection never emits one; caller-made lists may):
    # the sums over an empty key set, out = 0 and lse = log 0 = -inf
    q, k, v = rng_qkv(19, 12, 2, 1, 4)
    counts = np.array([[1, 0, 3], [0, 2, 0]], np.int32)
    idx = np.full((2, 3, 3), -1, np.int32)
    idx[0, 0, :1] = [0]
    idx[0, 2, :3] = [0, 1, 2]
    idx[1, 1, :2] = [0, 1]
    out, lse = so.sparse_attention(q, k, v, [0, 12], 4, counts, idx, 0.5)
    for h, r in [(0, 1), (1, 0), (1, 2)]:
        assert not out[r * 4:(r + 1) * 4, h].any() and np.isneginf(lse[h, r * 4:(r + 1) * 4]).all()
    for h, r in [(0, 0), (0, 2), (1, 1)]:
        assert np.isfinite(lse[h, r * 4:(r + 1) * 4]).all()


def test_token_level_metric_ranks_like_exact_contribution():
    # Appendix (rank-equivalent scoring): with B = 1, beta = 1, the 1/sqrt(d) routing scale and all
    # ||V_j|| >= 1 (clamp inactive), the top-k of the metric row equals the top-k of the exact
    # P_ij ||V_j||_2 of dense causal softmax attention, for every row and every k.
    N, d = 24, 16
    q, k, v = rng_qkv(5, N, 1, 1, d)
    v = v / np.linalg.norm(v, axis=2, keepdims=True) * np.random.default_rng(6).uniform(1.0, 6.0, (N, 1, 1))
    cu = [0, N]
    qb, kb, mv = so.pool_blocks(q, k, v, cu, 1)
    sc = so.oam_scores(qb, kb, mv, cu, 1, beta=1.0, route_scale=d ** -0.5)
    logits = (q[:, 0] @ k[:, 0].T) / math.sqrt(d)
    logits = np.where(np.tril(np.ones((N, N), bool)), logits, -np.inf)
    P = np.exp(logits - logits.max(axis=1, keepdims=True))
    P /= P.sum(axis=1, keepdims=True)
    contrib = P * np.linalg.norm(v[:, 0], axis=1)[None, :]
    for kk in (1, 3, 7):
        budget = np.full(N, kk, dtype=np.int32)
        counts, idx = so.select_blocks(sc, budget, cu, 1, n_sink=0, n_local=0)
        for i in range(N):
            want = sorted(np.argsort(-contrib[i, :i + 1], kind="stable")[:min(kk, i + 1)].tolist())
            assert idx[0, i, :counts[0, i]].tolist() == want


# ------------------------------------------------------------------------------------------------
# stage 2: schedule
# ------------------------------------------------------------------------------------------------

def test_schedule_endpoints_and_monotone():
    # catches: 0-based index inside Eq. 3, decay towards the wrong end, floor vs round,
    # binary rounding of mu eating an integer end point
    mu = PAPER["mu"]["value"]
    for n, ks in [(64, 12), (256, 25), (1024, 51), (1024, 102.4), (100, 10), (37, 20)]:
        ks_all = [so.tpd_k(i, n, ks, mu) for i in range(n)]
        assert ks_all[-1] == math.floor(mu * ks + 1e-9)            # k_end = mu * k_start
        assert ks_all[0] == math.floor(ks - ks * (1 - mu) / n + 1e-9)
        assert all(a >= b for a, b in zip(ks_all, ks_all[1:]))
        assert max(ks_all) <= ks
        # linear: never further than one block from the real-valued line
        for i, kk in enumerate(ks_all):
            line = ks - ks * (1 - mu) * (i + 1) / n
            assert line - 1 < kk <= line + 1e-6
    assert so.tpd_k(99, 100, 10, 0.7) == 7                         # not 6
    assert [so.tpd_k(i, 4, 8, 0.5) for i in range(4)] == [7, 6, 5, 4]   # hand-computed
    assert [so.tpd_k(i, 5, 3, 1.0) for i in range(5)] == [3] * 5        # mu = 1: uniform


def test_budget_windows_minimum_and_causal_clamp():
    # paper preset at 128K: k_start = 0.1 N_blk, 4 + 4 forced blocks, at least 54 blocks in total
    n = 1024
    ks = PAPER["k_start_ratio_over_16k"]["value"] * n
    b = so.tpd_budget(n, ks, PAPER["mu"]["value"], PAPER["min_total_budget_blocks"]["value"],
                      PAPER["initial_window_blocks"]["value"], PAPER["local_window_blocks"]["value"])
    assert b[0] == 1 and b[10] == 11 and b[53] == 54             # causal clamp: k_eff <= i + 1
    assert b.min() == 1 and b[200:].min() >= 54                   # minimum budget holds once causal allows
    assert b[-1] == max(54, math.floor(0.7 * ks + 1e-9)) == 71
    assert b.max() <= math.floor(ks)
    # at 64K the schedule (0.1 * 512 = 51.2 decaying to 35) sits below the 54-block minimum throughout
    b64 = so.tpd_budget(512, 0.1 * 512, 0.7, 54, 4, 4)
    assert set(b64[53:].tolist()) == {54} and b64[:54].tolist() == list(range(1, 55))
    # forced windows alone set the floor when the schedule asks for less
    b2 = so.tpd_budget(32, 2, 0.7, 0, 3, 2)
    assert b2.tolist()[:6] == [1, 2, 3, 4, 5, 5] and set(b2[5:].tolist()) == {5}
    assert so.forced_blocks(0, 2, 1) == [0]
    assert so.forced_blocks(1, 2, 1) == [0, 1]
    assert so.forced_blocks(7, 2, 1) == [0, 1, 7]
    assert so.forced_blocks(7, 2, 3) == [0, 1, 5, 6, 7]
    assert so.forced_blocks(2, 4, 4) == [0, 1, 2]
    assert so.forced_blocks(5, 0, 0) == []


def test_cost_closed_forms():
    # Eq. 2: sum_i min(i, k) = N k - k^2/2 (+ k/2 exactly); Eq. 4 for the decay schedule; both "~"
    mu = PAPER["mu"]["value"]
    for n, k in [(1024, 51), (512, 66), (256, 25), (4096, 300)]:
        uni = int(so.tpd_budget(n, k, 1.0, 0, 0, 0).sum())
        assert uni == n * k - k * (k - 1) // 2                       # exact
        assert abs(uni - (n * k - 0.5 * k * k)) <= k                 # Eq. 2
        dec = int(so.tpd_budget(n, k, mu, 0, 0, 0).sum())
        eq4 = n * k - 0.5 * k * k - 0.5 * k * (1 - mu) * (n - k)
        assert abs(dec - eq4) <= max(n, 0.2 * k * k)                 # Eq. 4
        assert dec < uni
        # equal-cost uniform budget is about (1 + mu)/2 = 0.85 of k_start (Ablation Studies)
        best = min(range(1, k + 1),
                   key=lambda ku: (abs(int(so.tpd_budget(n, ku, 1.0, 0, 0, 0).sum()) - dec), ku))
        assert best / k == pytest.approx(PAPER["k_uni_over_k_start"]["value"], abs=0.05)


def test_packed_budget_restarts_per_sequence():
    cu, B = [0, 256, 1280], 64
    b = so.packed_budget(cu, B, [3, 6], 0.7, 0, 1, 1)
    assert b[:4].tolist() == so.tpd_budget(4, 3, 0.7, 0, 1, 1).tolist()
    assert b[4:].tolist() == so.tpd_budget(16, 6, 0.7, 0, 1, 1).tolist()
    assert b[4] == 1 and len(b) == 20


# ------------------------------------------------------------------------------------------------
# stage 2: selection
# ------------------------------------------------------------------------------------------------

def best_subset(scores_row, free, need):
    """The size-`need` subset of `free` with the largest score sum (unique for distinct scores)."""
    best, best_sum = None, -np.inf
    for comb in itertools.combinations(free, need):
        s = sum(scores_row[j] for j in comb)
        if s > best_sum:
            best, best_sum = comb, s
    return list(best) if best is not None else []


def test_selection_is_the_max_sum_subset_plus_forced():
    # catches: ascending instead of descending rank, forced blocks counted twice or outside the
    # budget, acausal picks, unsorted output, wrong count
    r = np.random.default_rng(7)
    n, Hq = 9, 3
    sc = r.standard_normal((Hq, n, n))
    sc = np.where(np.tril(np.ones((n, n), bool))[None], sc, -np.inf)
    for n_sink, n_local, budget in [(1, 1, 4), (2, 2, 5), (0, 1, 3), (2, 1, 2), (0, 0, 3)]:
        bud = np.full(n, budget, dtype=np.int32)
        counts, idx = so.select_blocks(sc, bud, [0, n * 4], 4, n_sink, n_local)
        for h in range(Hq):
            for i in range(n):
                forced = so.forced_blocks(i, n_sink, n_local)
                k = min(i + 1, max(budget, len(forced)))
                got = idx[h, i, :counts[h, i]].tolist()
                assert counts[h, i] == k and got == sorted(set(got))
                assert all(0 <= j <= i for j in got) and set(forced) <= set(got)
                assert (idx[h, i, counts[h, i]:] == -1).all()
                free = [j for j in range(i + 1) if j not in forced]
                want = sorted(forced + best_subset(sc[h, i], free, k - len(forced)))
                assert got == want


def test_selection_ties_prefer_lower_index_and_permutation_equivariance():
    n = 8
    sc = np.full((1, n, n), -np.inf)
    for i in range(n):
        sc[0, i, :i + 1] = 1.0                                   # all equal
    sc[0, 7, 5] = 2.0
    counts, idx = so.select_blocks(sc, np.full(n, 4, np.int32), [0, n], 1, n_sink=1, n_local=1)
    assert idx[0, 6, :4].tolist() == [0, 1, 2, 6]                # forced 0 and 6, then lowest ties
    assert idx[0, 7, :4].tolist() == [0, 1, 5, 7]                # the 2.0, then the lowest tie
    # permuting the free key blocks of a row permutes its selection
    r = np.random.default_rng(8)
    row = r.standard_normal(n)
    sc2 = np.full((1, n, n), -np.inf)
    sc2[0, 7] = row
    perm = np.array([0, 4, 2, 6, 1, 5, 3, 7])                    # fixes forced blocks 0 and 7
    sc3 = sc2.copy()
    sc3[0, 7] = row[perm]                                        # new[j] = old[perm[j]]
    bud = np.zeros(n, np.int32)
    bud[7] = 5
    for i in range(7):                                           # only row 7 matters here
        sc2[0, i, :i + 1] = 0.0
        sc3[0, i, :i + 1] = 0.0
    _, a = so.select_blocks(sc2, bud, [0, n], 1, 1, 1, kmax=5)
    _, b = so.select_blocks(sc3, bud, [0, n], 1, 1, 1, kmax=5)
    assert sorted(perm[b[0, 7]].tolist()) == a[0, 7].tolist()


# ------------------------------------------------------------------------------------------------
# stage 3
# ------------------------------------------------------------------------------------------------

def dense_masked_attention(q, k, v, cu, allowed, scale):
    """Textbook softmax attention with an explicit token-level boolean mask `allowed[h]` [T,T]
    (already causal and sequence-local); GQA map written out."""
    T, Hq, d = q.shape
    G = Hq // k.shape[1]
    out = np.zeros((T, Hq, d))
    lse = np.zeros((Hq, T))
    for h in range(Hq):
        logits = scale * (q[:, h] @ k[:, h // G].T)
        logits = np.where(allowed[h], logits, -np.inf)
        for t in range(T):
            w = np.exp(logits[t] - logits[t].max())
            out[t, h] = (w / w.sum()) @ v[:, h // G]
            lse[h, t] = math.log(np.exp(logits[t]).sum())
    return out, lse


def token_mask_from_lists(cu, B, Hq, counts, idx):
    T = cu[-1]
    allowed = np.zeros((Hq, T, T), bool)
    for lo, hi, nb, row0 in so.sequence_table(cu, B):
        for i in range(nb):
            for h in range(Hq):
                for j in idx[h, row0 + i, :counts[h, row0 + i]]:
                    for t in range(lo + i * B, min(lo + (i + 1) * B, hi)):
                        for u in range(lo + j * B, min(lo + (j + 1) * B, hi)):
                            if u <= t:
                                allowed[h, t, u] = True
    return allowed


def full_budget_lists(cu, B, Hq):
    R, nbmax = so.total_rows(cu, B)
    counts = np.zeros((Hq, R), np.int32)
    idx = np.full((Hq, R, nbmax), -1, np.int32)
    for _, _, nb, row0 in so.sequence_table(cu, B):
        for i in range(nb):
            counts[:, row0 + i] = i + 1
            idx[:, row0 + i, :i + 1] = np.arange(i + 1)
    return counts, idx


def test_group_scores_brute_force_and_invariants():
    """The group reduction written out with loops; G = 1 is the identity; reordering the heads of
    a group changes nothing; max >= mean; the shared list is the per-head list when the heads of a
    group carry equal scores."""
    r = np.random.default_rng(11)
    Hq, Hkv, R, NB = 6, 2, 5, 5
    G = Hq // Hkv
    sc = r.normal(size=(Hq, R, NB))
    sc[:, np.triu_indices(R, 1)[0], np.triu_indices(R, 1)[1]] = -np.inf
    for how in ("max", "mean"):
        got = so.group_scores(sc, Hkv, how)
        assert got.shape == (Hkv, R, NB)
        for g in range(Hkv):
            for i in range(R):
                for j in range(NB):
                    vals = [sc[g * G + x, i, j] for x in range(G)]
                    want = max(vals) if how == "max" else sum(vals) / G
                    assert got[g, i, j] == want or abs(got[g, i, j] - want) < 1e-15
        assert np.array_equal(so.group_scores(sc, Hq, how), sc)
        perm = np.concatenate([r.permutation(G), G + r.permutation(G)])
        assert np.allclose(so.group_scores(sc[perm], Hkv, how), got, atol=1e-15)
    fin = np.isfinite(sc[0])
    assert (so.group_scores(sc, Hkv, "max")[:, fin] >= so.group_scores(sc, Hkv, "mean")[:, fin]).all()
    same = np.repeat(sc[::G], G, axis=0)                     # every head of a group equal to its first
    budget = np.array([1, 2, 2, 3, 3], dtype=np.int32)
    c1, i1 = so.select_blocks(same, budget, [0, R * 4], 4, 1, 1)
    c2, i2 = so.select_blocks(so.group_scores(same, Hkv, "max"), budget, [0, R * 4], 4, 1, 1)
    assert np.array_equal(c1[::G], c2) and np.array_equal(i1[::G], i2)
    with pytest.raises(ValueError):
        so.group_scores(sc, 4, "max")


def test_full_budget_equals_dense_causal_attention():
    # catches: missing intra-block causal mask, wrong GQA map, cross-sequence leakage, missing scale,
    # softmax over the wrong axis; ragged tails included
    B, Hq, Hkv, d = 4, 4, 2, 8
    cu = [0, 10, 23]
    q, k, v = rng_qkv(9, 23, Hq, Hkv, d)
    counts, idx = full_budget_lists(cu, B, Hq)
    out, lse = so.sparse_attention(q, k, v, cu, B, counts, idx, d ** -0.5)
    seq = np.zeros(23, int)
    seq[10:] = 1
    causal = (np.arange(23)[None, :] <= np.arange(23)[:, None]) & (seq[None, :] == seq[:, None])
    want, want_lse = dense_masked_attention(q, k, v, cu, np.broadcast_to(causal, (Hq, 23, 23)), d ** -0.5)
    assert np.abs(out - want).max() < 1e-12
    assert np.abs(lse - want_lse).max() < 1e-12
    # first token of each sequence attends to itself only
    assert np.allclose(out[0], v[0].repeat(2, axis=0)) and np.allclose(out[10], v[10].repeat(2, axis=0))
    # no leakage: changing sequence 0's keys/values leaves sequence 1 untouched
    k2, v2 = k.copy(), v.copy()
    k2[:10] += 1.0
    v2[:10] -= 2.0
    out2, _ = so.sparse_attention(q, k2, v2, cu, B, counts, idx, d ** -0.5)
    assert np.array_equal(out2[10:], out[10:])


def test_sparse_lists_equal_dense_attention_with_block_mask():
    B, Hq, Hkv, d = 4, 2, 1, 8
    cu = [0, 30]
    q, k, v = rng_qkv(10, 30, Hq, Hkv, d)
    qb, kb, mv = so.pool_blocks(q, k, v, cu, B)
    sc = so.oam_scores(qb, kb, mv, cu, B)
    bud = so.packed_budget(cu, B, [4], 0.7, 0, 1, 1)
    counts, idx = so.select_blocks(sc, bud, cu, B, 1, 1)
    assert counts.max() < 8                                       # really sparse
    out, lse = so.sparse_attention(q, k, v, cu, B, counts, idx, 0.3)
    allowed = token_mask_from_lists(cu, B, Hq, counts, idx)
    want, want_lse = dense_masked_attention(q, k, v, cu, allowed, 0.3)
    assert np.abs(out - want).max() < 1e-12 and np.abs(lse - want_lse).max() < 1e-12
    # subset request fills only what was asked for
    part, _ = so.sparse_attention(q, k, v, cu, B, counts, idx, 0.3, heads=[1], rows=[2, 7])
    assert np.array_equal(part[8:12, 1], out[8:12, 1]) and np.array_equal(part[28:30, 1], out[28:30, 1])
    assert np.isnan(part[:, 0]).all() and np.isnan(part[0:8, 1]).all()


def test_softmax_invariants():
    B, Hq, Hkv, d = 8, 2, 2, 4
    cu = [0, 64]
    q, k, v = rng_qkv(11, 64, Hq, Hkv, d)
    r = np.random.default_rng(12)
    counts = np.zeros((Hq, 8), np.int32)
    idx = np.full((Hq, 8, 8), -1, np.int32)
    for h in range(Hq):
        for i in range(8):
            pick = sorted(set(r.choice(i + 1, size=min(3, i + 1), replace=False).tolist()) | {i})
            counts[h, i] = len(pick)
            idx[h, i, :len(pick)] = pick
    # constant values: every convex combination returns the constant, whatever was selected
    vc = np.broadcast_to(r.standard_normal((1, Hkv, d)), (64, Hkv, d)).copy()
    out, _ = so.sparse_attention(q, k, vc, cu, B, counts, idx, 0.5)
    assert np.allclose(out, vc, atol=1e-12)
    # outputs stay inside the per-coordinate range of the visible values
    out, _ = so.sparse_attention(q, k, v, cu, B, counts, idx, 0.5)
    assert (out.max(axis=0) <= v.max(axis=0) + 1e-12).all()
    # shift invariance of softmax: adding a constant vector c to all keys adds <q,c> to every logit
    shift = r.standard_normal((1, Hkv, d))
    out_s, lse_s = so.sparse_attention(q, k + shift, v, cu, B, counts, idx, 0.5)
    assert np.allclose(out_s, out, atol=1e-10)


# ------------------------------------------------------------------------------------------------
# the benchmark configurations' budgets
# ------------------------------------------------------------------------------------------------

def _density(w, ks):
    total = int(so.packed_budget(w.cu_seqlens, w.block_size, ks, w.mu, w.k_min, w.n_sink, w.n_local).sum())
    return total, total / w.admissible_blocks


def test_benchmark_budgets_are_the_smallest_reaching_their_density():
    from paper_2603_06274_amd import workloads as wl
    expect_blocks = {"tiny_4k": 562, "llama8b_32k": 5028, "llama8b_128k": 42638}
    for w in wl.BENCHMARK_CONFIGS.values():
        total, dens = _density(w, w.k_start_blocks)
        assert dens >= w.target_density
        if w.name in expect_blocks:
            assert total == expect_blocks[w.name]
        if w.mu == 1.0:
            assert dens == 1.0
            continue
        if len(w.seq_lens) == 1:
            _, below = _density(w, [w.k_start_blocks[0] - 1])
            assert below < w.target_density
        else:
            # one ratio rho = k_start / n_blocks on a 1/1024 grid for all sequences
            nb = w.blocks_per_seq
            forced = w.n_sink + w.n_local
            def ks_for(rho1024):
                return [max(forced, round(rho1024 * n / 1024)) for n in nb]
            rho = next(x for x in range(1, 1025) if _density(w, ks_for(x))[1] >= w.target_density)
            assert tuple(ks_for(rho)) == w.k_start_blocks
