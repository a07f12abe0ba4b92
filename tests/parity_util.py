"""Helpers shared by the GPU parity tests: run the HIP path and the CPU oracle on the same seeded
tensors and compare them to the stated bars.

Bars (the benchmark spec):
  block scores   |gpu - oracle| <= 1e-4 * max(|oracle|, rms of the oracle row)
  index lists    bit-exact, except rows whose differing entries all sit within 1e-5 (relative) of the
                 oracle's selection threshold; those rows are counted and printed
  output         max-abs 1.5e-2 and relative L2 5e-3 against the fp64 oracle.  The max-abs bar is taken
                 as stated on every entry; an entry beyond it passes only if a rounding the prescribed
                 arithmetic makes can by itself exceed the bar there, and then only within that bound:
                 bf16 storage of the output (half an ulp <= 2^-8 |o|, beyond 1.5e-2 once |o| > 3.84) and
                 the bf16 probabilities of the second matrix product (<= 2^-8 D, D the mean absolute
                 deviation of the attended values, which reaches 3-6 on value rows scaled x4).  Such
                 entries are counted and printed.  The comparison is repeated after rounding the oracle
                 to bf16 and reported (max-abs, ulps, share of identical entries).
  lse            5e-3 absolute where the row sum is taken over the bf16-rounded probabilities (each
                 within 2^-8 relative of the fp32 one), which is what the library header promises
"""
from __future__ import annotations

import numpy as np
import torch

from oracle import stem_oracle as so
from paper_2603_06274_amd import workloads as wl
from paper_2603_06274_amd.prefill import StemPrefill

SCORE_RTOL = 1e-4
TIE_RTOL = 1e-5
OUT_MAX_ABS = 1.5e-2
OUT_REL_L2 = 5e-3


def host_arrays(data):
    """bf16 tensors widened exactly to fp32 numpy (the oracle widens further to fp64)."""
    return tuple(data[x].float().numpy() for x in "qkv")


def device_prefill(w: wl.Workload, data, want_lse=True, ad_stride=1) -> StemPrefill:
    dev = torch.device("cuda:0")
    q, k, v = (data[x].to(dev) for x in "qkv")
    return StemPrefill(q, k, v, w.cu_seqlens, w.block_size, w.k_start_blocks, w.mu, w.k_min, w.n_sink,
                       w.n_local, w.beta, w.route_scale, w.softmax_scale, want_lse=want_lse,
                       ad_stride=ad_stride, fill_scores=True)


def oracle_estimate(w: wl.Workload, qkv, ad_stride=1):
    """q_bar [Hq,R,S,d], k_bar [Hkv,R,S,d], m_v [Hkv,R], scores [Hq,R,NBmax] (fp64)."""
    q, k, v = qkv
    q_bar, k_bar, m_v = so.pool_blocks(q, k, v, w.cu_seqlens, w.block_size, ad_stride)
    scores = so.oam_scores(q_bar, k_bar, m_v, w.cu_seqlens, w.block_size, w.beta, w.route_scale)
    return q_bar, k_bar, m_v, scores


def oracle_select(w: wl.Workload, scores):
    budget = so.packed_budget(w.cu_seqlens, w.block_size, w.k_start_blocks, w.mu, w.k_min, w.n_sink,
                              w.n_local)
    counts, indices = so.select_blocks(scores, budget, w.cu_seqlens, w.block_size, w.n_sink, w.n_local)
    return budget, counts, indices


def check_pooled(pf: StemPrefill, q_bar, k_bar, m_v):
    gq, gk, gm = (t.cpu().double().numpy() for t in pf.pooled())
    assert np.abs(gq - q_bar).max() <= 2e-6 * max(1.0, np.abs(q_bar).max())
    assert np.abs(gk - k_bar).max() <= 2e-6 * max(1.0, np.abs(k_bar).max())
    fin = np.isfinite(m_v)
    assert np.array_equal(np.isfinite(gm), fin)
    assert np.abs(gm[fin] - m_v[fin]).max() <= 2e-6 * max(1.0, np.abs(m_v[fin]).max())


def check_scores(gpu_scores: np.ndarray, scores: np.ndarray):
    """gpu_scores fp32 [Hq,R,NB] as numpy, scores fp64 oracle.  -inf pattern must match exactly."""
    fin = np.isfinite(scores)
    assert np.array_equal(np.isfinite(gpu_scores), fin), "causal -inf pattern differs"
    assert (gpu_scores[~fin] == -np.inf).all()
    safe = np.where(fin, scores, 0.0)
    rms = np.sqrt((safe * safe).sum(axis=2, keepdims=True) / np.maximum(fin.sum(axis=2, keepdims=True), 1))
    tol = SCORE_RTOL * np.maximum(np.abs(safe), rms)
    err = np.abs(np.where(fin, gpu_scores.astype(np.float64), 0.0) - safe)
    worst = float((err / np.maximum(tol, 1e-300)).max())
    assert worst <= 1.0, "score error %.3g x tolerance" % worst
    return float(err.max())


def check_lists(w: wl.Workload, g_counts, g_idx, o_counts, o_idx, o_scores, log=print):
    """Exact equality of the lists except logged near-ties.  Returns a bool mask [Hq,R] of rows
    whose lists are identical."""
    assert np.array_equal(g_counts, o_counts), "counts differ"
    Hq, R = o_counts.shape
    same = np.ones((Hq, R), bool)
    kk = min(g_idx.shape[2], o_idx.shape[2])
    assert (g_idx[:, :, kk:] == -1).all() and (o_idx[:, :, kk:] == -1).all()
    diff_rows = np.argwhere((g_idx[:, :, :kk] != o_idx[:, :, :kk]).any(axis=2))
    near = 0
    for h, r in diff_rows:
        c = o_counts[h, r]
        a, b = set(g_idx[h, r, :c].tolist()), set(o_idx[h, r, :c].tolist())
        assert len(a) == c, "GPU list has repeats or padding inside the count"
        only_g, only_o = sorted(a - b), sorted(b - a)
        assert len(only_g) == len(only_o)
        # the oracle's threshold: the lowest score it kept among the blocks in dispute
        row = o_scores[h, r]
        tau = min(row[j] for j in only_o)
        for j in only_g + only_o:
            assert 0 <= j and np.isfinite(row[j]), "GPU picked a non-causal block"
            gap = abs(row[j] - tau)
            assert gap <= TIE_RTOL * max(abs(row[j]), abs(tau)), \
                "head %d row %d: block %d differs and is no near-tie (gap %.3g)" % (h, r, j, gap)
        same[h, r] = False
        near += 1
        log("near-tie: %s head %d row %d gpu-only %s oracle-only %s (threshold %.9g)"
            % (w.name, h, r, only_g, only_o, tau))
    # lists that agree as sets must agree in order too (ascending)
    for h, r in diff_rows:
        if same[h, r]:
            raise AssertionError("lists differ in order only")
    log("%s: %d of %d rows differ by near-ties" % (w.name, near, Hq * R))
    return same


OUT_EXACT_BAR_LIMIT = 3.84      # above this half a bf16 ulp alone can exceed OUT_MAX_ABS
LSE_ABS = 5e-3
ROUNDING_SLACK = 5e-4           # fp32 accumulation and second-order terms on top of the two rounding bounds


class ListedKeys:
    """What an output entry was computed from, so that the worst case of the second product's
    operand rounding can be evaluated for it: the probabilities enter the bf16 matrix instruction
    rounded to bf16 (relative error <= 2^-8 each, row sum taken from the rounded values), which moves
    out[t, h, c] by at most 2^-8 * D with D = sum_u p_u |V[u, c] - out[t, h, c]| (the mean absolute
    deviation of the attended values).  counts / indices are per query head."""

    def __init__(self, qkv, cu_seqlens, block_size, counts, indices, scale, q_token_of=None):
        self.q, self.k, self.v = qkv
        self.tab = so.sequence_table(cu_seqlens, block_size)
        self.B, self.counts, self.indices, self.scale = block_size, counts, indices, scale
        self.G = self.q.shape[1] // self.k.shape[1]

    def spread(self, t: int, h: int, want_out: np.ndarray) -> np.ndarray:
        """D[c] for all columns of out[t, h]; want_out is the oracle's out[t, h] (cross-checked)."""
        lo, hi, nb, row0 = next(x for x in self.tab if x[0] <= t < x[1])
        i = (t - lo) // self.B
        blocks = self.indices[h, row0 + i, :self.counts[h, row0 + i]]
        key_tok = np.concatenate([np.arange(lo + j * self.B, min(lo + (j + 1) * self.B, hi)) for j in blocks])
        key_tok = key_tok[key_tok <= t]
        g = h // self.G
        s = self.scale * (self.k[key_tok, g].astype(np.float64) @ self.q[t, h].astype(np.float64))
        p = np.exp(s - s.max())
        p /= p.sum()
        vv = self.v[key_tok, g].astype(np.float64)
        out = p @ vv
        assert np.abs(out - want_out).max() <= 1e-9 * max(1.0, np.abs(out).max())
        return p @ np.abs(vv - out[None, :])


def check_output(g_out, o_out: np.ndarray, what="", log=None, keys: ListedKeys = None):
    """g_out: the GPU output [T,Hq,d] (torch tensor, any device) ; o_out: the oracle's fp64 array of the
    same shape, NaN where the oracle was not asked to compute (those entries are skipped).

    Returns (max_abs, rel_l2) against the fp64 oracle; the other figures go to `log`."""
    sel = ~np.isnan(o_out[..., 0])
    assert sel.any()
    g = g_out.detach().cpu()[torch.from_numpy(sel)].double().numpy()
    return check_output_arrays(g, o_out[sel], np.argwhere(sel), what, log, keys)


def check_output_arrays(g: np.ndarray, o: np.ndarray, where: np.ndarray, what="", log=None,
                        keys: ListedKeys = None):
    """The output bars on two fp64 arrays [n, d]: g from the GPU (bf16 values), o the oracle;
    where[n] = (token, head) of each row.

    1. |g - o| <= 1.5e-2 as stated, on every entry, except where a rounding that the arithmetic
       prescribes (bf16 storage of the output, bf16 probabilities as matrix operands) can by itself
       exceed the bar: an entry beyond 1.5e-2 must have |o| > 3.84 or a value spread D with
       2^-8 (|o| + D) > 1.5e-2, and must then stay within 2^-8 (|o| + D) + ROUNDING_SLACK.  D needs
       `keys`; without it only the storage rounding above 3.84 is allowed.  The entries that needed
       the allowance are counted and printed.
    2. relative L2 <= 5e-3.
    3. The same after rounding the oracle to bf16 (what a perfect kernel would store): reported as
       max-abs, as ulps where |o| >= 2 and as the share of identical entries; an entry that met the
       bar in 1 lies within 1.5e-2 plus half an ulp of the rounded oracle."""
    assert not np.isnan(g).any(), "NaN in GPU output"
    d = np.abs(g - o)
    small = np.abs(o) <= OUT_EXACT_BAR_LIMIT
    max_abs = float(d.max())
    max_abs_small = float(d[small].max()) if small.any() else 0.0
    rel_l2 = float(np.sqrt((d * d).sum() / max((o * o).sum(), 1e-300)))
    over = np.argwhere(d > OUT_MAX_ABS)
    excused, worst_excess = 0, 0.0
    spread_cache = {}
    for n, c in over:
        storage = np.abs(o[n, c]) * 2.0 ** -8
        bound = storage if np.abs(o[n, c]) > OUT_EXACT_BAR_LIMIT else 0.0
        if d[n, c] > max(OUT_MAX_ABS, bound + ROUNDING_SLACK):
            assert keys is not None, "%s: entry %s col %d off by %.4g (oracle %.4g)" % (what, where[n], c, d[n, c], o[n, c])
            t, h = int(where[n][0]), int(where[n][1])
            if (t, h) not in spread_cache:
                spread_cache[(t, h)] = keys.spread(t, h, o[n])
            bound = storage + spread_cache[(t, h)][c] * 2.0 ** -8
            assert bound > OUT_MAX_ABS and d[n, c] <= bound + ROUNDING_SLACK, \
                "%s: token %d head %d col %d off by %.4g, oracle %.4g, rounding bound %.4g" % (what, t, h, c, d[n, c], o[n, c], bound)
        excused += 1
        worst_excess = max(worst_excess, float(d[n, c] - OUT_MAX_ABS))
    # the same after rounding the oracle to the output's storage type
    o_bf = torch.from_numpy(o).to(torch.bfloat16).double().numpy()
    d_bf = np.abs(g - o_bf)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(o_bf), 2.0 ** -126))) - 7)
    met = d <= OUT_MAX_ABS
    max_abs_bf = float(d_bf.max())
    max_ulps = float((d_bf / ulp)[np.abs(o_bf) >= 2.0].max()) if (np.abs(o_bf) >= 2.0).any() else 0.0
    rel_l2_bf = float(np.sqrt((d_bf * d_bf).sum() / max((o_bf * o_bf).sum(), 1e-300)))
    msg = ("%s output vs fp64 oracle: max-abs %.4g (%.4g where |o| <= %.2f), rel-L2 %.4g; %d of %d entries beyond "
           "%.3g, all within their rounding bound (worst excess %.4g); vs bf16-rounded oracle: max-abs %.4g, "
           "at most %.1f ulp where |o| >= 2, %.2f %% of entries identical, rel-L2 %.4g"
           % (what, max_abs, max_abs_small, OUT_EXACT_BAR_LIMIT, rel_l2, excused, d.size, OUT_MAX_ABS, worst_excess,
              max_abs_bf, max_ulps, 100.0 * float((d_bf == 0).mean()), rel_l2_bf))
    (log or print)(msg)
    assert (d_bf[met] <= OUT_MAX_ABS + 0.5 * ulp[met]).all(), msg
    assert rel_l2 <= OUT_REL_L2 and rel_l2_bf <= OUT_REL_L2, msg
    return max_abs, rel_l2


def check_lse(g_lse, o_lse: np.ndarray, what=""):
    """g_lse: GPU lse [Hq,T] (torch tensor); o_lse: oracle fp64, NaN where not computed; -inf must
    match exactly (a query with no visible key)."""
    m = ~np.isnan(o_lse)
    g = g_lse.detach().cpu().double().numpy()[m]
    o = o_lse[m]
    inf = np.isneginf(o)
    assert np.array_equal(np.isneginf(g), inf), "%s: -inf pattern of lse differs" % what
    err = float(np.abs(g[~inf] - o[~inf]).max()) if (~inf).any() else 0.0
    assert err <= LSE_ABS, "%s lse error %.4g" % (what, err)
    return err


def stratified_pairs(w: wl.Workload, random_per_head: int, seed: int):
    """(head, global query-block row) pairs to check at full size: for EVERY head and every packed
    sequence the first two rows, the rows around the end of the causal ramp (where the budget stops
    being clamped by causality), the last two rows, plus random rows per head.  The fixed rows hold
    both row parities, so with two XCDs per KV head (which take alternate rows) every head is seen
    on both of its XCDs; with one XCD per KV head every head means every XCD."""
    r = np.random.default_rng(seed)
    pairs = []
    total = w.total_rows
    for h in range(w.num_q_heads):
        rows = set()
        row0 = 0
        for s, nb in enumerate(w.blocks_per_seq):
            ks = int(w.k_start_blocks[s])
            for i in (0, 1, ks - 1, ks, ks + 1, nb - 2, nb - 1):
                if 0 <= i < nb:
                    rows.add(row0 + i)
            row0 += nb
        rows.update(int(x) for x in r.choice(total, size=min(random_per_head, total), replace=False))
        pairs += [(h, x) for x in sorted(rows)]
    return pairs


def oracle_attention_pairs(w: wl.Workload, qkv, counts, indices, pairs):
    """Oracle stage 3 for (head, global row) pairs, one by one.  Returns a list of
    (head, row, first token, one past the last token, out [n,d] fp64, lse [n] fp64)."""
    q, k, v = qkv
    G = w.num_q_heads // w.num_kv_heads
    tab = so.sequence_table(w.cu_seqlens, w.block_size)
    res = []
    for h, r in pairs:
        lo, hi, nb, row0 = next(t for t in tab if t[3] <= r < t[3] + t[2])
        i = r - row0
        o, l = so.sparse_attention_row(q, k, v, lo, hi, w.block_size, i, h, h // G,
                                       indices[h, r, :counts[h, r]], w.softmax_scale)
        t0 = lo + i * w.block_size
        res.append((h, r, t0, t0 + o.shape[0], o, l))
    return res
