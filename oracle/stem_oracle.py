"""CPU oracle for the Stem prefill hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the three stages compute, written from the paper and
sharing nothing with the HIP library (no code, headers, tables or helpers; neither imports the
other).  Only tests/, the smoke check and the benchmark's cpu_baseline leg may import it; the
product path never does.

What each function follows:
  pool_blocks        Algorithm 1, step 1 (block-wise representations Q-bar, K-bar, M-bar_V)
  oam_scores         Algorithm 1, step 3a and Eq. 7 (Output-Aware Metric on pooled blocks)
  tpd_budget         Eq. 3 (Token Position-Decay) in block units, Algorithm 1 step 3b, plus the
                     forced initial/local windows and minimum budget of Implementation Details
  select_blocks      Algorithm 1, step 3c (Top-k(i) of the metric row)
  group_scores       extension for grouped-query attention: the metric reduced over the query
                     heads of a KV head, so that one list serves the whole group
  sparse_attention   Algorithm 1, step 3d (exact softmax attention over the gathered blocks), with
                     the causal constraint j <= i of the Token Position-Decay analysis

Stages 1-2 are a heuristic (an approximation of attention mass followed by a top-k), so they are
written as the algorithm's steps in the paper's order.  Stage 3 reaches a result with a plain
definition (softmax attention restricted to a key set), so it is that definition written out.

Readings of points the paper leaves open (all also listed in the design notes):
  * Pool = per-block mean over the block's valid tokens, one d-vector per block: the only shape
    consistent with the 2 N^2 d / B^2 metric cost of Eq. 8 and with Q-bar_i K-bar^T in Algorithm 1.
    The general strided anti-diagonal sample (ad_stride = S) is kept as an option; S = 1 is the
    block mean.
  * log is the natural log (it inverts exp in Eq. 6); max(0, log 0) = 0.
  * The routing term carries `route_scale` (1.0 as printed in Eq. 7 / Algorithm 1; Eq. 6 has
    1/sqrt(d)).
  * The schedule runs on block indices of each packed sequence, 1-based inside Eq. 3, and the
    forced windows count inside the budget.  The floor of Eq. 3 is guarded by +1e-9.
  * Equal scores: the lower block index wins; lists are emitted ascending.
  * Softmax is normalised over the selected, causally unmasked keys.

Pins (tests/test_oracle_pins.py): every function here is pinned against brute force, closed forms or
a textbook definition; the paper prints no worked numerical example, so the end-to-end values are
otherwise unpinned.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np

NEG_INF = -np.inf


# ------------------------------------------------------------------------------------------------
# packed-sequence bookkeeping
# ------------------------------------------------------------------------------------------------

def sequence_table(cu_seqlens: Sequence[int], block_size: int) -> List[Tuple[int, int, int, int]]:
    """Per sequence: (first token, one-past-last token, number of blocks, first global row)."""
    table = []
    row = 0
    for s in range(len(cu_seqlens) - 1):
        lo, hi = int(cu_seqlens[s]), int(cu_seqlens[s + 1])
        nb = -(-(hi - lo) // block_size)
        table.append((lo, hi, nb, row))
        row += nb
    return table


def total_rows(cu_seqlens: Sequence[int], block_size: int) -> Tuple[int, int]:
    """(R, NBmax): query-block rows over all sequences, and the longest sequence in blocks."""
    tab = sequence_table(cu_seqlens, block_size)
    return sum(t[2] for t in tab), max([t[2] for t in tab], default=0)


# ------------------------------------------------------------------------------------------------
# stage 1: pooled representations and the Output-Aware Metric
# ------------------------------------------------------------------------------------------------

def pool_blocks(q: np.ndarray, k: np.ndarray, v: np.ndarray, cu_seqlens: Sequence[int],
                block_size: int, ad_stride: int = 1):
    """Algorithm 1 step 1.

    q [T,Hq,d], k, v [T,Hkv,d].  Returns
      q_bar [Hq,R,S,d], k_bar [Hkv,R,S,d]: for residue a < S, the mean of the block's valid token
        rows whose in-block position is congruent to a (mod S); with S = 1 the block mean,
      m_v [Hkv,R]: max over the block's valid tokens of ln ||V_t||_2  (-inf for an all-zero block).
    """
    S = int(ad_stride)
    if S < 1 or block_size % S:
        raise ValueError("ad_stride must divide the block size")
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    tab = sequence_table(cu_seqlens, block_size)
    R = sum(t[2] for t in tab)
    q_bar = np.zeros((Hq, R, S, d), dtype=np.float64)
    k_bar = np.zeros((Hkv, R, S, d), dtype=np.float64)
    m_v = np.full((Hkv, R), NEG_INF, dtype=np.float64)
    for lo, hi, nb, row0 in tab:
        for b in range(nb):
            t0 = lo + b * block_size
            t1 = min(t0 + block_size, hi)
            qb = q[t0:t1].astype(np.float64)          # [n,Hq,d]
            kb = k[t0:t1].astype(np.float64)
            vb = v[t0:t1].astype(np.float64)
            for a in range(S):
                if qb[a::S].shape[0]:
                    q_bar[:, row0 + b, a, :] = qb[a::S].mean(axis=0)
                    k_bar[:, row0 + b, a, :] = kb[a::S].mean(axis=0)
            norms = np.sqrt((vb * vb).sum(axis=2))    # [n,Hkv]
            with np.errstate(divide="ignore"):
                m_v[:, row0 + b] = np.log(norms).max(axis=0)
    return q_bar, k_bar, m_v


def oam_scores(q_bar: np.ndarray, k_bar: np.ndarray, m_v: np.ndarray, cu_seqlens: Sequence[int],
               block_size: int, beta: float = 0.2, route_scale: float = 1.0) -> np.ndarray:
    """Algorithm 1 step 3a / Eq. 7 on pooled blocks.

    scores[h, r, j] = route_scale * route(h, r, j) + beta * max(0, m_v[g(h), j])   for j <= i(r),
    -inf for j > i(r) or j beyond the row's sequence; j is local to the row's sequence and g(h) =
    h // (Hq/Hkv).  route is <q_bar, k_bar> for S = 1; for S > 1 it pairs residue a of the query
    block with residue S-1-a of the key block (the strided anti-diagonals) and averages over a.
    """
    Hq, R, S, d = q_bar.shape
    Hkv = k_bar.shape[0]
    G = Hq // Hkv
    tab = sequence_table(cu_seqlens, block_size)
    nbmax = max([t[2] for t in tab], default=0)
    scores = np.full((Hq, R, nbmax), NEG_INF, dtype=np.float64)
    magnitude = np.maximum(0.0, m_v)                  # max(0, -inf) = 0
    for _, _, nb, row0 in tab:
        for h in range(Hq):
            g = h // G
            qs = q_bar[h, row0:row0 + nb]             # [nb,S,d]
            ks = k_bar[g, row0:row0 + nb][:, ::-1, :]  # residue S-1-a against residue a
            route = (qs.reshape(nb, S * d) @ ks.reshape(nb, S * d).T) / S
            m = route_scale * route + beta * magnitude[g, row0:row0 + nb][None, :]
            causal = np.tril(np.ones((nb, nb), dtype=bool))
            scores[h, row0:row0 + nb, :nb] = np.where(causal, m, NEG_INF)
    return scores


# ------------------------------------------------------------------------------------------------
# stage 2: Token Position-Decay budget and selection
# ------------------------------------------------------------------------------------------------

def forced_blocks(i: int, n_sink: int, n_local: int) -> List[int]:
    """Always-kept key blocks of 0-based query block i: the first n_sink blocks and the last
    n_local causal blocks, diagonal included (Implementation Details).  Ascending, no repeats."""
    head = set(range(min(n_sink, i + 1)))
    tail = set(range(max(0, i - n_local + 1), i + 1))
    return sorted(head | tail)


FLOOR_GUARD = 1e-9


def tpd_k(i: int, n_blocks: int, k_start: float, mu: float) -> int:
    """Eq. 3 at block granularity: the budget of the (i+1)-th of n_blocks query blocks.

    The floor is taken after adding FLOOR_GUARD, so that a value which is an integer in decimal
    arithmetic (k_end = mu * k_start = 0.7 * 10) is not lost to the binary rounding of mu."""
    slope = (k_start * (1.0 - mu)) / n_blocks
    return int(math.floor(k_start - slope * (i + 1) + FLOOR_GUARD))


def tpd_budget(n_blocks: int, k_start: float, mu: float, k_min: int, n_sink: int,
               n_local: int) -> np.ndarray:
    """Effective per-row block budget of one sequence:
    k_eff(i) = min(i+1, max(k(i), k_min, |forced(i)|)) with k(i) from Eq. 3."""
    out = np.zeros(n_blocks, dtype=np.int32)
    for i in range(n_blocks):
        k = max(tpd_k(i, n_blocks, k_start, mu), int(k_min), len(forced_blocks(i, n_sink, n_local)))
        out[i] = min(i + 1, k)
    return out


def packed_budget(cu_seqlens: Sequence[int], block_size: int, k_start_blocks: Sequence[float],
                  mu: float, k_min: int, n_sink: int, n_local: int) -> np.ndarray:
    """tpd_budget per packed sequence, each restarting at its own first block; [R] int32."""
    parts = [tpd_budget(nb, k_start_blocks[s], mu, k_min, n_sink, n_local)
             for s, (_, _, nb, _) in enumerate(sequence_table(cu_seqlens, block_size))]
    return np.concatenate(parts) if parts else np.zeros(0, dtype=np.int32)


def select_blocks(scores: np.ndarray, budget: np.ndarray, cu_seqlens: Sequence[int],
                  block_size: int, n_sink: int, n_local: int, kmax: Optional[int] = None):
    """Algorithm 1 step 3c with the forced windows.

    For every head and row: the forced blocks, plus the best-scoring other causal blocks until the
    row holds k = min(i+1, max(budget[r], |forced|)) blocks; ties go to the lower block index.
    Returns counts [Hq,R] int32 and indices [Hq,R,kmax] int32, ascending, padded with -1.
    """
    Hq, R, _ = scores.shape
    tab = sequence_table(cu_seqlens, block_size)
    lists = [[None] * R for _ in range(Hq)]
    widest = 0
    for _, _, nb, row0 in tab:
        for i in range(nb):
            r = row0 + i
            forced = forced_blocks(i, n_sink, n_local)
            k = min(i + 1, max(int(budget[r]), len(forced)))
            free = np.setdiff1d(np.arange(i + 1), forced)      # ascending
            need = k - len(forced)
            for h in range(Hq):
                # descending score; the stable sort keeps ascending index among equal scores
                ranked = free[np.argsort(-scores[h, r, free], kind="stable")]
                chosen = sorted(forced + ranked[:need].tolist())
                lists[h][r] = chosen
                widest = max(widest, len(chosen))
    if kmax is None:
        kmax = widest
    if widest > kmax:
        raise ValueError("kmax too small for the budget")
    counts = np.zeros((Hq, R), dtype=np.int32)
    indices = np.full((Hq, R, kmax), -1, dtype=np.int32)
    for h in range(Hq):
        for r in range(R):
            c = lists[h][r]
            counts[h, r] = len(c)
            indices[h, r, :len(c)] = c
    return counts, indices


def group_scores(scores: np.ndarray, num_kv_heads: int, reduce: str = "max") -> np.ndarray:
    """Group-shared selection for grouped-query attention (an extension: the paper derives the
    method per head and names group sharing only for a comparison system in Related Work).

    scores [Hq,R,NB] -> [Hkv,R,NB]: the metric of KV head g for a block pair is the maximum
    ("max") or the mean ("mean") of the metric of its G = Hq/Hkv query heads h = g*G .. g*G+G-1.
    One list per (KV head, row) is then selected from it and used by all G heads.  Entries that
    are -inf (non-causal) for one head are -inf for all, and stay -inf.
    """
    Hq, R, NB = scores.shape
    G = Hq // num_kv_heads
    if G * num_kv_heads != Hq:
        raise ValueError("Hq must be a multiple of Hkv")
    grouped = scores.reshape(num_kv_heads, G, R, NB)
    if reduce == "max":
        return grouped.max(axis=1)
    if reduce == "mean":
        return grouped.sum(axis=1) / G
    raise ValueError("reduce must be 'max' or 'mean'")


# ------------------------------------------------------------------------------------------------
# stage 3: exact attention over the selected blocks
# ------------------------------------------------------------------------------------------------

def sparse_attention_row(q: np.ndarray, k: np.ndarray, v: np.ndarray, seq_lo: int, seq_hi: int,
                         block_size: int, i: int, head: int, kv_head: int,
                         blocks: Sequence[int], scale: float):
    """Algorithm 1 step 3d for one (head, query block i of the sequence [seq_lo, seq_hi)).

    out[t] = sum_u softmax_u(scale * <Q_t, K_u>) V_u over the tokens u of the listed key blocks
    with u <= t.  Returns (out [n,d] fp64, lse [n] fp64) for the block's n valid query tokens.
    A query with no visible key (possible only with an empty list, which the selection never
    emits) gets the empty sums: out = 0 and lse = log 0 = -inf.
    """
    t0 = seq_lo + i * block_size
    t1 = min(t0 + block_size, seq_hi)
    if len(blocks) == 0:
        return np.zeros((t1 - t0, q.shape[2])), np.full(t1 - t0, NEG_INF)
    key_tok = np.concatenate([
        np.arange(seq_lo + j * block_size, min(seq_lo + (j + 1) * block_size, seq_hi))
        for j in blocks])
    qt = q[t0:t1, head].astype(np.float64)            # [n,d]
    ks = k[key_tok, kv_head].astype(np.float64)       # [m,d]
    vs = v[key_tok, kv_head].astype(np.float64)
    s = scale * (qt @ ks.T)
    visible = key_tok[None, :] <= np.arange(t0, t1)[:, None]
    s = np.where(visible, s, NEG_INF)
    m = s.max(axis=1, keepdims=True)
    p = np.exp(s - m)
    z = p.sum(axis=1, keepdims=True)
    out = (p / z) @ vs
    lse = (m + np.log(z))[:, 0]
    return out, lse


def sparse_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, cu_seqlens: Sequence[int],
                     block_size: int, counts: np.ndarray, indices: np.ndarray, scale: float,
                     heads: Optional[Sequence[int]] = None, rows: Optional[Sequence[int]] = None):
    """Algorithm 1 step 3d for the requested heads and global rows (default: all).

    Returns out [T,Hq,d] fp64 and lse [Hq,T] fp64; entries of rows/heads not requested are NaN.
    """
    T, Hq, d = q.shape
    Hkv = k.shape[1]
    G = Hq // Hkv
    out = np.full((T, Hq, d), np.nan, dtype=np.float64)
    lse = np.full((Hq, T), np.nan, dtype=np.float64)
    wanted_rows = None if rows is None else set(int(r) for r in rows)
    head_list = range(Hq) if heads is None else heads
    for lo, hi, nb, row0 in sequence_table(cu_seqlens, block_size):
        for i in range(nb):
            r = row0 + i
            if wanted_rows is not None and r not in wanted_rows:
                continue
            t0 = lo + i * block_size
            t1 = min(t0 + block_size, hi)
            for h in head_list:
                blocks = indices[h, r, :counts[h, r]]
                o, l = sparse_attention_row(q, k, v, lo, hi, block_size, i, h, h // G, blocks, scale)
                out[t0:t1, h] = o
                lse[h, t0:t1] = l
    return out, lse


# ------------------------------------------------------------------------------------------------
# the whole path, as the benchmark's CPU baseline times it
# ------------------------------------------------------------------------------------------------

def stem_prefill(q, k, v, cu_seqlens, block_size, k_start_blocks, mu, k_min, n_sink, n_local,
                 beta, route_scale, scale, ad_stride=1, heads=None, rows=None):
    """Algorithm 1 end to end: pool -> metric -> budget -> top-k -> sparse attention."""
    q_bar, k_bar, m_v = pool_blocks(q, k, v, cu_seqlens, block_size, ad_stride)
    scores = oam_scores(q_bar, k_bar, m_v, cu_seqlens, block_size, beta, route_scale)
    budget = packed_budget(cu_seqlens, block_size, k_start_blocks, mu, k_min, n_sink, n_local)
    counts, indices = select_blocks(scores, budget, cu_seqlens, block_size, n_sink, n_local)
    out, lse = sparse_attention(q, k, v, cu_seqlens, block_size, counts, indices, scale, heads, rows)
    return dict(q_bar=q_bar, k_bar=k_bar, m_v=m_v, scores=scores, budget=budget, counts=counts,
                indices=indices, out=out, lse=lse)
