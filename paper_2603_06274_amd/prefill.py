"""Buffer plumbing around the C ABI: allocates the device buffers of one layer once and chains
stem_estimate -> stem_select -> stem_sparse_attn on the current stream.  No arithmetic here."""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as sb


class StemPrefill:
    """One attention layer's Stem pre-filling path on one GPU.

    q [T,Hq,d], k and v [Tk,Hkv,d]: bf16 CUDA tensors (k and v with equal strides).  With
    chunk = (starts, ends), q holds only the tokens of each sequence's chunk (T = their sum) while
    k and v keep all Tk = cu_seqlens[-1] rows; pass the same `workspace` to the calls of one
    prompt so that the pooled keys of earlier chunks are kept.
    """

    def __init__(self, q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, cu_seqlens: Sequence[int],
                 block_size: int, k_start_blocks: Sequence[float], mu: float = 0.7, k_min: int = 0,
                 n_sink: int = 4, n_local: int = 4, beta: float = 0.2, route_scale: float = 1.0,
                 softmax_scale: Optional[float] = None, want_lse: bool = False, ad_stride: int = 1,
                 chunk=None, workspace: Optional[torch.Tensor] = None, group_share: Optional[str] = None,
                 fill_scores: bool = False):
        if not (q.is_cuda and k.is_cuda and v.is_cuda):
            raise RuntimeError("StemPrefill needs device tensors; there is no CPU path")
        assert q.dtype == k.dtype == v.dtype == torch.bfloat16
        assert k.stride() == v.stride() and k.shape == v.shape
        self.q, self.k, self.v = q, k, v
        self.shape = sb.Shape.from_tensors(q, k, block_size, cu_seqlens, chunk)
        self.n_sink, self.n_local = int(n_sink), int(n_local)
        self.beta, self.route_scale = float(beta), float(route_scale)
        self.ad_stride = int(ad_stride)
        # False: the score kernel skips the tiles that hold no causal pair (the selection never reads
        # them); True: the whole [Hq, R, NBmax] rectangle is defined, -inf above the diagonal
        self.fill_scores = bool(fill_scores)
        # group_share "max" / "mean": one list per (KV head, row) from the group-reduced metric
        assert group_share in (None, "max", "mean")
        self.group_share = group_share
        self.softmax_scale = float(softmax_scale if softmax_scale is not None else q.shape[2] ** -0.5)
        self.rows, self.nbmax = sb.stem_rows(self.shape)
        budget_host, kmax = sb.stem_budget_schedule(self.shape, k_start_blocks, mu, k_min, n_sink, n_local)
        self.budget_host = budget_host
        self.kmax = max(kmax, 1)
        dev = q.device
        Hq, T = q.shape[1], q.shape[0]
        self.budget = budget_host.to(dev)
        need = sb.stem_workspace_bytes(self.shape, self.ad_stride)
        if workspace is not None:
            assert workspace.dtype == torch.uint8 and workspace.numel() >= need
        self.workspace = workspace if workspace is not None else torch.empty(need, dtype=torch.uint8, device=dev)
        self.scores = torch.empty((Hq, self.rows, self.nbmax), dtype=torch.float32, device=dev)
        Hl = k.shape[1] if group_share else Hq         # lists per row
        self.group_scores = (torch.empty((Hl, self.rows, self.nbmax), dtype=torch.float32, device=dev)
                             if group_share else None)
        self.counts = torch.empty((Hl, self.rows), dtype=torch.int32, device=dev)
        self.indices = torch.empty((Hl, self.rows, self.kmax), dtype=torch.int32, device=dev)
        self.out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=dev)  # O uses Q's strides
        self.lse = torch.empty((Hq, T), dtype=torch.float32, device=dev) if want_lse else None

    def estimate(self) -> None:
        sb.stem_estimate(self.shape, self.q, self.k, self.v, self.beta, self.route_scale,
                         self.ad_stride, self.scores, self.workspace, self.fill_scores)

    def pool(self) -> None:
        sb.stem_pool(self.shape, self.q, self.k, self.v, self.ad_stride, self.workspace)

    def block_scores(self) -> None:
        sb.stem_block_scores(self.shape, self.workspace, self.ad_stride, self.beta, self.route_scale,
                             self.scores, self.fill_scores)

    def select(self) -> None:
        if self.group_share:
            sb.stem_group_scores(self.shape, self.scores,
                                 sb.STEM_GROUP_MAX if self.group_share == "max" else sb.STEM_GROUP_MEAN,
                                 self.group_scores)
        sb.stem_select(self.shape, self.group_scores if self.group_share else self.scores, self.budget,
                       self.n_sink, self.n_local, self.counts, self.indices, self.kmax,
                       lists_per_kv_head=bool(self.group_share))

    def attend(self) -> None:
        sb.stem_sparse_attn(self.shape, self.q, self.k, self.v, self.counts, self.indices, self.kmax,
                            self.softmax_scale, self.out, self.lse, lists_per_kv_head=bool(self.group_share))

    def estimate_select(self, debug_scores: Optional[torch.Tensor] = None) -> None:
        """Stages 1-2 without the score tensor (per-head lists only)."""
        assert not self.group_share
        sb.stem_estimate_select(self.shape, self.q, self.k, self.v, self.beta, self.route_scale,
                                self.ad_stride, self.budget, self.n_sink, self.n_local, self.counts,
                                self.indices, self.kmax, debug_scores, self.workspace)

    def run(self, fused: bool = False) -> torch.Tensor:
        if fused:
            self.estimate_select()
        else:
            self.estimate()
            self.select()
        self.attend()
        return self.out

    def pooled(self):
        """Views of the pooled workspace: q_bar [Hq,R,S,d], k_bar [Hkv,Rk,S,d], m_v [Hkv,Rk] (fp32);
        Rk counts the blocks of all sequences."""
        S = self.ad_stride
        qo, ko, mo = sb.stem_workspace_layout(self.shape, S)
        Hq, Hkv, d, R = self.q.shape[1], self.k.shape[1], self.q.shape[2], self.rows
        B, cu = self.shape.c.block_size, self.shape.cu_seqlens
        Rk = sum(-(-(cu[s + 1] - cu[s]) // B) for s in range(len(cu) - 1))
        f = self.workspace
        q_bar = f[qo:qo + 4 * Hq * R * S * d].view(torch.float32).view(Hq, R, S, d)
        k_bar = f[ko:ko + 4 * Hkv * Rk * S * d].view(torch.float32).view(Hkv, Rk, S, d)
        m_v = f[mo:mo + 4 * Hkv * Rk].view(torch.float32).view(Hkv, Rk)
        return q_bar, k_bar, m_v
