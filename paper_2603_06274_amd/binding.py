"""Thin ctypes binding of libstem_hip.so: argument marshalling only.

Function names and argument order follow include/stem.h.  torch tensors are used for device
memory and for the current stream; every step of the path runs inside the library's HIP kernels.
There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence, Tuple

import torch

# STEM_HIP_LIBRARY overrides the in-tree build (to try another build of the same ABI).
_LIB_PATH = os.environ.get("STEM_HIP_LIBRARY") or os.path.join(
    os.path.dirname(os.path.abspath(__file__)), "libstem_hip.so")
_lib = None

STEM_OK = 0
STEM_ERR_INVALID_ARG = -1
STEM_ERR_UNSUPPORTED = -2
STEM_ERR_WORKSPACE = -3
STEM_ERR_HIP = -4


class StemError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, stem_strerror(status), status))


class stem_shape(ctypes.Structure):
    _fields_ = [
        ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("block_size", ctypes.c_int32), ("batch", ctypes.c_int32),
        ("host_cu_seqlens", ctypes.POINTER(ctypes.c_int32)),
        ("q_stride_token", ctypes.c_int64), ("q_stride_head", ctypes.c_int64),
        ("kv_stride_token", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
        ("host_chunk_start", ctypes.POINTER(ctypes.c_int32)),
        ("host_chunk_end", ctypes.POINTER(ctypes.c_int32)),
    ]


def library_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Load the library (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libstem_hip.so is not built: run `python -m paper_2603_06274_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, f32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float, ctypes.c_size_t
        shp = ctypes.POINTER(stem_shape)
        L.stem_version.restype = ctypes.c_int
        L.stem_version.argtypes = []
        L.stem_strerror.restype = ctypes.c_char_p
        L.stem_strerror.argtypes = [ctypes.c_int]
        sigs = {
            "stem_rows": [shp, ctypes.POINTER(i32), ctypes.POINTER(i32)],
            "stem_workspace_bytes": [shp, i32, ctypes.POINTER(sz)],
            "stem_workspace_layout": [shp, i32, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)],
            "stem_budget_schedule": [shp, ctypes.POINTER(ctypes.c_double), ctypes.c_double, i32, i32, i32,
                                     ctypes.POINTER(i32), ctypes.POINTER(i32)],
            "stem_pool": [shp, vp, vp, vp, i32, vp, sz, vp],
            "stem_block_scores": [shp, vp, sz, i32, f32, f32, i32, vp, vp],
            "stem_estimate": [shp, vp, vp, vp, f32, f32, i32, i32, vp, vp, sz, vp],
            "stem_estimate_static": [shp, vp, vp, vp, f32, f32, i32, vp, vp],
            "stem_group_scores": [shp, vp, i32, vp, vp],
            "stem_estimate_select": [shp, vp, vp, vp, f32, f32, i32, vp, i32, i32, vp, vp, i32, vp, vp, sz, vp],
            "stem_select": [shp, vp, vp, i32, i32, i32, vp, vp, i32, vp],
            "stem_sparse_attn": [shp, vp, vp, vp, vp, vp, i32, i32, f32, vp, vp, vp],
        }
        for name, args in sigs.items():
            fn = getattr(L, name)
            fn.restype = ctypes.c_int
            fn.argtypes = args
        _lib = L
    return _lib


EXPORTED = ["stem_version", "stem_strerror", "stem_rows", "stem_workspace_bytes",
            "stem_workspace_layout", "stem_budget_schedule", "stem_pool", "stem_block_scores",
            "stem_group_scores", "stem_estimate_select",
            "stem_estimate", "stem_estimate_static", "stem_select", "stem_sparse_attn"]


def _check(status: int, where: str) -> None:
    if status != STEM_OK:
        raise StemError(status, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


class Shape:
    """Owns the ctypes stem_shape and the host arrays it points to.  chunk = (starts, ends): per
    sequence, the query positions of a chunked call (None: whole sequences)."""

    def __init__(self, num_q_heads: int, num_kv_heads: int, head_dim: int, block_size: int,
                 cu_seqlens: Sequence[int], q_strides: Tuple[int, int], kv_strides: Tuple[int, int],
                 chunk: Optional[Tuple[Sequence[int], Sequence[int]]] = None):
        i32p = ctypes.POINTER(ctypes.c_int32)
        self._cu = (ctypes.c_int32 * len(cu_seqlens))(*[int(x) for x in cu_seqlens])
        batch = len(cu_seqlens) - 1
        if chunk is not None:
            assert len(chunk[0]) == batch and len(chunk[1]) == batch
            self._cs = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in chunk[0]])
            self._ce = (ctypes.c_int32 * max(batch, 1))(*[int(x) for x in chunk[1]])
            cs, ce = ctypes.cast(self._cs, i32p), ctypes.cast(self._ce, i32p)
        else:
            cs, ce = i32p(), i32p()
        self.c = stem_shape(num_q_heads, num_kv_heads, head_dim, block_size, batch,
                            ctypes.cast(self._cu, i32p),
                            q_strides[0], q_strides[1], kv_strides[0], kv_strides[1], cs, ce)
        self.cu_seqlens = [int(x) for x in cu_seqlens]
        self.chunk = None if chunk is None else ([int(x) for x in chunk[0]], [int(x) for x in chunk[1]])

    @classmethod
    def from_tensors(cls, q: torch.Tensor, k: torch.Tensor, block_size: int, cu_seqlens: Sequence[int],
                     chunk: Optional[Tuple[Sequence[int], Sequence[int]]] = None):
        """q [T,Hq,d], k [Tk,Hkv,d] (any token/head strides, last dim contiguous)."""
        assert q.dim() == 3 and k.dim() == 3 and q.stride(2) == 1 and k.stride(2) == 1
        return cls(q.shape[1], k.shape[1], q.shape[2], block_size, cu_seqlens,
                   (q.stride(0), q.stride(1)), (k.stride(0), k.stride(1)), chunk)

    def ref(self):
        return ctypes.byref(self.c)


def stem_version() -> int:
    return lib().stem_version()


def stem_strerror(status: int) -> str:
    return lib().stem_strerror(status).decode()


def stem_rows(shape: Shape) -> Tuple[int, int]:
    r, nb = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().stem_rows(shape.ref(), ctypes.byref(r), ctypes.byref(nb)), "stem_rows")
    return r.value, nb.value


def stem_workspace_bytes(shape: Shape, ad_stride: int = 1) -> int:
    n = ctypes.c_size_t()
    _check(lib().stem_workspace_bytes(shape.ref(), int(ad_stride), ctypes.byref(n)), "stem_workspace_bytes")
    return n.value


def stem_workspace_layout(shape: Shape, ad_stride: int = 1) -> Tuple[int, int, int]:
    a, b, c = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().stem_workspace_layout(shape.ref(), int(ad_stride), ctypes.byref(a), ctypes.byref(b),
                                       ctypes.byref(c)), "stem_workspace_layout")
    return a.value, b.value, c.value


def stem_budget_schedule(shape: Shape, k_start_blocks: Sequence[float], mu: float, k_min: int,
                         n_sink: int, n_local: int) -> Tuple[torch.Tensor, int]:
    """Returns (budget int32 CPU tensor [R], kmax)."""
    rows, _ = stem_rows(shape)
    ks = (ctypes.c_double * len(k_start_blocks))(*[float(x) for x in k_start_blocks])
    out = torch.zeros(max(rows, 1), dtype=torch.int32)
    kmax = ctypes.c_int32()
    _check(lib().stem_budget_schedule(shape.ref(), ks, float(mu), int(k_min), int(n_sink), int(n_local),
                                      ctypes.cast(out.data_ptr(), ctypes.POINTER(ctypes.c_int32)),
                                      ctypes.byref(kmax)), "stem_budget_schedule")
    return out[:rows], kmax.value


def stem_pool(shape: Shape, q, k, v, ad_stride: int, workspace: torch.Tensor) -> None:
    _check(lib().stem_pool(shape.ref(), _ptr(q), _ptr(k), _ptr(v), int(ad_stride), _ptr(workspace),
                           workspace.numel() * workspace.element_size(), _stream()), "stem_pool")


def stem_block_scores(shape: Shape, workspace: torch.Tensor, ad_stride: int, beta: float,
                      route_scale: float, scores: torch.Tensor, fill_non_causal: bool = True) -> None:
    _check(lib().stem_block_scores(shape.ref(), _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), int(ad_stride),
                                   float(beta), float(route_scale), int(bool(fill_non_causal)), _ptr(scores),
                                   _stream()), "stem_block_scores")


def stem_estimate(shape: Shape, q, k, v, beta: float, route_scale: float, ad_stride: int,
                  scores: torch.Tensor, workspace: torch.Tensor, fill_non_causal: bool = True) -> None:
    _check(lib().stem_estimate(shape.ref(), _ptr(q), _ptr(k), _ptr(v), float(beta), float(route_scale),
                               int(ad_stride), int(bool(fill_non_causal)), _ptr(scores), _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _stream()), "stem_estimate")


STEM_STATIC_WORKSPACE_BYTES = 32 << 20


def stem_estimate_static(shape: Shape, q, k, v, beta: float, route_scale: float, ad_stride: int,
                         scores: torch.Tensor) -> None:
    """stem_estimate on the library's own per-GPU array: no workspace argument, no allocation."""
    _check(lib().stem_estimate_static(shape.ref(), _ptr(q), _ptr(k), _ptr(v), float(beta), float(route_scale),
                                      int(ad_stride), _ptr(scores), _stream()), "stem_estimate_static")


STEM_GROUP_MAX, STEM_GROUP_MEAN = 0, 1


def stem_estimate_select(shape: Shape, q, k, v, beta: float, route_scale: float, ad_stride: int,
                         budget: torch.Tensor, n_sink: int, n_local: int, counts: torch.Tensor,
                         indices: torch.Tensor, kmax: int, debug_scores: Optional[torch.Tensor],
                         workspace: torch.Tensor) -> None:
    _check(lib().stem_estimate_select(shape.ref(), _ptr(q), _ptr(k), _ptr(v), float(beta), float(route_scale),
                                      int(ad_stride), _ptr(budget), int(n_sink), int(n_local), _ptr(counts),
                                      _ptr(indices), int(kmax), _ptr(debug_scores), _ptr(workspace),
                                      workspace.numel() * workspace.element_size(), _stream()),
           "stem_estimate_select")


def stem_group_scores(shape: Shape, scores: torch.Tensor, reduce: int, group_scores: torch.Tensor) -> None:
    _check(lib().stem_group_scores(shape.ref(), _ptr(scores), int(reduce), _ptr(group_scores), _stream()),
           "stem_group_scores")


def stem_select(shape: Shape, scores: torch.Tensor, budget: torch.Tensor, n_sink: int, n_local: int,
                counts: torch.Tensor, indices: torch.Tensor, kmax: int,
                lists_per_kv_head: bool = False) -> None:
    _check(lib().stem_select(shape.ref(), _ptr(scores), _ptr(budget), int(n_sink), int(n_local),
                             int(bool(lists_per_kv_head)), _ptr(counts), _ptr(indices), int(kmax), _stream()),
           "stem_select")


def stem_sparse_attn(shape: Shape, q, k, v, counts: torch.Tensor, indices: torch.Tensor, kmax: int,
                     softmax_scale: float, out: torch.Tensor, lse: Optional[torch.Tensor],
                     lists_per_kv_head: bool = False) -> None:
    _check(lib().stem_sparse_attn(shape.ref(), _ptr(q), _ptr(k), _ptr(v), _ptr(counts), _ptr(indices),
                                  int(kmax), int(bool(lists_per_kv_head)), float(softmax_scale), _ptr(out),
                                  _ptr(lse), _stream()), "stem_sparse_attn")
