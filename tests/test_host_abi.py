"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol,
does its shape bookkeeping and the Eq. 3 schedule on the host, and rejects bad arguments before
anything could be launched."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import stem_oracle as so
from paper_2603_06274_amd import binding as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def make_shape(cu, Hq=4, Hkv=2, d=128, B=64):
    return sb.Shape(Hq, Hkv, d, B, cu, (Hq * d, d), (Hkv * d, d))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "stem.h")).read()
    declared = set(re.findall(r"^\s*(?:int|const char\*)\s+(stem_\w+)\s*\(", header, flags=re.M))
    assert declared == set(sb.EXPORTED)
    L = ctypes.CDLL(sb.library_path())
    for name in declared:
        assert hasattr(L, name), name
    assert sb.stem_version() >= 100
    assert sb.stem_strerror(0) == "ok" and "workspace" in sb.stem_strerror(sb.STEM_ERR_WORKSPACE)


def test_rows_and_workspace():
    shape = make_shape([0, 100, 100, 740], B=64)
    assert sb.stem_rows(shape) == (2 + 0 + 10, 10)
    assert sb.stem_rows(shape) == so.total_rows([0, 100, 100, 740], 64)
    for S in (1, 2, 4, 8, 16):
        q_off, k_off, m_off = sb.stem_workspace_layout(shape, S)
        total = sb.stem_workspace_bytes(shape, S)
        assert k_off == 0 and m_off >= 2 * 12 * S * 128 * 4 and q_off >= m_off + 2 * 12 * 4
        assert total >= q_off + 4 * 12 * S * 128 * 4 and q_off % 256 == 0 and m_off % 256 == 0
        for d in (64, 256):                            # the pooled parts scale with the head size
            other = make_shape(shape.cu_seqlens, d=d)
            q_d, k_d, m_d = sb.stem_workspace_layout(other, S)
            assert k_d == 0 and m_d >= 2 * 12 * S * d * 4 and q_d >= m_d + 2 * 12 * 4
            assert sb.stem_workspace_bytes(other, S) >= q_d + 4 * 12 * S * d * 4
    n = ctypes.c_size_t()
    L = sb.lib()
    for S, want in ((0, sb.STEM_ERR_INVALID_ARG), (-2, sb.STEM_ERR_INVALID_ARG), (3, sb.STEM_ERR_INVALID_ARG),
                    (32, sb.STEM_ERR_UNSUPPORTED), (64, sb.STEM_ERR_UNSUPPORTED), (128, sb.STEM_ERR_INVALID_ARG)):
        assert L.stem_workspace_bytes(shape.ref(), S, ctypes.byref(n)) == want, S


@pytest.mark.parametrize("cu,B,ks,mu,k_min,n_sink,n_local", [
    ([0, 4096], 64, [12], 0.7, 0, 2, 1),
    ([0, 32768], 128, [25], 0.7, 0, 2, 2),
    ([0, 131072], 128, [51], 0.7, 0, 2, 2),
    ([0, 131072], 128, [102.4], 0.7, 54, 4, 4),
    ([0, 65536], 128, [51.2], 0.7, 54, 4, 4),
    ([0, 8192, 24576, 57344, 131072], 128, [4, 8, 16, 36], 0.7, 0, 2, 2),
    ([0, 65536], 128, [512], 1.0, 0, 2, 2),
    ([0, 65536], 128, [28], 1.0, 0, 2, 2),
    ([0, 100, 100, 777], 64, [3, 1, 5.5], 0.5, 2, 0, 0),
    ([0, 6400], 64, [10], 0.7, 0, 1, 3),
    ([0, 6400], 64, [0], 0.3, 0, 5, 7),
])
def test_budget_schedule_matches_oracle(cu, B, ks, mu, k_min, n_sink, n_local):
    shape = make_shape(cu, B=B)
    got, kmax = sb.stem_budget_schedule(shape, ks, mu, k_min, n_sink, n_local)
    want = so.packed_budget(cu, B, ks, mu, k_min, n_sink, n_local)
    assert got.numpy().tolist() == want.tolist()
    assert kmax == (int(want.max()) if len(want) else 0)


def test_budget_schedule_random_sweep():
    r = np.random.default_rng(0)
    for _ in range(200):
        n = int(r.integers(1, 400))
        ks = float(r.integers(0, 2 * n)) * (1.0 if r.random() < 0.5 else 0.1)
        mu = float(r.choice([0.5, 0.6, 0.7, 0.8, 0.9, 1.0]))
        k_min, n_sink, n_local = int(r.integers(0, 10)), int(r.integers(0, 6)), int(r.integers(0, 6))
        shape = make_shape([0, n * 64 - int(r.integers(0, 64))], B=64)
        got, _ = sb.stem_budget_schedule(shape, [ks], mu, k_min, n_sink, n_local)
        assert got.numpy().tolist() == so.tpd_budget(n, ks, mu, k_min, n_sink, n_local).tolist()


def test_chunked_shapes_rows_and_schedule():
    """A chunked call covers some query blocks of each sequence; rows keep their index in the
    sequence, so its budget is the matching slice of the whole-sequence schedule."""
    cu, B = [0, 1536, 2236], 128
    whole = make_shape(cu, B=B)
    assert sb.stem_rows(whole) == (12 + 6, 12)
    chunk = sb.Shape(4, 2, 128, B, cu, (4 * 128, 128), (2 * 128, 128), chunk=([512, 256], [1024, 700]))
    assert sb.stem_rows(chunk) == (4 + 4, 8)
    tail = sb.Shape(4, 2, 128, B, cu, (4 * 128, 128), (2 * 128, 128), chunk=([1024, 700], [1536, 700]))
    assert sb.stem_rows(tail) == (4, 12)
    ks, mu, k_min, n_sink, n_local = [7.5, 4], 0.7, 3, 1, 2
    full, _ = sb.stem_budget_schedule(whole, ks, mu, k_min, n_sink, n_local)
    want = so.packed_budget(cu, B, ks, mu, k_min, n_sink, n_local)
    assert full.numpy().tolist() == want.tolist()
    got, kmax = sb.stem_budget_schedule(chunk, ks, mu, k_min, n_sink, n_local)
    assert got.numpy().tolist() == want[4:8].tolist() + want[12 + 2:12 + 6].tolist()
    assert kmax == max(got.numpy().tolist())
    got, _ = sb.stem_budget_schedule(tail, ks, mu, k_min, n_sink, n_local)
    assert got.numpy().tolist() == want[8:12].tolist()
    # the key parts of the workspace do not move with the chunk
    assert sb.stem_workspace_layout(chunk, 2)[1:] == sb.stem_workspace_layout(whole, 2)[1:]
    n = ctypes.c_size_t()
    L = sb.lib()
    for starts, ends in (([100, 0], [1024, 700]), ([0, 0], [1000, 700]), ([512, 256], [256, 700]),
                         ([0, 0], [1536, 800]), ([-128, 0], [1536, 700])):
        bad = sb.Shape(4, 2, 128, B, cu, (4 * 128, 128), (2 * 128, 128), chunk=(starts, ends))
        assert L.stem_workspace_bytes(bad.ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG, (starts, ends)
    half = sb.Shape(4, 2, 128, B, cu, (4 * 128, 128), (2 * 128, 128), chunk=([0, 0], [1536, 700]))
    half.c.host_chunk_end = ctypes.POINTER(ctypes.c_int32)()
    assert L.stem_workspace_bytes(half.ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG


def test_bad_arguments_are_rejected_on_the_host():
    L = sb.lib()
    good = make_shape([0, 640])
    n = ctypes.c_size_t()
    # shape errors
    assert L.stem_workspace_bytes(make_shape([0, 640], Hq=3, Hkv=2).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_workspace_bytes(make_shape([0, 640], d=96).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_UNSUPPORTED
    assert L.stem_workspace_bytes(make_shape([0, 640], d=512).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_UNSUPPORTED
    assert L.stem_workspace_bytes(make_shape([0, 640], d=0).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    narrow = sb.Shape(4, 2, 256, 64, [0, 640], (4 * 128, 128), (2 * 128, 128))     # rows narrower than a head
    assert L.stem_workspace_bytes(narrow.ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_workspace_bytes(make_shape([0, 640], B=32).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_UNSUPPORTED
    assert L.stem_workspace_bytes(make_shape([0, 640, 600]).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_workspace_bytes(make_shape([1, 640]).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_workspace_bytes(make_shape(list(range(0, 66 * 64, 64))).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_workspace_bytes(make_shape([0, 64 * 5000]).ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_UNSUPPORTED
    bad_stride = sb.Shape(4, 2, 128, 64, [0, 640], (4 * 128 + 4, 128), (2 * 128, 128))
    assert L.stem_workspace_bytes(bad_stride.ref(), 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_workspace_bytes(None, 1, ctypes.byref(n)) == sb.STEM_ERR_INVALID_ARG
    # null / misaligned device pointers, short workspace: refused before any launch
    assert L.stem_pool(good.ref(), None, None, None, 1, None, 0, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_pool(good.ref(), 0x1000, 0x1000, 0x1008, 1, 0x1000, 1 << 30, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_pool(good.ref(), 0x1000, 0x1000, 0x1000, 1, 0x1000, 16, None) == sb.STEM_ERR_WORKSPACE
    assert L.stem_pool(good.ref(), 0x1000, 0x1000, 0x1000, 5, 0x1000, 1 << 30, None) == sb.STEM_ERR_INVALID_ARG
    # a workspace sized for block means is too small for four partial means per block
    small_ws = sb.stem_workspace_bytes(good, 1)
    assert L.stem_pool(good.ref(), 0x1000, 0x1000, 0x1000, 4, 0x1000, small_ws, None) == sb.STEM_ERR_WORKSPACE
    assert L.stem_estimate(good.ref(), 0x1000, 0x1000, 0x1000, 0.2, 1.0, 32, 1, 0x1000, 0x1000, 1 << 30, None) == sb.STEM_ERR_UNSUPPORTED
    assert L.stem_estimate(good.ref(), 0x1000, 0x1000, 0x1000, 0.2, 1.0, 0, 1, 0x1000, 0x1000, 1 << 30, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_estimate(good.ref(), 0x1000, 0x1000, 0x1000, 0.2, 1.0, 1, 2, 0x1000, 0x1000, 1 << 30, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_block_scores(good.ref(), 0x1000, 1 << 30, 1, float("nan"), 1.0, 1, 0x1000, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_block_scores(good.ref(), 0x1000, 1 << 30, 1, 0.2, 1.0, -1, 0x1000, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_select(good.ref(), 0x1000, 0x1000, 1, 1, 0, 0x1000, None, 8, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_select(good.ref(), 0x1000, 0x1000, -1, 1, 0, 0x1000, 0x1000, 8, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_select(good.ref(), 0x1000, 0x1000, 3, 3, 0, 0x1000, 0x1000, 4, None) == sb.STEM_ERR_INVALID_ARG
    # the diagonal is always kept: a local window of zero blocks is refused by both selection calls
    assert L.stem_select(good.ref(), 0x1000, 0x1000, 2, 0, 0, 0x1000, 0x1000, 8, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_estimate_select(good.ref(), 0x1000, 0x1000, 0x1000, 0.2, 1.0, 1, 0x1000, 2, 0, 0x1000, 0x1000, 8,
                                  None, 0x1000, 1 << 30, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_select(good.ref(), 0x1000, 0x1000, 1, 1, 2, 0x1000, 0x1000, 8, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_group_scores(good.ref(), 0x1000, 7, 0x1000, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_group_scores(good.ref(), None, 0, 0x1000, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_sparse_attn(good.ref(), 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0, 0, 0.1, 0x1000, None, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_sparse_attn(good.ref(), 0x1000, 0x1000, 0x1000, None, 0x1000, 4, 0, 0.1, 0x1000, None, None) == sb.STEM_ERR_INVALID_ARG
    assert L.stem_sparse_attn(good.ref(), 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 4, 0, -1.0, 0x1000, None, None) == sb.STEM_ERR_INVALID_ARG
    # one sequence of one KV head must stay below 2 GiB for the attention kernel's block addressing
    wide = sb.Shape(4, 2, 128, 64, [0, 4096], (4 * 128, 128), (1 << 19, 128))
    assert L.stem_sparse_attn(wide.ref(), 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 4, 0, 0.1, 0x1000, None, None) == sb.STEM_ERR_UNSUPPORTED
    wide64 = sb.Shape(4, 2, 64, 64, [0, 4096], (4 * 64, 64), (1 << 19, 64))       # the same for the other head sizes
    assert L.stem_sparse_attn(wide64.ref(), 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 4, 0, 0.1, 0x1000, None, None) == sb.STEM_ERR_UNSUPPORTED
    # an empty batch entry list is fine on the host and launches nothing
    empty = make_shape([0, 0])
    assert sb.stem_rows(empty) == (0, 0)
    assert L.stem_pool(empty.ref(), 0x1000, 0x1000, 0x1000, 1, 0x1000, 1 << 20, None) == sb.STEM_OK
    assert L.stem_sparse_attn(empty.ref(), 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 4, 0, 0.1, 0x1000, None, None) == sb.STEM_OK
    with pytest.raises(sb.StemError):
        sb.stem_rows(make_shape([0, 640], d=96))
