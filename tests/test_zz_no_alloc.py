"""stem_estimate_static, the stage-1 entry point for callers that cannot allocate: through the C ABI,
against stem_estimate (the entry point it is a variant of) and against the CPU oracle, on two calls
in a row, the second with a smaller input, so that what the first call left in the library's
per-GPU array must not show in the second."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2603_06274_amd import binding as sb
from paper_2603_06274_amd import workloads as wl

import parity_util as pu

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def test_static_workspace_estimate_matches_the_workspace_one_on_two_calls_in_a_row():
    dev = torch.device("cuda:0")
    L = sb.lib()
    first = wl.small("static_first", seed=81, num_q_heads=8, num_kv_heads=2, seq_lens=(3000, 1111),
                     block_size=128, k_start=(5, 3), outliers=(3, 2))
    second = wl.small("static_second", seed=82, num_q_heads=4, num_kv_heads=2, seq_lens=(700,),
                      block_size=64, k_start=(3,), outliers=(2,))
    for w, S in ((first, 1), (second, 2)):
        say("case", w.name, "seed", w.seed, "T", w.total_tokens, "ad_stride", S, "entry stem_estimate_static")
        data = wl.generate(w)
        qkv = pu.host_arrays(data)
        q, k, v = (data[x].to(dev) for x in "qkv")
        shape = sb.Shape.from_tensors(q, k, w.block_size, w.cu_seqlens)
        R, nbmax = sb.stem_rows(shape)
        # the existing entry point, on a caller-provided workspace
        ws = torch.empty(sb.stem_workspace_bytes(shape, S), dtype=torch.uint8, device=dev)
        want = torch.full((w.num_q_heads, R, nbmax), float("nan"), dtype=torch.float32, device=dev)
        sb.stem_estimate(shape, q, k, v, w.beta, w.route_scale, S, want, ws)
        # the new one: inputs and outputs only; it must not allocate, so none of torch's either
        got = torch.full_like(want, float("nan"))
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated(dev)
        status = L.stem_estimate_static(shape.ref(), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                        ctypes.c_float(w.beta), ctypes.c_float(w.route_scale), S,
                                        got.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert status == sb.STEM_OK, sb.stem_strerror(status)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated(dev) == before
        # same kernels on the same inputs: the same bits
        assert torch.equal(got.view(torch.int32), want.view(torch.int32))
        # and the stated bar against the oracle
        scores = pu.oracle_estimate(w, qkv, S)[3]
        err = pu.check_scores(got.cpu().numpy(), scores)
        say("%s: scores identical to stem_estimate; error against the oracle %.3g" % (w.name, err))


def test_static_workspace_estimate_refuses_what_does_not_fit():
    dev = torch.device("cuda:0")
    L = sb.lib()
    # 262144 tokens of 32/8 heads need 42 MB of pooled vectors: beyond the 32 MiB array
    big = sb.Shape(32, 8, 128, 128, [0, 262144], (32 * 128, 128), (8 * 128, 128))
    assert sb.stem_workspace_bytes(big, 1) > sb.STEM_STATIC_WORKSPACE_BYTES
    dummy = torch.zeros(64, dtype=torch.float32, device=dev)
    args = (dummy.data_ptr(), dummy.data_ptr(), dummy.data_ptr(), ctypes.c_float(0.2), ctypes.c_float(1.0))
    assert L.stem_estimate_static(big.ref(), *args, 1, dummy.data_ptr(), None) == sb.STEM_ERR_WORKSPACE
    # a chunked shape: the pooled keys of earlier chunks would have to survive in the shared array
    chunked = sb.Shape(4, 2, 128, 128, [0, 1024], (4 * 128, 128), (2 * 128, 128), chunk=([512], [1024]))
    assert L.stem_estimate_static(chunked.ref(), *args, 1, dummy.data_ptr(), None) == sb.STEM_ERR_UNSUPPORTED
    ok = sb.Shape(4, 2, 128, 128, [0, 1024], (4 * 128, 128), (2 * 128, 128))
    assert L.stem_estimate_static(ok.ref(), *args, 3, dummy.data_ptr(), None) == sb.STEM_ERR_INVALID_ARG
