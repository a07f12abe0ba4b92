#!/usr/bin/env python3
"""Benchmark of the Stem prefill hot path on one MI355X.

One step = stem_estimate -> stem_select -> stem_sparse_attn over one synthetic Llama-3-8B-shaped
attention layer at 128K tokens (32/8 GQA heads, head_dim 128, block 128, ~8 % block density), all
inputs resident in HBM.  Prints one JSON line.

  value      dense-equivalent TFLOP/s of the whole path: the FLOPs dense causal attention would
             spend on the layer (4 d B^2 A Hq) divided by the time of one step
  roofline   the sparse-attention kernel against the bf16 MFMA peak, from the FLOPs it really
             executes (4 d B^2 per listed block) and its duration measured with events on the
             launch stream
  cpu_baseline  the CPU oracle as it stands, timed on a bounded sample of the same layer and
             extrapolated by listed-block count (a reported baseline, not a target)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PAPER_H20_128K_DENSE_EQUIV_TFLOPS = 1.409e14 / 0.420 / 1e12   # dense-causal FLOPs of the layer / 420 ms

ATTN_SOURCE = os.path.join(ROOT, "paper_2603_06274_amd", "csrc", "stem_attn.hip")


def git_blob_sha1(path):
    """The hash git gives the file's content (what `git hash-object` prints)."""
    import hashlib
    data = open(path, "rb").read()
    return hashlib.sha1(b"blob %d\0" % len(data) + data).hexdigest()


def measured_attention_traffic(workload):
    """HBM-side bytes per sparse-attention launch as measured with rocprofv3 --pmc FETCH_SIZE and
    WRITE_SIZE runs of this script.  The figure lives beside the profile summary it comes from
    (profiles/sparse_attn_kernel_<workload>.md, a line `traffic_bytes_per_launch: <bytes> kernel_blob:
    <sha1>`), tagged with the git blob hash of the kernel source it was measured on; it is reported
    only while that hash is still the source's, otherwise null."""
    import re
    path = os.path.join(ROOT, "profiles", "sparse_attn_kernel_%s.md" % workload)
    current = git_blob_sha1(ATTN_SOURCE)
    info = {"profile": os.path.relpath(path, ROOT), "kernel_blob_now": current, "kernel_blob_measured": None}
    if not os.path.exists(path):
        return None, info
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)\s+kernel_blob:\s*([0-9a-f]{40})", open(path).read())
    if not m:
        return None, info
    info["kernel_blob_measured"] = m.group(2)
    return (float(m.group(1)) if m.group(2) == current else None), info


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def numpy_threads():
    """Threads of the BLAS behind numpy (the oracle's matrix products are its only parallel part)."""
    try:
        from threadpoolctl import threadpool_info
        blas = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
        if blas:
            return max(blas)
    except Exception:
        pass
    return 1


def cpu_baseline(w, data, dense_flops, gpu_counts, gpu_indices):
    """Times the oracle on KV group 0 (stages 1-2 in full, stage 3 on evenly spaced rows) and
    extrapolates to the layer."""
    import numpy as np
    from oracle import stem_oracle as so

    G = w.num_q_heads // w.num_kv_heads
    q = data["q"][:, :G].float().numpy()
    k = data["k"][:, :1].float().numpy()
    v = data["v"][:, :1].float().numpy()
    t0 = time.perf_counter()
    q_bar, k_bar, m_v = so.pool_blocks(q, k, v, w.cu_seqlens, w.block_size)
    scores = so.oam_scores(q_bar, k_bar, m_v, w.cu_seqlens, w.block_size, w.beta, w.route_scale)
    budget = so.packed_budget(w.cu_seqlens, w.block_size, w.k_start_blocks, w.mu, w.k_min, w.n_sink, w.n_local)
    counts, indices = so.select_blocks(scores, budget, w.cu_seqlens, w.block_size, w.n_sink, w.n_local)
    t12 = time.perf_counter() - t0
    n_rows = 512
    rows = [int(x) for x in np.linspace(0, w.total_rows - 1, n_rows)]
    t0 = time.perf_counter()
    so.sparse_attention(q, k, v, w.cu_seqlens, w.block_size, counts, indices, w.softmax_scale, rows=rows)
    t3 = time.perf_counter() - t0
    sampled_blocks = int(counts[:, rows].sum())
    group_blocks = int(counts.sum())
    t_layer = w.num_kv_heads * (t12 + t3 * group_blocks / max(sampled_blocks, 1))
    # rows of this KV group whose GPU list differs from the oracle's (near-ties of the fp32 metric)
    kk = min(indices.shape[2], gpu_indices.shape[2])
    differ = ((gpu_indices[:G, :, :kk] != indices[:, :, :kk]).any(axis=2) | (gpu_counts[:G] != counts))
    return {
        "value": round(dense_flops / t_layer / 1e12, 4), "unit": "TFLOP/s (dense-equivalent)",
        "cores": numpy_threads(), "host_cpu_count": os.cpu_count(), "kind": "oracle",
        "list_rows_differing_from_oracle": int(differ.sum()), "list_rows_compared": int(differ.size),
        "sample": "KV group 0 (%d of %d query heads): stages 1-2 in full (%.1f s), stage 3 on %d of %d "
                  "query-block rows (%.1f s, %d listed blocks); layer time extrapolated by listed-block "
                  "count to %.0f s" % (G, w.num_q_heads, t12, n_rows, w.total_rows, t3, sampled_blocks, t_layer),
        "extrapolated_layer_seconds": round(t_layer, 1),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_128k")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ad-stride", type=int, default=1, help="anti-diagonal stride of the estimate (1, 2, 4, 8, 16)")
    ap.add_argument("--fused", action="store_true", help="stages 1-2 through stem_estimate_select (no score tensor)")
    ap.add_argument("--group-share", choices=["max", "mean"], default=None,
                    help="one list per (KV head, row) from the group-reduced metric")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy, the known-size dispatch the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="after the timed steps, also time the vendor library's dense bf16 GEMM (16384^3, "
                         "torch.matmul) in the same process: what dense matrix work sustains on this box")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a one-GPU hot path (no collectives, no sharding); run with --gpus 1")

    import torch
    from paper_2603_06274_amd import binding, workloads
    from paper_2603_06274_amd.prefill import StemPrefill

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    binding.lib()
    w = {**workloads.BENCHMARK_CONFIGS, **workloads.EXTRA_CONFIGS}[args.workload]
    data = workloads.generate(w)
    dev = torch.device("cuda:0")
    if args.fused and args.group_share:
        sys.exit("bench.py: --fused gives per-head lists only")
    options = {"ad_stride": args.ad_stride, "fused": args.fused, "group_share": args.group_share}
    default_options = args.ad_stride == 1 and not args.fused and not args.group_share
    pf = StemPrefill(*(data[x].to(dev) for x in "qkv"), w.cu_seqlens, w.block_size, w.k_start_blocks, w.mu,
                     w.k_min, w.n_sink, w.n_local, w.beta, w.route_scale, w.softmax_scale,
                     ad_stride=args.ad_stride, group_share=args.group_share)

    d, B, Hq, Hkv, T, R = w.head_dim, w.block_size, w.num_q_heads, w.num_kv_heads, w.total_tokens, w.total_rows
    dense_flops = 4.0 * d * B * B * w.admissible_blocks * Hq

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        pf.run(fused=args.fused)
    torch.cuda.synchronize()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        ev[s][0].record()
        if args.fused:                                 # both stages in one call: booked under "estimate"
            pf.estimate_select()
            ev[s][1].record()
        else:
            pf.estimate()
            ev[s][1].record()
            pf.select()
        ev[s][2].record()
        pf.attend()
        ev[s][3].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    t_est = median([e[0].elapsed_time(e[1]) for e in ev])
    t_sel = median([e[1].elapsed_time(e[2]) for e in ev])
    attn_ms = [e[2].elapsed_time(e[3]) for e in ev]
    t_attn_avg = sum(attn_ms) / len(attn_ms)

    listed = int(pf.counts.sum().item())
    if args.group_share:                               # a list serves the G heads of its KV head
        listed *= Hq // Hkv
    density = listed / (w.admissible_blocks * Hq)
    attn_flops = 4.0 * d * B * B * listed
    attn_tflops = attn_flops / (t_attn_avg * 1e-3) / 1e12

    # the two kernels of stage 1, timed on their own (outside the timed region above)
    def time_call(fn, n=15):
        fn()
        torch.cuda.synchronize()
        pairs = []
        for _ in range(n):                             # queued back to back: no host gap inside a pair
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            pairs.append((a, b))
        torch.cuda.synchronize()
        return median([a.elapsed_time(b) for a, b in pairs])

    t_pool = time_call(pf.pool)
    t_scores = time_call(pf.block_scores)
    pool_bytes = 2.0 * d * T * (Hq + 2 * Hkv) + 4.0 * d * R * (Hq + Hkv) * args.ad_stride + 4.0 * R * Hkv
    pool_gbs = pool_bytes / (t_pool * 1e-3) / 1e9

    value = dense_flops / (ms_per_step * 1e-3) / 1e12
    traffic, traffic_info = measured_attention_traffic(w.name)
    # the whole estimation stage against the HBM roofline: what the method itself has to move is Q, K, V
    # once, the pooled vectors out and back in, and the causal half of the score tensor out
    est_bytes = pool_bytes + 4.0 * d * (R * Hq + w.total_rows * Hkv) * args.ad_stride + 4.0 * w.admissible_blocks * Hq
    est_gbs = est_bytes / (t_est * 1e-3) / 1e9
    # The paper's only number for this path: 420 ms per 128K layer with its default schedule on an
    # NVIDIA H20 (Empirical Latency), i.e. 335 dense-equivalent TFLOP/s for these shapes.  It applies
    # to that schedule only and is another machine's figure: context, not a target.
    vs_baseline = value / PAPER_H20_128K_DENSE_EQUIV_TFLOPS if w.name == "llama8b_128k_paper_preset" else None
    result = {
        "metric": "sparse prefill attention, dense-equivalent TFLOP/s at 128K (estimate + select + attention, one layer)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None if vs_baseline is None else round(vs_baseline, 2),
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "tokens": T, "q_heads": Hq, "kv_heads": Hkv, "head_dim": d, "block": B,
                   "k_start_blocks": list(w.k_start_blocks), "mu": w.mu, "beta": w.beta,
                   "n_sink": w.n_sink, "n_local": w.n_local, "density": round(density, 5),
                   "listed_blocks": listed, "score_tensor": "tiles without a causal pair not written",
                   **({} if default_options else options)},
        "stages_ms": {"estimate": round(t_est, 4), "select": round(t_sel, 4), "attention": round(t_attn_avg, 4),
                      "pool_kernel": round(t_pool, 4), "scores_kernel": round(t_scores, 4)},
        "attention_dense_equiv_tflops": round(dense_flops / (t_attn_avg * 1e-3) / 1e12, 2),
        "roofline": {"kernel": "sparse_attn_kernel", "bound": "mfma", "achieved": round(attn_tflops, 2),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(attn_tflops / PEAK_BF16_TFLOPS, 4),
                     "traffic": traffic if default_options else None, "traffic_source": traffic_info},
        "estimate_roofline": {"kernel": "pool_kernel", "bound": "hbm", "achieved": round(pool_gbs, 1),
                              "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(pool_gbs / PEAK_HBM_GBS, 4),
                              "algorithmic_bytes": pool_bytes},
        "estimate_stage_roofline": {"kernels": "pool_kernel + block_scores_kernel" if not args.fused else
                                    "pool_kernel + score_select_kernel (selection included)",
                                    "bound": "hbm", "achieved": round(est_gbs, 1), "peak": PEAK_HBM_GBS,
                                    "unit": "GB/s", "frac": round(est_gbs / PEAK_HBM_GBS, 4),
                                    "algorithmic_bytes": est_bytes},
    }
    if args.vendor_gemm:                               # context for the roofline fraction, not part of the path
        n = 16384
        a = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
        b = torch.randn(n, n, device=dev, dtype=torch.bfloat16)
        c = torch.empty(n, n, device=dev, dtype=torch.bfloat16)
        t_gemm = time_call(lambda: torch.matmul(a, b, out=c), n=20)
        result["vendor_gemm"] = {"what": "torch.matmul, bf16, 16384^3, random normal data", "ms": round(t_gemm, 4),
                                 "tflops": round(2.0 * n ** 3 / (t_gemm * 1e-3) / 1e12, 1),
                                 "attention_over_gemm": round(attn_tflops / (2.0 * n ** 3 / (t_gemm * 1e-3) / 1e12), 4)}
        del a, b, c
    if not args.no_cpu_baseline and default_options:   # the oracle leg times the default path only
        result["cpu_baseline"] = cpu_baseline(w, data, dense_flops, pf.counts.cpu().numpy(), pf.indices.cpu().numpy())
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
