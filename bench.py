#!/usr/bin/env python3
"""Benchmark of the Quick ADC hot path on one MI355X.

Workload (BASELINE config 2, "single-query bandwidth scan"): d=128 mixture
data, PQ m=16 x 16 centroids (64-bit codes), N = 10,000,000 codes contiguous
in HBM, queries issued one at a time, uint8 tables, R = 100.

One "step" is one query through the whole path on one stream:
    qadc_build_luts -> qadc_quantize_luts (init = 200) -> qadc_scan_topk
over 10 M codes already resident in HBM.  Successive steps scan successive
code buffers out of `--buffers` distinct ones (default 8 x 80 MB = 640 MB),
so that the scan streams from HBM and not from the 256 MB last-level cache.

Prints ONE JSON line: whole-path throughput in G codes/s, the roofline of the
dominant kernel (the code-streaming scan kernel, timed with HIP events on its
own stream by the library's profiling hooks), and the CPU oracle timed on the
host cores on a bounded sample of the same workload.
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--n", type=int, default=10_000_000, help="codes per query scan")
    ap.add_argument("--buffers", type=int, default=8, help="distinct code buffers rotated over")
    ap.add_argument("--m", type=int, default=16)
    ap.add_argument("--R", type=int, default=100)
    ap.add_argument("--init", type=int, default=200)
    ap.add_argument("--queries", type=int, default=1000)
    ap.add_argument("--cpu-queries", type=int, default=32, help="queries of the CPU-oracle sample (0 = skip)")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event timing pass")
    return ap.parse_args()


def build_database(Q, torch, spec, m, n_total, dev):
    """Codebooks + n_total encoded mixture vectors, all produced on the GPU."""
    from workloads import SEED_TRAIN, SEED_BASE, kmeans_init_rows
    from workloads.mixture_torch import mixture_vectors_torch, BLOCK
    d = spec.d
    dsub = d // m
    # Codebooks: the sub-vectors of 16 seeded learning-set rows (a k-means start state).
    train = mixture_vectors_torch(spec, SEED_TRAIN, 0, 20_000, dev)
    rows = torch.from_numpy(kmeans_init_rows(20_000, 16)).to(dev)
    cb = train[rows].reshape(16, m, dsub).permute(1, 0, 2).contiguous()
    codes = torch.empty((n_total, m // 2), dtype=torch.uint8, device=dev)
    chunk = 4 * BLOCK
    for s in range(0, n_total, chunk):
        cnt = min(chunk, n_total - s)
        x = mixture_vectors_torch(spec, SEED_BASE, s, cnt, dev)
        Q.qadc_pq_encode(cb, x, out=codes[s:s + cnt])
    torch.cuda.synchronize()
    return cb, codes


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
              "(no collectives, no sharding in this library)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_1704_07355_amd as Q
    from workloads import MixtureSpec, SEED_QUERY
    from workloads.mixture_torch import mixture_vectors_torch

    Q.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    spec = MixtureSpec(d=128)
    m, n, R, init = args.m, args.n, args.R, args.init
    row = m // 2

    t0 = time.time()
    cb, codes = build_database(Q, torch, spec, m, n * args.buffers, dev)
    queries = mixture_vectors_torch(spec, SEED_QUERY, 0, args.queries, dev)
    t_build = time.time() - t0
    bufs = [codes[b * n:(b + 1) * n] for b in range(args.buffers)]

    ws_bytes = Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_TOPK, n, m, 1, R)
    ws = Q.qadc_workspace_init(torch.empty(ws_bytes, dtype=torch.uint8, device=dev))
    luts = torch.empty((1, m, 16), dtype=torch.float32, device=dev)
    out_idx = torch.empty((1, R), dtype=torch.int32, device=dev)
    out_dist = torch.empty((1, R), dtype=torch.uint8, device=dev)

    def step(i):
        qi = i % args.queries
        buf = bufs[i % args.buffers]
        Q.qadc_build_luts(cb, queries[qi:qi + 1], out=luts)
        ql, _, _, _ = Q.qadc_quantize_luts(luts, buf[:init], R)
        Q.qadc_scan_topk(Q.QADC_U8_4BIT, buf, ql, R, workspace=ws, out_idx=out_idx, out_dist=out_dist)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    ms_total = e0.elapsed_time(e1)
    ms_per_step = ms_total / args.steps
    gcodes = n / (ms_per_step * 1e-3) / 1e9

    # Per-kernel timing of the scan kernel (HIP events recorded by the library around the
    # kernel on the stream it runs on), same launch configuration, same rotation.
    roofline = None
    scan_only = None
    if not args.no_profile:
        nprof = min(args.steps, 200)
        Q.qadc_profile_enable(True)
        for i in range(nprof):
            step(args.warmup + i)
        torch.cuda.synchronize()
        ms_scan, launches = Q.qadc_profile_read(Q.QADC_PROF_SCAN)
        ms_merge, _ = Q.qadc_profile_read(Q.QADC_PROF_MERGE)
        ms_seed, _ = Q.qadc_profile_read(Q.QADC_PROF_SEED)
        Q.qadc_profile_enable(False)
        avg_ms = ms_scan / max(1, launches)
        achieved = n * row / (avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "scan_u8_kernel", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                    "traffic": None, "avg_kernel_us": round(avg_ms * 1e3, 2),
                    "bytes_per_launch": n * row, "launches_timed": launches}
        scan_only = {"scan_kernel_us": round(avg_ms * 1e3, 2),
                     "merge_kernel_us": round(ms_merge / max(1, launches) * 1e3, 2),
                     "seed_kernel_us": round(ms_seed / max(1, launches) * 1e3, 2)}

    # CPU oracle (plain C twin, one query per thread) on a bounded sample: same codes, same tables.
    cpu = None
    if args.cpu_queries > 0:
        from oracle import cref
        nqc = args.cpu_queries
        h_codes = bufs[0].cpu().numpy()
        l = Q.qadc_build_luts(cb, queries[:nqc].contiguous())
        ql, _, _, _ = Q.qadc_quantize_luts(l, bufs[0][:init], R)
        gi, gd = Q.qadc_scan_topk(Q.QADC_U8_4BIT, bufs[0], ql, R)
        torch.cuda.synchronize()
        h_ql = ql.cpu().numpy()
        t0 = time.time()
        ci, cd = cref.scan_topk_u8(h_codes, h_ql, R)
        dt = time.time() - t0
        same = bool(np.array_equal(gi.cpu().numpy().view(np.uint32), ci)
                    and np.array_equal(gd.cpu().numpy(), cd))
        cpu = {"value": round(nqc * n / dt / 1e9, 4), "unit": "Gcodes/s", "cores": cref.num_threads(),
               "kind": "oracle", "sample": "%d queries x %d codes, one query per thread, scan + top-R "
               "on the GPU's quantized tables" % (nqc, n), "seconds": round(dt, 2),
               "gpu_matches_oracle": same}

    rec = {
        "metric": "G PQ codes scanned/s (single-query 4-bit Quick ADC scan, whole path per query)",
        "value": round(gcodes, 2), "unit": "Gcodes/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config 2: single-query scan, d=128 mixture, PQ m=%d x 4-bit, N=%d codes "
                   "contiguous, queries one at a time, R=%d, init=%d, %d rotating code buffers"
                   % (m, n, R, init, args.buffers),
                   "n": n, "m": m, "R": R, "init": init, "nbins": 255, "buffers": args.buffers,
                   "codebooks": "16 seeded learning-set rows per sub-space"},
        "hbm_gbps_whole_path": round(n * row / (ms_per_step * 1e-3) / 1e9, 1),
        "pct_hbm_peak_whole_path": round(100 * n * row / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        "roofline": roofline, "kernels": scan_only, "cpu_baseline": cpu,
        "database_build_s": round(t_build, 2),
    }
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
