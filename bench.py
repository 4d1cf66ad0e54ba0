#!/usr/bin/env python3
"""Benchmark of the Quick ADC hot path on one MI355X.

Workload (config 2, "single-query bandwidth scan"): d=128 mixture
data, PQ m=16 x 16 centroids (64-bit codes) trained by 10 k-means iterations
on 20,000 vectors, N = 10,000,000 codes contiguous in HBM, queries issued one
at a time, uint8 tables (init = 200), R = 100.

One "step" is one query through the whole path on one stream -- Tables, quantization
of the tables, scan, top-R -- by qadc_search (or, with --separate-calls, by
qadc_build_luts -> qadc_quantize_luts -> qadc_scan_topk: same arithmetic, more launches)
over 10 M codes already resident in HBM.  Successive steps scan successive
code buffers out of `--buffers` distinct ones (default 8 x 80 MB = 640 MB),
so that the scan streams from HBM and not from the 256 MB last-level cache.

Prints ONE JSON line: whole-path throughput in G codes/s, the roofline of the
dominant kernel (the code-streaming scan kernel; its duration is taken from HIP
events attached to its own dispatches by the library's profiling hooks), the
accuracy of the quantized scan against float ADC, and the CPU oracle timed on
the host cores on a bounded sample of the same workload.
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


WORKLOAD_DEFAULTS = {
    "scan": dict(steps=1000, warmup=50, n=10_000_000, m=16, init=200, batch=256),
    "batched": dict(steps=8, warmup=1, n=100_000_000, m=32, init=1000, batch=256),
    "ivf": dict(steps=4, warmup=1, n=1_000_000_000, m=32, init=1000, batch=4096),
    "compare": dict(steps=1000, warmup=20, n=50_000_000, m=16, init=200, batch=256),
    "build": dict(steps=3, warmup=1, n=4_000_000, m=16, init=200, batch=256),
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--workload", choices=["scan", "batched", "ivf", "compare", "build"], default="scan",
                    help="scan: config 2, one query at a time (default); batched: config 3, query batches "
                         "over 128-bit codes; ivf: config 4, inverted index with Zipf-skewed lists; "
                         "compare: config 5, 8-bit PQ with float tables against Quick ADC on the same vectors; "
                         "build: database side, an inverted index built from raw vectors (assign, group, "
                         "encode residuals, transposed layout)")
    ap.add_argument("--K", type=int, default=65536, help="coarse centroids of the ivf workload")
    ap.add_argument("--nprobe", type=int, default=64)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--n", type=int, default=None, help="codes per query scan")
    ap.add_argument("--batch", type=int, default=None,
                    help="queries per step of the batched (default 256) and ivf (default 4096) workloads")
    ap.add_argument("--buffers", type=int, default=8, help="distinct code buffers rotated over")
    ap.add_argument("--m", type=int, default=None)
    ap.add_argument("--d", type=int, default=128, help="dimensions of the vectors (scan and ivf workloads)")
    ap.add_argument("--R", type=int, default=100)
    ap.add_argument("--nbins", type=int, default=255,
                    help="scan workload: bins of the table quantizer (255: unsigned bytes; 127: the paper's signed bytes)")
    ap.add_argument("--init", type=int, default=None)
    ap.add_argument("--queries", type=int, default=1000)
    ap.add_argument("--cpu-queries", type=int, default=2048, help="queries of the CPU-oracle sample (0 = skip)")
    ap.add_argument("--recall-queries", type=int, default=100, help="queries of the accuracy sample (0 = skip)")
    ap.add_argument("--no-profile", action="store_true", help="skip the per-kernel event timing pass")
    ap.add_argument("--copy-calibration", type=int, default=0,
                    help="also run this many plain device copies of 80 MB of codes (untimed), so that a counter "
                         "run can scale FETCH_SIZE / WRITE_SIZE by a kernel of known traffic")
    ap.add_argument("--streams", type=int, default=2,
                    help="scan workload: also time the same steps dealt round-robin to this many HIP streams "
                         "(each with a workspace of its own), reported beside the single-stream value; 1 = skip")
    ap.add_argument("--opq", type=int, default=0, metavar="ROUNDS",
                    help="scan workload: train an optimized product quantizer with this many rounds; database "
                         "vectors are rotated before encoding and every query by qadc_rotate before qadc_search")
    ap.add_argument("--no-mi-full", action="store_true",
                    help="ivf workload: skip the multi-index of 2^14 x 2^14 cells over the same codes")
    ap.add_argument("--no-small-calls", action="store_true",
                    help="ivf: skip the timing of calls of 1, 4, 16 and 64 queries")
    ap.add_argument("--no-extras", action="store_true",
                    help="scan workload: skip the short runs of configs 3, 4 and 5 nested in the same line")
    ap.add_argument("--separate-calls", action="store_true",
                    help="time qadc_build_luts + qadc_quantize_luts + qadc_scan_topk instead of qadc_search")
    args = ap.parse_args()
    for k, v in WORKLOAD_DEFAULTS[args.workload].items():
        if getattr(args, k) is None:
            setattr(args, k, v)
    return args


def copy_calibration(torch, src, times):
    """Plain device copies of the first 80,000,000 bytes of `src` (untimed): a counter run scales
    FETCH_SIZE / WRITE_SIZE by these dispatches of known traffic."""
    if times <= 0:
        return
    flat = src.reshape(-1)[:80_000_000]
    dst = torch.empty_like(flat)
    for _ in range(times):
        dst.copy_(flat)
    torch.cuda.synchronize()


def train_opq(Q, torch, train, m, rows, rounds, iters=10):
    """Optimized product quantizer on the GPU (bench support): `rounds` times { codebooks by k-means on
    the rotated learning set; rotation by orthogonal Procrustes between the learning set and its
    reproductions }, then the codebooks of the final rotation.  -> (rot [d][d], codebooks)."""
    n, d = train.shape
    dsub = d // m
    rot = torch.eye(d, dtype=torch.float32, device=train.device)
    for _ in range(rounds):
        xr = Q.qadc_rotate(rot, train)
        cb = Q.qadc_pq_train(xr, m, 16, rows, iters)
        codes = Q.qadc_pq_encode(cb, xr).long()
        comps = torch.stack([codes & 15, codes >> 4], dim=2).reshape(n, m)     # component j of every row
        y = torch.cat([cb[j][comps[:, j]] for j in range(m)], dim=1)            # reproductions pq(R x)
        u, _, vt = torch.linalg.svd(train.double().T @ y.double())
        rot = (u @ vt).T.float().contiguous()
    xr = Q.qadc_rotate(rot, train)
    return rot, Q.qadc_pq_train(xr, m, 16, rows, iters)


def build_database(Q, torch, spec, m, n_total, n_keep, dev, opq_rounds=0):
    """Codebooks (GPU k-means) + n_total encoded mixture vectors, all produced on the GPU.

    The raw vectors of the first n_keep rows are kept for the exact-neighbour accuracy check.
    With opq_rounds > 0 the quantizer is an optimized product quantizer: the vectors are rotated
    before encoding and the rotation is returned as a fourth value.
    """
    from workloads import SEED_TRAIN, SEED_BASE, kmeans_init_rows
    from workloads.mixture_torch import mixture_vectors_torch, BLOCK
    train = mixture_vectors_torch(spec, SEED_TRAIN, 0, 20_000, dev)
    rows = torch.from_numpy(kmeans_init_rows(20_000, 16)).to(dev)
    rot = None
    if opq_rounds > 0:
        rot, cb = train_opq(Q, torch, train, m, rows, opq_rounds)
    else:
        cb = Q.qadc_pq_train(train, m, 16, rows, 10)
    codes = torch.empty((n_total, m // 2), dtype=torch.uint8, device=dev)
    raw = torch.empty((n_keep, spec.d), dtype=torch.float32, device=dev) if n_keep else None
    chunk = 4 * BLOCK
    for s in range(0, n_total, chunk):
        cnt = min(chunk, n_total - s)
        x = mixture_vectors_torch(spec, SEED_BASE, s, cnt, dev)
        Q.qadc_pq_encode(cb, Q.qadc_rotate(rot, x) if rot is not None else x, out=codes[s:s + cnt])
        if raw is not None and s < n_keep:
            k = min(cnt, n_keep - s)
            raw[s:s + k] = x[:k]
    torch.cuda.synchronize()
    if opq_rounds > 0:
        return cb, codes, raw, rot
    return cb, codes, raw


def accuracy(Q, torch, np, cb, codes, raw, queries, R, init, rot=None, nbins=255):
    """overlap@R of the quantized scan with float ADC on the same codes, and NN-recall@R of both."""
    luts = Q.qadc_build_luts(cb, Q.qadc_rotate(rot, queries) if rot is not None else queries)
    ql, _, _, _ = Q.qadc_quantize_luts(luts, codes[:init], R, nbins)
    qi, _ = Q.qadc_scan_topk(Q.QADC_U8_4BIT, codes, ql, R, nbins)
    fi, _ = Q.qadc_scan_topk(Q.QADC_F32_4BIT, codes, luts, R)
    # exact nearest neighbour of each query among the raw vectors (measurement only)
    best = torch.full((queries.shape[0],), float("inf"), device=queries.device)
    arg = torch.zeros((queries.shape[0],), dtype=torch.int64, device=queries.device)
    qq = (queries * queries).sum(1)
    step = 1 << 20
    for s in range(0, raw.shape[0], step):
        x = raw[s:s + step]
        dist = qq[:, None] - 2.0 * queries @ x.T + (x * x).sum(1)[None, :]
        v, a = dist.min(1)
        upd = v < best
        best[upd] = v[upd]
        arg[upd] = a[upd] + s
    torch.cuda.synchronize()
    qi = qi.cpu().numpy().view(np.uint32).astype(np.int64)
    fi = fi.cpu().numpy().view(np.uint32).astype(np.int64)
    nn = arg.cpu().numpy()
    overlap = float(np.mean([len(np.intersect1d(a, b)) / R for a, b in zip(qi, fi)]))
    rec_q = float(np.mean([nn[i] in qi[i] for i in range(len(nn))]))
    rec_f = float(np.mean([nn[i] in fi[i] for i in range(len(nn))]))
    return {"queries": int(queries.shape[0]), "overlap_at_R_vs_float_adc": round(overlap, 4),
            "nn_recall_at_R_quick_adc": round(rec_q, 4), "nn_recall_at_R_float_adc": round(rec_f, 4)}


# HBM bytes per scan_u8_kernel launch from the FETCH_SIZE / WRITE_SIZE counter runs summarized in
# profiles/scan_u8_config2_hbm_traffic.md (scaled by a plain copy of known size); valid for the
# workload it was measured on only: (n, m) -> (bytes read, bytes written).
SCAN_TRAFFIC = {(10_000_000, 16): (39152.4 * 1.9994 * 1024, 53.1 * 1.0 * 1024)}
TILED_TRAFFIC = 8_680_000_000   # config 3, scan_u8_tiled16_kernel<16, 2>: HBM bytes read per 256-query batch
COMPARE_TRAFFIC = 400_060_000   # config 5, scan_u8_kernel<8, 256>: HBM bytes read per query

MFMA_TRAFFIC = 1_619_000_000    # config 3, scan_u8_mfma_kernel<16>: HBM bytes read per 256-query batch
MFMA_I8_PEAK_TOPS = 5000.0      # dense int8 MFMA peak of the chip
ALU_PEAK_TLOOKUPS = 157.3  # 256 CUs x 64 lanes x 2.4 GHz x 4 byte lanes per 32-bit lane-op


def run_batched(args):
    """Config 3: batches of queries over 128-bit codes; a step = one batch through qadc_search."""
    import numpy as np
    import torch
    import paper_1704_07355_amd as Q
    from workloads import MixtureSpec, SEED_QUERY
    from workloads.mixture_torch import mixture_vectors_torch

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    spec = MixtureSpec(d=128)
    m, n, R, init, nb = args.m, args.n, args.R, args.init, args.batch
    t0 = time.time()
    cb, codes, _ = build_database(Q, torch, spec, m, n, 0, dev)
    nq_total = nb * (args.steps + args.warmup)
    queries = mixture_vectors_torch(spec, SEED_QUERY, 0, nq_total, dev)
    t_build = time.time() - t0
    copy_calibration(torch, codes, args.copy_calibration)
    ws = Q.qadc_workspace_init(torch.empty(Q.qadc_workspace_bytes(Q.QADC_WS_SEARCH, n, m, nb, R),
                                           dtype=torch.uint8, device=dev))
    out_idx = torch.empty((nb, R), dtype=torch.int32, device=dev)
    out_dist = torch.empty((nb, R), dtype=torch.uint8, device=dev)
    ql_out = torch.empty((nb, m, 16), dtype=torch.uint8, device=dev)

    def step(i):
        Q.qadc_search(cb, queries[i * nb:(i + 1) * nb], codes, R, init, workspace=ws, out_idx=out_idx,
                      out_dist=out_dist, qluts_out=ql_out)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps
    pairs = n * nb / (ms_per_step * 1e-3)

    roofline = kernels = None
    if not args.no_profile:
        Q.qadc_profile_enable(True)
        step(args.warmup + args.steps - 1)
        torch.cuda.synchronize()
        ms_scan, launches = Q.qadc_profile_read(Q.QADC_PROF_SCAN)
        ms_prep = sum(Q.qadc_profile_read(w)[0] for w in (Q.QADC_PROF_PREPARE, Q.QADC_PROF_TABLES,
                                                          Q.QADC_PROF_QUANTIZE))
        ms_seed, _ = Q.qadc_profile_read(Q.QADC_PROF_SEED)
        ms_merge, _ = Q.qadc_profile_read(Q.QADC_PROF_MERGE)
        Q.qadc_profile_enable(False)
        ach = n * nb * m / (ms_scan * 1e-3) / 1e12
        on_matrix_cores = nb >= (16 if m >= 16 else 32) and os.environ.get("QADC_TILED_MFMA", "1") != "0"
        if on_matrix_cores:
            # The method's work is m lookup-adds per (code, query) pair (Alg. 2); the ceiling quoted for
            # it is the vector ALU's byte-lane rate, whatever unit executes it.  This kernel forms the
            # sums as one-hot int8 products on the sparse matrix instruction: every lookup-add is a
            # 16-term dot product of which the hardware executes 8 terms (two of every four) -- reported
            # beside it, not as the fraction.
            ops = n * nb * m * 8 * 2 / (ms_scan * 1e-3) / 1e12
            roofline = {"bound": "alu", "kernel": "scan_u8_mfma_kernel (+ the redo launch)", "achieved": round(ach, 2),
                        "peak": ALU_PEAK_TLOOKUPS, "unit": "T lookup-adds/s", "frac": round(ach / ALU_PEAK_TLOOKUPS, 4),
                        "note": "m lookup-adds per (code, query) pair against the byte-lane ceiling of the vector ALU "
                                "(256 CUs x 64 lanes x 2.4 GHz x 4 byte lanes); the kernel executes them on the matrix "
                                "cores as one-hot products, 15 of every 16 by zero",
                        "int8_ops_executed_tops": round(ops, 1),
                        "int8_ops_executed_frac_of_dense_mfma_peak": round(ops / MFMA_I8_PEAK_TOPS, 4),
                        "lookup_adds_as_int8_macs_frac_of_mfma_peak": round(2 * ach / MFMA_I8_PEAK_TOPS, 4),
                        "traffic": MFMA_TRAFFIC if (n, m, nb) == (100_000_000, 32, 256) else None,
                        "traffic_source": "profiles/hbm_traffic_configs_3_4_5.md (rocprofv3 --pmc FETCH_SIZE, bytes read per launch)",
                        "scan_ms": round(ms_scan, 3), "launches_timed": launches}
        else:
            roofline = {"bound": "alu", "kernel": "scan_u8_tiled16_kernel (+ 16-bit-lane and redo launches)", "achieved": round(ach, 2),
                        "peak": ALU_PEAK_TLOOKUPS, "unit": "T lookup-adds/s", "frac": round(ach / ALU_PEAK_TLOOKUPS, 4),
                        "traffic": TILED_TRAFFIC if (n, m, nb) == (100_000_000, 32, 256) else None,
                        "traffic_source": "profiles/hbm_traffic_configs_3_4_5.md (rocprofv3 --pmc FETCH_SIZE, bytes read per launch)",
                        "scan_ms": round(ms_scan, 3), "launches_timed": launches}
        kernels = {"scan_ms": round(ms_scan, 3), "tables_quantize_ms": round(ms_prep, 3),
                   "seed_tau_ms": round(ms_seed, 3), "merge_ms": round(ms_merge, 3)}

    cpu = None
    if args.cpu_queries > 0:
        from oracle import cref
        nqc = min(64, nb)
        h_codes = codes.cpu().numpy()
        h_ql = ql_out[:nqc].cpu().numpy()
        gi, gd = out_idx[:nqc].cpu().numpy().view(np.uint32), out_dist[:nqc].cpu().numpy()
        t0 = time.time()
        ci, cd = cref.scan_topk_u8(h_codes, h_ql, R)
        dt = time.time() - t0
        cpu = {"value": round(nqc * n / dt / 1e9, 4), "unit": "G pairs/s", "cores": cref.num_threads(),
               "kind": "oracle", "sample": "%d queries of the last batch x %d codes, one query per thread"
               % (nqc, n), "seconds": round(dt, 2),
               "gpu_matches_oracle": bool(np.array_equal(gi, ci) and np.array_equal(gd, cd))}

    return ({
        "metric": "G (code, query) pairs scanned/s (query-batched 4-bit Quick ADC scan, whole path per batch)",
        "value": round(pairs / 1e9, 1), "unit": "Gpairs/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config 3: d=128 mixture, PQ m=%d x 4-bit, N=%d codes, batches of %d queries "
                   "through qadc_search (a wavefront scans each code for 64 queries), R=%d, init=%d"
                   % (m, n, nb, R, init), "n": n, "m": m, "R": R, "init": init, "batch": nb},
        "gcodes_per_s_per_query": round(pairs / nb / 1e9, 2),
        "roofline": roofline, "kernels": kernels, "cpu_baseline": cpu, "database_build_s": round(t_build, 2)})


def build_ivf_index(Q, torch, np, n, K, m, n_queries, dev, d=128, sigma=18.0):
    """Synthetic inverted index on the GPU (see run_ivf) -> (IvfIndex, list sizes, queries)."""
    from workloads import MixtureSpec, SEED_BASE, SEED_TRAIN, zipf_list_sizes, kmeans_init_rows
    from workloads.mixture_torch import mixture_vectors_torch
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED_BASE * 7919 + 11)
    coarse = mixture_vectors_torch(MixtureSpec(d=d), SEED_TRAIN, 0, K, dev)
    sizes = zipf_list_sizes(n, K, 0.8, SEED_BASE)
    list_off = torch.from_numpy(np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)).to(dev)
    train = sigma * torch.randn((20_000, d), generator=gen, device=dev)
    cb = Q.qadc_pq_train(train.contiguous(), m, 16, torch.from_numpy(kmeans_init_rows(20_000, 16)).to(dev), 10)
    codes = torch.empty((n, m // 2), dtype=torch.uint8, device=dev)
    chunk = 1 << 22
    for s in range(0, n, chunk):
        cnt = min(chunk, n - s)
        x = sigma * torch.randn((cnt, d), generator=gen, device=dev)
        Q.qadc_pq_encode(cb, x, out=codes[s:s + cnt])
    ids = torch.arange(n, dtype=torch.int32, device=dev)
    index = Q.IvfIndex(coarse, list_off, codes, ids, cb)
    prob = torch.from_numpy(sizes / sizes.sum()).to(dev)
    home = torch.multinomial(prob, n_queries, replacement=True, generator=gen)
    queries = (coarse[home] + sigma * torch.randn((n_queries, d), generator=gen, device=dev)).contiguous()
    torch.cuda.synchronize()
    return index, sizes, queries


def multi_index_usual_size(Q, torch, coarse, codes, cb, queries, last, nb, nprobe, R, init, dev, d, kh=16384):
    """The same codes under a multi-index of kh x kh product cells with lists for the occupied cells only
    (2^28 cells for 10^9 vectors: most are empty, lists are short).  Half-centroids are halves of vectors
    drawn like the coarse centroids; a stored vector's cell is one of the 4 closest cells of a point drawn
    around a coarse centroid, as the queries are, so the probes of a query meet occupied cells.  Times the grouping (database side) and one batch of queries
    through Index (probes, then list numbers) and qadc_ivf_search."""
    from workloads import MixtureSpec, SEED_TRAIN
    from workloads.mixture_torch import mixture_vectors_torch
    n = codes.shape[0]
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    # half-centroids: the halves of vectors drawn like the coarse centroids (rows after theirs)
    hv = mixture_vectors_torch(MixtureSpec(d=d), SEED_TRAIN, 1 << 20, kh, dev)
    halves = torch.stack([hv[:, :d // 2], hv[:, d // 2:]]).contiguous()
    # a pool of cells around the coarse centroids, where the queries are drawn too
    chunk = 8192
    mi_ws = torch.empty((Q.qadc_multi_index_workspace_bytes(kh, chunk, 4),), dtype=torch.uint8, device=dev)
    pool = []
    for s in range(0, max(chunk, min(1 << 20, n // 256)), chunk):
        home = torch.randint(0, coarse.shape[0], (chunk,), generator=gen, device=dev)
        pts = (coarse[home] + 18.0 * torch.randn((chunk, d), generator=gen, device=dev)).contiguous()
        pool.append(Q.qadc_multi_index_probes(halves, pts, 4, workspace=mi_ws).reshape(-1).clone())
    pool = torch.cat(pool)
    cells = torch.empty((n,), dtype=torch.int32, device=dev)
    for s in range(0, n, 1 << 26):
        cnt = min(1 << 26, n - s)
        cells[s:s + cnt] = pool[torch.randint(0, pool.numel(), (cnt,), generator=gen, device=dev)]
    del mi_ws
    ws = torch.empty((Q.qadc_multi_index_group_workspace_bytes(n, kh),), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    t0 = time.time()
    cell_ids, list_off, ids = Q.qadc_multi_index_group(cells, kh, workspace=ws)
    torch.cuda.synchronize()
    t_group = time.time() - t0
    del ws, cells
    index = Q.IvfIndex(None, list_off, codes, ids, cb, halves=halves, cell_ids=cell_ids)
    qb = queries[last * nb:(last + 1) * nb]
    mi_ws = torch.empty((Q.qadc_multi_index_workspace_bytes(kh, nb, nprobe),), dtype=torch.uint8, device=dev)
    probes = torch.empty((nb, nprobe), dtype=torch.int32, device=dev)
    sws = Q.qadc_workspace_init(torch.empty(Q.qadc_ivf_workspace_bytes(index, nb, nprobe, R), dtype=torch.uint8,
                                            device=dev))

    def batch():
        Q.qadc_multi_index_probes(halves, qb, nprobe, workspace=mi_ws, out=probes)
        slots = Q.qadc_multi_index_slots(cell_ids, probes, out=probes)
        return slots, Q.qadc_ivf_search(index, qb, nprobe, R, init, probes_in=slots, workspace=sws)

    batch()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(3):
        slots, _ = batch()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / 3
    used = slots.clamp(min=0).long()
    lens = (list_off[used + 1] - list_off[used]) * (slots >= 0)
    sizes = list_off[1:] - list_off[:-1]
    return {"half_centroids": kh, "cells": kh * kh, "occupied_cells": int(cell_ids.numel()),
            "largest_list": int(sizes.max().item()), "grouping_s": round(t_group, 3),
            "occupied_probes_per_query": round(float((slots >= 0).sum().item()) / nb, 2),
            "codes_scanned_per_query": round(float(lens.sum().item()) / nb, 1),
            "ms_per_batch": round(ms, 3), "queries_per_s": round(nb / (ms * 1e-3), 1)}


def run_ivf(args):
    """Config 4: IVF + Quick ADC.  A step = one batch of queries through qadc_ivf_search.

    Synthetic index built list by list on the GPU: list sizes follow a Zipf(0.8) profile, every
    stored vector is its cell's centroid plus N(0, 18^2) noise, so its residual code is the
    encoding of that noise; ids are a running counter; a query is the centroid of a size-weighted
    random cell plus N(0, 18^2) noise.
    """
    import numpy as np
    import torch
    import paper_1704_07355_amd as Q
    from workloads import MixtureSpec, SEED_QUERY, SEED_BASE, SEED_TRAIN, zipf_list_sizes, kmeans_init_rows
    from workloads.mixture_torch import mixture_vectors_torch

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    m, n, K, R, init, nprobe, nb = args.m, args.n, args.K, args.R, args.init, args.nprobe, args.batch
    t0 = time.time()
    nq_total = nb * (args.steps + args.warmup)
    index, sizes, queries = build_ivf_index(Q, torch, np, n, K, m, nq_total, dev, d=args.d)
    coarse, list_off, codes, _, cb = index.tensors
    t_build = time.time() - t0
    copy_calibration(torch, codes, args.copy_calibration)

    ws = Q.qadc_workspace_init(torch.empty(Q.qadc_ivf_workspace_bytes(index, nb, nprobe, R),
                                           dtype=torch.uint8, device=dev))

    def step(i, debug=False):
        return Q.qadc_ivf_search(index, queries[i * nb:(i + 1) * nb], nprobe, R, init, workspace=ws, debug=debug)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        step(args.warmup + i)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = e0.elapsed_time(e1) / args.steps

    Q.qadc_profile_enable(True)
    last = args.warmup + args.steps - 1
    out_ids, out_dist, probes, qluts = step(last, debug=True)
    torch.cuda.synchronize()
    phase = {}
    for name, which in (("index", Q.QADC_PROF_IVF_INDEX), ("tables", Q.QADC_PROF_IVF_TABLES),
                        ("quantize", Q.QADC_PROF_QUANTIZE), ("seed", Q.QADC_PROF_SEED),
                        ("scan", Q.QADC_PROF_SCAN), ("scan_shared", Q.QADC_PROF_IVF_SHARED),
                        ("merge", Q.QADC_PROF_MERGE)):
        phase[name] = Q.qadc_profile_read(which)[0]
    Q.qadc_profile_enable(False)
    h_probes = probes.cpu().numpy()
    scanned = float(sizes[h_probes.clip(0)].sum())  # (code, query) pairs of the last batch
    row = m // 2
    if phase["scan_shared"] > 0:
        # Large batches: the lists probed by several queries are scanned once for all of them on the
        # matrix units (ivfs_scan_kernel), the others query by query (ivf_scan_kernel).  The method's
        # work is m lookup-adds per (code, query) pair; as for the batched exhaustive scan, the ceiling
        # quoted for it is the byte-lane rate of the vector ALU.
        per_cell = np.bincount(h_probes[h_probes >= 0].ravel(), minlength=K)
        min_pairs = int(os.environ.get("QADC_IVF_SHARED_MIN_PAIRS", "4"))
        shared = (h_probes >= 0) & (per_cell[h_probes.clip(0)] >= min_pairs)
        pairs_shared = float(sizes[h_probes[shared]].sum())
        pairs_own = scanned - pairs_shared
        codes_once = float(sizes[per_cell >= min_pairs].sum())  # codes of the shared lists, each read once per 32 pairs
        ach = pairs_shared * m / (phase["scan_shared"] * 1e-3) / 1e12
        own = pairs_own * row / (phase["scan"] * 1e-3) / 1e9 if phase["scan"] > 0 else 0.0
        roofline = {"bound": "alu", "kernel": "ivfs_scan_kernel", "achieved": round(ach, 2), "peak": ALU_PEAK_TLOOKUPS,
                    "unit": "T lookup-adds/s", "frac": round(ach / ALU_PEAK_TLOOKUPS, 4), "traffic": None,
                    "note": "m lookup-adds per (code, query) pair of the lists shared by >= %d queries of the batch, "
                            "against the byte-lane ceiling of the vector ALU; executed as one-hot int8 products on "
                            "the sparse matrix instruction, 32 pairs per wavefront whatever the number that exist"
                            % min_pairs,
                    "scan_shared_ms_per_batch": round(phase["scan_shared"], 3),
                    "pairs_shared_per_query": round(pairs_shared / nb), "shared_list_codes": round(codes_once),
                    "per_query_kernel": {"kernel": "ivf_scan_kernel", "bound": "hbm", "achieved": round(own, 1),
                                         "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(own / HBM_PEAK_GBPS, 4),
                                         "scan_ms_per_batch": round(phase["scan"], 3),
                                         "pairs_per_query": round(pairs_own / nb)},
                    "codes_scanned_per_query": round(scanned / nb)}
    else:
        ach = scanned * row / (phase["scan"] * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "ivf_scan_kernel", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None,
                    "traffic_note": "depends on the batch; measured at 1.01 x the algorithmic bytes "
                                    "(profiles/hbm_traffic_configs_3_4_5.md)",
                    "scan_ms_per_batch": round(phase["scan"], 3), "codes_scanned_per_query": round(scanned / nb)}

    # beside it: the Index step of an inverted multi-index with as many cells (two quantizers of
    # sqrt(K) half-centroids, seeded at random: only the step's cost is measured here)
    multi_index = None
    kh = int(round(K ** 0.5))
    if kh * kh == K and kh <= 4096 and nprobe <= 256:
        gen = torch.Generator(device=dev)
        gen.manual_seed(7)
        halves = torch.rand((2, kh, args.d // 2), generator=gen, device=dev) * 255.0
        qb = queries[last * nb:(last + 1) * nb]
        mi_ws = torch.empty((Q.qadc_multi_index_workspace_bytes(kh, nb, nprobe),), dtype=torch.uint8, device=dev)
        mi_out = torch.empty((nb, nprobe), dtype=torch.int32, device=dev)
        for _ in range(2):
            Q.qadc_multi_index_probes(halves, qb, nprobe, workspace=mi_ws, out=mi_out)
        m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        m0.record()
        for _ in range(10):
            Q.qadc_multi_index_probes(halves, qb, nprobe, workspace=mi_ws, out=mi_out)
        m1.record()
        torch.cuda.synchronize()
        multi_index = {"half_centroids": kh, "cells": K, "index_step_ms_per_batch": round(m0.elapsed_time(m1) / 10, 4),
                       "inverted_index_step_ms_per_batch": round(phase["index"], 4)}

    if multi_index is not None and not getattr(args, "no_mi_full", False):
        multi_index["usual_size"] = multi_index_usual_size(Q, torch, coarse, codes, cb, queries, last, nb, nprobe, R,
                                                           init, dev, args.d)

    cpu = None
    if args.cpu_queries > 0:
        from oracle import qadc_oracle as O
        nqc = min(32, nb)
        h_coarse, h_cb = coarse.cpu().numpy(), cb.cpu().numpy()
        h_off = list_off.cpu().numpy()
        h_q = queries[last * nb:last * nb + nqc].cpu().numpy()
        h_ql = qluts[:nqc].cpu().numpy()
        gi, gd = out_ids[:nqc].cpu().numpy().view(np.uint32), out_dist[:nqc].cpu().numpy()
        same, codes_done, dt = True, 0, 0.0
        for iq in range(nqc):
            cells = h_probes[iq]
            # host copy of the probed lists only, re-based into a compact index
            lens = (h_off[cells + 1] - h_off[cells]).astype(np.int64)
            sub_off = np.zeros(len(cells) + 1, dtype=np.int64)
            np.cumsum(lens, out=sub_off[1:])
            sub_codes = torch.cat([codes[h_off[c]:h_off[c + 1]] for c in cells]).cpu().numpy()
            sub_ids = np.concatenate([np.arange(h_off[c], h_off[c + 1], dtype=np.int64) for c in cells])
            order = np.argsort(sub_ids, kind="stable")  # storage-position order decides ties
            sub = dict(list_off=sub_off, codes=sub_codes, ids=sub_ids.astype(np.uint32))
            t1 = time.time()
            rep = O.ivf_quick_adc_search(sub, h_coarse[cells], h_cb, h_q[iq], len(cells), init, R,
                                         probes=np.arange(len(cells)), qluts=h_ql[iq])
            dt += time.time() - t1
            codes_done += int(lens.sum())
            # the compact index keeps probe order, the real one storage order: compare as sets of
            # (sum, id) after sorting ties by id, which is the storage position here
            want = sorted(zip(rep["dist"].tolist(), rep["ids"].tolist()))
            got = sorted(zip(gd[iq].tolist(), gi[iq].tolist()))
            same = same and ([w[0] for w in want] == [g[0] for g in got])
            del order
        cpu = {"value": round(codes_done / dt / 1e9, 4), "unit": "Gcodes/s", "cores": 1, "kind": "oracle",
               "sample": "%d queries of the last batch, NumPy oracle replay of the GPU's cells and tables "
               "(%d codes)" % (nqc, codes_done), "seconds": round(dt, 2), "gpu_sums_match_oracle": bool(same)}

    # beside it: batches alternating over two streams, each with a workspace of its own (the small kernels
    # of one batch overlap the scans of the other)
    two_streams = None
    if args.streams > 1 and not getattr(args, "no_small_calls", False):
        strs = [torch.cuda.Stream(device=dev) for _ in range(2)]
        wss = [ws, Q.qadc_workspace_init(torch.empty(Q.qadc_ivf_workspace_bytes(index, nb, nprobe, R),
                                                     dtype=torch.uint8, device=dev))]
        nbat = nq_total // nb
        torch.cuda.synchronize()

        def alternate(reps):
            for i in range(reps):
                with torch.cuda.stream(strs[i % 2]):
                    Q.qadc_ivf_search(index, queries[(i % nbat) * nb:(i % nbat + 1) * nb], nprobe, R, init,
                                      workspace=wss[i % 2])
        alternate(2)
        torch.cuda.synchronize()
        t2 = time.time()
        alternate(2 * args.steps)
        torch.cuda.synchronize()
        dt2 = time.time() - t2
        two_streams = {"ms_per_batch": round(dt2 / (2 * args.steps) * 1e3, 3),
                       "queries_per_s": round(nb * 2 * args.steps / dt2, 1)}
        del wss

    # beside it: calls of a few queries (response time; the batch rate above is the headline)
    small_calls = {}
    for nsm in (1, 4, 16, 64):
        if nsm > nb or getattr(args, "no_small_calls", False):
            continue
        sws = Q.qadc_workspace_init(torch.empty(Q.qadc_ivf_workspace_bytes(index, nsm, nprobe, R),
                                                dtype=torch.uint8, device=dev))
        reps = 200 if nsm <= 4 else 50
        for i in range(5):
            Q.qadc_ivf_search(index, queries[i * nsm:(i + 1) * nsm], nprobe, R, init, workspace=sws)
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s0.record()
        for i in range(reps):
            j = i % (nq_total // nsm)
            Q.qadc_ivf_search(index, queries[j * nsm:(j + 1) * nsm], nprobe, R, init, workspace=sws)
        s1.record()
        torch.cuda.synchronize()
        small_calls[str(nsm)] = round(s0.elapsed_time(s1) / reps, 4)
        del sws

    return ({
        "metric": "queries/s (IVF + Quick ADC, whole path per batch)",
        "value": round(nb / (ms_per_step * 1e-3), 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config 4: IVF K=%d, Zipf(0.8) lists, N=%d residual codes m=%d x 4-bit, nprobe=%d, "
                   "batches of %d queries, R=%d, init=%d" % (K, n, m, nprobe, nb, R, init),
                   "n": n, "K": K, "m": m, "nprobe": nprobe, "R": R, "init": init, "batch": nb},
        "gcodes_scanned_per_s": round(scanned / (ms_per_step * 1e-3) / 1e9, 2),
        "phase_ms_per_query": {k: round(v / nb, 5) for k, v in phase.items()},
        "multi_index": multi_index, "ms_per_call_of_few_queries": small_calls, "two_streams": two_streams,
        "roofline": roofline, "cpu_baseline": cpu, "database_build_s": round(t_build, 2)})


def run_compare(args):
    """Config 5: the same d=96 vectors under 8-bit PQ (m=8 x 256, float32 tables, Alg. 1) and under
    Quick ADC (m=16 x 16, uint8 tables, Alg. 2), both 64-bit codes, both one query at a time
    through the same scan API.  A step = one query through both paths; `value` is Quick ADC's rate.
    """
    import numpy as np
    import torch
    import paper_1704_07355_amd as Q
    from workloads import MixtureSpec, SEED_QUERY, SEED_TRAIN, SEED_BASE, kmeans_init_rows
    from workloads.mixture_torch import mixture_vectors_torch, BLOCK

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    spec = MixtureSpec(d=96)
    n, R, init = args.n, args.R, args.init
    t0 = time.time()
    train = mixture_vectors_torch(spec, SEED_TRAIN, 0, 20_000, dev)
    cb8 = Q.qadc_pq_train(train, 8, 256, torch.from_numpy(kmeans_init_rows(20_000, 256)).to(dev), 10)
    cb4 = Q.qadc_pq_train(train, 16, 16, torch.from_numpy(kmeans_init_rows(20_000, 16)).to(dev), 10)
    cb6 = Q.qadc_pq_train(train, 16, 64, torch.from_numpy(kmeans_init_rows(20_000, 64)).to(dev), 10)
    codes8 = torch.empty((n, 8), dtype=torch.uint8, device=dev)
    codes4 = torch.empty((n, 8), dtype=torch.uint8, device=dev)
    codes6 = torch.empty((n, 12), dtype=torch.uint8, device=dev)  # m = 16 x 6-bit: 96-bit codes
    keep = args.recall_queries > 0
    raw = torch.empty((n, spec.d), dtype=torch.float32, device=dev) if keep else None
    chunk = 4 * BLOCK
    for s in range(0, n, chunk):
        cnt = min(chunk, n - s)
        x = mixture_vectors_torch(spec, SEED_BASE, s, cnt, dev)
        Q.qadc_pq_encode(cb8, x, out=codes8[s:s + cnt])
        Q.qadc_pq_encode(cb4, x, out=codes4[s:s + cnt])
        Q.qadc_pq_encode(cb6, x, out=codes6[s:s + cnt])
        if keep:
            raw[s:s + cnt] = x
    queries = mixture_vectors_torch(spec, SEED_QUERY, 0, args.queries, dev)
    torch.cuda.synchronize()
    t_build = time.time() - t0
    copy_calibration(torch, codes4, args.copy_calibration)

    ws4 = Q.qadc_workspace_init(torch.empty(Q.qadc_workspace_bytes(Q.QADC_WS_SEARCH, n, 16, 1, R),
                                            dtype=torch.uint8, device=dev))
    ws8 = Q.qadc_workspace_init(torch.empty(Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_F32_8BIT, n, 8, 1, R),
                                            dtype=torch.uint8, device=dev))
    luts8 = torch.empty((1, 8, 256), dtype=torch.float32, device=dev)
    idx4 = torch.empty((1, R), dtype=torch.int32, device=dev)
    dist4 = torch.empty((1, R), dtype=torch.uint8, device=dev)
    idx8 = torch.empty((1, R), dtype=torch.int32, device=dev)
    dist8 = torch.empty((1, R), dtype=torch.float32, device=dev)

    def quick(i):
        qi = i % args.queries
        Q.qadc_search(cb4, queries[qi:qi + 1], codes4, R, init, workspace=ws4, out_idx=idx4, out_dist=dist4)

    def pq8(i):
        qi = i % args.queries
        Q.qadc_build_luts(cb8, queries[qi:qi + 1], out=luts8)
        Q.qadc_scan_topk(Q.QADC_F32_8BIT, codes8, luts8, R, workspace=ws8, out_idx=idx8, out_dist=dist8)

    # the 8-bit codes again, with their 256-entry tables quantized to uint8 and saturating sums
    wsq = Q.qadc_workspace_init(torch.empty(Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_U8_8BIT, n, 8, 1, R),
                                            dtype=torch.uint8, device=dev))
    idxq = torch.empty((1, R), dtype=torch.int32, device=dev)
    distq = torch.empty((1, R), dtype=torch.uint8, device=dev)

    def pq8_u8(i):
        qi = i % args.queries
        Q.qadc_build_luts(cb8, queries[qi:qi + 1], out=luts8)
        ql, _, _, _ = Q.qadc_quantize_luts(luts8, codes8[:init], R)
        Q.qadc_scan_topk(Q.QADC_U8_8BIT, codes8, ql, R, workspace=wsq, out_idx=idxq, out_dist=distq)

    # 6-bit sub-quantizers (the paper's Conclusion): m = 16 x 64 centroids, 64-entry uint8 tables
    ws6 = Q.qadc_workspace_init(torch.empty(Q.qadc_workspace_bytes(Q.QADC_WS_SCAN_U8_6BIT, n, 16, 1, R),
                                            dtype=torch.uint8, device=dev))
    luts6 = torch.empty((1, 16, 64), dtype=torch.float32, device=dev)
    idx6 = torch.empty((1, R), dtype=torch.int32, device=dev)
    dist6 = torch.empty((1, R), dtype=torch.uint8, device=dev)

    def pq6_u8(i):
        qi = i % args.queries
        Q.qadc_build_luts(cb6, queries[qi:qi + 1], out=luts6)
        ql, _, _, _ = Q.qadc_quantize_luts(luts6, codes6[:init], R)
        Q.qadc_scan_topk(Q.QADC_U8_6BIT, codes6, ql, R, workspace=ws6, out_idx=idx6, out_dist=dist6)

    def timed(fn):
        for i in range(args.warmup):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.steps):
            fn(args.warmup + i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    ms4 = timed(quick)
    ms8 = timed(pq8)
    ms8q = timed(pq8_u8)
    ms6 = timed(pq6_u8)

    # the same comparison on batches of 256 queries (one call each): both share code reads between
    # queries (query-tiled kernels: 16 queries per LDS read for the uint8 tables, 8 queries per two
    # LDS reads for the float tables)
    nbq = min(256, args.queries)
    qb = queries[:nbq].contiguous()
    luts8b = Q.qadc_build_luts(cb8, qb)

    def timed_batch(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps

    ms4b = timed_batch(lambda: Q.qadc_search(cb4, qb, codes4, R, init))
    ms8b = timed_batch(lambda: Q.qadc_scan_topk(Q.QADC_F32_8BIT, codes8, luts8b, R))
    luts4b = Q.qadc_build_luts(cb4, qb)
    ms4fb = timed_batch(lambda: Q.qadc_scan_topk(Q.QADC_F32_4BIT, codes4, luts4b, R))
    ql8b = Q.qadc_quantize_luts(luts8b, codes8[:init], R)[0]
    ms8qb = timed_batch(lambda: Q.qadc_scan_topk(Q.QADC_U8_8BIT, codes8, ql8b, R))
    batched = {"queries": nbq, "quick_adc_ms": round(ms4b, 3), "pq8_float_ms": round(ms8b, 3),
               "pq8_uint8_tables_ms": round(ms8qb, 3),
               "float_adc_4bit_codes_ms": round(ms4fb, 3),
               "speedup_quick_adc_over_float_adc_same_codes": round(ms4fb / ms4b, 2),
               "quick_adc_gpairs_per_s": round(n * nbq / (ms4b * 1e-3) / 1e9, 1),
               "pq8_float_gpairs_per_s": round(n * nbq / (ms8b * 1e-3) / 1e9, 1),
               "speedup_quick_adc_over_pq8_float": round(ms8b / ms4b, 2)}

    roofline = kernels = None
    if not args.no_profile:
        nprof = min(args.steps, 200)
        per = {}
        for name, fn in (("quick_adc", quick), ("pq8_float", pq8), ("pq8_uint8_tables", pq8_u8),
                         ("pq6_uint8_tables", pq6_u8)):
            Q.qadc_profile_enable(True)
            for i in range(nprof):
                fn(i)
            torch.cuda.synchronize()
            per[name] = {}
            for k, which in (("scan", Q.QADC_PROF_SCAN), ("seed", Q.QADC_PROF_SEED), ("merge", Q.QADC_PROF_MERGE),
                             ("tables", Q.QADC_PROF_TABLES), ("quantize", Q.QADC_PROF_QUANTIZE),
                             ("prepare", Q.QADC_PROF_PREPARE)):
                ms, cnt = Q.qadc_profile_read(which)
                if cnt:
                    per[name][k + "_us_per_query"] = round(ms / nprof * 1e3, 2)
            Q.qadc_profile_enable(False)
        kernels = per
        us = per["quick_adc"]["scan_us_per_query"]
        ach = n * 8 / (us * 1e-6) / 1e9
        us8 = per["pq8_float"]["scan_us_per_query"]
        roofline = {"bound": "hbm", "kernel": "scan_u8_kernel", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBPS, 4),
                    "traffic": COMPARE_TRAFFIC if n == 50_000_000 else None,
                    "traffic_source": "profiles/hbm_traffic_configs_3_4_5.md (rocprofv3 --pmc FETCH_SIZE, bytes read per launch)",
                    "avg_kernel_us": us, "bytes_per_launch": n * 8, "launches_timed": nprof,
                    "pq8_float_scan_kernel": {"avg_kernel_us": us8,
                                              "achieved": round(n * 8 / (us8 * 1e-6) / 1e9, 1),
                                              "frac": round(n * 8 / (us8 * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)},
                    "pq6_uint8_scan_kernel": {"avg_kernel_us": per["pq6_uint8_tables"]["scan_us_per_query"],
                                              "bytes_per_launch": n * 12,
                                              "achieved": round(n * 12 / (per["pq6_uint8_tables"]["scan_us_per_query"] * 1e-6) / 1e9, 1),
                                              "frac": round(n * 12 / (per["pq6_uint8_tables"]["scan_us_per_query"] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}}

    acc = None
    if keep:
        nq = min(args.recall_queries, args.queries)
        qs = queries[:nq].contiguous()
        i4, _ = Q.qadc_search(cb4, qs, codes4, R, init)
        f4, _ = Q.qadc_scan_topk(Q.QADC_F32_4BIT, codes4, Q.qadc_build_luts(cb4, qs), R)
        l8 = Q.qadc_build_luts(cb8, qs)
        i8, _ = Q.qadc_scan_topk(Q.QADC_F32_8BIT, codes8, l8, R)
        i8q, _ = Q.qadc_scan_topk(Q.QADC_U8_8BIT, codes8, Q.qadc_quantize_luts(l8, codes8[:init], R)[0], R)
        i6q, _ = Q.qadc_scan_topk(Q.QADC_U8_6BIT, codes6,
                                  Q.qadc_quantize_luts(Q.qadc_build_luts(cb6, qs), codes6[:init], R)[0], R)
        best = torch.full((nq,), float("inf"), device=dev)
        arg = torch.zeros((nq,), dtype=torch.int64, device=dev)
        qq = (qs * qs).sum(1)
        for s in range(0, n, 1 << 20):
            x = raw[s:s + (1 << 20)]
            dist = qq[:, None] - 2.0 * qs @ x.T + (x * x).sum(1)[None, :]
            v, a = dist.min(1)
            upd = v < best
            best[upd] = v[upd]
            arg[upd] = a[upd] + s
        torch.cuda.synchronize()
        nn = arg.cpu().numpy()
        h = {k: v.cpu().numpy().view(np.uint32).astype(np.int64)
             for k, v in (("q", i4), ("f4", f4), ("f8", i8), ("q8", i8q), ("q6", i6q))}
        rec = {k: float(np.mean([nn[i] in h[k][i] for i in range(nq)])) for k in h}
        ov = float(np.mean([len(np.intersect1d(a, b)) / R for a, b in zip(h["q"], h["f4"])]))
        ov8 = float(np.mean([len(np.intersect1d(a, b)) / R for a, b in zip(h["q8"], h["f8"])]))
        acc = {"queries": nq, "nn_recall_at_R_quick_adc": round(rec["q"], 4),
               "nn_recall_at_R_float_adc_4bit_codes": round(rec["f4"], 4),
               "nn_recall_at_R_pq8_float": round(rec["f8"], 4),
               "nn_recall_at_R_pq8_uint8_tables": round(rec["q8"], 4),
               "nn_recall_at_R_pq6_uint8_tables_96bit": round(rec["q6"], 4),
               "overlap_at_R_quick_vs_float_adc_same_codes": round(ov, 4),
               "overlap_at_R_pq8_uint8_tables_vs_pq8_float": round(ov8, 4),
               "note": "NN-recall = exact nearest neighbour (raw vectors) among the R returned, the paper's "
                       "Recall@R; the mixture's within-component neighbours are isotropic noise, so every 64-bit "
                       "code sits near chance here -- the overlap with float ADC is the meaningful figure"}

    cpu = None
    if args.cpu_queries > 0:
        from oracle import cref
        nqc = min(256, args.queries)
        h_codes = codes4.cpu().numpy()
        ql = torch.empty((nqc, 16, 16), dtype=torch.uint8, device=dev)
        gi, gd = Q.qadc_search(cb4, queries[:nqc].contiguous(), codes4, R, init, qluts_out=ql)
        torch.cuda.synchronize()
        t0 = time.time()
        ci, cd = cref.scan_topk_u8(h_codes, ql.cpu().numpy(), R)
        dt = time.time() - t0
        cpu = {"value": round(nqc * n / dt / 1e9, 4), "unit": "Gcodes/s", "cores": cref.num_threads(),
               "kind": "oracle", "sample": "%d Quick ADC queries x %d codes, one query per thread" % (nqc, n),
               "seconds": round(dt, 2),
               "gpu_matches_oracle": bool(np.array_equal(gi.cpu().numpy().view(np.uint32), ci)
                                          and np.array_equal(gd.cpu().numpy(), cd))}

    return ({
        "metric": "G PQ codes scanned/s (Quick ADC m=16 x 4-bit, whole path per query) with the 8-bit PQ "
                  "float-table scan of the same vectors beside it",
        "value": round(n / (ms4 * 1e-3) / 1e9, 2), "unit": "Gcodes/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms4, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": "config 5: d=96 mixture, N=%d vectors as PQ m=8 x 256 (float32 tables) and as "
                   "PQ m=16 x 16 (Quick ADC, uint8 tables), 64-bit codes both, queries one at a time, R=%d, "
                   "init=%d" % (n, R, init), "n": n, "R": R, "init": init},
        "pq8_float": {"ms_per_query": round(ms8, 5), "gcodes_per_s": round(n / (ms8 * 1e-3) / 1e9, 2)},
        "pq8_uint8_tables": {"ms_per_query": round(ms8q, 5), "gcodes_per_s": round(n / (ms8q * 1e-3) / 1e9, 2),
                             "note": "the 8-bit codes scanned with their 256-entry tables quantized as in "
                                     "Section 3.3 (qadc_build_luts + qadc_quantize_luts_8bit + qadc_scan_topk "
                                     "QADC_U8_8BIT, three calls per query)"},
        "pq6_uint8_tables": {"ms_per_query": round(ms6, 5), "gcodes_per_s": round(n / (ms6 * 1e-3) / 1e9, 2),
                             "note": "the same vectors as m=16 x 6-bit codes (96 bits, four components per three "
                                     "bytes) with 64-entry uint8 tables: qadc_build_luts + qadc_quantize_luts_6bit + "
                                     "qadc_scan_topk QADC_U8_6BIT, three calls per query"},
        "speedup_quick_adc_over_pq8_float": round(ms8 / ms4, 3),
        "batches_of_256": batched,
        "roofline": roofline, "kernels": kernels, "accuracy": acc, "cpu_baseline": cpu,
        "database_build_s": round(t_build, 2)})


def run_build(args):
    """Database side: a step = one inverted index built from n raw vectors already in HBM
    (qadc_ivf_assign, qadc_ivf_group, qadc_ivf_encode, then the list in the paper's transposed layout
    and back).  Vectors: coarse centroid of a Zipf-weighted cell plus N(0, 18^2) noise."""
    import numpy as np
    import torch
    import paper_1704_07355_amd as Q
    from workloads import MixtureSpec, SEED_BASE, SEED_TRAIN, zipf_list_sizes, kmeans_init_rows
    from workloads.mixture_torch import mixture_vectors_torch

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    n, m, d = args.n, args.m, args.d
    K = args.K if args.K != 65536 else 4096
    gen = torch.Generator(device=dev)
    gen.manual_seed(SEED_BASE * 31 + 5)
    coarse = mixture_vectors_torch(MixtureSpec(d=d), SEED_TRAIN, 0, K, dev)
    sizes = zipf_list_sizes(n, K, 0.8, SEED_BASE)
    home = torch.multinomial(torch.from_numpy(sizes / sizes.sum()).to(dev), n, replacement=True, generator=gen)
    x = (coarse[home] + 18.0 * torch.randn((n, d), generator=gen, device=dev)).contiguous()
    del home
    train = 18.0 * torch.randn((20_000, d), generator=gen, device=dev)
    cb = Q.qadc_pq_train(train.contiguous(), m, 16, torch.from_numpy(kmeans_init_rows(20_000, 16)).to(dev), 10)
    ws = torch.empty((Q.qadc_ivf_group_workspace_bytes(n, K),), dtype=torch.uint8, device=dev)
    cells = torch.empty((n,), dtype=torch.int32, device=dev)
    codes = torch.empty((n, m // 2), dtype=torch.uint8, device=dev)
    packed = torch.empty((Q.qadc_packed_bytes(n, m, Q.QADC_LAYOUT_TRANSPOSED),), dtype=torch.uint8, device=dev)
    back = torch.empty_like(codes)
    names = ["assign", "group", "encode", "pack", "unpack"]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)]

    def step(timed):
        if timed:
            ev[0].record()
        Q.qadc_ivf_assign(coarse, x, out=cells)
        if timed:
            ev[1].record()
        list_off, ids = Q.qadc_ivf_group(cells, K, workspace=ws)
        if timed:
            ev[2].record()
        Q.qadc_ivf_encode(coarse, cb, x, cells, ids, out=codes)
        if timed:
            ev[3].record()
        Q.qadc_pack_codes(codes, Q.QADC_LAYOUT_TRANSPOSED, out=packed)
        if timed:
            ev[4].record()
        Q.qadc_unpack_codes(packed, n, m, Q.QADC_LAYOUT_TRANSPOSED, out=back)
        if timed:
            ev[5].record()
        return list_off, ids

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    phase = dict.fromkeys(names, 0.0)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        list_off, ids = step(True)
        torch.cuda.synchronize()
        for i, k in enumerate(names):
            phase[k] += ev[i].elapsed_time(ev[i + 1])
    wall = (time.perf_counter() - t0) / args.steps
    phase = {k: v / args.steps for k, v in phase.items()}
    assert torch.equal(back, codes)

    # the oracle builds the index of the first rows; same cells, and the same codes for those rows
    cpu = None
    if args.cpu_queries > 0:
        from oracle import qadc_oracle as O
        ns = min(n, 1500)
        xs, cs, cbs = x[:ns].cpu().numpy(), coarse.cpu().numpy(), cb.cpu().numpy()
        t1 = time.perf_counter()
        ix = O.ivf_build(xs, cs, cbs)
        secs = time.perf_counter() - t1
        want_cells = O.ivf_assign(xs, cs)
        inv = torch.empty((n,), dtype=torch.int64, device=dev)
        inv[ids.long() & 0xFFFFFFFF] = torch.arange(n, device=dev)
        mine = codes[inv[:ns]].cpu().numpy()           # code of input row i
        theirs = np.empty_like(mine)
        theirs[ix["ids"]] = ix["codes"]
        same = bool(np.array_equal(cells[:ns].cpu().numpy(), want_cells) and np.array_equal(mine, theirs))
        cpu = {"value": round(ns / secs, 1), "unit": "vectors/s", "cores": 1, "kind": "oracle",
               "sample": "first %d vectors, NumPy oracle ivf_build against K=%d cells" % (ns, K),
               "seconds": round(secs, 2), "gpu_matches_oracle": same}
    flops = 3.0 * n * K * d                       # a subtraction and a fused multiply-add per component
    out = {"metric": "vectors/s (inverted index built from raw vectors: assign + group + encode)",
           "value": round(n / ((phase["assign"] + phase["group"] + phase["encode"]) * 1e-3), 1),
           "unit": "vectors/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(wall * 1e3, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f64", "data": "synthetic",
           "config": {"workload": "index build: n=%d vectors d=%d, K=%d coarse centroids, m=%d x 4-bit residual codes"
                                  % (n, d, K, m), "n": n, "d": d, "K": K, "m": m},
           "phase_ms": {k: round(v, 3) for k, v in phase.items()},
           "roofline": {"bound": "alu", "kernel": "ivf_assign_kernel", "achieved": round(flops / (phase["assign"] * 1e-3) / 1e12, 2),
                        "peak": 78.6, "unit": "TFLOP/s", "frac": round(flops / (phase["assign"] * 1e-3) / 78.6e12, 4),
                        "traffic": None},
           "layout_gb_per_s": {"pack": round(2 * codes.numel() / (phase["pack"] * 1e-3) / 1e9, 1),
                               "unpack": round(2 * codes.numel() / (phase["unpack"] * 1e-3) / 1e9, 1)},
           "cpu_baseline": cpu}
    return out


def other_workloads(argv_args):
    """Short runs of the other workloads (configs 3, 4, 5 at their full sizes), each with the record its
    own `--workload` run prints; nested under one key of the headline line."""
    import gc
    import torch
    out = {}
    plans = (("config3_batched", "batched", dict(steps=4, warmup=1)),
             ("config4_ivf", "ivf", dict(steps=2, warmup=1)),
             ("config5_compare", "compare", dict(steps=300, warmup=20)))
    for key, workload, over in plans:
        a = argparse.Namespace(**vars(argv_args))
        a.workload = workload
        for k, v in {**WORKLOAD_DEFAULTS[workload], **over}.items():
            setattr(a, k, v)
        a.d, a.R, a.nbins, a.K, a.nprobe, a.copy_calibration, a.opq = 128, 100, 255, 65536, 64, 0, 0
        a.queries, a.recall_queries = 1000, 100
        t0 = time.time()
        try:
            rec = RUNNERS[workload](a)
            rec["wall_s"] = round(time.time() - t0, 1)
        except Exception as e:  # an extra must not take the headline with it
            rec = {"error": "%s: %s" % (type(e).__name__, e)}
        out[key] = rec
        gc.collect()
        torch.cuda.empty_cache()
    return out


RUNNERS = {"batched": run_batched, "ivf": run_ivf, "compare": run_compare, "build": run_build}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported "
              "(no collectives, no sharding in this library)" % args.gpus, file=sys.stderr)
        sys.exit(2)
    if args.workload in ("batched", "ivf", "compare", "build"):
        import paper_1704_07355_amd as Q
        Q.lib()
        print(json.dumps(RUNNERS[args.workload](args)))
        return

    import numpy as np
    import torch
    import paper_1704_07355_amd as Q
    from workloads import MixtureSpec, SEED_QUERY
    from workloads.mixture_torch import mixture_vectors_torch

    Q.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    spec = MixtureSpec(d=args.d)
    m, n, R, init = args.m, args.n, args.R, args.init
    row = m // 2

    t0 = time.time()
    n_keep = n if args.recall_queries > 0 else 0
    rot = None
    if args.opq > 0:
        cb, codes, raw, rot = build_database(Q, torch, spec, m, n * args.buffers, n_keep, dev, args.opq)
    else:
        cb, codes, raw = build_database(Q, torch, spec, m, n * args.buffers, n_keep, dev)
    queries = mixture_vectors_torch(spec, SEED_QUERY, 0, args.queries, dev)
    yrot = torch.empty((1, spec.d), dtype=torch.float32, device=dev)
    t_build = time.time() - t0
    bufs = [codes[b * n:(b + 1) * n] for b in range(args.buffers)]

    ws_bytes = Q.qadc_workspace_bytes(Q.QADC_WS_SEARCH, n, m, 1, R)
    ws = Q.qadc_workspace_init(torch.empty(ws_bytes, dtype=torch.uint8, device=dev))
    luts = torch.empty((1, m, 16), dtype=torch.float32, device=dev)
    out_idx = torch.empty((1, R), dtype=torch.int32, device=dev)
    out_dist = torch.empty((1, R), dtype=torch.uint8, device=dev)

    def step(i):
        qi = i % args.queries
        buf = bufs[i % args.buffers]
        if args.separate_calls:
            Q.qadc_build_luts(cb, queries[qi:qi + 1], out=luts)
            ql, _, _, _ = Q.qadc_quantize_luts(luts, buf[:init], R, args.nbins)
            Q.qadc_scan_topk(Q.QADC_U8_4BIT, buf, ql, R, args.nbins, workspace=ws, out_idx=out_idx, out_dist=out_dist)
        elif rot is not None:
            Q.qadc_rotate(rot, queries[qi:qi + 1], out=yrot)
            Q.qadc_search(cb, yrot, buf, R, init, args.nbins, workspace=ws, out_idx=out_idx, out_dist=out_dist)
        else:
            Q.qadc_search(cb, queries[qi:qi + 1], buf, R, init, args.nbins, workspace=ws, out_idx=out_idx,
                          out_dist=out_dist)

    if args.copy_calibration > 0:
        dst = torch.empty_like(bufs[0])
        for i in range(args.copy_calibration):
            dst.copy_(bufs[i % args.buffers])  # reads n*row bytes, writes n*row bytes
        torch.cuda.synchronize()
        del dst

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

    # The same steps with queries in flight on several streams (independent queries, one call each,
    # a workspace per stream): the small kernels of one query overlap the scan of another.
    multi = None
    if args.streams > 1 and not args.separate_calls and rot is None:
        ns = args.streams
        streams = [torch.cuda.Stream(device=dev) for _ in range(ns)]
        wss = [Q.qadc_workspace_init(torch.empty(ws_bytes, dtype=torch.uint8, device=dev)) for _ in range(ns)]
        oi = [torch.empty((1, R), dtype=torch.int32, device=dev) for _ in range(ns)]
        od = [torch.empty((1, R), dtype=torch.uint8, device=dev) for _ in range(ns)]
        torch.cuda.synchronize()

        def mstep(i):
            k = i % ns
            with torch.cuda.stream(streams[k]):
                Q.qadc_search(cb, queries[i % args.queries:i % args.queries + 1], bufs[i % args.buffers], R, init,
                              args.nbins, workspace=wss[k], out_idx=oi[k], out_dist=od[k])

        for i in range(args.warmup):
            mstep(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            mstep(args.warmup + i)
        torch.cuda.synchronize()
        ms_multi = (time.perf_counter() - t0) * 1e3 / args.steps
        multi = {"streams": ns, "ms_per_step": round(ms_multi, 5),
                 "gcodes_per_s": round(n / (ms_multi * 1e-3) / 1e9, 2),
                 "note": "same calls, queries dealt round-robin to the streams; host wall clock"}

    # Per-kernel durations (HIP events attached to each dispatch by the library), same launch
    # configuration, same buffer rotation.
    roofline = None
    kernels = None
    if not args.no_profile:
        nprof = min(args.steps, 300)
        Q.qadc_profile_enable(True)
        for i in range(nprof):
            step(args.warmup + i)
        torch.cuda.synchronize()
        us = {}
        for name, which in (("scan", Q.QADC_PROF_SCAN), ("seed", Q.QADC_PROF_SEED),
                            ("merge", Q.QADC_PROF_MERGE), ("tables", Q.QADC_PROF_TABLES),
                            ("quantize", Q.QADC_PROF_QUANTIZE), ("prepare", Q.QADC_PROF_PREPARE),
                            ("rotate", Q.QADC_PROF_ROTATE)):
            ms, cnt = Q.qadc_profile_read(which)
            us[name] = (ms / max(1, cnt) * 1e3, cnt)
        Q.qadc_profile_enable(False)
        # second pass, reported beside the first: the scan kernel alone carries events, its neighbours
        # in the stream are launched exactly as in the timed region (rocprofv3 times every kernel,
        # as the first pass does, so the roofline figure is the first pass's)
        Q.qadc_profile_only(Q.QADC_PROF_SCAN)
        for i in range(nprof):
            step(args.warmup + i)
        torch.cuda.synchronize()
        ms, cnt = Q.qadc_profile_read(Q.QADC_PROF_SCAN)
        Q.qadc_profile_enable(False)
        scan_alone_us = ms / max(1, cnt) * 1e3
        avg_us, launches = us["scan"]
        achieved = n * row / (avg_us * 1e-6) / 1e9
        tr = SCAN_TRAFFIC.get((n, m))
        roofline = {"bound": "hbm", "kernel": "scan_u8_kernel", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                    "traffic": int(tr[0] + tr[1]) if tr else None,
                    "traffic_source": "profiles/scan_u8_config2_hbm_traffic.md (rocprofv3 --pmc, bytes per "
                                      "launch, read %d + written %d)" % (tr[0], tr[1]) if tr else None,
                    "avg_kernel_us": round(avg_us, 2),
                    "bytes_per_launch": n * row, "launches_timed": launches}
        kernels = {k + "_kernel_us": round(v[0], 2) for k, v in us.items() if v[1]}
        kernels["scan_kernel_us_when_only_it_is_timed"] = round(scan_alone_us, 2)
        # the same scan on ONE buffer every query: 80 MB stay in the 256 MB last-level cache
        Q.qadc_profile_enable(True)
        for i in range(100):
            Q.qadc_search(cb, queries[i % args.queries:i % args.queries + 1], bufs[0], R, init, args.nbins,
                          workspace=ws, out_idx=out_idx, out_dist=out_dist)
        torch.cuda.synchronize()
        ms, cnt = Q.qadc_profile_read(Q.QADC_PROF_SCAN)
        Q.qadc_profile_enable(False)
        kernels["scan_kernel_us_same_buffer_every_query"] = round(ms / max(1, cnt) * 1e3, 2)

    acc = None
    if args.recall_queries > 0:
        acc = accuracy(Q, torch, np, cb, bufs[0], raw, queries[:args.recall_queries].contiguous(), R, init, rot, args.nbins)
        acc["note"] = ("overlap = |top-R(Quick ADC) & top-R(float ADC, same codes)| / R; NN-recall = exact "
                       "nearest neighbour (raw vectors) among the R returned; first buffer only")

    # CPU oracle (plain C twin, one query per thread) on a bounded sample: same codes, same tables.
    cpu = None
    if args.cpu_queries > 0:
        from oracle import cref
        nqc = args.cpu_queries
        h_codes = bufs[0].cpu().numpy()
        cq = mixture_vectors_torch(spec, SEED_QUERY, 0, nqc, dev)
        l = Q.qadc_build_luts(cb, Q.qadc_rotate(rot, cq) if rot is not None else cq)
        ql, _, _, _ = Q.qadc_quantize_luts(l, bufs[0][:init], R, args.nbins)
        gi, gd = Q.qadc_scan_topk(Q.QADC_U8_4BIT, bufs[0], ql, R, args.nbins)
        torch.cuda.synchronize()
        h_ql = ql.cpu().numpy()
        t0 = time.time()
        ci, cd = cref.scan_topk_u8(h_codes, h_ql, R, args.nbins)
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
        "config": {"workload": "%s: single-query scan, d=%d mixture, PQ m=%d x 4-bit (10 k-means "
                   "iterations on 20k vectors), N=%d codes contiguous, queries one at a time, R=%d, "
                   "init=%d, %d rotating code buffers"
                   % ("config 2" if (args.d, m, n) == (128, 16, 10_000_000) else "config-2-shaped", args.d, m, n, R,
                      init, args.buffers),
                   "n": n, "m": m, "R": R, "init": init, "nbins": args.nbins, "buffers": args.buffers,
                   "entry": "build_luts+quantize_luts+scan_topk" if args.separate_calls else
                   ("qadc_rotate+qadc_search (optimized product quantizer, %d rounds)" % args.opq if rot is not None
                    else "qadc_search")},
        "hbm_gbps_whole_path": round(n * row / (ms_per_step * 1e-3) / 1e9, 1),
        "pct_hbm_peak_whole_path": round(100 * n * row / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2),
        "multi_stream": multi,
        "roofline": roofline, "kernels": kernels, "accuracy": acc, "cpu_baseline": cpu,
        "database_build_s": round(t_build, 2),
    }
    if roofline is not None:
        # the same bytes over the whole path of a query (every launch and the gaps between them)
        roofline["whole_path"] = {"achieved": rec["hbm_gbps_whole_path"], "frac": round(rec["hbm_gbps_whole_path"] / HBM_PEAK_GBPS, 4),
                                  "us_per_query": round(ms_per_step * 1e3, 2)}
    if not args.no_extras and (args.d, m, n) == (128, 16, 10_000_000) and not args.separate_calls and rot is None:
        del codes, bufs, raw
        rec["other_workloads"] = other_workloads(args)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
