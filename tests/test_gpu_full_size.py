"""GPU parity at the full sizes of the benchmark configurations, through the entry points and launch
shapes bench.py times.  The plain-C oracle twin scans the same codes on the host (it needs a few
seconds per configuration), so the comparison is complete, not sampled, for the queries checked."""

import numpy as np
import pytest

from gpu_common import idx_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    assert torch.cuda.is_available()
    import paper_1704_07355_amd as Q
    Q.lib()
    import bench
    from oracle import qadc_oracle as O, cref
    return Q, torch, bench, O, cref


def test_config2_single_query_search_10m_codes(env):
    """N = 10 M, m = 16: qadc_search one query at a time (fused prepare kernel, sampled bound)."""
    Q, torch, bench, O, cref = env
    from workloads import MixtureSpec, SEED_QUERY
    from workloads.mixture_torch import mixture_vectors_torch
    dev = torch.device("cuda:0")
    n, m, R, init, nq = 10_000_000, 16, 100, 200, 12
    cb, codes, _ = bench.build_database(Q, torch, MixtureSpec(d=128), m, n, 0, dev)
    queries = mixture_vectors_torch(MixtureSpec(d=128), SEED_QUERY, 0, nq, dev)
    ws = Q.qadc_workspace_init(torch.empty(Q.qadc_workspace_bytes(Q.QADC_WS_SEARCH, n, m, 1, R),
                                           dtype=torch.uint8, device=dev))
    ql = torch.empty((nq, m, 16), dtype=torch.uint8, device=dev)
    gi = torch.empty((nq, R), dtype=torch.int32, device=dev)
    gd = torch.empty((nq, R), dtype=torch.uint8, device=dev)
    for iq in range(nq):
        Q.qadc_search(cb, queries[iq:iq + 1], codes, R, init, workspace=ws, out_idx=gi[iq:iq + 1],
                      out_dist=gd[iq:iq + 1], qluts_out=ql[iq:iq + 1])
    torch.cuda.synchronize()
    h_codes, h_ql = codes.cpu().numpy(), ql.cpu().numpy()
    wi, wd = cref.scan_topk_u8(h_codes, h_ql, R)
    assert np.array_equal(idx_np(gi), wi)
    assert np.array_equal(gd.cpu().numpy(), wd)
    # tables and quantizer of the same calls against the oracle's (entries within one step)
    h_cb, h_q = cb.cpu().numpy(), queries.cpu().numpy()
    for iq in (0, nq - 1):
        want = O.quick_adc_tables(h_cb, h_q[iq], h_codes[:init], init, R)["qlut"]
        assert np.abs(h_ql[iq].astype(int) - want.astype(int)).max() <= 1


def test_config3_query_batch_100m_codes(env):
    """N = 100 M, m = 32: a 256-query batch through qadc_search (matrix-core batched scan); 12 of
    its queries are rescanned in full by the oracle."""
    Q, torch, bench, O, cref = env
    from workloads import MixtureSpec, SEED_QUERY
    from workloads.mixture_torch import mixture_vectors_torch
    dev = torch.device("cuda:0")
    n, m, R, init, nb = 100_000_000, 32, 100, 1000, 256
    cb, codes, _ = bench.build_database(Q, torch, MixtureSpec(d=128), m, n, 0, dev)
    queries = mixture_vectors_torch(MixtureSpec(d=128), SEED_QUERY, 0, nb, dev)
    ql = torch.empty((nb, m, 16), dtype=torch.uint8, device=dev)
    gi, gd = Q.qadc_search(cb, queries, codes, R, init, qluts_out=ql)
    torch.cuda.synchronize()
    pick = np.array([0, 1, 7, 8, 63, 64, 100, 127, 128, 200, 254, 255])
    h_codes = codes.cpu().numpy()
    wi, wd = cref.scan_topk_u8(h_codes, ql.cpu().numpy()[pick], R)
    assert np.array_equal(idx_np(gi)[pick], wi)
    assert np.array_equal(gd.cpu().numpy()[pick], wd)
    # the same queries in tiles of 64 and of 32 (other launch shapes: 32 queries per wavefront, more
    # and shorter chunks) give the same rows
    for t0, t1 in ((0, 64), (64, 96)):
        ti, td = Q.qadc_search(cb, queries[t0:t1], codes, R, init)
        torch.cuda.synchronize()
        assert np.array_equal(idx_np(ti), idx_np(gi)[t0:t1])
        assert np.array_equal(td.cpu().numpy(), gd.cpu().numpy()[t0:t1])


def test_config5_float_and_quantized_scans_50m_codes(env):
    """N = 50 M, d = 96: 8-bit PQ with float tables (Alg. 1) and Quick ADC on the same vectors."""
    Q, torch, bench, O, cref = env
    from workloads import MixtureSpec, SEED_QUERY, SEED_TRAIN, SEED_BASE, kmeans_init_rows
    from workloads.mixture_torch import mixture_vectors_torch, BLOCK
    dev = torch.device("cuda:0")
    spec = MixtureSpec(d=96)
    n, R, init, nq = 50_000_000, 100, 200, 6
    train = mixture_vectors_torch(spec, SEED_TRAIN, 0, 20_000, dev)
    cb8 = Q.qadc_pq_train(train, 8, 256, torch.from_numpy(kmeans_init_rows(20_000, 256)).to(dev), 10)
    cb4 = Q.qadc_pq_train(train, 16, 16, torch.from_numpy(kmeans_init_rows(20_000, 16)).to(dev), 10)
    codes8 = torch.empty((n, 8), dtype=torch.uint8, device=dev)
    codes4 = torch.empty((n, 8), dtype=torch.uint8, device=dev)
    for s in range(0, n, 4 * BLOCK):
        cnt = min(4 * BLOCK, n - s)
        x = mixture_vectors_torch(spec, SEED_BASE, s, cnt, dev)
        Q.qadc_pq_encode(cb8, x, out=codes8[s:s + cnt])
        Q.qadc_pq_encode(cb4, x, out=codes4[s:s + cnt])
    queries = mixture_vectors_torch(spec, SEED_QUERY, 0, nq, dev)
    luts8 = Q.qadc_build_luts(cb8, queries)
    fi = torch.empty((nq, R), dtype=torch.int32, device=dev)
    fd = torch.empty((nq, R), dtype=torch.float32, device=dev)
    ql = torch.empty((nq, 16, 16), dtype=torch.uint8, device=dev)
    gi = torch.empty((nq, R), dtype=torch.int32, device=dev)
    gd = torch.empty((nq, R), dtype=torch.uint8, device=dev)
    for iq in range(nq):  # one query at a time, as the benchmark issues them
        Q.qadc_scan_topk(Q.QADC_F32_8BIT, codes8, luts8[iq:iq + 1], R, out_idx=fi[iq:iq + 1],
                         out_dist=fd[iq:iq + 1])
        Q.qadc_search(cb4, queries[iq:iq + 1], codes4, R, init, out_idx=gi[iq:iq + 1],
                      out_dist=gd[iq:iq + 1], qluts_out=ql[iq:iq + 1])
    torch.cuda.synchronize()
    wi, wd = cref.scan_topk_f32(codes8.cpu().numpy(), luts8.cpu().numpy(), R)
    assert np.array_equal(idx_np(fi), wi)
    assert np.array_equal(fd.cpu().numpy().view(np.uint32), wd.view(np.uint32))
    wi, wd = cref.scan_topk_u8(codes4.cpu().numpy(), ql.cpu().numpy(), R)
    assert np.array_equal(idx_np(gi), wi)
    assert np.array_equal(gd.cpu().numpy(), wd)


@pytest.mark.parametrize("n", [100_000_000, 1_000_000_000])
def test_config4_ivf_search(env, n):
    """Inverted index of the benchmark's shape (K = 65536, Zipf(0.8) lists, m = 32, nprobe = 64) at
    N = 1e8 and at the full N = 1e9: a 4096-query batch, the benchmark's; for a sample of its queries the oracle
    rescans every probed list with the GPU's cells and tables and selects by (sum, storage
    position); vector ids are a hash of the position."""
    Q, torch, bench, O, cref = env
    dev = torch.device("cuda:0")
    K, m, R, init, nprobe, nb = 65536, 32, 100, 1000, 64, 4096
    index, sizes, queries = bench.build_ivf_index(Q, torch, np, n, K, m, nb, dev)
    coarse, list_off, codes, _, cb = index.tensors
    # vector ids that are not the storage positions: id(p) = (p * 2654435761 + 12345) mod 2^32
    vid = torch.arange(n, dtype=torch.int64, device=dev)
    vid.mul_(2654435761).add_(12345).bitwise_and_(0xFFFFFFFF)
    vid = torch.where(vid >= 2 ** 31, vid - 2 ** 32, vid).to(torch.int32)   # the same 32 bits, as int32
    index = Q.IvfIndex(coarse, list_off, codes, vid, cb)
    ids, dist, probes, qluts = Q.qadc_ivf_search(index, queries, nprobe, R, init, debug=True)
    torch.cuda.synchronize()
    h_off = list_off.cpu().numpy()
    h_probes = probes.cpu().numpy()
    for iq in (0, 1, 7, 63, 64, 255, 256, 1000, 2047, 2048, 3333, 4095):
        h_ql = qluts[iq].cpu().numpy()
        sums, pos = [], []
        for t, c in enumerate(h_probes[iq]):
            lo, hi = int(h_off[c]), int(h_off[c + 1])
            if hi > lo:
                sums.append(O.scan_saturating(h_ql[t], codes[lo:hi].cpu().numpy()))
                pos.append(np.arange(lo, hi, dtype=np.int64))
        sums, pos = np.concatenate(sums), np.concatenate(pos)
        order = np.argsort(pos, kind="stable")  # storage position decides ties
        sel, d = O.top_r(sums[order], R, pad_dist=255)
        want_ids = (pos[order][sel] * 2654435761 + 12345) & 0xFFFFFFFF
        assert np.array_equal(idx_np(ids)[iq].astype(np.int64), want_ids), iq
        assert np.array_equal(dist[iq].cpu().numpy(), d), iq
    # the float side at this size: the oracle's own cells, tables and quantizer for a few queries
    h_coarse, h_cb = coarse.cpu().numpy(), cb.cpu().numpy()
    for iq in (0, 1000, 4095):
        y = queries[iq].cpu().numpy()
        want_probes = O.ivf_probes(y, h_coarse, nprobe)
        if not np.array_equal(h_probes[iq], want_probes):   # float32 against float64 distances: near-ties may swap
            dq = O.sq_l2(y[None], h_coarse)[0]
            np.testing.assert_allclose(dq[h_probes[iq]], dq[want_probes], rtol=1e-5)
            continue
        cells = h_probes[iq]
        lens = (h_off[cells + 1] - h_off[cells]).astype(np.int64)
        sub_off = np.zeros(len(cells) + 1, dtype=np.int64)
        np.cumsum(lens, out=sub_off[1:])
        sub_codes = torch.cat([codes[h_off[c]:h_off[c + 1]] for c in cells]).cpu().numpy()
        sub = dict(list_off=sub_off, codes=sub_codes, ids=np.zeros(int(sub_off[-1]), dtype=np.uint32))
        full = O.ivf_quick_adc_search(sub, h_coarse[cells], h_cb, y, nprobe, init, R, probes=np.arange(nprobe))
        assert np.abs(qluts[iq].cpu().numpy().astype(int) - full["qluts"].astype(int)).max() <= 1, iq
