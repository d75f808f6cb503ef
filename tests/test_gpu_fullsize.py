"""Parity at the benchmark's full size (1M x 128, 10,000 queries, the launch configuration
bench.py times), on sampled outputs the CPU oracle can compute one by one, plus the
integer stages in full."""
import numpy as np
import pytest

import oracle
from paper_2308_15136_amd import datagen

pytestmark = pytest.mark.gpu


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def test_large_batch_workload_at_full_size():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2308_15136_amd as cagra
    cagra.load_library()
    w = datagen.workload("sift1m")
    N, dim = w.base.shape
    d, d_init = w.degree, w.init_degree
    print(f"case fullsize N={N} dim={dim} d={d}", flush=True)
    base = torch.from_numpy(w.base).cuda()
    queries = torch.from_numpy(w.queries).cuda()

    # initial k-NN graph: sampled rows against the oracle's brute force
    knn = cagra.exact_search(base, base, d_init, w.metric, exclude_self=True, return_dists=False)
    knn_np = _u32(knn)
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(N, size=96, replace=False)).astype(np.int64)
    print("  knn rows", flush=True)
    np.testing.assert_array_equal(knn_np[rows], oracle.knn_graph(w.base, d_init, w.metric, rows=rows))
    assert knn_np.max() < N and not np.any(knn_np == np.arange(N, dtype=np.uint32)[:, None])

    # optimisation: prune on sampled nodes, reversed graph and merge in full
    graph, pruned, rev, rlen = cagra.optimize(knn, d, return_stages=True)
    pruned_np, rev_np, rlen_np, graph_np = _u32(pruned), _u32(rev), _u32(rlen), _u32(graph)
    rows = np.sort(rng.choice(N, size=3000, replace=False)).astype(np.int64)
    print("  prune rows", flush=True)
    cnt = oracle.detour_count(knn_np, rows=rows)
    np.testing.assert_array_equal(pruned_np[rows], oracle.prune(knn_np[rows], cnt, d))
    print("  reverse + merge", flush=True)
    o_rev, o_len = oracle.reverse(pruned_np)
    np.testing.assert_array_equal(rlen_np, o_len)
    np.testing.assert_array_equal(rev_np, o_rev)
    np.testing.assert_array_equal(graph_np, oracle.merge(pruned_np, o_rev, o_len))
    # the one-call build gives the same graph
    np.testing.assert_array_equal(_u32(cagra.build(base, d, d_init, w.metric)), graph_np)

    # search: whole batch on the GPU, a sample of it on the oracle (integer data: bit-exact)
    print("  search", flush=True)
    # (search_width, itopk): the point bench.py times (320 candidates per pass, taken in chunks of 256), two of
    # its short-list points (448 and 512 candidates), the best with at most 256 candidates, the one-parent search
    for width, itopk in ((5, 32), (7, 16), (8, 10), (4, 48), (1, 128)):
        print(f"    search_width {width} itopk {itopk}", flush=True)
        opts = cagra.SearchOptions(seed=20230815, mode=1)
        ids, dists, st = cagra.search(graph, base, queries, w.k, itopk, width, w.metric, opts, return_stats=True)
        ids_np, d_np, st_np = _u32(ids), dists.cpu().numpy(), _u32(st)
        assert not np.any(st_np[:, 3] & 2)
        sample = np.sort(rng.choice(w.queries.shape[0], size=1500, replace=False))
        # the seed generator is keyed by the query's index in the batch, so the oracle gets the
        # batch prefix up to the last sampled query
        upto = int(sample.max()) + 1
        o_ids, o_d, o_st = oracle.search(graph_np, w.base, w.queries[:upto], w.k, itopk, width, w.metric,
                                         seed=20230815, return_stats=True)
        np.testing.assert_array_equal(ids_np[sample], o_ids[sample])
        np.testing.assert_array_equal(d_np[sample], o_d[sample])
        np.testing.assert_array_equal(st_np[sample, :2], o_st[sample, :2])
        # properties that hold for every query of the batch
        assert ids_np.max() < N
        assert np.all(np.diff(d_np, axis=1) >= 0)
        srt = np.sort(ids_np, axis=1)
        assert np.all(srt[:, 1:] != srt[:, :-1])
        # the same rows stored as uint8 / fp16 hold the same integers: same answer, bit for bit
        for code in (cagra.U8, cagra.F16):
            n_ids, n_d = cagra.search(graph, cagra.convert_dataset(base, code), queries, w.k, itopk, width,
                                      w.metric, opts)
            assert torch.equal(n_ids, ids) and torch.equal(n_d, dists)


@pytest.mark.parametrize("name,cases", [
    ("deep1m", ((10, 128, 1), (100, 256, 1), (10, 64, 4), (10, 32, 16), (10, 64, 8), (100, 128, 4))),   # 1M x 96 unit-norm rows, L2, degree 32; the last two cases: bench.py's timed points
    ("glove200", ((10, 256, 1), (10, 128, 2), (10, 64, 8), (10, 256, 16))),   # 1,183,514 x 200 unit-norm rows, inner product; the last case: bench.py's timed point
])
def test_float_workloads_at_full_size(name, cases):
    """The lower-dimensional and the inner-product configuration at their full sizes: whole batch on
    the GPU, a sample of the queries on the oracle, the stated bars for floating-point data
    (distances within 1e-5 relative, id agreement >= 99.5 %, recall within 0.003)."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2308_15136_amd as cagra
    cagra.load_library()
    w = datagen.workload(name)
    N, dim = w.base.shape
    print(f"case fullsize {name} N={N} dim={dim} d={w.degree}", flush=True)
    base = torch.from_numpy(w.base).cuda()
    queries = torch.from_numpy(w.queries).cuda()
    graph = cagra.build(base, w.degree, w.init_degree, w.metric)
    graph_np = _u32(graph)
    assert graph_np.max() < N
    # the initial lists behind the graph: sampled rows of the exhaustive search against the oracle
    rng = np.random.default_rng(1)
    rows = np.sort(rng.choice(N, size=48, replace=False)).astype(np.int64)
    knn_rows = torch.cat([cagra.exact_search(base, base[int(r):int(r) + 1], w.init_degree, w.metric, exclude_self=True,
                                             self_offset=int(r), return_dists=False) for r in rows])
    np.testing.assert_array_equal(_u32(knn_rows), oracle.knn_graph(w.base, w.init_degree, w.metric, rows=rows))
    nq = 1200                                    # the oracle runs the first nq queries of the batch
    gt = _u32(cagra.exact_search(base, queries[:nq], 100, w.metric, return_dists=False))
    for k, itopk, width in cases:
        print(f"    k {k} itopk {itopk} search_width {width}", flush=True)
        opts = cagra.SearchOptions(seed=7, mode=1)
        ids, dists, st = cagra.search(graph, base, queries, k, itopk, width, w.metric, opts, return_stats=True)
        ids_np, d_np = _u32(ids), dists.cpu().numpy()
        o_ids, o_d = oracle.search(graph_np, w.base, w.queries[:nq], k, itopk, width, w.metric, seed=7)
        agree = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids_np[:nq], o_ids)) / float(o_ids.size)
        assert agree >= 0.995, f"id agreement {agree}"
        same = ids_np[:nq] == o_ids
        denom = np.maximum(np.abs(o_d), 1.0 if w.metric == oracle.IP else 0.0)
        rel = np.abs(d_np[:nq] - o_d)[same] / np.maximum(denom[same], 1e-30)
        assert rel.max() <= 1e-5, f"distance error {rel.max()}"
        r_gpu, r_ora = oracle.recall(ids_np[:nq], gt[:, :k]), oracle.recall(o_ids, gt[:, :k])
        print(f"      id agreement {agree:.5f}  max rel dist err {rel.max():.2e}  recall gpu {r_gpu:.4f} oracle {r_ora:.4f}",
              flush=True)
        assert abs(r_gpu - r_ora) <= 0.003
        # every query of the batch: sorted, unique, valid ids
        valid = ids_np != oracle.INVALID_ID
        assert np.all(ids_np[valid] < N) and np.all(np.diff(d_np, axis=1) >= 0)
        srt = np.sort(ids_np, axis=1)
        assert np.all((srt[:, 1:] != srt[:, :-1]) | (srt[:, 1:] == oracle.INVALID_ID))
        assert not np.any(_u32(st)[:, 3] & 2)


def test_small_batch_workload_at_full_size():
    """The 10M x 96 configuration (Table I, DEEP-10M shape; Sec. IV-C.2): graph stages on sampled rows,
    the single mode on 1,000 queries at the floating-point bars, the multi mode (device-memory visited
    table) with 8 and 32 workers at batch sizes 1, 10, 100 and 1,000, and the same searches over rows
    padded to a stride of 128 floats, so that row offsets pass 2^32 bytes."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2308_15136_amd as cagra
    cagra.load_library()
    w = datagen.workload("deep10m")
    N, dim = w.base.shape
    d, d_init, k = w.degree, w.init_degree, w.k
    print(f"case fullsize deep10m N={N} dim={dim} d={d}", flush=True)
    base = torch.from_numpy(w.base).cuda()
    queries = torch.from_numpy(w.queries).cuda()
    nq = queries.shape[0]

    # initial k-NN graph in slices of rows (the filtered exhaustive search), so that the long step reports progress
    knn = torch.empty((N, d_init), dtype=torch.int32, device="cuda")
    redone = torch.zeros(1, dtype=torch.int32, device="cuda")
    step = 1_000_000
    for lo in range(0, N, step):
        hi = min(N, lo + step)
        knn[lo:hi] = cagra.exact_search(base, base[lo:hi], d_init, w.metric, exclude_self=True, self_offset=lo,
                                        return_dists=False, blocks_redone=redone)
        torch.cuda.synchronize()
        print(f"  k-NN graph rows {hi}/{N}, blocks redone by the plain kernels so far: {int(redone.item())}", flush=True)
    knn_np = _u32(knn)
    rng = np.random.default_rng(4)
    rows = np.sort(rng.choice(N, size=48, replace=False)).astype(np.int64)
    print("  knn rows against the oracle", flush=True)
    np.testing.assert_array_equal(knn_np[rows], oracle.knn_graph(w.base, d_init, w.metric, rows=rows))

    graph, pruned, rev, rlen = cagra.optimize(knn, d, return_stages=True)
    graph_np, pruned_np = _u32(graph), _u32(pruned)
    rows = np.sort(rng.choice(N, size=2000, replace=False)).astype(np.int64)
    print("  prune rows against the oracle", flush=True)
    np.testing.assert_array_equal(pruned_np[rows], oracle.prune(knn_np[rows], oracle.detour_count(knn_np, rows=rows), d))
    # merged rows: d distinct ids below N, no self edge, first entry = nearest neighbour
    assert graph_np.max() < N and not np.any(graph_np == np.arange(N, dtype=np.uint32)[:, None])
    np.testing.assert_array_equal(graph_np[:, 0], knn_np[:, 0])
    srt = np.sort(graph_np[rows], axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1])
    del knn, pruned, rev, rlen, knn_np, pruned_np

    # the same rows with a stride of 128 floats: 10M x 512 bytes = 5.12 GB, offsets beyond 2^32
    padded = torch.zeros((N, 128), dtype=torch.float32, device="cuda")
    padded[:, :dim] = base
    base_ld = padded[:, :dim]
    assert base_ld.stride(0) == 128 and N * 128 * 4 > 2**32

    gt = _u32(cagra.exact_search(base, queries, k, w.metric, return_dists=False))

    def bars(ids_np, d_np, o_ids, o_d, what):
        agree = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids_np, o_ids)) / float(o_ids.size)
        same = ids_np == o_ids
        rel = np.abs(d_np - o_d)[same] / np.maximum(np.abs(o_d[same]), 1e-30)
        r_gpu, r_ora = oracle.recall(ids_np, gt[:len(ids_np)]), oracle.recall(o_ids, gt[:len(ids_np)])
        print(f"      {what}: id agreement {agree:.5f}  max rel dist err {rel.max():.2e}  recall gpu {r_gpu:.4f} oracle {r_ora:.4f}",
              flush=True)
        return agree, rel.max(), r_gpu, r_ora

    def invariants(ids_np, d_np):
        valid = ids_np != oracle.INVALID_ID
        assert np.all(ids_np[valid] < N) and np.all(np.diff(d_np, axis=1) >= 0)
        s = np.sort(ids_np, axis=1)
        assert np.all((s[:, 1:] != s[:, :-1]) | (s[:, 1:] == oracle.INVALID_ID))
        for b in range(0, ids_np.shape[0], 7):          # distances belong to the ids
            for t in range(ids_np.shape[1]):
                if valid[b, t]:
                    ref = oracle.distance(w.queries[b], w.base[ids_np[b, t]], w.metric)
                    assert abs(d_np[b, t] - ref) <= 1e-5 * abs(ref)

    print("  single mode", flush=True)
    for itopk, width in ((64, 1), (128, 4), (64, 16), (128, 2)):     # the last: bench.py's timed point at batch 10,000
        opts = cagra.SearchOptions(seed=7, mode=1)
        ids, dists, st = cagra.search(graph, base, queries, k, itopk, width, w.metric, opts, return_stats=True)
        ids_np, d_np = _u32(ids), dists.cpu().numpy()
        o_ids, o_d = oracle.search(graph_np, w.base, w.queries, k, itopk, width, w.metric, seed=7)
        agree, rel, r_gpu, r_ora = bars(ids_np, d_np, o_ids, o_d, f"itopk {itopk} search_width {width}")
        assert agree >= 0.995 and rel <= 1e-5 and abs(r_gpu - r_ora) <= 0.003
        invariants(ids_np, d_np)
        assert not np.any(_u32(st)[:, 3] & 2)
        p_ids, p_d = cagra.search(graph, base_ld, queries, k, itopk, width, w.metric, opts)
        assert torch.equal(p_ids, ids) and torch.equal(p_d, dists), "padded rows give another answer"

    print("  multi mode", flush=True)
    for workers in (8, 32):
        itopk = 32 * workers
        opts = cagra.SearchOptions(seed=7, mode=2, wg_per_query=workers)
        plan = cagra.describe(d, dim, nq, k, itopk, 1, opts)
        local, cap = plan["itopk_local"], plan["max_iterations"]
        assert plan["mode"] == 2 and plan["wg_per_query"] == workers and local == 32
        o_ids, o_d = oracle.search_multi(graph_np, w.base, w.queries, k, local, workers, w.metric, seed=7,
                                         max_iterations=cap)
        for data, what in ((base, "rows dense"), (base_ld, "rows padded")):
            ids, dists, st = cagra.search(graph, data, queries, k, itopk, 1, w.metric, opts, return_stats=True)
            ids_np, d_np, st_np = _u32(ids), dists.cpu().numpy(), _u32(st)
            agree, rel, r_gpu, r_ora = bars(ids_np, d_np, o_ids, o_d, f"W {workers} {what}")
            # the workers interleave freely on the GPU and in lock step in the oracle: recall is the bar,
            # id agreement is reported
            assert abs(r_gpu - r_ora) <= 0.003 and rel <= 1e-5
            invariants(ids_np, d_np)
            assert not np.any(st_np[:, 3] & 2), "visited table overflowed"
            assert st_np[:, 0].max() <= cap
        # the batch sizes the configuration names; a query's seeds depend on its index in the call
        for nb in (1, 10, 100):
            hits = 0
            for lo in range(0, 200, nb):
                ids, dists = cagra.search(graph, base, queries[lo:lo + nb], k, itopk, 1, w.metric, opts)
                ids_np, d_np = _u32(ids), dists.cpu().numpy()
                assert np.all(np.diff(d_np, axis=1) >= 0) and ids_np.max() < N
                hits += sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids_np, gt[lo:lo + nb]))
            print(f"      W {workers} batch {nb}: recall over 200 queries {hits / (200.0 * k):.4f}", flush=True)
            assert hits / (200.0 * k) >= oracle.recall(o_ids[:200], gt[:200]) - 0.02
