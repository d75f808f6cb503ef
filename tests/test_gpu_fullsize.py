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
    # (search_width, itopk): the point bench.py times (4, 48), and the one-parent search at the same recall
    for width, itopk in ((4, 48), (1, 128)):
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
