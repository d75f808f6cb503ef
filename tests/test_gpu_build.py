"""GPU parity of the build side (exhaustive search, k-NN graph, optimisation, whole build)
against the CPU oracle, through the C ABI.  Everything here is integer or decided by a
fixed-order fp32 accumulation, so the bar is bit-exact."""
import numpy as np
import pytest

import oracle
from paper_2308_15136_amd import datagen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def cagra():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2308_15136_amd as m
    m.load_library()
    return m


def _dev(a):
    import torch
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("name,n,nq,k", [
    ("tiny", 10_000, 100, 10),
    ("tiny", 10_000, 37, 1),
    ("deep1m", 5_003, 129, 100),       # N and B off the tile size
    ("glove200", 3_000, 64, 512),      # inner product, largest k
    ("sift1m", 4_097, 50, 64),
])
def test_exact_search_bit_exact(cagra, name, n, nq, k):
    print(f"case exact {name} n={n} nq={nq} k={k}", flush=True)
    w = datagen.workload(name, n=n, n_queries=nq)
    ids, dists = cagra.exact_search(_dev(w.base), _dev(w.queries), k, w.metric)
    ref_ids, ref_d = oracle.exact_search(w.base, w.queries, k, w.metric)
    np.testing.assert_array_equal(_u32(ids), ref_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), ref_d)


@pytest.mark.parametrize("name,n,d_init", [("tiny", 10_000, 64), ("glove200", 2_500, 128), ("deep1m", 1_000, 512)])
def test_knn_graph_bit_exact(cagra, name, n, d_init):
    print(f"case knn {name} n={n} d_init={d_init}", flush=True)
    w = datagen.workload(name, n=n, n_queries=1)
    b = _dev(w.base)
    ids = cagra.exact_search(b, b, d_init, w.metric, exclude_self=True, return_dists=False)
    np.testing.assert_array_equal(_u32(ids), oracle.knn_graph(w.base, d_init, w.metric))
    # a slice of rows addressed through self_offset
    part = cagra.exact_search(b, b[100:300], d_init, w.metric, exclude_self=True, self_offset=100,
                              return_dists=False)
    np.testing.assert_array_equal(_u32(part), _u32(ids)[100:300])


def _stagewise(cagra, g0, d):
    graph, pruned, rev, rlen = cagra.optimize(_dev(g0), d, return_stages=True)
    cnt = oracle.detour_count(g0)
    o_pr = oracle.prune(g0, cnt, d)
    o_rev, o_len = oracle.reverse(o_pr)
    o_graph = oracle.merge(o_pr, o_rev, o_len)
    np.testing.assert_array_equal(_u32(pruned), o_pr)
    np.testing.assert_array_equal(_u32(rlen), o_len)
    np.testing.assert_array_equal(_u32(rev), o_rev)
    np.testing.assert_array_equal(_u32(graph), o_graph)


@pytest.mark.parametrize("name,n,d", [("tiny", 10_000, 32), ("sift1m", 6_000, 64), ("deep1m", 3_000, 2),
                                      ("glove200", 1_500, 128)])
def test_optimize_stagewise_bit_exact(cagra, name, n, d):
    print(f"case optimize {name} n={n} d={d}", flush=True)
    w = datagen.workload(name, n=n, n_queries=1)
    _stagewise(cagra, oracle.knn_graph(w.base, 2 * d, w.metric), d)


def test_optimize_with_hub_nodes(cagra):
    # node 0 is everybody's first neighbour, node 1 everybody's second: in-degrees of N-1,
    # far beyond the reversed list's cap and the select kernel's pool.
    n, d_init, d = 5_000, 16, 8
    rng = np.random.default_rng(3)
    g0 = np.empty((n, d_init), np.uint32)
    for x in range(n):
        head = [v for v in (0, 1) if v != x]
        pool = np.setdiff1d(rng.choice(n, size=d_init + 3, replace=False), np.array(head + [x]))
        g0[x] = head + pool[: d_init - len(head)].tolist()
    print("case optimize hubs", flush=True)
    _stagewise(cagra, g0, d)


@pytest.mark.parametrize("name,n,d,d_init", [("tiny", 10_000, 32, 0), ("sift1m", 20_000, 64, 0),
                                             ("glove200", 4_000, 16, 48)])
def test_build_bit_exact(cagra, name, n, d, d_init):
    print(f"case build {name} n={n} d={d}", flush=True)
    w = datagen.workload(name, n=n, n_queries=1)
    g = cagra.build(_dev(w.base), d, d_init, w.metric)
    np.testing.assert_array_equal(_u32(g), oracle.build(w.base, d, d_init, w.metric))


def test_build_rejections(cagra):
    w = datagen.workload("tiny", n=500, n_queries=1)
    b = _dev(w.base)
    for d, di in [(7, 14), (0, 0), (32, 16), (300, 600), (250, 512 + 2)]:
        with pytest.raises(cagra.CagraError):
            cagra.build(b, d, di)
    with pytest.raises(cagra.CagraError):
        cagra.exact_search(b, b, 513)
    with pytest.raises(cagra.CagraError):
        cagra.build(b[:, :30].contiguous(), 8, 16)          # a row stride that is not a multiple of 4 floats


def test_exact_search_beyond_one_slice_of_dataset_rows(cagra):
    # More than 2^20 dataset rows: the exhaustive search walks the dataset in slices and carries the
    # k best of a row from slice to slice.  Checked on runs of rows at the start, across the slice
    # boundary and at the end, against the oracle's brute force (integer data: bit-exact).
    import torch
    n, dim, k = 1_100_000, 16, 48
    base = datagen.sift_like(n, dim, 64, seed=5, stream=1)
    bd = torch.from_numpy(base).cuda()
    for lo, hi in [(0, 40), (2**20 - 20, 2**20 + 20), (n - 40, n)]:
        print(f"case sliced exact search rows {lo}..{hi}", flush=True)
        rows = np.arange(lo, hi, dtype=np.int64)
        ref, ref_d = oracle.knn_graph(base, k, oracle.L2, rows=rows, return_dists=True)
        for algo in (cagra.EXACT_PLAIN, cagra.EXACT_FILTERED):      # the slices are the plain algorithm's
            ids = cagra.exact_search(bd, bd[lo:hi], k, cagra.L2, exclude_self=True, self_offset=lo, return_dists=False,
                                     algo=algo)
            np.testing.assert_array_equal(_u32(ids), ref)
            ids2, d2 = cagra.exact_search(bd, bd[lo:hi], k, cagra.L2, exclude_self=True, self_offset=lo, algo=algo)
            np.testing.assert_array_equal(_u32(ids2), ref)
            np.testing.assert_array_equal(d2.cpu().numpy(), ref_d)
    # plain queries (nothing left out), fewer valid neighbours than k cannot happen here; k = 1 edge
    q = datagen.sift_like(16, dim, 64, seed=5, stream=2)
    ids, d = cagra.exact_search(bd, torch.from_numpy(q).cuda(), 1, cagra.L2)
    r_ids, r_d = oracle.exact_search(base, q, 1, oracle.L2)
    np.testing.assert_array_equal(_u32(ids), r_ids)
    np.testing.assert_array_equal(d.cpu().numpy(), r_d)


@pytest.mark.parametrize("name,n,d", [("tiny", 10_000, 32), ("sift1m", 6_000, 64), ("deep1m", 3_000, 2),
                                      ("glove200", 1_500, 128)])
def test_distance_based_reordering_bit_exact(cagra, name, n, d):
    # Sec. III-B.2, the variant with distances as the weights of Eq. 3: the distance table is the
    # exhaustive search's own output (bit-exact against the oracle's), the counts are integers.
    print(f"case distance-based reordering {name} n={n} d={d}", flush=True)
    w = datagen.workload(name, n=n, n_queries=1)
    b = _dev(w.base)
    g0, gd = oracle.knn_graph(w.base, 2 * d, w.metric, return_dists=True)
    ids, dists = cagra.exact_search(b, b, 2 * d, w.metric, exclude_self=True)
    np.testing.assert_array_equal(_u32(ids), g0)
    np.testing.assert_array_equal(dists.cpu().numpy(), gd)
    graph, pruned, rev, rlen = cagra.optimize(ids, d, return_stages=True, knn_dists=dists)
    o_pr = oracle.prune(g0, oracle.detour_count_distance(g0, gd), d)
    np.testing.assert_array_equal(_u32(pruned), o_pr)
    np.testing.assert_array_equal(_u32(graph), oracle.optimize(g0, d, g0_dist=gd))
    np.testing.assert_array_equal(_u32(cagra.build(b, d, 0, w.metric, reorder=cagra.REORDER_DISTANCE)),
                                  oracle.build(w.base, d, 0, w.metric, reorder=oracle.DISTANCE))
    # integer data has many equal distances (strict comparisons matter); the two reorderings differ
    assert not np.array_equal(_u32(graph), oracle.optimize(g0, d))


def _check_filtered(cagra, base, queries, k, metric, exclude_self=False, expect_redone=None):
    import torch
    bd = _dev(base)
    qd = bd if queries is None else _dev(queries)
    redone = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    ids, dists = cagra.exact_search(bd, qd, k, metric, exclude_self=exclude_self, algo=cagra.EXACT_FILTERED,
                                    blocks_redone=redone)
    if exclude_self:
        ref, ref_d = oracle.knn_graph(base, k, metric, return_dists=True)
    else:
        ref, ref_d = oracle.exact_search(base, queries, k, metric)
    np.testing.assert_array_equal(_u32(ids), ref)
    np.testing.assert_array_equal(dists.cpu().numpy(), ref_d)
    n = int(redone.item())
    if expect_redone is not None:
        assert (n > 0) == expect_redone, f"blocks redone by the plain kernels: {n}"
    return n


def test_filtered_exact_search_bit_exact(cagra):
    # The matrix-core filter in front of the exact arithmetic: same ids and distances as the oracle's brute
    # force, and on ordinary data no block of query rows has to be handed to the plain kernels.
    print("case filtered: integer rows, distinct queries", flush=True)
    w = datagen.workload("sift1m", n=20_000, n_queries=300)
    _check_filtered(cagra, w.base, w.queries, 64, w.metric, expect_redone=False)
    print("case filtered: unit-norm rows, k-NN graph (rows of the dataset as queries, self left out)", flush=True)
    w = datagen.workload("deep1m", n=8_000, n_queries=1)
    _check_filtered(cagra, w.base, None, 64, w.metric, exclude_self=True, expect_redone=False)
    print("case filtered: inner product, dim 200 (padded to 224), k = 128", flush=True)
    w = datagen.workload("glove200", n=6_000, n_queries=130)
    _check_filtered(cagra, w.base, w.queries, 128, w.metric, expect_redone=False)
    print("case filtered: largest k on the smallest N the filter takes", flush=True)
    w = datagen.workload("tiny", n=4_096, n_queries=70)
    _check_filtered(cagra, w.base, w.queries, 512, w.metric)
    print("case filtered: k = 1", flush=True)
    _check_filtered(cagra, w.base, w.queries, 1, w.metric, expect_redone=False)


def test_filtered_exact_search_scales(cagra):
    # magnitudes far outside the fp16 range are brought into it by a power of two
    w = datagen.workload("deep1m", n=5_000, n_queries=64)
    for scale in (1e6, 1e-6, 3e4):
        print(f"case filtered: rows scaled by {scale}", flush=True)
        _check_filtered(cagra, (w.base * np.float32(scale)).astype(np.float32),
                        (w.queries * np.float32(scale)).astype(np.float32), 32, w.metric, expect_redone=False)
    # queries of a very different magnitude than the dataset
    _check_filtered(cagra, w.base, (w.queries * np.float32(1e3)).astype(np.float32), 32, oracle.IP, expect_redone=False)


def test_filtered_exact_search_falls_back_when_it_cannot_certify(cagra):
    # 20,000 rows that are copies of 3 vectors: more rows tie below any threshold than the candidate buffer
    # holds (4,096), so the block must be done again by the plain kernels, with the plain result (ties by id).
    rng = np.random.default_rng(11)
    protos = rng.integers(0, 50, size=(3, 32)).astype(np.float32)
    base = protos[rng.integers(0, 3, size=20_000)]
    queries = protos[[0, 1, 2, 0]] + np.float32(1.0)
    print("case filtered: massive duplicates", flush=True)
    _check_filtered(cagra, base, queries, 100, oracle.L2, expect_redone=True)
    _check_filtered(cagra, base, None, 16, oracle.L2, exclude_self=True, expect_redone=True)
    # the same without a distance output: the plain kernels keep their running distances in the workspace
    ids = cagra.exact_search(_dev(base), _dev(queries), 100, cagra.L2, return_dists=False, algo=cagra.EXACT_FILTERED)
    np.testing.assert_array_equal(_u32(ids), oracle.exact_search(base, queries, 100, oracle.L2)[0])


def test_build_with_either_exact_algorithm_gives_the_same_graph(cagra):
    w = datagen.workload("sift1m", n=12_000, n_queries=1)
    b = _dev(w.base)
    plain = cagra.build(b, 32, 64, w.metric, exact_algo=cagra.EXACT_PLAIN)
    filtered = cagra.build(b, 32, 64, w.metric, exact_algo=cagra.EXACT_FILTERED)
    np.testing.assert_array_equal(_u32(plain), _u32(filtered))
    np.testing.assert_array_equal(_u32(filtered), oracle.build(w.base, 32, 64, w.metric))
    # distance-based reordering takes the distances of the initial graph from the filtered search's re-rank
    by_dist = cagra.build(b, 32, 64, w.metric, reorder=cagra.REORDER_DISTANCE, exact_algo=cagra.EXACT_FILTERED)
    np.testing.assert_array_equal(_u32(by_dist), oracle.build(w.base, 32, 64, w.metric, reorder=oracle.DISTANCE))
    with pytest.raises(cagra.CagraError):
        cagra.exact_search(b[:2000], b[:10], 8, algo=cagra.EXACT_FILTERED)      # N below 4096
    with pytest.raises(cagra.CagraError):
        cagra.exact_search(b, b[:10], 8, algo=7)


def test_filtered_exact_search_with_padded_rows(cagra):
    # rows further apart than dim (views into wider matrices), a dimension that the fp16 copies pad (48 -> 64)
    import torch
    w = datagen.workload("sift1m", n=9_000, n_queries=150)
    dim = 48
    base, queries = np.ascontiguousarray(w.base[:, :dim]), np.ascontiguousarray(w.queries[:, :dim])
    wide_b = torch.full((base.shape[0], dim + 8), 9.0, dtype=torch.float32, device="cuda")
    wide_b[:, :dim] = torch.from_numpy(base).cuda()
    wide_q = torch.full((queries.shape[0], dim + 4), -3.0, dtype=torch.float32, device="cuda")
    wide_q[:, :dim] = torch.from_numpy(queries).cuda()
    print("case filtered: padded rows", flush=True)
    redone = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    ids, dists = cagra.exact_search(wide_b[:, :dim], wide_q[:, :dim], 40, cagra.L2, algo=cagra.EXACT_FILTERED,
                                    blocks_redone=redone)
    ref, ref_d = oracle.exact_search(base, queries, 40, oracle.L2)
    np.testing.assert_array_equal(_u32(ids), ref)
    np.testing.assert_array_equal(dists.cpu().numpy(), ref_d)
    assert int(redone.item()) == 0
    # the k-NN graph over the padded view: the query rows are the dataset rows
    g = cagra.exact_search(wide_b[:, :dim], wide_b[:, :dim], 24, cagra.L2, exclude_self=True, return_dists=False,
                           algo=cagra.EXACT_FILTERED)
    np.testing.assert_array_equal(_u32(g), oracle.knn_graph(base, 24, oracle.L2))


def _filtered_cases():
    rng = np.random.default_rng(123)
    cases = []
    for i in range(36):
        n = int(rng.choice([4096, 5000, 8191, 12000]))
        dim = int(rng.choice([4, 8, 20, 32, 36, 64, 96, 100, 128, 200]))
        k = int(rng.choice([1, 7, 32, 64, 128, 300, 512]))
        metric = int(rng.choice([0, 1]))
        kind = str(rng.choice(["gauss", "ints", "unit", "clusters", "dups", "scaled", "sparse"]))
        own = bool(rng.integers(0, 2))
        cases.append((i, n, dim, k, metric, kind, own, int(rng.integers(0, 2**31))))
    return cases


@pytest.mark.parametrize("i,n,dim,k,metric,kind,own,seed", _filtered_cases())
def test_filtered_exact_search_over_data_kinds(cagra, i, n, dim, k, metric, kind, own, seed):
    # shapes off every tile size, value distributions that stress the filter: ties by the thousand, sparse rows,
    # magnitudes from 1e-8 to 1e8; whatever the filter certifies or hands back, the answer is the oracle's
    print(f"case filtered kinds {i}: n={n} dim={dim} k={k} metric={metric} {kind} own={own}", flush=True)
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((n, dim)).astype(np.float32)
    if kind == "ints":
        x = np.clip(np.round(x * 20), -128, 127)
    elif kind == "unit":
        x /= np.linalg.norm(x, axis=1, keepdims=True)
    elif kind == "clusters":
        x = (rng.standard_normal((50, dim)) * 3)[rng.integers(0, 50, n)] + 0.2 * x
    elif kind == "dups":
        c = np.round(rng.standard_normal((int(rng.choice([3, 40, 1000])), dim)) * 5)
        x = c[rng.integers(0, c.shape[0], n)]
    elif kind == "scaled":
        x = x * np.float32(10.0 ** rng.uniform(-8, 8))
    elif kind == "sparse":
        x = x * (rng.random((n, dim)) < 0.15)
    x = np.ascontiguousarray(x, dtype=np.float32)
    if own:
        _check_filtered(cagra, x, None, k, metric, exclude_self=True)
    else:
        nq = int(rng.choice([1, 100, 129]))
        q = (x[rng.integers(0, n, nq)] + 0.05 * rng.standard_normal((nq, dim)) * np.abs(x).mean()).astype(np.float32)
        _check_filtered(cagra, x, q, k, metric)


def test_filtered_exact_search_falls_back_across_slices(cagra):
    # More than 2^20 dataset rows that are copies of a few vectors: the filter cannot certify, and the plain
    # kernels that take the block back walk the dataset in slices, carrying the k best from slice to slice.
    import torch
    rng = np.random.default_rng(17)
    n, dim, k = 1_150_000, 16, 70
    protos = rng.integers(0, 40, size=(5, dim)).astype(np.float32)
    base = protos[rng.integers(0, 5, size=n)]
    queries = (protos[[0, 3, 4]] + np.float32(0.5)).astype(np.float32)
    print("case filtered: duplicates beyond one slice of dataset rows", flush=True)
    bd = _dev(base)
    redone = torch.zeros(1, dtype=torch.int32, device="cuda")
    ids, dists = cagra.exact_search(bd, _dev(queries), k, cagra.L2, algo=cagra.EXACT_FILTERED, blocks_redone=redone)
    ref, ref_d = oracle.exact_search(base, queries, k, oracle.L2)
    np.testing.assert_array_equal(_u32(ids), ref)
    np.testing.assert_array_equal(dists.cpu().numpy(), ref_d)
    assert int(redone.item()) == 1
