"""Pins for the search half of the CPU oracle (no GPU).  Expected values come
from float64 brute force on integer-valued data, from breadth-first closure of
the seeds, from closed forms on a line, or from published SplitMix64 outputs --
never from the oracle itself."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2308_15136_amd import datagen

MASK = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15


def _fin(z):
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK
    return z ^ (z >> 31)


def _seed_id(seed, q, slot, n):
    h = _fin((seed + GAMMA * (q + 1)) & MASK)
    h = _fin((h + GAMMA * (slot + 1)) & MASK)
    return ((h >> 32) * n) >> 32


def test_seed_generator_published_vectors(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "splitmix64.json")))
    gamma = int(g["gamma"], 16)
    for n, want in enumerate(g["outputs_from_state_0"], start=1):
        assert oracle.splitmix_fin((gamma * n) & MASK) == int(want, 16)
    for seed, q, slot, n in [(0, 0, 0, 10), (7, 3, 5, 1000), (2**63 + 5, 9999, 63, 2**31 - 1),
                             (123, 0, 4095, 1_000_000)]:
        assert oracle.seed_id(seed, q, slot, n) == _seed_id(seed, q, slot, n)


def test_seed_generator_uniform():
    n = 50
    counts = np.zeros(n)
    for q in range(200):
        for s in range(100):
            counts[oracle.seed_id(42, q, s, n)] += 1
    exp = 200 * 100 / n
    chi2 = ((counts - exp) ** 2 / exp).sum()
    assert chi2 < 100.0          # 49 degrees of freedom: 99.99th percentile is about 97
    assert counts.min() > 0


def _int_data(n, dim, nq, seed):
    base = datagen.sift_like(n, dim, 4, seed=seed, stream=1)
    qs = datagen.sift_like(nq, dim, 4, seed=seed, stream=2)
    return base, qs


def _exact_keys(base, q):
    d = ((base.astype(np.float64) - q.astype(np.float64)[None, :]) ** 2).sum(1)
    return d


def _closure(graph, seeds):
    seen = set(seeds)
    frontier = list(seen)
    while frontier:
        nxt = []
        for v in frontier:
            for u in graph[v]:
                u = int(u)
                if u not in seen:
                    seen.add(u)
                    nxt.append(u)
        frontier = nxt
    return seen


@pytest.mark.parametrize("p", [1, 3])
def test_large_M_returns_best_of_the_seed_closure(p):
    # random sparse graph (degree 3) on 400 nodes: the closure of the seeds is a
    # strict subset for many queries, which is what makes this test sharp.
    n, d, k = 400, 3, 12
    base, qs = _int_data(n, 10, 30, seed=21)
    rng = np.random.default_rng(5)
    graph = np.empty((n, d), np.uint32)
    for x in range(n):
        graph[x] = rng.choice(np.delete(np.arange(n), x)[: 40 + x % 7], size=d, replace=False)
    ids, dists, st = oracle.search(graph, base, qs, k, itopk=n, search_width=p, seed=99,
                                   max_iterations=10 * n, return_stats=True)
    strict = 0
    for b in range(qs.shape[0]):
        seeds = [_seed_id(99, b, s, n) for s in range(p * d)]
        reach = sorted(_closure(graph, seeds))
        strict += len(reach) < n
        keys = _exact_keys(base, qs[b])
        order = sorted(reach, key=lambda v: (keys[v], v))[:k]
        want_ids = order + [oracle.INVALID_ID] * (k - len(order))
        assert ids[b].tolist() == want_ids
        assert dists[b, :len(order)].astype(np.float64).tolist() == [keys[v] for v in order]
        assert np.all(dists[b, len(order):] == np.float32(oracle.FLT_MAX))
        # every reachable node is expanded exactly once and measured exactly once
        assert st[b, 1] == len(reach) and st[b, 2] == len(reach) and st[b, 3] == 0
    assert strict > 0


@pytest.mark.parametrize("M", [5, 16, 64])
def test_complete_graph_gives_exact_topk(M):
    n, k = 60, 5
    base, qs = _int_data(n, 8, 25, seed=31)
    graph = np.array([[y for y in range(n) if y != x] for x in range(n)], np.uint32)
    ids, dists = oracle.search(graph, base, qs, k, itopk=M, search_width=1, seed=1)
    for b in range(qs.shape[0]):
        keys = _exact_keys(base, qs[b])
        order = sorted(range(n), key=lambda v: (keys[v], v))[:k]
        assert ids[b].tolist() == order
        assert dists[b].astype(np.float64).tolist() == [keys[v] for v in order]


@pytest.mark.parametrize("M,k", [(1, 1), (2, 2), (4, 2), (9, 6)])
def test_line_world_walks_to_the_exact_answer(M, k):
    # nodes at x = 0..n-1, each linked to its two neighbours on the line: the greedy
    # walk must reach the query from any seed and finish with the M nearest nodes.
    n = 300
    base = np.arange(n, dtype=np.float32)[:, None]
    graph = np.array([[x - 1 if x > 0 else 2, x + 1 if x < n - 1 else n - 3] for x in range(n)], np.uint32)
    qs = np.array([[17.3], [150.8], [299.4], [0.2], [77.5]], np.float32)
    ids, dists, st = oracle.search(graph, base, qs, k, itopk=M, search_width=1, seed=3,
                                   max_iterations=2 * n, return_stats=True)
    for b, q in enumerate(qs[:, 0]):
        order = sorted(range(n), key=lambda v: ((np.float32(v) - q) ** 2, v))[:k]
        assert ids[b].tolist() == order
        seeds = [_seed_id(3, b, s, n) for s in range(2)]
        nearest = order[0]
        assert st[b, 0] >= min(abs(s - nearest) for s in seeds)
        assert st[b, 3] == 0


def test_iteration_cap_stops_the_walk():
    n = 300
    base = np.arange(n, dtype=np.float32)[:, None]
    graph = np.array([[x - 1 if x > 0 else 2, x + 1 if x < n - 1 else n - 3] for x in range(n)], np.uint32)
    qs = np.array([[150.0]], np.float32)
    seeds = [_seed_id(8, 0, s, n) for s in range(2)]
    start = min(seeds, key=lambda s: (abs(s - 150), s))
    assert abs(start - 150) > 6
    ids, dists, st = oracle.search(graph, base, qs, 1, itopk=1, seed=8, max_iterations=5, return_stats=True)
    step = 1 if start < 150 else -1
    # M = 1: one step towards the query per pass, the fifth pass's candidates are still merged
    assert ids[0, 0] == start + 5 * step
    assert st[0, 0] == 5 and st[0, 1] == 5 and st[0, 3] == 1


def test_connected_blob_reaches_recall_one_when_M_covers_everything():
    import scipy.sparse as sp
    from scipy.sparse.csgraph import connected_components
    n, d, k = 1500, 16, 10
    base = datagen.gaussian_mixture(n, 8, 1, 0.0, 1.0, seed=13, stream=1)
    qs = datagen.gaussian_mixture(50, 8, 1, 0.0, 1.0, seed=13, stream=2)
    g = oracle.build(base, d, 2 * d)
    adj = sp.csr_matrix((np.ones(n * d), (np.repeat(np.arange(n), d), g.ravel().astype(np.int64))), shape=(n, n))
    ncomp, _ = connected_components(adj, directed=True, connection="strong")
    assert ncomp == 1
    gt, _ = oracle.exact_search(base, qs, k)
    ids, _ = oracle.search(g, base, qs, k, itopk=n, max_iterations=4 * n)
    assert oracle.recall(ids, gt) == 1.0
    np.testing.assert_array_equal(ids, gt)


@pytest.mark.parametrize("p", [1, 2])
def test_forgetting_does_not_change_the_answer(p):
    # Sec. IV-B.3: resetting the visited set costs extra distance computations only
    w = datagen.workload("tiny", n=3000, n_queries=60)
    g = oracle.build(w.base, 16, 32)
    ref_ids, ref_d, ref_st = oracle.search(g, w.base, w.queries, 10, 48, p, seed=5, return_stats=True)
    more = 0
    for interval in (1, 2, 5):
        ids, d, st = oracle.search(g, w.base, w.queries, 10, 48, p, seed=5, reset_interval=interval,
                                   return_stats=True)
        np.testing.assert_array_equal(ids, ref_ids)
        np.testing.assert_array_equal(d, ref_d)
        np.testing.assert_array_equal(st[:, :2], ref_st[:, :2])
        assert np.all(st[:, 2] >= ref_st[:, 2])
        more += int((st[:, 2] > ref_st[:, 2]).sum())
    assert more > 0


def test_output_is_sorted_unique_and_self_consistent():
    w = datagen.workload("deep1m", n=4000, n_queries=80)
    g = oracle.build(w.base, 16, 32)
    for p in (1, 2):
        ids, dists, st = oracle.search(g, w.base, w.queries, 10, 32, p, seed=2, return_stats=True)
        assert ids.max() < 4000
        for b in range(80):
            assert len(set(ids[b].tolist())) == 10
            keys = list(zip(dists[b].tolist(), ids[b].tolist()))
            assert keys == sorted(keys)
            for t in range(10):
                assert dists[b, t] == np.float32(oracle.distance(w.queries[b], w.base[ids[b, t]]))
        assert np.all(st[:, 1] <= st[:, 0] * p)
        assert np.all(st[:, 1] >= 1)


def test_recall_rises_with_M_and_matches_eq2():
    w = datagen.workload("deep1m", n=6000, n_queries=100)
    g = oracle.build(w.base, 16, 32)
    gt, _ = oracle.exact_search(w.base, w.queries, 10)
    rs = []
    for M in (10, 32, 128):
        ids, _ = oracle.search(g, w.base, w.queries, 10, M, seed=4)
        rs.append(oracle.recall(ids, gt))
    assert rs[0] <= rs[1] <= rs[2] and rs[2] > 0.9
    # Eq. 2 on a hand case
    assert oracle.recall(np.array([[1, 2, 3, 4]]), np.array([[4, 9, 1, 7]])) == 0.5


def test_multi_worker_degenerates_to_single_and_keeps_invariants():
    w = datagen.workload("tiny", n=3000, n_queries=40)
    g = oracle.build(w.base, 16, 32)
    a = oracle.search(g, w.base, w.queries, 10, 32, 1, seed=6, max_iterations=50)
    b = oracle.search_multi(g, w.base, w.queries, 10, 32, 1, seed=6, max_iterations=50)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])
    ids, dists, st = oracle.search_multi(g, w.base, w.queries, 10, 32, 4, seed=6, max_iterations=50,
                                         return_stats=True)
    gt, _ = oracle.exact_search(w.base, w.queries, 10)
    for q in range(40):
        valid = ids[q] != oracle.INVALID_ID
        assert len(set(ids[q][valid].tolist())) == valid.sum()
        keys = list(zip(dists[q].tolist(), ids[q].tolist()))
        assert keys == sorted(keys)
        for t in np.nonzero(valid)[0]:
            assert dists[q, t] == np.float32(oracle.distance(w.queries[q], w.base[ids[q, t]]))
    # four workers look at more nodes per pass than one (Sec. IV-C.2)
    assert st[:, 2].mean() > oracle.search(g, w.base, w.queries, 10, 32, 1, seed=6, max_iterations=50,
                                           return_stats=True)[2][:, 2].mean()
    assert oracle.recall(ids, gt) >= oracle.recall(a[0], gt) - 0.02


def test_argument_checks():
    w = datagen.workload("tiny", n=500, n_queries=3)
    g = oracle.build(w.base, 8, 16)
    with pytest.raises(ValueError):
        oracle.search(g, w.base, w.queries, 10, 5)          # k > M
    with pytest.raises(ValueError):
        oracle.build(w.base, 7, 14)                          # odd degree
    assert oracle.auto_max_iterations(64, 1) == 160


# ---- several workers per query (Sec. IV-C.2) ----------------------------------------------------

def _multi_case(n=300, dim=16, nq=30, degree=8, seed=31):
    base, qs = _int_data(n, dim, nq, seed)
    g = oracle.build(base, degree, 2 * degree)
    return base, qs, g


@pytest.mark.parametrize("workers", [2, 4, 7])
def test_multi_worker_lists_that_hold_every_node_give_brute_force(workers):
    # Local lists longer than the dataset never drop a node; on a strongly connected graph every node
    # is reached and owned by exactly one worker, so the merged answer is the exact one (float64 brute
    # force on integer data, ties by id).  A merge that leaves a worker out cannot pass.
    base, qs, g = _multi_case()
    n = base.shape[0]
    assert oracle.strong_components(g) == 1
    k = 10
    ids, dists, st, lists = oracle.search_multi(g, base, qs, k, n, workers, seed=3, max_iterations=10 * n,
                                                return_stats=True, return_lists=True)
    contributed = set()
    for b in range(qs.shape[0]):
        d64 = _exact_keys(base, qs[b])
        order = sorted(range(n), key=lambda i: (d64[i], i))[:k]
        assert ids[b].tolist() == order
        assert dists[b].astype(np.float64).tolist() == [d64[i] for i in order]
        # every node sits in exactly one worker's list
        held = lists[b][lists[b] != oracle.INVALID_ID]
        assert sorted(held.tolist()) == list(range(n))
        owner = {int(v): w for w in range(workers) for v in lists[b, w] if v != oracle.INVALID_ID}
        contributed |= {owner[i] for i in order}
    assert st[:, 2].tolist() == [n] * qs.shape[0]          # every node measured exactly once
    assert not st[:, 3].any()
    assert len(contributed) == workers                      # over the batch every worker fed the result


@pytest.mark.parametrize("workers", [2, 5])
def test_multi_worker_one_pass_by_hand(workers):
    # One pass (I_max = 1) followed here by hand: worker w draws the seed slots w*d .. w*d + d - 1, a node
    # belongs to the first worker (in the order 0, 1, ...) that draws it, every worker then expands its
    # nearest seed, again worker 0 first.  The lists, the number of distances and the result follow.
    base, qs, g = _multi_case(n=500, nq=20, seed=32)
    n, d, k, local = base.shape[0], g.shape[1], 5, 64
    ids, dists, st, lists = oracle.search_multi(g, base, qs, k, local, workers, seed=9, max_iterations=1,
                                                return_stats=True, return_lists=True)
    for b in range(qs.shape[0]):
        d64 = _exact_keys(base, qs[b])
        seen, own = set(), [[] for _ in range(workers)]
        for w in range(workers):
            for t in range(d):
                v = _seed_id(9, b, w * d + t, n)
                if v not in seen:
                    seen.add(v)
                    own[w].append(v)
        n_seeds = len(seen)
        parents = []
        for w in range(workers):
            par = min(own[w], key=lambda i: (d64[i], i)) if own[w] else None
            parents.append(par)
            if par is None:
                continue
            for v in g[par].tolist():
                if v not in seen:
                    seen.add(v)
                    own[w].append(v)
        for w in range(workers):
            want = sorted(own[w], key=lambda i: (d64[i], i))
            got = [int(v) for v in lists[b, w] if v != oracle.INVALID_ID]
            assert got == want, (b, w)
        assert st[b, 2] == len(seen) and st[b, 1] == sum(p is not None for p in parents)
        assert n_seeds <= workers * d
        merged = sorted(seen, key=lambda i: (d64[i], i))[:k]
        assert ids[b].tolist() == merged
        assert st[b, 3] == 1                                   # stopped by the pass limit


def test_multi_worker_result_is_the_merge_of_disjoint_lists():
    # Ordinary list lengths (nodes do get dropped): the lists stay disjoint, each is sorted, and the result
    # is the first k of their union, recomputed here from float64 distances.
    base, qs = _int_data(3000, 24, 40, 33)
    g = oracle.build(base, 16, 32)
    k, local, workers = 10, 32, 6
    ids, dists, lists = oracle.search_multi(g, base, qs, k, local, workers, seed=4, max_iterations=80,
                                            return_lists=True)
    beyond_first = 0
    for b in range(qs.shape[0]):
        d64 = _exact_keys(base, qs[b])
        held = []
        for w in range(workers):
            row = [int(v) for v in lists[b, w] if v != oracle.INVALID_ID]
            assert row == sorted(row, key=lambda i: (d64[i], i))
            held += row
        assert len(held) == len(set(held))
        merged = sorted(held, key=lambda i: (d64[i], i))[:k]
        assert ids[b].tolist() == merged
        assert dists[b].astype(np.float64).tolist() == [d64[i] for i in merged]
        beyond_first += len(set(merged) - set(int(v) for v in lists[b, 0]))
    assert beyond_first > 0                                    # the answers do not come from worker 0 alone
