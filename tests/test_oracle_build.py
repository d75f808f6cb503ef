"""Pins for the build half of the CPU oracle (no GPU): each test checks the
oracle against something other than itself -- float64 brute force on data
where every formula is exact, hand-worked fixtures, or invariants that the
paper states (Sec. III)."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2308_15136_amd import datagen


def _bruteforce_lists(base64, K, metric, exclude_self=True):
    """Exact (dist, id)-ordered neighbour lists in float64 (exact on integer data)."""
    if metric == oracle.L2:
        sq = (base64 * base64).sum(1)
        D = sq[:, None] + sq[None, :] - 2.0 * base64 @ base64.T
    else:
        D = -(base64 @ base64.T)
    n = D.shape[0]
    out = np.empty((n, K), np.uint32)
    ids = np.arange(n)
    for x in range(n):
        order = np.lexsort((ids, D[x]))
        if exclude_self:
            order = order[order != x]
        out[x] = order[:K]
    return out, D


@pytest.mark.parametrize("metric", [oracle.L2, oracle.IP])
def test_knn_matches_float64_bruteforce_on_integer_data(metric):
    # integer values 0..255 in dim 24: squared distances and dot products are
    # integers below 2^24, so fp32 in any order and float64 agree exactly.
    base = datagen.sift_like(1200, 24, 6, seed=11, stream=1)
    assert np.all(base == np.rint(base)) and base.min() >= 0 and base.max() <= 255
    want, D = _bruteforce_lists(base.astype(np.float64), 20, metric)
    got, gd = oracle.knn_graph(base, 20, metric, return_dists=True)
    np.testing.assert_array_equal(got, want)
    np.testing.assert_array_equal(gd.astype(np.float64), np.take_along_axis(D, want.astype(np.int64), 1))


def test_knn_ties_by_id_on_a_line(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "line6_build.json")))
    pts = np.array(g["points"], np.float32)[:, None]
    np.testing.assert_array_equal(oracle.knn_graph(pts, g["d_init"]), np.array(g["knn"], np.uint32))
    # longer line: interior node i has neighbours i-1, i+1, i-2, i+2 in that order
    pts = np.arange(50, dtype=np.float32)[:, None]
    got = oracle.knn_graph(pts, 4)
    for i in range(2, 48):
        assert got[i].tolist() == [i - 1, i + 1, i - 2, i + 2]
    assert got[0].tolist() == [1, 2, 3, 4] and got[49].tolist() == [48, 47, 46, 45]


def test_knn_rows_subset_equals_full():
    base = datagen.gaussian_mixture(700, 12, 4, 1.0, 1.0, seed=5, stream=1)
    full = oracle.knn_graph(base, 16)
    rows = np.array([0, 13, 699, 350], np.int64)
    np.testing.assert_array_equal(oracle.knn_graph(base, 16, rows=rows), full[rows])


def test_exact_search_is_eq1():
    base = datagen.sift_like(900, 16, 5, seed=3, stream=1)
    qs = datagen.sift_like(40, 16, 5, seed=3, stream=2)
    b64, q64 = base.astype(np.float64), qs.astype(np.float64)
    D = ((q64[:, None, :] - b64[None, :, :]) ** 2).sum(-1)
    ids, dists = oracle.exact_search(base, qs, 7)
    for b in range(40):
        order = np.lexsort((np.arange(900), D[b]))[:7]
        assert ids[b].tolist() == order.tolist()
        assert dists[b].astype(np.float64).tolist() == D[b][order].tolist()


def test_distance_definitions():
    x = np.array([1.0, 2.0, 3.0, 4.0], np.float32)
    y = np.array([0.5, -2.0, 3.0, 8.0], np.float32)
    assert oracle.distance(x, y, oracle.L2) == 0.25 + 16.0 + 0.0 + 16.0
    assert oracle.distance(x, y, oracle.IP) == -(0.5 - 4.0 + 9.0 + 32.0)
    assert oracle.distance(x, x, oracle.L2) == 0.0
    # squared L2 is symmetric, inner product too
    assert oracle.distance(x, y, oracle.L2) == oracle.distance(y, x, oracle.L2)


def test_hand_worked_line_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "line6_build.json")))
    g0 = np.array(g["knn"], np.uint32)
    cnt = oracle.detour_count(g0)
    np.testing.assert_array_equal(cnt, np.array(g["count"], np.uint32))
    pr = oracle.prune(g0, cnt, g["d"])
    np.testing.assert_array_equal(pr, np.array(g["pruned"], np.uint32))
    rev, rlen = oracle.reverse(pr)
    for y, want in enumerate(g["reversed"]):
        assert rev[y, :rlen[y]].tolist() == want
    np.testing.assert_array_equal(oracle.merge(pr, rev, rlen), np.array(g["graph"], np.uint32))
    pts = np.array(g["points"], np.float32)[:, None]
    np.testing.assert_array_equal(oracle.build(pts, g["d"], g["d_init"]), np.array(g["graph"], np.uint32))


def test_merge_hand_cases(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "merge_cases.json")))
    d = g["d"]
    for case in g["cases"]:
        # node 0 carries the case; the other rows are filler so that every id is a valid node
        n = 40
        pr = np.tile(np.arange(1, d + 1, dtype=np.uint32), (n, 1))
        rev = np.full((n, d), oracle.INVALID_ID, np.uint32)
        rlen = np.zeros(n, np.uint32)
        pr[0] = case["pruned"]
        rlen[0] = len(case["reversed"])
        rev[0, :rlen[0]] = case["reversed"]
        out = oracle.merge(pr, rev, rlen)
        assert out[0].tolist() == case["expect"], case["why"]


def _detour_by_sets(g0):
    """Eq. 3 with ranks, restated through set membership instead of loops over l."""
    n, D = g0.shape
    cnt = np.zeros((n, D), np.uint32)
    for x in range(n):
        for j in range(D):
            y = int(g0[x, j])
            cnt[x, j] = sum(1 for i in range(j) if y in set(g0[int(g0[x, i]), :j].tolist()))
    return cnt


def test_detour_count_definition_and_bounds():
    base = datagen.gaussian_mixture(300, 8, 3, 1.0, 1.0, seed=7, stream=1)
    g0 = oracle.knn_graph(base, 12)
    cnt = oracle.detour_count(g0)
    np.testing.assert_array_equal(cnt, _detour_by_sets(g0))
    assert np.all(cnt[:, 0] == 0)
    assert np.all(cnt <= np.arange(12)[None, :])


def test_detour_count_closed_form_on_complete_lists():
    # d_init = N-1: every node lists every other node, so "Y is within the first
    # j entries of Z's list" is "rank of Y seen from Z is < j", computable from
    # the distance ranks alone.
    base = datagen.sift_like(24, 6, 2, seed=9, stream=1).astype(np.float64)
    base += np.arange(24)[:, None] * 1e-3          # no exact ties
    g0 = oracle.knn_graph(base.astype(np.float32), 23)
    b = base.astype(np.float32).astype(np.float64)
    D = ((b[:, None, :] - b[None, :, :]) ** 2).sum(-1)
    rank = np.empty((24, 24), np.int64)            # rank[z, y] = position of y in z's list
    for z in range(24):
        order = [v for v in np.argsort(D[z], kind="stable") if v != z]
        assert order == g0[z].tolist()
        for r, y in enumerate(order):
            rank[z, y] = r
    cnt = oracle.detour_count(g0)
    for x in range(24):
        for j in range(23):
            y = g0[x, j]
            want = sum(1 for i in range(j) if rank[g0[x, i], y] < j)
            assert cnt[x, j] == want


@pytest.mark.parametrize("name,n,d", [("tiny", 2500, 16), ("deep1m", 2000, 8)])
def test_graph_invariants(name, n, d):
    w = datagen.workload(name, n=n, n_queries=4)
    g0 = oracle.knn_graph(w.base, 2 * d, w.metric)
    cnt = oracle.detour_count(g0)
    pr = oracle.prune(g0, cnt, d)
    rev, rlen = oracle.reverse(pr)
    out = oracle.merge(pr, rev, rlen)
    ids = np.arange(n, dtype=np.uint32)[:, None]
    # pruned: d-subset of the initial list, first entry is the nearest neighbour
    np.testing.assert_array_equal(pr[:, 0], g0[:, 0])
    for x in range(0, n, 97):
        assert set(pr[x].tolist()) <= set(g0[x].tolist()) and len(set(pr[x].tolist())) == d
        # order is by (count, rank)
        pos = [g0[x].tolist().index(v) for v in pr[x]]
        keys = [(int(cnt[x, p]), p) for p in pos]
        assert keys == sorted(keys)
        assert keys[-1] <= min((int(cnt[x, p]), p) for p in range(2 * d) if p not in pos)
    # reversed: capped at d; every listed source really has that edge; ranks non-decreasing
    assert rlen.max() <= d
    indeg = np.bincount(pr.ravel(), minlength=n)
    np.testing.assert_array_equal(np.minimum(indeg, d), rlen)
    for y in range(0, n, 61):
        ranks = []
        for xsrc in rev[y, :rlen[y]]:
            row = pr[xsrc].tolist()
            assert y in row
            ranks.append((row.index(y), int(xsrc)))
        assert ranks == sorted(ranks)
    # final graph: fixed out-degree, no self loop, no duplicate, ids valid
    assert out.shape == (n, d) and out.max() < n
    assert not np.any(out == ids)
    assert all(len(set(r.tolist())) == d for r in out)
    np.testing.assert_array_equal(out[:, 0], g0[:, 0])
    # d/2 from each side whenever the reversed list has enough entries new to the node
    for y in range(0, n, 53):
        from_rev = [v for t, v in enumerate(out[y]) if t % 2 == 1 and v in set(rev[y, :rlen[y]].tolist())]
        if rlen[y] == 0:
            assert out[y].tolist() == pr[y].tolist()
        assert len(from_rev) <= d // 2
    np.testing.assert_array_equal(oracle.optimize(g0, d), out)
    np.testing.assert_array_equal(oracle.build(w.base, d, 2 * d, w.metric), out)


def test_two_hop_bound():
    # Sec. III-A: a node reaches at most d + d^2 nodes in two hops
    w = datagen.workload("tiny", n=1500, n_queries=1)
    d = 8
    g = oracle.build(w.base, d, 16)
    for x in range(0, 1500, 37):
        two = set(g[x].tolist())
        for z in g[x]:
            two |= set(g[z].tolist())
        assert len(two) <= d + d * d


def test_detour_count_rows_subset_equals_full():
    base = datagen.gaussian_mixture(400, 8, 3, 1.0, 1.0, seed=17, stream=1)
    g0 = oracle.knn_graph(base, 12)
    full = oracle.detour_count(g0)
    rows = np.array([399, 0, 17, 200], np.int64)
    np.testing.assert_array_equal(oracle.detour_count(g0, rows=rows), full[rows])


# ---- distance-based reordering (Sec. III-B.2, the variant the paper compares with) ------------

def test_distance_based_count_on_a_line_by_hand():
    # Five points on a line at 0, 1, 3, 7, 15 (squared distances are integers), d_init = 4: every
    # node lists every other node.  A route X -> Z -> Y counts iff both hops are shorter than the
    # direct edge.  From the end point 0 every nearer point is a detour to every farther one:
    # counts 0, 1, 2, 3 along its list (1, 3, 7, 15).  From the point at 3 (list 1, 0, 7, 15 at
    # squared distances 4, 9, 16, 144): to 0 via 1 (4 < 9, 1 < 9): 1 route; to 7 none (1 -> 7 is
    # 36, 0 -> 7 is 49, both >= 16); to 15 only via 7 (16 < 144, 64 < 144): 1 route.
    pts = np.array([[0.0], [1.0], [3.0], [7.0], [15.0]], np.float32)
    g0, gd = oracle.knn_graph(pts, 4, return_dists=True)
    assert g0[0].tolist() == [1, 2, 3, 4] and g0[2].tolist() == [1, 0, 3, 4] and g0[4].tolist() == [3, 2, 1, 0]
    assert gd[2].tolist() == [4.0, 9.0, 16.0, 144.0]
    cnt = oracle.detour_count_distance(g0, gd)
    assert cnt[0].tolist() == [0, 1, 2, 3]
    assert cnt[2].tolist() == [0, 1, 0, 1]
    assert cnt[4].tolist() == [0, 1, 2, 3]


def test_distance_based_count_is_the_lune_count_on_complete_lists():
    # d_init = N-1: every edge exists, so the count for X -> Y is the number of points Z that are
    # closer than |XY| to both X and Y (the lune of the relative neighbourhood graph) -- a property
    # of the metric alone, computed here from float64 distances (exact on integer data).
    n = 40
    base = datagen.sift_like(n, 8, 3, seed=11, stream=1)
    g0, gd = oracle.knn_graph(base, n - 1, return_dists=True)
    b = base.astype(np.float64)
    D = ((b[:, None, :] - b[None, :, :]) ** 2).sum(-1)
    cnt = oracle.detour_count_distance(g0, gd)
    for x in range(n):
        for j in range(n - 1):
            y = int(g0[x, j])
            want = sum(1 for z in range(n) if z != x and z != y and D[x, z] < D[x, y] and D[z, y] < D[x, y])
            assert cnt[x, j] == want


def test_distance_based_count_bounds_and_subset():
    w = datagen.workload("deep1m", n=1500, n_queries=1)
    g0, gd = oracle.knn_graph(w.base, 24, return_dists=True)
    cnt = oracle.detour_count_distance(g0, gd)
    assert np.all(cnt[:, 0] == 0)
    # a detour's first hop is strictly shorter than the edge, so it sits earlier in the sorted list
    assert np.all(cnt <= np.arange(24)[None, :])
    rows = np.array([0, 7, 700, 1499], np.int64)
    np.testing.assert_array_equal(oracle.detour_count_distance(g0, gd, rows=rows), cnt[rows])
    # literal set form: routes through Z need Y in Z's list
    member = [set(r.tolist()) for r in g0]
    for x in (3, 999):
        for j in range(24):
            y = int(g0[x, j])
            want = 0
            for i in range(24):
                z = int(g0[x, i])
                if y in member[z] and gd[x, i] < gd[x, j] and gd[z, g0[z].tolist().index(y)] < gd[x, j]:
                    want += 1
            assert cnt[x, j] == want


def test_distance_based_build_keeps_the_graph_invariants():
    w = datagen.workload("tiny", n=1200, n_queries=1)
    g = oracle.build(w.base, 16, 32, w.metric, reorder=oracle.DISTANCE)
    n = g.shape[0]
    assert g.shape == (n, 16) and g.max() < n
    assert not np.any(g == np.arange(n, dtype=np.uint32)[:, None])
    assert all(len(set(r.tolist())) == 16 for r in g)
    g0, gd = oracle.knn_graph(w.base, 32, w.metric, return_dists=True)
    np.testing.assert_array_equal(g, oracle.optimize(g0, 16, g0_dist=gd))
    assert np.all(g[:, 0] == g0[:, 0])      # the nearest neighbour has no detour and stays first


# ---- reachability measures of Sec. III-A ------------------------------------------------------

def _adjacency(g):
    n = g.shape[0]
    a = np.zeros((n, n), bool)
    a[np.repeat(np.arange(n), g.shape[1]), g.reshape(-1)] = True
    return a


def test_two_hop_counts_against_the_adjacency_matrix():
    rng = np.random.default_rng(5)
    n, d = 300, 5
    g = np.stack([rng.choice(np.setdiff1d(np.arange(n), [x]), size=d, replace=False) for x in range(n)]).astype(np.uint32)
    a = _adjacency(g)
    reach = a | ((a.astype(np.int32) @ a.astype(np.int32)) > 0)     # one or two steps
    reach[np.arange(n), np.arange(n)] = False                         # the node itself does not count
    np.testing.assert_array_equal(oracle.two_hop_counts(g), reach.sum(1).astype(np.uint32))
    # closed forms: a ring with one edge per node reaches 2 nodes, a complete graph all others,
    # and nothing exceeds d + d^2
    ring = ((np.arange(10) + 1) % 10).astype(np.uint32)[:, None]
    assert oracle.two_hop_counts(ring).tolist() == [2] * 10
    full = np.stack([np.setdiff1d(np.arange(7), [x]) for x in range(7)]).astype(np.uint32)
    assert oracle.two_hop_counts(full).tolist() == [6] * 7
    assert oracle.two_hop_counts(g).max() <= d + d * d


def test_component_counts_against_scipy_and_by_hand():
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import connected_components
    rng = np.random.default_rng(8)
    for n, d in [(400, 1), (400, 2), (2000, 3), (50, 6)]:
        g = np.stack([rng.choice(np.setdiff1d(np.arange(n), [x]), size=d, replace=False) for x in range(n)]).astype(np.uint32)
        adj = csr_matrix(_adjacency(g))
        assert oracle.strong_components(g) == connected_components(adj, directed=True, connection="strong")[0]
        assert oracle.weak_components(g) == connected_components(adj, directed=True, connection="weak")[0]
    # a directed ring is one strong component; a chain that ends in a 2-cycle has one component per
    # chain node plus the cycle; two separate rings are two of each
    ring = ((np.arange(9) + 1) % 9).astype(np.uint32)[:, None]
    assert oracle.strong_components(ring) == 1 and oracle.weak_components(ring) == 1
    chain = np.array([1, 2, 3, 4, 3], np.uint32)[:, None]           # 0->1->2->3<->4
    assert oracle.strong_components(chain) == 4 and oracle.weak_components(chain) == 1
    two = np.array([1, 2, 0, 4, 5, 3], np.uint32)[:, None]
    assert oracle.strong_components(two) == 2 and oracle.weak_components(two) == 2
    # a long path does not overflow anything (the recursion is unrolled)
    n = 200_000
    path = np.minimum(np.arange(n) + 1, n - 1).astype(np.uint32)[:, None]
    path[-1, 0] = n - 2
    assert oracle.strong_components(path) == n - 1


# ---- NN-descent in synchronous rounds (Sec. III-B.1 names NN-descent; the rounds are this build's) --

def _lists_ok(base, ids, dists, metric=oracle.L2):
    n, k = ids.shape
    for x in range(0, n, max(1, n // 60)):
        valid = ids[x] != oracle.INVALID_ID
        row = ids[x][valid]
        assert x not in row.tolist() and len(set(row.tolist())) == len(row)
        assert np.all(valid[: valid.sum()])                                    # unused slots come last
        keys = list(zip(dists[x][valid].tolist(), row.tolist()))
        assert keys == sorted(keys)
        for j in (0, len(row) // 2, len(row) - 1):
            assert dists[x, j] == oracle.distance(base[x], base[row[j]], metric)


def test_nn_descent_round_zero_is_the_best_of_the_drawn_nodes():
    base = datagen.sift_like(500, 8, 4, seed=2, stream=1)
    k = 12
    ids, dists = oracle.nn_descent(base, k, 0, 4, seed=77)
    b = base.astype(np.float64)
    for x in (0, 1, 250, 499):
        drawn = sorted({oracle.seed_id(77, x, j, 500) for j in range(k)} - {x},
                       key=lambda c: (((b[x] - b[c]) ** 2).sum(), c))
        assert ids[x][: len(drawn)].tolist() == drawn
        assert np.all(ids[x][len(drawn):] == oracle.INVALID_ID)
    _lists_ok(base, ids, dists)


def test_nn_descent_one_round_follows_the_stated_rule():
    # L_t from L_{t-1} re-derived with sets and float64 distances (exact on integer data)
    n, k, s = 400, 10, 4
    base = datagen.sift_like(n, 8, 4, seed=3, stream=1)
    b = base.astype(np.float64)
    for t in (1, 2, 3, 4):      # windows 0, 4, 6 (clipped to k - s), 0
        prev, _ = oracle.nn_descent(base, k, t - 1, s, seed=5)
        cur, _ = oracle.nn_descent(base, k, t, s, seed=5)
        win = min(((t - 1) % -(-k // s)) * s, k - s)       # the sample's first rank moves from round to round
        forward = [[int(v) for v in prev[x][win:win + s] if v != oracle.INVALID_ID] for x in range(n)]
        reverse = [[] for _ in range(n)]
        for r in range(win, win + s):            # sources ordered by (rank, source), at most s each
            for y in range(n):
                if prev[y][r] != oracle.INVALID_ID and len(reverse[prev[y][r]]) < s:
                    reverse[int(prev[y][r])].append(y)
        for x in range(0, n, 7):
            pool = {int(v) for v in prev[x] if v != oracle.INVALID_ID}
            for v in forward[x] + reverse[x]:
                pool |= {int(c) for c in prev[v] if c != oracle.INVALID_ID}
            pool.discard(x)
            want = sorted(pool, key=lambda c: (((b[x] - b[c]) ** 2).sum(), c))[:k]
            assert cur[x][: len(want)].tolist() == want


def test_nn_descent_improves_monotonically_and_converges():
    w = datagen.workload("tiny", n=3000, n_queries=1)
    k, s = 16, 8
    exact = oracle.knn_graph(w.base, k)
    last_kth, recalls = None, []
    for t in (0, 1, 2, 4, 8):
        ids, dists = oracle.nn_descent(w.base, k, t, s, seed=1)
        _lists_ok(w.base, ids, dists)
        if last_kth is not None:
            assert np.all(dists[:, -1] <= last_kth)          # a list only ever gets better
        last_kth = dists[:, -1].copy()
        recalls.append(np.mean([len(set(a.tolist()) & set(e.tolist())) for a, e in zip(ids, exact)]) / k)
    assert recalls == sorted(recalls) and recalls[0] < 0.05 and recalls[-1] > 0.9
    # with everything sampled on a small set the lists become the exact ones
    base = datagen.sift_like(60, 8, 2, seed=4, stream=1)
    ids, _ = oracle.nn_descent(base, 20, 6, 20, seed=9)
    np.testing.assert_array_equal(ids, oracle.knn_graph(base, 20))
    # the exact lists are a fixed point of a round: feeding them back changes nothing is implied by
    # "a list only gets better" + optimality; inner product works the same way
    wg = datagen.workload("glove200", n=800, n_queries=1)
    ids, dists = oracle.nn_descent(wg.base, 8, 5, 8, metric=oracle.IP, seed=2)
    _lists_ok(wg.base, ids, dists, oracle.IP)
