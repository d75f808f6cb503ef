"""GPU multi-workgroup search (Sec. IV-C.2) against the CPU oracle, through the C ABI.

With one worker the mode is the single search with one parent per pass, so results must
match the oracle exactly (integer data).  With several workers the GPU interleaves them
freely while the oracle runs them in lock step, so the node sets differ legitimately:
only what is unique is compared (sortedness, uniqueness, distances of the returned ids)
and recall against the exact neighbours must stay close to the lock-step oracle's.
"""
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


_cache = {}


def _setup(name, n, nq, degree):
    key = (name, n, nq, degree)
    if key not in _cache:
        import torch
        w = datagen.workload(name, n=n, n_queries=nq)
        g = oracle.build(w.base, degree, 2 * degree, w.metric)
        gt, _ = oracle.exact_search(w.base, w.queries, 10, w.metric)
        dev = (torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(w.base).cuda(),
               torch.from_numpy(w.queries).cuda())
        _cache[key] = (w, g, gt, dev)
    return _cache[key]


def _local(k, itopk, workers):
    return max(k, 32, -(-itopk // workers))


def _check_invariants(ids, ds, w):
    n = w.base.shape[0]
    for b in range(ids.shape[0]):
        valid = ids[b] != oracle.INVALID_ID
        assert np.all(ids[b][valid] < n)
        assert len(set(ids[b][valid].tolist())) == valid.sum()
        keys = list(zip(ds[b].tolist(), ids[b].tolist()))
        assert keys == sorted(keys)
    for b in range(0, ids.shape[0], 5):
        for t in range(ids.shape[1]):
            if ids[b, t] != oracle.INVALID_ID:
                ref = oracle.distance(w.queries[b], w.base[ids[b, t]], w.metric)
                assert abs(ds[b, t] - ref) <= 1e-5 * max(abs(ref), 1.0 if w.metric == oracle.IP else 1e-30)


@pytest.mark.parametrize("name,n,degree,itopk,k", [("sift1m", 20_000, 64, 64, 10), ("sift1m", 20_000, 64, 200, 100)])
def test_one_worker_equals_single_search(cagra, name, n, degree, itopk, k):
    print(f"case multi W=1 {name} M={itopk} k={k}", flush=True)
    w, g, gt, (gd, bd, qd) = _setup(name, n, 200, degree)
    opts = cagra.SearchOptions(seed=11, mode=2, wg_per_query=1)
    ids, dists, st = cagra.search(gd, bd, qd, k, itopk, 1, w.metric, opts, return_stats=True)
    local = _local(k, itopk, 1)
    r_ids, r_d, r_st = oracle.search(g, w.base, w.queries, k, local, 1, w.metric, seed=11, return_stats=True)
    np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    st = st.cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(st[:, :3], r_st[:, :3])
    m_ids, m_d = oracle.search_multi(g, w.base, w.queries, k, local, 1, w.metric, seed=11,
                                     max_iterations=oracle.auto_max_iterations(local, 1))
    np.testing.assert_array_equal(m_ids, r_ids)


@pytest.mark.parametrize("name,n,degree,itopk,workers,nq", [
    ("deep1m", 50_000, 32, 64, 4, 1000),
    ("deep1m", 50_000, 32, 256, 8, 1000),
    ("sift1m", 20_000, 64, 128, 4, 1000),
    ("glove200", 20_000, 64, 128, 16, 500),
    ("deep1m", 50_000, 32, 64, 8, 1),        # batch of one
    ("deep1m", 50_000, 32, 64, 8, 10),
])
def test_several_workers(cagra, name, n, degree, itopk, workers, nq):
    print(f"case multi {name} M={itopk} W={workers} B={nq}", flush=True)
    w, g, gt, (gd, bd, qd) = _setup(name, n, 1000, degree)
    k = 10
    opts = cagra.SearchOptions(seed=5, mode=2, wg_per_query=workers)
    ids, dists, st = cagra.search(gd, bd, qd[:nq], k, itopk, 1, w.metric, opts, return_stats=True)
    ids = ids.cpu().numpy().view(np.uint32)
    ds = dists.cpu().numpy()
    st = st.cpu().numpy().view(np.uint32)
    assert not np.any(st[:, 3] & 2), "visited table overflowed"
    import dataclasses
    ww = dataclasses.replace(w, queries=w.queries[:nq])
    _check_invariants(ids, ds, ww)
    local = _local(k, itopk, workers)
    cap = oracle.auto_max_iterations(local, 1)
    o_ids, o_d, o_st = oracle.search_multi(g, w.base, w.queries[:nq], k, local, workers, w.metric, seed=5,
                                           max_iterations=cap, return_stats=True)
    # a worker never makes more passes than the cap, and every pass expands one parent
    assert st[:, 0].max() <= cap and np.all(st[:, 1] <= st[:, 0].astype(np.int64) * workers)
    if nq >= 500:
        r_gpu, r_ora = oracle.recall(ids, gt[:nq]), oracle.recall(o_ids, gt[:nq])
        agree = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids, o_ids)) / float(ids.size)
        print(f"  recall gpu {r_gpu:.4f} oracle {r_ora:.4f} id agreement {agree:.4f} "
              f"dists gpu {st[:, 2].mean():.0f} oracle {o_st[:, 2].mean():.0f}", flush=True)
        assert abs(r_gpu - r_ora) <= 0.003
        assert agree >= 0.97          # measured, not a parity bar: the workers' interleaving differs


def test_auto_mode_rule(cagra):
    # Sec. IV-C.3: multi when the batch is smaller than the number of compute units or itopk > 512
    assert cagra.auto_mode(1, 64) == 2
    assert cagra.auto_mode(10_000, 64) == 1
    assert cagra.auto_mode(10_000, 1024) == 2
    w, g, gt, (gd, bd, qd) = _setup("deep1m", 50_000, 1000, 32)
    ids, dists = cagra.search(gd, bd, qd[:8], 10, 64, 4, w.metric, cagra.SearchOptions(seed=1))
    _check_invariants(ids.cpu().numpy().view(np.uint32), dists.cpu().numpy(),
                      __import__("dataclasses").replace(w, queries=w.queries[:8]))
    # itopk beyond the single-workgroup limit goes to the multi mode
    ids, dists = cagra.search(gd, bd, qd, 10, 1024, 8, w.metric, cagra.SearchOptions(seed=1))
    assert oracle.recall(ids.cpu().numpy().view(np.uint32), gt) > 0.9


def test_prepared_search_gives_the_same_answers(cagra):
    import torch
    w, g, gt, (gd, bd, qd) = _setup("sift1m", 20_000, 200, 64)
    # single mode: deterministic, so the prepared call must reproduce search() exactly, call after call
    opts = cagra.SearchOptions(seed=3, mode=1)
    qbuf = qd[:50].clone()
    prepared = cagra.PreparedSearch(gd, bd, qbuf, 10, 64, 2, w.metric, opts)
    for lo in (0, 50, 150):
        qbuf.copy_(qd[lo:lo + 50])
        ids, dists = prepared()
        e_ids, e_d = cagra.search(gd, bd, qd[lo:lo + 50], 10, 64, 2, w.metric, opts)
        assert torch.equal(ids, e_ids) and torch.equal(dists, e_d)
        ids, dists = prepared(qd[150 - lo:200 - lo])         # another tensor of the same shape, no copy
        e_ids, e_d = cagra.search(gd, bd, qd[150 - lo:200 - lo], 10, 64, 2, w.metric, opts)
        assert torch.equal(ids, e_ids) and torch.equal(dists, e_d)
    with pytest.raises(ValueError):
        prepared(qd[:49])
    # multi mode, one query at a time
    mopts = cagra.SearchOptions(seed=3, mode=2, wg_per_query=8, max_iterations=12)
    q1 = qd[:1].clone()
    one = cagra.PreparedSearch(gd, bd, q1, 10, 256, 1, w.metric, mopts)
    hits = 0
    for b in range(60):
        q1.copy_(qd[b:b + 1])
        ids, dists = one()
        row = ids.cpu().numpy().view(np.uint32)[0]
        hits += len(set(row.tolist()) & set(gt[b].tolist()))
        assert np.all(np.diff(dists.cpu().numpy()[0]) >= 0) and len(set(row.tolist())) == 10
    assert hits / 600.0 > 0.9


@pytest.mark.parametrize("workers", [2, 4, 7])
def test_lists_that_hold_every_node_give_the_exact_answer(cagra, workers):
    # However the workers interleave: a node belongs to the worker that registered it first, and with
    # local lists longer than the dataset no list ever drops a node, so every node reachable from the
    # seeds ends up in exactly one list and the merged result is the exact k nearest of those.  On a
    # strongly connected graph that is the brute-force answer, id for id (integer data: distances too).
    import torch
    n, nq, degree, k = 400, 60, 8, 10
    w = datagen.workload("sift1m", n=n, n_queries=nq)
    g = oracle.build(w.base, degree, 2 * degree, w.metric)
    assert oracle.strong_components(g) == 1
    ref_ids, ref_d = oracle.exact_search(w.base, w.queries, k, w.metric)
    print(f"case multi exhaustive lists W={workers}", flush=True)
    opts = cagra.SearchOptions(seed=21, mode=2, wg_per_query=workers, max_iterations=600)
    ids, dists = cagra.search(torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(w.base).cuda(),
                              torch.from_numpy(w.queries).cuda(), k, 512 * workers, 1, w.metric, opts)
    plan = cagra.describe(degree, w.base.shape[1], nq, k, 512 * workers, 1, opts)
    assert plan["itopk_local"] >= n and plan["wg_per_query"] == workers
    np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), ref_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), ref_d)


def _workspace_is_clean(cagra, ws, plan, batch):
    """The clean state of a multi-mode workspace: ticket counters zero, and of the two tables of every query the one
    that is in use next has every slot empty."""
    import torch
    words = ws.view(torch.int32)
    t0, d0, w0 = plan["ws_tables_offset"] // 4, plan["ws_tickets_offset"] // 4, plan["ws_which_offset"] // 4
    tickets, which = words[d0:d0 + batch], words[w0:w0 + batch]
    tables = words[t0:t0 + 2 * batch * plan["table_entries"]].view(batch, 2, plan["table_entries"])
    if not (bool((tickets == 0).all().item()) and bool(((which == 0) | (which == 1)).all().item())):
        return False
    in_use = tables[torch.arange(batch, device=ws.device), which.long()]
    return bool((in_use == -1).all().item())


@pytest.mark.parametrize("workers,itopk,max_it", [(1, 64, 0), (8, 256, 12), (32, 1024, 4)])
def test_every_search_hands_the_workspace_back_clean(cagra, workers, itopk, max_it):
    # Sec. IV-C.2's device-memory table is emptied by the last worker of each query, so a caller who keeps the
    # workspace may vouch for it and the search is one kernel launch.  Checked slot by slot after every call.
    import torch
    w, g, gt, (gd, bd, qd) = _setup("sift1m", 20_000, 200, 64)
    k, nb = 10, 7
    opts = cagra.SearchOptions(seed=3, mode=2, wg_per_query=workers, max_iterations=max_it)
    plan = cagra.describe(64, 128, nb, k, itopk, 1, opts)
    ws = torch.empty(cagra.search_workspace_bytes(20_000, 64, nb, k, itopk, 1, opts), dtype=torch.uint8, device="cuda")
    ws.random_(0, 256)                                    # whatever was there before
    cagra.search_workspace_init(ws, 20_000, 64, 128, nb, k, itopk, 1, opts)
    torch.cuda.synchronize()
    assert _workspace_is_clean(cagra, ws, plan, nb)
    import dataclasses
    vouch = dataclasses.replace(opts, workspace_clean=1)
    print(f"case clean workspace W={workers} M={itopk} I_max={max_it}", flush=True)
    hits = 0
    for call in range(12):
        lo = call * nb
        ids, dists, st = cagra.search(gd, bd, qd[lo:lo + nb], k, itopk, 1, w.metric, vouch, workspace=ws, return_stats=True)
        torch.cuda.synchronize()
        assert _workspace_is_clean(cagra, ws, plan, nb), f"call {call} left something behind"
        ids_np = ids.cpu().numpy().view(np.uint32)
        st_np = st.cpu().numpy().view(np.uint32)
        assert not np.any(st_np[:, 3] & 2) and np.all(st_np[:, 2] > 0) and np.all(st_np[:, 1] <= st_np[:, 0].astype(np.int64) * workers)
        if workers == 1:
            # one worker is deterministic: the vouched-for call must equal the call that cleans first, bit for bit
            e_ids, e_d, e_st = cagra.search(gd, bd, qd[lo:lo + nb], k, itopk, 1, w.metric, opts, return_stats=True)
            assert torch.equal(ids, e_ids) and torch.equal(dists, e_d) and torch.equal(st, e_st)
        srt = np.sort(ids_np, axis=1)
        assert np.all(srt[:, 1:] != srt[:, :-1]) and np.all(np.diff(dists.cpu().numpy(), axis=1) >= 0)
        hits += sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids_np, gt[lo:lo + nb]))
    assert hits / (12.0 * nb * k) > (0.9 if workers > 1 else 0.85)


def test_vouched_workspace_gives_the_exact_answer_call_after_call(cagra):
    # lists longer than the dataset: the answer is unique whatever the interleaving, so a table slot left behind by an
    # earlier call (a node wrongly taken for visited) would show as a missing neighbour
    import torch
    n, nq, degree, k, workers = 400, 60, 8, 10, 4
    w = datagen.workload("sift1m", n=n, n_queries=nq)
    g = oracle.build(w.base, degree, 2 * degree, w.metric)
    ref_ids, ref_d = oracle.exact_search(w.base, w.queries, k, w.metric)
    gd, bd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(w.base).cuda(), torch.from_numpy(w.queries).cuda()
    opts = cagra.SearchOptions(seed=21, mode=2, wg_per_query=workers, max_iterations=600)
    nb = 5
    call = cagra.PreparedSearch(gd, bd, qd[:nb].clone(), k, 512 * workers, 1, w.metric, opts)
    for lo in range(0, nq, nb):
        ids, dists = call(qd[lo:lo + nb])
        np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), ref_ids[lo:lo + nb])
        np.testing.assert_array_equal(dists.cpu().numpy(), ref_d[lo:lo + nb])
