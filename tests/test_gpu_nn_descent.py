"""GPU NN-descent (synchronous rounds; Sec. III-B.1 names NN-descent for the initial graph) against
the CPU oracle, through the C ABI.  A round's result is a set property (the k best of a pool of
nodes), so on integer data, where fp32 distances are exact in any order, lists and distances
must match bit for bit after any number of rounds; on float data the usual search bars apply."""
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


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("n,dim,k,s,rounds", [
    (6_000, 128, 64, 16, 0),      # only the random lists
    (6_000, 128, 64, 16, 1),
    (6_000, 128, 64, 16, 3),
    (4_000, 32, 100, 32, 2),      # two list registers, a ragged second chunk of every row
    (4_000, 32, 16, 4, 5),
    (3_000, 16, 130, 64, 2),      # four list registers, the largest sample
    (300, 16, 299, 8, 2),         # k = N - 1: every list ends up complete
])
def test_rounds_bit_exact_on_integer_data(cagra, n, dim, k, s, rounds):
    import torch
    print(f"case nn-descent sift-like n={n} dim={dim} k={k} s={s} rounds={rounds}", flush=True)
    base = datagen.sift_like(n, dim, 16, seed=6, stream=1)
    ids, dists = cagra.nn_descent(torch.from_numpy(base).cuda(), k, rounds, s, cagra.L2, seed=31)
    r_ids, r_d = oracle.nn_descent(base, k, rounds, s, oracle.L2, seed=31)
    np.testing.assert_array_equal(_u32(ids), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)


@pytest.mark.parametrize("name,n,k,s", [("deep1m", 8_000, 64, 32), ("glove200", 5_000, 32, 16)])
def test_float_data_within_the_search_bars(cagra, name, n, k, s):
    import torch
    print(f"case nn-descent {name} n={n} k={k} s={s}", flush=True)
    w = datagen.workload(name, n=n, n_queries=1)
    ids, dists = cagra.nn_descent(torch.from_numpy(w.base).cuda(), k, 4, s, w.metric, seed=8)
    r_ids, r_d = oracle.nn_descent(w.base, k, 4, s, w.metric, seed=8)
    got, gd = _u32(ids), dists.cpu().numpy()
    agree = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(got, r_ids)) / float(r_ids.size)
    assert agree >= 0.995, f"id agreement {agree}"
    same = got == r_ids
    denom = np.maximum(np.abs(r_d), 1.0 if w.metric == oracle.IP else 0.0)
    rel = np.abs(gd - r_d)[same] / np.maximum(denom[same], 1e-30)
    assert rel.max() <= 1e-5
    # rows sorted, unique, without the node itself
    assert np.all(np.diff(gd, axis=1) >= 0)
    srt = np.sort(got, axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1]) and not np.any(got == np.arange(n, dtype=np.uint32)[:, None])
    exact = oracle.knn_graph(w.base, k, w.metric)
    rec = np.mean([len(set(a.tolist()) & set(e.tolist())) for a, e in zip(got, exact)]) / k
    print(f"  recall of the k-NN lists after 4 rounds {rec:.4f}", flush=True)
    assert rec > 0.85


def test_build_from_nn_descent_and_rejections(cagra):
    import torch
    n, d = 8_000, 32
    base = datagen.sift_like(n, 64, 16, seed=7, stream=1)
    bd = torch.from_numpy(base).cuda()
    g = cagra.build(bd, d, 0, cagra.L2, nn_descent=True, nnd_rounds=5, nnd_sample=16, seed=3)
    k_ids, k_d = oracle.nn_descent(base, 2 * d, 5, 16, oracle.L2, seed=3)
    np.testing.assert_array_equal(_u32(g), oracle.optimize(k_ids, d))
    g2 = cagra.build(bd, d, 0, cagra.L2, reorder=cagra.REORDER_DISTANCE, nn_descent=True, nnd_rounds=5,
                     nnd_sample=16, seed=3)
    np.testing.assert_array_equal(_u32(g2), oracle.optimize(k_ids, d, g0_dist=k_d))
    # automatic rounds and sample: the lists are close to the exact ones, and the graph searches well
    ids, _ = cagra.nn_descent(bd, 2 * d)
    exact = oracle.knn_graph(base, 2 * d)
    rec = np.mean([len(set(a.tolist()) & set(e.tolist())) for a, e in zip(_u32(ids), exact)]) / (2 * d)
    print(f"  recall of the k-NN lists, automatic parameters: {rec:.4f}", flush=True)
    assert rec > 0.97
    for kw in (dict(k=0), dict(k=n), dict(k=16, sample=17), dict(k=16, sample=65), dict(k=600)):
        with pytest.raises(cagra.CagraError):
            cagra.nn_descent(bd, kw["k"], 2, kw.get("sample", 0))
    torch.cuda.synchronize()
