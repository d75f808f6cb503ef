"""Rows whose width is not a whole number of 16-byte pieces (Sec. IV-B.1 fetches rows in 128-bit loads).

The library takes such rows on a stride rounded up to whole pieces with ZEROS between `dim` and the stride, the form
its conversion call writes; zeros add nothing to a squared distance or an inner product, so every result must equal
the oracle's on the unpadded rows -- bit for bit on integer-valued data, where fp32 sums are exact in any order, and
for the build path (one fused multiply-add per dimension, in order) on any data.
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


def _integer_rows(dim, n, nq):
    """Integer-valued rows 0..255 of any width: columns of the 128-dimensional stand-in, repeated as needed."""
    key = (dim, n, nq)
    if key not in _cache:
        w = datagen.workload("sift1m", n=n, n_queries=nq)
        cols = np.arange(dim) % w.base.shape[1]
        base = np.ascontiguousarray(w.base[:, cols])
        queries = np.ascontiguousarray(w.queries[:, cols])
        g = oracle.build(base, 32, 64, oracle.L2)
        _cache[key] = (base, queries, g)
    return _cache[key]


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


@pytest.mark.parametrize("storage", ["f32", "f16", "u8"])
@pytest.mark.parametrize("dim", [13, 50, 127, 200])
def test_search_over_rows_of_any_width(cagra, dim, storage):
    import torch
    base, queries, g = _integer_rows(dim, 6_000, 150)
    dt = {"f32": cagra.F32, "f16": cagra.F16, "u8": cagra.U8}[storage]
    piece = {"f32": 4, "f16": 8, "u8": 16}[storage]
    rows = cagra.convert_dataset(torch.from_numpy(base).cuda(), dt)
    assert rows.shape == (base.shape[0], dim) and rows.stride(0) == -(-dim // piece) * piece
    # the whole padded matrix: the values, then zeros
    full = torch.as_strided(rows, (rows.shape[0], rows.stride(0)), (rows.stride(0), 1)).cpu().numpy()
    np.testing.assert_array_equal(full[:, :dim].astype(np.float32), base)
    assert not full[:, dim:].any()
    gd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(queries).cuda()
    for metric in (oracle.L2, oracle.IP):
        for k, itopk, width, mode, waves in ((10, 64, 1, 1, 1), (10, 32, 12, 1, 1), (10, 64, 4, 1, 2), (10, 96, 1, 2, 1)):
            print(f"case padded dim={dim} {storage} metric={metric} M={itopk} p={width} mode={mode} waves={waves}", flush=True)
            o = cagra.SearchOptions(seed=5, mode=mode, waves_per_query=waves if mode == 1 else 0,
                                    wg_per_query=1 if mode == 2 else 0)
            ids, dists, st = cagra.search(gd, rows, qd, k, itopk, width, metric, o, return_stats=True)
            r_ids, r_d, r_st = oracle.search(g, base, queries, k, itopk, width, metric, seed=5, return_stats=True)
            np.testing.assert_array_equal(_u32(ids), r_ids)
            np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
            if waves == 1 and mode == 1:
                np.testing.assert_array_equal(_u32(st)[:, :2], r_st[:, :2])
    # a stride that is not whole pieces, or shorter than the rounded width, is refused
    if dim % piece:
        tight = torch.zeros((base.shape[0], dim), dtype=rows.dtype, device="cuda")
        with pytest.raises(cagra.CagraError):
            cagra.search(gd, tight, qd, 10, 64, 1)
    torch.cuda.synchronize()


@pytest.mark.parametrize("dim", [13, 50, 99])
def test_build_over_rows_of_any_width(cagra, dim):
    import torch
    w = datagen.workload("glove200" if dim > 60 else "deep1m", n=5_000, n_queries=40)
    base = np.ascontiguousarray(w.base[:, :dim])
    queries = np.ascontiguousarray(w.queries[:, :dim])
    rows = cagra.convert_dataset(torch.from_numpy(base).cuda(), cagra.F32)
    qrows = cagra.convert_dataset(torch.from_numpy(queries).cuda(), cagra.F32)
    assert rows.stride(0) == (dim + 3) // 4 * 4
    for metric in (oracle.L2, oracle.IP):
        print(f"case padded build dim={dim} metric={metric}", flush=True)
        for algo in (cagra.EXACT_PLAIN, cagra.EXACT_FILTERED):
            ids, dists = cagra.exact_search(rows, qrows, 20, metric, algo=algo)
            r_ids, r_d = oracle.exact_search(base, queries, 20, metric)
            np.testing.assert_array_equal(_u32(ids), r_ids)
            np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
        g = cagra.build(rows, 16, 32, metric)
        np.testing.assert_array_equal(_u32(g), oracle.build(base, 16, 32, metric))
    # NN-descent is compared bit for bit on integer-valued rows (its distances are summed lane-wise)
    whole = datagen.sift_like(3_000, dim, 16, seed=6, stream=1)
    ids, dists = cagra.nn_descent(cagra.convert_dataset(torch.from_numpy(whole).cuda(), cagra.F32), 16, rounds=3, sample=8,
                                  metric=oracle.L2, seed=9)
    r_ids, r_d = oracle.nn_descent(whole, 16, 3, 8, oracle.L2, seed=9)
    np.testing.assert_array_equal(_u32(ids), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    torch.cuda.synchronize()
