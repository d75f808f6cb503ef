"""GPU search over a dataset stored as fp16 or uint8 (Sec. IV-C.1, last paragraph; Sec. V-D uses
fp16 storage) against the CPU oracle, through the C ABI.

The kernels widen the stored values to fp32 and accumulate in fp32, so the search over a
narrow dataset is, by definition, the fp32 search over the widened values: the oracle is given
the dataset rounded by numpy (round to nearest even, the same rule the library's conversion
states) and every bar of the fp32 search applies unchanged.  Integer data 0..255 is exact in
both narrow types, so there the results must equal the oracle's on the original fp32 rows
bit for bit.
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
        w = datagen.workload(name, n=n, n_queries=nq)
        g = oracle.build(w.base, degree, 2 * degree, w.metric)
        gt, _ = oracle.exact_search(w.base, w.queries, 10, w.metric)
        _cache[key] = (w, g, gt)
    return _cache[key]


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def test_conversion_rounds_like_numpy(cagra):
    import torch
    rng = np.random.default_rng(3)
    x = rng.normal(0, 40, size=(257, 48)).astype(np.float32)
    # halfway cases, range ends, values beyond the range of either type
    x[0, :12] = [0.5, 1.5, 2.5, 254.5, 255.5, 300.0, -0.5, -3.0, 2049.0, 65504.0, 65520.0, 1e-8]
    x[1, :4] = [np.float32(1) + np.float32(2) ** -11, np.float32(1) + 3 * np.float32(2) ** -11, 6.1e-5, 5.96e-8]
    xd = torch.from_numpy(x).cuda()
    with np.errstate(over="ignore"):
        want16 = x.astype(np.float16)
    got16 = cagra.convert_dataset(xd, cagra.F16).cpu().numpy()
    np.testing.assert_array_equal(got16.view(np.uint16), want16.view(np.uint16))
    want8 = np.clip(np.rint(x), 0, 255).astype(np.uint8)
    np.testing.assert_array_equal(cagra.convert_dataset(xd, cagra.U8).cpu().numpy(), want8)


@pytest.mark.parametrize("dtype_name", ["u8", "f16"])
@pytest.mark.parametrize("k,itopk,width", [(10, 64, 1), (10, 150, 1), (40, 300, 2)])
def test_integer_data_is_exact_in_narrow_storage(cagra, dtype_name, k, itopk, width):
    import torch
    w, g, gt = _setup("sift1m", 20_000, 300, 64)
    print(f"case storage {dtype_name} sift1m k={k} M={itopk} p={width}", flush=True)
    base = torch.from_numpy(w.base).cuda()
    narrow = cagra.convert_dataset(base, cagra.U8 if dtype_name == "u8" else cagra.F16)
    gd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(w.queries).cuda()
    ids, dists, st = cagra.search(gd, narrow, qd, k, itopk, width, w.metric,
                                  cagra.SearchOptions(seed=99, mode=1), return_stats=True)
    r_ids, r_d, r_st = oracle.search(g, w.base, w.queries, k, itopk, width, w.metric, seed=99, return_stats=True)
    np.testing.assert_array_equal(_u32(ids), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    np.testing.assert_array_equal(_u32(st)[:, :2], r_st[:, :2])


@pytest.mark.parametrize("name,degree,itopk,team", [("deep1m", 32, 128, 0), ("deep1m", 32, 64, 4),
                                                    ("deep1m", 32, 64, 16), ("glove200", 64, 128, 0),
                                                    ("tiny", 32, 64, 0)])
def test_fp16_storage_matches_oracle_on_rounded_rows(cagra, name, degree, itopk, team):
    import torch
    n, nq = (10_000, 100) if name == "tiny" else (20_000, 300)
    w, g, gt = _setup(name, n, nq, degree)
    print(f"case storage f16 {name} M={itopk} team={team}", flush=True)
    rounded = w.base.astype(np.float16).astype(np.float32)
    half = cagra.convert_dataset(torch.from_numpy(w.base).cuda(), cagra.F16)
    gd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(w.queries).cuda()
    k = 10
    ids, dists = cagra.search(gd, half, qd, k, itopk, 1, w.metric, cagra.SearchOptions(seed=4, mode=1, team_size=team))
    r_ids, r_d = oracle.search(g, rounded, w.queries, k, itopk, 1, w.metric, seed=4)
    ids_np, d_np = _u32(ids), dists.cpu().numpy()
    agreement = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids_np, r_ids)) / float(r_ids.size)
    assert agreement >= 0.995, f"id agreement {agreement}"
    same = ids_np == r_ids
    denom = np.maximum(np.abs(r_d), 1.0 if w.metric == oracle.IP else 0.0)
    rel = np.abs(d_np - r_d)[same] / np.maximum(denom[same], 1e-30)
    assert rel.max() <= 1e-5, f"distance error {rel.max()}"
    r_half, r_ref = oracle.recall(ids_np, gt), oracle.recall(r_ids, gt)
    assert abs(r_half - r_ref) <= 0.003
    # Sec. V-D: fp16 storage does not cost recall; compare with the fp32 oracle on the original rows
    f_ids, _ = oracle.search(g, w.base, w.queries, k, itopk, 1, w.metric, seed=4)
    r_f32 = oracle.recall(f_ids, gt)
    print(f"  recall f16 {r_half:.4f}  oracle on rounded rows {r_ref:.4f}  fp32 oracle {r_f32:.4f}", flush=True)
    assert abs(r_half - r_f32) <= 0.01


def test_narrow_storage_in_multi_mode_and_rejections(cagra):
    import torch
    w, g, gt = _setup("sift1m", 20_000, 300, 64)
    base = torch.from_numpy(w.base).cuda()
    gd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(w.queries).cuda()
    bytes8 = cagra.convert_dataset(base, cagra.U8)
    # one worker in multi mode is the single search with one parent per pass
    ids, dists = cagra.search(gd, bytes8, qd, 10, 64, 1, w.metric, cagra.SearchOptions(seed=11, mode=2, wg_per_query=1))
    r_ids, r_d = oracle.search(g, w.base, w.queries, 10, 64, 1, w.metric, seed=11)
    np.testing.assert_array_equal(_u32(ids), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    # several workers: invariants and recall close to the lock-step oracle
    ids, dists = cagra.search(gd, bytes8, qd, 10, 128, 1, w.metric, cagra.SearchOptions(seed=11, mode=2, wg_per_query=4))
    ids_np, d_np = _u32(ids), dists.cpu().numpy()
    assert np.all(np.diff(d_np, axis=1) >= 0)
    for b in range(0, 300, 9):
        for t in range(10):
            assert d_np[b, t] == oracle.distance(w.queries[b], w.base[ids_np[b, t]], w.metric)
    o_ids, _ = oracle.search_multi(g, w.base, w.queries, 10, 32, 4, w.metric, seed=11,
                                   max_iterations=oracle.auto_max_iterations(32, 1))
    assert abs(oracle.recall(ids_np, gt) - oracle.recall(o_ids, gt)) <= 0.01
    # a row stride must be whole 16-byte pieces of the storage type: 200 bytes is not (208 with zeros would be)
    wg, gg, _ = _setup("glove200", 20_000, 300, 64)
    gb = torch.from_numpy(wg.base).cuda()
    bad = torch.zeros(gb.shape, dtype=torch.uint8, device="cuda")
    with pytest.raises(cagra.CagraError):
        cagra.search(torch.from_numpy(gg.view(np.int32)).cuda(), bad, torch.from_numpy(wg.queries).cuda(), 10, 64, 1)
    torch.cuda.synchronize()
