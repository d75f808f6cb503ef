"""A seeded sweep of search configurations on small integer-valued data (exact fp32 arithmetic, so
GPU and oracle must agree bit for bit): dimensions that leave team lanes idle, degrees that are not
powers of two, padded row strides, k = itopk, tiny and huge tables, both table policies, every
storage type, all team sizes.  One wavefront per query throughout (tests/test_gpu_team.py covers the teams of
several wavefronts, which small batches would otherwise get automatically)."""
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


def _cases():
    rng = np.random.default_rng(2023)
    cases = []
    for i in range(48):
        dim = int(rng.choice([16, 32, 48, 80, 96, 112, 128, 208, 256, 400]))
        degree = int(rng.choice([4, 6, 10, 16, 24, 32, 48, 64]))
        width = int(rng.choice([1, 1, 2, 3, 4, 7]))
        while width * degree > 256:
            width -= 1
        itopk = int(rng.choice([1, 7, 10, 33, 64, 65, 100, 128, 200, 256, 384, 512]))
        k = int(rng.choice([1, min(10, itopk), itopk]))
        storage = str(rng.choice(["f32", "f32", "f16", "u8"]))
        if storage == "u8" and dim % 16:
            storage = "f16" if dim % 8 == 0 else "f32"
        policy = int(rng.choice([0, 1, 2]))
        entries = int(rng.choice([0, 0, 256, 512, 1024, 2048, 8192]))
        if policy == 1 and entries and itopk + width * degree > entries // 8 * 7:
            entries = 0
        team = int(rng.choice([0, 0, 4, 8, 16, 32]))
        pad = int(rng.choice([0, 0, 16, 64]))
        cases.append((i, dim, degree, width, itopk, k, storage, policy, entries, team, pad))
    # rows longer than one sweep of a team's lanes (more than four 16-byte loads per lane), as for the
    # 960-dimensional descriptors of Table I
    cases += [(48, 960, 16, 1, 64, 10, "f32", 0, 0, 0, 0), (49, 960, 16, 2, 100, 10, "f16", 0, 0, 8, 32),
              (50, 2048, 16, 1, 32, 10, "u8", 1, 0, 4, 0), (51, 1536, 32, 1, 64, 10, "f32", 2, 1024, 16, 0)]
    # a periodic-reset table that just holds the list and two passes (32 + 2 * 96 of 224) but not the seeds and
    # the two passes before the first reset (3 * 96): the automatic interval must be 1, and nothing overflows
    cases += [(52, 16, 24, 4, 32, 32, "f16", 1, 256, 32, 0)]
    return cases


_built = {}


def _index(dim, degree):
    key = (dim, degree)
    if key not in _built:
        base = datagen.sift_like(3000, dim, 12, seed=100 + dim, stream=1, rank=min(64, dim))
        queries = datagen.sift_like(64, dim, 12, seed=100 + dim, stream=2)
        _built[key] = (base, queries, oracle.build(base, degree, 2 * degree))
    return _built[key]


@pytest.mark.parametrize("i,dim,degree,width,itopk,k,storage,policy,entries,team,pad", _cases())
def test_sweep(cagra, i, dim, degree, width, itopk, k, storage, policy, entries, team, pad):
    import torch
    print(f"case sweep {i}: dim={dim} d={degree} p={width} M={itopk} k={k} {storage} policy={policy} "
          f"entries={entries} team={team} pad={pad}", flush=True)
    base, queries, g = _index(dim, degree)
    dev_base = torch.from_numpy(base).cuda()
    data = dev_base if storage == "f32" else cagra.convert_dataset(dev_base, cagra.F16 if storage == "f16" else cagra.U8)
    if pad:                                   # rows further apart than dim: a view into a wider matrix
        wide = torch.zeros((data.shape[0], dim + pad), dtype=data.dtype, device="cuda")
        wide[:, :dim] = data
        data = wide[:, :dim]
        qwide = torch.full((queries.shape[0], dim + 4), 7.0, dtype=torch.float32, device="cuda")
        qwide[:, :dim] = torch.from_numpy(queries).cuda()
        qd = qwide[:, :dim]
    else:
        qd = torch.from_numpy(queries).cuda()
    opts = cagra.SearchOptions(seed=1000 + i, mode=1, table_policy=policy, table_entries=entries, team_size=team,
                               waves_per_query=1)
    ids, dists, st = cagra.search(torch.from_numpy(g.view(np.int32)).cuda(), data, qd, k, itopk, width, cagra.L2, opts,
                                  return_stats=True)
    r_ids, r_d, r_st = oracle.search(g, base, queries, k, itopk, width, oracle.L2, seed=1000 + i, return_stats=True)
    np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    st = st.cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(st[:, :2], r_st[:, :2])
    assert np.all(st[:, 2] >= r_st[:, 2]) and not np.any(st[:, 3] & 2)


# More than 256 candidates per pass (Sec. IV-B.2's large candidate lists): the pass takes them in chunks.
# Ragged last chunks, degrees that do not divide the chunk, both table policies, tables far too small.
_WIDE = [
    # dim, degree, width, itopk, k, storage, policy, entries
    (32, 64, 5, 64, 10, "f32", 0, 0),          # 320
    (48, 96, 5, 128, 10, "f16", 1, 0),         # 480, periodic reset
    (16, 48, 11, 200, 200, "u8", 2, 1024),     # 528, table much smaller than two passes
    (128, 64, 16, 512, 10, "f32", 0, 0),       # 1024
    (32, 32, 64, 256, 100, "f32", 2, 0),       # 2048, the most parents per pass
    (64, 128, 16, 100, 10, "f32", 1, 8192),    # 2048, periodic reset every pass or two
    (32, 24, 40, 33, 7, "f32", 0, 256),        # 960 candidates into a 256-entry table
    (96, 256, 8, 512, 512, "f16", 0, 0),       # 2048 from the largest degree, k = itopk
]

_wide_built = {}


def _wide_index(dim, degree):
    key = (dim, degree)
    if key not in _wide_built:
        base = datagen.sift_like(8000, dim, 12, seed=300 + dim, stream=1, rank=min(64, dim))
        queries = datagen.sift_like(48, dim, 12, seed=300 + dim, stream=2)
        _wide_built[key] = (base, queries, oracle.build(base, degree, 2 * degree))
    return _wide_built[key]


@pytest.mark.parametrize("dim,degree,width,itopk,k,storage,policy,entries", _WIDE)
def test_wide_passes(cagra, dim, degree, width, itopk, k, storage, policy, entries):
    import torch
    print(f"case wide: dim={dim} d={degree} p={width} M={itopk} k={k} {storage} policy={policy} entries={entries}",
          flush=True)
    base, queries, g = _wide_index(dim, degree)
    dev_base = torch.from_numpy(base).cuda()
    data = dev_base if storage == "f32" else cagra.convert_dataset(dev_base, cagra.F16 if storage == "f16" else cagra.U8)
    opts = cagra.SearchOptions(seed=77, mode=1, table_policy=policy, table_entries=entries, waves_per_query=1)
    ids, dists, st = cagra.search(torch.from_numpy(g.view(np.int32)).cuda(), data, torch.from_numpy(queries).cuda(),
                                  k, itopk, width, cagra.L2, opts, return_stats=True)
    r_ids, r_d, r_st = oracle.search(g, base, queries, k, itopk, width, oracle.L2, seed=77, return_stats=True)
    np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    st = st.cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(st[:, :2], r_st[:, :2])
    assert np.all(st[:, 2] >= r_st[:, 2]) and not np.any(st[:, 3] & 2)


def test_wide_limits(cagra):
    import torch
    base, queries, g = _wide_index(32, 64)
    gd, bd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(base).cuda(), torch.from_numpy(queries).cuda()
    one = cagra.SearchOptions(mode=1)
    with pytest.raises(cagra.CagraError):
        cagra.search(gd, bd, qd, 10, 64, 33, cagra.L2, one)        # 2112 candidates
    with pytest.raises(cagra.CagraError):
        cagra.search(gd[:, :16].contiguous(), bd, qd, 10, 128, 65, cagra.L2, one)   # 65 parents
    torch.cuda.synchronize()


def _mixed_cases():
    # a second seeded batch over narrow and wide passes alike (search_width up to 64)
    rng = np.random.default_rng(77)
    cases = []
    for i in range(150):
        dim = int(rng.choice([16, 32, 48, 64, 96, 128, 208]))
        degree = int(rng.choice([4, 8, 16, 24, 32, 48, 64]))
        width = int(rng.choice([1, 2, 3, 4, 5, 6, 8, 11, 16, 23, 32, 64]))
        while width * degree > 2048:
            width //= 2
        itopk = int(rng.choice([1, 5, 10, 16, 32, 33, 64, 100, 128, 256, 512]))
        k = int(rng.choice([1, min(10, itopk), itopk]))
        storage = str(rng.choice(["f32", "f32", "f16", "u8"]))
        if storage == "u8" and dim % 16:
            storage = "f16" if dim % 8 == 0 else "f32"
        policy = int(rng.choice([0, 1, 2]))
        entries = int(rng.choice([0, 0, 256, 1024, 4096, 8192]))
        if policy == 1 and entries and max(itopk + width * degree, 2 * width * degree) > entries // 8 * 7:
            entries = 0                      # a periodic-reset table must hold at least one window
        team = int(rng.choice([0, 0, 4, 8, 16, 32]))
        cases.append((i, dim, degree, width, itopk, k, storage, policy, entries, team))
    return cases


_mixed_built = {}


def _mixed_index(dim, degree):
    key = (dim, degree)
    if key not in _mixed_built:
        base = datagen.sift_like(2500, dim, 12, seed=500 + dim + degree, stream=1, rank=min(64, dim))
        queries = datagen.sift_like(40, dim, 12, seed=500 + dim + degree, stream=2)
        _mixed_built[key] = (base, queries, oracle.build(base, degree, 2 * degree))
    return _mixed_built[key]


@pytest.mark.parametrize("i,dim,degree,width,itopk,k,storage,policy,entries,team", _mixed_cases())
def test_mixed_sweep(cagra, i, dim, degree, width, itopk, k, storage, policy, entries, team):
    import torch
    print(f"case mixed {i}: dim={dim} d={degree} p={width} M={itopk} k={k} {storage} policy={policy} "
          f"entries={entries} team={team}", flush=True)
    base, queries, g = _mixed_index(dim, degree)
    dev_base = torch.from_numpy(base).cuda()
    data = dev_base if storage == "f32" else cagra.convert_dataset(dev_base, cagra.F16 if storage == "f16" else cagra.U8)
    opts = cagra.SearchOptions(seed=4000 + i, mode=1, table_policy=policy, table_entries=entries, team_size=team,
                               waves_per_query=1)
    ids, dists, st = cagra.search(torch.from_numpy(g.view(np.int32)).cuda(), data, torch.from_numpy(queries).cuda(),
                                  k, itopk, width, cagra.L2, opts, return_stats=True)
    r_ids, r_d, r_st = oracle.search(g, base, queries, k, itopk, width, oracle.L2, seed=4000 + i, return_stats=True)
    np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    st = st.cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(st[:, :2], r_st[:, :2])
    assert np.all(st[:, 2] >= r_st[:, 2]) and not np.any(st[:, 3] & 2)


def _float_cases():
    # floating-point rows (unit norm) and both metrics through narrow and wide passes: the bars are the stated
    # ones for data on which rounding can differ (distances within 1e-5, id agreement >= 99.5 % per batch)
    rng = np.random.default_rng(99)
    cases = []
    for i in range(36):
        dim = int(rng.choice([32, 64, 96, 128, 200]))
        degree = int(rng.choice([8, 16, 32, 64]))
        width = int(rng.choice([1, 2, 4, 8, 16, 32]))
        while width * degree > 2048:
            width //= 2
        itopk = int(rng.choice([16, 32, 64, 100, 128, 256]))
        k = int(rng.choice([1, min(10, itopk), min(100, itopk)]))
        metric = int(rng.choice([0, 1]))
        storage = str(rng.choice(["f32", "f32", "f16"]))
        if storage == "f16" and dim % 8:
            storage = "f32"
        waves = int(rng.choice([1, 1, 2, 4]))
        cases.append((i, dim, degree, width, itopk, k, metric, storage, waves))
    return cases


_float_built = {}


def _float_index(dim, degree, metric):
    key = (dim, degree, metric)
    if key not in _float_built:
        base = datagen.unit_mixture(4000, dim, 24, min(32, dim), 1.5, 0.3, seed=900 + dim, stream=1)
        queries = datagen.unit_mixture(100, dim, 24, min(32, dim), 1.5, 0.3, seed=900 + dim, stream=2)
        _float_built[key] = (base, queries, oracle.build(base, degree, 2 * degree, metric))
    return _float_built[key]


@pytest.mark.parametrize("i,dim,degree,width,itopk,k,metric,storage,waves", _float_cases())
def test_float_sweep(cagra, i, dim, degree, width, itopk, k, metric, storage, waves):
    import torch
    print(f"case float {i}: dim={dim} d={degree} p={width} M={itopk} k={k} metric={metric} {storage} waves={waves}", flush=True)
    base, queries, g = _float_index(dim, degree, metric)
    dev_base = torch.from_numpy(base).cuda()
    if storage == "f16":
        data = cagra.convert_dataset(dev_base, cagra.F16)
        ref_base = base.astype(np.float16).astype(np.float32)      # the search over fp16 rows is the search over their values
    else:
        data, ref_base = dev_base, base
    opts = cagra.SearchOptions(seed=8000 + i, mode=1, waves_per_query=waves)
    ids, dists, st = cagra.search(torch.from_numpy(g.view(np.int32)).cuda(), data, torch.from_numpy(queries).cuda(),
                                  k, itopk, width, metric, opts, return_stats=True)
    ids, dists = ids.cpu().numpy().view(np.uint32), dists.cpu().numpy()
    r_ids, r_d = oracle.search(g, ref_base, queries, k, itopk, width, metric, seed=8000 + i)
    agree = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(ids, r_ids)) / float(r_ids.size)
    assert agree >= 0.995, f"id agreement {agree}"
    same = ids == r_ids
    # unit-norm rows and queries: |x||q| = 1, so for the inner product the bar is 1e-5 absolute (a relative bar has
    # no meaning for values that pass through zero); for L2 it is relative
    denom = np.maximum(np.abs(r_d), 1.0) if metric == oracle.IP else np.maximum(np.abs(r_d), 1e-30)
    assert (np.abs(dists - r_d)[same] / denom[same]).max() <= 1e-5
    assert np.all(np.diff(dists, axis=1) >= 0) and not np.any(st.cpu().numpy().view(np.uint32)[:, 3] & 2)
