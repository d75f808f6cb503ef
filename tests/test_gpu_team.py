"""Wave teams (several wavefronts of one workgroup on one query, Sec. IV-C.1) against the CPU oracle, through the
C ABI.  A team splits the candidates of a pass among its wavefronts and keeps one list copy per wavefront;
the result must be that of the one-wavefront search, i.e. the oracle's, bit for bit on integer-valued data."""
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
    rng = np.random.default_rng(4242)
    cases = []
    for i in range(72):
        dim = int(rng.choice([16, 32, 48, 96, 128, 208]))
        degree = int(rng.choice([4, 8, 16, 24, 32, 48, 64]))
        width = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 11, 16, 32, 64]))
        while width * degree > 2048:
            width //= 2
        itopk = int(rng.choice([1, 5, 10, 16, 32, 33, 64, 100, 128, 256, 512]))
        k = int(rng.choice([1, min(10, itopk), itopk]))
        storage = str(rng.choice(["f32", "f32", "f16", "u8"]))
        if storage == "u8" and dim % 16:
            storage = "f16" if dim % 8 == 0 else "f32"
        entries = int(rng.choice([0, 0, 256, 1024, 4096]))
        team = int(rng.choice([0, 0, 4, 8, 16, 32]))
        waves = int(rng.choice([2, 4]))
        cases.append((i, dim, degree, width, itopk, k, storage, entries, team, waves))
    return cases


_built = {}


def _index(dim, degree):
    key = (dim, degree)
    if key not in _built:
        base = datagen.sift_like(2500, dim, 12, seed=700 + dim + degree, stream=1, rank=min(64, dim))
        queries = datagen.sift_like(40, dim, 12, seed=700 + dim + degree, stream=2)
        _built[key] = (base, queries, oracle.build(base, degree, 2 * degree))
    return _built[key]


@pytest.mark.parametrize("i,dim,degree,width,itopk,k,storage,entries,team,waves", _cases())
def test_team_sweep(cagra, i, dim, degree, width, itopk, k, storage, entries, team, waves):
    import torch
    print(f"case team {i}: dim={dim} d={degree} p={width} M={itopk} k={k} {storage} entries={entries} team={team} "
          f"waves={waves}", flush=True)
    base, queries, g = _index(dim, degree)
    dev_base = torch.from_numpy(base).cuda()
    data = dev_base if storage == "f32" else cagra.convert_dataset(dev_base, cagra.F16 if storage == "f16" else cagra.U8)
    opts = cagra.SearchOptions(seed=6000 + i, mode=1, table_entries=entries, team_size=team, waves_per_query=waves)
    plan = cagra.describe(degree, dim, queries.shape[0], k, itopk, width, opts)
    assert plan["waves_per_query"] == waves and plan["table_policy"] == 2
    ids, dists, st = cagra.search(torch.from_numpy(g.view(np.int32)).cuda(), data, torch.from_numpy(queries).cuda(),
                                  k, itopk, width, cagra.L2, opts, return_stats=True)
    r_ids, r_d, r_st = oracle.search(g, base, queries, k, itopk, width, oracle.L2, seed=6000 + i, return_stats=True)
    np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
    st = st.cpu().numpy().view(np.uint32)
    np.testing.assert_array_equal(st[:, :2], r_st[:, :2])
    assert np.all(st[:, 2] >= r_st[:, 2]) and not np.any(st[:, 3] & 3)


def test_team_rejections(cagra):
    import torch
    base, queries, g = _index(32, 16)
    gd, bd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(base).cuda(), torch.from_numpy(queries).cuda()
    for bad in (cagra.SearchOptions(mode=1, waves_per_query=3), cagra.SearchOptions(mode=1, waves_per_query=8),
                cagra.SearchOptions(mode=1, waves_per_query=2, table_policy=1),       # teams share a replacement table
                cagra.SearchOptions(mode=1, waves_per_query=4, hash_bits=12)):
        with pytest.raises(cagra.CagraError):
            cagra.search(gd, bd, qd, 10, 64, 2, cagra.L2, bad)
    torch.cuda.synchronize()


def test_small_batches_get_teams_automatically(cagra):
    import torch
    base, queries, g = _index(32, 32)
    n_cu_plus = 40                       # far fewer queries than compute units
    plan = cagra.describe(32, 32, n_cu_plus, 10, 64, 8, cagra.SearchOptions(mode=1))
    assert plan["waves_per_query"] == 4
    assert cagra.describe(32, 32, 100_000, 10, 64, 8, cagra.SearchOptions(mode=1))["waves_per_query"] == 1
    assert cagra.describe(32, 32, n_cu_plus, 10, 64, 2, cagra.SearchOptions(mode=1))["waves_per_query"] == 1   # 64 candidates
    assert cagra.describe(32, 32, n_cu_plus, 10, 64, 8, cagra.SearchOptions(mode=1, table_policy=1))["waves_per_query"] == 1
    gd, bd, qd = torch.from_numpy(g.view(np.int32)).cuda(), torch.from_numpy(base).cuda(), torch.from_numpy(queries).cuda()
    ids, dists = cagra.search(gd, bd, qd, 10, 64, 8, cagra.L2, cagra.SearchOptions(seed=9, mode=1))
    r_ids, r_d = oracle.search(g, base, queries, 10, 64, 8, oracle.L2, seed=9)
    np.testing.assert_array_equal(ids.cpu().numpy().view(np.uint32), r_ids)
    np.testing.assert_array_equal(dists.cpu().numpy(), r_d)
