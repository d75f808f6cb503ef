"""The synthetic inputs are reproducible and have the value ranges the
workload descriptions promise."""
import numpy as np

from paper_2308_15136_amd import datagen


def test_deterministic_and_prefix_stable():
    a = datagen.workload("tiny", n=3000, n_queries=10)
    b = datagen.workload("tiny", n=1000, n_queries=10)
    np.testing.assert_array_equal(a.base[:1000], b.base)
    np.testing.assert_array_equal(a.queries, b.queries)
    c = datagen.sift_like(70000, 8, 4, seed=1, stream=1)
    d = datagen.sift_like(66000, 8, 4, seed=1, stream=1)
    np.testing.assert_array_equal(c[:66000], d)


def test_value_ranges():
    s = datagen.workload("sift1m", n=5000, n_queries=50)
    assert s.base.dtype == np.float32 and s.base.shape == (5000, 128)
    assert np.all(s.base == np.rint(s.base)) and s.base.min() == 0 and s.base.max() <= 255
    assert (s.base == 0).mean() > 0.1
    for name, dim in (("deep1m", 96), ("glove200", 200)):
        w = datagen.workload(name, n=2000, n_queries=20)
        assert w.base.shape == (2000, dim)
        np.testing.assert_allclose(np.linalg.norm(w.base.astype(np.float64), axis=1), 1.0, atol=1e-6)
    assert datagen.workload("glove200", n=100, n_queries=5).metric == datagen.IP
    # queries are not rows of the base set
    assert not (s.queries[:, None, :] == s.base[None, :200, :]).all(-1).any()
