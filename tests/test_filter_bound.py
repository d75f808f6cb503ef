"""The error bound behind the matrix-core filter of the exhaustive search, checked on the CPU with
numpy's fp16 rounding: for vectors x, q scaled by a power of two that brings the largest magnitude into
[2^13, 2^14) and rounded to fp16, the distance formed from the rounded copies and fp32 norms stays within
    eps = 2 * 1.01 * 2^-10 * |x||q| + (12 dim + 48) * 2^-24 * (|x|^2 + |q|^2)       (squared L2)
    eps = 2 * (1.01 * 2^-10 + (12 dim + 48) * 2^-24) * |x||q|                         (inner product)
of the true distance, with the share of eps that is reserved for the rounding of the exact fp32 chain
and of the MFMA's own accumulation left unused.  The filter keeps a dataset row when its approximate
distance is at most threshold + eps, so a bound that failed here would let it drop true neighbours."""
import numpy as np
import pytest

U = 2.0 ** -24


def _scale(m):
    mx = float(np.max(np.abs(m)))
    if mx == 0.0:
        return 1.0
    return 2.0 ** (13 - int(np.floor(np.log2(mx))))


def _approx(x, q, metric):
    """What the filter computes, its dot product in float64 (the hardware accumulates in fp32: covered by
    the (12 dim + 48) u term, of which this test only grants the part for norms and final additions)."""
    sx, sq = _scale(x), _scale(q)
    x16 = (x * np.float32(sx)).astype(np.float16).astype(np.float64)
    q16 = (q * np.float32(sq)).astype(np.float16).astype(np.float64)
    dot = (q16 @ x16.T) / (sx * sq)
    if metric == "ip":
        return -dot
    nx = np.sum(x.astype(np.float32) ** 2, axis=1, dtype=np.float32).astype(np.float64)
    nq = np.sum(q.astype(np.float32) ** 2, axis=1, dtype=np.float32).astype(np.float64)
    return (nq[:, None] + nx[None, :]) - 2.0 * dot


def _true(x, q, metric):
    x64, q64 = x.astype(np.float64), q.astype(np.float64)
    if metric == "ip":
        return -(q64 @ x64.T)
    return ((q64[:, None, :] - x64[None, :, :]) ** 2).sum(axis=2)


def _cases():
    rng = np.random.default_rng(5)
    out = []
    for dim in (4, 96, 128, 960):
        unit = rng.standard_normal((60, dim)).astype(np.float32)
        unit /= np.linalg.norm(unit, axis=1, keepdims=True)
        out.append((f"unit-norm dim {dim}", unit[:40], unit[40:]))
        ints = rng.integers(0, 256, size=(60, dim)).astype(np.float32)
        out.append((f"integers dim {dim}", ints[:40], ints[40:]))
        mixed = (rng.standard_normal((60, dim)) * 10.0 ** rng.uniform(-3, 3, size=(60, dim))).astype(np.float32)
        out.append((f"magnitudes over six decades dim {dim}", mixed[:40], mixed[40:]))
        sparse = mixed * (rng.random((60, dim)) < 0.1)
        out.append((f"sparse dim {dim}", sparse[:40].astype(np.float32), sparse[40:].astype(np.float32)))
        out.append((f"queries a thousand times larger dim {dim}", unit[:40], unit[40:] * np.float32(1e3)))
        out.append((f"tiny values dim {dim}", unit[:40] * np.float32(1e-9), unit[40:] * np.float32(1e-9)))
    return out


@pytest.mark.parametrize("name,x,q", _cases(), ids=[c[0] for c in _cases()])
@pytest.mark.parametrize("metric", ["l2", "ip"])
def test_fp16_filter_error_bound(name, x, q, metric):
    dim = x.shape[1]
    nx = (x.astype(np.float64) ** 2).sum(axis=1)
    nq = (q.astype(np.float64) ** 2).sum(axis=1)
    g = np.sqrt(nq[:, None] * nx[None, :])
    s = nq[:, None] + nx[None, :]
    c16, c32 = 1.01 * 2.0 ** -10, (12 * dim + 48) * U
    # reserved and not granted here: the chain's own rounding ((2 dim + 4) u S resp. (dim + 2) u g), and the
    # accumulation inside the matrix instruction, whose accumulators start at minus the right-hand side of the
    # test, so that a partial sum is bounded by 1.01 S resp. 2.01 g in scaled units and every one of the dim
    # additions errs by at most 2 u of that (truncation), plus the two roundings of the start value:
    # (4.1 dim + 3) u S resp. (4.1 dim + 3) u g
    if metric == "l2":
        eps = 2 * c16 * g + c32 * s - (2 * dim + 4) * U * s - (4.1 * dim + 3) * U * s
    else:
        eps = 2 * (c16 + c32) * g - (dim + 2) * U * g - (4.1 * dim + 3) * U * g
    err = np.abs(_approx(x, q, metric) - _true(x, q, metric))
    assert np.all(eps >= 0)
    assert np.all(err <= eps), f"{name}: the bound fails for {int(np.sum(err > eps))} pairs"
    # and the bound is not idle: fp16 rounding uses a visible part of it on dense data of moderate dimension
    if "unit-norm" in name and metric == "ip" and dim in (96, 128):
        assert float(np.max(err[eps > 0] / eps[eps > 0])) > 0.02
