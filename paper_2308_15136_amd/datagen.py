"""Seeded synthetic inputs shaped like the paper's workloads (Table I).

This module only draws random numbers and shapes them into base/query
matrices.  It holds none of the method's arithmetic (no distances, no graph
logic, no search) so that both the CPU oracle's tests and the HIP path's tests
may take their inputs from it without sharing any code of the method itself.

The paper's datasets (SIFT-1M, DEEP-1M/10M, GloVe-200) are not available
offline; each generator below produces a stand-in with the same shape, value
range and rough cluster structure.  Every draw comes from a Philox stream
keyed by (seed, stream, chunk), so a matrix is reproducible bit for bit on any
machine and independent of how many rows are requested after it.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

_CHUNK = 65536  # rows per independently keyed Philox stream

L2 = 0
IP = 1


def _rng(seed: int, stream: int, chunk: int) -> np.random.Generator:
    # Philox takes a 2-word key and a 4-word counter; the counter's top words
    # name the stream and the chunk so that streams never overlap.
    return np.random.Generator(
        np.random.Philox(key=[seed & 0xFFFFFFFFFFFFFFFF, 0x243F6A8885A308D3],
                         counter=[0, 0, chunk, stream]))


def _chunks(n: int):
    for c, lo in enumerate(range(0, n, _CHUNK)):
        yield c, lo, min(n, lo + _CHUNK)


def _normalize_rows(x: np.ndarray) -> None:
    nrm = np.sqrt(np.einsum("ij,ij->i", x, x, dtype=np.float64))
    nrm[nrm == 0] = 1.0
    x /= nrm[:, None].astype(np.float32)


def gaussian_mixture(n: int, dim: int, n_comp: int, center_std: float, sigma: float,
                     seed: int, stream: int, unit_norm: bool = False,
                     log_var_range: Optional[tuple] = None) -> np.ndarray:
    """Rows drawn from an n_comp-component Gaussian mixture.

    Centres ~ N(0, center_std^2 I).  Within-component noise is sigma * N(0, I),
    or, when log_var_range = (lo, hi) is given, N(0, diag(v_c)) * sigma with the
    per-component per-dimension variances v_c log-uniform in [lo, hi].
    The component table depends on `seed` only; `stream` separates base rows
    from query rows drawn from the same mixture.
    """
    g0 = _rng(seed, 0, 0)
    centers = (g0.standard_normal((n_comp, dim)) * center_std).astype(np.float32)
    if log_var_range is not None:
        lo, hi = log_var_range
        var = np.exp(g0.uniform(np.log(lo), np.log(hi), size=(n_comp, dim)))
        std = (np.sqrt(var) * sigma).astype(np.float32)
    else:
        std = None
    out = np.empty((n, dim), dtype=np.float32)
    for c, lo_r, hi_r in _chunks(n):
        g = _rng(seed, stream, c)
        m = hi_r - lo_r
        # always draw the whole chunk so that a shorter matrix is a prefix of a longer one
        comp = g.integers(0, n_comp, size=_CHUNK)[:m]
        z = g.standard_normal((_CHUNK, dim), dtype=np.float32)[:m]
        if std is None:
            z *= np.float32(sigma)
        else:
            z *= std[comp]
        z += centers[comp]
        out[lo_r:hi_r] = z
    if unit_norm:
        _normalize_rows(out)
    return out


def latent_mixture(n: int, dim: int, n_comp: int, rank: int, spread: float, noise: float,
                   seed: int, stream: int, log_var_range: Optional[tuple] = None) -> np.ndarray:
    """Rows of a Gaussian mixture whose components share a low-dimensional structure.

    A latent point z = mu_c + e lives in R^rank: component means mu_c ~ N(0, spread^2 I),
    e ~ N(0, I) (or N(0, diag(v_c)) with per-component variances log-uniform in
    log_var_range).  The row is z A + noise * N(0, I_dim) with one fixed random map
    A[rank, dim] (entries N(0, 1/rank)).  In R^dim this is a mixture of n_comp Gaussians
    with low-rank-plus-isotropic covariances; neighbouring components overlap when
    `spread` is around 1-2, which keeps the k-NN graph of the rows connected the way
    the graphs of real descriptor sets are, instead of falling apart into islands.
    """
    g0 = _rng(seed, 0, 0)
    mu = (g0.standard_normal((n_comp, rank)) * spread).astype(np.float32)
    A = (g0.standard_normal((rank, dim)) / np.sqrt(rank)).astype(np.float32)
    std = None
    if log_var_range is not None:
        lo, hi = log_var_range
        std = np.sqrt(np.exp(g0.uniform(np.log(lo), np.log(hi), size=(n_comp, rank)))).astype(np.float32)
    out = np.empty((n, dim), dtype=np.float32)
    for c, lo_r, hi_r in _chunks(n):
        g = _rng(seed, stream, c)
        m = hi_r - lo_r
        # always draw the whole chunk so that a shorter matrix is a prefix of a longer one
        comp = g.integers(0, n_comp, size=_CHUNK)[:m]
        z = g.standard_normal((_CHUNK, rank), dtype=np.float32)[:m]
        e = g.standard_normal((_CHUNK, dim), dtype=np.float32)[:m]
        if std is not None:
            z *= std[comp]
        z += mu[comp]
        x = z @ A
        x += np.float32(noise) * e
        out[lo_r:hi_r] = x
    return out


def sift_like(n: int, dim: int, n_comp: int, seed: int, stream: int,
              rank: int = 64, spread: float = 1.5, noise: float = 0.3) -> np.ndarray:
    """Integer-valued rows in 0..255 stored as fp32 (stand-in for SIFT-1M).

    A latent mixture (see latent_mixture) is scaled per dimension (log-normal scales, so
    a few dimensions carry most of the energy), shifted by a heavy-tailed per-dimension
    offset, rounded and clipped to [0, 255].  The clipping at zero leaves many exact
    zeros and a heavy right tail, like gradient-histogram descriptors.
    """
    g0 = _rng(seed, 7, 0)
    dim_scale = (42.0 * np.exp(0.45 * g0.standard_normal(dim))).astype(np.float32)
    offset = (g0.gamma(0.9, 24.0, size=dim) - 6.0).astype(np.float32)
    x = latent_mixture(n, dim, n_comp, rank, spread, noise, seed, stream)
    x *= dim_scale / np.float32(np.sqrt(1.0 + spread * spread))
    x += offset
    np.rint(x, out=x)
    np.clip(x, 0.0, 255.0, out=x)
    return x


def unit_mixture(n: int, dim: int, n_comp: int, rank: int, spread: float, noise: float,
                 seed: int, stream: int, log_var_range: Optional[tuple] = None) -> np.ndarray:
    """Latent Gaussian mixture rows scaled to unit L2 norm (stand-in for DEEP / GloVe)."""
    x = latent_mixture(n, dim, n_comp, rank, spread, noise, seed, stream, log_var_range)
    _normalize_rows(x)
    return x


@dataclass
class Workload:
    """One benchmark / parity configuration: inputs plus the parameters to run it with."""
    name: str
    base: np.ndarray          # [N, dim] fp32, C-contiguous
    queries: np.ndarray       # [B, dim] fp32
    metric: int               # L2 or IP
    degree: int               # d of the final graph
    init_degree: int          # d_init of the exact kNN graph
    k: int
    itopk: tuple              # sweep of M values
    search_width: int = 1
    search_widths: tuple = (1, 2, 4)   # sweep of p values (Sec. IV-A: parents per pass)
    notes: str = ""
    extra: dict = field(default_factory=dict)


def workload(name: str, n: Optional[int] = None, n_queries: Optional[int] = None) -> Workload:
    """Build one of the named configurations; n / n_queries shrink it (prefix-stable:
    a smaller n yields the first n rows of the full matrix)."""
    if name == "tiny":          # plumbing: 10k x 32, 16 isotropic components
        n = n or 10_000
        b = n_queries or 100
        base = gaussian_mixture(n, 32, 16, 2.0, 1.0, seed=0, stream=1)
        qs = gaussian_mixture(b, 32, 16, 2.0, 1.0, seed=0, stream=2)
        return Workload(name, base, qs, L2, 32, 64, 10, (64,))
    if name == "sift1m":        # large batch: 1M x 128, integers 0..255
        n = n or 1_000_000
        b = n_queries or 10_000
        base = sift_like(n, 128, 256, seed=1, stream=1)
        qs = sift_like(b, 128, 256, seed=1, stream=2)
        # itopk 32..256 is the sweep the benchmark configuration names; the shorter lists are reported beside it
        return Workload(name, base, qs, L2, 64, 128, 10, (32, 48, 64, 96, 128, 192, 256),
                        search_widths=(1, 2, 4, 5, 6, 7, 8), extra={"short_itopk": (10, 12, 16, 20, 24)})
    if name == "deep1m":        # large batch, lower dim: 1M x 96 unit norm
        n = n or 1_000_000
        b = n_queries or 10_000
        base = unit_mixture(n, 96, 1024, 40, 1.5, 0.1, seed=2, stream=1)
        qs = unit_mixture(b, 96, 1024, 40, 1.5, 0.1, seed=2, stream=2)
        return Workload(name, base, qs, L2, 32, 64, 10, (16, 32, 64, 128, 256, 512), search_widths=(1, 2, 4, 8, 16, 32))
    if name == "glove200":      # angular, higher dim: 1,183,514 x 200, inner product
        n = n or 1_183_514
        b = n_queries or 10_000
        kw = dict(seed=3, log_var_range=(0.1, 10.0))
        base = unit_mixture(n, 200, 2000, 128, 1.5, 0.1, stream=1, **kw)
        qs = unit_mixture(b, 200, 2000, 128, 1.5, 0.1, stream=2, **kw)
        return Workload(name, base, qs, IP, 64, 128, 10, (32, 64, 128, 256, 512), search_widths=(1, 2, 4, 8, 16))
    if name == "deep10m":       # small batch / scale: 10M x 96 unit norm
        n = n or 10_000_000
        b = n_queries or 1_000
        base = unit_mixture(n, 96, 4096, 40, 1.5, 0.1, seed=4, stream=1)
        qs = unit_mixture(b, 96, 4096, 40, 1.5, 0.1, seed=4, stream=2)
        return Workload(name, base, qs, L2, 32, 64, 10, (64, 128, 256), search_width=4, search_widths=(1, 2, 4, 8, 16))
    raise ValueError(f"unknown workload {name!r}")


WORKLOADS = ("tiny", "sift1m", "deep1m", "glove200", "deep10m")
