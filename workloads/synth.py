"""Seeded synthetic inputs shaped like the IVF-TQ paper's workloads.

This module only draws random inputs (database vectors, queries, a Gaussian
matrix to be orthogonalised, k-means initial indices).  It holds none of the
method's arithmetic: no coarse assignment, no rotation, no quantiser (a
workload whose data are specified as unit-norm is scaled here because that is
part of the data's definition, not a step of the method).  Both the
CPU oracle's tests and the HIP path's tests/bench read their inputs from here
so that the two sides see bit-identical fp32 arrays.

The paper measures on public descriptor sets (1M x 128, 10M x 96, 10M x 200;
Section "Streaming Experiments" and the million-scale comparison table).
Those sets are not available here; the mixtures below stand in for them and
only reproduce their shapes and a clustered structure.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def _rng(seed: int, stream: int) -> np.random.Generator:
    """Counter-based generator: one independent Philox stream per purpose."""
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


# stream ids (kept fixed so every consumer sees the same numbers)
_S_MEANS, _S_SIGMA, _S_DB, _S_QUERY, _S_ROT, _S_INIT, _S_SHIFT, _S_SAMPLE = range(8)


@dataclass
class Workload:
    """Shape and distribution of one benchmark configuration."""

    name: str
    n: int                 # database vectors
    d: int                 # dimension
    nlist: int             # coarse cells L
    b: int                 # bits per coordinate
    nq: int                # queries
    k: int                 # results per query
    nprobe: tuple          # probe counts swept
    n_components: int      # mixture components
    train_n: int           # coarse-training sample size
    kmeans_iters: int = 10
    seed: int = 42
    kind: str = "iso"      # iso | iso_var | aniso | aniso_ood
    sigma: float = 0.3     # iso: fixed sigma; aniso: sigma_0
    unit_norm: bool = False
    extra: dict = field(default_factory=dict)


def config_tiny() -> Workload:
    """20k x 64, 16 isotropic components, sigma 0.3, L=64, b=4, seed 0."""
    return Workload("tiny", 20_000, 64, 64, 4, 200, 10, (8,), 16, 20_000,
                    kmeans_iters=10, seed=0, kind="iso", sigma=0.3)


def config_1m() -> Workload:
    """1M x 128, 1000 components with per-component sigma ~ U(0.2, 0.6)."""
    return Workload("1m_d128", 1_000_000, 128, 1024, 4, 10_000, 10,
                    (8, 16, 32, 64), 1000, 100_000, kind="iso_var")


def config_10m_d96(b: int = 4) -> Workload:
    """10M x 96 unit-norm, 4096 anisotropic components (one decade of variances)."""
    return Workload("10m_d96", 10_000_000, 96, 4096, b, 10_000, 10,
                    (16, 32, 64, 128), 4096, 500_000, kind="aniso",
                    sigma=0.5, unit_norm=True)


def config_10m_d200() -> Workload:
    """10M x 200 inner-product search with out-of-distribution queries, k=100."""
    return Workload("10m_d200", 10_000_000, 200, 4096, 4, 10_000, 100,
                    (32, 64, 128), 4096, 500_000, kind="aniso_ood", sigma=0.5)


def scaled(w: Workload, n: int, nq: int | None = None, nlist: int | None = None,
           train_n: int | None = None) -> Workload:
    """Same distribution, smaller counts (for parity cases the oracle finishes fast)."""
    from dataclasses import replace
    return replace(w, n=n, nq=nq if nq is not None else w.nq,
                   nlist=nlist if nlist is not None else w.nlist,
                   train_n=min(train_n if train_n is not None else w.train_n, n))


def _mixture_params(w: Workload):
    means = _rng(w.seed, _S_MEANS).standard_normal((w.n_components, w.d)).astype(np.float32)
    rs = _rng(w.seed, _S_SIGMA)
    if w.kind == "iso":
        sig = np.full((w.n_components, 1), w.sigma, dtype=np.float32)
    elif w.kind == "iso_var":
        sig = rs.uniform(0.2, 0.6, size=(w.n_components, 1)).astype(np.float32)
    else:  # per-component diagonal variances, log-uniform over one decade
        var = (w.sigma ** 2) * np.power(10.0, rs.uniform(-0.5, 0.5, size=(w.n_components, w.d)))
        sig = np.sqrt(var).astype(np.float32)
    return means, sig


def _draw(w: Workload, count: int, stream: int, offset_block: int = 0,
          ood: bool = False, chunk: int = 1 << 18) -> np.ndarray:
    """count points of the mixture; drawn chunk by chunk so memory stays bounded."""
    means, sig = _mixture_params(w)
    out = np.empty((count, w.d), dtype=np.float32)
    if ood:
        dirs = _rng(w.seed, _S_SHIFT).standard_normal((w.n_components, w.d)).astype(np.float32)
        dirs /= np.linalg.norm(dirs, axis=1, keepdims=True)
    pos = 0
    blk = offset_block
    while pos < count:
        m = min(chunk, count - pos)
        r = np.random.Generator(np.random.Philox(key=[int(w.seed), int(stream)],
                                                 counter=[0, 0, 0, blk]))
        comp = r.integers(0, w.n_components, size=m)
        noise = r.standard_normal((m, w.d), dtype=np.float32)
        s = sig[comp]
        mu = means[comp]
        if ood:  # mean moved by half a sigma along a fixed direction, twice the variance
            mu = mu + 0.5 * s.mean(axis=1, keepdims=True) * dirs[comp]
            s = s * np.float32(np.sqrt(2.0))
        x = mu + s * noise
        if w.unit_norm:
            x /= np.linalg.norm(x, axis=1, keepdims=True)
        out[pos:pos + m] = x
        pos += m
        blk += 1
    return out


def database(w: Workload, start: int = 0, count: int | None = None,
             chunk: int = 1 << 18) -> np.ndarray:
    """Rows [start, start+count) of the database; start must be a multiple of chunk."""
    count = w.n - start if count is None else count
    assert start % chunk == 0, "database slices start on chunk boundaries"
    return _draw(w, count, _S_DB, offset_block=start // chunk, chunk=chunk)


def queries(w: Workload, count: int | None = None) -> np.ndarray:
    count = w.nq if count is None else count
    return _draw(w, count, _S_QUERY, ood=(w.kind == "aniso_ood"))


def train_sample_indices(w: Workload, n_available: int | None = None) -> np.ndarray:
    """Sorted indices of the coarse-training sample (all rows when train_n >= n)."""
    n = w.n if n_available is None else n_available
    if w.train_n >= n:
        return np.arange(n, dtype=np.int64)
    idx = _rng(w.seed, _S_SAMPLE).choice(n, size=w.train_n, replace=False)
    return np.sort(idx).astype(np.int64)


def kmeans_init_indices(seed: int, n: int, nlist: int) -> np.ndarray:
    """nlist distinct row indices used as initial k-means centres."""
    return _rng(seed, _S_INIT).choice(n, size=nlist, replace=False).astype(np.int64)


def gaussian_matrix(seed: int, d: int) -> np.ndarray:
    """d x d iid N(0,1) in float64: the raw draw a Haar rotation is built from."""
    return _rng(seed, _S_ROT).standard_normal((d, d))


def random_unit_vectors(seed: int, n: int, d: int, stream: int = 100) -> np.ndarray:
    """n points uniform on the unit sphere (float64)."""
    g = _rng(seed, stream).standard_normal((n, d))
    return g / np.linalg.norm(g, axis=1, keepdims=True)
