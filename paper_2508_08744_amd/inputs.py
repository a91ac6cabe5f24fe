"""Seeded synthetic inputs shaped like the paper's workloads (Table 2).

Holds no arithmetic of the method itself: only Gaussian-mixture point clouds.
Both the HIP path's tests/bench and the CPU oracle's tests draw from here.
The public datasets the paper uses (SIFT, Gist, Deep, ...) are not available;
these stand in for them by shape, value range and cluster structure.
"""
from __future__ import annotations

import numpy as np

DATA_SEED_BASE = 250808744

# name: (n, d, k, metric, components)
CONFIGS = {
    "C1": dict(n=10_000, d=32, k=16, metric="l2", comps=10),
    "C2": dict(n=1_000_000, d=128, k=32, metric="l2", comps=1000),
    "C3": dict(n=1_000_000, d=960, k=32, metric="l2", comps=500),
    "C4": dict(n=10_000_000, d=96, k=32, metric="cosine", comps=10_000),
    "C5": dict(n=100_000_000, d=96, k=32, metric="l2", comps=10_000),
}


def _mixture(rng, n, d, centers, sigma, chunk=1 << 18):
    out = np.empty((n, d), dtype=np.float32)
    ncomp = centers.shape[0]
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        comp = rng.integers(0, ncomp, size=e - s)
        out[s:e] = centers[comp] + sigma * rng.standard_normal((e - s, d), dtype=np.float32)
    return out


def make(config: str, n: int | None = None, seed: int | None = None, d: int | None = None,
         comps: int | None = None) -> np.ndarray:
    """Row-major fp32 ``n x d`` points of the named configuration.

    ``n``/``d``/``comps`` override the configuration's size (same generator, smaller
    draw) for tests and for the bounded CPU-baseline sample.
    """
    cfg = CONFIGS[config]
    idx = int(config[1:])
    n = cfg["n"] if n is None else n
    d = cfg["d"] if d is None else d
    ncomp = cfg["comps"] if comps is None else comps
    rng = np.random.Generator(np.random.PCG64(DATA_SEED_BASE + idx if seed is None else seed))
    if config == "C1":
        centers = rng.uniform(-1.0, 1.0, size=(ncomp, d)).astype(np.float32)
        return _mixture(rng, n, d, centers, np.float32(0.15))
    if config == "C2":
        # byte-valued features: round and clip to [0, 255], stored as fp32
        centers = rng.uniform(0.0, 255.0, size=(ncomp, d)).astype(np.float32)
        X = _mixture(rng, n, d, centers, np.float32(20.0))
        np.rint(X, out=X)
        np.clip(X, 0.0, 255.0, out=X)
        return X
    if config == "C3":
        centers = rng.standard_normal((ncomp, d), dtype=np.float32)
        X = _mixture(rng, n, d, centers, np.float32(0.3))
        lo = X.min(axis=0, keepdims=True)
        hi = X.max(axis=0, keepdims=True)
        X -= lo
        X /= np.maximum(hi - lo, np.float32(1e-12))
        return X
    if config in ("C4", "C5"):
        centers = rng.standard_normal((ncomp, d), dtype=np.float32)
        X = _mixture(rng, n, d, centers, np.float32(0.3))
        X /= np.linalg.norm(X, axis=1, keepdims=True).astype(np.float32)
        return X
    raise KeyError(config)


def sample_rows(n: int, q: int, seed: int = 7) -> np.ndarray:
    """Fixed random sample of row indices used for ground-truth recall."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if q >= n:
        return np.arange(n, dtype=np.int64)
    return np.sort(rng.choice(n, size=q, replace=False)).astype(np.int64)


def make_on_device(config: str, device, n: int | None = None, seed: int | None = None, chunk: int = 1 << 21):
    """The C4 / C5 recipe (unit-norm Gaussian mixture) drawn on the device with torch's generator, in
    chunks, for sizes the host should not have to hold (1e8 x 96 fp32 is 38.4 GB).  Same distribution
    as ``make``, other random numbers: no oracle input comes from here."""
    import torch
    if config not in ("C4", "C5"):
        raise KeyError(config)
    cfg = CONFIGS[config]
    idx = int(config[1:])
    n = cfg["n"] if n is None else n
    d, ncomp = cfg["d"], cfg["comps"]
    gen = torch.Generator(device=device).manual_seed(DATA_SEED_BASE + idx if seed is None else seed)
    centers = torch.randn((ncomp, d), generator=gen, device=device, dtype=torch.float32)
    X = torch.empty((n, d), device=device, dtype=torch.float32)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        comp = torch.randint(0, ncomp, (e - s,), generator=gen, device=device)
        x = centers[comp] + 0.3 * torch.randn((e - s, d), generator=gen, device=device, dtype=torch.float32)
        x /= x.norm(dim=1, keepdim=True)
        X[s:e] = x
    return X
