"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws numbers. It holds none of the method's arithmetic and is
the one module that both the oracle-side tests and the GPU-side tests/bench
use, so both see the same inputs. The paper's datasets (Glove1.2M etc.) are
not available offline; these inputs take their shape (size, dimension, unit
norm, low cross-dimension correlation, equal per-dimension variance -- the
properties Section 7.8 of the paper names) and stand in for them.

Generation is chunked: chunk c of a stream is drawn from
numpy.random.default_rng([seed, stream, c]) and covers rows
[c * CHUNK, (c+1) * CHUNK), so any slice can be regenerated on its own.
Streams: 0 mixture centers, 1 datapoints, 2 queries, 3 log-norms.
"""
import numpy as np

CHUNK = 1 << 18

STREAM_CENTERS, STREAM_DATA, STREAM_QUERIES, STREAM_NORMS = 0, 1, 2, 3


def _normalize(a):
    nrm = np.linalg.norm(a.astype(np.float64), axis=1, keepdims=True)
    nrm[nrm == 0] = 1.0
    return (a / nrm).astype(np.float32)


def _chunks(n):
    for c in range((n + CHUNK - 1) // CHUNK):
        yield c, c * CHUNK, min(n, (c + 1) * CHUNK)


def gaussian_unit(n, d, seed, stream=STREAM_DATA):
    """i.i.d. N(0,1) rows, L2-normalised (the tiny configuration)."""
    out = np.empty((n, d), np.float32)
    for c, lo, hi in _chunks(n):
        rng = np.random.default_rng([seed, stream, c])
        out[lo:hi] = _normalize(rng.standard_normal((hi - lo, d), dtype=np.float32))
    return out


def mixture_centers(n_comp, d, seed):
    rng = np.random.default_rng([seed, STREAM_CENTERS, 0])
    return _normalize(rng.standard_normal((n_comp, d), dtype=np.float32))


def mixture_chunk(c, rows, d, centers, sigma, seed, stream, lognormal_sigma=None):
    """`rows` rows of chunk c: center of a uniformly drawn component plus
    sigma * N(0, I_d) (sigma per coordinate), L2-normalised; then, if
    lognormal_sigma is given, scaled by exp(N(0, lognormal_sigma^2))."""
    rng = np.random.default_rng([seed, stream, c])
    comp = rng.integers(0, centers.shape[0], size=rows)
    x = centers[comp] + np.float32(sigma) * rng.standard_normal((rows, d), dtype=np.float32)
    x = _normalize(x)
    if lognormal_sigma is not None:
        rn = np.random.default_rng([seed, STREAM_NORMS, c])
        x = (x * np.exp(lognormal_sigma * rn.standard_normal((rows, 1))).astype(np.float32))
        x = x.astype(np.float32)
    return x


def mixture(n, d, n_comp, sigma, seed, stream=STREAM_DATA, lognormal_sigma=None, centers=None):
    if centers is None:
        centers = mixture_centers(n_comp, d, seed)
    out = np.empty((n, d), np.float32)
    for c, lo, hi in _chunks(n):
        out[lo:hi] = mixture_chunk(c, hi - lo, d, centers, sigma, seed, stream, lognormal_sigma)
    return out


# ---- the benchmark configurations ----------------------------------------------------

CONFIGS = {
    # name: n, d, M, bits, T, generator, nq, k, reorder_k
    "tiny": dict(n=10_000, d=32, M=16, bits=4, T=0.2, nq=100, k=10, reorder_k=100,
                 kind="gaussian", seed=0),
    "glove": dict(n=1_183_514, d=100, M=50, bits=4, T=0.2, nq=10_000, k=10, reorder_k=100,
                  kind="mixture", n_comp=1000, sigma=0.3, seed=1),
    # the paper's 100-bit setting on the same data: 25 subspaces of 4 dims x 16 codewords
    "glove100": dict(n=1_183_514, d=100, M=25, bits=4, T=0.2, nq=10_000, k=10, reorder_k=100,
                     kind="mixture", n_comp=1000, sigma=0.3, seed=1),
    # 8-bit codes on the same data: 25 subspaces of 4 dims x 256 codewords (200 bits, 25 B/point)
    "glove8": dict(n=1_183_514, d=100, M=25, bits=8, T=0.2, nq=10_000, k=10, reorder_k=100,
                   kind="mixture", n_comp=1000, sigma=0.3, seed=1),
    "glove_ivf": dict(n=1_183_514, d=100, M=50, bits=4, T=0.2, nq=10_000, k=10, reorder_k=100,
                      kind="mixture", n_comp=1000, sigma=0.3, seed=1, n_leaves=2000,
                      leaves_to_search=100),
    "large4": dict(n=10_000_000, d=128, M=64, bits=4, T=0.2, nq=1024, k=10, reorder_k=200,
                   kind="mixture", n_comp=10_000, sigma=0.3, seed=2),
    "large8": dict(n=50_000_000, d=256, M=32, bits=8, T=0.2, nq=1024, k=100, reorder_k=500,
                   kind="mixture", n_comp=10_000, sigma=0.3, seed=3, lognormal_sigma=0.25),
}


def make_data(cfg, n=None):
    """Datapoints of a configuration (optionally only the first n rows)."""
    n = cfg["n"] if n is None else n
    if cfg["kind"] == "gaussian":
        return gaussian_unit(n, cfg["d"], cfg["seed"])
    return mixture(n, cfg["d"], cfg["n_comp"], cfg["sigma"], cfg["seed"],
                   lognormal_sigma=cfg.get("lognormal_sigma"))


def make_queries(cfg, nq=None):
    """Queries of a configuration: same law as the data, unit norm."""
    nq = cfg["nq"] if nq is None else nq
    if cfg["kind"] == "gaussian":
        return gaussian_unit(nq, cfg["d"], cfg["seed"], stream=STREAM_QUERIES)
    return mixture(nq, cfg["d"], cfg["n_comp"], cfg["sigma"], cfg["seed"], stream=STREAM_QUERIES)
