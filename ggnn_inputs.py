"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle checks.

This module only draws random data (numpy / torch generators); it contains none of
the method's arithmetic and imports neither the oracle nor the HIP binding.

The public ANN benchmark sets the paper measures on are not available here; these
generators produce stand-ins with the same shapes, value ranges and cluster
structure (mixtures of Gaussians for SIFT-like integer-valued vectors, a random
linear map with a decaying spectrum for DEEP-like unit vectors, a von Mises-Fisher
mixture with log-normal norms for GloVe-like vectors).
"""
from __future__ import annotations

import numpy as np

CONFIGS = {
    # name: generator kind and the build / query parameters of the workload
    "sift10k": dict(kind="gmm", N=10_000, D=128, Q=1_000, components=32, sigma=20.0, dtype="f32",
                    metric="l2", K=24, levels=3, k=10, beam=64, data_seed=1001, query_seed=2001),
    "sift1m": dict(kind="gmm", N=1_000_000, D=128, Q=10_000, components=1024, sigma=25.0, dtype="f32",
                   metric="l2", K=24, levels=4, k=10, beam=10, data_seed=1002, query_seed=2002),
    "deep1m": dict(kind="spectrum", N=1_000_000, D=96, Q=10_000, dtype="f32",
                   metric="l2", K=24, levels=4, k=10, beam=10, data_seed=1003, query_seed=2003),
    "glove1m": dict(kind="vmf", N=1_200_000, D=100, Q=10_000, components=2000, kappa=20.0, norm_sigma=0.5,
                    dtype="f32", metric="cosine", K=40, levels=4, k=10, beam=10, data_seed=1004, query_seed=2004),
    # a high-dimensional configuration in the shape of GIST1M (960 floats per vector, 1 000 queries)
    "gist1m": dict(kind="spectrum", N=1_000_000, D=960, Q=1_000, dtype="f32",
                   metric="l2", K=24, levels=4, k=10, beam=10, data_seed=1006, query_seed=2006),
    "sift100m_u8": dict(kind="gmm", N=100_000_000, D=128, Q=10_000, components=65536, sigma=25.0, dtype="u8",
                        metric="l2", K=24, levels=4, k=10, beam=10, data_seed=1005, query_seed=2005),
}


def _gmm_centres(components: int, D: int, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.uniform(0.0, 255.0, size=(components, D)).astype(np.float32)


def gmm_int(n: int, D: int, components: int, sigma: float, centre_seed: int, draw_seed: int,
            dtype: str = "f32", chunk: int = 262_144) -> np.ndarray:
    """Integer-valued vectors in [0,255]: centres ~ U[0,255]^D, uniform component choice,
    isotropic Gaussian noise, clipped and rounded."""
    centres = _gmm_centres(components, D, centre_seed)
    rng = np.random.default_rng(draw_seed)
    out = np.empty((n, D), dtype=np.uint8 if dtype == "u8" else np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        comp = rng.integers(0, components, size=hi - lo)
        x = centres[comp] + rng.standard_normal((hi - lo, D), dtype=np.float32) * np.float32(sigma)
        x = np.rint(np.clip(x, 0.0, 255.0))
        out[lo:hi] = x.astype(out.dtype)
    return out


def _orthogonal(D: int, rng: np.random.Generator) -> np.ndarray:
    q, r = np.linalg.qr(rng.standard_normal((D, D)))
    return q * np.sign(np.diag(r))


def spectrum_unit(n: int, D: int, map_seed: int, draw_seed: int, chunk: int = 262_144) -> np.ndarray:
    """Unit vectors: i.i.d. N(0,1) passed through U diag(i^-1/2) V^T, then normalised."""
    rng = np.random.default_rng(map_seed)
    U = _orthogonal(D, rng)
    V = _orthogonal(D, rng)
    A = (U * (1.0 / np.sqrt(np.arange(1, D + 1)))) @ V.T
    A = A.astype(np.float32)
    rng = np.random.default_rng(draw_seed)
    out = np.empty((n, D), dtype=np.float32)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        x = rng.standard_normal((hi - lo, D), dtype=np.float32) @ A.T
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        out[lo:hi] = x
    return out


def vmf_lognormal(n: int, D: int, components: int, kappa: float, norm_sigma: float, centre_seed: int,
                  draw_seed: int, chunk: int = 131_072) -> np.ndarray:
    """Directions from a mixture of von Mises-Fisher lobes (Wood's rejection sampler for
    the cosine to the mean direction, uniform tangent component) times log-normal norms."""
    rng = np.random.default_rng(centre_seed)
    mu = rng.standard_normal((components, D))
    mu /= np.linalg.norm(mu, axis=1, keepdims=True)
    rng = np.random.default_rng(draw_seed)
    out = np.empty((n, D), dtype=np.float32)
    b = (-2.0 * kappa + np.sqrt(4.0 * kappa * kappa + (D - 1.0) ** 2)) / (D - 1.0)
    x0 = (1.0 - b) / (1.0 + b)
    c = kappa * x0 + (D - 1.0) * np.log(1.0 - x0 * x0)
    for lo in range(0, n, chunk):
        m = min(n, lo + chunk) - lo
        w = np.empty(m)
        todo = np.arange(m)
        while todo.size:
            z = rng.beta((D - 1.0) / 2.0, (D - 1.0) / 2.0, size=todo.size)
            u = rng.uniform(size=todo.size)
            cand = (1.0 - (1.0 + b) * z) / (1.0 - (1.0 - b) * z)
            ok = kappa * cand + (D - 1.0) * np.log(1.0 - x0 * cand) - c >= np.log(u)
            w[todo[ok]] = cand[ok]
            todo = todo[~ok]
        comp = rng.integers(0, components, size=m)
        m_dir = mu[comp]
        v = rng.standard_normal((m, D))
        v -= (v * m_dir).sum(1, keepdims=True) * m_dir
        v /= np.linalg.norm(v, axis=1, keepdims=True)
        x = w[:, None] * m_dir + np.sqrt(np.maximum(0.0, 1.0 - w * w))[:, None] * v
        norms = np.exp(rng.normal(0.0, norm_sigma, size=m))
        out[lo:lo + m] = (x * norms[:, None]).astype(np.float32)
    return out


def make(name: str, n: int | None = None, q: int | None = None):
    """Returns (base, queries, cfg) for one of CONFIGS; n / q override the sizes (the
    distribution, and for a prefix the data, stay the same)."""
    cfg = dict(CONFIGS[name])
    N = cfg["N"] if n is None else n
    Q = cfg["Q"] if q is None else q
    cfg["N"], cfg["Q"] = N, Q
    if cfg["kind"] == "gmm":
        base = gmm_int(N, cfg["D"], cfg["components"], cfg["sigma"], cfg["data_seed"], cfg["data_seed"] + 1, cfg["dtype"])
        queries = gmm_int(Q, cfg["D"], cfg["components"], cfg["sigma"], cfg["data_seed"], cfg["query_seed"], cfg["dtype"])
    elif cfg["kind"] == "spectrum":
        base = spectrum_unit(N, cfg["D"], cfg["data_seed"], cfg["data_seed"] + 1)
        queries = spectrum_unit(Q, cfg["D"], cfg["data_seed"], cfg["query_seed"])
    elif cfg["kind"] == "vmf":
        base = vmf_lognormal(N, cfg["D"], cfg["components"], cfg["kappa"], cfg["norm_sigma"], cfg["data_seed"], cfg["data_seed"] + 1)
        queries = vmf_lognormal(Q, cfg["D"], cfg["components"], cfg["kappa"], cfg["norm_sigma"], cfg["data_seed"], cfg["query_seed"])
    else:
        raise ValueError(cfg["kind"])
    return base, queries, cfg


def gmm_int_torch(n: int, D: int, components: int, sigma: float, centre_seed: int, draw_seed: int,
                  device, dtype: str = "u8", chunk: int = 4_194_304):
    """Same distribution as gmm_int, drawn with torch on `device` (for sets too large to
    ship from the host).  Not bit-identical to the numpy generator."""
    import torch

    centres = torch.from_numpy(_gmm_centres(components, D, centre_seed)).to(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(draw_seed)
    out = torch.empty((n, D), dtype=torch.uint8 if dtype == "u8" else torch.float32, device=device)
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        comp = torch.randint(0, components, (hi - lo,), generator=gen, device=device)
        x = centres[comp] + torch.randn((hi - lo, D), generator=gen, device=device) * sigma
        out[lo:hi] = x.clamp_(0.0, 255.0).round_().to(out.dtype)
    return out
