"""Seeded generators: mixture database, Zipf-skewed queries.

Everything is keyed by (seed, chunk index) so that any slice of a large
database can be regenerated without materialising the rest.  Streams differ
between CPU and GPU generators of torch; a fixture is always generated and
consumed on one machine, so only per-device reproducibility is needed.
"""
import math

import numpy as np
import torch

from .workloads import WorkloadSpec

GEN_CHUNK = 65536  # vectors per RNG chunk (fixed: part of the recipe)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def mixture_centers(spec: WorkloadSpec, device="cpu") -> torch.Tensor:
    """Mixture centres, coordinates ~ N(0, 1); fp32 [n_centers, d]."""
    g = _gen(device, spec.seed_data * 1_000_003 + 999_983)
    return torch.randn(spec.n_centers, spec.d, generator=g, device=device,
                       dtype=torch.float32)


def _finish(x: torch.Tensor, normalize: bool) -> torch.Tensor:
    if normalize:
        x = x / x.norm(dim=1, keepdim=True).clamp_min(1e-20)
    return x.contiguous()


def database_chunk(spec: WorkloadSpec, centers: torch.Tensor, start: int,
                   count: int) -> torch.Tensor:
    """Vectors [start, start+count) of the database, fp32 [count, d].

    Vector i = centre(u_i) + sigma * N(0, I), u_i uniform over centres,
    L2-normalised when the spec says so.  `start` must be a multiple of
    GEN_CHUNK so chunk seeds line up.
    """
    assert start % GEN_CHUNK == 0
    device = centers.device
    out = []
    done = 0
    while done < count:
        c = (start + done) // GEN_CHUNK
        n_here = min(GEN_CHUNK, spec.n - (start + done), count - done)
        g = _gen(device, spec.seed_data * 1_000_003 + c)
        which = torch.randint(0, spec.n_centers, (GEN_CHUNK,), generator=g,
                              device=device)[:n_here]
        noise = torch.randn(GEN_CHUNK, spec.d, generator=g, device=device,
                            dtype=torch.float32)[:n_here]
        out.append(_finish(centers[which] + spec.sigma * noise, spec.normalize))
        done += n_here
    return torch.cat(out, 0) if len(out) > 1 else out[0]


def zipf_probabilities(n: int, s: float) -> np.ndarray:
    """P(rank r) proportional to r^-s, r = 1..n (float64, sums to 1)."""
    w = np.arange(1, n + 1, dtype=np.float64) ** (-float(s))
    return w / w.sum()


def zipf_center_choice(n_centers: int, s, nq: int, seed: int,
                       perm_seed: int) -> np.ndarray:
    """Centre index for each of nq queries.

    Rank r ~ Zipf(s) over a seeded random permutation of centres; s=None
    gives a uniform choice.  Inverse-CDF sampling with numpy's PCG64.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if s is None:
        return rng.integers(0, n_centers, size=nq, dtype=np.int64)
    perm = np.random.Generator(np.random.PCG64(perm_seed)).permutation(n_centers)
    cdf = np.cumsum(zipf_probabilities(n_centers, s))
    cdf[-1] = 1.0
    ranks = np.searchsorted(cdf, rng.random(nq), side="right")
    ranks = np.minimum(ranks, n_centers - 1)
    return perm[ranks].astype(np.int64)


def make_queries(spec: WorkloadSpec, centers: torch.Tensor, nq: int = None,
                 seed: int = None, perm_seed: int = None):
    """Queries fp32 [nq, d] and the centre each was drawn around."""
    nq = spec.nq if nq is None else nq
    seed = spec.seed_queries if seed is None else seed
    perm_seed = spec.seed_perm if perm_seed is None else perm_seed
    device = centers.device
    which = zipf_center_choice(spec.n_centers, spec.zipf_s, nq, seed, perm_seed)
    g = _gen(device, seed * 1_000_003 + 7)
    noise = torch.randn(nq, spec.d, generator=g, device=device, dtype=torch.float32)
    idx = torch.from_numpy(which).to(device)
    q = _finish(centers[idx] + spec.sigma * noise, spec.normalize)
    return q, which


def harmonic(n: int, s: float) -> float:
    return float(sum(math.pow(r, -s) for r in range(1, n + 1)))
