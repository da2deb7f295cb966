"""Seeded synthetic inputs for the ASGD K-Means path (no method arithmetic here).

The paper builds its synthetic collection by sampling k cluster centres and then
drawing every sample from a distribution attached to one centre, with overlap set
by distance and variance parameters it never prints (Section 5.3, "Synthetic Data
Sets").  These generators follow that recipe with the parameters of the five
benchmark workloads; they stand in for the paper's synthetic sets and, for the
d=128 workload, for its HOG codebook features (Section 5.3, "Image
Classification"), which are not public.

This module is the only code shared by the HIP path's callers and the CPU oracle's
callers: it produces bytes, nothing else.  Both sides must be fed the SAME array
(generate once, hand it to both), never two independently generated copies.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    N: int            # samples
    d: int            # dimensions
    k: int            # centroids (and mixture components)
    W: int            # workers
    b: int            # mini-batch size
    lr: float         # step size epsilon
    E: int            # exchange interval in mini-batches
    epochs: int
    sigma: float      # isotropic std of every component
    centres: str      # "uniform10" | "sphere10"
    weights: str      # "equal" | "zipf1.1"
    data_seed: int = 1234
    schedule_seed: int = 1

    @property
    def H(self) -> int:          # shard length, Alg. 5, partition of the data
        return self.N // self.W

    @property
    def S(self) -> int:          # mini-batch steps per epoch (tail of a shard is dropped)
        return self.H // self.b

    @property
    def processed_per_epoch(self) -> int:
        return self.W * self.S * self.b

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five benchmark workloads (index = config number).
CONFIGS = (
    Workload("cfg0_tiny", 100_000, 10, 10, 4, 500, 0.05, 4, 5, 1.0, "uniform10", "equal"),
    Workload("cfg1_streaming", 100_000_000, 10, 10, 1024, 1000, 0.05, 8, 1, 1.0, "uniform10", "equal"),
    Workload("cfg2_wider", 20_000_000, 100, 100, 512, 2000, 0.02, 8, 2, 1.0, "uniform10", "zipf1.1"),
    Workload("cfg3_hbm_scale", 2_500_000_000, 10, 10, 4096, 1000, 0.05, 16, 1, 2.0, "uniform10", "equal"),
    Workload("cfg4_contraction", 5_000_000, 128, 1024, 256, 4096, 0.01, 4, 2, 1.0, "sphere10", "equal"),
)


def mixture_parameters(wl: Workload):
    """Centres (k x d, float32) and component probabilities (k, float64) of a workload."""
    rng = np.random.default_rng([wl.data_seed, 0xC0FFEE])
    if wl.centres == "uniform10":
        c = rng.uniform(0.0, 10.0, size=(wl.k, wl.d))
    elif wl.centres == "sphere10":
        g = rng.standard_normal((wl.k, wl.d))
        c = 10.0 * g / np.linalg.norm(g, axis=1, keepdims=True)
    else:
        raise ValueError(wl.centres)
    if wl.weights == "equal":
        p = np.full(wl.k, 1.0 / wl.k)
    elif wl.weights == "zipf1.1":
        p = 1.0 / np.arange(1, wl.k + 1, dtype=np.float64) ** 1.1
        p /= p.sum()
    else:
        raise ValueError(wl.weights)
    return c.astype(np.float32), p


def generate_host(wl: Workload, chunk_rows: int = 1 << 20) -> np.ndarray:
    """N x d float32 row-major samples on the host (NumPy generator, seeded)."""
    centres, p = mixture_parameters(wl)
    rng = np.random.default_rng([wl.data_seed, 1])
    X = np.empty((wl.N, wl.d), dtype=np.float32)
    for lo in range(0, wl.N, chunk_rows):
        hi = min(wl.N, lo + chunk_rows)
        comp = rng.choice(wl.k, size=hi - lo, p=p)
        noise = rng.standard_normal((hi - lo, wl.d), dtype=np.float32)
        X[lo:hi] = centres[comp] + np.float32(wl.sigma) * noise
    return X


def generate_device(wl: Workload, device="cuda:0", chunk_rows: int = 1 << 24):
    """N x d float32 row-major samples generated chunk-wise in device memory (torch tensor).

    Uses torch's seeded device generator only to fill memory.  The bytes differ from
    `generate_host`; a caller that also needs them on the host copies this tensor back.
    """
    import torch

    centres, p = mixture_parameters(wl)
    gen = torch.Generator(device=device)
    gen.manual_seed(wl.data_seed)
    c_dev = torch.from_numpy(centres).to(device)
    p_dev = torch.from_numpy(p).to(device=device, dtype=torch.float32)
    X = torch.empty((wl.N, wl.d), dtype=torch.float32, device=device)
    for lo in range(0, wl.N, chunk_rows):
        hi = min(wl.N, lo + chunk_rows)
        comp = torch.multinomial(p_dev, hi - lo, replacement=True, generator=gen)
        out = X[lo:hi]
        out.normal_(0.0, wl.sigma, generator=gen)
        out += c_dev[comp]
        del comp
    return X


def centre_error(w: np.ndarray, wl: Workload) -> float:
    """Error against the generator's centres as the paper uses it for its synthetic data (Sec. 5.3, last
    paragraph: the distance between the centres of the generation step and the centres returned; a relative
    measure only).  The paper gives no formula; reading: for every generated centre the Euclidean distance
    to the nearest returned centroid, averaged.  Evaluation helper on the host, not part of the hot path."""
    c, _ = mixture_parameters(wl)
    c = c.astype(np.float64)
    w = np.asarray(w, dtype=np.float64).reshape(-1, wl.d)
    d2 = ((c[:, None, :] - w[None, :, :]) ** 2).sum(-1)
    return float(np.sqrt(d2.min(1)).mean())
