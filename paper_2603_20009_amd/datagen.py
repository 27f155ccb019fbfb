"""Seeded synthetic embedding-shaped inputs (no k-means arithmetic in here).

The paper measures on public embedding collections that are not available to
this build; these generators produce stand-ins with the same shapes and the
properties that matter for the method: fp32 rows of unit L2 norm, a mixture
structure (so clusters exist) and a skewed per-dimension variance (which the
random rotation then spreads out).

Two recipes, both a Gaussian mixture followed by row normalisation:

``linear``   means ~ N(0, I); within-component std decays linearly from 1.0
             (first dimension) to 0.1 (last dimension).
``embed``    per-dimension variance v_j = 1 / (1 + j/64); means ~ N(0, v_j);
             within-component noise sigma_w * sqrt(v_j) * N(0, 1).

The same function runs on the CPU (numpy-backed torch generator) and on a GPU
(device generator, chunked so that 10^7 rows never need a second full copy).
A CPU call and a GPU call with the same seed do NOT give the same numbers:
whichever buffer is generated is the one handed to both the library and the
oracle.
"""
from __future__ import annotations

import torch

SIGMA_W = 0.5  # within/between ratio of the ``embed`` recipe


def mixture(n: int, d: int, components: int, seed: int, recipe: str = "embed", device: str = "cpu",
            chunk: int = 1 << 18, return_labels: bool = False, sample_seed: int | None = None):
    """n x d fp32 rows of unit norm drawn from a `components`-component mixture.

    `seed` fixes the mixture (its means); `sample_seed` (default: seed + 1) fixes the rows drawn from
    it, so that held-out rows of the same mixture are a second call with another `sample_seed`."""
    dev = torch.device(device)
    g = torch.Generator(device=dev)
    g.manual_seed(int(seed))
    j = torch.arange(d, device=dev, dtype=torch.float32)
    if recipe == "linear":
        mean_scale = torch.ones(d, device=dev)
        noise_scale = 1.0 - 0.9 * j / max(d - 1, 1)
    elif recipe == "embed":
        v = 1.0 / (1.0 + j / 64.0)
        mean_scale = v.sqrt()
        noise_scale = SIGMA_W * v.sqrt()
    else:
        raise ValueError(recipe)
    means = torch.randn(components, d, generator=g, device=dev, dtype=torch.float32) * mean_scale
    g.manual_seed(int(seed) + 1 if sample_seed is None else int(sample_seed))
    out = torch.empty(n, d, device=dev, dtype=torch.float32)
    labels = torch.empty(n, device=dev, dtype=torch.int64) if return_labels else None
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        comp = torch.randint(0, components, (e - s,), generator=g, device=dev)
        x = torch.randn(e - s, d, generator=g, device=dev, dtype=torch.float32)
        x.mul_(noise_scale).add_(means[comp])
        x.div_(x.norm(dim=1, keepdim=True).clamp_min_(1e-30))
        out[s:e] = x
        if labels is not None:
            labels[s:e] = comp
    return (out, labels) if return_labels else out


# The five workloads of this build (shapes of the paper's collections).
CONFIGS = {
    "C1": dict(n=20_000, d=128, components=100, recipe="linear", k=100, iters=10),
    "C2": dict(n=1_000_000, d=1536, components=4096, recipe="embed", k=1024, iters=10),
    "C3": dict(n=1_000_000, d=768, components=8192, recipe="embed", k=4096, iters=10, etr=True, nq=1000),
    "C4": dict(n=1_000_000, d=1536, components=16384, recipe="embed", k=16384, iters=10),
    "C5": dict(n=10_000_000, d=384, components=32768, recipe="embed", k=32768, iters=5),
}
SEED_DATA = 1234
SEED_FIT = 42
SEED_QUERY = 4321


def config_data(name: str, device: str = "cpu", n: int | None = None):
    c = CONFIGS[name]
    return mixture(n or c["n"], c["d"], c["components"], SEED_DATA, c["recipe"], device)


def config_queries(name: str, device: str = "cpu", nq: int | None = None):
    """Held-out queries: rows of the same mixture as the data (same means) drawn with their own seed."""
    c = CONFIGS[name]
    return mixture(nq or c.get("nq", 1000), c["d"], c["components"], SEED_DATA, c["recipe"], device,
                   sample_seed=SEED_QUERY)
