"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and rounds them to the storage dtype.  It holds none of the
operator's arithmetic and imports neither the HIP binding nor the CPU oracle, so both sides can be
fed the same bits.

Recipe (one ``numpy.random.Generator(PCG64(seed))`` per workload, draws in the order q, k, v, then
filters): activations q, k, v ~ N(0, 1) i.i.d., drawn in fp32 and, for bf16 workloads, rounded to
bf16 with round-to-nearest-even; short filters h[c, j] ~ N(0, 1/l_h) (variance 1/l_h); medium filters
h[g, j] = w[g, j] * exp(-alpha_g * j) with w ~ N(0, 1/l_h) and alpha_g ~ U(0.01, 0.1), the exponential
decay regulariser of the paper's Hyena-MR (Sec. 2.1), materialised on the host in fp64 and stored as
fp32.  The paper's own operator benchmark (Sec. 3.2.2, batch 1, width 4096, sequence length swept)
runs on synthetic tensors as well; no dataset is involved.
"""
from __future__ import annotations

import numpy as np
import torch

# name -> shape of the workload; order matches the list of benchmark configurations.
CONFIGS = {
    "c0": dict(kind="se", B=1, L=1024, D=256, lh=7, group=1, dtype="f32"),
    "c1": dict(kind="se", B=1, L=8192, D=4096, lh=7, group=1, dtype="bf16"),
    "c2": dict(kind="mr", B=1, L=8192, D=4096, lh=128, group=16, dtype="bf16"),
    "c3": dict(kind="mr", B=1, L=131072, D=4096, lh=128, group=16, dtype="bf16"),
    "c4": dict(kind="chain", B=4, L=32768, D=4096, lh=128, group=16, lf=7, feat_group=1, dtype="bf16"),
    # not one of the five: c2 with a filter per channel (no grouping), the shape of the chunk-parallel path (App. A.1)
    "c2u": dict(kind="mr", B=1, L=8192, D=4096, lh=128, group=1, dtype="bf16"),
    # not of the five either: Hyena-LI (long implicit filter, Sec. 2.1) at the shapes of c2 and c3
    "li2": dict(kind="li", B=1, L=8192, D=4096, order=16, group=16, dtype="bf16"),
    "li3": dict(kind="li", B=1, L=131072, D=4096, order=16, group=16, dtype="bf16"),
}

_BASE_SEED = 186800


def config(name: str, **overrides) -> dict:
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    cfg["name"] = name
    return cfg


def seed_for(name: str, variant: int = 0) -> int:
    return _BASE_SEED + list(CONFIGS).index(name) + 1000 * variant


def torch_dtype(dtype: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def normal_tensor(rng: np.random.Generator, shape, dtype: str) -> torch.Tensor:
    """N(0,1) draws in fp32, stored as ``dtype`` (bf16: round-to-nearest-even). CPU tensor."""
    x = torch.from_numpy(rng.standard_normal(size=shape, dtype=np.float32))
    return x if dtype == "f32" else x.to(torch.bfloat16)


def short_filter(rng: np.random.Generator, n_filters: int, lh: int) -> np.ndarray:
    """h[c, j] ~ N(0, 1/l_h): standard deviation l_h**-0.5.  fp32 [n_filters, l_h]."""
    w = rng.standard_normal(size=(n_filters, lh), dtype=np.float32)
    return (w * np.float32(lh ** -0.5)).astype(np.float32)


def decay_filter(rng: np.random.Generator, n_filters: int, lh: int) -> np.ndarray:
    """h[g, j] = w[g, j] * exp(-alpha_g * j), w ~ N(0, 1/l_h), alpha_g ~ U(0.01, 0.1).  fp32."""
    w = rng.standard_normal(size=(n_filters, lh)).astype(np.float64) * lh ** -0.5
    alpha = rng.uniform(0.01, 0.1, size=(n_filters, 1))
    j = np.arange(lh, dtype=np.float64)[None, :]
    return (w * np.exp(-alpha * j)).astype(np.float32)


def li_params(rng: np.random.Generator, n_filters: int, order: int):
    """Residues and poles of the long implicit filter h[g, j] = sum_n R[g, n] lam[g, n]^j (Sec. 2.1):
    R ~ N(0, 1/order); lam = exp(-a) with a log-uniform in [1e-3, 1], i.e. time constants from one step to a
    thousand steps, every pole real and inside the unit circle.  fp32 [n_filters, order] each."""
    R = rng.standard_normal(size=(n_filters, order)) * order ** -0.5
    a = np.exp(rng.uniform(np.log(1e-3), np.log(1.0), size=(n_filters, order)))
    return R.astype(np.float32), np.exp(-a).astype(np.float32)


def make(name: str, variant: int = 0, **overrides) -> dict:
    """Build one workload on the host.

    Returns a dict with the shape fields of the configuration plus CPU tensors ``q, k, v`` (storage
    dtype), fp32 numpy filter ``h`` [D // group, l_h] and, for the chain workload, the three
    featurizer filters ``hq, hk, hv`` [D // feat_group, l_f].
    """
    cfg = config(name, **overrides)
    rng = np.random.Generator(np.random.PCG64(seed_for(name, variant)))
    shape = (cfg["B"], cfg["L"], cfg["D"])
    out = dict(cfg)
    for key in ("q", "k", "v"):
        out[key] = normal_tensor(rng, shape, cfg["dtype"])
    n_filters = cfg["D"] // cfg["group"]
    if cfg["kind"] == "li":
        out["R"], out["lam"] = li_params(rng, n_filters, cfg["order"])
        return out
    if cfg["kind"] == "se":
        out["h"] = short_filter(rng, n_filters, cfg["lh"])
    else:
        out["h"] = decay_filter(rng, n_filters, cfg["lh"])
    if cfg["kind"] == "chain":
        nf = cfg["D"] // cfg["feat_group"]
        for key in ("hq", "hk", "hv"):
            out[key] = short_filter(rng, nf, cfg["lf"])
    return out


def sample_points(seed: int, B: int, L: int, D: int, n: int, lh: int) -> np.ndarray:
    """n output coordinates (b, t, c) for spot checks: uniform draws plus the corners that matter
    for a causal filter (first rows of every batch item, t around l_h, last row, first/last channel)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    pts = np.stack(
        [rng.integers(0, B, n), rng.integers(0, L, n), rng.integers(0, D, n)], axis=1
    ).astype(np.int64)
    edge_t = sorted({t for t in (0, 1, lh - 2, lh - 1, lh, L - 1) if 0 <= t < L})
    edges = [(b, t, c) for b in sorted({0, B - 1}) for t in edge_t for c in sorted({0, D - 1})]
    return np.concatenate([np.asarray(edges, dtype=np.int64).reshape(-1, 3), pts], axis=0)
