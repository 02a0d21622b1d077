"""Seeded synthetic inputs shaped like the paper's workloads.

This module draws random numbers and nothing else: it holds none of the
encoding's arithmetic (no level table, no hashing, no interpolation), so the GPU
library's tests and the CPU oracle can both be fed from it without sharing
method code.  The number of table entries is an argument, obtained by the
caller from whichever implementation it is exercising.

Workloads (they stand in for data sets that are not available here):
  tiny2d   small 2D case the CPU oracle finishes instantly
  image2d  i.i.d. pixel coordinates of gigapixel-image fitting (Section 5.1 of the paper)
  sdf3d    signed-distance training batch: mostly near-surface points plus a
           uniform share (Appendix C.1 describes the real sampler)
  nerf3d   ray-marching batch: samples ordered ray by ray (Appendix E.1)
  large3d  table far larger than the on-chip caches (the regime right of the
           performance cliff in Fig. 4)
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

_ONE_BELOW = np.float32(1.0) - np.float32(2.0 ** -24)  # largest fp32 below 1


@dataclass(frozen=True)
class Workload:
    name: str
    d: int
    L: int
    F: int
    T: int
    N_min: int
    N_max: int
    B: int
    param_dtype: str   # "f32" | "f16"
    io_dtype: str      # "f32" | "f16"
    points: str        # "uniform" | "sdf" | "rays"
    seed: int


WORKLOADS = {
    "tiny2d": Workload("tiny2d", 2, 4, 2, 1 << 10, 4, 32, 4096, "f32", "f32", "uniform", 0),
    "image2d": Workload("image2d", 2, 16, 2, 1 << 22, 16, 32768, 1 << 18, "f16", "f16", "uniform", 1),
    "sdf3d": Workload("sdf3d", 3, 16, 2, 1 << 19, 16, 2048, 1 << 18, "f16", "f16", "sdf", 2),
    "nerf3d": Workload("nerf3d", 3, 16, 2, 1 << 19, 16, 2048, 1 << 20, "f16", "f16", "rays", 3),
    "large3d": Workload("large3d", 3, 16, 2, 1 << 24, 16, 524288, 1 << 21, "f16", "f16", "uniform", 4),
}


def _np_dtype(name: str):
    return {"f32": np.float32, "f16": np.float16}[name]


def _rngs(seed: int):
    """Three independent streams: positions, tables, upstream gradients."""
    return [np.random.default_rng(s) for s in np.random.SeedSequence(seed).spawn(3)]


def _unit_vectors(rng, n: int, d: int) -> np.ndarray:
    v = rng.standard_normal((n, d))
    return v / np.linalg.norm(v, axis=1, keepdims=True)


def _clamp_unit(x: np.ndarray) -> np.ndarray:
    return np.clip(x.astype(np.float32), np.float32(0.0), _ONE_BELOW)


def points_uniform(rng, B: int, d: int) -> np.ndarray:
    return _clamp_unit(rng.random((B, d)))


def points_sdf(rng, B: int, d: int = 3) -> np.ndarray:
    """80% on a sphere of radius 0.3 about the cube centre with N(0, 0.01^2)
    jitter per axis, 20% uniform, shuffled (training batches are drawn i.i.d.)."""
    n_surf = (B * 4) // 5
    surf = 0.5 + 0.3 * _unit_vectors(rng, n_surf, d) + 0.01 * rng.standard_normal((n_surf, d))
    unif = rng.random((B - n_surf, d))
    x = np.concatenate([surf, unif], axis=0)
    return _clamp_unit(x[rng.permutation(B)])


def points_rays(rng, B: int, d: int = 3, samples_per_ray: int = 256) -> np.ndarray:
    """Rays from a sphere of radius 1.5 about the cube centre aimed at uniform
    targets in [0.25,0.75]^d; stratified samples between the entry and exit of
    the unit cube, kept in ray-major order."""
    n_rays = (B + samples_per_ray - 1) // samples_per_ray
    o = 0.5 + 1.5 * _unit_vectors(rng, n_rays, d)
    t = rng.uniform(0.25, 0.75, (n_rays, d))
    direc = t - o
    direc /= np.linalg.norm(direc, axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        t0 = (0.0 - o) / direc
        t1 = (1.0 - o) / direc
    t_near = np.max(np.minimum(t0, t1), axis=1)
    t_far = np.min(np.maximum(t0, t1), axis=1)
    k = np.arange(samples_per_ray)[None, :] + rng.random((n_rays, samples_per_ray))
    ts = t_near[:, None] + k / samples_per_ray * (t_far - t_near)[:, None]
    x = o[:, None, :] + ts[:, :, None] * direc[:, None, :]
    return _clamp_unit(x.reshape(-1, d)[:B])


def make_points(kind: str, rng, B: int, d: int) -> np.ndarray:
    if kind == "uniform":
        return points_uniform(rng, B, d)
    if kind == "sdf":
        return points_sdf(rng, B, d)
    if kind == "rays":
        return points_rays(rng, B, d)
    raise ValueError(kind)


def make_tables(rng, n_entries: int, F: int, dtype: str, scale: float = 1e-4) -> np.ndarray:
    """U(-scale, scale) drawn in fp32, rounded to the storage type (round to
    nearest even, subnormals kept).  scale=1e-4 is the paper's initialisation;
    tests also use scale=1 so that fp16 tolerances are not vacuous."""
    t = rng.uniform(-scale, scale, (n_entries, F)).astype(np.float32)
    return t.astype(_np_dtype(dtype))


def make_dy(rng, B: int, LF: int, dtype: str) -> np.ndarray:
    return rng.standard_normal((B, LF), dtype=np.float32).astype(_np_dtype(dtype))


def make_inputs(w: Workload, n_entries: int, B: int | None = None, table_scale: float = 1e-4):
    """(x [B,d] fp32, theta [n_entries,F], dy [B,L*F]) for a workload; ``B``
    overrides the workload's batch size (a prefix-like smaller draw, same recipe)."""
    B = w.B if B is None else B
    rx, rt, rg = _rngs(w.seed)
    x = make_points(w.points, rx, B, w.d)
    theta = make_tables(rt, n_entries, w.F, w.param_dtype, table_scale)
    dy = make_dy(rg, B, w.L * w.F, w.io_dtype)
    return x, theta, dy
