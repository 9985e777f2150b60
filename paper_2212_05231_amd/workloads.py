"""Seeded synthetic inputs and parameter sets for the five benchmark workloads.

This module holds no arithmetic of the method itself: it draws random numbers,
lays out rays, and derives the per-level grid descriptor that both the HIP
library and the CPU oracle receive as plain integers.  It depends on numpy only
and is the one module the tests hand to both sides.

The paper trains on calibrated multi-view image sets that are not available
here; the ray batches below stand in for them (Sec. 3 "Background": n samples
p(t_i) = o + t_i v along each camera ray).  What is kept from the real workload
is the structure that matters to the kernels: 64 consecutive samples are
collinear, samples concentrate near the centre of the unit cube, tables start as
tiny uniform noise.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

MAX_LEVELS = 32


@dataclass
class Config:
    """Shape descriptor shared by oracle and library (mirrors `neus2_config`)."""
    n_levels: int
    n_features: int
    log2_table_size: int
    active_levels: int
    table_dtype: str                 # "f32" | "f16"
    res: List[int]
    dense: List[int]
    sdf_dims: List[int]              # e.g. [32, 64, 64, 16]
    color_dims: List[int]            # e.g. [38, 64, 64, 3] or [] when there is no colour net
    samples_per_ray: int
    loss_kind: int                   # 0: mean(d^2) + beta*eikonal ; 1: L1 colour + beta*eikonal ; 2: Huber colour
    s: float
    beta: float
    name: str = ""
    huber_delta: float = 0.1
    frozen_levels: int = 0           # levels [0, frozen) are inputs (they carry x), not parameters

    @property
    def table_size(self) -> int:
        return 1 << self.log2_table_size

    @property
    def enc_dim(self) -> int:
        return self.n_levels * self.n_features


def level_resolutions(n_levels: int, res_min: int, res_max: Optional[int] = None,
                      growth: Optional[float] = None) -> List[int]:
    """Grid resolution per level, geometric between res_min and res_max."""
    if growth is None:
        growth = math.exp(math.log(res_max / res_min) / (n_levels - 1))
    res = [int(math.floor(res_min * growth ** l + 1e-9)) for l in range(n_levels)]
    if res_max is not None:
        res[-1] = int(res_max)
    return res


def dense_flags(res: List[int], table_size: int) -> List[int]:
    """A level is stored densely when all (res+1)^3 vertices fit in its table."""
    return [1 if (r + 1) ** 3 <= table_size else 0 for r in res]


def make_config(k: int) -> Config:
    """Descriptor of benchmark workload k (1..5)."""
    if k == 1:
        res = level_resolutions(8, 16, growth=1.5)
        return Config(8, 2, 14, 8, "f32", res, dense_flags(res, 1 << 14), [16, 64, 16], [],
                      1, 0, 20.0, 0.1, "cfg1-tiny-sdf")
    if k in (2, 3, 5):
        res = level_resolutions(16, 16, 2048)
        return Config(16, 2, 19, 8 if k == 3 else 16, "f16", res, dense_flags(res, 1 << 19),
                      [32, 64, 64, 16], [38, 64, 64, 3], 64, 1, 20.0, 0.1,
                      {2: "cfg2-static-4096x64", 3: "cfg3-progressive-8192x64",
                       5: "cfg5-dynamic-20x8192x64"}[k])
    if k == 4:
        res = level_resolutions(16, 16, 4096)
        return Config(16, 2, 21, 16, "f16", res, dense_flags(res, 1 << 21),
                      [32, 64, 64, 16], [38, 64, 64, 3], 64, 1, 20.0, 0.1, "cfg4-large-16384x64")
    raise ValueError(f"unknown workload {k}")


def default_rays(k: int) -> int:
    return {1: 4096, 2: 4096, 3: 8192, 4: 16384, 5: 8192}[k]


def _xavier(rng: np.random.Generator, n_out: int, n_in: int) -> np.ndarray:
    bound = math.sqrt(6.0 / (n_in + n_out))
    return rng.uniform(-bound, bound, size=(n_out, n_in)).astype(np.float32)


def make_params(cfg: Config, seed: int) -> Dict[str, object]:
    """Tables (stored dtype), SDF matrices H_l [n_l, n_{l-1}], colour matrices W_l."""
    rng = np.random.default_rng(seed)
    T, L, F = cfg.table_size, cfg.n_levels, cfg.n_features
    tab = rng.uniform(-1e-4, 1e-4, size=(L, T, F))
    tables = tab.astype(np.float16 if cfg.table_dtype == "f16" else np.float32)
    H = [_xavier(rng, cfg.sdf_dims[i + 1], cfg.sdf_dims[i]) for i in range(len(cfg.sdf_dims) - 1)]
    W = [_xavier(rng, cfg.color_dims[i + 1], cfg.color_dims[i]) for i in range(len(cfg.color_dims) - 1)]
    return {"tables": tables, "H": H, "W": W}


def make_points(n: int, seed: int) -> np.ndarray:
    """Workload 1: points uniform in the unit cube, fp32."""
    rng = np.random.default_rng(seed)
    pos = rng.uniform(0.0, 1.0, size=(n, 3)).astype(np.float32)
    return np.minimum(pos, np.float32(1.0 - 2.0 ** -24))


def make_rays(n_rays: int, samples_per_ray: int, seed: int, to_cube: bool = True) -> Dict[str, np.ndarray]:
    """Workloads 2-5: cameras on a radius-3 sphere looking at the origin with
    +-0.3 jitter, stratified samples between the two unit-sphere intersections.

    Returns pos [R*n,3] (unit-cube coordinates if `to_cube`, else world), dirs
    [R,3], target rgb [R,3], all fp32.
    """
    rng = np.random.default_rng(seed)
    u = rng.normal(size=(n_rays, 3))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    o = 3.0 * u
    tgt = rng.uniform(-0.3, 0.3, size=(n_rays, 3))
    v = tgt - o
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    # |o + t v| = 1  ->  t^2 + 2 (o.v) t + |o|^2 - 1 = 0
    b = np.sum(o * v, axis=1)
    disc = b * b - (np.sum(o * o, axis=1) - 1.0)
    root = np.sqrt(disc)
    near, far = -b - root, -b + root
    jit = rng.uniform(0.0, 1.0, size=(n_rays, samples_per_ray))
    kk = np.arange(samples_per_ray)[None, :]
    t = near[:, None] + (kk + jit) * ((far - near)[:, None] / samples_per_ray)
    p = o[:, None, :] + t[:, :, None] * v[:, None, :]
    if to_cube:
        p = np.clip((p + 1.0) * 0.5, 0.0, 1.0 - 2.0 ** -24)
    rgb = rng.uniform(0.0, 1.0, size=(n_rays, 3))
    return {"pos": p.reshape(-1, 3).astype(np.float32), "dirs": v.astype(np.float32),
            "target": rgb.astype(np.float32)}


def make_ragged_rays(n_rays: int, seed: int, max_len: int = 200) -> Dict[str, np.ndarray]:
    """Rays with their own sample counts, the shape an occupancy-grid ray marcher hands to the
    step: a fixed marching step dt = 2/128 along the chord through the unit sphere, samples only
    on one occupied interval per ray.  Length mix: 10 % of the rays have no sample (they miss
    the occupied cells), 75 % have 4..64, 15 % have 65..max_len (longer than one wavefront).

    Returns pos [N,3] (unit cube), dirs [R,3], target [R,3] (fp32), ray_offsets [R+1] and
    sample_ray [N] (int32).
    """
    rng = np.random.default_rng(seed)
    u = rng.normal(size=(n_rays, 3))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    o = 3.0 * u
    tgt = rng.uniform(-0.3, 0.3, size=(n_rays, 3))
    v = tgt - o
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    b = np.sum(o * v, axis=1)
    root = np.sqrt(b * b - (np.sum(o * o, axis=1) - 1.0))
    near, far = -b - root, -b + root
    dt = 2.0 / 128.0
    kind = rng.uniform(size=n_rays)
    count = np.where(kind < 0.10, 0, np.where(kind < 0.85, rng.integers(min(4, max_len), min(64, max_len) + 1, size=n_rays),
                                              rng.integers(min(65, max_len), max_len + 1, size=n_rays)))
    count = np.minimum(count, np.floor((far - near) / dt).astype(np.int64))
    offsets = np.zeros(n_rays + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(count)
    N = int(offsets[-1])
    sample_ray = np.repeat(np.arange(n_rays), count)
    k = np.arange(N) - offsets[sample_ray]
    t0 = near + rng.uniform(size=n_rays) * np.maximum(far - near - count * dt, 0.0)
    t = t0[sample_ray] + (k + rng.uniform(size=N)) * dt
    p = o[sample_ray] + t[:, None] * v[sample_ray]
    p = np.clip((p + 1.0) * 0.5, 0.0, 1.0 - 2.0 ** -24)
    rgb = rng.uniform(0.0, 1.0, size=(n_rays, 3))
    return {"pos": p.astype(np.float32), "dirs": v.astype(np.float32), "target": rgb.astype(np.float32),
            "ray_offsets": offsets.astype(np.int32), "sample_ray": sample_ray.astype(np.int32)}


def make_camera_rays(n_rays: int, seed: int) -> Dict[str, np.ndarray]:
    """Rays for the ray marcher, in unit-cube coordinates: the cameras of `make_rays` (on a
    sphere of radius 3 around the scene, looking at the origin with +-0.3 jitter, world cube
    [-1,1]^3 mapped to [0,1]^3), plus 3 % of rays that miss the cube and 2 % that start
    inside it.  Returns origins [R,3], dirs [R,3] (unit), jitter [R] in [0,1), target [R,3], fp32.
    """
    rng = np.random.default_rng(seed)
    u = rng.normal(size=(n_rays, 3))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    o = 3.0 * u
    tgt = rng.uniform(-0.3, 0.3, size=(n_rays, 3))
    kind = rng.uniform(size=n_rays)
    tgt[kind < 0.03] += 4.0 * u[kind < 0.03][:, [1, 2, 0]]          # looks past the scene
    inside = kind > 0.98
    o[inside] = rng.uniform(-0.9, 0.9, size=(int(inside.sum()), 3))
    v = tgt - o
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    return {"origins": ((o + 1.0) * 0.5).astype(np.float32), "dirs": v.astype(np.float32),
            "jitter": rng.uniform(0.0, 1.0, size=n_rays).astype(np.float32),
            "target": rng.uniform(0.0, 1.0, size=(n_rays, 3)).astype(np.float32)}


def make_shell_cells(log2_res: int, radius: float = 0.3, half_width: float = 0.03) -> np.ndarray:
    """Occupied cells of a trained scene, as a bool array [G,G,G] indexed [x,y,z]: the cells
    whose centre lies within `half_width` of a sphere of `radius` around the cube's centre
    (cells near the surface are the ones an SDF-driven update keeps)."""
    G = 1 << log2_res
    c = (np.arange(G) + 0.5) / G - 0.5
    r = np.sqrt(c[:, None, None] ** 2 + c[None, :, None] ** 2 + c[None, None, :] ** 2)
    return np.abs(r - radius) <= half_width


def make_candidate_cells(log2_res: int, m: int, seed: int, duplicates: bool = True) -> Dict[str, np.ndarray]:
    """Candidate cells of one grid update: m cell numbers (uniform over the grid, so some are
    drawn twice unless `duplicates` is off) and a point offset in [0,1)^3 inside each."""
    rng = np.random.default_rng(seed)
    n_cells = 1 << (3 * log2_res)
    cells = rng.integers(0, n_cells, size=m) if duplicates else rng.permutation(n_cells)[:m]
    jit = rng.uniform(0.0, 1.0, size=(m, 3)).astype(np.float32)
    return {"cells": cells.astype(np.int32), "jitter": np.minimum(jit, np.float32(1.0 - 2.0 ** -24))}


def make_rigid(seed: int, max_angle_deg: float = 5.0, max_shift: float = 0.05) -> Dict[str, np.ndarray]:
    """Workload 5: a small axis-angle vector omega and a translation, float64."""
    rng = np.random.default_rng(seed)
    axis = rng.normal(size=3)
    axis /= np.linalg.norm(axis)
    angle = math.radians(rng.uniform(0.0, max_angle_deg))
    shift = rng.normal(size=3)
    shift *= rng.uniform(0.0, max_shift) / np.linalg.norm(shift)
    return {"omega": axis * angle, "shift": shift}


def make_workload(k: int, n_rays: Optional[int] = None, frame: int = 0) -> Dict[str, object]:
    """Config, parameters and one batch for workload k; sizes may be overridden."""
    cfg = make_config(k)
    params = make_params(cfg, 2000 + k)
    R = default_rays(k) if n_rays is None else n_rays
    if k == 1:
        batch = {"pos": make_points(R, 1000 + k)}
    elif k == 5:
        batch = make_rays(R, cfg.samples_per_ray, 1000 + k + 100 * frame, to_cube=False)
        batch.update(make_rigid(3000 + k + 100 * frame))
    else:
        batch = make_rays(R, cfg.samples_per_ray, 1000 + k)
    return {"cfg": cfg, "params": params, "batch": batch}
