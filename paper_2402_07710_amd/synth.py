"""Seeded synthetic inputs for the sparse-convolution path.

This module only *makes inputs*: voxel coordinate sets shaped like the workloads a sparse 3-D
convolution layer sees (uniform random cells, rotating-LiDAR sweeps, indoor surfaces), feature
rows and weights.  It holds none of the method's arithmetic (no hashing, no kernel map, no
convolution) and is the only module that both the CPU oracle's tests and the HIP path's tests
and benchmark draw from.  Everything is numpy on the host and fully determined by the seed.

Coordinates follow the sparse-tensor index structure of the paper (Section II-A, Fig. 2): one
int32 row (batch, x, y, z) per active voxel, rows distinct.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "uniform_cells", "lidar_sweep", "lidar_scene", "lidar_batch", "indoor_scene",
    "features", "weights", "round_to_dtype", "CONFIGS", "make_config",
]


# --------------------------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------------------------
def _dedup_first(cells: np.ndarray) -> np.ndarray:
    """Drop repeated rows, keeping the first occurrence of each and the original order."""
    if len(cells) == 0:
        return cells.reshape(0, cells.shape[1])
    _, first = np.unique(cells, axis=0, return_index=True)
    return cells[np.sort(first)]


def _with_batch(xyz: np.ndarray, b: int) -> np.ndarray:
    out = np.empty((len(xyz), 4), dtype=np.int32)
    out[:, 0] = b
    out[:, 1:] = xyz
    return out


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float values to the nearest value representable in `dtype` ("f32", "f16", "bf16")
    and hand them back as float32 (exact: all three formats embed in float32)."""
    x = np.asarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        import torch
        return torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    raise ValueError(f"unknown dtype {dtype!r}")


# --------------------------------------------------------------------------------------------
# coordinate sets
# --------------------------------------------------------------------------------------------
def uniform_cells(n: int, grid: int, seed: int, batch: int = 0) -> np.ndarray:
    """`n` distinct cells drawn uniformly without replacement from a grid³ cube, in random row
    order (no spatial coherence between neighbouring rows)."""
    rng = np.random.default_rng(seed)
    lin = rng.choice(grid ** 3, size=n, replace=False)
    x, rem = np.divmod(lin, grid * grid)
    y, z = np.divmod(rem, grid)
    return _with_batch(np.stack([x, y, z], axis=1).astype(np.int32), batch)


# LiDAR model constants: a 64-ring spinning sensor 1.73 m above a flat ground plane.
LIDAR_RINGS = 64
LIDAR_AZIMUTHS = 2048
LIDAR_ELEV_DEG = (-24.8, 2.0)
LIDAR_HEIGHT = 1.73
LIDAR_RANGE = (2.0, 70.0)
LIDAR_NOISE = 0.01
LIDAR_VOXEL = 0.05
LIDAR_GRID = (1408, 1600, 41)
LIDAR_Z0 = -1.85            # z of the grid's lowest cell face, sensor frame (ground is -1.73)
LIDAR_BOXES = 40


def _random_boxes(rng: np.random.Generator, n_boxes: int):
    """Axis-aligned boxes resting on the ground: footprint 1.5-6 m, height 1-3 m, centres at
    horizontal range 5-60 m from the origin."""
    rng_r = rng.uniform(5.0, 60.0, n_boxes)
    ang = rng.uniform(0.0, 2 * np.pi, n_boxes)
    cx, cy = rng_r * np.cos(ang), rng_r * np.sin(ang)
    sx = rng.uniform(1.5, 6.0, n_boxes)
    sy = rng.uniform(1.5, 6.0, n_boxes)
    h = rng.uniform(1.0, 3.0, n_boxes)
    lo = np.stack([cx - sx / 2, cy - sy / 2, np.full(n_boxes, -LIDAR_HEIGHT)], axis=1)
    hi = np.stack([cx + sx / 2, cy + sy / 2, -LIDAR_HEIGHT + h], axis=1)
    return lo, hi


def lidar_sweep(rng: np.random.Generator, lo: np.ndarray, hi: np.ndarray,
                sensor_xy=(0.0, 0.0)) -> np.ndarray:
    """One revolution of the sensor: first hit of every ray against the ground plane and the
    boxes, range-gated, with Gaussian range noise.  Returns float64 points [M,3] in the scene
    frame, in ring-major / azimuth-minor order."""
    elev = np.deg2rad(np.linspace(LIDAR_ELEV_DEG[0], LIDAR_ELEV_DEG[1], LIDAR_RINGS))
    azim = np.arange(LIDAR_AZIMUTHS) * (2 * np.pi / LIDAR_AZIMUTHS)
    ce, se = np.cos(elev)[:, None], np.sin(elev)[:, None]
    d = np.stack([ce * np.cos(azim)[None, :], ce * np.sin(azim)[None, :],
                  np.broadcast_to(se, (LIDAR_RINGS, LIDAR_AZIMUTHS))], axis=-1).reshape(-1, 3)
    o = np.array([sensor_xy[0], sensor_xy[1], 0.0])

    t_hit = np.full(len(d), np.inf)
    # ground plane z = -LIDAR_HEIGHT
    down = d[:, 2] < -1e-9
    t_hit[down] = (-LIDAR_HEIGHT - o[2]) / d[down, 2]
    # boxes (slab test), one box at a time to bound memory
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = 1.0 / d
        for b in range(len(lo)):
            t0 = (lo[b] - o) * inv
            t1 = (hi[b] - o) * inv
            tn = np.minimum(t0, t1).max(axis=1)
            tf = np.maximum(t0, t1).min(axis=1)
            ok = (tn <= tf) & (tn > 0)
            t_hit = np.where(ok & (tn < t_hit), tn, t_hit)
    keep = np.isfinite(t_hit) & (t_hit >= LIDAR_RANGE[0]) & (t_hit <= LIDAR_RANGE[1])
    t = t_hit[keep] + rng.normal(0.0, LIDAR_NOISE, int(keep.sum()))
    return o[None, :] + d[keep] * t[:, None]


def lidar_scene(seed: int, batch: int = 0, n_sweeps: int = 1) -> np.ndarray:
    """Voxelised LiDAR-shaped scene: ground plane + 40 random boxes seen by a 64x2048 sweep,
    voxelised at 0.05 m into a 1408x1600x41 grid centred (x, y) on the first sensor position,
    out-of-grid returns dropped, duplicates removed (first occurrence kept, ring-major order).
    `n_sweeps` > 1 adds sweeps of the same scene from sensor positions displaced by 1 m steps
    along x (a denser set with the same local structure)."""
    rng = np.random.default_rng(seed)
    lo, hi = _random_boxes(rng, LIDAR_BOXES)
    pts = [lidar_sweep(rng, lo, hi, sensor_xy=(1.0 * s, 0.0)) for s in range(n_sweeps)]
    pts = np.concatenate(pts, axis=0)
    origin = np.array([-LIDAR_GRID[0] * LIDAR_VOXEL / 2, -LIDAR_GRID[1] * LIDAR_VOXEL / 2, LIDAR_Z0])
    cells = np.floor((pts - origin) / LIDAR_VOXEL).astype(np.int64)
    inside = np.all((cells >= 0) & (cells < np.array(LIDAR_GRID)), axis=1)
    cells = _dedup_first(cells[inside].astype(np.int32))
    return _with_batch(cells, batch)


def lidar_batch(seeds, n_sweeps: int = 1) -> np.ndarray:
    """Independent scenes concatenated, scene s carrying batch index s."""
    return np.concatenate([lidar_scene(s, batch=b, n_sweeps=n_sweeps) for b, s in enumerate(seeds)], axis=0)


# Indoor-style scene constants: surfaces inside a 512³ grid of 2 cm cells (a 10.24 m cube).
INDOOR_GRID = 512
INDOOR_VOXEL = 0.02
INDOOR_SAMPLE = 0.01
INDOOR_TRIANGLES = 120
INDOOR_SPHERES = 80
INDOOR_TRI_LEG = (0.6, 2.5)
INDOOR_SPHERE_R = (0.2, 0.7)


def indoor_scene(seed: int, batch: int = 0, scale: float = 1.0) -> np.ndarray:
    """Dense-surface scene: random right triangles (planes patches) and spheres, sampled on a
    1 cm lattice over each surface and voxelised at 2 cm into a 512³ grid; samples outside the
    grid dropped; duplicates removed keeping generation order (surface by surface, scanline
    within a surface).  `scale` shrinks the number of surfaces (for small test cases)."""
    rng = np.random.default_rng(seed)
    ext = INDOOR_GRID * INDOOR_VOXEL
    n_tri = max(1, int(round(INDOOR_TRIANGLES * scale)))
    n_sph = max(1, int(round(INDOOR_SPHERES * scale)))
    chunks = []
    for _ in range(n_tri):
        p0 = rng.uniform(0.0, ext, 3)
        # two orthogonal unit vectors spanning the triangle's plane
        a = rng.normal(size=3)
        a /= np.linalg.norm(a)
        b = np.cross(a, rng.normal(size=3))
        b /= np.linalg.norm(b)
        la, lb = rng.uniform(*INDOOR_TRI_LEG, 2)
        na, nb = int(la / INDOOR_SAMPLE) + 1, int(lb / INDOOR_SAMPLE) + 1
        u, v = np.meshgrid(np.arange(na), np.arange(nb), indexing="ij")
        inside = (u / max(na - 1, 1) + v / max(nb - 1, 1)) <= 1.0
        u, v = u[inside] * INDOOR_SAMPLE, v[inside] * INDOOR_SAMPLE
        chunks.append(p0[None, :] + u[:, None] * a[None, :] + v[:, None] * b[None, :])
    for _ in range(n_sph):
        c = rng.uniform(0.0, ext, 3)
        r = rng.uniform(*INDOOR_SPHERE_R)
        n_lat = int(np.pi * r / INDOOR_SAMPLE) + 1
        for th in np.linspace(0.0, np.pi, n_lat):
            n_lon = max(1, int(2 * np.pi * r * np.sin(th) / INDOOR_SAMPLE))
            ph = np.arange(n_lon) * (2 * np.pi / n_lon)
            ring = np.stack([r * np.sin(th) * np.cos(ph), r * np.sin(th) * np.sin(ph),
                             np.full(n_lon, r * np.cos(th))], axis=1)
            chunks.append(c[None, :] + ring)
    pts = np.concatenate(chunks, axis=0)
    cells = np.floor(pts / INDOOR_VOXEL).astype(np.int64)
    inside = np.all((cells >= 0) & (cells < INDOOR_GRID), axis=1)
    cells = _dedup_first(cells[inside].astype(np.int32))
    return _with_batch(cells, batch)


# --------------------------------------------------------------------------------------------
# features and weights
# --------------------------------------------------------------------------------------------
def features(n: int, c: int, dtype: str, seed: int) -> np.ndarray:
    """Feature rows ~ N(0,1), rounded to `dtype`, returned as float32 [n, c]."""
    rng = np.random.default_rng(seed + 1_000_003)
    return round_to_dtype(rng.standard_normal((n, c), dtype=np.float32), dtype)


def weights(k3: int, c_in: int, c_out: int, dtype: str, seed: int) -> np.ndarray:
    """Weights [K³, C_in, C_out] ~ N(0, sigma) with sigma = 1/sqrt(K³·C_in) (fan-in scaling, so
    outputs are O(1)), rounded to `dtype`, returned as float32."""
    rng = np.random.default_rng(seed + 2_000_003)
    w = rng.standard_normal((k3, c_in, c_out), dtype=np.float32) / np.float32(np.sqrt(k3 * c_in))
    return round_to_dtype(w, dtype)


# --------------------------------------------------------------------------------------------
# the five named configurations (+ the C=64 target layer)
# --------------------------------------------------------------------------------------------
CONFIGS = {
    # name: (coords builder, K, stride, mode, C_in, C_out, dtype)
    # box = (B, X, Y, Z): the voxel grid the coordinates are confined to
    "cfg1": dict(coords=lambda: uniform_cells(2000, 64, seed=0), K=3, stride=1, mode="subm",
                 C_in=16, C_out=16, dtype="f32", box=(1, 64, 64, 64)),
    "cfg2": dict(coords=lambda: lidar_scene(0), K=3, stride=1, mode="subm",
                 C_in=32, C_out=32, dtype="f16", box=(1, 1408, 1600, 41)),
    "cfg3": dict(coords=lambda: lidar_scene(0), K=2, stride=2, mode="strided",
                 C_in=32, C_out=64, dtype="f16", box=(1, 1408, 1600, 41)),
    # the down-sampling layer most encoders use: 3x3x3 kernel, stride 2, no padding (K != stride)
    "cfg3k3": dict(coords=lambda: lidar_scene(0), K=3, stride=2, mode="strided",
                   C_in=32, C_out=64, dtype="f16", box=(1, 1408, 1600, 41)),
    "cfg4": dict(coords=lambda: lidar_batch([0, 1, 2, 3]), K=3, stride=1, mode="subm",
                 C_in=64, C_out=64, dtype="bf16", box=(4, 1408, 1600, 41)),
    "cfg5": dict(coords=lambda: indoor_scene(0), K=3, stride=1, mode="subm",
                 C_in=128, C_out=128, dtype="f16", box=(1, 512, 512, 512)),
    # the ~100k-voxel C=64 fp16 submanifold layer the target statement names: three sweeps of
    # one scene (sensor displaced in 1 m steps), same local structure as cfg2
    "target64": dict(coords=lambda: lidar_scene(0, n_sweeps=3), K=3, stride=1, mode="subm",
                     C_in=64, C_out=64, dtype="f16", box=(1, 1408, 1600, 41)),
}


def make_config(name: str, seed: int = 0) -> dict:
    """Materialise one named configuration: coords int32 [N,4], feat float32 [N,C_in] and
    weight float32 [K³,C_in,C_out] (both already rounded to the config's dtype)."""
    spec = CONFIGS[name]
    coords = np.ascontiguousarray(spec["coords"](), dtype=np.int32)
    k3 = spec["K"] ** 3
    return dict(
        name=name, coords=coords, K=spec["K"], stride=spec["stride"], mode=spec["mode"],
        C_in=spec["C_in"], C_out=spec["C_out"], dtype=spec["dtype"], box=spec["box"],
        feat=features(len(coords), spec["C_in"], spec["dtype"], seed),
        weight=weights(k3, spec["C_in"], spec["C_out"], spec["dtype"], seed),
    )
