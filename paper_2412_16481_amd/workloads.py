"""Seeded synthetic inputs for the PSH + Bucket-Swin path.

This module only draws input data (point coordinates and bf16 feature rows). It holds none of
the method's arithmetic (no voxelisation, hashing, grouping or attention) and is the one module
that both the CPU oracle's tests and the HIP path's tests/bench import.

The paper measures on LiDAR driving scans and shows an indoor building sample (Section 5,
Fig. 3); those datasets are not available here, so the generators below produce point sets of
the same nature: surface-like samples (points on planes and box faces, not volume-filling),
about 1e5 points per scan, batches of scans stored back to back.

All randomness comes from ``numpy.random.default_rng(seed)``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

# --------------------------------------------------------------------------- bf16 plumbing


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even) and return the 16-bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to fp32, exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def features_bf16(rng: np.random.Generator, n: int, channels: int) -> np.ndarray:
    """N(0,1) features rounded to bf16; returned as uint16 bit patterns of shape [n, channels]."""
    out = np.empty((n, channels), dtype=np.uint16)
    step = max(1, (1 << 22) // max(channels, 1))
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        out[lo:hi] = f32_to_bf16_bits(rng.standard_normal((hi - lo, channels), dtype=np.float32))
    return out


# --------------------------------------------------------------------------- point generators


def uniform_cube(rng: np.random.Generator, n: int, side: float = 4.0) -> np.ndarray:
    """n points uniform in [0, side)^3, fp32 [n,3]."""
    return (rng.random((n, 3), dtype=np.float32) * np.float32(side)).astype(np.float32)


def _sample_rects(rng, origins, eu, ev, n):
    """Sample n points area-proportionally over rectangles origin + a*eu + b*ev, a,b in [0,1)."""
    areas = np.linalg.norm(np.cross(eu, ev), axis=1)
    p = areas / areas.sum()
    which = rng.choice(len(areas), size=n, p=p)
    a = rng.random(n)[:, None]
    b = rng.random(n)[:, None]
    return origins[which] + a * eu[which] + b * ev[which]


def indoor_room(rng: np.random.Generator, n: int = 200_000, n_boxes: int = 30,
                room: Tuple[float, float, float] = (10.0, 10.0, 3.0), jitter: float = 0.005) -> np.ndarray:
    """Points on the floor, the four walls and the visible faces of random boxes standing on the
    floor of a room, with Gaussian jitter; fp32 [n,3]."""
    X, Y, Z = room
    org, eu, ev = [], [], []

    def rect(o, u, v):
        org.append(o)
        eu.append(u)
        ev.append(v)

    rect((0, 0, 0), (X, 0, 0), (0, Y, 0))          # floor
    rect((0, 0, 0), (X, 0, 0), (0, 0, Z))          # wall y=0
    rect((0, Y, 0), (X, 0, 0), (0, 0, Z))          # wall y=Y
    rect((0, 0, 0), (0, Y, 0), (0, 0, Z))          # wall x=0
    rect((X, 0, 0), (0, Y, 0), (0, 0, Z))          # wall x=X
    cx = rng.uniform(0.0, X, n_boxes)
    cy = rng.uniform(0.0, Y, n_boxes)
    ex = rng.uniform(0.3, 2.0, n_boxes)
    ey = rng.uniform(0.3, 2.0, n_boxes)
    ez = rng.uniform(0.3, 2.0, n_boxes)
    for i in range(n_boxes):
        x0, y0 = cx[i] - ex[i] / 2, cy[i] - ey[i] / 2
        rect((x0, y0, ez[i]), (ex[i], 0, 0), (0, ey[i], 0))       # top
        rect((x0, y0, 0), (ex[i], 0, 0), (0, 0, ez[i]))           # side y=y0
        rect((x0, y0 + ey[i], 0), (ex[i], 0, 0), (0, 0, ez[i]))   # side y=y1
        rect((x0, y0, 0), (0, ey[i], 0), (0, 0, ez[i]))           # side x=x0
        rect((x0 + ex[i], y0, 0), (0, ey[i], 0), (0, 0, ez[i]))   # side x=x1
    pts = _sample_rects(rng, np.asarray(org, np.float64), np.asarray(eu, np.float64),
                        np.asarray(ev, np.float64), n)
    pts = pts + rng.normal(0.0, jitter, pts.shape)
    return pts.astype(np.float32)


def lidar_scan(rng: np.random.Generator, n_beams: int = 64, n_azimuth: int = 1800,
               max_range: float = 70.0, n_boxes: int = 50, sensor_height: float = 1.8,
               range_noise: float = 0.02) -> np.ndarray:
    """One sweep of a spinning multi-beam range sensor over a ground plane and random boxes.
    Rays are cast from (0,0,sensor_height); returns beyond max_range are dropped; fp32 [n,3]."""
    elev = np.deg2rad(np.linspace(-25.0, -1.4, n_beams))
    azim = np.deg2rad(np.arange(n_azimuth) * (360.0 / n_azimuth))
    el, az = np.meshgrid(elev, azim, indexing="ij")
    d = np.stack([np.cos(el) * np.cos(az), np.cos(el) * np.sin(az), np.sin(el)], axis=-1).reshape(-1, 3)
    o = np.array([0.0, 0.0, sensor_height])
    t = sensor_height / (-d[:, 2])                       # ground z = 0
    bc = rng.uniform(-max_range, max_range, (n_boxes, 2))
    bf = rng.uniform(1.0, 6.0, (n_boxes, 2))
    bh = rng.uniform(1.0, 4.0, n_boxes)
    lo = np.concatenate([bc - bf / 2, np.zeros((n_boxes, 1))], axis=1)
    hi = np.concatenate([bc + bf / 2, bh[:, None]], axis=1)
    keep = ~((lo[:, 0] < 1.0) & (hi[:, 0] > -1.0) & (lo[:, 1] < 1.0) & (hi[:, 1] > -1.0))
    lo, hi = lo[keep], hi[keep]
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = 1.0 / d
        for b in range(lo.shape[0]):                     # slab test, one box at a time
            t0 = (lo[b] - o) * inv
            t1 = (hi[b] - o) * inv
            tn = np.minimum(t0, t1).max(axis=1)
            tf = np.maximum(t0, t1).min(axis=1)
            hit = (tn <= tf) & (tn > 0.0)
            t = np.where(hit & (tn < t), tn, t)
    t = t + rng.normal(0.0, range_noise, t.shape)
    ok = (t <= max_range) & (t > 0.5)
    pts = o + d[ok] * t[ok, None]
    return pts.astype(np.float32)


# --------------------------------------------------------------------------- the five workloads


@dataclass
class Workload:
    name: str
    coords: np.ndarray            # fp32 [n,3], scans back to back
    batch_offsets: np.ndarray     # int32 [n_scans+1]
    voxel_size: float
    bucket_cap: int               # attention scope capacity (rows per group)
    heads: int
    head_dim: int
    modes: List[str] = field(default_factory=list)   # attention passes, in order
    seed: int = 0
    scope_buckets: int = 4

    @property
    def n(self) -> int:
        return int(self.coords.shape[0])

    @property
    def n_scans(self) -> int:
        return int(self.batch_offsets.shape[0] - 1)

    @property
    def channels(self) -> int:
        return self.heads * self.head_dim

    def qkv(self) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
        """Three independent bf16 feature arrays [n, heads*head_dim] (uint16 bit patterns)."""
        rng = np.random.default_rng([self.seed, 0x51C0FFEE])
        return tuple(features_bf16(rng, self.n, self.channels) for _ in range(3))


def _stack_scans(scans: List[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    off = np.zeros(len(scans) + 1, dtype=np.int32)
    off[1:] = np.cumsum([s.shape[0] for s in scans])
    return np.ascontiguousarray(np.concatenate(scans, axis=0), dtype=np.float32), off


CONFIG_NAMES = ("tiny", "indoor", "lidar4", "wide", "lidar8")
EXTRA_NAMES = ("scope8k",)


def make_workload(name: str, seed: int = 0) -> Workload:
    """The five benchmark/parity configurations (sizes, voxel, channels, capacity, passes)."""
    if name == "tiny":
        rng = np.random.default_rng(seed)
        c, off = _stack_scans([uniform_cube(rng, 4096, 4.0)])
        return Workload(name, c, off, 0.02, 128, 4, 16, ["plain", "shift"], seed)
    if name == "indoor":
        rng = np.random.default_rng(seed)
        c, off = _stack_scans([indoor_room(rng, 200_000)])
        return Workload(name, c, off, 0.02, 1024, 4, 16, ["plain", "shift"], seed)
    if name == "lidar4":
        c, off = _stack_scans([lidar_scan(np.random.default_rng(seed + s)) for s in range(4)])
        return Workload(name, c, off, 0.05, 1024, 8, 16, ["plain", "shift"], seed)
    if name == "wide":
        rng = np.random.default_rng(seed)
        c, off = _stack_scans([indoor_room(rng, 200_000)])
        return Workload(name, c, off, 0.02, 4096, 16, 16, ["plain", "shift", "stride"], seed)
    if name == "lidar8":
        c, off = _stack_scans([lidar_scan(np.random.default_rng(seed + s)) for s in range(8)])
        return Workload(name, c, off, 0.05, 1024, 8, 32, ["shift", "stride", "shift", "stride"], seed)
    if name == "scope8k":    # beyond the five configurations: the largest scope of the paper's scope-scaling study
        rng = np.random.default_rng(seed)
        c, off = _stack_scans([indoor_room(rng, 200_000)])
        return Workload(name, c, off, 0.02, 8192, 8, 16, ["plain", "shift", "stride"], seed)
    raise ValueError(f"unknown workload {name!r}; choose from {CONFIG_NAMES + EXTRA_NAMES}")


def many_scans(n_scans: int, points_per_scan: int, seed: int = 0, side: float = 20.0) -> Tuple[np.ndarray, np.ndarray]:
    """A large batch of uniform-cube scans, used to show bucketize in its bandwidth regime."""
    rng = np.random.default_rng(seed)
    coords = (rng.random((n_scans * points_per_scan, 3), dtype=np.float32) * np.float32(side)).astype(np.float32)
    off = (np.arange(n_scans + 1, dtype=np.int64) * points_per_scan).astype(np.int32)
    return coords, off
