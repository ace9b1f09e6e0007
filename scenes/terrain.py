"""Terrain inputs: a flat plane or a seeded synthetic heightfield.

The heightfield stands in for the paper's uneven terrain with static
rectangular obstacles (Section 4.1, complex-terrain task): a sum of four
sinusoid octaves plus axis-aligned box steps that add their height to the
samples they cover.  Heights are stored as fp32 samples, row-major [ny][nx].
"""
from dataclasses import dataclass
import numpy as np

PLANE, HEIGHTFIELD = 0, 1


@dataclass
class Terrain:
    kind: int
    nx: int = 0
    ny: int = 0
    cell: float = 0.0
    origin: tuple = (0.0, 0.0)
    heights: np.ndarray = None      # fp32 [ny][nx]

    @property
    def extent(self):
        return ((self.nx - 1) * self.cell, (self.ny - 1) * self.cell)


def make_plane():
    return Terrain(kind=PLANE, nx=0, ny=0, cell=1.0, origin=(0.0, 0.0),
                   heights=np.zeros((0, 0), np.float32))


def make_heightfield(seed=7, nx=256, ny=256, cell=0.1, amplitude=0.3, n_boxes=200,
                     box_half=(0.2, 1.0), box_height=(0.05, 0.3)):
    rng = np.random.Generator(np.random.Philox(key=int(seed)))
    xs = np.arange(nx, dtype=np.float64) * cell
    ys = np.arange(ny, dtype=np.float64) * cell
    gx, gy = np.meshgrid(xs, ys)                     # [ny][nx]
    h = np.zeros((ny, nx), np.float64)
    # octave amplitudes halve from amplitude*8/15 so that they sum to `amplitude`
    amps = amplitude * np.array([8.0, 4.0, 2.0, 1.0]) / 15.0
    lams = np.array([12.8, 6.4, 3.2, 1.6])
    for a, lam in zip(amps, lams):
        ang = rng.uniform(0.0, 2.0 * np.pi)
        ph = rng.uniform(0.0, 2.0 * np.pi)
        k = 2.0 * np.pi / lam
        h += a * np.sin(k * (np.cos(ang) * gx + np.sin(ang) * gy) + ph)
    ex, ey = (nx - 1) * cell, (ny - 1) * cell
    for _ in range(n_boxes):
        cx, cy = rng.uniform(0.0, ex), rng.uniform(0.0, ey)
        hx, hy = rng.uniform(*box_half), rng.uniform(*box_half)
        bh = rng.uniform(*box_height)
        inside = (np.abs(gx - cx) <= hx) & (np.abs(gy - cy) <= hy)
        h[inside] += bh
    return Terrain(kind=HEIGHTFIELD, nx=nx, ny=ny, cell=float(cell), origin=(0.0, 0.0),
                   heights=np.ascontiguousarray(h.astype(np.float32)))


def make_flat_heightfield(nx=16, ny=16, cell=0.1, height=0.0, origin=(0.0, 0.0)):
    return Terrain(kind=HEIGHTFIELD, nx=nx, ny=ny, cell=float(cell), origin=tuple(origin),
                   heights=np.full((ny, nx), height, np.float32))


def make_tilted_heightfield(nx=16, ny=16, cell=0.1, slope_x=0.0, slope_y=0.0, z0=0.0,
                            origin=(0.0, 0.0)):
    xs = np.arange(nx, dtype=np.float64) * cell
    ys = np.arange(ny, dtype=np.float64) * cell
    gx, gy = np.meshgrid(xs, ys)
    h = z0 + slope_x * gx + slope_y * gy
    return Terrain(kind=HEIGHTFIELD, nx=nx, ny=ny, cell=float(cell), origin=tuple(origin),
                   heights=np.ascontiguousarray(h.astype(np.float32)))


def terrain_height_max_near(terrain, x, y, radius):
    """Largest height sample within `radius` (in xy) of the point; 0 on a plane."""
    if terrain.kind == PLANE:
        return 0.0
    c = terrain.cell
    i0 = max(0, int(np.floor((x - terrain.origin[0] - radius) / c)))
    i1 = min(terrain.nx - 1, int(np.ceil((x - terrain.origin[0] + radius) / c)))
    j0 = max(0, int(np.floor((y - terrain.origin[1] - radius) / c)))
    j1 = min(terrain.ny - 1, int(np.ceil((y - terrain.origin[1] + radius) / c)))
    if i1 < i0 or j1 < j0:
        return 0.0
    return float(terrain.heights[j0:j1 + 1, i0:i1 + 1].max())
