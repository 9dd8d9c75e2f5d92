"""Seeded generators: stroke images (2-D), shell volumes (3-D), sparse filters.

Layouts produced (all numpy, host memory):
  coords  int32  [rows, 1+d]   (b, c_1..c_d), rows sorted ascending by (b, lin),
                               lin = row-major site index, last coordinate fastest
  feats   float32 [rows, C]    one channel vector per occupied site; 0.0 = absent
  w       float32 [T, C_in, C_out]  T = prod(ksize); tap index row-major over
                               (delta_1..delta_d) + h;  0.0 = pruned weight
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

BASE_SEED = 180110585


@dataclass
class LayerSpec:
    c_in: int
    c_out: int
    ksize: Tuple[int, ...]
    filter_density: float
    sigma: float
    rho_up: float
    relu: bool
    pool: bool


@dataclass
class Workload:
    name: str
    ndim: int
    extent: Tuple[int, ...]
    batch: int
    coords: np.ndarray
    feats: np.ndarray
    layers: List[LayerSpec]
    filters: List[np.ndarray] = field(default_factory=list)
    density: float = 0.0
    seed: int = 0


def lin_index(coords: np.ndarray, extent: Sequence[int]) -> np.ndarray:
    """Row-major linear site index (last coordinate fastest) of coords[:, 1:]."""
    lin = np.zeros(coords.shape[0], dtype=np.int64)
    for a, e in enumerate(extent):
        lin = lin * int(e) + coords[:, 1 + a].astype(np.int64)
    return lin


def sort_rows(coords: np.ndarray, feats: np.ndarray, extent: Sequence[int]):
    """Sort rows ascending by (b, lin)."""
    n = int(np.prod([int(e) for e in extent]))
    key = coords[:, 0].astype(np.int64) * n + lin_index(coords, extent)
    order = np.argsort(key, kind="stable")
    return np.ascontiguousarray(coords[order]), np.ascontiguousarray(feats[order])


def occupancy_to_rows(occ: np.ndarray) -> np.ndarray:
    """Boolean [B, E_1..E_d] -> sorted int32 coords [rows, 1+d]."""
    idx = np.argwhere(occ)  # argwhere is already row-major sorted
    return np.ascontiguousarray(idx.astype(np.int32))


# ----------------------------------------------------------------------------
# 2-D: thick polyline strokes
# ----------------------------------------------------------------------------
def _stroke_mask(rng: np.random.Generator, h: int, w: int) -> np.ndarray:
    yy, xx = np.mgrid[0:h, 0:w].astype(np.float64)
    mask = np.zeros((h, w), dtype=bool)
    n_lines = int(rng.integers(3, 7))
    for _ in range(n_lines):
        n_seg = int(rng.integers(2, 5))
        pts = rng.uniform([2.0, 2.0], [h - 3.0, w - 3.0], size=(n_seg + 1, 2))
        half = 0.5 * float(rng.uniform(2.0, 3.0))
        for s in range(n_seg):
            (y0, x0), (y1, x1) = pts[s], pts[s + 1]
            dy, dx = y1 - y0, x1 - x0
            L2 = dy * dy + dx * dx + 1e-12
            t = np.clip(((yy - y0) * dy + (xx - x0) * dx) / L2, 0.0, 1.0)
            d2 = (yy - (y0 + t * dy)) ** 2 + (xx - (x0 + t * dx)) ** 2
            mask |= d2 <= half * half
    return mask


def stroke_image(rng: np.random.Generator, h: int = 28, w: int = 28,
                 density: float = 0.19, tol: float = 0.03, max_tries: int = 10000) -> np.ndarray:
    """Boolean [h, w] mask of 3-6 random thick polylines with density in band."""
    for _ in range(max_tries):
        m = _stroke_mask(rng, h, w)
        if abs(m.mean() - density) <= tol:
            return m
    raise RuntimeError("stroke_image: density band not reached")


# ----------------------------------------------------------------------------
# 3-D: thin shells of spheres / boxes / cylinders
# ----------------------------------------------------------------------------
def _shape_shell(rng: np.random.Generator, r: int, grids) -> np.ndarray:
    z, y, x = grids
    kind = int(rng.integers(0, 3))
    size = rng.uniform(0.15, 0.4, size=3) * r
    centre = rng.uniform(0.25 * r, 0.75 * r, size=3)
    pz, py, px = z - centre[0], y - centre[1], x - centre[2]
    if kind == 0:  # sphere
        sd = np.sqrt(pz * pz + py * py + px * px) - size[0]
    elif kind == 1:  # axis-aligned box, half extents size[0..2]
        qz, qy, qx = np.abs(pz) - size[0], np.abs(py) - size[1], np.abs(px) - size[2]
        outside = np.sqrt(np.maximum(qz, 0) ** 2 + np.maximum(qy, 0) ** 2 + np.maximum(qx, 0) ** 2)
        inside = np.minimum(np.maximum(qz, np.maximum(qy, qx)), 0.0)
        sd = outside + inside
    else:  # axis-aligned cylinder, random axis, radius size[0], half height size[1]
        axis = int(rng.integers(0, 3))
        p = [pz, py, px]
        a = p.pop(axis)
        rad = np.sqrt(p[0] * p[0] + p[1] * p[1]) - size[0]
        hh = np.abs(a) - size[1]
        outside = np.sqrt(np.maximum(rad, 0) ** 2 + np.maximum(hh, 0) ** 2)
        inside = np.minimum(np.maximum(rad, hh), 0.0)
        sd = outside + inside
    return np.abs(sd) < 0.5


def shell_volume(rng: np.random.Generator, r: int, density: float, tol: float,
                 max_tries: int = 2000) -> np.ndarray:
    """Boolean [r, r, r]: union of 2-5 voxelised shape surfaces, density in band."""
    ax = np.arange(r, dtype=np.float32) + 0.5
    grids = np.meshgrid(ax, ax, ax, indexing="ij", sparse=True)
    for _ in range(max_tries):
        occ = np.zeros((r, r, r), dtype=bool)
        for n_shapes in range(1, 6):
            occ |= _shape_shell(rng, r, grids)
            d = occ.mean()
            if n_shapes >= 2 and abs(d - density) <= tol:
                return occ
            if d > density + tol:
                break
    raise RuntimeError("shell_volume: density band not reached")


def random_sparse_sites(rng: np.random.Generator, extent: Sequence[int], batch: int,
                        density: float) -> np.ndarray:
    """Uniformly scattered occupancy (the paper's own runtime workload, Sec. 4.1)."""
    occ = rng.random((batch, *extent)) < density
    return occupancy_to_rows(occ)


# ----------------------------------------------------------------------------
# filters
# ----------------------------------------------------------------------------
def make_filter(rng: np.random.Generator, ksize: Sequence[int], c_in: int, c_out: int,
                density: float, sigma: float) -> np.ndarray:
    """w[T, C_in, C_out]; each weight kept independently with prob `density`."""
    t = int(np.prod(ksize))
    w = rng.normal(0.0, sigma, size=(t, c_in, c_out)).astype(np.float32)
    if density < 1.0:
        keep = rng.random((t, c_in, c_out)) < density
        w = np.where(keep, w, np.float32(0.0)).astype(np.float32)
    return np.ascontiguousarray(w)


def _uniform_open_closed(rng: np.random.Generator, shape) -> np.ndarray:
    """U(0, 1] as float32, never exactly zero."""
    v = (1.0 - rng.random(shape)).astype(np.float32)
    v[v <= 0.0] = np.float32(1.0)
    return v


# ----------------------------------------------------------------------------
# the five configurations
# ----------------------------------------------------------------------------
CONFIGS = {
    1: dict(name="cfg1_2d28_strokes", ndim=2, r=28, batch=1, density=0.19, tol=0.03,
            layers=[LayerSpec(1, 8, (3, 3), 0.5, 0.3, 0.15, True, True)]),
    2: dict(name="cfg2_3d32_shells", ndim=3, r=32, batch=8, density=0.09, tol=0.015,
            layers=[LayerSpec(1, 16, (3, 3, 3), 0.5, 0.2, 0.15, True, False)]),
    3: dict(name="cfg3_3d64_shells_2layer", ndim=3, r=64, batch=8, density=0.05, tol=0.01,
            layers=[LayerSpec(16, 32, (3, 3, 3), 0.5, 0.2, 0.10, True, True),
                    LayerSpec(32, 32, (3, 3, 3), 0.5, 0.2, 0.10, True, False)]),
    4: dict(name="cfg4_3d128_shells_dense_filter", ndim=3, r=128, batch=4, density=0.027, tol=0.005,
            layers=[LayerSpec(32, 64, (3, 3, 3), 1.0, 0.2, 0.05, True, False)]),
    5: dict(name="cfg5_3d256_shells_5x5x5", ndim=3, r=256, batch=1, density=0.013, tol=0.003,
            layers=[LayerSpec(64, 64, (5, 5, 5), 0.3, 0.2, 0.05, False, False)]),
}
CFG5_RHO_SWEEP = (0.02, 0.05, 0.10)


def make_config(index: int, seed: int | None = None, *, r: int | None = None,
                batch: int | None = None) -> Workload:
    """Build configuration `index` (1..5).  `r` / `batch` override the size
    (same recipe on a smaller grid) for quick tests."""
    cfg = CONFIGS[index]
    seed = BASE_SEED + index if seed is None else seed
    rng = np.random.default_rng(seed)
    rr = cfg["r"] if r is None else r
    bb = cfg["batch"] if batch is None else batch
    ndim = cfg["ndim"]
    layers: List[LayerSpec] = cfg["layers"]
    c_in = layers[0].c_in
    if ndim == 2:
        occ = np.stack([stroke_image(rng, rr, rr, cfg["density"], cfg["tol"]) for _ in range(bb)])
        coords = occupancy_to_rows(occ)
        feats = _uniform_open_closed(rng, (coords.shape[0], c_in))
        extent = (rr, rr)
    else:
        # the density targets follow ~3/r; when r is overridden keep that law
        dens = cfg["density"] * cfg["r"] / rr if r is not None else cfg["density"]
        tol = cfg["tol"] * cfg["r"] / rr if r is not None else cfg["tol"]
        occ = np.stack([shell_volume(rng, rr, dens, tol) for _ in range(bb)])
        coords = occupancy_to_rows(occ)
        if index == 2:
            feats = np.ones((coords.shape[0], c_in), dtype=np.float32)
        else:
            feats = _uniform_open_closed(rng, (coords.shape[0], c_in))
        extent = (rr, rr, rr)
    filters = [make_filter(rng, L.ksize, L.c_in, L.c_out, L.filter_density, L.sigma) for L in layers]
    return Workload(name=cfg["name"], ndim=ndim, extent=extent, batch=bb, coords=coords,
                    feats=np.ascontiguousarray(feats), layers=list(layers), filters=filters,
                    density=float(occ.mean()), seed=seed)


def make_paper_runtime(r: int, rho_f: float, seed: int | None = None) -> Workload:
    """The paper's own runtime experiment (Sec. 4.1): one r^3 grid whose sites are occupied independently with
    probability 1/r and hold random non-zero values, one input channel, eight output channels, a 3x3x3 filter whose
    weights are kept with probability rho_f, rho_up = 1/r, batch 1."""
    seed = BASE_SEED + 1000 + r if seed is None else seed
    rng = np.random.default_rng(seed)
    extent = (r, r, r)
    coords = random_sparse_sites(rng, extent, 1, 1.0 / r)
    feats = _uniform_open_closed(rng, (coords.shape[0], 1))
    layer = LayerSpec(c_in=1, c_out=8, ksize=(3, 3, 3), filter_density=rho_f, sigma=0.2, rho_up=1.0 / r,
                      relu=False, pool=False)
    w = make_filter(rng, layer.ksize, 1, 8, rho_f, layer.sigma)
    return Workload(name=f"paper_runtime_r{r}_rhof{rho_f:g}", ndim=3, extent=extent, batch=1, coords=coords,
                    feats=np.ascontiguousarray(feats), layers=[layer], filters=[w],
                    density=coords.shape[0] / float(r) ** 3, seed=seed)


# Upper density bounds of the three sparse blocks of the paper's OctNet3 variants (appendix, network architectures).
OCTNET3_RHO = {32: (0.14, 0.33, 0.66), 64: (0.06, 0.14, 0.33), 128: (0.02, 0.06, 0.14)}


def make_octnet3_stack(r: int, batch: int = 2, seed: int | None = None) -> Workload:
    """The sparse part of the paper's OctNet3-r^3 network (appendix table of architectures) with random weights:
    three blocks of three 3x3x3 convolutions, 1 -> 8 -> 8 -> 8 | 8 -> 16 -> 16 -> 16 | 16 -> 24 -> 24 -> 24 channels,
    block i bounded by rho_i, a 2^3 max-pooling after the first two blocks, sparseToDense after the third.  Every
    convolution is followed by ReLU (a reading: the table lists the convolutions only).  Input: occupancy (value 1)
    of shell surfaces at density about 3/r, as in the other 3-D workloads.  `pool` of a layer means "pool after it"."""
    rho = OCTNET3_RHO[r]
    seed = BASE_SEED + 2000 + r if seed is None else seed
    rng = np.random.default_rng(seed)
    dens, tol = 2.9 / r, 0.6 / r
    occ = np.stack([shell_volume(rng, r, dens, tol) for _ in range(batch)])
    coords = occupancy_to_rows(occ)
    feats = np.ones((coords.shape[0], 1), dtype=np.float32)
    chans = [(1, 8), (8, 8), (8, 8), (8, 16), (16, 16), (16, 16), (16, 24), (24, 24), (24, 24)]
    layers = [LayerSpec(c_in=ci, c_out=co, ksize=(3, 3, 3), filter_density=1.0, sigma=float(np.sqrt(2.0 / (27 * ci))),
                        rho_up=rho[i // 3], relu=True, pool=(i in (2, 5))) for i, (ci, co) in enumerate(chans)]
    filters = [make_filter(rng, L.ksize, L.c_in, L.c_out, 1.0, L.sigma) for L in layers]
    return Workload(name=f"octnet3_{r}_sparse_part", ndim=3, extent=(r, r, r), batch=batch, coords=coords,
                    feats=feats, layers=layers, filters=filters, density=float(occ.mean()), seed=seed)
