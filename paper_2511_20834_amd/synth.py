"""Seeded synthetic voxel clouds, features and weights.

This module only draws inputs: raw integer ``(b, x, y, z)`` voxel coordinates
(unique rows, in shuffled order), feature matrices and weight tensors.  It holds
none of the sparse-convolution arithmetic (no packing, no downsampling, no
kernel maps, no contractions), so that the CPU oracle and the HIP path can both
be fed from it without sharing any part of the method.

The clouds stand in for the outdoor LiDAR and indoor RGB-D datasets the paper
evaluates on (Section 6.1), which are licensed and not redistributable; the
random-volume generators follow the paper's ablation set-up (Section 6.6).
"""
from __future__ import annotations

import numpy as np

SEED_BASE = 20834 * 10


def _unique_rows_shuffled(coords: np.ndarray, rng: np.random.Generator) -> np.ndarray:
    coords = np.unique(coords.astype(np.int32), axis=0)
    rng.shuffle(coords, axis=0)
    return np.ascontiguousarray(coords, dtype=np.int32)


def _with_batch(xyz: np.ndarray, b: int) -> np.ndarray:
    out = np.empty((xyz.shape[0], 4), dtype=np.int32)
    out[:, 0] = b
    out[:, 1:] = xyz
    return out


# ----------------------------------------------------------------------------
# config 0: tiny surface cloud in a 64^3 grid
# ----------------------------------------------------------------------------
def tiny_cloud(seed: int = SEED_BASE + 0, n_plane: int = 1100, n_sphere: int = 450) -> np.ndarray:
    """Plane z=4 over x,y in [0,64) plus three spheres (r ~ U(8,15)), sampled at
    random surface points, quantised to the unit grid and deduplicated."""
    rng = np.random.default_rng(seed)
    pts = [np.stack([rng.uniform(0, 64, n_plane), rng.uniform(0, 64, n_plane),
                     np.full(n_plane, 4.5)], axis=1)]
    for _ in range(3):
        r = rng.uniform(8, 15)
        c = rng.uniform(16, 48, size=3)
        d = rng.normal(size=(n_sphere, 3))
        d /= np.linalg.norm(d, axis=1, keepdims=True)
        pts.append(c + r * d)
    p = np.floor(np.concatenate(pts)).astype(np.int64)
    keep = np.all((p >= 0) & (p < 64), axis=1)
    return _unique_rows_shuffled(_with_batch(p[keep], 0), rng)


# ----------------------------------------------------------------------------
# config 1: LiDAR-like scene
# ----------------------------------------------------------------------------
def _ray_box(o, d, lo, hi):
    """Slab test; returns entry distance (inf where missed). o:(3,), d:(R,3)."""
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = 1.0 / d
        t0 = (lo - o) * inv
        t1 = (hi - o) * inv
    tmin = np.minimum(t0, t1).max(axis=1)
    tmax = np.maximum(t0, t1).min(axis=1)
    hit = (tmax >= np.maximum(tmin, 0.0)) & (tmin > 0)
    return np.where(hit, tmin, np.inf)


def _ray_cylinder(o, d, cx, cy, r, h):
    """Vertical cylinder of radius r, z in [0,h]; side surface only."""
    ox, oy = o[0] - cx, o[1] - cy
    a = d[:, 0] ** 2 + d[:, 1] ** 2
    b = 2 * (ox * d[:, 0] + oy * d[:, 1])
    c = ox * ox + oy * oy - r * r
    disc = b * b - 4 * a * c
    with np.errstate(divide="ignore", invalid="ignore"):
        t = (-b - np.sqrt(np.maximum(disc, 0))) / (2 * a)
    z = o[2] + t * d[:, 2]
    hit = (disc > 0) & (t > 0) & (z >= 0) & (z <= h) & (a > 0)
    return np.where(hit, t, np.inf)


def lidar_cloud(seed: int = SEED_BASE + 1, target: int = 120_000, beams: int = 64,
                azimuths: int = 2048, voxel: float = 0.1) -> np.ndarray:
    """64-beam spinning sensor at z=1.8 m over the ground plane z=0 with 40
    random boxes and cylinders; hits quantised to 0.1 m voxels inside
    x,y in [-51.2,51.2) m, z in [-3,5) m.  One revolution of 64x2048 rays gives
    fewer than ``target`` unique voxels (sky misses, duplicates), so further
    revolutions with a sub-step azimuth shift, taken 0.7 m further along x each
    (a moving vehicle aggregating sweeps), are accumulated until ``target`` is
    reached; the surplus of the last revolution is trimmed by a seeded choice."""
    rng = np.random.default_rng(seed)
    boxes, cyls = [], []
    for i in range(40):
        ang, dist = rng.uniform(0, 2 * np.pi), rng.uniform(4, 45)
        cx, cy = dist * np.cos(ang), dist * np.sin(ang)
        if i % 2 == 0:
            sx, sy, sz = rng.uniform(1, 5, size=3)
            boxes.append((np.array([cx - sx / 2, cy - sy / 2, 0.0]),
                          np.array([cx + sx / 2, cy + sy / 2, sz])))
        else:
            cyls.append((cx, cy, rng.uniform(0.2, 1.0), rng.uniform(1, 5)))
    elev = np.deg2rad(np.linspace(-25.0, 3.0, beams))
    vox = np.empty((0, 3), dtype=np.int64)
    rev = 0
    while vox.shape[0] < target and rev < 16:
        az = (np.arange(azimuths) + rng.uniform(0, 1)) * (2 * np.pi / azimuths)
        o = np.array([0.7 * rev + rng.normal(0, 0.05), rng.normal(0, 0.05), 1.8 + rng.normal(0, 0.02)])
        e, a = np.meshgrid(elev + rng.normal(0, 2e-4, beams), az, indexing="ij")
        d = np.stack([np.cos(e) * np.cos(a), np.cos(e) * np.sin(a), np.sin(e)], axis=-1).reshape(-1, 3)
        with np.errstate(divide="ignore"):
            t = np.where(d[:, 2] < 0, -o[2] / d[:, 2], np.inf)
        for lo, hi in boxes:
            t = np.minimum(t, _ray_box(o, d, lo, hi))
        for cx, cy, r, h in cyls:
            t = np.minimum(t, _ray_cylinder(o, d, cx, cy, r, h))
        ok = np.isfinite(t)
        p = o + t[ok, None] * d[ok]
        p[:, 2] = np.maximum(p[:, 2], 0.0) + 1e-6  # ground hits sit in the z=0 voxel layer
        ok2 = (np.abs(p[:, 0]) < 51.2) & (np.abs(p[:, 1]) < 51.2) & (p[:, 2] >= -3) & (p[:, 2] < 5)
        v = np.floor(p[ok2] / voxel).astype(np.int64)
        vox = np.unique(np.concatenate([vox, v]), axis=0)
        rev += 1
    if vox.shape[0] > target:
        # keep whole revolutions' structure but trim to the target with a seeded choice
        vox = vox[np.sort(rng.choice(vox.shape[0], target, replace=False))]
    return _unique_rows_shuffled(_with_batch(vox, 0), rng)


# ----------------------------------------------------------------------------
# config 3: indoor-like rooms, batch 4
# ----------------------------------------------------------------------------
def _room_surface_voxels(rng: np.random.Generator, nx=500, ny=500, nz=150) -> np.ndarray:
    occ = []
    X, Y = np.meshgrid(np.arange(nx), np.arange(ny), indexing="ij")
    for z in (0, nz - 1):  # floor, ceiling
        occ.append(np.stack([X.ravel(), Y.ravel(), np.full(X.size, z)], 1))
    Xw, Zw = np.meshgrid(np.arange(nx), np.arange(nz), indexing="ij")
    for y in (0, ny - 1):
        occ.append(np.stack([Xw.ravel(), np.full(Xw.size, y), Zw.ravel()], 1))
    Yw, Zw = np.meshgrid(np.arange(ny), np.arange(nz), indexing="ij")
    for x in (0, nx - 1):
        occ.append(np.stack([np.full(Yw.size, x), Yw.ravel(), Zw.ravel()], 1))
    for _ in range(30):  # furniture: axis-aligned boxes standing on the floor, 0.3-2 m sides
        s = rng.integers(15, 100, size=3)
        x0, y0 = rng.integers(1, nx - 1 - s[0]), rng.integers(1, ny - 1 - s[1])
        x1, y1, z1 = x0 + s[0], y0 + s[1], min(int(s[2]), nz - 2)
        xs, ys, zs = np.arange(x0, x1 + 1), np.arange(y0, y1 + 1), np.arange(1, z1 + 1)
        A, B = np.meshgrid(xs, ys, indexing="ij")
        occ.append(np.stack([A.ravel(), B.ravel(), np.full(A.size, z1)], 1))  # top
        A, B = np.meshgrid(xs, zs, indexing="ij")
        for y in (y0, y1):
            occ.append(np.stack([A.ravel(), np.full(A.size, y), B.ravel()], 1))
        A, B = np.meshgrid(ys, zs, indexing="ij")
        for x in (x0, x1):
            occ.append(np.stack([np.full(A.size, x), A.ravel(), B.ravel()], 1))
    return np.unique(np.concatenate(occ).astype(np.int32), axis=0)


def indoor_cloud(seed: int = SEED_BASE + 3, batch: int = 4, per_scene: int = 60_000) -> np.ndarray:
    """``batch`` rooms of 10 m x 10 m x 3 m at 2 cm voxels (floor, ceiling, four
    walls, 30 boxes); every scene's surface voxels are subsampled uniformly at
    random to ``per_scene`` voxels.  The batch index is the first column."""
    rng = np.random.default_rng(seed)
    scenes = []
    for b in range(batch):
        v = _room_surface_voxels(rng)
        sel = rng.choice(v.shape[0], min(per_scene, v.shape[0]), replace=False)
        scenes.append(_with_batch(v[sel], b))
    return _unique_rows_shuffled(np.concatenate(scenes), rng)


# ----------------------------------------------------------------------------
# random volumes (ablation set-up of Section 6.6)
# ----------------------------------------------------------------------------
def random_cloud(n_voxels: int, dims=(200, 200, 200), seed: int = SEED_BASE + 7, batch: int = 1) -> np.ndarray:
    """``n_voxels`` distinct voxels drawn uniformly from a ``dims`` volume per batch item."""
    rng = np.random.default_rng(seed)
    vol = int(dims[0]) * int(dims[1]) * int(dims[2])
    out = []
    for b in range(batch):
        if n_voxels * 8 > vol:
            lin = rng.choice(vol, n_voxels, replace=False)
        else:
            lin = np.unique(rng.integers(0, vol, size=int(n_voxels * 1.05) + 16))
            while lin.size < n_voxels:
                lin = np.unique(np.concatenate([lin, rng.integers(0, vol, size=n_voxels)]))
            lin = rng.choice(lin, n_voxels, replace=False)
        x, r = np.divmod(lin, dims[1] * dims[2])
        y, z = np.divmod(r, dims[2])
        out.append(_with_batch(np.stack([x, y, z], 1), b))
    return _unique_rows_shuffled(np.concatenate(out), rng)


def scaled_random_cloud(n_voxels: int, density: float = 0.0125, seed: int = SEED_BASE + 8) -> np.ndarray:
    """Volume [n, n, 200] with n chosen so that ``n_voxels`` voxels give ``density``."""
    n = max(8, int(round(np.sqrt(n_voxels / (density * 200.0)))))
    return random_cloud(n_voxels, (n, n, 200), seed)


def full_grid(n: int, batch: int = 1) -> np.ndarray:
    """Every voxel of an n^3 grid (closed-form kernel maps exist for it)."""
    g = np.stack(np.meshgrid(np.arange(n), np.arange(n), np.arange(n), indexing="ij"), -1).reshape(-1, 3)
    return np.concatenate([_with_batch(g, b) for b in range(batch)]).astype(np.int32)


# ----------------------------------------------------------------------------
# features and weights
# ----------------------------------------------------------------------------
def features(n: int, c: int, dtype=np.float16, seed: int = 1) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, c), dtype=np.float32).astype(dtype)


def weights(k_vol: int, cin: int, cout: int, dtype=np.float16, seed: int = 2, std: float | None = None) -> np.ndarray:
    """Weights [K^3, Cin, Cout]; He initialisation (std sqrt(2 / (K^3 Cin))) unless ``std`` is given."""
    rng = np.random.default_rng(seed)
    if std is None:
        std = float(np.sqrt(2.0 / (k_vol * cin)))
    return (rng.standard_normal((k_vol, cin, cout), dtype=np.float32) * np.float32(std)).astype(dtype)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


CONFIGS = {
    0: dict(cloud="tiny", K=3, layer_stride=1, cin=16, cout=16, dtype="f32"),
    1: dict(cloud="lidar", K=3, layer_stride=1, cin=64, cout=64, dtype="f16"),
    2: dict(cloud="lidar", K=3, layer_stride=2, cin=64, cout=128, dtype="f16"),
    3: dict(cloud="indoor", K=5, layer_stride=1, cin=32, cout=32, dtype="f16"),
}

_cloud_cache: dict = {}


def cloud(name: str) -> np.ndarray:
    """Named clouds of the benchmark configurations (memoised per process)."""
    if name not in _cloud_cache:
        _cloud_cache[name] = {"tiny": tiny_cloud, "lidar": lidar_cloud, "indoor": indoor_cloud}[name]()
    return _cloud_cache[name]


def layer_tensors(cfg: int, n_in: int):
    """(features, weights) for single-layer configuration ``cfg`` with ``n_in`` input voxels."""
    c = CONFIGS[cfg]
    dt = np.float32 if c["dtype"] == "f32" else np.float16
    k3 = c["K"] ** 3
    std = float(1.0 / np.sqrt(27 * 16)) if cfg == 0 else None
    f = features(n_in, c["cin"], dt, seed=SEED_BASE + 100 + cfg)
    w = weights(k3, c["cin"], c["cout"], dt, seed=SEED_BASE + 200 + cfg, std=std)
    return f, w


# ----------------------------------------------------------------------------
# config 4: UNet-style layer stack (a workload description, no arithmetic)
# ----------------------------------------------------------------------------
def unet_layers(cin: int = 4, widths=(32, 64, 128, 256)):
    """The 25 SpC layers of benchmark configuration 4 as dicts with keys
    name, K, in_stride, layer_stride, transposed, cin, cout, relu, src, skip, save.

    ``src`` / ``skip`` name the tensors a layer reads (``skip`` is concatenated after
    ``src`` along channels), ``save`` the name under which its output is kept.  Encoder:
    a 3x3x3 stem, then per stage a 2x2x2 stride-2 layer and two 3x3x3 submanifold
    layers.  Decoder: per stage a 2x2x2 transposed layer, concatenation with the encoder
    tensor of that level, and two 3x3x3 submanifold layers.  ReLU after every layer but
    the last; batch norm is folded into the weights (weights only, no bias)."""
    L = []
    w0 = widths[0]
    L.append(dict(name="stem", K=3, in_stride=1, layer_stride=1, transposed=0, cin=cin, cout=w0, src="input", skip=None,
                  save="enc0"))
    prev, c_prev = "enc0", w0
    for i, w in enumerate(widths):
        s = 2 ** i
        L.append(dict(name="down%d" % (i + 1), K=2, in_stride=s, layer_stride=2, transposed=0, cin=c_prev, cout=w, src=prev,
                      skip=None, save="d%d" % (i + 1)))
        L.append(dict(name="enc%da" % (i + 1), K=3, in_stride=2 * s, layer_stride=1, transposed=0, cin=w, cout=w,
                      src="d%d" % (i + 1), skip=None, save="e%da" % (i + 1)))
        L.append(dict(name="enc%db" % (i + 1), K=3, in_stride=2 * s, layer_stride=1, transposed=0, cin=w, cout=w,
                      src="e%da" % (i + 1), skip=None, save="enc%d" % (i + 1)))
        prev, c_prev = "enc%d" % (i + 1), w
    skip_w = [w0] + list(widths[:-1])  # widths of enc0 .. enc3
    for i in range(len(widths) - 1, -1, -1):
        s = 2 ** i  # stride of the finer level this stage produces
        c_up = skip_w[i]
        L.append(dict(name="up%d" % (i + 1), K=2, in_stride=s, layer_stride=2, transposed=1, cin=c_prev, cout=c_up, src=prev,
                      skip=None, save="u%d" % (i + 1)))
        L.append(dict(name="dec%da" % (i + 1), K=3, in_stride=s, layer_stride=1, transposed=0, cin=2 * c_up, cout=c_up,
                      src="u%d" % (i + 1), skip="enc%d" % i, save="g%da" % (i + 1)))
        L.append(dict(name="dec%db" % (i + 1), K=3, in_stride=s, layer_stride=1, transposed=0, cin=c_up, cout=c_up,
                      src="g%da" % (i + 1), skip=None, save="dec%d" % (i + 1)))
        prev, c_prev = "dec%d" % (i + 1), c_up
    for j, l in enumerate(L):
        l["relu"] = j != len(L) - 1
    return L


def unet_weights(layers, dtype=np.float16, seed: int = SEED_BASE + 400):
    return [weights(l["K"] ** 3, l["cin"], l["cout"], dtype, seed=seed + j) for j, l in enumerate(layers)]
