"""Seeded synthetic inputs for the KiloNeRF rendering path.

This module serves both the HIP library's callers (tests, benchmark) and the CPU oracle's tests.
It only *draws inputs*: random weights, occupancy grids, cameras / rays, query points.  None of
the method's arithmetic (cell assignment, encoding, network layers, marching, compositing) lives
here.  Every generator is a pure function of its arguments and an integer seed (numpy Philox).

The paper measures on trained scenes of four public datasets (Sec. 4.1) that are not available
here; these generators stand in for them with the same shapes: image sizes 800x800 and
1920x1080, network grids up to 16^3 with a 16x finer occupancy grid, tiny MLPs with 4 hidden
layers of 32 units, eps = 0.01.
"""
from __future__ import annotations

import math

import numpy as np

BASE_SEED = 210313744


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(int(seed)))


# ---------------------------------------------------------------------------------------------
# canonical weight layout (an interface shared by every consumer; sizes only, no arithmetic)
# ---------------------------------------------------------------------------------------------
def layer_shapes(hidden: int, L_pos: int = 10, L_dir: int = 4):
    """[(fan_in, fan_out)] of the five affine layers, in storage order."""
    ex, ed = 3 + 6 * L_pos, 3 + 6 * L_dir
    H = hidden
    return [(ex, H), (H, H), (H, H + 1), (H + ed, H), (H, 3)]


def params_per_net(hidden: int, L_pos: int = 10, L_dir: int = 4) -> int:
    return sum(i * o + o for i, o in layer_shapes(hidden, L_pos, L_dir))


def layer_views(weights: np.ndarray, hidden: int, L_pos: int = 10, L_dir: int = 4):
    """Views [(W_l, b_l)] into an (N, P) canonical weight array; W_l is (N, fan_in, fan_out)."""
    out, off = [], 0
    for i, o in layer_shapes(hidden, L_pos, L_dir):
        W = weights[:, off:off + i * o].reshape(-1, i, o)
        off += i * o
        b = weights[:, off:off + o]
        off += o
        out.append((W, b))
    assert off == weights.shape[1]
    return out


def kaiming_weights(n_nets: int, hidden: int, seed: int, L_pos: int = 10, L_dir: int = 4,
                    sigma_scale: float = 1.0) -> np.ndarray:
    """(N, P) float32: W ~ U(+-sqrt(6/fan_in)), b ~ U(+-1/sqrt(fan_in)) per layer.

    ``sigma_scale`` multiplies the density column of layer 3 (weights and bias) so that random
    networks give opaque-looking scenes; it is part of the input, not of the method."""
    g = rng(seed)
    P = params_per_net(hidden, L_pos, L_dir)
    w = np.empty((n_nets, P), np.float32)
    for (W, b), (fi, fo) in zip(layer_views(w, hidden, L_pos, L_dir), layer_shapes(hidden, L_pos, L_dir)):
        bw, bb = math.sqrt(6.0 / fi), 1.0 / math.sqrt(fi)
        W[...] = g.uniform(-bw, bw, size=W.shape).astype(np.float32)
        b[...] = g.uniform(-bb, bb, size=b.shape).astype(np.float32)
    if sigma_scale != 1.0:
        W3, b3 = layer_views(w, hidden, L_pos, L_dir)[2]
        W3[:, :, 0] *= np.float32(sigma_scale)
        b3[:, 0] *= np.float32(sigma_scale)
    return w


def round_to_storage(weights: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the storage type ('f32' | 'f16' | 'bf16', round to nearest even)
    and return them as float32, so both consumers receive exactly representable values."""
    w = np.ascontiguousarray(weights, np.float32)
    if dtype == "f32":
        return w.copy()
    if dtype == "f16":
        return w.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = w.view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(w.shape)
    raise ValueError(dtype)


def to_storage_bits(weights_f32_rounded: np.ndarray, dtype: str) -> np.ndarray:
    """Bit pattern array handed to the device for a storage type (float32 / float16 / uint16 for bf16)."""
    if dtype == "f32":
        return np.ascontiguousarray(weights_f32_rounded, np.float32)
    if dtype == "f16":
        return weights_f32_rounded.astype(np.float16)
    if dtype == "bf16":
        return (np.ascontiguousarray(weights_f32_rounded, np.float32).view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(dtype)


# ---------------------------------------------------------------------------------------------
# occupancy grids
# ---------------------------------------------------------------------------------------------
def blob_occupancy(res, n_blobs: int, occupied_fraction: float, seed: int) -> np.ndarray:
    """uint8 (ox, oy, oz): 1 where a sum of seeded isotropic Gaussian blobs, sampled at voxel
    centres of the unit-normalised box, exceeds the (1 - occupied_fraction) quantile."""
    g = rng(seed)
    res = tuple(int(r) for r in res)
    mu = g.uniform(0.2, 0.8, size=(n_blobs, 3))          # central 60 % of the box
    s = g.uniform(0.04, 0.12, size=n_blobs)               # std. dev. as a fraction of the extent
    amp = g.uniform(0.5, 1.0, size=n_blobs)
    axes = [(np.arange(r) + 0.5) / r for r in res]
    gx = np.exp(-0.5 * ((axes[0][None, :] - mu[:, 0:1]) / s[:, None]) ** 2) * amp[:, None]
    gy = np.exp(-0.5 * ((axes[1][None, :] - mu[:, 1:2]) / s[:, None]) ** 2)
    gz = np.exp(-0.5 * ((axes[2][None, :] - mu[:, 2:3]) / s[:, None]) ** 2)
    gyz = (gy[:, :, None] * gz[:, None, :]).reshape(n_blobs, -1).astype(np.float32)
    field = (gx.T.astype(np.float32) @ gyz)               # (ox, oy*oz)
    kth = int((1.0 - occupied_fraction) * field.size)
    thr = np.partition(field.ravel(), kth)[kth]
    return (field >= thr).astype(np.uint8).reshape(res)


# ---------------------------------------------------------------------------------------------
# cameras, rays, points
# ---------------------------------------------------------------------------------------------
def camera_rays(width: int, height: int, fov_x_deg: float, radius: float, azimuth_deg: float,
                elevation_deg: float, center=(0.0, 0.0, 0.0)):
    """Pinhole camera on a sphere around ``center`` looking at it (up = +z).  One ray through
    each pixel centre; returns (rays_o, rays_d) float32 (H*W, 3), directions of unit length."""
    az, el = math.radians(azimuth_deg), math.radians(elevation_deg)
    c = np.asarray(center, np.float64)
    eye = c + radius * np.array([math.cos(el) * math.cos(az), math.cos(el) * math.sin(az), math.sin(el)])
    fwd = (c - eye) / np.linalg.norm(c - eye)
    right = np.cross(fwd, np.array([0.0, 0.0, 1.0]))
    right /= np.linalg.norm(right)
    up = np.cross(right, fwd)
    half = math.tan(math.radians(fov_x_deg) / 2.0)
    px = ((np.arange(width) + 0.5) / width * 2.0 - 1.0) * half
    py = (1.0 - (np.arange(height) + 0.5) / height * 2.0) * half * (height / width)
    d = fwd[None, None, :] + px[None, :, None] * right[None, None, :] + py[:, None, None] * up[None, None, :]
    d /= np.linalg.norm(d, axis=-1, keepdims=True)
    o = np.broadcast_to(eye, d.shape)
    return (np.ascontiguousarray(o.reshape(-1, 3), np.float32),
            np.ascontiguousarray(d.reshape(-1, 3), np.float32))


def sphere_dirs(m: int, seed: int) -> np.ndarray:
    g = rng(seed)
    z = g.uniform(-1.0, 1.0, size=m)
    phi = g.uniform(0.0, 2.0 * math.pi, size=m)
    s = np.sqrt(np.maximum(0.0, 1.0 - z * z))
    return np.stack([s * np.cos(phi), s * np.sin(phi), z], axis=1).astype(np.float32)


def uniform_points(m: int, seed: int, lo=(0.0, 0.0, 0.0), hi=(1.0, 1.0, 1.0)) -> np.ndarray:
    g = rng(seed)
    lo, hi = np.asarray(lo, np.float64), np.asarray(hi, np.float64)
    return (lo + g.random(size=(m, 3)) * (hi - lo)).astype(np.float32)


def skewed_points(m: int, res, seed: int, hot_cell_fraction: float = 0.05, hot_point_fraction: float = 0.9,
                  lo=(0.0, 0.0, 0.0), hi=(1.0, 1.0, 1.0)) -> np.ndarray:
    """Load-skew input: ``hot_point_fraction`` of the points cluster (Gaussian, clamped) inside a
    seeded ``hot_cell_fraction`` of the cells of a grid ``res``; the rest is uniform; shuffled."""
    g = rng(seed)
    res = np.asarray(res, np.int64)
    lo, hi = np.asarray(lo, np.float64), np.asarray(hi, np.float64)
    n_cells = int(res.prod())
    n_hot = max(1, int(round(hot_cell_fraction * n_cells)))
    hot = g.choice(n_cells, size=n_hot, replace=False)
    m_hot = int(round(hot_point_fraction * m))
    which = hot[g.integers(0, n_hot, size=m_hot)]
    iz = which % res[2]
    iy = (which // res[2]) % res[1]
    ix = which // (res[1] * res[2])
    cell = (hi - lo) / res
    centre = lo + (np.stack([ix, iy, iz], axis=1) + 0.5) * cell
    off = np.clip(g.normal(0.0, 0.2, size=(m_hot, 3)), -0.49, 0.49) * cell
    pts = np.concatenate([centre + off, lo + g.random(size=(m - m_hot, 3)) * (hi - lo)], axis=0)
    g.shuffle(pts, axis=0)
    return pts.astype(np.float32)
