"""Rounding model of a 16-bit evaluation of Eq. 7 (TEST INFRASTRUCTURE, numpy, not part of the product path).

The oracle proper keeps every activation in fp64, so its distance to a 16-bit evaluation mixes two things: the
rounding that any evaluation with 16-bit operands has, and whatever a kernel may do wrong.  This module is the
first of the two on its own: Eq. 7 with the architecture of Sec. 3.2 exactly as `kn_oracle.c` computes it, except
that every operand of a matrix product is first rounded to the storage type (round to nearest even): the encoded
inputs gamma(x) and gamma(d), the hidden vectors after layers 1, 2 and 4, and the feature vector out of layer 3.
Sums are kept in fp64 (an fp32 accumulator differs from that by about 1e-7 relative, three orders of magnitude
below a 16-bit rounding); the density and the colour are not rounded.  It says nothing about any kernel's
internals beyond "operands are 16 bit, sums are not", and shares no code with the HIP path.

`fold=True` is the same model for an evaluation that takes layer 3's feature vector and layer 4 as one affine map:
Sec. 3.2 puts no activation between them, so W4f^T (W3f^T h2 + b3f) + W4d^T gamma(d) + b4 equals
(W3f W4f)^T h2 + W4d^T gamma(d) + (b4 + W4f^T b3f).  The operands of that product are h2, gamma(d), the matrix
W3f W4f and the bias b4 + W4f^T b3f, the last two rounded to the storage type like every other operand; the feature
vector itself is then never rounded.

Uses: tests compare it with the fp64 oracle to measure how much of an error budget rounding alone takes (the
answer depends on the scene: a density error is multiplied by the sample spacing in Eq. 4), and compare the HIP
path with it at a far tighter tolerance than the 16-bit bar allows against the fp64 oracle.
"""
from __future__ import annotations

import numpy as np


def round_operand(a, dtype: str) -> np.ndarray:
    """fp64/fp32 array -> values representable in `dtype` ('f16' | 'bf16' | 'f32'), round to nearest even, as fp64."""
    a32 = np.asarray(a, np.float64).astype(np.float32)
    if dtype == "f32":
        return a32.astype(np.float64)
    if dtype == "f16":
        return a32.astype(np.float16).astype(np.float64)
    if dtype == "bf16":
        u = np.ascontiguousarray(a32).view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(np.float32).reshape(a32.shape).astype(np.float64)
    raise ValueError(dtype)


def _gamma(p32: np.ndarray, L: int) -> np.ndarray:
    """[p, then per k: sin(2^k p) (xyz), cos(2^k p) (xyz)] of fp32 3-vectors (M, 3) -> (M, 3 + 6L) in fp64."""
    out = [p32.astype(np.float64)]
    for k in range(L):
        a = (p32 * np.float32(2.0 ** k)).astype(np.float64)      # 2^k p is exact in fp32
        out += [np.sin(a), np.cos(a)]
    return np.concatenate(out, axis=1)


def _layers(w: np.ndarray, H: int, L_pos: int, L_dir: int):
    ex, ed = 3 + 6 * L_pos, 3 + 6 * L_dir
    shapes = [(ex, H), (H, H), (H, H + 1), (H + ed, H), (H, 3)]
    out, off = [], 0
    for i, o in shapes:
        W = w[off:off + i * o].reshape(i, o).astype(np.float64)
        off += i * o
        out.append((W, w[off:off + o].astype(np.float64)))
        off += o
    assert off == len(w)
    return out


def mlp_one_network(w, H: int, x, d, dtype: str, L_pos: int = 10, L_dir: int = 4, fold: bool = False):
    """One network (its P canonical parameters, already representable in `dtype`) on M inputs -> sigma (M), rgb (M, 3).
    fold: feature layer and layer 4 as one affine map of the second hidden vector (see the module's header)."""
    (W1, b1), (W2, b2), (W3, b3), (W4, b4), (W5, b5) = _layers(np.asarray(w), H, L_pos, L_dir)
    rnd = lambda a: round_operand(a, dtype)
    gx = rnd(_gamma(np.asarray(x, np.float32).reshape(-1, 3), L_pos))
    gd = rnd(_gamma(np.asarray(d, np.float32).reshape(-1, 3), L_dir))
    h1 = rnd(np.maximum(gx @ W1 + b1, 0.0))
    h2 = rnd(np.maximum(h1 @ W2 + b2, 0.0))
    o3 = h2 @ W3 + b3
    sigma = np.maximum(o3[:, 0], 0.0)
    if fold:
        W34, b34 = rnd(W3[:, 1:] @ W4[:H]), rnd(b4 + b3[1:] @ W4[:H])
        h4 = rnd(np.maximum(h2 @ W34 + gd @ W4[H:] + b34, 0.0))
    else:
        feat = rnd(o3[:, 1:])
        h4 = rnd(np.maximum(np.concatenate([feat, gd], axis=1) @ W4 + b4, 0.0))
    rgb = 1.0 / (1.0 + np.exp(-(h4 @ W5 + b5)))
    return sigma, rgb


def eval_points(weights, H: int, ids, points, dirs, dtype: str, fold: bool = False):
    """eval_grouped under the rounding model: `ids` are the network ids of the points (-1: none -> zeros)."""
    ids = np.asarray(ids)
    M = len(ids)
    sigma, rgb = np.zeros(M), np.zeros((M, 3))
    for n in np.unique(ids[ids >= 0]):
        sel = np.nonzero(ids == n)[0]
        sigma[sel], rgb[sel] = mlp_one_network(weights[n], H, points[sel], dirs[sel], dtype, fold=fold)
    return sigma, rgb


def fma32(a, b, c) -> np.ndarray:
    """fp32 fused multiply-add of fp32 operands (the product of two fp32 numbers is exact in fp64; the one rounding
    of the sum to fp64 in front of the rounding to fp32 matters in about one case in 2^29)."""
    return (np.asarray(a, np.float64) * np.asarray(b, np.float64) + np.asarray(c, np.float64)).astype(np.float32)


def render_midpoint(orc, weights, H: int, dtype: str, rays_o, rays_d, t_near, step, K, eps, bg):
    """Sec. 3.4 / Eq. 2-4 with the rounding model in place of the networks: the oracle marches (`orc.march`), the
    samples' positions are the lattice points t_k = t_near + (k + 1/2) step, x = o + t_k d in fp32, the model
    evaluates them, the oracle blends (`oracle.composite`).  Midpoint lattice only.  -> image (R, 3) fp64."""
    from . import composite
    step32, tn32 = np.float32(step), np.float32(t_near)
    img = np.tile(np.asarray(bg, np.float64), (len(rays_o), 1))
    pts, dirs, owner = [], [], []
    for r in range(len(rays_o)):
        kk = orc.march(rays_o[r], rays_d[r], t_near, step, K)
        if len(kk) == 0:
            continue
        t = fma32(kk.astype(np.float64) + 0.5, step32, tn32)
        pts.append(np.stack([fma32(t, rays_d[r, a], rays_o[r, a]) for a in range(3)], axis=1))
        dirs.append(np.tile(rays_d[r], (len(kk), 1)))
        owner.append(np.full(len(kk), r))
    if not pts:
        return img
    pts, dirs, owner = np.concatenate(pts), np.concatenate(dirs), np.concatenate(owner)
    sg, rgb = eval_points(weights, H, orc.cell_ids(pts), pts, dirs, dtype)
    cuts = np.flatnonzero(np.diff(owner)) + 1
    for s, e in zip(np.concatenate([[0], cuts]), np.concatenate([cuts, [len(owner)]])):
        img[owner[s]] = composite(sg[s:e], rgb[s:e], float(step32), eps, bg)[0]
    return img


def extract_occupancy(orc, weights, H: int, dtype: str, occ_res, tau, voxels=None):
    """Sec. 3.4 occupancy extraction with the rounding model in place of the networks: 27 probes per voxel at the
    sub-cell centres (offsets 1/6, 1/2, 5/6; x = fma((float)v + c, cell, b_min) in fp32, as the oracle places them),
    marked iff a density is above tau.  -> (occupancy bytes, min over the probes of |sigma - tau|), per voxel given
    (linear indices, x slowest) or for the whole grid (flat)."""
    res = np.asarray(occ_res, np.int64)
    vox = np.arange(int(res.prod()), dtype=np.int64) if voxels is None else np.asarray(voxels, np.int64)
    v = np.stack([vox // (res[1] * res[2]), (vox // res[2]) % res[1], vox % res[2]], axis=1)
    cell = ((orc.aabb_max - orc.aabb_min) / res.astype(np.float32)).astype(np.float32)
    sub = np.array([1.0 / 6.0, 0.5, 5.0 / 6.0], np.float32)
    pick = np.stack(np.meshgrid(sub, sub, sub, indexing="ij"), -1).reshape(27, 3)
    at = (v[:, None, :].astype(np.float32) + pick[None, :, :]).astype(np.float32)          # (n, 27, 3), fp32 sums
    x = fma32(at, cell[None, None, :], orc.aabb_min[None, None, :]).reshape(-1, 3)
    d = np.tile(np.float32([0.0, 0.0, 1.0]), (len(x), 1))
    sg = eval_points(weights, H, orc.cell_ids(x), x, d, dtype)[0].reshape(-1, 27)
    return (sg > float(np.float32(tau))).any(axis=1).astype(np.uint8), np.abs(sg - float(np.float32(tau))).min(axis=1)
