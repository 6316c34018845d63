"""The five benchmark workloads, as seeded synthetic inputs.

Each ``configN`` returns a dict of numpy arrays and call arguments.  ``weights`` are float32
values already rounded to the config's storage type (so the oracle and the device receive the
same numbers); ``wdtype`` names that type.  Image size and point counts can be reduced for
quick tests through the keyword arguments; the defaults are the full sizes.
"""
from __future__ import annotations

import math

import numpy as np

from . import (BASE_SEED, blob_occupancy, camera_rays, kaiming_weights, round_to_storage,
               skewed_points, sphere_dirs, uniform_points)


def _scene(res, lo, hi, hidden, wdtype, seed, sigma_scale=1.0, occ=None):
    n = int(np.prod(res))
    w = round_to_storage(kaiming_weights(n, hidden, seed, sigma_scale=sigma_scale), wdtype)
    return dict(res=tuple(res), aabb_min=tuple(float(v) for v in lo), aabb_max=tuple(float(v) for v in hi),
                hidden=hidden, wdtype=wdtype, weights=w, occupancy=occ, L_pos=10, L_dir=4)


def config1(width=64, height=64):
    """Tiny fp32 render: 2^3 networks, unit cube, camera at distance 2.5, 32 samples per ray,
    no occupancy grid, no early termination."""
    sc = _scene((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, "f32", BASE_SEED + 1)
    o, d = camera_rays(width, height, 40.0, 2.5, 30.0, 20.0, center=(0.5, 0.5, 0.5))
    r = math.sqrt(3.0) / 2.0
    return dict(scene=sc, rays_o=o, rays_d=d, t_near=2.5 - r, step=2 * r / 32, K=32, term_eps=0.0,
                bg=(0.0, 0.0, 0.0), width=width, height=height, name="cfg1_tiny_f32")


def config2(m=1 << 22, wdtype="f16"):
    """Isolated grouped MLP: 16^3 networks, uniform points in the unit cube, uniform directions."""
    sc = _scene((16, 16, 16), (0, 0, 0), (1, 1, 1), 32, wdtype, BASE_SEED + 2)
    return dict(scene=sc, points=uniform_points(m, BASE_SEED + 20), dirs=sphere_dirs(m, BASE_SEED + 21),
                name="cfg2_mlp_%s" % wdtype)


def _render_config(net_res, occ_res, hidden, wdtype, n_blobs, frac, width, height, steps, seed,
                   azimuth, sigma_scale, name):
    occ = blob_occupancy((occ_res,) * 3, n_blobs, frac, seed + 7)
    sc = _scene((net_res,) * 3, (-1, -1, -1), (1, 1, 1), hidden, wdtype, seed, sigma_scale=sigma_scale, occ=occ)
    o, d = camera_rays(width, height, 40.0, 4.0, azimuth, 30.0)
    diag = 2.0 * math.sqrt(3.0)
    return dict(scene=sc, rays_o=o, rays_d=d, t_near=4.0 - math.sqrt(3.0), step=diag / steps, K=steps,
                term_eps=0.01, bg=(1.0, 1.0, 1.0), width=width, height=height, name=name)


def config3(width=800, height=800, azimuth=45.0, sigma_scale=100.0, wdtype="f16"):
    """Full render: 16^3 networks, 256^3 occupancy grid (8 % occupied, 32 blobs), camera on a
    sphere of radius 4, 40 degree field of view, step = diagonal / 512, eps = 0.01."""
    return _render_config(16, 256, 32, wdtype, 32, 0.08, width, height, 512, BASE_SEED + 3, azimuth,
                          sigma_scale, "cfg3_render_%s" % wdtype)


def config4(m=1 << 23, wdtype="bf16"):
    """Load skew: 90 % of the points in 5 % of the cells."""
    sc = _scene((16, 16, 16), (0, 0, 0), (1, 1, 1), 32, wdtype, BASE_SEED + 4)
    return dict(scene=sc, points=skewed_points(m, (16, 16, 16), BASE_SEED + 40),
                dirs=sphere_dirs(m, BASE_SEED + 41), name="cfg4_skew_%s" % wdtype)


def config5(width=1920, height=1080, azimuth=45.0, sigma_scale=100.0, wdtype="bf16", net_res=32, occ_res=512):
    """Large render: 32^3 networks of width 64, 512^3 occupancy grid (5 % occupied, 64 blobs),
    1920x1080 rays, step = diagonal / 1024."""
    return _render_config(net_res, occ_res, 64, wdtype, 64, 0.05, width, height, 1024, BASE_SEED + 5, azimuth,
                          sigma_scale, "cfg5_large_%s" % wdtype)


def sparsify(scene, present, seed):
    """Turn a dense scene dict into a sparse one: the cells flagged in ``present`` keep their network, the networks
    are stored in shuffled order, ``cell_net`` maps cell -> row of ``weights`` (-1: no network)."""
    present = np.asarray(present, bool).reshape(-1)
    n = int(present.sum())
    table = np.full(present.size, -1, np.int32)
    table[present] = np.random.default_rng(seed).permutation(n).astype(np.int32)
    w = np.empty((n, scene["weights"].shape[1]), np.float32)
    w[table[present]] = scene["weights"][present]
    out = dict(scene)
    out["weights"] = w
    out["cell_net"] = table
    return out


def config_sparse(width=800, height=800, azimuth=45.0, sigma_scale=100.0, wdtype="f16", net_res=48, occ_res=192,
                  hidden=32, frac=0.04):
    """A finer network grid than a dense scene could hold (48^3 = 110,592 cells), with networks only in the cells
    that contain occupied voxels (the sparse instantiation Sec. 5 proposes); camera and lattice as config 3."""
    occ = blob_occupancy((occ_res,) * 3, 32, frac, BASE_SEED + 67)
    f = occ_res // net_res
    assert f * net_res == occ_res
    present = occ.reshape(net_res, f, net_res, f, net_res, f).any(axis=(1, 3, 5)).reshape(-1)
    n = int(present.sum())
    table = np.full(present.size, -1, np.int32)
    table[present] = np.random.default_rng(BASE_SEED + 68).permutation(n).astype(np.int32)
    w = round_to_storage(kaiming_weights(n, hidden, BASE_SEED + 6, sigma_scale=sigma_scale), wdtype)
    sc = dict(res=(net_res,) * 3, aabb_min=(-1.0, -1.0, -1.0), aabb_max=(1.0, 1.0, 1.0), hidden=hidden, wdtype=wdtype,
              weights=w, occupancy=occ, L_pos=10, L_dir=4, cell_net=table)
    o, d = camera_rays(width, height, 40.0, 4.0, azimuth, 30.0)
    diag = 2.0 * math.sqrt(3.0)
    return dict(scene=sc, rays_o=o, rays_d=d, t_near=4.0 - math.sqrt(3.0), step=diag / 512, K=512, term_eps=0.01,
                bg=(1.0, 1.0, 1.0), width=width, height=height, name="sparse_render_%s" % wdtype)
