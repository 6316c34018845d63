"""ctypes binding of the CPU oracle (TEST INFRASTRUCTURE, not part of the product path).

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` import
this package.  It compiles ``kn_oracle.c`` with gcc into two shared objects next to the source:
``libkn_oracle.so`` (one thread: the definition) and ``libkn_oracle_omp.so`` (same source with
OpenMP over independent rays / points, used only to time the oracle on all host cores).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kn_oracle.c")
_LIBS = {False: os.path.join(_HERE, "libkn_oracle.so"), True: os.path.join(_HERE, "libkn_oracle_omp.so")}
_CFLAGS = ["-O2", "-ffp-contract=off", "-fPIC", "-shared", "-std=c99", "-Wall", "-Wextra"]


def build(force: bool = False) -> None:
    """Compile both oracle libraries (skipped when up to date unless ``force``)."""
    for omp, out in _LIBS.items():
        fresh = os.path.exists(out) and os.path.getmtime(out) >= max(
            os.path.getmtime(_SRC), os.path.getmtime(os.path.join(_HERE, "kn_oracle.h")))
        if fresh and not force:
            continue
        cmd = ["gcc", *_CFLAGS, *(["-fopenmp"] if omp else []), _SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


class Scene(C.Structure):
    _fields_ = [("res", C.c_int32 * 3), ("aabb_min", C.c_float * 3), ("aabb_max", C.c_float * 3),
                ("hidden", C.c_int32), ("L_pos", C.c_int32), ("L_dir", C.c_int32),
                ("weights", C.c_void_p), ("occ_res", C.c_int32 * 3), ("occupancy", C.c_void_p),
                ("cell_net", C.c_void_p), ("n_nets", C.c_int32)]


_f32p = np.ctypeslib.ndpointer(np.float32, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(np.float64, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_loaded = {}


def _lib(omp: bool = False):
    if omp not in _loaded:
        # KN_ORACLE_LIB: load this shared object instead (the mutation test points the pins at deliberately broken
        # builds of the oracle to show that they notice)
        override = os.environ.get("KN_ORACLE_LIB")
        if not override:
            build()
        L = C.CDLL(override or _LIBS[omp])
        L.kno_params_per_net.restype = C.c_int64
        L.kno_params_per_net.argtypes = [C.c_int32] * 3
        L.kno_posenc.restype = None
        L.kno_posenc.argtypes = [_f32p, C.c_int32, _f64p]
        L.kno_grid_index.restype = C.c_int32
        L.kno_grid_index.argtypes = [_f32p, _f32p, _i32p, _f32p]
        L.kno_cell_ids.argtypes = [C.POINTER(Scene), _f32p, C.c_int64, _i32p]
        L.kno_bucket.argtypes = [_i32p, C.c_int64, C.c_int32, _i32p, _i32p, _i32p]
        L.kno_mlp.argtypes = [C.POINTER(Scene), C.c_int32, _f32p, _f32p, _f64p, _f64p]
        L.kno_eval_points.argtypes = [C.POINTER(Scene), _f32p, _f32p, C.c_int64, _f64p, _f64p, C.c_void_p]
        L.kno_march.restype = C.c_int32
        L.kno_march.argtypes = [C.POINTER(Scene), _f32p, _f32p, C.c_float, C.c_float, C.c_int32, _i32p]
        L.kno_stratified_offset.restype = C.c_float
        L.kno_stratified_offset.argtypes = [C.c_uint32, C.c_uint32, C.c_int32]
        L.kno_march_stratified.restype = C.c_int32
        L.kno_march_stratified.argtypes = [C.POINTER(Scene), _f32p, _f32p, C.c_float, C.c_float, C.c_int32,
                                           C.c_uint32, C.c_uint32, _i32p]
        L.kno_render_stratified.argtypes = [C.POINTER(Scene), _f32p, _f32p, C.c_int64, C.c_float, C.c_float,
                                            C.c_int32, C.c_float, _f32p, C.c_uint32, C.c_void_p, _f64p, C.c_void_p,
                                            C.c_void_p, C.c_void_p]
        L.kno_composite.restype = C.c_int32
        L.kno_composite.argtypes = [_f64p, _f64p, C.c_int32, C.c_double, C.c_double, _f64p, _f64p,
                                    C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.kno_composite_deltas.restype = C.c_int32
        L.kno_composite_deltas.argtypes = [_f64p, _f64p, _f64p, C.c_int32, C.c_double, _f64p, _f64p,
                                           C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.kno_render.argtypes = [C.POINTER(Scene), _f32p, _f32p, C.c_int64, C.c_float, C.c_float,
                                 C.c_int32, C.c_float, _f32p, _f64p, C.c_void_p, C.c_void_p, C.c_void_p]
        _u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")
        _i64p = np.ctypeslib.ndpointer(np.int64, flags="C_CONTIGUOUS")
        L.kno_extract_occupancy_at.argtypes = [C.POINTER(Scene), _i32p, C.c_float, _i64p, C.c_int64, _u8p, _f64p, _f64p]
        L.kno_extract_occupancy.argtypes = [C.POINTER(Scene), _i32p, C.c_float, _u8p, _f64p, _f64p]
        L.kno_num_threads.restype = C.c_int
        _loaded[omp] = L
    return _loaded[omp]


def params_per_net(hidden: int, L_pos: int = 10, L_dir: int = 4) -> int:
    return int(_lib().kno_params_per_net(hidden, L_pos, L_dir))


class OracleScene:
    """Host-side scene for the oracle.  ``weights``: (N, P) float32 in the canonical layout
    (values already rounded to the storage type under test); ``occupancy``: uint8 (ox, oy, oz) or None;
    ``cell_net``: None, or for a sparse grid an int32 array with one entry per cell (network index, or -1
    for a cell without a network); N is then the number of rows of ``weights``."""

    def __init__(self, res, aabb_min, aabb_max, hidden, weights, occupancy=None, L_pos=10, L_dir=4,
                 threads: bool = False, cell_net=None):
        self.omp = bool(threads)
        self.L = _lib(self.omp)
        self.res = tuple(int(v) for v in res)
        self.cells = self.res[0] * self.res[1] * self.res[2]
        self.cell_net = None if cell_net is None else np.ascontiguousarray(cell_net, dtype=np.int32).reshape(-1)
        if self.cell_net is not None:
            assert self.cell_net.size == self.cells
        self.N = self.cells if self.cell_net is None else int(np.asarray(weights).shape[0])
        self.hidden, self.L_pos, self.L_dir = int(hidden), int(L_pos), int(L_dir)
        self.P = params_per_net(hidden, L_pos, L_dir)
        self.weights = np.ascontiguousarray(weights, dtype=np.float32).reshape(self.N, self.P)
        self.occupancy = None if occupancy is None else np.ascontiguousarray(occupancy, dtype=np.uint8)
        s = Scene()
        s.res[:] = self.res
        s.aabb_min[:] = [float(v) for v in aabb_min]
        s.aabb_max[:] = [float(v) for v in aabb_max]
        s.hidden, s.L_pos, s.L_dir = self.hidden, self.L_pos, self.L_dir
        s.weights = self.weights.ctypes.data
        if self.occupancy is None:
            s.occ_res[:] = [0, 0, 0]
            s.occupancy = None
        else:
            assert self.occupancy.ndim == 3
            s.occ_res[:] = list(self.occupancy.shape)
            s.occupancy = self.occupancy.ctypes.data
        s.cell_net = None if self.cell_net is None else self.cell_net.ctypes.data
        s.n_nets = 0 if self.cell_net is None else self.N
        self.c = s
        self.aabb_min = np.array(aabb_min, np.float32)
        self.aabb_max = np.array(aabb_max, np.float32)

    # -- steps ---------------------------------------------------------------------------
    def cell_ids(self, points):
        points = np.ascontiguousarray(points, np.float32).reshape(-1, 3)
        ids = np.empty(len(points), np.int32)
        assert self.L.kno_cell_ids(C.byref(self.c), points, len(points), ids) == 0
        return ids

    def grid_index(self, x, res=None):
        res = np.array(self.res if res is None else res, np.int32)
        return int(self.L.kno_grid_index(self.aabb_min, self.aabb_max, res, np.asarray(x, np.float32)))

    def mlp(self, n, x, d):
        sg = np.zeros(1)
        rgb = np.zeros(3)
        assert self.L.kno_mlp(C.byref(self.c), int(n), np.asarray(x, np.float32), np.asarray(d, np.float32), sg, rgb) == 0
        return float(sg[0]), rgb

    def eval_points(self, points, dirs):
        points = np.ascontiguousarray(points, np.float32).reshape(-1, 3)
        dirs = np.ascontiguousarray(dirs, np.float32).reshape(-1, 3)
        M = len(points)
        sg, rgb, ids = np.empty(M), np.empty((M, 3)), np.empty(M, np.int32)
        assert self.L.kno_eval_points(C.byref(self.c), points, dirs, M, sg, rgb, ids.ctypes.data) == 0
        return sg, rgb, ids

    def march(self, o, d, t_near, step, K):
        ks = np.empty(max(K, 1), np.int32)
        n = self.L.kno_march(C.byref(self.c), np.asarray(o, np.float32), np.asarray(d, np.float32),
                             float(t_near), float(step), int(K), ks)
        return ks[:n].copy()

    def march_stratified(self, o, d, t_near, step, K, seed, ray):
        ks = np.empty(max(K, 1), np.int32)
        n = self.L.kno_march_stratified(C.byref(self.c), np.asarray(o, np.float32), np.asarray(d, np.float32),
                                        float(t_near), float(step), int(K), int(seed), int(ray), ks)
        return ks[:n].copy()

    def render(self, rays_o, rays_d, t_near, step, K, term_eps=0.0, bg=(0.0, 0.0, 0.0), seed=None, ray_ids=None):
        """``seed`` None: midpoint lattice; else stratified sampling with that seed; ray number = row, or
        ``ray_ids[row]`` when the rays are a subset of a frame."""
        rays_o = np.ascontiguousarray(rays_o, np.float32).reshape(-1, 3)
        rays_d = np.ascontiguousarray(rays_d, np.float32).reshape(-1, 3)
        R = len(rays_o)
        rgb, n_eval, T, mg = np.empty((R, 3)), np.empty(R, np.int32), np.empty(R), np.empty(R)
        ids = None if ray_ids is None else np.ascontiguousarray(ray_ids, np.uint32)
        assert ids is None or len(ids) == R
        if seed is None:
            rc = self.L.kno_render(C.byref(self.c), rays_o, rays_d, R, float(t_near), float(step), int(K),
                                   float(term_eps), np.asarray(bg, np.float32), rgb, n_eval.ctypes.data,
                                   T.ctypes.data, mg.ctypes.data)
        else:
            rc = self.L.kno_render_stratified(C.byref(self.c), rays_o, rays_d, R, float(t_near), float(step), int(K),
                                              float(term_eps), np.asarray(bg, np.float32), int(seed),
                                              None if ids is None else ids.ctypes.data, rgb,
                                              n_eval.ctypes.data, T.ctypes.data, mg.ctypes.data)
        assert rc == 0
        return rgb, n_eval, T, mg

    def extract_occupancy(self, occ_res, tau, voxels=None):
        """Sec. 3.4 occupancy extraction -> (occupancy bytes, largest probe density, margin to tau), for the
        whole grid (arrays of shape occ_res) or for the voxels given by linear index."""
        occ_res = np.asarray(occ_res, np.int32)
        if voxels is None:
            n = int(np.prod(occ_res.astype(np.int64)))
            occ, top, mg = np.empty(n, np.uint8), np.empty(n), np.empty(n)
            assert self.L.kno_extract_occupancy(C.byref(self.c), occ_res, float(tau), occ, top, mg) == 0
            shape = tuple(int(r) for r in occ_res)
            return occ.reshape(shape), top.reshape(shape), mg.reshape(shape)
        voxels = np.ascontiguousarray(voxels, np.int64)
        occ, top, mg = np.empty(len(voxels), np.uint8), np.empty(len(voxels)), np.empty(len(voxels))
        assert self.L.kno_extract_occupancy_at(C.byref(self.c), occ_res, float(tau), voxels, len(voxels), occ, top, mg) == 0
        return occ, top, mg

    def num_threads(self):
        return int(self.L.kno_num_threads())


def posenc(p, L):
    out = np.empty(3 + 6 * L)
    _lib().kno_posenc(np.asarray(p, np.float32), int(L), out)
    return out


def stratified_offset(seed, ray, k):
    return float(_lib().kno_stratified_offset(int(seed), int(ray), int(k)))


def bucket(ids, N):
    ids = np.ascontiguousarray(ids, np.int32)
    counts, offsets, perm = np.empty(N + 1, np.int32), np.empty(N + 2, np.int32), np.empty(len(ids), np.int32)
    assert _lib().kno_bucket(ids, len(ids), int(N), counts, offsets, perm) == 0
    return counts, offsets, perm


def composite(sigma, rgb, step, eps=0.0, bg=(0.0, 0.0, 0.0)):
    """``step``: the constant delta, or an array with a delta per sample."""
    sigma = np.ascontiguousarray(sigma, np.float64)
    rgb = np.ascontiguousarray(rgb, np.float64).reshape(-1, 3)
    out = np.empty(3)
    T, mg = C.c_double(), C.c_double()
    if np.ndim(step) == 0:
        used = _lib().kno_composite(sigma, rgb, len(sigma), float(step), float(eps),
                                    np.asarray(bg, np.float64), out, C.byref(T), C.byref(mg))
    else:
        delta = np.ascontiguousarray(step, np.float64)
        assert len(delta) == len(sigma)
        used = _lib().kno_composite_deltas(sigma, rgb, delta, len(sigma), float(eps), np.asarray(bg, np.float64), out,
                                           C.byref(T), C.byref(mg))
    return out, T.value, int(used), mg.value
