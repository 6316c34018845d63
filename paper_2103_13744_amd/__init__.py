"""Python binding of libkilonerf_hip.so: argument marshalling only.

Every step of the rendering path (cell assignment, bucketing, the grouped tiny MLPs, marching,
blending) runs in the HIP kernels behind the C ABI declared in ``include/kilonerf.h``; this
module turns torch device tensors into pointers, sizes and a stream handle and checks status
codes.  There is no CPU or PyTorch fallback: if the library is missing or a call fails, an
exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkilonerf_hip.so")

KN_F32, KN_F16, KN_BF16 = 0, 1, 2
DTYPES = {"f32": KN_F32, "f16": KN_F16, "bf16": KN_BF16}

EXPORTS = ["kn_error_string", "kn_last_hip_error", "kn_params_per_net", "kn_create", "kn_destroy", "kn_set_option",
           "kn_scene_bytes", "kn_scene_create", "kn_scene_destroy",
           "kn_extract_workspace_bytes", "kn_extract_occupancy", "kn_layered_workspace_bytes", "kn_eval_grouped_layered",
           "kn_workspace_bytes", "kn_cell_ids", "kn_bucket", "kn_eval_grouped", "kn_eval_grouped_static", "kn_march", "kn_composite",
           "kn_render", "kn_composite_deltas", "kn_march_stratified", "kn_render_stratified", "kn_set_render_params", "kn_profile_enable", "kn_profile_read"]


class KnError(RuntimeError):
    pass


class SceneDesc(C.Structure):
    _fields_ = [("res", C.c_int32 * 3), ("aabb_min", C.c_float * 3), ("aabb_max", C.c_float * 3),
                ("hidden", C.c_int32), ("L_pos", C.c_int32), ("L_dir", C.c_int32), ("wdtype", C.c_int32),
                ("weights", C.c_void_p), ("occ_res", C.c_int32 * 3), ("occupancy", C.c_void_p),
                ("cell_net", C.c_void_p), ("n_nets", C.c_int32)]


class RenderStats(C.Structure):
    _fields_ = [("rays", C.c_int64), ("waves", C.c_int64), ("samples_evaluated", C.c_int64),
                ("samples_blended", C.c_int64), ("slots", C.c_int64)]


class Profile(C.Structure):
    _fields_ = [("ms_cell", C.c_double), ("ms_march", C.c_double), ("ms_bucket", C.c_double), ("ms_mlp", C.c_double),
                ("ms_blend", C.c_double), ("mlp_launches", C.c_int64), ("mlp_samples", C.c_int64),
                ("bucket_keys", C.c_int64), ("calls", C.c_int64), ("ms_setup", C.c_double)]


_lib = None


def load_library(build_if_missing: bool = True):
    """dlopen the in-tree library (building it first only if it does not exist)."""
    global _lib
    if _lib is not None:
        return _lib
    # torch ships its own HIP runtime; it must be the one already loaded when the library is opened,
    # so that device pointers and streams created by torch are valid inside the library
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise KnError("libkilonerf_hip.so has not been built (run paper_2103_13744_amd/build.py)")
        from .build import build
        build(force=True)
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_float
    L.kn_error_string.restype = C.c_char_p
    L.kn_error_string.argtypes = [C.c_int]
    L.kn_last_hip_error.restype = C.c_int
    L.kn_params_per_net.restype = i64
    L.kn_params_per_net.argtypes = [i32, i32, i32]
    L.kn_create.argtypes = [C.POINTER(vp), C.c_int]
    L.kn_destroy.argtypes = [vp]
    L.kn_set_option.argtypes = [vp, i32, i64]
    L.kn_scene_bytes.argtypes = [C.POINTER(SceneDesc), C.POINTER(i64)]
    L.kn_scene_create.argtypes = [vp, C.POINTER(SceneDesc), vp, vp, i64, C.POINTER(vp)]
    L.kn_scene_destroy.argtypes = [vp]
    L.kn_workspace_bytes.argtypes = [vp, vp, i64, i64, C.POINTER(i64)]
    L.kn_cell_ids.argtypes = [vp, vp, vp, i64, vp]
    L.kn_bucket.argtypes = [vp, vp, vp, vp, i64, vp, vp, vp, vp, i64]
    L.kn_eval_grouped.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, i64]
    L.kn_eval_grouped_static.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp, vp, vp, vp]
    L.kn_march.argtypes = [vp, vp, vp, vp, i64, f32, f32, i32, vp, i32, vp, vp, vp]
    L.kn_extract_workspace_bytes.argtypes = [vp, C.POINTER(i64)]
    L.kn_layered_workspace_bytes.argtypes = [vp, i64, C.POINTER(i64)]
    L.kn_eval_grouped_layered.argtypes = [vp, vp, vp, vp, vp, i64, vp, vp, vp, i64]
    L.kn_extract_occupancy.argtypes = [vp, vp, vp, C.POINTER(i32 * 3), f32, vp, vp, i64]
    L.kn_composite.argtypes = [vp, vp, vp, vp, i64, f32, f32, C.POINTER(f32 * 3), vp, vp, vp]
    L.kn_composite_deltas.argtypes = [vp, vp, vp, vp, vp, i64, f32, C.POINTER(f32 * 3), vp, vp, vp]
    L.kn_render.argtypes = [vp, vp, vp, vp, vp, i64, f32, f32, i32, f32, C.POINTER(f32 * 3), vp,
                            C.POINTER(RenderStats), vp, i64]
    u32 = C.c_uint32
    L.kn_march_stratified.argtypes = [vp, vp, vp, vp, i64, f32, f32, i32, u32, vp, i32, vp, vp, vp]
    L.kn_render_stratified.argtypes = [vp, vp, vp, vp, vp, i64, f32, f32, i32, f32, C.POINTER(f32 * 3), u32, vp,
                                       C.POINTER(RenderStats), vp, i64]
    L.kn_set_render_params.argtypes = [vp, i32, i32, i32]
    L.kn_profile_enable.argtypes = [vp, C.c_int]
    L.kn_profile_read.argtypes = [vp, C.POINTER(Profile), C.c_int]
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        L = load_library()
        raise KnError("%s failed: %s (status %d, hip error %d)" %
                      (what, L.kn_error_string(rc).decode(), rc, L.kn_last_hip_error()))


def _ptr(t, dtype=None, allow_none=False, shape=None):
    """Device pointer of a contiguous device tensor; ``dtype`` and ``shape`` (None entries are free) are checked,
    because the library sees only the address: it cannot tell a float64 or short tensor from the one it expects."""
    if t is None:
        if allow_none:
            return None
        raise KnError("missing tensor argument")
    if not t.is_cuda or not t.is_contiguous():
        raise KnError("tensor arguments must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise KnError("expected dtype %s, got %s" % (dtype, t.dtype))
    if shape is not None:
        if t.dim() != len(shape) or any(w is not None and int(w) != int(h) for w, h in zip(shape, t.shape)):
            raise KnError("expected shape %s, got %s" % (tuple(shape), tuple(t.shape)))
    return t.data_ptr()


def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def params_per_net(hidden: int, L_pos: int = 10, L_dir: int = 4) -> int:
    return int(load_library().kn_params_per_net(hidden, L_pos, L_dir))


OPT_GROUP_FUSED_MAX, OPT_GROUP_HASH_SLOTS, OPT_PROFILE_EVERY = 1, 2, 3


class Context:
    """kn_ctx: the mutable state of the library on one device (wave schedule, timing, mailboxes)."""

    def __init__(self, device: int = 0):
        self.L = load_library()
        h = C.c_void_p()
        _check(self.L.kn_create(C.byref(h), int(device)), "kn_create")
        self.h = h
        self.device = int(device)

    def close(self):
        if getattr(self, "h", None):
            self.L.kn_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_render_params(self, first_wave_samples: int = 0, slots_per_ray: int = 0, wave_growth: int = 0):
        _check(self.L.kn_set_render_params(self.h, first_wave_samples, slots_per_ray, wave_growth), "kn_set_render_params")

    def set_option(self, option: int, value: int):
        _check(self.L.kn_set_option(self.h, int(option), int(value)), "kn_set_option")

    def profile_enable(self, on):
        """False / 0: off; True / 1: every stage; 2: only the grouped-MLP kernel; 3: only the marching kernel."""
        _check(self.L.kn_profile_enable(self.h, int(on)), "kn_profile_enable")

    def profile_read(self, reset: bool = True) -> dict:
        p = Profile()
        _check(self.L.kn_profile_read(self.h, C.byref(p), 1 if reset else 0), "kn_profile_read")
        return {k: getattr(p, k) for k, _ in Profile._fields_}


_default_ctx = {}


def default_context(device=None) -> Context:
    """One shared context per device, created on first use (scenes and the module-level helpers use it unless told otherwise)."""
    import torch
    dev = torch.cuda.current_device() if device is None else int(device)
    if dev not in _default_ctx:
        _default_ctx[dev] = Context(dev)
    return _default_ctx[dev]


def set_render_params(first_wave_samples: int = 0, slots_per_ray: int = 0, wave_growth: int = 0):
    default_context().set_render_params(first_wave_samples, slots_per_ray, wave_growth)


def profile_enable(on):
    default_context().profile_enable(on)


def profile_read(reset: bool = True) -> dict:
    return default_context().profile_read(reset)


class Scene:
    """Device-resident KiloNeRF scene.  ``weights``: device tensor (N, P) of float32 / float16 /
    bfloat16 in the canonical layout; ``occupancy``: device uint8 tensor (ox, oy, oz) or None; ``cell_net``: None, or
    for a sparse grid a device int32 tensor with one entry per cell (network index, -1 = no network); N is then the
    number of rows of ``weights``.  ``ctx``: the context the scene is created and, by default, used through (the shared
    default context of the device if None); every method that runs kernels takes ``ctx=`` to go through another one.
    ``lend_buffer``: the scene's device data lives in a torch tensor this object owns (kn_scene_bytes, buffer
    argument of kn_scene_create) instead of memory the library allocates."""

    def __init__(self, res, aabb_min, aabb_max, hidden, weights, occupancy=None, L_pos=10, L_dir=4, cell_net=None, ctx=None,
                 lend_buffer=True):
        import torch
        self.L = load_library()
        self.ctx = default_context(weights.device.index) if ctx is None else ctx
        wd = {torch.float32: KN_F32, torch.float16: KN_F16, torch.bfloat16: KN_BF16}.get(weights.dtype)
        if wd is None:
            raise KnError("unsupported weight dtype %s" % weights.dtype)
        d = SceneDesc()
        d.res[:] = [int(v) for v in res]
        d.aabb_min[:] = [float(v) for v in aabb_min]
        d.aabb_max[:] = [float(v) for v in aabb_max]
        d.hidden, d.L_pos, d.L_dir, d.wdtype = int(hidden), int(L_pos), int(L_dir), wd
        self.N = int(res[0]) * int(res[1]) * int(res[2])
        n_rows = self.N if cell_net is None else int(weights.shape[0])
        P = int(self.L.kn_params_per_net(int(hidden), int(L_pos), int(L_dir)))
        d.weights = _ptr(weights, shape=(n_rows, P) if P > 0 else None)
        if occupancy is None:
            d.occ_res[:] = [0, 0, 0]
            d.occupancy = None
        else:
            d.occ_res[:] = list(occupancy.shape)
            d.occupancy = _ptr(occupancy, torch.uint8, shape=(None, None, None))
        if cell_net is not None:
            if cell_net.numel() != self.N:
                raise KnError("cell_net must have one entry per cell")
            d.cell_net = _ptr(cell_net, torch.int32)
            d.n_nets = self.N = n_rows
        self.hidden = int(hidden)
        self.device = weights.device
        self._buffer = None
        if lend_buffer:
            need = C.c_int64()
            _check(self.L.kn_scene_bytes(C.byref(d), C.byref(need)), "kn_scene_bytes")
            self._buffer = torch.empty(int(need.value), dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        _check(self.L.kn_scene_create(self.ctx.h, C.byref(d), _stream(), _ptr(self._buffer, allow_none=True),
                                      0 if self._buffer is None else self._buffer.numel(), C.byref(h)), "kn_scene_create")
        self.h = h
        self._ws = None

    def close(self):
        if getattr(self, "h", None):
            self.L.kn_scene_destroy(self.h)
            self.h = None
            self._buffer = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _ctx(self, ctx):
        return (self.ctx if ctx is None else ctx).h

    # -- workspace -----------------------------------------------------------------------
    def workspace_bytes(self, max_points=0, max_rays=0, ctx=None) -> int:
        out = C.c_int64()
        _check(self.L.kn_workspace_bytes(self._ctx(ctx), self.h, int(max_points), int(max_rays), C.byref(out)), "kn_workspace_bytes")
        return out.value

    def _workspace(self, max_points=0, max_rays=0, ctx=None):
        import torch
        need = self.workspace_bytes(max_points, max_rays, ctx)
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    # -- stages --------------------------------------------------------------------------
    def cell_ids(self, points):
        import torch
        M = points.shape[0]
        ids = torch.empty(M, dtype=torch.int32, device=self.device)
        _check(self.L.kn_cell_ids(self.h, _stream(), _ptr(points, torch.float32, shape=(M, 3)) if M else None, M,
                                  _ptr(ids) if M else None), "kn_cell_ids")
        return ids

    def bucket(self, ids, ctx=None):
        import torch
        M = ids.shape[0]
        counts = torch.empty(self.N + 1, dtype=torch.int32, device=self.device)
        offsets = torch.empty(self.N + 2, dtype=torch.int32, device=self.device)
        perm = torch.empty(M, dtype=torch.int32, device=self.device)
        ws = self._workspace(max_points=max(M, 1), ctx=ctx)
        _check(self.L.kn_bucket(self._ctx(ctx), self.h, _stream(), _ptr(ids, torch.int32, shape=(M,)) if M else None, M,
                                _ptr(counts), _ptr(offsets), _ptr(perm) if M else None, _ptr(ws), ws.numel()), "kn_bucket")
        return counts, offsets, perm

    def _eval_args(self, points, dirs, out, aux):
        """Checked pointers of an eval_grouped call: points, dirs (M, 3) float32; out = (sigma (M,), rgb (M, 3)) float32;
        aux = None or (ids (M,), counts (N + 1,), perm (M,)) int32."""
        import torch
        M = points.shape[0]
        sigma, rgb = out
        ids, counts, perm = aux if aux is not None else (None, None, None)
        f, i = torch.float32, torch.int32
        if M == 0:
            return 0, (None, None), (None, None), (None, _ptr(counts, i, allow_none=True, shape=(self.N + 1,)), None)
        return M, (_ptr(points, f, shape=(M, 3)), _ptr(dirs, f, shape=(M, 3))), \
            (_ptr(sigma, f, shape=(M,)), _ptr(rgb, f, shape=(M, 3))), \
            (_ptr(ids, i, allow_none=True, shape=(M,)), _ptr(counts, i, allow_none=True, shape=(self.N + 1,)),
             _ptr(perm, i, allow_none=True, shape=(M,)))

    def eval_grouped(self, points, dirs, want_aux=False, out=None, ctx=None):
        import torch
        M = points.shape[0]
        if out is None:
            out = (torch.empty(M, dtype=torch.float32, device=self.device),
                   torch.empty((M, 3), dtype=torch.float32, device=self.device))
        aux = None
        if want_aux:
            aux = (torch.empty(M, dtype=torch.int32, device=self.device),
                   torch.empty(self.N + 1, dtype=torch.int32, device=self.device),
                   torch.empty(M, dtype=torch.int32, device=self.device))
        ws = self._workspace(max_points=max(M, 1), ctx=ctx)
        M, pin, pout, paux = self._eval_args(points, dirs, out, aux)
        _check(self.L.kn_eval_grouped(self._ctx(ctx), self.h, _stream(), *pin, M, *pout, *paux, _ptr(ws), ws.numel()),
               "kn_eval_grouped")
        if want_aux:
            return (*out, *aux)
        return out

    def eval_grouped_static(self, points, dirs, out, aux=None, ctx=None):
        """kn_eval_grouped_static: eval_grouped on the library's static scratch array (nothing is allocated, so
        ``out`` = (sigma, rgb) is required; ``aux`` = (ids, counts, perm) optional outputs)."""
        M, pin, pout, paux = self._eval_args(points, dirs, out, aux)
        _check(self.L.kn_eval_grouped_static(self._ctx(ctx), self.h, _stream(), *pin, M, *pout, *paux), "kn_eval_grouped_static")
        return out

    def eval_grouped_layered(self, points, dirs, out=None, workspace=None, ctx=None):
        """eval_grouped one layer at a time (grouped matrix products with activations in device memory): the
        comparison point for the fused kernel.  16-bit scenes only."""
        import torch
        M = points.shape[0]
        if out is None:
            out = (torch.empty(M, dtype=torch.float32, device=self.device),
                   torch.empty((M, 3), dtype=torch.float32, device=self.device))
        if workspace is None:
            need = C.c_int64()
            _check(self.L.kn_layered_workspace_bytes(self.h, max(M, 1), C.byref(need)), "kn_layered_workspace_bytes")
            workspace = torch.empty(int(need.value), dtype=torch.uint8, device=self.device)
        M, pin, pout, _ = self._eval_args(points, dirs, out, None)
        _check(self.L.kn_eval_grouped_layered(self._ctx(ctx), self.h, _stream(), *pin, M, *pout, _ptr(workspace),
                                              workspace.numel()), "kn_eval_grouped_layered")
        return out

    def extract_occupancy(self, occ_res, tau, out=None, ctx=None):
        """Occupancy grid of resolution ``occ_res`` from the scene's own density field (27 probes per voxel,
        marked where any density is above ``tau``): a uint8 device tensor of shape ``occ_res``."""
        import torch
        res = tuple(int(r) for r in occ_res)
        occ = torch.empty(res, dtype=torch.uint8, device=self.device) if out is None else out
        need = C.c_int64()
        _check(self.L.kn_extract_workspace_bytes(self.h, C.byref(need)), "kn_extract_workspace_bytes")
        ws = torch.empty(int(need.value), dtype=torch.uint8, device=self.device)
        _check(self.L.kn_extract_occupancy(self._ctx(ctx), self.h, _stream(), C.byref((C.c_int32 * 3)(*res)), float(tau),
                                           _ptr(occ, torch.uint8, shape=res), _ptr(ws), ws.numel()), "kn_extract_occupancy")
        return occ

    def march(self, rays_o, rays_d, t_near, step, K, S=None, k_begin=None, seed=None):
        """``seed`` None: midpoint lattice (kn_march); else stratified sampling (kn_march_stratified)."""
        import torch
        R = rays_o.shape[0]
        S = int(K if S is None else S)
        out_k = torch.empty((R, S), dtype=torch.int32, device=self.device)
        cnt = torch.empty(R, dtype=torch.int32, device=self.device)
        nxt = torch.empty(R, dtype=torch.int32, device=self.device)
        head = (self.h, _stream(), _ptr(rays_o, torch.float32, shape=(R, 3)), _ptr(rays_d, torch.float32, shape=(R, 3)), R,
                float(t_near), float(step), int(K))
        tail = (_ptr(k_begin, torch.int32, allow_none=True, shape=(R,)), S, _ptr(out_k), _ptr(cnt), _ptr(nxt))
        if seed is None:
            _check(self.L.kn_march(*head, *tail), "kn_march")
        else:
            _check(self.L.kn_march_stratified(*head, int(seed), *tail), "kn_march_stratified")
        return out_k, cnt, nxt

    def render(self, rays_o, rays_d, t_near, step, K, term_eps=0.0, bg=(0.0, 0.0, 0.0), want_stats=False, out=None,
               workspace=None, seed=None, ctx=None):
        """``seed`` None: midpoint lattice (kn_render); else stratified sampling (kn_render_stratified).  ``workspace``: a uint8 device tensor of at least ``workspace_bytes(max_rays=R)`` bytes; by default one
        cached workspace per scene is used.  Calls that are in flight at the same time (on different streams) need
        a workspace each."""
        import torch
        R = rays_o.shape[0]
        rgb = torch.empty((R, 3), dtype=torch.float32, device=self.device) if out is None else out
        ws = self._workspace(max_rays=max(R, 1), ctx=ctx) if workspace is None else workspace
        st = RenderStats()
        bgc = (C.c_float * 3)(*[float(v) for v in bg])
        f = torch.float32
        head = (self._ctx(ctx), self.h, _stream(), _ptr(rays_o, f, shape=(R, 3)) if R else None,
                _ptr(rays_d, f, shape=(R, 3)) if R else None, R, float(t_near), float(step), int(K), float(term_eps), C.byref(bgc))
        tail = (_ptr(rgb, f, shape=(R, 3)) if R else None, C.byref(st) if want_stats else None, _ptr(ws, torch.uint8), ws.numel())
        if seed is None:
            _check(self.L.kn_render(*head, *tail), "kn_render")
        else:
            _check(self.L.kn_render_stratified(*head, int(seed), *tail), "kn_render_stratified")
        if want_stats:
            return rgb, {k: getattr(st, k) for k, _ in RenderStats._fields_}
        return rgb


def composite(sigma, rgb, offsets, step, term_eps=0.0, bg=(0.0, 0.0, 0.0)):
    """``step``: the constant sample spacing (kn_composite), or a float32 device tensor with a spacing per sample
    (kn_composite_deltas)."""
    import torch
    L = load_library()
    R = offsets.shape[0] - 1
    out = torch.empty((R, 3), dtype=torch.float32, device=offsets.device)
    T = torch.empty(R, dtype=torch.float32, device=offsets.device)
    used = torch.empty(R, dtype=torch.int32, device=offsets.device)
    bgc = (C.c_float * 3)(*[float(v) for v in bg])
    n = sigma.shape[0]
    if torch.is_tensor(step):
        if step.shape[0] != n:
            raise KnError("one delta per sample expected")
        _check(L.kn_composite_deltas(_stream(), _ptr(sigma, torch.float32) if n else None,
                                     _ptr(rgb, torch.float32) if n else None, _ptr(step, torch.float32) if n else None,
                                     _ptr(offsets, torch.int32), R, float(term_eps), C.byref(bgc), _ptr(out), _ptr(T),
                                     _ptr(used)), "kn_composite_deltas")
        return out, T, used
    _check(L.kn_composite(_stream(), _ptr(sigma, torch.float32) if n else None, _ptr(rgb, torch.float32) if n else None,
                          _ptr(offsets, torch.int32), R, float(step), float(term_eps), C.byref(bgc), _ptr(out), _ptr(T),
                          _ptr(used)), "kn_composite")
    return out, T, used
