"""The C-ABI library loads, exports every symbol the public header declares, and rejects bad
arguments on the host (no GPU needed: nothing here launches a kernel)."""
import ctypes as C
import os
import re

import pytest

import paper_2103_13744_amd as kn

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return kn.load_library()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "kilonerf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kn_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(kn.EXPORTS) == names


def test_params_per_net_and_error_strings(lib):
    assert lib.kn_params_per_net(32, 10, 4) == 6212          # the paper's "6k parameters" (Sec. 4.3)
    assert lib.kn_params_per_net(64, 10, 4) == 18564
    assert lib.kn_params_per_net(0, 10, 4) == -1
    assert lib.kn_error_string(0) == b"ok"
    for code in (-1, -2, -3, -4, -5, -6):
        assert lib.kn_error_string(code) not in (b"ok", b"unknown status")
    assert lib.kn_error_string(-99) == b"unknown status"


def test_host_side_argument_validation(lib):
    h = C.c_void_p()
    n = C.c_int64()
    fake_ctx = 256                                                      # never dereferenced: the descriptor is checked first
    assert lib.kn_scene_create(None, None, None, None, 0, C.byref(h)) == -1
    assert lib.kn_scene_create(fake_ctx, None, None, None, 0, C.byref(h)) == -1
    d = kn.SceneDesc()
    assert lib.kn_scene_create(fake_ctx, C.byref(d), None, None, 0, None) == -1
    assert lib.kn_scene_bytes(None, C.byref(n)) == -1 and lib.kn_scene_bytes(C.byref(d), None) == -1

    def check(desc):            # the descriptor checks are the same in both calls
        rc = lib.kn_scene_bytes(C.byref(desc), C.byref(n))
        assert rc != 0 and lib.kn_scene_create(fake_ctx, C.byref(desc), None, None, 0, C.byref(h)) == rc
        return rc

    d.res[:] = [2, 2, 2]
    d.aabb_min[:] = [0, 0, 0]
    d.aabb_max[:] = [1, 1, 1]
    d.hidden, d.L_pos, d.L_dir, d.wdtype = 32, 10, 4, 0
    d.weights = None
    assert check(d) == -1       # no weights
    d.weights = 256                                                     # never dereferenced below
    d.aabb_max[:] = [1, 0, 1]
    assert check(d) == -1       # empty box
    d.aabb_max[:] = [1, 1, 1]
    d.res[:] = [0, 2, 2]
    assert check(d) == -1       # zero grid component
    d.res[:] = [64, 64, 64]
    assert check(d) == -2       # too many networks
    d.cell_net, d.n_nets = 256, 0                                       # sparse grid (table never dereferenced below)
    assert check(d) == -1       # no networks behind the table
    d.n_nets = 70000
    assert check(d) == -2       # too many networks
    d.res[:] = [300, 300, 300]
    d.n_nets = 100
    assert check(d) == -2       # too many cells
    d.cell_net, d.n_nets = None, 0
    d.res[:] = [2, 2, 2]
    d.hidden = 48
    assert check(d) == -2       # no kernel for this width
    d.hidden, d.wdtype = 32, 7
    assert check(d) == -1       # bad dtype
    d.wdtype = 0
    d.occ_res[:] = [4, 4, 4]
    d.occupancy = None
    assert check(d) == -1       # grid announced, not given
    # a valid descriptor: the size of the scene's device data, without a device
    d.occupancy = 256
    d.occ_res[:] = [64, 64, 64]
    assert lib.kn_scene_bytes(C.byref(d), C.byref(n)) == 0
    f32_small = n.value
    assert f32_small >= 8 * 124 * 64 * 4 + 64 ** 3 // 8 + 2 * 16 ** 3      # weight image, occupancy bits, skip field twice
    d.wdtype, d.res[:] = 1, [16, 16, 16]
    assert lib.kn_scene_bytes(C.byref(d), C.byref(n)) == 0 and n.value >= 4096 * (12 * 1024 + 36 * 4)
    out = C.c_int64()
    assert lib.kn_create(None, 0) == -1
    assert lib.kn_destroy(None) == 0
    assert lib.kn_workspace_bytes(None, None, 10, 10, C.byref(out)) == -1
    assert lib.kn_cell_ids(None, None, None, 0, None) == -1
    assert lib.kn_render(None, None, None, None, None, 0, 0.0, 1.0, 8, 0.0, None, None, None, None, 0) == -1
    bg = (C.c_float * 3)(0, 0, 0)
    assert lib.kn_render_stratified(None, None, None, None, None, 0, 0.0, 1.0, 8, 0.0, C.byref(bg), 1, None, None, None, 0) == -1
    assert lib.kn_march_stratified(None, None, None, None, 0, 0.0, 1.0, 8, 1, None, 4, None, None, None) == -1
    assert lib.kn_composite(None, None, None, None, -1, 0.1, 0.0, C.byref(bg), None, None, None) == -1
    assert lib.kn_composite(None, None, None, None, 0, 0.0, 0.0, C.byref(bg), None, None, None) == -1   # step <= 0
    assert lib.kn_composite(None, None, None, None, 0, 0.1, 1.5, C.byref(bg), None, None, None) == -1   # eps >= 1
    assert lib.kn_composite(None, None, None, None, 0, 0.1, 0.01, C.byref(bg), None, None, None) == 0   # R = 0: no-op
    assert lib.kn_composite_deltas(None, None, None, None, None, -1, 0.0, C.byref(bg), None, None, None) == -1
    assert lib.kn_composite_deltas(None, None, None, None, None, 0, 1.5, C.byref(bg), None, None, None) == -1   # eps >= 1
    assert lib.kn_composite_deltas(None, None, None, None, None, 0, 0.0, C.byref(bg), None, None, None) == 0    # R = 0
    assert lib.kn_set_render_params(None, 0, 0, 0) == -1
    assert lib.kn_set_option(None, 1, 0) == -1
    assert lib.kn_profile_enable(None, 1) == -1
    assert lib.kn_profile_read(None, None, 0) == -1
    res = (C.c_int32 * 3)(4, 4, 4)
    assert lib.kn_extract_occupancy(None, None, None, C.byref(res), 1.0, None, None, 0) == -1
    assert lib.kn_extract_workspace_bytes(None, C.byref(out)) == -1
    assert lib.kn_layered_workspace_bytes(None, 10, C.byref(out)) == -1
    assert lib.kn_eval_grouped_layered(None, None, None, None, None, 0, None, None, None, 0) == -1
    assert lib.kn_eval_grouped(None, None, None, None, None, 0, None, None, None, None, None, None, 0) == -1
    assert lib.kn_eval_grouped_static(None, None, None, None, None, 0, None, None, None, None, None) == -1
    assert lib.kn_bucket(None, None, None, None, 0, None, None, None, None, 0) == -1


def test_a_context_needs_a_gfx950_device():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a device is present: contexts are covered by the GPU tests")
    h = C.c_void_p()
    assert kn.load_library().kn_create(C.byref(h), 0) == -5 and not h.value
    with pytest.raises(kn.KnError, match="gfx950"):
        kn.Context(0)


def test_binding_checks_dtypes_and_shapes_before_it_passes_pointers():
    """The library sees addresses only; the binding refuses tensors of the wrong type, shape or device."""
    import torch

    class Dev:                      # stands in for a device tensor: _ptr only looks at these attributes
        def __init__(self, shape, dtype, cuda=True, contiguous=True):
            self.shape, self.dtype, self.is_cuda, self._c = tuple(shape), dtype, cuda, contiguous

        def is_contiguous(self):
            return self._c

        def dim(self):
            return len(self.shape)

        def data_ptr(self):
            return 4096

    assert kn._ptr(Dev((5, 3), torch.float32), torch.float32, shape=(5, 3)) == 4096
    assert kn._ptr(Dev((5, 3), torch.float32), shape=(None, 3)) == 4096
    assert kn._ptr(None, allow_none=True) is None
    for bad, kw in ((Dev((5, 3), torch.float64), dict(dtype=torch.float32)),
                    (Dev((5, 4), torch.float32), dict(shape=(5, 3))),
                    (Dev((15,), torch.float32), dict(shape=(5, 3))),
                    (Dev((4, 3), torch.float32), dict(shape=(5, 3))),
                    (Dev((5, 3), torch.float32, cuda=False), {}),
                    (Dev((5, 3), torch.float32, contiguous=False), {}),
                    (None, {})):
        with pytest.raises(kn.KnError):
            kn._ptr(bad, **kw)


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(kn, "_lib", None)
    monkeypatch.setattr(kn, "LIB_PATH", "/nonexistent/libkilonerf_hip.so")
    with pytest.raises(kn.KnError):
        kn.load_library(build_if_missing=False)
