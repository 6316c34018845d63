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
    for code in (-1, -2, -3, -4, -5):
        assert lib.kn_error_string(code) not in (b"ok", b"unknown status")
    assert lib.kn_error_string(-99) == b"unknown status"


def test_host_side_argument_validation(lib):
    h = C.c_void_p()
    assert lib.kn_scene_create(None, None, C.byref(h)) == -1
    d = kn.SceneDesc()
    assert lib.kn_scene_create(C.byref(d), None, None) == -1
    d.res[:] = [2, 2, 2]
    d.aabb_min[:] = [0, 0, 0]
    d.aabb_max[:] = [1, 1, 1]
    d.hidden, d.L_pos, d.L_dir, d.wdtype = 32, 10, 4, 0
    d.weights = None
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -1       # no weights
    d.weights = 256                                                     # never dereferenced below
    d.aabb_max[:] = [1, 0, 1]
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -1       # empty box
    d.aabb_max[:] = [1, 1, 1]
    d.res[:] = [0, 2, 2]
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -1       # zero grid component
    d.res[:] = [64, 64, 64]
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -2       # too many networks
    d.cell_net, d.n_nets = 256, 0                                       # sparse grid (table never dereferenced below)
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -1       # no networks behind the table
    d.n_nets = 70000
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -2       # too many networks
    d.res[:] = [300, 300, 300]
    d.n_nets = 100
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -2       # too many cells
    d.cell_net, d.n_nets = None, 0
    d.res[:] = [2, 2, 2]
    d.hidden = 48
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -2       # no kernel for this width
    d.hidden, d.wdtype = 32, 7
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -1       # bad dtype
    d.wdtype = 0
    d.occ_res[:] = [4, 4, 4]
    d.occupancy = None
    assert lib.kn_scene_create(C.byref(d), None, C.byref(h)) == -1       # grid announced, not given
    out = C.c_int64()
    assert lib.kn_workspace_bytes(None, 10, 10, C.byref(out)) == -1
    assert lib.kn_cell_ids(None, None, None, 0, None) == -1
    assert lib.kn_render(None, None, None, None, 0, 0.0, 1.0, 8, 0.0, None, None, None, None, 0) == -1
    bg = (C.c_float * 3)(0, 0, 0)
    assert lib.kn_render_stratified(None, None, None, None, 0, 0.0, 1.0, 8, 0.0, C.byref(bg), 1, None, None, None, 0) == -1
    assert lib.kn_march_stratified(None, None, None, None, 0, 0.0, 1.0, 8, 1, None, 4, None, None, None) == -1
    assert lib.kn_composite(None, None, None, None, -1, 0.1, 0.0, C.byref(bg), None, None, None) == -1
    assert lib.kn_composite(None, None, None, None, 0, 0.0, 0.0, C.byref(bg), None, None, None) == -1   # step <= 0
    assert lib.kn_composite(None, None, None, None, 0, 0.1, 1.5, C.byref(bg), None, None, None) == -1   # eps >= 1
    assert lib.kn_composite(None, None, None, None, 0, 0.1, 0.01, C.byref(bg), None, None, None) == 0   # R = 0: no-op
    assert lib.kn_composite_deltas(None, None, None, None, None, -1, 0.0, C.byref(bg), None, None, None) == -1
    assert lib.kn_composite_deltas(None, None, None, None, None, 0, 1.5, C.byref(bg), None, None, None) == -1   # eps >= 1
    assert lib.kn_composite_deltas(None, None, None, None, None, 0, 0.0, C.byref(bg), None, None, None) == 0    # R = 0
    assert lib.kn_set_render_params(0, 0, 0) == 0
    res = (C.c_int32 * 3)(4, 4, 4)
    assert lib.kn_extract_occupancy(None, None, C.byref(res), 1.0, None, None, 0) == -1
    assert lib.kn_extract_workspace_bytes(None, C.byref(out)) == -1
    assert lib.kn_layered_workspace_bytes(None, 10, C.byref(out)) == -1
    assert lib.kn_eval_grouped_layered(None, None, None, None, 0, None, None, None, 0) == -1


def test_binding_refuses_to_run_without_the_library(monkeypatch):
    monkeypatch.setattr(kn, "_lib", None)
    monkeypatch.setattr(kn, "LIB_PATH", "/nonexistent/libkilonerf_hip.so")
    with pytest.raises(kn.KnError):
        kn.load_library(build_if_missing=False)
