"""The rounding model of a 16-bit evaluation (oracle/lowprec.py) pinned to the oracle and to the number formats, and
what it says about the pixel bar: how far rounding alone moves a pixel depends on density unit x sample spacing,
because Eq. 4 multiplies a density error by delta.  CPU only."""
import math

import numpy as np

import kn_synth as ks
from kn_synth import configs
from oracle import OracleScene, lowprec
from tests.util import scene_dict


def oracle_scene(sc):
    return OracleScene(sc["res"], sc["aabb_min"], sc["aabb_max"], sc["hidden"], sc["weights"], sc["occupancy"], threads=True)


def test_round_operand_is_round_to_nearest_even_of_the_format():
    r = lowprec.round_operand
    # bf16 keeps 8 significant bits: spacing 2^-7 in [1, 2)
    assert r(1.0 + 2.0 ** -8, "bf16") == 1.0                      # tie -> even (1.0)
    assert r(1.0 + 3 * 2.0 ** -8, "bf16") == 1.0 + 2.0 ** -6      # tie -> even (1 + 2 * 2^-7)
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -20, "bf16") == 1.0 + 2.0 ** -7
    assert r(-3.0e38, "bf16") < -2.9e38 and r(1e-30, "bf16") > 0   # fp32's exponent range
    # fp16 keeps 11 significant bits: spacing 2^-10 in [1, 2)
    assert r(1.0 + 2.0 ** -11, "f16") == 1.0 and r(1.0 + 3 * 2.0 ** -11, "f16") == 1.0 + 2.0 ** -9
    assert r(65504.0, "f16") == 65504.0
    x = np.linspace(-4, 4, 10001)
    for dt, bits in (("bf16", 8), ("f16", 11)):
        y = r(x, dt)
        assert np.all(np.abs(y - x) <= np.abs(x) * 2.0 ** -bits + 1e-12)      # half a unit in the last place
        assert np.array_equal(r(y, dt), y)                                      # idempotent
    assert np.array_equal(r(x.astype(np.float32), "f32"), x.astype(np.float32).astype(np.float64))


def test_model_without_rounding_is_the_oracle():
    """dtype 'f32' rounds operands to fp32 only: then the model is Eq. 7 as the oracle computes it (a wrong layer
    connection, activation or feature order in the model would show here)."""
    for H in (32, 64):
        sc = scene_dict((2, 3, 2), (-1, -1, -1), (1, 1, 1), H, "f32", 31 + H, sigma_scale=20.0)
        orc = oracle_scene(sc)
        pts, dirs = ks.uniform_points(3000, 1, lo=(-1.05,) * 3, hi=(1.05,) * 3), ks.sphere_dirs(3000, 2)
        so, co, ids = orc.eval_points(pts, dirs)
        sm, cm = lowprec.eval_points(sc["weights"], H, ids, pts, dirs, "f32")
        assert np.abs(sm - so).max() < 2e-5 and np.abs(cm - co).max() < 1e-6
        assert np.all(sm[ids < 0] == 0) and (ids < 0).sum() > 50
        # feature layer and layer 4 taken as one affine map (no activation between them, Sec. 3.2): the same function
        sf, cf = lowprec.eval_points(sc["weights"], H, ids, pts, dirs, "f32", fold=True)
        assert np.array_equal(sf, sm) and 0 < np.abs(cf - cm).max() < 1e-6 and np.abs(cf - co).max() < 1e-6
    want, _, mg = orc.extract_occupancy((8, 12, 8), 5.0)
    occ, m = lowprec.extract_occupancy(orc, sc["weights"], 64, "f32", (8, 12, 8), 5.0)
    far = mg.ravel() > 1e-4
    assert np.array_equal(occ[far], want.ravel()[far]) and np.abs(m - mg.ravel()).max() < 1e-4 and 0.05 < want.mean() < 0.99
    pick = np.array([0, 5, 100, 767], np.int64)
    occ2, m2 = lowprec.extract_occupancy(orc, sc["weights"], 64, "f32", (8, 12, 8), 5.0, voxels=pick)
    assert np.array_equal(occ2, occ[pick]) and np.array_equal(m2, m[pick])


def test_density_rounding_error_is_a_fraction_of_the_density_unit():
    """The model's distance to the oracle: about 2^-6 of the density unit for bf16 and 2^-9 for fp16 at most (a
    pre-activation is a sum of some tens of products of operands rounded to 8 / 11 bits), the same for every unit."""
    for unit in (1.0, 100.0):
        sc16 = {}
        for dt, rho in (("bf16", 2.0 ** -6), ("f16", 2.0 ** -9)):
            sc = scene_dict((3, 3, 3), (-1, -1, -1), (1, 1, 1), 32, dt, 7, sigma_scale=unit)
            orc = oracle_scene(sc)
            pts, dirs = ks.uniform_points(20000, 3, lo=(-1,) * 3, hi=(1,) * 3), ks.sphere_dirs(20000, 4)
            so, co, ids = orc.eval_points(pts, dirs)
            sm, cm = lowprec.eval_points(sc["weights"], 32, ids, pts, dirs, dt)
            e = np.abs(sm - so) / unit
            sc16[dt] = e.max()
            assert rho / 4 < e.max() < 1.25 * rho, (dt, unit, e.max())
            assert np.abs(cm - co).max() < (8e-3 if dt == "bf16" else 1e-3)
            # with the feature layer folded into layer 4 the rounding of the product matrix takes the place of the
            # rounding of the feature vector: the same density, a colour error of the same size
            sf, cf = lowprec.eval_points(sc["weights"], 32, ids, pts, dirs, dt, fold=True)
            assert np.array_equal(sf, sm) and np.abs(cf - co).max() < (8e-3 if dt == "bf16" else 1e-3)
            assert 0.5 < np.abs(cf - co).mean() / np.abs(cm - co).mean() < 1.5
        assert 4 < sc16["bf16"] / sc16["f16"] < 16         # three more bits


def test_pixel_error_of_rounding_alone_grows_with_density_unit_times_step():
    """Eq. 4: alpha = 1 - exp(-sigma delta), so a density error e moves alpha by up to delta e.  On a fine lattice
    (density unit x step below 1: the benchmark scenes have 0.68 and 0.34) bf16 rounding moves pixels by well under the
    2e-2 bar; the same networks sampled with one coarse step per ray (unit x step in the hundreds) are beyond it
    although every density is as accurate as before.  No 16-bit evaluation can meet an absolute pixel bar there."""
    cfg = configs.config3(20, 20, wdtype="bf16")
    sc = cfg["scene"]
    orc = oracle_scene(sc)
    o, d = cfg["rays_o"], cfg["rays_d"]
    fine = lowprec.render_midpoint(orc, sc["weights"], 32, "bf16", o, d, cfg["t_near"], cfg["step"], cfg["K"], 0.0, cfg["bg"])
    ref = orc.render(o, d, cfg["t_near"], cfg["step"], cfg["K"], 0.0, cfg["bg"])[0]
    assert 100.0 * cfg["step"] < 1.0
    assert 1e-4 < np.abs(fine - ref).max() < 1e-2
    # one lattice point per ray, in the middle of the box, no occupancy grid: unit x step = 350
    sc1 = dict(sc, occupancy=None)
    orc1 = oracle_scene(sc1)
    o, d = ks.camera_rays(48, 48, 30.0, 4.0, 45.0, 30.0)
    step = 2.0 * math.sqrt(3.0)
    coarse = lowprec.render_midpoint(orc1, sc["weights"], 32, "bf16", o, d, 4.0 - step / 2, step, 1, 0.0, cfg["bg"])
    ref1 = orc1.render(o, d, 4.0 - step / 2, step, 1, 0.0, cfg["bg"])[0]
    err = np.abs(coarse - ref1).max(axis=1)
    assert err.max() > 2e-2 and np.mean(err > 2e-2) < 0.05      # a few pixels far off, most untouched
