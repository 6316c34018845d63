"""Parity of the HIP path against the CPU oracle, element by element, through the C ABI.

Bars: cell ids, bucket counts and the sample permutation bit-exact; fp32 outputs within 1e-4
absolute; 16-bit matrix-core outputs within 2e-2 absolute (density: 2e-2 absolute + 2e-2 relative,
because its scale is free).  Rays whose transmittance comes within MARGIN (relative) of the
termination threshold may legitimately stop one sample earlier or later than the oracle; the
skipped / extra sample contributes at most eps, so those rays are compared at tolerance + eps.

A 16-bit pixel bar needs a regime: Eq. 4 multiplies a density error by the sample spacing, and the density of a
16-bit evaluation is off by up to RHO density units by rounding alone (tests/test_lowprec_model.py), so one
sample can move a pixel by 1 - exp(-RHO * unit * step).  The 2e-2 bar is asserted where RHO * unit * step <= 2e-2
(unit * step <= 1 for bf16, <= 8 for fp16: every benchmark workload, 0.34 to 0.68); beyond that regime the bar is
widened by exactly that term.
"""
import math
import os

import numpy as np
import pytest

import kn_synth as ks
import oracle
from kn_synth import configs
from tests.util import cuda, make_pair, scene_dict

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "f16": 2e-2, "bf16": 2e-2}
# relative distance of a ray's transmittance to eps below which the ray may stop one sample apart from the oracle: a few
# times the relative error of T, which is the summed density error times the step (16-bit: about 3e-3 / 4e-4 density
# units per sample, tens of samples, unit * step below 1)
MARGIN = {"f32": 1e-3, "f16": 0.01, "bf16": 0.03}
# largest density error of a 16-bit evaluation by rounding alone, in density units (the bar on sigma, and an eighth
# of it: fp16 keeps three more bits)
RHO = {"f16": 2.5e-3, "bf16": 2e-2}


def pixel_bar(wdtype, unit_times_step):
    """The pixel bar of a 16-bit scene: 2e-2 inside the supported regime, widened beyond it by what the rounding of
    one sample's density can move a pixel (module docstring)."""
    if wdtype == "f32":
        return TOL["f32"]
    worst = RHO[wdtype] * unit_times_step
    return TOL[wdtype] + (0.0 if worst <= TOL[wdtype] else 1.0 - math.exp(-worst))


def log(*a):
    print(*a, flush=True)


# ------------------------------------------------------------------ a2: cell ids
@pytest.mark.parametrize("res,lo,hi", [((2, 2, 2), (0, 0, 0), (1, 1, 1)), ((3, 4, 5), (-1, 0, 0.5), (1, 2, 4.5)),
                                       ((10, 16, 10), (-0.67, -1.07, -0.67), (0.67, 1.07, 0.67)),
                                       ((16, 16, 16), (-1, -1, -1), (1, 1, 1)), ((32, 32, 32), (0, 0, 0), (1, 1, 1))])
def test_cell_ids_bit_exact(res, lo, hi):
    log("cell ids", res)
    sc = scene_dict(res, lo, hi, 32, "f32", 1)
    dev, orc = make_pair(sc)
    g = ks.rng(17)
    lo_, hi_ = np.array(lo), np.array(hi)
    M = 200_003
    pts = (lo_ - 0.05 + g.random((M, 3)) * (hi_ - lo_ + 0.1)).astype(np.float32)
    # points exactly on cell faces and on the box faces
    faces = lo_ + (hi_ - lo_) * g.integers(0, np.array(res) + 1, size=(5000, 3)) / np.array(res)
    pts[:5000] = faces.astype(np.float32)
    pts[5000] = [np.nan, 0, 0]
    pts[5001] = [np.inf, 0, 0]
    got = dev.cell_ids(cuda(pts)).cpu().numpy()
    want = orc.cell_ids(pts)
    np.testing.assert_array_equal(got, want)
    assert (want < 0).sum() > 100 and len(np.unique(want)) > 0.9 * int(np.prod(res))


# ------------------------------------------------------------------ a3: bucketing
@pytest.mark.parametrize("N,M,mode", [(8, 0, "uniform"), (8, 1, "uniform"), (8, 63, "uniform"), (8, 4097, "uniform"),
                                      (4096, 300_001, "uniform"), (4096, 500_000, "skew"), (4096, 70_000, "single"),
                                      (4096, 5000, "outside"), (32768, 1_000_003, "uniform"), (60, 10_000, "uniform")])
def test_bucket_bit_exact(N, M, mode):
    log("bucket", N, M, mode)
    res = {8: (2, 2, 2), 4096: (16, 16, 16), 32768: (32, 32, 32), 60: (3, 4, 5)}[N]
    dev, _ = make_pair(scene_dict(res, (0, 0, 0), (1, 1, 1), 32, "f32", 1))
    g = ks.rng(23 + N + M)
    if mode == "uniform":
        ids = g.integers(-1, N, size=M)
    elif mode == "skew":
        hot = g.integers(0, N, size=20)
        ids = np.where(g.random(M) < 0.9, hot[g.integers(0, 20, size=M)], g.integers(-1, N, size=M))
    elif mode == "single":
        ids = np.full(M, 1234)
    else:
        ids = np.full(M, -1)
    ids = ids.astype(np.int32)
    counts, offsets, perm = dev.bucket(cuda(ids))
    c, o, p = oracle.bucket(ids, N)
    np.testing.assert_array_equal(counts.cpu().numpy(), c)
    np.testing.assert_array_equal(offsets.cpu().numpy(), o)
    np.testing.assert_array_equal(perm.cpu().numpy(), p)


# ------------------------------------------------------------------ a4: grouped MLP through eval_grouped
def check_eval(sc, pts, dirs, sample=None, tol=None, sigma_unit=1.0):
    """sigma_unit: density scale of the scene (the factor its density head was multiplied by);
    the density tolerance is stated in that unit."""
    import torch
    dev, orc = make_pair(sc, threads=True)
    tol = TOL[sc["wdtype"]] if tol is None else tol
    sg, rgb, ids, counts, perm = dev.eval_grouped(cuda(pts), cuda(dirs), want_aux=True)
    torch.cuda.synchronize()
    ids_o = orc.cell_ids(pts)
    np.testing.assert_array_equal(ids.cpu().numpy(), ids_o)
    c, o, p = oracle.bucket(ids_o, orc.N)
    np.testing.assert_array_equal(counts.cpu().numpy(), c)
    np.testing.assert_array_equal(perm.cpu().numpy(), p)
    sel = np.arange(len(pts)) if sample is None else sample
    s_o, c_o, _ = orc.eval_points(pts[sel], dirs[sel])
    s_g, c_g = sg.cpu().numpy()[sel].astype(np.float64), rgb.cpu().numpy()[sel].astype(np.float64)
    err_c = np.abs(c_g - c_o).max()
    s_g, s_o = s_g / sigma_unit, s_o / sigma_unit
    err_s = (np.abs(s_g - s_o) / (1.0 + (0 if tol < 1e-3 else 1) * np.abs(s_o))).max()
    log("  eval %s H=%d M=%d: max |rgb err| %.3g, max sigma err (abs or abs/(1+|s|)) %.3g" %
        (sc["wdtype"], sc["hidden"], len(pts), err_c, err_s))
    assert err_c <= tol and err_s <= tol
    outside = ids_o[sel] < 0
    assert np.all(s_g[outside] == 0) and np.all(c_g[outside] == 0)
    return dev


@pytest.mark.parametrize("H", [32, 64])
def test_eval_grouped_fp32(H):
    sc = scene_dict((2, 2, 2), (0, 0, 0), (1, 1, 1), H, "f32", 5)
    M = 20_011
    pts = ks.uniform_points(M, 1, lo=(-0.05,) * 3, hi=(1.05,) * 3)
    check_eval(sc, pts, ks.sphere_dirs(M, 2))


def test_eval_grouped_fp32_noncubic_grid():
    sc = scene_dict((10, 16, 10), (-0.67, -1.07, -0.67), (0.67, 1.07, 0.67), 32, "f32", 6)   # the Lego grid of Sec. 4.3
    M = 30_000
    pts = ks.uniform_points(M, 3, lo=(-0.7, -1.1, -0.7), hi=(0.7, 1.1, 0.7))
    check_eval(sc, pts, ks.sphere_dirs(M, 4))


def test_eval_grouped_fp32_large_box():
    # 2^9 p reaches tens of thousands of radians: the encoding's range reduction has to stay accurate there
    sc = scene_dict((3, 2, 4), (-40, -10, 5), (40, 30, 45), 32, "f32", 18)
    M = 10_003
    pts = ks.uniform_points(M, 19, lo=(-41, -11, 4), hi=(41, 31, 46))
    check_eval(sc, pts, ks.sphere_dirs(M, 20))


@pytest.mark.parametrize("wdtype,H", [("f16", 32), ("bf16", 32), ("f16", 64), ("bf16", 64)])
def test_eval_grouped_matrix_cores(wdtype, H):
    sc = scene_dict((4, 4, 4), (-1, -1, -1), (1, 1, 1), H, wdtype, 7)
    M = 50_021
    pts = ks.uniform_points(M, 5, lo=(-1.02,) * 3, hi=(1.02,) * 3)
    check_eval(sc, pts, ks.sphere_dirs(M, 6))


@pytest.mark.parametrize("wdtype,H,unit", [("bf16", 32, 1.0), ("bf16", 64, 100.0), ("f16", 32, 100.0), ("f16", 64, 1.0)])
def test_matrix_core_kernel_follows_the_rounding_model(wdtype, H, unit):
    """Rounding or defect?  The kernel against Eq. 7 with every matrix operand rounded to the storage type and
    nothing else changed (oracle/lowprec.py).  The two can differ only where a sum or a sine lands within the kernel's
    own fp32 / hardware-sine error of a rounding boundary and one operand comes out one unit in the last place apart,
    so they agree far more closely than the kernel and the fp64 oracle do: what separates kernel and oracle is the
    rounding of the operands, which any 16-bit evaluation has."""
    from oracle import lowprec
    sc = scene_dict((4, 3, 5), (-1, -1, -1), (1, 1, 1), H, wdtype, 141, sigma_scale=unit)
    M = 40_009
    pts, dirs = ks.uniform_points(M, 142, lo=(-1,) * 3, hi=(1,) * 3), ks.sphere_dirs(M, 143)
    dev, orc = make_pair(sc, threads=True)
    s_g, c_g = [t.cpu().numpy().astype(np.float64) for t in dev.eval_grouped(cuda(pts), cuda(dirs))]
    s_o, c_o, ids = orc.eval_points(pts, dirs)
    s_m, c_m = lowprec.eval_points(sc["weights"], H, ids, pts, dirs, wdtype, fold=True)  # (the kernels fold the feature layer)
    to_oracle, to_model = np.abs(s_g - s_o) / unit, np.abs(s_g - s_m) / unit
    q = lambda a: float(np.quantile(a, 0.99))
    log("  %s H=%d unit %g: density error / unit, kernel - oracle max %.2e p99 %.2e; kernel - model max %.2e p99 %.2e; "
        "model - oracle max %.2e; colour: kernel - oracle %.2e, kernel - model p99 %.2e" %
        (wdtype, H, unit, to_oracle.max(), q(to_oracle), to_model.max(), q(to_model), (np.abs(s_m - s_o) / unit).max(),
         np.abs(c_g - c_o).max(), q(np.abs(c_g - c_m))))
    assert to_oracle.max() <= RHO[wdtype] and (np.abs(s_m - s_o) / unit).max() <= RHO[wdtype]     # both within the rounding bound
    assert q(to_model) <= {"bf16": 3e-3, "f16": 1e-3}[wdtype]
    assert np.mean(to_model <= 1e-5) > 0.5          # most samples: the model's value up to fp32 summation
    if wdtype == "bf16":
        assert q(to_model) < 0.5 * q(to_oracle)
    assert q(np.abs(c_g - c_m)) <= {"bf16": 2e-3, "f16": 5e-4}[wdtype]


def test_render_refuses_more_rays_than_its_32_bit_indices_hold():
    """kn_render's limits on the number of rays (packed (ray, k) records, slot numbers, byte offsets into the table of
    encoded directions): one ray beyond a limit is KN_E_UNSUPPORTED (-2), at the limit the call goes on to its next check
    (the workspace, which is too small here: -3).  Nothing is launched either way."""
    import ctypes as C
    import torch
    import paper_2103_13744_amd as kn
    sc = scene_dict((1, 1, 1), (0, 0, 0), (1, 1, 1), 32, "f16", 171)
    dev, _ = make_pair(sc)
    L = kn.load_library()
    buf = torch.zeros(1024, dtype=torch.float32, device="cuda")
    ws = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    bg = (C.c_float * 3)(0, 0, 0)

    def call(R, K):
        return L.kn_render(dev._ctx(None), dev.h, None, C.c_void_p(buf.data_ptr()), C.c_void_p(buf.data_ptr()), C.c_int64(R),
                           C.c_float(0.0), C.c_float(0.1), C.c_int32(K), C.c_float(0.0), C.byref(bg), C.c_void_p(buf.data_ptr()), None,
                           C.c_void_p(ws.data_ptr()), C.c_int64(ws.numel()))
    assert call(2 ** 23, 512) == -3 and call(2 ** 23 + 1, 512) == -2            # ray << 9 | k in 32 bits
    assert call((2 ** 31 - 1) // 128, 2) == -3 and call((2 ** 31 - 1) // 128 + 1, 2) == -2     # 128 slots per ray
    kn.set_render_params(0, 16, 0)
    try:
        assert call(2 ** 26, 2) == -3 and call(2 ** 26 + 1, 2) == -2            # 64 bytes of encoded direction per ray
    finally:
        kn.set_render_params(0, 0, 0)


def test_stage_timing_on_one_call_in_n():
    """KN_OPT_PROFILE_EVERY: events are recorded on one call in n, counted from the moment timing is switched on; the
    results do not depend on it."""
    import paper_2103_13744_amd as kn
    sc = scene_dict((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, "f16", 181)
    dev, _ = make_pair(sc)
    ctx = kn.Context()
    pts, dirs = cuda(ks.uniform_points(5000, 182)), cuda(ks.sphere_dirs(5000, 183))
    want = dev.eval_grouped(pts, dirs)
    for every, timed in ((1, 7), (3, 3), (0, 7), (100, 1)):
        ctx.set_option(kn.OPT_PROFILE_EVERY, every)
        ctx.profile_enable(1)
        for _ in range(7):
            got = dev.eval_grouped(pts, dirs, ctx=ctx)
        prof = ctx.profile_read()
        ctx.profile_enable(0)
        assert prof["calls"] == timed and prof["mlp_launches"] == timed and prof["ms_mlp"] > 0
        assert all(bool((a == b).all()) for a, b in zip(got, want))
    with pytest.raises(kn.KnError):
        ctx.set_option(kn.OPT_PROFILE_EVERY, 2 ** 31)


def test_folded_feature_layer_out_of_fp16_range_is_refused():
    """The 16-bit kernels take layer 3's feature vector and layer 4 as one affine map (Sec. 3.2 puts no activation between
    them) whose matrix is rounded to the scene's type.  fp16 weights whose products sum beyond 65504 cannot be carried
    that way: scene creation refuses them; the same numbers in bf16 (fp32's range) make a scene."""
    import paper_2103_13744_amd as kn
    H = 32
    sc = scene_dict((2, 1, 1), (0, 0, 0), (1, 1, 1), H, "f16", 151)
    P = sc["weights"].shape[1]
    oW3 = 63 * H + H + H * H + H
    oW4 = oW3 + H * (H + 1) + (H + 1)
    w = sc["weights"].copy()
    w[1, oW3:oW3 + H * (H + 1)] = 60.0                  # network 1: every feature weight 60, every layer-4 weight 60:
    w[1, oW4:oW4 + (H + 27) * H] = 60.0                 # 32 x 3600 = 115,200 per element of the product
    assert oW4 + (H + 27) * H + H + 3 * H + 3 == P
    with pytest.raises(kn.KnError, match="-2|unsupported|UNSUPPORTED"):
        make_pair(dict(sc, weights=w))
    make_pair(dict(sc, weights=w, wdtype="bf16"))       # 60 is a bf16 number as well
    make_pair(sc)


def test_eval_grouped_matrix_cores_large_box():
    # coordinates large enough that 2^9 p leaves the range the sine hardware reduces by itself (f16 only: the
    # raw coordinates are network inputs too, and rounding 45.0 to bf16 alone costs more than the tolerance)
    sc = scene_dict((3, 2, 4), (-40, -10, 5), (40, 30, 45), 32, "f16", 17)
    M = 20_003
    pts = ks.uniform_points(M, 15, lo=(-41, -11, 4), hi=(41, 31, 46))
    check_eval(sc, pts, ks.sphere_dirs(M, 16))


def test_eval_grouped_density_scaled_and_tiny_groups():
    # sigma_scale as in the render workload; 16^3 networks with few points each => many partial tiles
    sc = scene_dict((16, 16, 16), (-1, -1, -1), (1, 1, 1), 32, "f16", 8, sigma_scale=100.0)
    M = 40_000
    pts = ks.uniform_points(M, 7, lo=(-1,) * 3, hi=(1,) * 3)
    check_eval(sc, pts, ks.sphere_dirs(M, 8), sigma_unit=100.0)


def test_eval_grouped_empty_and_permutation_invariance():
    import torch
    sc = scene_dict((4, 4, 4), (0, 0, 0), (1, 1, 1), 32, "f16", 9)
    dev, _ = make_pair(sc)
    e = torch.empty((0, 3), dtype=torch.float32, device="cuda")
    sg, rgb = dev.eval_grouped(e, e)
    assert sg.numel() == 0 and rgb.numel() == 0
    M = 30_000
    pts, dirs = ks.uniform_points(M, 1), ks.sphere_dirs(M, 2)
    s1, c1 = [t.cpu().numpy() for t in dev.eval_grouped(cuda(pts), cuda(dirs))]
    p = ks.rng(3).permutation(M)
    s2, c2 = [t.cpu().numpy() for t in dev.eval_grouped(cuda(pts[p]), cuda(dirs[p]))]
    np.testing.assert_array_equal(s2, s1[p])      # each sample's arithmetic is independent of its tile mates
    np.testing.assert_array_equal(c2, c1[p])


@pytest.mark.parametrize("res,M,mode", [((1, 1, 1), 5_000, "mixed"),         # one network: keys 0 / 1, one pass of one bit
                                        ((3, 5, 17), 20_000, "mixed"),       # 255 networks + "outside" = 256 keys: one pass of 8 bits
                                        ((4, 8, 8), 12_289, "mixed"),        # 257 keys: two passes (5 + 4 bits); 3 blocks + 1 record
                                        ((4, 8, 8), 1, "inside"), ((4, 8, 8), 4096, "inside"), ((4, 8, 8), 4097, "outside"),
                                        ((16, 16, 16), 70_001, "skewed")])
def test_eval_grouped_reordering_edge_cases(res, M, mode):
    """kn_eval_grouped moves the samples themselves into grouped order (a radix sort of 32-byte records, one or two
    passes by the number of key bits): ids, counts and the stable permutation bit-exact, results within the bar, and
    equal bit for bit to the evaluation that sorts indices instead (kn_eval_grouped_static)."""
    import torch
    sc = scene_dict(res, (-1, -1, -1), (1, 1, 1), 32, "f16", 61)
    span = {"mixed": 1.15, "inside": 0.999, "outside": 1.0, "skewed": 1.0}[mode]
    pts = ks.uniform_points(M, 62, lo=(-span,) * 3, hi=(span,) * 3)
    if mode == "outside":
        pts = pts + np.float32(3.0)
        pts[::7] = np.nan
    if mode == "skewed":        # nine points in ten in a twentieth of the box
        pts[: 9 * M // 10, 0] = pts[: 9 * M // 10, 0] * np.float32(0.05)
        pts = pts[ks.rng(63).permutation(M)]
    dirs = ks.sphere_dirs(M, 64)
    sel = None if M <= 20_000 else ks.rng(65).choice(M, size=5_000, replace=False)
    dev = check_eval(sc, pts, dirs, sample=sel)
    out = dev.eval_grouped(cuda(pts), cuda(dirs), want_aux=True)
    ref = (torch.empty(M, dtype=torch.float32, device="cuda"), torch.empty((M, 3), dtype=torch.float32, device="cuda"))
    aux = (torch.empty(M, dtype=torch.int32, device="cuda"), torch.empty(dev.N + 1, dtype=torch.int32, device="cuda"),
           torch.empty(M, dtype=torch.int32, device="cuda"))
    dev.eval_grouped_static(cuda(pts), cuda(dirs), ref, aux=aux)
    torch.cuda.synchronize()
    for a, b in zip(out, (*ref, *aux)):
        assert torch.equal(a, b)


def test_eval_grouped_on_arrays_that_start_off_a_sixteen_byte_boundary():
    """Points and directions are fp32 arrays with 4-byte alignment as far as the interface goes; the key kernel reads
    whole tiles of an aligned array 16 bytes at a time and anything else element by element.  Same results either way."""
    import torch
    sc = scene_dict((5, 4, 6), (-1, -1, -1), (1, 1, 1), 32, "f16", 71)
    dev, _ = make_pair(sc)
    M = 3 * 4096 + 17
    pts, dirs = ks.uniform_points(M, 72, lo=(-1.05,) * 3, hi=(1.05,) * 3), ks.sphere_dirs(M, 73)
    want = dev.eval_grouped(cuda(pts), cuda(dirs), want_aux=True)
    for shift in (1, 2, 3):                                      # floats in front of the arrays
        flat_p = torch.zeros(3 * M + shift, dtype=torch.float32, device="cuda")
        flat_d = torch.zeros(3 * M + shift, dtype=torch.float32, device="cuda")
        p_off, d_off = flat_p[shift:].view(M, 3), flat_d[shift:].view(M, 3)
        p_off.copy_(cuda(pts))
        d_off.copy_(cuda(dirs))
        assert p_off.data_ptr() % 16 == 4 * shift and p_off.is_contiguous()
        got = dev.eval_grouped(p_off, d_off, want_aux=True)
        torch.cuda.synchronize()
        for a, b in zip(got, want):
            assert torch.equal(a, b)


def test_eval_grouped_reordering_with_sixteen_key_bits():
    """32^3 networks: keys need 16 bits, two passes of 8."""
    sc = scene_dict((32, 32, 32), (0, 0, 0), (1, 1, 1), 32, "f16", 66)
    M = 300_007
    pts = ks.uniform_points(M, 67, lo=(-0.01,) * 3, hi=(1.01,) * 3)
    check_eval(sc, pts, ks.sphere_dirs(M, 68), sample=ks.rng(69).choice(M, size=4_000, replace=False))


@pytest.mark.parametrize("wdtype,H", [("f16", 32), ("bf16", 32), ("f16", 64), ("bf16", 64)])
def test_layer_at_a_time_equals_fused_and_oracle(wdtype, H):
    """Sec. 3.5's grouped matrix products, one launch per layer: same operands and order of operations as the fused
    kernel, so the same bits; and within the 16-bit bar of the oracle."""
    import torch
    sc = scene_dict((4, 3, 5), (-1, -1, -1), (1, 1, 1), H, wdtype, 41, sigma_scale=3.0)
    M = 23_017                                                   # ragged groups, a ragged last tile, points outside
    pts, dirs = ks.uniform_points(M, 42, lo=(-1.03,) * 3, hi=(1.03,) * 3), ks.sphere_dirs(M, 43)
    dev, orc = make_pair(sc, threads=True)
    s_f, c_f = [t.cpu().numpy() for t in dev.eval_grouped(cuda(pts), cuda(dirs))]
    s_l, c_l = [t.cpu().numpy() for t in dev.eval_grouped_layered(cuda(pts), cuda(dirs))]
    np.testing.assert_array_equal(s_l, s_f)
    np.testing.assert_array_equal(c_l, c_f)
    s_o, c_o, ids = orc.eval_points(pts, dirs)
    assert np.abs(c_l - c_o).max() <= TOL[wdtype]
    assert (np.abs(s_l - s_o) / 3.0 / (1 + s_o / 3.0)).max() <= TOL[wdtype]
    assert np.all(s_l[ids < 0] == 0) and np.all(c_l[ids < 0] == 0) and (ids < 0).sum() > 100
    e = torch.empty((0, 3), dtype=torch.float32, device="cuda")
    assert dev.eval_grouped_layered(e, e)[0].numel() == 0


def test_layer_at_a_time_is_refused_for_fp32_scenes():
    import paper_2103_13744_amd as kn
    sc = scene_dict((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, "f32", 44)
    dev, _ = make_pair(sc)
    pts, dirs = ks.uniform_points(100, 45), ks.sphere_dirs(100, 46)
    with pytest.raises(kn.KnError):
        dev.eval_grouped_layered(cuda(pts), cuda(dirs))


def test_eval_grouped_random_configurations_fp32():
    """Thirty seeded random cases: grid shapes, boxes, batch sizes from 0 to a few thousand, points partly outside."""
    g = np.random.default_rng(20210314)
    for it in range(30):
        H = [32, 64][g.integers(0, 2)]
        nres = tuple(int(v) for v in g.integers(1, 9, size=3))
        lo = g.uniform(-3, 1, size=3)
        hi = lo + g.uniform(0.3, 4, size=3)
        sc = scene_dict(nres, tuple(lo), tuple(hi), H, "f32", int(g.integers(1, 1 << 30)))
        M = int(g.choice([0, 1, 2, 63, 64, 65, 1000, 4097]))
        pad = 0.05 * (hi - lo)
        pts = ks.uniform_points(M, int(g.integers(1, 1 << 30)), lo=tuple(lo - pad), hi=tuple(hi + pad))
        dirs = ks.sphere_dirs(M, int(g.integers(1, 1 << 30)))
        if M == 0:
            dev, _ = make_pair(sc)
            assert dev.eval_grouped(cuda(pts.reshape(0, 3)), cuda(dirs.reshape(0, 3)))[0].numel() == 0
        else:
            check_eval(sc, pts, dirs)


def test_extract_occupancy_random_configurations_fp32():
    """Fifteen seeded random pairs of network grid and occupancy resolution (mostly not nested), every voxel checked."""
    g = np.random.default_rng(20210315)
    for it in range(15):
        nres = tuple(int(v) for v in g.integers(1, 6, size=3))
        ores = tuple(int(v) for v in g.integers(1, 14, size=3))
        lo = g.uniform(-2, 0, size=3)
        hi = lo + g.uniform(0.5, 3, size=3)
        sc = scene_dict(nres, tuple(lo), tuple(hi), [32, 64][g.integers(0, 2)], "f32", int(g.integers(1, 1 << 30)), sigma_scale=20.0)
        orc = make_pair(sc, threads=True)[1]
        top = orc.extract_occupancy(ores, 0.0)[1]
        tau = float(np.quantile(top, g.uniform(0.2, 0.8)))
        dev = make_pair(sc)[0]
        got = dev.extract_occupancy(ores, tau).cpu().numpy()
        want, _, mg = orc.extract_occupancy(ores, tau)
        close = mg <= 1e-4 * 20.0
        np.testing.assert_array_equal(got[~close], want[~close])
        assert close.sum() <= 2 + 0.01 * close.size


def test_eval_grouped_replays_from_a_hip_graph():
    """kn_eval_grouped neither allocates nor waits on the host, so it can be captured into a graph: three replays on
    fresh inputs, with eager calls in between, each equal to the eager result of the same inputs."""
    import torch
    sc = scene_dict((4, 4, 4), (0, 0, 0), (1, 1, 1), 32, "f16", 61)
    dev, _ = make_pair(sc)
    M = 20_000
    pts, dirs = torch.empty((M, 3), device="cuda"), torch.empty((M, 3), device="cuda")
    out = (torch.empty(M, device="cuda"), torch.empty((M, 3), device="cuda"))
    batches = [(cuda(ks.uniform_points(M, 62 + i, lo=(-0.05,) * 3, hi=(1.05,) * 3)), cuda(ks.sphere_dirs(M, 72 + i)))
               for i in range(3)]
    pts.copy_(batches[0][0])
    dirs.copy_(batches[0][1])
    dev.eval_grouped(pts, dirs, out=out)                       # warm-up: workspace allocated, kernels loaded
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            dev.eval_grouped(pts, dirs, out=out)
    torch.cuda.current_stream().wait_stream(side)
    for p, d in batches:
        want_s, want_c = [t.clone() for t in dev.eval_grouped(p, d)]      # eager, own output buffers
        torch.cuda.synchronize()
        pts.copy_(p)
        dirs.copy_(d)
        out[0].zero_()
        out[1].zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out[0], want_s) and torch.equal(out[1], want_c)
        assert float(want_s.abs().sum()) > 0


# ------------------------------------------------------------------ a1: marching
def test_march_bit_exact_and_resumable():
    cfg = configs.config3(40, 40)
    dev, orc = make_pair(cfg["scene"])
    o, d = cfg["rays_o"], cfg["rays_d"]
    K = cfg["K"]
    out_k, cnt, nxt = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], K)
    out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
    total = 0
    for r in range(len(o)):
        want = orc.march(o[r], d[r], cfg["t_near"], cfg["step"], K)
        assert cnt[r] == len(want), r
        np.testing.assert_array_equal(out_k[r, :cnt[r]], want)
        assert np.all(out_k[r, cnt[r]:] == -1)
        total += len(want)
    assert total > 5000
    # in chunks of 5 samples, resuming where the previous chunk stopped
    kb = cuda(np.zeros(len(o), np.int32))
    got = [[] for _ in range(len(o))]
    for _ in range(K):
        ck, cc, kb = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], K, S=5, k_begin=kb)
        ck, cc = ck.cpu().numpy(), cc.cpu().numpy()
        for r in np.nonzero(cc)[0]:
            got[r] += ck[r, :cc[r]].tolist()
        if cc.sum() == 0:
            break
    for r in range(0, len(o), 7):
        assert got[r] == out_k[r, :cnt[r]].tolist()


def test_march_without_grid_and_axis_parallel_rays():
    cfg = configs.config1(24, 24)
    dev, orc = make_pair(cfg["scene"])
    o, d = cfg["rays_o"].copy(), cfg["rays_d"].copy()
    o[:4] = [[-1, 0.3, 0.6], [0.5, 0.5, -2], [0.2, 3, 0.2], [0.5, 1.0, 0.5]]
    d[:4] = [[1, 0, 0], [0, 0, 1], [0, -1, 0], [1, 0, 0]]        # zero components; last one rides the upper face
    out_k, cnt, _ = dev.march(cuda(o), cuda(d), 0.25, 1 / 16, 80)
    out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
    for r in range(len(o)):
        want = orc.march(o[r], d[r], 0.25, 1 / 16, 80)
        assert cnt[r] == len(want), r
        np.testing.assert_array_equal(out_k[r, :cnt[r]], want)
    assert cnt[0] == 16 and cnt[3] == 0


# ------------------------------------------------------------------ a5: blending
def test_composite_stage():
    import paper_2103_13744_amd as kn
    g = ks.rng(31)
    R = 3000
    n = g.integers(0, 40, size=R)
    n[:3] = 0
    off = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    sg = g.uniform(0, 60, size=off[-1]).astype(np.float32)
    col = g.random((off[-1], 3)).astype(np.float32)
    for eps in (0.0, 0.01):
        out, T, used = kn.composite(cuda(sg), cuda(col), cuda(off), 0.05, eps, (1.0, 0.5, 0.25))
        out, T, used = out.cpu().numpy(), T.cpu().numpy(), used.cpu().numpy()
        for r in range(R):
            o_, T_, u_, mg = oracle.composite(sg[off[r]:off[r + 1]], col[off[r]:off[r + 1]], 0.05, eps, (1.0, 0.5, 0.25))
            if mg > 1e-3:
                assert used[r] == u_
                assert np.abs(out[r] - o_).max() < 1e-5 and abs(T[r] - T_) < 1e-6
            else:
                assert abs(used[r] - u_) <= 1 and np.abs(out[r] - o_).max() < 1e-5 + eps


def test_composite_stage_with_a_delta_per_sample():
    import paper_2103_13744_amd as kn
    g = ks.rng(32)
    R = 2000
    n = g.integers(0, 40, size=R)
    n[:2] = 0
    off = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
    sg = g.uniform(0, 60, size=off[-1]).astype(np.float32)
    col = g.random((off[-1], 3)).astype(np.float32)
    delta = g.uniform(0.01, 0.1, size=off[-1]).astype(np.float32)
    for eps in (0.0, 0.01):
        out, T, used = kn.composite(cuda(sg), cuda(col), cuda(off), cuda(delta), eps, (1.0, 0.5, 0.25))
        out, T, used = out.cpu().numpy(), T.cpu().numpy(), used.cpu().numpy()
        for r in range(R):
            s_ = slice(off[r], off[r + 1])
            o_, T_, u_, mg = oracle.composite(sg[s_], col[s_], delta[s_], eps, (1.0, 0.5, 0.25))
            if mg > 1e-3:
                assert used[r] == u_
                assert np.abs(out[r] - o_).max() < 1e-5 and abs(T[r] - T_) < 1e-6
            else:
                assert abs(used[r] - u_) <= 1 and np.abs(out[r] - o_).max() < 1e-5 + eps
    # equal deltas: the bits of the constant-step call
    a = kn.composite(cuda(sg), cuda(col), cuda(off), cuda(np.full(off[-1], 0.05, np.float32)), 0.01, (1.0, 0.5, 0.25))
    b = kn.composite(cuda(sg), cuda(col), cuda(off), 0.05, 0.01, (1.0, 0.5, 0.25))
    for x, y in zip(a, b):
        np.testing.assert_array_equal(x.cpu().numpy(), y.cpu().numpy())


# ------------------------------------------------------------------ a1-a6: render
def render_check(cfg, sel=None, margin=None):
    """Render on the device, compare (a subset of) pixels with the oracle."""
    import torch
    sc = cfg["scene"]
    tol = TOL[sc["wdtype"]]
    margin = MARGIN[sc["wdtype"]] if margin is None else margin
    dev, orc = make_pair(sc, threads=True)
    o, d = cfg["rays_o"], cfg["rays_d"]
    seed = cfg.get("seed")          # stratified sampling with this seed; None: the midpoint lattice
    img, stats = dev.render(cuda(o), cuda(d), cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"], want_stats=True,
                            seed=seed)
    torch.cuda.synchronize()
    img = img.cpu().numpy().astype(np.float64)
    sel = np.arange(len(o)) if sel is None else sel
    ref, n_eval, T, mg = orc.render(o[sel], d[sel], cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"], seed=seed,
                                    ray_ids=None if seed is None else sel)       # the draws are keyed by the ray's row
    err = np.abs(img[sel] - ref).max(axis=1)
    straddle = mg < margin
    log("  render %s: %d rays, waves %d, evaluated %d, blended %d; oracle blended (subset) %d; max err %.3g "
        "(straddling rays: %d, max err there %.3g)" % (cfg["name"], len(o), stats["waves"], stats["samples_evaluated"],
                                                     stats["samples_blended"], n_eval.sum(), err[~straddle].max(),
                                                     straddle.sum(), err[straddle].max() if straddle.any() else 0))
    assert err[~straddle].max() <= tol
    if straddle.any():
        assert err[straddle].max() <= tol + cfg["term_eps"]
    assert straddle.mean() < {"f32": 0.002, "f16": 0.02, "bf16": 0.06}[sc["wdtype"]]     # observed: 0.001, 0.005, 0.04
    assert stats["rays"] == len(o) and stats["samples_evaluated"] >= stats["samples_blended"]
    if sel is None or len(sel) == len(o):
        if not straddle.any():
            assert stats["samples_blended"] == n_eval.sum()
        else:
            assert abs(stats["samples_blended"] - n_eval.sum()) <= straddle.sum()
    return dev, img, stats


def test_render_config1_fp32():
    cfg = configs.config1()
    render_check(cfg)


def test_render_config1_fp32_with_termination():
    cfg = configs.config1(48, 48)
    cfg["scene"] = scene_dict((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, "f32", 77, sigma_scale=60.0)
    cfg["term_eps"] = 0.01
    cfg["bg"] = (1.0, 1.0, 1.0)
    render_check(cfg)


@pytest.mark.parametrize("wdtype", ["f16", "bf16"])
def test_render_config3_small(wdtype):
    cfg = configs.config3(96, 96, wdtype=wdtype)
    render_check(cfg)


def test_render_config3_fp32_weights():
    cfg = configs.config3(64, 64, wdtype="f32")
    render_check(cfg)


def test_render_config5_small():
    cfg = configs.config5(96, 54, net_res=8, occ_res=128)
    render_check(cfg)


def test_render_without_counts_equals_render_with_counts():
    """A frame whose second wave is known to be the last leaves out the sums that close a wave unless the caller asks
    for the frame's counts: the image must not depend on that."""
    cfg = configs.config3(80, 80)
    dev, _ = make_pair(cfg["scene"])
    o, d = cuda(cfg["rays_o"]), cuda(cfg["rays_d"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    plain = [dev.render(o, d, *args).cpu().numpy() for _ in range(3)]
    counted, st = dev.render(o, d, *args, want_stats=True)
    assert st["waves"] == 2
    for img in plain:
        np.testing.assert_array_equal(img, counted.cpu().numpy())
    np.testing.assert_array_equal(dev.render(o, d, *args).cpu().numpy(), plain[0])  # and again after a counted frame


def test_render_is_independent_of_wave_cut_and_deterministic():
    import paper_2103_13744_amd as kn
    cfg = configs.config3(80, 80)
    dev, _ = make_pair(cfg["scene"])
    o, d = cuda(cfg["rays_o"]), cuda(cfg["rays_d"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    imgs = []
    try:
        for first, slots in ((8, 8), (8, 8), (1, 1), (3, 5), (64, 64)):
            kn.set_render_params(first, slots)
            img, st = dev.render(o, d, *args, want_stats=True)
            imgs.append((img.cpu().numpy(), st))
    finally:
        kn.set_render_params(0, 0)
    for img, st in imgs[1:]:
        np.testing.assert_array_equal(img, imgs[0][0])
        assert st["samples_blended"] == imgs[0][1]["samples_blended"]
    assert imgs[2][1]["waves"] > imgs[0][1]["waves"] > imgs[4][1]["waves"] >= 1


def test_render_large_grid_code_paths():
    """Grids with too many networks for a counter each in LDS are grouped with separate histogram, offset and fill
    kernels and an LDS hash table; a second context whose limits force those paths on a small scene must produce the
    same image as the default context on the same scene."""
    import paper_2103_13744_amd as kn
    cfg = configs.config3(64, 64)
    dev, _ = make_pair(cfg["scene"])
    o, d = cuda(cfg["rays_o"]), cuda(cfg["rays_d"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    here = dev.render(o, d, *args).cpu().numpy()
    forced = kn.Context()
    # the path of large grids (counters in an LDS hash table), then the same with a table so small that most bins
    # overflow into the global-memory path
    for slots in (0, 16):
        forced.set_option(kn.OPT_GROUP_FUSED_MAX, 0)
        forced.set_option(kn.OPT_GROUP_HASH_SLOTS, slots)
        np.testing.assert_array_equal(dev.render(o, d, *args, ctx=forced).cpu().numpy(), here)
        np.testing.assert_array_equal(dev.render(o, d, *args).cpu().numpy(), here)          # the default context is untouched
    # the same paths under the sparse-grid and stratified variants of the marching kernel
    cfg = _sparse_cfg3("f16", 64, 64)
    dev, _ = make_pair(cfg["scene"])
    here = dev.render(o, d, *args, seed=3).cpu().numpy()
    forced.set_option(kn.OPT_GROUP_HASH_SLOTS, 0)
    np.testing.assert_array_equal(dev.render(o, d, *args, seed=3, ctx=forced).cpu().numpy(), here)
    with pytest.raises(kn.KnError):
        forced.set_option(kn.OPT_GROUP_HASH_SLOTS, 100)       # not a power of two
    with pytest.raises(kn.KnError):
        forced.set_option(99, 1)
    forced.close()


def test_bucket_over_more_blocks_than_one_scan_step():
    """The per-digit scan of the (digit, block) count table takes 1,024 blocks of 4,096 keys at a time: 5 M keys need two
    steps.  One pass (20 networks) and two (4,096).  Same counts, offsets and permutation as the oracle."""
    M = 5_000_011
    for res in ((5, 2, 2), (16, 16, 16)):
        N = int(np.prod(res))
        dev, _ = make_pair(scene_dict(res, (0, 0, 0), (1, 1, 1), 32, "f32", 1))
        ids = ks.rng(29 + N).integers(-1, N, size=M).astype(np.int32)
        c, o, p = oracle.bucket(ids, N)
        counts, offsets, perm = dev.bucket(cuda(ids))
        np.testing.assert_array_equal(counts.cpu().numpy(), c)
        np.testing.assert_array_equal(offsets.cpu().numpy(), o)
        np.testing.assert_array_equal(perm.cpu().numpy(), p)


def test_two_contexts_with_different_schedules_from_two_threads():
    """A context owns the wave schedule, the timing state and the mailboxes; a scene is immutable.  Two threads render
    the same scene through a context each, with different schedules and one of them timing its stages: the images are
    the bits of a one-at-a-time render, and neither context sees the other's settings."""
    import threading
    import torch
    import paper_2103_13744_amd as kn
    cfg = configs.config3(96, 96)
    dev, _ = make_pair(cfg["scene"])
    o, d = cuda(cfg["rays_o"]), cuda(cfg["rays_d"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    ref, ref_stats = dev.render(o, d, *args, want_stats=True)
    ref = ref.cpu().numpy()
    torch.cuda.synchronize()
    R = len(cfg["rays_o"])
    ctxs = [kn.Context(), kn.Context()]
    ctxs[0].set_render_params(8, 16, 2)
    ctxs[1].set_render_params(64, 512, 4)
    ctxs[1].profile_enable(1)
    results, waves, errors = [None, None], [None, None], []

    def worker(t):
        try:
            torch.cuda.set_device(0)
            st = torch.cuda.Stream()
            ws = torch.empty(dev.workspace_bytes(max_rays=R, ctx=ctxs[t]), dtype=torch.uint8, device="cuda")
            out = torch.empty((R, 3), dtype=torch.float32, device="cuda")
            with torch.cuda.stream(st):
                for _ in range(15):
                    _, stats = dev.render(o, d, *args, out=out, workspace=ws, ctx=ctxs[t], want_stats=True)
            st.synchronize()
            results[t], waves[t] = out.cpu().numpy(), stats["waves"]
        except Exception as e:       # (an exception in a thread would otherwise be lost)
            errors.append(e)

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(2)]
    for x in threads:
        x.start()
    for x in threads:
        x.join()
    assert not errors, errors
    np.testing.assert_array_equal(results[0], ref)
    np.testing.assert_array_equal(results[1], ref)
    assert waves[0] > ref_stats["waves"] >= waves[1]              # each ran its own schedule
    prof = ctxs[1].profile_read()
    assert prof["calls"] == 15 and prof["ms_mlp"] > 0 and ctxs[0].profile_read()["calls"] == 0
    # a workspace sized for one context's schedule is refused by a context whose schedule needs more
    small = torch.empty(dev.workspace_bytes(max_rays=R, ctx=ctxs[0]), dtype=torch.uint8, device="cuda")
    with pytest.raises(kn.KnError, match="workspace"):
        dev.render(o, d, *args, workspace=small, ctx=ctxs[1])
    for c in ctxs:
        c.close()


def test_scene_in_a_buffer_the_caller_lends():
    """kn_scene_bytes + the buffer argument of kn_scene_create: the scene's device data (packed weights, occupancy
    bits, skip field, table of a sparse grid) in caller memory, or, without a buffer, in memory the library allocates.
    Same image either way; buffers that are too small or misaligned are refused."""
    import ctypes as C
    import torch
    import paper_2103_13744_amd as kn
    from tests.util import device_weights
    cfg = _sparse_cfg3("f16", 48, 48)
    sc = cfg["scene"]
    o, d = cuda(cfg["rays_o"]), cuda(cfg["rays_d"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    w, occ, table = device_weights(sc["weights"], "f16"), cuda(sc["occupancy"]), cuda(sc["cell_net"])
    mk = lambda lend: kn.Scene(sc["res"], sc["aabb_min"], sc["aabb_max"], 32, w, occ, cell_net=table, lend_buffer=lend)
    lent, own = mk(True), mk(False)
    assert lent._buffer is not None and lent._buffer.numel() > w.numel() * 2 and own._buffer is None
    np.testing.assert_array_equal(lent.render(o, d, *args).cpu().numpy(), own.render(o, d, *args).cpu().numpy())
    # raw calls: size query, then refusals
    desc = kn.SceneDesc()
    desc.res[:] = sc["res"]
    desc.aabb_min[:] = sc["aabb_min"]
    desc.aabb_max[:] = sc["aabb_max"]
    desc.hidden, desc.L_pos, desc.L_dir, desc.wdtype = 32, 10, 4, kn.KN_F16
    desc.weights, desc.occupancy, desc.cell_net, desc.n_nets = w.data_ptr(), occ.data_ptr(), table.data_ptr(), w.shape[0]
    desc.occ_res[:] = list(occ.shape)
    need = C.c_int64()
    L = lent.L
    assert L.kn_scene_bytes(C.byref(desc), C.byref(need)) == 0 and need.value == lent._buffer.numel()
    buf = torch.empty(need.value + 256, dtype=torch.uint8, device="cuda")
    h = C.c_void_p()
    ctx = lent.ctx.h
    assert L.kn_scene_create(ctx, C.byref(desc), None, buf.data_ptr(), need.value - 1, C.byref(h)) == -3
    assert L.kn_scene_create(ctx, C.byref(desc), None, buf.data_ptr() + 64, need.value, C.byref(h)) == -3
    assert L.kn_scene_create(None, C.byref(desc), None, buf.data_ptr(), need.value, C.byref(h)) == -1
    assert L.kn_scene_create(ctx, C.byref(desc), None, buf.data_ptr(), need.value, C.byref(h)) == 0
    assert L.kn_scene_destroy(h) == 0


def test_render_network_grid_above_the_fused_grouping_limit():
    """21^3 = 9,261 networks: more than the grouping keeps a counter each for in LDS (hash tables instead), and not a
    multiple of four (the offset arrays then start at odd alignments)."""
    occ = ks.blob_occupancy((42, 42, 42), 5, 0.3, 881)
    sc = configs._scene((21, 21, 21), (-1, -1, -1), (1, 1, 1), 32, "f16", 882, sigma_scale=30.0, occ=occ)
    o, d = ks.camera_rays(40, 30, 40.0, 4.0, 20.0, 30.0)
    diag = 2.0 * math.sqrt(3.0)
    cfg = dict(scene=sc, rays_o=o, rays_d=d, t_near=4.0 - math.sqrt(3.0), step=diag / 128, K=128, term_eps=0.01,
               bg=(1.0, 1.0, 1.0), name="odd_large_grid_f16")
    _, _, stats = render_check(cfg)
    assert stats["samples_blended"] > 5000


def test_render_calls_in_flight_on_one_scene():
    """Calls on different streams (own workspace and output each) may overlap on one scene: every stream gets its
    own host mailbox.  Each result must equal the one-at-a-time image of the same rays."""
    import threading
    import torch
    cfg = configs.config3(96, 96)
    dev, _ = make_pair(cfg["scene"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    views = []
    for az in (10.0, 100.0, 190.0):
        o, d = configs.camera_rays(96, 96, 40.0, 4.0, az, 30.0)
        o, d = cuda(o), cuda(d)
        views.append((o, d, dev.render(o, d, *args).cpu().numpy()))
    torch.cuda.synchronize()
    R = 96 * 96
    results = [None] * len(views)

    def worker(t):
        st = torch.cuda.Stream()
        ws = torch.empty(dev.workspace_bytes(max_rays=R), dtype=torch.uint8, device="cuda")
        out = torch.empty((R, 3), dtype=torch.float32, device="cuda")
        with torch.cuda.stream(st):
            for _ in range(20):
                dev.render(views[t][0], views[t][1], *args, out=out, workspace=ws)
        st.synchronize()
        results[t] = out.cpu().numpy()

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(len(views))]
    for x in threads:
        x.start()
    for x in threads:
        x.join()
    for t, (_, _, ref) in enumerate(views):
        np.testing.assert_array_equal(results[t], ref)


def test_render_random_configurations_fp32():
    """Forty seeded random scenes: grid shapes (nested and not, with and without occupancy), boxes, cameras, K from 1 to
    600, termination thresholds and wave schedules (down to one sample per ray and wave, four slots per ray), fp32 so
    that the pixel bar is tight.  Every pixel against the oracle."""
    import torch
    import paper_2103_13744_amd as kn
    g = np.random.default_rng(20210313)
    try:
        for it in range(40):
            H = [32, 64][g.integers(0, 2)]
            nres = tuple(int(v) for v in g.integers(1, 7, size=3))
            if g.random() < 0.5:
                ores = tuple(int(n * 2 ** g.integers(0, 4)) for n in nres)
            else:
                ores = tuple(int(v) for v in g.integers(1, 40, size=3))
            lo = g.uniform(-2, 0, size=3)
            hi = lo + g.uniform(0.5, 3, size=3)
            seed = int(g.integers(1, 1 << 30))
            occ = ks.blob_occupancy(ores, int(g.integers(1, 6)), float(g.uniform(0.05, 0.6)), seed) if g.random() < 0.8 else None
            sc = configs._scene(nres, lo, hi, H, "f32", seed, sigma_scale=float(g.choice([1.0, 10.0, 100.0])), occ=occ)
            W, Hh = int(g.integers(1, 40)), int(g.integers(1, 40))
            diag = float(np.linalg.norm(hi - lo))
            rad = diag * g.uniform(0.8, 1.5)
            o, d = ks.camera_rays(W, Hh, float(g.uniform(20, 70)), rad, float(g.uniform(0, 360)), float(g.uniform(-60, 60)),
                                  center=tuple(0.5 * (lo + hi)))
            K = int(g.choice([1, 7, 32, 100, 257, 600]))
            t_near = max(rad - diag / 2, 0.0) * g.uniform(0.9, 1.0)
            step = diag / K * g.uniform(0.8, 1.3)
            eps = float(g.choice([0.0, 0.01, 0.1]))
            sched = (int(g.choice([0, 1, 3, 16, 48])), int(g.choice([0, 4, 32, 128])), int(g.choice([0, 2, 4, 32])))
            kn.set_render_params(*sched)
            dev, orc = make_pair(sc, threads=True)
            img, st = dev.render(cuda(o), cuda(d), t_near, step, K, eps, (0.3, 0.6, 0.9), want_stats=True)
            torch.cuda.synchronize()
            ref, n_eval, _, mg = orc.render(o, d, t_near, step, K, eps, (0.3, 0.6, 0.9))
            err = np.abs(img.cpu().numpy().astype(np.float64) - ref).max(axis=1)
            straddle = mg < 1e-3
            what = "case %d: H %d grid %s occupancy %s K %d eps %g schedule %s" % (it, H, nres, ores if occ is not None else None, K, eps, sched)
            assert err[~straddle].max(initial=0.0) <= 1e-4, what
            assert err[straddle].max(initial=0.0) <= 1e-4 + eps, what
            assert abs(st["samples_blended"] - n_eval.sum()) <= straddle.sum(), what
            assert st["samples_evaluated"] >= st["samples_blended"], what
    finally:
        kn.set_render_params(0, 0, 0)


def test_render_random_configurations_16bit():
    """Sixty seeded random scenes in fp16 and bf16: widths 32 and 64, grid shapes (nested and not, with and without
    occupancy, dense and sparse), midpoint and stratified lattices, K from 1 to 600, density units 1 to 100, termination
    thresholds, wave schedules.  Every pixel against the oracle at `pixel_bar`: 2e-2 wherever density unit x step is in
    the supported regime, the derived wider bar beyond it (K = 1 and K = 7 with steep density heads); straddling rays
    (MARGIN, times unit x step beyond 1) at + eps; the blended-sample count equal to the oracle's up to the straddlers."""
    import torch
    import paper_2103_13744_amd as kn
    g = np.random.default_rng(20210316)
    inside = outside = 0
    worst_inside = 0.0
    try:
        for it in range(60):
            wd = ["f16", "bf16"][it % 2]
            H = [32, 64][g.integers(0, 2)]
            nres = tuple(int(v) for v in g.integers(1, 7, size=3))
            if g.random() < 0.5:
                ores = tuple(int(n * 2 ** g.integers(0, 4)) for n in nres)
            else:
                ores = tuple(int(v) for v in g.integers(1, 40, size=3))
            lo = g.uniform(-2, 0, size=3)
            hi = lo + g.uniform(0.5, 3, size=3)
            seed = int(g.integers(1, 1 << 30))
            occ = ks.blob_occupancy(ores, int(g.integers(1, 6)), float(g.uniform(0.05, 0.6)), seed) if g.random() < 0.8 else None
            unit = float(g.choice([1.0, 10.0, 100.0]))
            sc = configs._scene(nres, lo, hi, H, wd, seed, sigma_scale=unit, occ=occ)
            if g.random() < 0.4:
                present = g.random(int(np.prod(nres))) < g.uniform(0.3, 1.0)
                present[0] = True
                sc = configs.sparsify(sc, present, seed + 5)
            W, Hh = int(g.integers(1, 40)), int(g.integers(1, 40))
            diag = float(np.linalg.norm(hi - lo))
            rad = diag * g.uniform(0.8, 1.5)
            o, d = ks.camera_rays(W, Hh, float(g.uniform(20, 70)), rad, float(g.uniform(0, 360)), float(g.uniform(-60, 60)),
                                  center=tuple(0.5 * (lo + hi)))
            K = int([1, 7, 32, 100, 257, 600][it % 6 if it < 12 else g.integers(0, 6)])      # K = 1 and K = 7 for both types at least
            t_near = max(rad - diag / 2, 0.0) * g.uniform(0.9, 1.0)
            step = diag / K * g.uniform(0.8, 1.3)
            eps = float(g.choice([0.0, 0.01, 0.1]))
            rseed = int(g.integers(0, 1 << 32)) if g.random() < 0.5 else None
            sched = (int(g.choice([0, 1, 3, 16, 48])), int(g.choice([0, 4, 32, 128])), int(g.choice([0, 2, 4, 32])))
            kn.set_render_params(*sched)
            dev, orc = make_pair(sc, threads=True)
            img, st = dev.render(cuda(o), cuda(d), t_near, step, K, eps, (0.3, 0.6, 0.9), want_stats=True, seed=rseed)
            torch.cuda.synchronize()
            ref, n_eval, _, mg = orc.render(o, d, t_near, step, K, eps, (0.3, 0.6, 0.9), seed=rseed)
            err = np.abs(img.cpu().numpy().astype(np.float64) - ref).max(axis=1)
            a = unit * float(np.float32(step))
            straddle = mg < MARGIN[wd] * max(1.0, a)      # the relative error of T is the summed density error x step
            bar = pixel_bar(wd, a)
            what = "case %d: %s H %d grid %s occupancy %s sparse %s K %d unit x step %.3g eps %g stratified %s schedule %s" % (
                it, wd, H, nres, ores if occ is not None else None, "cell_net" in sc, K, a, eps, rseed is not None, sched)
            log("  %s: bar %.3g, max err %.3g (straddlers: %d, there %.3g)" % (what, bar, err[~straddle].max(initial=0.0),
                                                                             straddle.sum(), err[straddle].max(initial=0.0)))
            assert err[~straddle].max(initial=0.0) <= bar, what
            assert err[straddle].max(initial=0.0) <= bar + eps, what
            assert abs(st["samples_blended"] - n_eval.sum()) <= straddle.sum(), what
            assert st["samples_evaluated"] >= st["samples_blended"], what
            if bar == TOL[wd]:
                inside += 1
                worst_inside = max(worst_inside, err[~straddle].max(initial=0.0))
            else:
                outside += 1
                assert np.mean(err > TOL[wd] + eps) <= 0.02, what       # rounding throws few pixels that far
    finally:
        kn.set_render_params(0, 0, 0)
    log("  inside the regime: %d cases, worst pixel %.3g; outside: %d cases" % (inside, worst_inside, outside))
    assert inside >= 30 and outside >= 5


def test_render_on_more_streams_than_mailboxes():
    """A context has eight host mailboxes, one per stream with a call in flight; a mailbox whose last call has
    reported is handed on to the next stream that needs one (calls that find none wait for their stream instead).
    Same image on every one of eleven streams, used one after the other and then all at once."""
    import torch
    cfg = configs.config3(48, 48)
    dev, _ = make_pair(cfg["scene"])
    o, d = cuda(cfg["rays_o"]), cuda(cfg["rays_d"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    ref = dev.render(o, d, *args).cpu().numpy()
    for _ in range(11):
        st = torch.cuda.Stream()
        st.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(st):
            img, stats = dev.render(o, d, *args, want_stats=True)
        st.synchronize()
        np.testing.assert_array_equal(img.cpu().numpy(), ref)
        assert stats["waves"] >= 1 and stats["samples_blended"] > 0
    # all at once: eleven calls enqueued back to back, each on its own stream with its own workspace and output
    R = o.shape[0]
    jobs = []
    for _ in range(11):
        st = torch.cuda.Stream()
        st.wait_stream(torch.cuda.current_stream())
        ws = torch.empty(dev.workspace_bytes(max_rays=R), dtype=torch.uint8, device="cuda")
        out = torch.empty((R, 3), dtype=torch.float32, device="cuda")
        jobs.append((st, ws, out))
    for _ in range(3):
        for st, ws, out in jobs:
            with torch.cuda.stream(st):
                dev.render(o, d, *args, out=out, workspace=ws)
    torch.cuda.synchronize()
    for _, _, out in jobs:
        np.testing.assert_array_equal(out.cpu().numpy(), ref)


def test_render_edge_cases():
    import torch
    cfg = configs.config3(16, 16)
    sc = dict(cfg["scene"])
    # nothing occupied -> background everywhere
    sc["occupancy"] = np.zeros((8, 8, 8), np.uint8)
    dev, _ = make_pair(sc)
    img = dev.render(cuda(cfg["rays_o"]), cuda(cfg["rays_d"]), cfg["t_near"], cfg["step"], cfg["K"], 0.01, (0.25, 0.5, 0.75))
    np.testing.assert_array_equal(img.cpu().numpy(), np.tile(np.float32([0.25, 0.5, 0.75]), (256, 1)))
    # zero rays, zero lattice points
    e = torch.empty((0, 3), dtype=torch.float32, device="cuda")
    assert dev.render(e, e, 1.0, 0.1, 16).shape == (0, 3)
    img = dev.render(cuda(cfg["rays_o"]), cuda(cfg["rays_d"]), cfg["t_near"], cfg["step"], 0, 0.0, (1, 0, 0))
    np.testing.assert_array_equal(img.cpu().numpy(), np.tile(np.float32([1, 0, 0]), (256, 1)))


def test_march_and_render_on_grids_that_do_not_nest():
    """Non-cubic box, network grid (3, 5, 2), occupancy grid (20, 17, 9): neither a multiple of the other nor of
    the skip block, so network cells cannot be derived from voxel coordinates by a shift."""
    occ = ks.blob_occupancy((20, 17, 9), 6, 0.2, 991)
    sc = configs._scene((3, 5, 2), (-1, 0, 0.5), (1, 2, 4.5), 32, "f32", 992, sigma_scale=5.0, occ=occ)
    o, d = ks.camera_rays(36, 28, 50.0, 6.0, 35.0, 25.0, center=(0.0, 1.0, 2.5))
    diag = math.sqrt(4 + 4 + 16)
    cfg = dict(scene=sc, rays_o=o, rays_d=d, t_near=6.0 - diag / 2, step=diag / 96, K=96, term_eps=0.01,
               bg=(0.2, 0.3, 0.4), name="non_nested_f32")
    dev, img, stats = render_check(cfg)
    assert stats["samples_blended"] > 1000
    orc = make_pair(sc)[1]
    out_k, cnt, _ = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], 96)
    out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
    for r in range(0, len(o), 3):
        want = orc.march(o[r], d[r], cfg["t_near"], cfg["step"], 96)
        assert cnt[r] == len(want), r
        np.testing.assert_array_equal(out_k[r, :cnt[r]], want)


# ------------------------------------------------------------------ occupancy extraction (Sec. 3.4)
def extraction_check(sc, occ_res, tau, sigma_unit=1.0, voxels=None):
    """Occupancy bytes against the oracle's.  The decision sigma > tau rests on a floating-point density, so a
    voxel with a probe whose oracle density lies within the density tolerance of tau may legitimately come out
    either way; all other voxels must agree exactly, and the undecided ones must be few."""
    import torch
    dev, orc = make_pair(sc, threads=True)
    got = dev.extract_occupancy(occ_res, tau)
    torch.cuda.synchronize()
    assert got.dtype == torch.uint8 and tuple(got.shape) == tuple(occ_res)
    got = got.cpu().numpy()
    assert set(np.unique(got)) <= {0, 1}
    if voxels is None:
        want, top, mg = orc.extract_occupancy(occ_res, tau)
    else:
        want, top, mg = orc.extract_occupancy(occ_res, tau, voxels=voxels)
        got = got.ravel()[voxels]
    # fp32: the density bar itself.  16-bit: a voxel with a probe within the rounding bound RHO of tau may differ from
    # the fp64 oracle; with 27 probes per voxel that is a third of the voxels in bf16, so those are checked against the
    # rounding model instead (Eq. 7 with 16-bit operands, oracle/lowprec.py), which the kernel follows eight times more
    # closely (test_matrix_core_kernel_follows_the_rounding_model): only voxels that are close to tau there as well
    # are left undecided.
    wd = sc["wdtype"]
    rel = 1e-4 if wd == "f32" else RHO[wd]
    tol = rel * sigma_unit * (1.0 + (0 if wd == "f32" else 1) * tau / sigma_unit)
    close = (mg <= tol).ravel()
    got, want = got.ravel(), want.ravel()
    np.testing.assert_array_equal(got[~close], want[~close])
    undecided = close
    if wd != "f32" and close.any():
        from oracle import lowprec
        idx = np.flatnonzero(close) if voxels is None else np.asarray(voxels)[close]
        m_occ, m_mg = lowprec.extract_occupancy(orc, sc["weights"], sc["hidden"], wd, occ_res, tau, voxels=idx)
        near = m_mg <= tol / 8
        np.testing.assert_array_equal(got[close][~near], m_occ[~near])
        undecided = np.zeros_like(close)
        undecided[np.flatnonzero(close)[near]] = True
    log("  extraction %s H=%d %s: %d voxels, %.1f %% marked, %d within the rounding bound of tau for the oracle, %d left "
        "undecided by the rounding model, %d of those differ from the oracle"
        % (wd, sc["hidden"], tuple(occ_res), want.size, 100 * want.mean(), close.sum(), undecided.sum(),
           (got != want)[undecided].sum()))
    assert 0.02 < want.mean() < 0.98
    assert undecided.mean() < {"f32": 0.003, "f16": 0.02, "bf16": 0.09}[wd]               # observed: 0.002, 0.01, 0.063
    assert (got != want)[undecided].sum() <= 0.25 * undecided.sum() + 2     # and even those mostly agree
    return dev, got.reshape(occ_res) if voxels is None else got


def median_density(sc, occ_res):
    """A threshold inside the range of a random scene's densities: the median over voxels of the largest probe."""
    orc = make_pair(sc, threads=True)[1]
    n = int(np.prod(occ_res))
    pick = np.arange(0, n, max(1, n // 2000), dtype=np.int64)
    return float(np.median(orc.extract_occupancy(occ_res, 0.0, voxels=pick)[1]))


@pytest.mark.parametrize("wdtype,H", [("f32", 32), ("f32", 64), ("f16", 32), ("bf16", 32), ("f16", 64), ("bf16", 64)])
def test_extract_occupancy_nested_grid(wdtype, H):
    # 16 voxels per network cell and axis do not fill whole 64-probe tiles (27 * 8^3 = 216 tiles, the last ragged)
    sc = scene_dict((2, 3, 2), (-1, -1, -1), (1, 1, 1), H, wdtype, 31, sigma_scale=20.0)
    res = (16, 24, 16)
    extraction_check(sc, res, median_density(sc, res), sigma_unit=20.0)


@pytest.mark.parametrize("wdtype", ["f32", "f16"])
def test_extract_occupancy_grids_that_do_not_nest(wdtype):
    # voxels straddle network cells: their probes are evaluated by different networks; one axis has fewer voxels
    # than cells, so some cells own no voxel at all
    sc = scene_dict((3, 5, 2), (-1, 0, 0.5), (1, 2, 4.5), 32, wdtype, 32, sigma_scale=20.0)
    res = (20, 3, 9)
    extraction_check(sc, res, median_density(sc, res), sigma_unit=20.0)


def test_extract_occupancy_threshold_cases_and_single_network():
    import torch
    sc = scene_dict((1, 1, 1), (0, 0, 0), (1, 1, 1), 32, "f16", 33, sigma_scale=20.0)
    dev, _ = make_pair(sc)
    assert int(dev.extract_occupancy((5, 7, 3), 1e30).sum()) == 0          # nothing is above
    assert int(dev.extract_occupancy((5, 7, 3), -1.0).sum()) == 105        # densities are >= 0: everything is above
    assert int(dev.extract_occupancy((1, 1, 1), -1.0).sum()) == 1
    extraction_check(sc, (12, 10, 14), median_density(sc, (12, 10, 14)), sigma_unit=20.0)
    # the result is what kn_scene_create takes as an occupancy grid
    occ = dev.extract_occupancy((8, 8, 8), median_density(sc, (8, 8, 8)))
    sc2 = dict(sc)
    sc2["occupancy"] = occ.cpu().numpy()
    cfg = configs.config3(16, 16)
    dev2, orc2 = make_pair(sc2)
    o, d = cfg["rays_o"] * 0.25 + 0.5, cfg["rays_d"]
    k, cnt, _ = dev2.march(cuda(o), cuda(d), 0.0, 0.02, 100)
    for r in range(0, len(o), 17):
        np.testing.assert_array_equal(k[r, :cnt[r]].cpu().numpy(), orc2.march(o[r], d[r], 0.0, 0.02, 100))


def test_error_statuses_of_extraction_and_layered_evaluation():
    """Bad arguments are turned into status codes on the host, before any launch."""
    import ctypes as C
    import torch
    import paper_2103_13744_amd as kn
    sc = scene_dict((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, "f16", 51)
    dev, _ = make_pair(sc)
    L, h = dev.L, dev.h
    occ = torch.empty(64, dtype=torch.uint8, device="cuda")
    ws = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    res = lambda *v: C.byref((C.c_int32 * 3)(*v))
    call = lambda r, tau, o, w, nb: L.kn_extract_occupancy(dev.ctx.h, h, None, r, tau, o, w, nb)
    assert call(res(4, 4, 4), 1.0, occ.data_ptr(), ws.data_ptr(), ws.numel()) == 0
    assert call(res(4, 0, 4), 1.0, occ.data_ptr(), ws.data_ptr(), ws.numel()) == -1          # empty resolution
    assert call(res(4, 4, 4), float("nan"), occ.data_ptr(), ws.data_ptr(), ws.numel()) == -1
    assert call(res(4, 4, 4), 1.0, None, ws.data_ptr(), ws.numel()) == -1                    # no output
    assert call(res(4, 4, 4), 1.0, occ.data_ptr(), None, 0) == -3                            # no workspace
    assert call(res(4, 4, 4), 1.0, occ.data_ptr(), ws.data_ptr(), 16) == -3                  # workspace too small
    assert call(res(4, 4, 4), 1.0, occ.data_ptr(), ws.data_ptr() + 4, ws.numel() - 4) == -3  # misaligned
    assert call(res(2048, 2048, 2048), 1.0, occ.data_ptr(), ws.data_ptr(), ws.numel()) == -2 # more than 2^31 - 1 voxels
    assert call(res(1300, 1300, 1200), 1.0, occ.data_ptr(), ws.data_ptr(), ws.numel()) == -2 # too many voxels per network
    pts = cuda(ks.uniform_points(10, 52))
    out_s, out_c = torch.empty(10, device="cuda"), torch.empty((10, 3), device="cuda")
    lay = lambda m, w, nb: L.kn_eval_grouped_layered(dev.ctx.h, h, None, pts.data_ptr(), pts.data_ptr(), m, out_s.data_ptr(),
                                                      out_c.data_ptr(), w, nb)
    assert lay(-1, ws.data_ptr(), ws.numel()) == -1
    assert lay(10, ws.data_ptr(), 64) == -3
    assert lay(10, None, 0) == -3
    torch.cuda.synchronize()


# ------------------------------------------------------------------ full-size workloads (sampled comparison)
def test_full_config2_sampled():
    cfg = configs.config2()
    M = len(cfg["points"])
    sel = ks.rng(99).choice(M, size=20_000, replace=False)
    check_eval(cfg["scene"], cfg["points"], cfg["dirs"], sample=sel)


def test_full_config4_sampled():
    cfg = configs.config4()
    M = len(cfg["points"])
    sel = ks.rng(98).choice(M, size=20_000, replace=False)
    check_eval(cfg["scene"], cfg["points"], cfg["dirs"], sample=sel)


def test_full_config3_sampled():
    cfg = configs.config3()
    R = len(cfg["rays_o"])
    sel = np.sort(ks.rng(97).choice(R, size=6000, replace=False))
    _, img, stats = render_check(cfg, sel=sel)
    assert stats["samples_blended"] > 1_000_000


def test_full_config5_sampled():
    cfg = configs.config5()
    R = len(cfg["rays_o"])
    sel = np.sort(ks.rng(96).choice(R, size=3000, replace=False))
    render_check(cfg, sel=sel)


def test_full_config3_stratified_sampled():
    cfg = configs.config3()
    cfg["seed"] = 2024
    cfg["name"] += "_stratified"
    sel = np.sort(ks.rng(95).choice(len(cfg["rays_o"]), size=5000, replace=False))
    _, img, stats = render_check(cfg, sel=sel)
    assert stats["samples_blended"] > 1_000_000


def test_full_sparse_grid_sampled():
    cfg = configs.config_sparse()
    sel = np.sort(ks.rng(94).choice(len(cfg["rays_o"]), size=6000, replace=False))
    _, img, stats = render_check(cfg, sel=sel)
    assert stats["samples_blended"] > 500_000


def test_full_extraction_config3_sampled():
    """Extraction at the size of the render workload (16^3 networks, 256^3 voxels, 4.5e8 probes), fp16; the oracle
    checks a sample of the voxels."""
    sc = configs.config3(8, 8)["scene"]
    res = (256, 256, 256)
    pick = np.unique(ks.rng(77).integers(0, 256 ** 3, size=1500)).astype(np.int64)
    orc = make_pair(sc, threads=True)[1]
    tau = float(np.median(orc.extract_occupancy(res, 0.0, voxels=pick[:300])[1]))
    extraction_check(sc, res, tau, sigma_unit=100.0, voxels=pick)


# ------------------------------------------------------------------ sparse network grids (Sec. 5)
def _sparse_cfg3(wdtype, width=64, height=64, keep=0.6, seed=31):
    cfg = configs.config3(width, height, wdtype=wdtype)
    n = int(np.prod(cfg["scene"]["res"]))
    cfg["scene"] = configs.sparsify(cfg["scene"], np.random.default_rng(seed).random(n) < keep, seed + 1)
    cfg["name"] += "_sparse"
    return cfg


@pytest.mark.parametrize("wdtype", ["f32", "f16"])
def test_sparse_grid_ids_eval_march_render(wdtype):
    cfg = _sparse_cfg3(wdtype)
    sc = cfg["scene"]
    log("sparse grid", wdtype, "networks", len(sc["weights"]), "of", sc["cell_net"].size, "cells")
    g = ks.rng(91)
    M = 150_001
    pts = (-1.05 + g.random((M, 3)) * 2.1).astype(np.float32)
    dev = check_eval(sc, pts, ks.sphere_dirs(M, 92), sample=np.arange(0, M, 7), sigma_unit=100.0)
    _, orc = make_pair(sc)
    ids = orc.cell_ids(pts)
    assert (ids < 0).mean() > 0.3 and len(np.unique(ids)) == len(sc["weights"]) + 1
    np.testing.assert_array_equal(dev.cell_ids(cuda(pts)).cpu().numpy(), ids)
    # marching: the kept lattice points, bit-exact
    o, d = cfg["rays_o"], cfg["rays_d"]
    out_k, cnt, _ = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], cfg["K"])
    out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
    total = 0
    for r in range(0, len(o), 3):
        want = orc.march(o[r], d[r], cfg["t_near"], cfg["step"], cfg["K"])
        assert cnt[r] == len(want), r
        np.testing.assert_array_equal(out_k[r, :cnt[r]], want)
        total += len(want)
    assert total > 3000
    render_check(cfg)


def test_sparse_grid_entries_out_of_range_mean_no_network():
    import torch
    import paper_2103_13744_amd as kn
    cfg = _sparse_cfg3("f32", 8, 8)
    sc = cfg["scene"]
    bad = sc["cell_net"].copy()
    gone = bad < 0
    bad[gone] = np.where(np.random.default_rng(3).random(int(gone.sum())) < 0.5, len(sc["weights"]), -9)
    dev, orc = make_pair(dict(sc, cell_net=bad))
    pts = (-1 + ks.rng(5).random((20_000, 3)) * 2).astype(np.float32)
    np.testing.assert_array_equal(dev.cell_ids(cuda(pts)).cpu().numpy(), orc.cell_ids(pts))
    np.testing.assert_array_equal(orc.cell_ids(pts), make_pair(sc)[1].cell_ids(pts))
    # descriptor checks
    w = torch.zeros((4, kn.params_per_net(32)), device="cuda")
    with pytest.raises(kn.KnError, match="one entry per cell"):
        kn.Scene((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, w, cell_net=torch.zeros(7, dtype=torch.int32, device="cuda"))
    with pytest.raises(kn.KnError, match="unsupported"):
        kn.Scene((300, 300, 300), (0, 0, 0), (1, 1, 1), 32, w, cell_net=torch.zeros(27_000_000, dtype=torch.int32, device="cuda"))


@pytest.mark.parametrize("wdtype", ["f32", "bf16"])
def test_sparse_grid_extraction(wdtype):
    sc = scene_dict((6, 5, 7), (-1, -1, -1), (1, 1, 1), 32, wdtype, 41, sigma_scale=5.0)
    sc = configs.sparsify(sc, np.random.default_rng(8).random(6 * 5 * 7) < 0.7, 9)
    for occ_res in ((24, 20, 28), (25, 23, 30)):          # nested, and not
        tau = median_density(sc, occ_res)
        dev, got = extraction_check(sc, occ_res, max(tau, 0.05), sigma_unit=5.0)
        if occ_res != (24, 20, 28):
            continue          # (a voxel that straddles cell faces can reach a network cell through a corner)
        # nested grids: a voxel whose cell has no network is never marked
        _, orc = make_pair(sc)
        ctr = (np.stack(np.meshgrid(*[np.arange(r) + 0.5 for r in occ_res], indexing="ij"), -1) / np.array(occ_res) * 2 - 1)
        ids = orc.cell_ids(ctr.reshape(-1, 3).astype(np.float32)).reshape(occ_res)
        assert (ids < 0).sum() > 1000 and not got[ids < 0].any()


def test_sparse_grid_with_more_cells_than_a_dense_grid_may_have():
    cfg = configs.config_sparse(96, 96)
    sc = cfg["scene"]
    log("sparse 48^3:", len(sc["weights"]), "networks in", sc["cell_net"].size, "cells")
    assert sc["cell_net"].size > 65535 and 1000 < len(sc["weights"]) < 65535
    dev, img, stats = render_check(cfg)
    assert stats["samples_blended"] > 10_000
    # networks only where something is occupied: the table drops no sample, so the march equals the dense rule
    _, orc = make_pair(sc)
    o, d = cfg["rays_o"], cfg["rays_d"]
    out_k, cnt, _ = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], cfg["K"])
    out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
    for r in range(0, len(o), 97):
        np.testing.assert_array_equal(out_k[r, :cnt[r]], orc.march(o[r], d[r], cfg["t_near"], cfg["step"], cfg["K"]))
    g = ks.rng(93)
    pts = (-1 + g.random((100_000, 3)) * 2).astype(np.float32)
    check_eval(sc, pts, ks.sphere_dirs(100_000, 94), sample=np.arange(0, 100_000, 11), sigma_unit=100.0)


# ------------------------------------------------------------------ stratified sampling (Sec. 3.4)
def test_stratified_march_bit_exact_and_resumable():
    cfg = configs.config3(40, 40)
    dev, orc = make_pair(cfg["scene"])
    o, d, K = cfg["rays_o"], cfg["rays_d"], cfg["K"]
    differ = 0
    for seed in (0, 7, 2 ** 32 - 1):
        out_k, cnt, nxt = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], K, seed=seed)
        out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
        total = 0
        for r in range(0, len(o), 2):
            want = orc.march_stratified(o[r], d[r], cfg["t_near"], cfg["step"], K, seed, r)
            assert cnt[r] == len(want), (seed, r)
            np.testing.assert_array_equal(out_k[r, :cnt[r]], want)
            differ += want.tolist() != orc.march(o[r], d[r], cfg["t_near"], cfg["step"], K).tolist()
            total += len(want)
        assert total > 2500
    assert differ > 100           # the draws do move lattice points across voxel faces
    seed = 7
    kb = cuda(np.zeros(len(o), np.int32))
    got = [[] for _ in range(len(o))]
    for _ in range(K):
        ck, cc, kb = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], K, S=6, k_begin=kb, seed=seed)
        ck, cc = ck.cpu().numpy(), cc.cpu().numpy()
        for r in np.nonzero(cc)[0]:
            got[r] += ck[r, :cc[r]].tolist()
        if cc.sum() == 0:
            break
    out_k, cnt, _ = dev.march(cuda(o), cuda(d), cfg["t_near"], cfg["step"], K, seed=seed)
    out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
    for r in range(0, len(o), 5):
        assert got[r] == out_k[r, :cnt[r]].tolist()


def test_stratified_march_without_grid_and_coarse_steps():
    # no occupancy grid; steps much longer than a skip block would be; rays that graze and miss the box
    cfg = configs.config1(24, 24)
    dev, orc = make_pair(cfg["scene"])
    o, d = cfg["rays_o"], cfg["rays_d"]
    for K, seed in ((32, 1), (5, 2), (1, 3)):
        step = cfg["step"] * 32 / K
        out_k, cnt, _ = dev.march(cuda(o), cuda(d), cfg["t_near"], step, K, seed=seed)
        out_k, cnt = out_k.cpu().numpy(), cnt.cpu().numpy()
        for r in range(len(o)):
            want = orc.march_stratified(o[r], d[r], cfg["t_near"], step, K, seed, r)
            assert cnt[r] == len(want)
            np.testing.assert_array_equal(out_k[r, :cnt[r]], want)


@pytest.mark.parametrize("wdtype,H", [("f32", 32), ("f16", 32), ("bf16", 64), ("f32", 64)])
def test_stratified_render(wdtype, H):
    if H == 32:
        cfg = configs.config3(72, 72, wdtype=wdtype)
    else:
        cfg = configs.config5(64, 40, net_res=8, occ_res=128, wdtype=wdtype)
    cfg["seed"] = 1234
    cfg["name"] += "_stratified"
    dev, img, _ = render_check(cfg)
    mid = dev.render(cuda(cfg["rays_o"]), cuda(cfg["rays_d"]), cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"],
                     cfg["bg"]).cpu().numpy()
    assert np.abs(mid - img).max() > 0.01            # not the midpoint picture


def test_stratified_render_without_termination_fp32():
    cfg = configs.config1(48, 48)
    cfg["seed"] = 99
    render_check(cfg)


def test_stratified_render_is_seeded_and_independent_of_the_wave_cut():
    import paper_2103_13744_amd as kn
    cfg = configs.config3(80, 80)
    dev, _ = make_pair(cfg["scene"])
    o, d = cuda(cfg["rays_o"]), cuda(cfg["rays_d"])
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    try:
        imgs = []
        for first, slots, growth in ((0, 0, 0), (4, 32, 2), (1, 8, 3), (512, 512, 2)):
            kn.set_render_params(first, slots, growth)
            imgs.append(dev.render(o, d, *args, seed=5).cpu().numpy())
            again = dev.render(o, d, *args, seed=5).cpu().numpy()
            np.testing.assert_array_equal(imgs[-1], again)
        for im in imgs[1:]:
            np.testing.assert_array_equal(im, imgs[0])
        other = dev.render(o, d, *args, seed=6).cpu().numpy()
        assert np.abs(other - imgs[0]).max() > 0.01
    finally:
        kn.set_render_params(0, 0, 0)


def test_stratified_render_on_a_sparse_grid_and_on_grids_that_do_not_nest():
    cfg = _sparse_cfg3("f32", 56, 56)
    cfg["seed"] = 77
    render_check(cfg)
    occ = ks.blob_occupancy((50, 45, 61), 12, 0.15, 5)
    cfg = configs.config3(48, 48, wdtype="f32")
    cfg["scene"] = scene_dict((5, 8, 5), (-1, -1, -1), (1, 1, 1), 32, "f32", 13, occ=occ, sigma_scale=60.0)
    cfg["seed"] = 78
    render_check(cfg)


def test_sparse_and_stratified_edge_cases():
    import torch
    import paper_2103_13744_amd as kn
    # a grid in which no cell has a network: everything is empty space
    sc = scene_dict((3, 2, 4), (-1, -1, -1), (1, 1, 1), 32, "f32", 5, sigma_scale=50.0)
    sc = dict(sc, weights=sc["weights"][:1].copy(), cell_net=np.full(24, -1, np.int32))
    dev, orc = make_pair(sc)
    cfg = configs.config1(12, 12)
    o, d = ks.camera_rays(12, 12, 40.0, 4.0, 30.0, 20.0)
    bg = (0.2, 0.4, 0.6)
    for seed in (None, 3):
        img, st = dev.render(cuda(o), cuda(d), 2.0, 0.05, 80, 0.01, bg, want_stats=True, seed=seed)
        assert st["samples_evaluated"] == 0 and np.allclose(img.cpu().numpy(), np.tile(np.float32(bg), (144, 1)))
        assert np.allclose(orc.render(o, d, 2.0, 0.05, 80, 0.01, bg, seed=seed)[0], np.tile(bg, (144, 1)))
    pts = (-1 + ks.rng(2).random((5000, 3)) * 2).astype(np.float32)
    sg, rgb, ids, counts, perm = dev.eval_grouped(cuda(pts), cuda(ks.sphere_dirs(5000, 3)), want_aux=True)
    assert (ids.cpu().numpy() == -1).all() and not sg.cpu().numpy().any() and not rgb.cpu().numpy().any()
    assert counts.cpu().numpy().tolist() == [0, 5000]
    assert not dev.extract_occupancy((9, 8, 12), 0.0).cpu().numpy().any()
    # stratified rendering with no lattice points, one lattice point, no rays
    dev, orc = make_pair(cfg["scene"])
    o, d = cfg["rays_o"], cfg["rays_d"]
    img = dev.render(cuda(o), cuda(d), cfg["t_near"], cfg["step"], 0, 0.0, bg, seed=1).cpu().numpy()
    assert np.allclose(img, np.tile(np.float32(bg), (len(o), 1)))
    img = dev.render(cuda(o), cuda(d), cfg["t_near"] + 0.5, 0.3, 1, 0.0, bg, seed=2).cpu().numpy()
    ref = orc.render(o, d, cfg["t_near"] + 0.5, 0.3, 1, 0.0, bg, seed=2)[0]
    assert np.abs(img - ref).max() < 1e-4 and np.abs(ref - np.array(bg)).max() > 1e-3
    empty = torch.empty((0, 3), dtype=torch.float32, device="cuda")
    assert dev.render(empty, empty, 1.0, 0.1, 8, 0.0, bg, seed=3).shape == (0, 3)
    k, c, nx = dev.march(cuda(o[:5]), cuda(d[:5]), cfg["t_near"], cfg["step"], 0, S=4, seed=4)
    assert (c.cpu().numpy() == 0).all() and (k.cpu().numpy() == -1).all()
