"""Pins of the CPU oracle against things other than itself: constants the paper prints, closed
forms, invariants, library routines and brute force.  No GPU needed."""
import math
from fractions import Fraction

import numpy as np
import pytest

import kn_synth as ks
import oracle
from oracle import OracleScene


def zero_net(H=32, n=1):
    return np.zeros((n, ks.params_per_net(H)), np.float32)


def unit_scene(weights, res=(1, 1, 1), H=32, occ=None, lo=(0, 0, 0), hi=(1, 1, 1)):
    return OracleScene(res, lo, hi, H, weights, occ)


# ------------------------------------------------------------------ printed constants
def test_parameter_count_is_the_papers_6k(golden):
    g = golden("paper_constants.txt")
    assert g["hidden_layers"] == 4 and g["hidden_units"] == 32
    p = oracle.params_per_net(32)
    assert p == 6212 and round(p / 1000) == g["params_per_net_thousands"]
    # four hidden layers: L1, L2, L4 output H; L3 outputs H + 1 (density + feature); output layer 3
    shapes = ks.layer_shapes(32)
    assert [o for _, o in shapes] == [32, 32, 33, 32, 3] and shapes[0][0] == 63 and shapes[3][0] == 59
    assert oracle.params_per_net(64) == 18564
    # whole-scene storage at the largest grid stays under the paper's bound in fp16 (Sec. 5)
    assert g["max_networks"] * p * 2 / 1e6 < g["storage_mb_upper"]


# ------------------------------------------------------------------ positional encoding
def test_posenc_dims_and_identities():
    p = np.array([0.3, -0.7, 0.9], np.float32)
    for L, dims in ((10, 63), (4, 27)):
        e = oracle.posenc(p, L)
        assert e.shape == (dims,)
        np.testing.assert_array_equal(e[:3], p.astype(np.float64))
        s = e[3:].reshape(L, 2, 3)[:, 0]
        c = e[3:].reshape(L, 2, 3)[:, 1]
        np.testing.assert_allclose(s * s + c * c, 1.0, atol=1e-12)
        # frequency doubles from one block to the next and there is no factor pi:
        np.testing.assert_allclose(s[1:], 2 * s[:-1] * c[:-1], atol=1e-9)
        np.testing.assert_allclose(c[1:], 1 - 2 * s[:-1] ** 2, atol=1e-9)
        np.testing.assert_allclose(s[0], np.sin(p.astype(np.float64)), atol=1e-15)


def test_posenc_at_zero_and_known_angle():
    e = oracle.posenc(np.zeros(3, np.float32), 10)
    assert np.all(e[:3] == 0)
    np.testing.assert_array_equal(e[3:].reshape(10, 2, 3)[:, 0], 0.0)
    np.testing.assert_array_equal(e[3:].reshape(10, 2, 3)[:, 1], 1.0)
    x = np.float32(math.pi / 6)
    e = oracle.posenc(np.array([x, 0, 0], np.float32), 2)
    assert abs(e[3] - 0.5) < 1e-7 and abs(e[6] - math.sqrt(3) / 2) < 1e-7        # sin, cos of pi/6
    assert abs(e[9] - math.sqrt(3) / 2) < 1e-7 and abs(e[12] - 0.5) < 1e-7       # sin, cos of pi/3


# ------------------------------------------------------------------ spatial binning (Eq. 6)
@pytest.mark.parametrize("res", [(2, 2, 2), (3, 4, 5), (10, 16, 10), (16, 16, 16)])
def test_grid_index_matches_exact_interval_search(res):
    lo, hi = (-1.0, 0.0, 0.5), (1.0, 2.0, 4.5)
    sc = OracleScene(res, lo, hi, 32, zero_net(n=int(np.prod(res))))
    g = ks.rng(5)
    pts = (np.array(lo) + g.random((4000, 3)) * (np.array(hi) - np.array(lo))).astype(np.float32)
    ids = sc.cell_ids(pts)
    checked = 0
    for p, got in zip(pts[:1500], ids[:1500]):
        idx = []
        near_face = False
        for a in range(3):
            # exact rational position in cell units; brute-force search over all cells of the axis
            u = (Fraction(float(p[a])) - Fraction(lo[a])) * res[a] / (Fraction(hi[a]) - Fraction(lo[a]))
            cells = [i for i in range(res[a]) if i <= u < i + 1]
            assert len(cells) == 1
            idx.append(cells[0])
            near_face |= min(u - cells[0], cells[0] + 1 - u) < Fraction(1, 10 ** 4)
        if near_face:      # fp32 rounding may legitimately move such a point across the face
            continue
        checked += 1
        assert got == (idx[0] * res[1] + idx[1]) * res[2] + idx[2]      # x slowest, z fastest
    assert checked > 1400


def test_grid_index_faces_and_outside():
    sc = unit_scene(zero_net(n=8), res=(2, 2, 2))
    assert sc.grid_index([0.0, 0.0, 0.0]) == 0
    assert sc.grid_index([0.5, 0.0, 0.0]) == 4          # lower face of the second x cell
    assert sc.grid_index([0.0, 0.0, 0.5]) == 1          # z is the fastest axis
    assert sc.grid_index([0.0, 0.5, 0.0]) == 2
    assert sc.grid_index([0.75, 0.75, 0.75]) == 7
    for bad in ([1.0, 0.2, 0.2], [-1e-6, 0.2, 0.2], [0.2, 1.5, 0.2], [0.2, 0.2, np.nan], [0.2, np.inf, 0.2]):
        assert sc.grid_index(bad) == -1                 # upper face excluded, outside, non-finite


# ------------------------------------------------------------------ bucketing
def test_bucket_equals_stable_argsort():
    g = ks.rng(11)
    N = 37
    ids = g.integers(-1, N, size=5000).astype(np.int32)
    counts, offsets, perm = oracle.bucket(ids, N)
    key = np.where(ids < 0, N, ids)
    np.testing.assert_array_equal(perm, np.argsort(key, kind="stable").astype(np.int32))
    np.testing.assert_array_equal(counts, np.bincount(key, minlength=N + 1))
    np.testing.assert_array_equal(offsets, np.concatenate([[0], np.cumsum(counts)]))
    assert offsets[-1] == len(ids) and sorted(perm.tolist()) == list(range(len(ids)))
    c0, o0, p0 = oracle.bucket(np.zeros(0, np.int32), 4)
    assert c0.sum() == 0 and o0[-1] == 0 and len(p0) == 0


# ------------------------------------------------------------------ the tiny MLP (Eq. 7, Sec. 3.2)
def dense_reference(w, H, x, d):
    """The same network through numpy float64 matrix products (library routine reduction)."""
    (W1, b1), (W2, b2), (W3, b3), (W4, b4), (W5, b5) = [(W[0].astype(np.float64), b[0].astype(np.float64))
                                                         for W, b in ks.layer_views(w, H)]

    def enc(p, L):
        p = np.asarray(p, np.float32).astype(np.float64)
        parts = [p]
        for k in range(L):
            parts += [np.sin(2.0 ** k * p), np.cos(2.0 ** k * p)]
        return np.concatenate(parts)
    h = np.maximum(enc(x, 10) @ W1 + b1, 0)
    h = np.maximum(h @ W2 + b2, 0)
    o3 = h @ W3 + b3
    h4 = np.maximum(np.concatenate([o3[1:], enc(d, 4)]) @ W4 + b4, 0)
    return max(o3[0], 0.0), 1 / (1 + np.exp(-(h4 @ W5 + b5)))


@pytest.mark.parametrize("H", [32, 64])
def test_single_cell_grid_is_one_dense_mlp(H):
    w = ks.kaiming_weights(1, H, 77)
    sc = unit_scene(w, H=H)
    g = ks.rng(3)
    pts = g.random((50, 3)).astype(np.float32)
    dirs = ks.sphere_dirs(50, 4)
    sg, rgb, ids = sc.eval_points(pts, dirs)
    assert np.all(ids == 0)
    for i in range(50):
        s_ref, c_ref = dense_reference(w, H, pts[i], dirs[i])
        assert abs(sg[i] - s_ref) < 1e-12 and np.abs(rgb[i] - c_ref).max() < 1e-12


def probe_net(H=32):
    w = zero_net(H)
    return w, ks.layer_views(w, H)


def test_mlp_wiring_probes_have_closed_forms():
    x = np.array([0.3, 0.1, 0.2], np.float32)
    d = np.array([0.6, 0.0, 0.8], np.float32)
    xd, dd = x.astype(np.float64), d.astype(np.float64)
    sig = lambda v: 1 / (1 + math.exp(-v))
    # (a) position feature "sin(2^3 * y)" (index 3 + 6*3 + 1) -> h1[5] -> h2[7] -> density (x2) and
    #     feature 2 -> h4[9] -> green.
    w, ((W1, b1), (W2, b2), (W3, b3), (W4, b4), (W5, b5)) = probe_net()
    W1[0, 3 + 18 + 1, 5] = 1
    W2[0, 5, 7] = 1
    W3[0, 7, 0] = 2
    W3[0, 7, 1 + 2] = 1
    W4[0, 2, 9] = 1
    W5[0, 9, 1] = 3
    s, c = unit_scene(w).mlp(0, x, d)
    v = math.sin(8 * xd[1])
    assert v > 0 and abs(s - 2 * v) < 1e-12
    np.testing.assert_allclose(c, [0.5, sig(3 * v), 0.5], atol=1e-12)
    # (b) the cos block follows the sin block inside each frequency: cos(2^0 * z) is index 3 + 3 + 2
    w, ((W1, b1), (W2, b2), (W3, b3), (W4, b4), (W5, b5)) = probe_net()
    W1[0, 8, 0] = 1
    W2[0, 0, 0] = 1
    W3[0, 0, 0] = 1
    s, _ = unit_scene(w).mlp(0, x, d)
    assert abs(s - math.cos(xd[2])) < 1e-12
    # (c) the identity part of the encoding comes first, and the global (not cell-local) x is encoded
    w8 = zero_net(n=8)
    lv = ks.layer_views(w8, 32)
    lv[0][0][:, 0, 0] = 1          # h1[0] = x_x
    lv[1][0][:, 0, 0] = 1
    lv[2][0][:, 0, 0] = 1          # sigma = x_x
    sc8 = unit_scene(w8, res=(2, 2, 2))
    sg, _, ids = sc8.eval_points(np.array([[0.75, 0.1, 0.1]], np.float32), d[None])
    assert ids[0] == 4 and abs(sg[0] - 0.75) < 1e-12
    # (d) direction enters the last hidden layer after the H feature inputs: sin(2^1 * d_z) is
    #     index 3 + 6 + 2 of gamma(d), i.e. row H + 11 of W4; the density does not see it
    w, ((W1, b1), (W2, b2), (W3, b3), (W4, b4), (W5, b5)) = probe_net()
    W4[0, 32 + 11, 4] = 1
    W5[0, 4, 2] = -2
    s, c = unit_scene(w).mlp(0, x, d)
    assert s == 0
    np.testing.assert_allclose(c, [0.5, 0.5, sig(-2 * math.sin(2 * dd[2]))], atol=1e-12)
    # (e) no activation on the feature vector (a negative feature survives), ReLU on the density
    w, ((W1, b1), (W2, b2), (W3, b3), (W4, b4), (W5, b5)) = probe_net()
    b3[0, 1 + 6] = -5
    b3[0, 0] = -3
    W4[0, 6, 0] = -1
    W5[0, 0, 0] = 1
    s, c = unit_scene(w).mlp(0, x, d)
    assert s == 0 and abs(c[0] - sig(5.0)) < 1e-12
    # (f) ReLU after the first, second and last hidden layer: a negative pre-activation is cut
    for layer in (0, 1, 3):
        w, lv = probe_net()
        lv[layer][1][0, 0] = -1.0            # bias of unit 0 of that layer
        nxt = {0: (1, (0, 0)), 1: (2, (0, 0)), 3: (4, (0, 0))}[layer]
        lv[nxt[0]][0][0, nxt[1][0], nxt[1][1]] = 1.0
        if layer == 0:
            lv[2][0][0, 0, 0] = 1.0
        s, c = unit_scene(w).mlp(0, x, d)
        assert s == 0 and abs(c[0] - 0.5) < 1e-12
    # (g) saturation of the sigmoid and bias-only colour
    w, lv = probe_net()
    lv[4][1][0, :] = [40, -40, 0]
    _, c = unit_scene(w).mlp(0, x, d)
    np.testing.assert_allclose(c, [1, 0, 0.5], atol=1e-15)


def test_gamma_zero_gives_bias_plus_cos_rows():
    w = ks.kaiming_weights(1, 32, 5)
    lv = ks.layer_views(w, 32)
    for l in (1, 2, 3, 4):
        lv[l][0][...] = 0
        lv[l][1][...] = 0
    # route h1 unit j to the density one at a time
    W1, b1 = lv[0][0][0].astype(np.float64), lv[0][1][0].astype(np.float64)
    cos_rows = [3 + 6 * k + 3 + a for k in range(10) for a in range(3)]
    expect = np.maximum(b1 + W1[cos_rows].sum(0), 0)
    for j in (0, 13, 31):
        lv[1][0][0, :, :] = 0
        lv[1][0][0, j, 0] = 1
        lv[2][0][0, 0, 0] = 1
        s, _ = unit_scene(w, lo=(-1, -1, -1), hi=(1, 1, 1)).mlp(0, [0, 0, 0], [0, 0, 1])
        assert abs(s - expect[j]) < 1e-12


def test_identical_cells_equal_single_cell_and_order_is_irrelevant():
    w1 = ks.kaiming_weights(1, 32, 9)
    one = unit_scene(w1)
    many = unit_scene(np.repeat(w1, 27, axis=0), res=(3, 3, 3))
    pts = ks.uniform_points(300, 1)
    dirs = ks.sphere_dirs(300, 2)
    s1, c1, _ = one.eval_points(pts, dirs)
    s2, c2, ids = many.eval_points(pts, dirs)
    np.testing.assert_array_equal(s1, s2)
    np.testing.assert_array_equal(c1, c2)
    assert len(np.unique(ids)) == 27
    p = ks.rng(8).permutation(300)
    s3, c3, ids3 = many.eval_points(pts[p], dirs[p])
    np.testing.assert_array_equal(s3, s2[p])
    np.testing.assert_array_equal(c3, c2[p])
    np.testing.assert_array_equal(ids3, ids[p])


def test_each_point_uses_the_network_of_its_cell():
    # network n has density bias n + 1 and nothing else: sigma reveals which network answered
    res = (3, 4, 5)
    w = zero_net(n=60)
    ks.layer_views(w, 32)[2][1][:, 0] = np.arange(60) + 1
    sc = unit_scene(w, res=res, lo=(-1, 0, 0.5), hi=(1, 2, 4.5))
    pts = ks.uniform_points(2000, 3, lo=(-1, 0, 0.5), hi=(1, 2, 4.5))
    sg, _, ids = sc.eval_points(pts, ks.sphere_dirs(2000, 4))
    np.testing.assert_array_equal(sg, ids + 1.0)
    out = np.array([[1.5, 1, 1], [0, -0.1, 1]], np.float32)
    sg, rgb, ids = sc.eval_points(out, ks.sphere_dirs(2, 4))
    assert np.all(ids == -1) and np.all(sg == 0) and np.all(rgb == 0)


# ------------------------------------------------------------------ compositing (Eq. 2-4) and ERT
def test_alpha_blend_worked_example(golden):
    g = golden("alpha_blend_example.txt")
    rgb = np.array([[1, 1, 1], [0, 0, 0], [1, 1, 1]], float)
    out, T, used, _ = oracle.composite([g["sigma"]] * 3, rgb, g["delta"])
    np.testing.assert_allclose(out, g["c_hat"], atol=1e-15)
    assert abs(T - g["T_end"]) < 1e-15 and used == 3
    out, _, _, _ = oracle.composite([g["sigma"]] * 3, rgb, g["delta"], bg=(1, 1, 1))
    np.testing.assert_allclose(out, g["c_hat_bg1"], atol=1e-15)
    # early termination with constant alpha = 1/2
    n = 20
    out, T, used, _ = oracle.composite([g["sigma"]] * n, np.ones((n, 3)), 1.0, eps=0.01)
    assert used == g["ert_samples_at_eps_0p01"] and abs(T - 2.0 ** -7) < 1e-15
    np.testing.assert_allclose(out, 1 - 2.0 ** -7, atol=1e-15)


def test_constant_density_gives_exponential_transmittance():
    g = ks.rng(2)
    for _ in range(5):
        sigma, step, n = g.uniform(0.1, 5), g.uniform(0.01, 0.2), int(g.integers(1, 60))
        col = g.random(3)
        bg = g.random(3)
        out, T, used, _ = oracle.composite([sigma] * n, np.tile(col, (n, 1)), step, bg=bg)
        Texp = math.exp(-sigma * step * n)
        assert abs(T - Texp) < 1e-12 and used == n
        np.testing.assert_allclose(out, col * (1 - Texp) + bg * Texp, atol=1e-12)


def test_composite_with_a_delta_per_sample():
    g = ks.rng(61)
    n = 50
    sg, col, delta = g.uniform(0, 8, n), g.random((n, 3)), g.uniform(0.01, 0.2, n)
    bg = (0.2, 0.4, 0.6)
    out, T, used, _ = oracle.composite(sg, col, delta, 0.0, bg)
    # transmittance: exp(-sum sigma_i delta_i); a uniform colour c gives c (1 - T) + T bg whatever the deltas
    assert used == n and abs(T - math.exp(-float(np.dot(sg, delta)))) < 1e-12
    flat, Tf, _, _ = oracle.composite(sg, np.tile([0.3, 0.5, 0.7], (n, 1)), delta, 0.0, bg)
    np.testing.assert_allclose(flat, np.array([0.3, 0.5, 0.7]) * (1 - Tf) + np.array(bg) * Tf, atol=1e-12)
    # equal deltas: the constant-step form; a delta is tied to its own sample (reversing only the deltas changes T's path)
    same = oracle.composite(sg, col, np.full(n, 0.05), 0.01, bg)
    ref = oracle.composite(sg, col, 0.05, 0.01, bg)
    assert np.array_equal(same[0], ref[0]) and same[1:] == ref[1:]
    # sample i is weighted by T_(i-1) (1 - exp(-sigma_i delta_i)), written out
    Tr, C = 1.0, np.zeros(3)
    for i in range(n):
        a = 1 - math.exp(-sg[i] * delta[i])
        C += Tr * a * col[i]
        Tr *= 1 - a
    np.testing.assert_allclose(out, C + Tr * np.array(bg), atol=1e-12)
    assert np.abs(oracle.composite(sg, col, delta[::-1].copy(), 0.0, bg)[0] - out).max() > 1e-3
    # early termination looks at the same T
    cut, Tc, used_c, _ = oracle.composite(sg, col, delta, 0.05, bg)
    T_after = np.exp(-np.cumsum(sg * delta))
    first_below = int(np.argmax(T_after < 0.05))
    assert used_c == first_below + 1 < n and abs(Tc - T_after[first_below]) < 1e-12 and np.abs(cut - out).max() <= 0.05


def test_ert_error_is_bounded_by_eps_and_eps_zero_is_off():
    g = ks.rng(6)
    for _ in range(20):
        n = 80
        sg, col = g.uniform(0, 30, n), g.random((n, 3))
        full, Tf, used_f, _ = oracle.composite(sg, col, 0.05)
        cut, Tc, used_c, mg = oracle.composite(sg, col, 0.05, eps=0.01)
        assert used_f == n and used_c <= n and np.abs(full - cut).max() <= 0.01
        # it stops right after the first sample that leaves T = exp(-0.05 * sum of the densities so far) below eps
        T_after = np.exp(-0.05 * np.cumsum(sg))
        first_below = int(np.argmax(T_after < 0.01))
        assert T_after[first_below] < 0.01 and used_c == first_below + 1 < n
        assert Tc < 0.01 and abs(Tc - T_after[first_below]) < 1e-12 and mg >= 0
        again, _, u2, m2 = oracle.composite(sg, col, 0.05, eps=0.0)
        np.testing.assert_array_equal(again, full)
        assert u2 == n and math.isinf(m2)


# ------------------------------------------------------------------ marching and rendering
def const_scene(sigma, colour, res=(2, 2, 2), occ=None, lo=(0, 0, 0), hi=(1, 1, 1)):
    """Every network outputs density `sigma` and colour `colour` everywhere (bias only)."""
    n = int(np.prod(res))
    w = zero_net(n=n)
    lv = ks.layer_views(w, 32)
    lv[2][1][:, 0] = sigma
    c = np.asarray(colour, np.float64)
    lv[4][1][:, :] = np.log(c / (1 - c))
    return OracleScene(res, lo, hi, 32, w, occ)


def test_march_counts_lattice_points_inside_the_box():
    sc = const_scene(1.0, (0.5, 0.5, 0.5))
    # axis-parallel ray entering the unit cube at t = 1: midpoints t_k = 0.5 + (k + 1/2)/16
    o, d = np.array([-1.0, 0.3, 0.6], np.float32), np.array([1.0, 0.0, 0.0], np.float32)
    ks_ = sc.march(o, d, 0.5, 1 / 16, 40)
    expect = [k for k in range(40) if 0 <= Fraction(-1) + Fraction(1, 2) + Fraction(2 * k + 1, 32) < 1]
    assert ks_.tolist() == expect and len(expect) == 16
    # lattice points sit in the middle of their steps: shifted by 3/64 the box holds the midpoints 7..22
    # (x_k = (4k - 27)/64), whereas the starts of the steps inside it would be 8..23
    assert sc.march(o, d, 0.5 + 3 / 64, 1 / 16, 40).tolist() == list(range(7, 23))
    # a ray that misses the box keeps nothing
    assert len(sc.march(np.array([-1, 2.0, 0.5], np.float32), d, 0.5, 1 / 16, 40)) == 0


def test_march_skips_unoccupied_voxels():
    occ = np.zeros((8, 8, 8), np.uint8)
    occ[2:4, :, :] = 1                       # slab 0.25 <= x < 0.5
    occ[6, 2, 4] = 1                         # one voxel: x in [.75,.875), y in [.25,.375), z in [.5,.625)
    sc = const_scene(1.0, (0.5, 0.5, 0.5), occ=occ)
    o, d = np.array([-1.0, 0.3, 0.6], np.float32), np.array([1.0, 0.0, 0.0], np.float32)
    got = sc.march(o, d, 1.0, 1 / 64, 64).tolist()       # x_k = (k + 1/2)/64
    want = [k for k in range(64) if 16 <= k < 32 or 48 <= k < 56]
    assert got == want
    full = const_scene(1.0, (0.5, 0.5, 0.5), occ=np.ones((8, 8, 8), np.uint8))
    none = const_scene(1.0, (0.5, 0.5, 0.5))
    assert full.march(o, d, 1.0, 1 / 64, 64).tolist() == none.march(o, d, 1.0, 1 / 64, 64).tolist() == list(range(64))


def test_render_constant_density_closed_form():
    colour, bg, sigma = np.array([0.2, 0.5, 0.9]), np.array([1.0, 0.25, 0.0]), 3.0
    occ = np.zeros((8, 8, 8), np.uint8)
    occ[2:4, :, :] = 1
    for o_, n_expect in ((None, 16), (occ, 4)):
        sc = const_scene(sigma, colour, occ=o_)
        o = np.array([[-1.0, 0.3, 0.6]], np.float32)
        d = np.array([[1.0, 0.0, 0.0]], np.float32)
        step = 1 / 16
        rgb, n_eval, T, _ = sc.render(o, d, 0.5, step, 40, 0.0, bg)
        assert n_eval[0] == n_expect
        Texp = math.exp(-sigma * n_expect * step)
        assert abs(T[0] - Texp) < 1e-12
        np.testing.assert_allclose(rgb[0], colour * (1 - Texp) + bg.astype(np.float32) * Texp, atol=1e-7)
    # nothing occupied: the pixel is the background
    sc = const_scene(sigma, colour, occ=np.zeros((4, 4, 4), np.uint8))
    rgb, n_eval, T, _ = sc.render(o, d, 0.5, step, 40, 0.01, bg)
    assert n_eval[0] == 0 and T[0] == 1.0
    np.testing.assert_allclose(rgb[0], bg, atol=1e-7)
    # zero density (negative density bias is cut by the ReLU): background again
    sc = const_scene(-2.0, colour)
    rgb, n_eval, _, _ = sc.render(o, d, 0.5, step, 40, 0.0, bg)
    assert n_eval[0] == 16
    np.testing.assert_allclose(rgb[0], bg, atol=1e-7)


def test_render_is_march_then_networks_then_blend():
    from kn_synth import configs
    cfg = configs.config1(16, 16)
    s = cfg["scene"]
    sc = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], s["weights"])
    rgb, n_eval, T, _ = sc.render(cfg["rays_o"], cfg["rays_d"], cfg["t_near"], cfg["step"], cfg["K"], 0.0, cfg["bg"])
    assert n_eval.max() > 20 and n_eval.min() >= 0
    step32, tn32 = np.float32(cfg["step"]), np.float32(cfg["t_near"])
    for r in (0, 37, 100, 255):
        kk = sc.march(cfg["rays_o"][r], cfg["rays_d"][r], cfg["t_near"], cfg["step"], cfg["K"])
        assert len(kk) == n_eval[r]
        t = (kk.astype(np.float64) + 0.5) * float(step32) + float(tn32)
        x = cfg["rays_o"][r].astype(np.float64) + t[:, None] * cfg["rays_d"][r].astype(np.float64)
        sg, col, ids = sc.eval_points(x.astype(np.float32), np.tile(cfg["rays_d"][r], (len(kk), 1)))
        assert np.all(ids >= 0)
        out, Tr, _, _ = oracle.composite(sg, col, float(step32))
        np.testing.assert_allclose(out, rgb[r], atol=1e-5)      # x recomputed in fp64 here, fp32 lattice there
        assert abs(Tr - T[r]) < 1e-5


def test_render_stops_where_the_blend_of_its_samples_stops():
    """Early termination inside the render (Sec. 3.4): a ray's image, final transmittance and number of evaluated
    samples equal those of blending all its marched samples with the same threshold (the blend stops by itself)."""
    from kn_synth import configs
    cfg = configs.config3(16, 16)
    s = cfg["scene"]
    sc = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], s["weights"], s["occupancy"])
    o, d, eps = cfg["rays_o"], cfg["rays_d"], 0.05
    rgb, n_eval, T, mg = sc.render(o, d, cfg["t_near"], cfg["step"], cfg["K"], eps, cfg["bg"])
    step32, tn32 = np.float32(cfg["step"]), np.float32(cfg["t_near"])
    stopped = 0
    for r in np.flatnonzero(n_eval > 0)[::3]:
        kk = sc.march(o[r], d[r], cfg["t_near"], cfg["step"], cfg["K"])
        t = ((kk.astype(np.float64) + 0.5) * float(step32) + float(tn32)).astype(np.float32)
        x = (o[r].astype(np.float64) + t[:, None].astype(np.float64) * d[r].astype(np.float64)).astype(np.float32)
        sg, col, _ = sc.eval_points(x, np.tile(d[r], (len(kk), 1)))
        out, Tr, used, m = oracle.composite(sg, col, float(step32), eps, cfg["bg"])
        if m < 1e-3:
            continue                                      # (positions recomputed here: a ray on the threshold may differ)
        assert used == n_eval[r] and abs(Tr - T[r]) < 1e-4
        np.testing.assert_allclose(out, rgb[r], atol=1e-4)
        stopped += used < len(kk)
    assert stopped >= 10                                  # rays that ended early, with samples left behind


def test_render_ert_bound_and_straddle_margin():
    from kn_synth import configs
    cfg = configs.config3(24, 24)
    s = cfg["scene"]
    sc = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], s["weights"], s["occupancy"])
    args = (cfg["rays_o"], cfg["rays_d"], cfg["t_near"], cfg["step"], cfg["K"])
    full, n_full, _, _ = sc.render(*args, 0.0, cfg["bg"])
    cut, n_cut, T, mg = sc.render(*args, cfg["term_eps"], cfg["bg"])
    assert np.abs(full - cut).max() <= cfg["term_eps"] + 1e-12
    assert np.all(n_cut <= n_full) and n_cut.sum() < n_full.sum()
    assert np.all((T < 0.01) == (n_cut < n_full) | (T < 0.01))
    assert np.all(mg[n_cut > 0] >= 0)


# ------------------------------------------------------------------ occupancy extraction (Sec. 3.4)


# ------------------------------------------------------------------ sparse network grids (Sec. 5)
def _sparse_fixture():
    from kn_synth import configs
    cfg = configs.config3(20, 20)
    s = cfg["scene"]
    dense = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], s["weights"], s["occupancy"])
    return cfg, s, dense


def test_sparse_grid_with_every_cell_present_equals_the_dense_grid_whatever_the_order():
    cfg, s, dense = _sparse_fixture()
    n = dense.N
    args = (cfg["rays_o"], cfg["rays_d"], cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    want = dense.render(*args)
    rng = np.random.default_rng(5)
    pts = rng.uniform(-1.1, 1.1, (4000, 3)).astype(np.float32)
    dirs = ks.sphere_dirs(4000, 3)
    want_pts = dense.eval_points(pts, dirs)
    for table in (np.arange(n, dtype=np.int32), rng.permutation(n).astype(np.int32)):
        w = np.empty_like(s["weights"])
        w[table] = s["weights"]                 # network table[c] holds the weights of cell c
        sp = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], w, s["occupancy"], cell_net=table)
        got = sp.render(*args)
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
        sg, rgb, ids = sp.eval_points(pts, dirs)
        assert np.array_equal(sg, want_pts[0]) and np.array_equal(rgb, want_pts[1])
        inside = want_pts[2] >= 0
        assert np.array_equal(ids[inside], table[want_pts[2][inside]]) and np.all(ids[~inside] == -1)
        assert np.array_equal(sp.cell_ids(pts), ids)


def test_a_cell_without_a_network_is_empty_space():
    cfg, s, dense = _sparse_fixture()
    n = dense.N
    rng = np.random.default_rng(6)
    present = rng.random(n) < 0.6
    table = np.full(n, -1, np.int32)
    table[present] = rng.permutation(int(present.sum())).astype(np.int32)
    w = np.empty((int(present.sum()), s["weights"].shape[1]), np.float32)
    w[table[present]] = s["weights"][present]
    sp = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], w, s["occupancy"], cell_net=table)
    # the same field on the dense grid: the absent cells' networks put out density 0 (layer 3, output 0)
    wz = s["weights"].copy()
    lv = ks.layer_views(wz, s["hidden"])
    lv[2][0][~present, :, 0] = 0.0
    lv[2][1][~present, 0] = 0.0
    dz = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], wz, s["occupancy"])
    args = (cfg["rays_o"], cfg["rays_d"], cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    rgb_s, n_s, T_s, _ = sp.render(*args)
    rgb_z, n_z, T_z, _ = dz.render(*args)
    np.testing.assert_allclose(rgb_s, rgb_z, atol=1e-12)
    np.testing.assert_allclose(T_s, T_z, atol=1e-12)
    assert np.all(n_s <= n_z) and n_s.sum() < n_z.sum()          # the absent cells' samples are never evaluated
    # marching: exactly the dense ray's samples whose cell has a network
    for r in (0, 111, 210, 399):
        kk = dense.march(cfg["rays_o"][r], cfg["rays_d"][r], cfg["t_near"], cfg["step"], cfg["K"])
        t = np.float32(cfg["t_near"]) + (kk.astype(np.float32) + np.float32(0.5)) * np.float32(cfg["step"])
        x = cfg["rays_o"][r] + t[:, None] * cfg["rays_d"][r]
        keep = present[dense.cell_ids(x.astype(np.float32))]
        got = sp.march(cfg["rays_o"][r], cfg["rays_d"][r], cfg["t_near"], cfg["step"], cfg["K"])
        # (x is recomputed without the fused multiply-add: a point within rounding of a cell face may differ)
        assert len(set(got.tolist()) ^ set(kk[keep].tolist())) <= 1
    # points: density and colour 0 and id -1 in absent cells, the dense values elsewhere
    pts = rng.uniform(-1, 1, (3000, 3)).astype(np.float32)
    dirs = np.tile(np.float32([0.6, 0.0, 0.8]), (3000, 1))
    sg, rgb, ids = sp.eval_points(pts, dirs)
    sg_d, rgb_d, ids_d = dense.eval_points(pts, dirs)
    gone = ~present[ids_d]
    assert gone.sum() > 500 and np.all(ids[gone] == -1) and np.all(sg[gone] == 0) and np.all(rgb[gone] == 0)
    assert np.array_equal(sg[~gone], sg_d[~gone]) and np.array_equal(rgb[~gone], rgb_d[~gone])
    # table entries outside [0, n_nets) also mean "no network"
    bad = table.copy()
    bad[~present] = np.where(rng.random(int((~present).sum())) < 0.5, len(w), -7)
    sb = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], w, s["occupancy"], cell_net=bad)
    assert np.array_equal(sb.eval_points(pts, dirs)[2], ids)
    # extraction: the occupancy of the zeroed dense field
    occ_s = sp.extract_occupancy((12, 12, 12), 0.5)[0]
    occ_z = dz.extract_occupancy((12, 12, 12), 0.5)[0]
    assert np.array_equal(occ_s, occ_z) and 0 < occ_s.sum() < occ_s.size


# ------------------------------------------------------------------ stratified sampling (Sec. 3.4)
def test_stratified_offsets_are_uniform_draws_per_seed_ray_and_sample():
    u = np.array([[[oracle.stratified_offset(s_, r, k) for k in range(64)] for r in range(48)] for s_ in (0, 1, 77)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert np.array_equal(u * 2 ** 24, np.floor(u * 2 ** 24))          # 24-bit fractions
    n = u.size
    assert abs(u.mean() - 0.5) < 4 * math.sqrt(1 / 12 / n) and abs(u.var() - 1 / 12) < 0.004
    hist = np.histogram(u, bins=16, range=(0, 1))[0]
    assert ((hist - n / 16) ** 2 / (n / 16)).sum() < 45                 # chi-square, 15 degrees of freedom
    c = u - 0.5
    for a, b in ((c[:, :, 1:], c[:, :, :-1]), (c[:, 1:], c[:, :-1]), (c[1:], c[:-1])):   # along k, ray, seed
        assert abs((a * b).mean() * 12) < 5 / math.sqrt(a.size)
    assert len(np.unique(u)) > 0.99 * n
    # the function is its published definition (32-bit finalizer of MurmurHash3, nested)
    def mix(v):
        v ^= v >> 16; v = (v * 0x85EBCA6B) & 0xFFFFFFFF; v ^= v >> 13; v = (v * 0xC2B2AE35) & 0xFFFFFFFF
        return v ^ (v >> 16)
    assert mix(0) == 0 and mix(1) == 0x514E28B7
    for s_, r, k in ((0, 0, 0), (1, 2, 3), (210313744, 639999, 511), (2 ** 32 - 1, 2 ** 32 - 1, 1023)):
        want = (mix(mix((mix(s_) + r) & 0xFFFFFFFF) ^ k) >> 8) / 2 ** 24
        assert oracle.stratified_offset(s_, r, k) == want


def test_stratified_march_tests_one_point_per_interval():
    occ = np.zeros((8, 8, 8), np.uint8)
    occ[2:4, :, :] = 1                       # slab 0.25 <= x < 0.5
    sc = const_scene(1.0, (0.5, 0.5, 0.5), occ=occ)
    o, d = np.array([-1.0, 0.3, 0.6], np.float32), np.array([1.0, 0.0, 0.0], np.float32)
    differs = 0
    for seed, ray in ((3, 0), (3, 1), (4, 0), (9, 12345)):
        got = sc.march_stratified(o, d, 1.0, 1 / 64, 64, seed, ray).tolist()
        # x_k = (k + u_k) / 64 exactly (all quantities are small dyadic fractions): in the slab iff 16 <= k + u_k < 32
        want = [k for k in range(64) if 16 <= k + oracle.stratified_offset(seed, ray, k) < 32]
        assert got == want == list(range(16, 32))        # interval k lies inside the slab or outside it
        # intervals of 1/40 shifted by 1/128: the slab's faces cut intervals 9 and 19 at 0.6875 of their length
        tn = 1.0 + 1 / 128
        got = sc.march_stratified(o, d, tn, 1 / 40, 40, seed, ray).tolist()
        want = [k for k in range(40) if 9.6875 <= k + oracle.stratified_offset(seed, ray, k) < 19.6875]
        assert got == want and set(range(10, 19)) <= set(got) <= set(range(9, 20))
        differs += got != sc.march(o, d, tn, 1 / 40, 40).tolist()
    assert differs >= 1                                    # the boundary intervals do depend on the draw


def test_stratified_render_of_a_constant_medium_telescopes():
    colour, bg, sigma = np.array([0.2, 0.5, 0.9]), np.array([1.0, 0.25, 0.0]), 3.0
    sc = const_scene(sigma, colour, res=(1, 1, 1), lo=(-4, -4, -4), hi=(4, 4, 4))
    o = np.tile(np.float32([-1.0, 0.3, 0.6]), (5, 1))
    d = np.tile(np.float32([1.0, 0.0, 0.0]), (5, 1))
    step, t_near, K, seed = 1 / 16, 0.5, 24, 11
    rgb, n_eval, T, _ = sc.render(o, d, t_near, step, K, 0.0, bg, seed=seed)
    assert np.all(n_eval == K)
    for r in range(5):
        # sum of delta_k = t_K - t_0 = (K + u_K - u_0) * step
        length = (K + oracle.stratified_offset(seed, r, K) - oracle.stratified_offset(seed, r, 0)) * step
        assert abs(T[r] - math.exp(-sigma * length)) < 1e-6
        np.testing.assert_allclose(rgb[r], colour * (1 - T[r]) + bg * T[r], atol=1e-7)
    assert len(np.unique(T)) == 5                           # each ray has its own draws
    T_mid = sc.render(o, d, t_near, step, K, 0.0, bg)[2]
    assert np.allclose(T_mid, math.exp(-sigma * K * step), atol=1e-12)
    # rays rendered as a subset of a frame carry their numbers in the frame
    T_sub = sc.render(o[:2], d[:2], t_near, step, K, 0.0, bg, seed=seed, ray_ids=[3, 1])[2]
    assert np.array_equal(T_sub, T[[3, 1]])
    # other seed, other draws; same seed, same picture
    assert not np.array_equal(sc.render(o, d, t_near, step, K, 0.0, bg, seed=12)[2], T)
    assert np.array_equal(sc.render(o, d, t_near, step, K, 0.0, bg, seed=seed)[2], T)


def test_stratified_render_is_march_then_networks_then_blend_with_its_own_deltas():
    from kn_synth import configs
    cfg = configs.config3(16, 16)
    s = cfg["scene"]
    sc = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], s["weights"], s["occupancy"])
    seed = 5
    rgb, n_eval, T, _ = sc.render(cfg["rays_o"], cfg["rays_d"], cfg["t_near"], cfg["step"], cfg["K"], 0.0, cfg["bg"], seed=seed)
    mid = sc.render(cfg["rays_o"], cfg["rays_d"], cfg["t_near"], cfg["step"], cfg["K"], 0.0, cfg["bg"])
    assert n_eval.sum() > 500 and 1e-4 < np.abs(rgb - mid[0]).max() < 0.3
    step, tn = float(np.float32(cfg["step"])), float(np.float32(cfg["t_near"]))
    checked = 0
    for r in np.argsort(-n_eval)[:6]:
        kk = sc.march_stratified(cfg["rays_o"][r], cfg["rays_d"][r], cfg["t_near"], cfg["step"], cfg["K"], seed, r)
        assert len(kk) == n_eval[r]
        u = np.array([oracle.stratified_offset(seed, r, k) for k in range(cfg["K"] + 1)])
        t = tn + (np.arange(cfg["K"] + 1) + u) * step
        x = cfg["rays_o"][r].astype(np.float64) + t[kk, None] * cfg["rays_d"][r].astype(np.float64)
        sg, col, ids = sc.eval_points(x.astype(np.float32), np.tile(cfg["rays_d"][r], (len(kk), 1)))
        delta = t[kk + 1] - t[kk]
        Tr, C = 1.0, np.zeros(3)
        for i in range(len(kk)):                              # Eq. 2-4 with a delta per sample
            a = 1 - math.exp(-sg[i] * delta[i])
            C += Tr * a * col[i]
            Tr *= 1 - a
        np.testing.assert_allclose(C + Tr * np.asarray(cfg["bg"]), rgb[r], atol=2e-4)   # x in fp64 here, fp32 lattice there
        assert abs(Tr - T[r]) < 2e-4
        checked += 1
    assert checked == 6


def _probe_coords(lo, hi, res):
    """(res, 3) positions of the three sub-cell centres of every voxel along one axis, fp64."""
    v = np.arange(res)[:, None]
    return lo + (v + np.array([1 / 6, 1 / 2, 5 / 6])[None, :]) * ((hi - lo) / res)


def test_extraction_constant_density_and_strict_threshold():
    w = zero_net(n=8)
    ks.layer_views(w, 32)[2][1][:, 0] = 10.0                      # b3[0]: sigma = 10 everywhere
    sc = unit_scene(w, res=(2, 2, 2))
    occ, top, mg = sc.extract_occupancy((3, 4, 5), 9.999)
    assert occ.shape == (3, 4, 5) and occ.dtype == np.uint8 and np.all(occ == 1)
    np.testing.assert_array_equal(top, 10.0)
    np.testing.assert_allclose(mg, 0.001, atol=1e-6)            # tau is rounded to fp32 first
    occ, _, mg = sc.extract_occupancy((3, 4, 5), 10.0)            # "above tau" is strict
    assert np.all(occ == 0) and np.all(mg == 0)


@pytest.mark.parametrize("axis", [0, 1, 2])
@pytest.mark.parametrize("sign", [1.0, -1.0])
def test_extraction_linear_field_marks_voxels_by_their_extreme_probe(axis, sign):
    # sigma = relu(sign * k * (x_axis - mid) + 4), k = 8 / extent: rising (or falling) from 0 to 8 along one axis of
    # the box [-1,1]x[0,2]x[1,5].
    # A voxel is marked iff the probe with the largest density, the one at offset 5/6 (rising) or 1/6 (falling)
    # of the voxel along that axis, is above tau.  Which axis of the output array follows the field pins the
    # x-slowest layout.
    lo, hi, res = np.array([-1.0, 0.0, 1.0]), np.array([1.0, 2.0, 5.0]), (7, 6, 9)
    w = zero_net(n=6)
    lv = ks.layer_views(w, 32)
    k, mid = 8.0 / (hi[axis] - lo[axis]), 0.5 * (lo[axis] + hi[axis])
    lv[0][0][:, axis, 0] = sign * k                                # identity input `axis` -> h1[0]
    lv[0][1][:, 0] = -sign * k * mid + 4.0
    lv[1][0][:, 0, 0] = 1.0
    lv[2][0][:, 0, 0] = 1.0
    sc = unit_scene(w, res=(1, 2, 3), lo=lo, hi=hi)
    tau = 5.0
    occ, top, mg = sc.extract_occupancy(res, tau)
    pc = _probe_coords(lo[axis], hi[axis], res[axis])               # (res, 3)
    dens = np.maximum(sign * k * (pc - mid) + 4.0, 0.0)
    want_line = dens.max(axis=1) > tau
    assert 0 < want_line.sum() < res[axis]
    assert np.abs(dens - tau).min() > 1e-3                        # no probe sits on the threshold
    shape = [1, 1, 1]
    shape[axis] = res[axis]
    want = np.broadcast_to(want_line.reshape(shape), res)
    np.testing.assert_array_equal(occ, want.astype(np.uint8))
    np.testing.assert_allclose(top, np.broadcast_to(dens.max(axis=1).reshape(shape), res), atol=1e-5)
    np.testing.assert_allclose(mg, np.broadcast_to(np.abs(dens - tau).min(axis=1).reshape(shape), res), atol=1e-5)


def test_extraction_sees_the_centre_probe():
    # A tent of half-width 0.02 around the centre of voxel 3 of 8 along y (unit cube): narrower than the distance to
    # the neighbouring probes (1/24), so only the probe at offset 1/2 of that voxel is above tau.
    c = (3 + 0.5) / 8
    w = zero_net()
    lv = ks.layer_views(w, 32)
    lv[0][0][0, 1, 0], lv[0][1][0, 0] = 1.0, -c                  # h1[0] = relu(y - c)
    lv[0][0][0, 1, 1], lv[0][1][0, 1] = -1.0, c                  # h1[1] = relu(c - y)
    lv[1][0][0, 0, 0] = lv[1][0][0, 1, 0] = -50.0                # h2[0] = relu(1 - 50 |y - c|)
    lv[1][1][0, 0] = 1.0
    lv[2][0][0, 0, 0] = 20.0                                       # sigma = 20 h2[0]
    occ, top, _ = unit_scene(w).extract_occupancy((2, 8, 2), 10.0)
    want = np.zeros((2, 8, 2), np.uint8)
    want[:, 3, :] = 1
    np.testing.assert_array_equal(occ, want)
    np.testing.assert_allclose(top[:, 3, :], 20.0, atol=1e-4)
    # moved to offset 1/6 of the same voxel, then to the voxel boundary where no probe sits
    for centre, hit in (((3 + 1 / 6) / 8, True), (3 / 8, False)):
        lv[0][1][0, 0], lv[0][1][0, 1] = -centre, centre
        occ, _, _ = unit_scene(w).extract_occupancy((2, 8, 2), 10.0)
        assert bool(occ[:, 3, :].all()) == hit and occ.sum() == (4 if hit else 0)


def test_extraction_uses_the_network_of_the_probes_cell_and_the_voxel_list_form():
    # 2x1x1 networks with different constant densities, 3 voxels along x: the middle voxel straddles the cell
    # boundary, its probes at offsets 1/6 (x = 0.389) and 1/2 (x = 0.5) fall into different cells.
    w = zero_net(n=2)
    ks.layer_views(w, 32)[2][1][0, 0] = 1.0
    ks.layer_views(w, 32)[2][1][1, 0] = 7.0
    sc = unit_scene(w, res=(2, 1, 1))
    occ, top, _ = sc.extract_occupancy((3, 1, 1), 5.0)
    assert occ.ravel().tolist() == [0, 1, 1] and top.ravel().tolist() == [1.0, 7.0, 7.0]
    occ, top, _ = sc.extract_occupancy((3, 1, 1), 0.5)
    assert occ.ravel().tolist() == [1, 1, 1]
    # the per-voxel form agrees with the whole-grid form on a random scene
    sc = OracleScene((2, 3, 2), (0, 0, 0), (1, 1, 1), 32, ks.kaiming_weights(12, 32, 77, sigma_scale=20.0))
    tau = float(np.median(sc.extract_occupancy((5, 4, 6), 0.0)[1]))   # random weights: take tau inside the range
    full, ftop, fmg = sc.extract_occupancy((5, 4, 6), tau)
    assert 0 < full.sum() < full.size
    np.testing.assert_array_equal(full, (ftop > np.float32(tau)).astype(np.uint8))
    pick = np.array([0, 7, 33, 64, 119], np.int64)
    o, t, m = sc.extract_occupancy((5, 4, 6), tau, voxels=pick)
    np.testing.assert_array_equal(o, full.ravel()[pick])
    np.testing.assert_array_equal(t, ftop.ravel()[pick])
    np.testing.assert_array_equal(m, fmg.ravel()[pick])
    # and with 27 explicit evaluations per voxel at independently computed probe positions
    for vox in pick:
        ix, iy, iz = np.unravel_index(vox, (5, 4, 6))
        offs = np.array([1 / 6, 1 / 2, 5 / 6])
        gx, gy, gz = np.meshgrid((ix + offs) / 5, (iy + offs) / 4, (iz + offs) / 6, indexing="ij")
        pts = np.stack([gx.ravel(), gy.ravel(), gz.ravel()], 1).astype(np.float32)
        sg, _, _ = sc.eval_points(pts, np.tile(np.float32([0, 0, 1]), (27, 1)))
        assert abs(sg.max() - ftop.ravel()[vox]) < 1e-4 * (1 + sg.max())


def test_threaded_build_gives_identical_results():
    w = ks.kaiming_weights(8, 32, 1)
    a = OracleScene((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, w)
    b = OracleScene((2, 2, 2), (0, 0, 0), (1, 1, 1), 32, w, threads=True)
    pts, dirs = ks.uniform_points(500, 1), ks.sphere_dirs(500, 2)
    for u, v in zip(a.eval_points(pts, dirs), b.eval_points(pts, dirs)):
        np.testing.assert_array_equal(u, v)
    assert a.num_threads() == 1 and b.num_threads() >= 1
