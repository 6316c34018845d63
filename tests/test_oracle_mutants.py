"""The pins of tests/test_oracle_pins.py must notice plausible mistakes in the oracle.

Each mutant below is the oracle's source with one such mistake planted (a sign, an index, a transposed operand, a
dropped term, an off-by-one), compiled on the CPU into a shared object of its own; the pin tests named with it are run
against that build in a child process and have to fail.  The unchanged source, built the same way, has to pass."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "kn_oracle.c")

# (name, text in the source, what a mistaken author might have written, pins that must catch it)
MUTANTS = [
    ("alpha_sign_as_printed", "double alpha = 1.0 - exp(-sigma[i] * (delta ? delta[i] : step));",
     "double alpha = 1.0 - exp(sigma[i] * (delta ? delta[i] : step));",
     "alpha_blend or constant_density"),
    ("render_alpha_sign", "double alpha = 1.0 - exp(-sg * lattice_delta(t_near, step, k, &j));",
     "double alpha = 1.0 - exp(sg * lattice_delta(t_near, step, k, &j));", "render_constant_density"),
    ("background_dropped", "rgb_out[3 * r + c] = C[c] + T * (double)bg[c];", "rgb_out[3 * r + c] = C[c];", "render_constant_density"),
    ("transmittance_before_colour", "for (int c = 0; c < 3; ++c) C[c] += T * alpha * rgb[3 * i + c]; /* Eq. 2 */\n        T *= (1.0 - alpha);",
     "T *= (1.0 - alpha);\n        for (int c = 0; c < 3; ++c) C[c] += T * alpha * rgb[3 * i + c];", "alpha_blend"),
    ("sin_cos_swapped", "out[3 + 6 * k + a] = sin(f * (double)p[a]);\n            out[3 + 6 * k + 3 + a] = cos(f * (double)p[a]);",
     "out[3 + 6 * k + a] = cos(f * (double)p[a]);\n            out[3 + 6 * k + 3 + a] = sin(f * (double)p[a]);", "posenc"),
    ("encoding_with_pi", "double f = ldexp(1.0, k); /* 2^k */", "double f = ldexp(1.0, k) * 3.14159265358979323846;", "posenc"),
    ("encoding_axis_major", "out[3 + 6 * k + a] = sin(f * (double)p[a]);\n            out[3 + 6 * k + 3 + a] = cos(f * (double)p[a]);",
     "out[3 + 2 * k + 2 * L * a - 2 * k * 0 + 0] = sin(f * (double)p[a]);\n            out[3 + 2 * k + 2 * L * a + 1] = cos(f * (double)p[a]);",
     "posenc or mlp_wiring or gamma_zero"),
    ("z_slowest", "return (idx[0] * res[1] + idx[1]) * res[2] + idx[2];", "return (idx[2] * res[1] + idx[1]) * res[0] + idx[0];",
     "grid_index"),
    ("upper_face_inside", "if (!(fl >= 0.0f) || !(fl < (float)res[a])) return -1;", "if (!(fl >= 0.0f) || !(fl <= (float)res[a])) return -1;",
     "grid_index_faces"),
    ("weights_transposed", "acc += in[i] * (double)W[(size_t)i * n_out + o];", "acc += in[i] * (double)W[(size_t)o * n_in + i];",
     "single_cell_grid or mlp_wiring"),
    ("bias_dropped", "double acc = (double)b[o];", "double acc = 0.0;", "mlp_wiring or gamma_zero or single_cell"),
    ("relu_on_feature", "in4[i] = o3[1 + i]; /* feature vector: no activation */", "in4[i] = relu(o3[1 + i]);", "mlp_wiring or single_cell"),
    ("density_is_last_output", "*sigma = relu(o3[0]);\n    for (int i = 0; i < H; ++i) in4[i] = o3[1 + i];",
     "*sigma = relu(o3[H]);\n    for (int i = 0; i < H; ++i) in4[i] = o3[i];", "mlp_wiring or single_cell or parameter_count"),
    ("direction_before_feature", "kno_posenc(d, s->L_dir, in4 + H);", "for (int i = H - 1; i >= 0; --i) in4[i + ed] = in4[i];\n    kno_posenc(d, s->L_dir, in4);",
     "mlp_wiring or single_cell"),
    ("cell_local_position", "kno_posenc(x, s->L_pos, gx);", "{ float xl[3]; for (int a = 0; a < 3; ++a) { float cs = (s->aabb_max[a] - s->aabb_min[a]) / (float)s->res[a]; xl[a] = x[a] - s->aabb_min[a] - cs * floorf((x[a] - s->aabb_min[a]) / cs); } kno_posenc(xl, s->L_pos, gx); }",
     "mlp_wiring or identical_cells or each_point"),
    ("wrong_network", "} else if (kno_mlp(s, id, points + 3 * m, dirs + 3 * m, sigma + m, rgb + 3 * m) != 0) {",
     "} else if (kno_mlp(s, 0, points + 3 * m, dirs + 3 * m, sigma + m, rgb + 3 * m) != 0) {", "each_point_uses"),
    ("lattice_at_interval_start", "return (j && j->on) ? kno_stratified_offset(j->seed, j->ray, k) : 0.5f;",
     "return (j && j->on) ? kno_stratified_offset(j->seed, j->ray, k) : 0.0f;", "march_counts or march_skips"),
    ("occupancy_ignored", "return v >= 0 && s->occupancy[v] != 0;", "return v >= 0;", "march_skips or render_constant_density"),
    ("unstable_bucket", "for (int64_t m = 0; m < M; ++m) { /* ascending m => stable */\n        int32_t b = ids[m] < 0 ? N : ids[m];\n        perm[cursor[b]++] = (int32_t)m;",
     "for (int64_t m = M - 1; m >= 0; --m) {\n        int32_t b = ids[m] < 0 ? N : ids[m];\n        perm[cursor[b]++] = (int32_t)m;", "bucket_equals"),
    ("termination_never", "if (T < eps) break;                               /* Sec. 3.4, ERT */", ";", "ert_error"),
    ("render_never_terminates", "                if (T < eps) break;\n            }\n        }\n        for (int c = 0; c < 3; ++c) rgb_out[3 * r + c]",
     "                ;\n            }\n        }\n        for (int c = 0; c < 3; ++c) rgb_out[3 * r + c]", "render_stops_where"),
    ("delta_looks_backwards", "return (double)lattice_t(t_near, step, k + 1, j) - (double)lattice_t(t_near, step, k, j);",
     "return (double)lattice_t(t_near, step, k, j) - (double)lattice_t(t_near, step, k - 1, j);", "stratified_render"),
    ("delta_constant_under_stratification", "if (!(j && j->on)) return (double)step;", "if (1) return (double)step;", "stratified_render"),
    ("draws_shared_by_all_rays", "uint32_t per_ray = mix32(mix32(seed) + ray);", "uint32_t per_ray = mix32(mix32(seed));", "stratified"),
    ("draw_of_the_next_sample", "return fmaf((float)k + lattice_offset(j, k), step, t_near);", "return fmaf((float)k + lattice_offset(j, k + 1), step, t_near);",
     "stratified_march or stratified_render"),
    ("offset_23_bits", "return (float)(word >> 8) * (1.0f / 16777216.0f);", "return (float)(word >> 9) * (1.0f / 16777216.0f);", "stratified_offsets"),
    ("sparse_table_ignored_by_march", "if (network_of(s, x) < 0) return 0;", "if (kno_grid_index(s->aabb_min, s->aabb_max, s->res, x) < 0) return 0;",
     "without_a_network"),
    ("sparse_table_not_applied_to_ids", "for (int64_t m = 0; m < M; ++m) ids[m] = network_of(s, points + 3 * m);",
     "for (int64_t m = 0; m < M; ++m) ids[m] = kno_grid_index(s->aabb_min, s->aabb_max, s->res, points + 3 * m);", "sparse_grid or without_a_network"),
    ("probes_on_voxel_corners", "static const float sub[3] = {1.0f / 6.0f, 0.5f, 5.0f / 6.0f};", "static const float sub[3] = {0.0f, 0.5f, 1.0f};",
     "extraction"),
    ("threshold_not_strict", "if (sg > (double)tau) any = 1;", "if (sg >= (double)tau) any = 1;", "extraction_constant_density"),
    ("only_the_centre_probe", "for (int i = 0; i < 3; ++i)\n        for (int j = 0; j < 3; ++j)\n            for (int k = 0; k < 3; ++k) {",
     "for (int i = 1; i < 2; ++i)\n        for (int j = 1; j < 2; ++j)\n            for (int k = 1; k < 2; ++k) {", "extraction"),
    ("occupancy_at_network_resolution", "int32_t v = kno_grid_index(s->aabb_min, s->aabb_max, s->occ_res, x);",
     "int32_t v = kno_grid_index(s->aabb_min, s->aabb_max, s->res, x);", "march_skips or render_constant_density"),
    ("sigmoid_sign", "rgb[c] = 1.0 / (1.0 + exp(-o5[c]));", "rgb[c] = 1.0 / (1.0 + exp(o5[c]));", "mlp_wiring or single_cell"),
    ("density_without_relu", "*sigma = relu(o3[0]);", "*sigma = o3[0];", "render_constant_density or mlp_wiring"),
    ("second_layer_without_relu", "for (int i = 0; i < H; ++i) h2[i] = relu(h2[i]);", ";", "single_cell or mlp_wiring"),
    ("probes_use_the_voxels_home_network", "int32_t id = network_of(s, x);\n                if (id >= 0 && kno_mlp(s, id, x, dir, &sg, rgb) != 0) return -1;",
     "float ctr[3]; for (int a = 0; a < 3; ++a) ctr[a] = fmaf((float)v[a] + 0.5f, cell[a], s->aabb_min[a]);\n"
     "                int32_t id = network_of(s, ctr);\n                if (id >= 0 && kno_mlp(s, id, x, dir, &sg, rgb) != 0) return -1;",
     "extraction_uses_the_network"),
    ("delta_of_the_previous_sample", "double alpha = 1.0 - exp(-sigma[i] * (delta ? delta[i] : step));",
     "double alpha = 1.0 - exp(-sigma[i] * (delta ? delta[i > 0 ? i - 1 : 0] : step));", "delta_per_sample"),
    ("one_parameter_short", "((int64_t)H * (H + 1) + (H + 1))", "((int64_t)H * (H + 1) + H)", "parameter_count"),
]


def _build(source_text, out):
    src = out.replace(".so", ".c")
    with open(src, "w") as f:
        f.write(source_text)
    subprocess.run(["gcc", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-std=c99", "-I", os.path.join(ROOT, "oracle"), src, "-o", out,
                    "-lm"], check=True)


def _pins(lib, select):
    cmd = [sys.executable, "-m", "pytest", os.path.join(HERE, "test_oracle_pins.py"), "-x", "-q", "-p", "no:cacheprovider"]
    if select:
        cmd += ["-k", select]
    return subprocess.run(cmd, env=dict(os.environ, KN_ORACLE_LIB=lib), cwd=ROOT, capture_output=True, text=True, timeout=600)


def test_the_unchanged_oracle_passes_its_pins_when_built_this_way(tmp_path):
    lib = str(tmp_path / "plain.so")
    _build(open(SRC).read(), lib)
    r = _pins(lib, "")
    assert r.returncode == 0, r.stdout[-2000:]


@pytest.mark.parametrize("name,old,new,select", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(tmp_path, name, old, new, select):
    text = open(SRC).read()
    assert text.count(old) == 1, "the mutation site of %s is not unique in the oracle source" % name
    lib = str(tmp_path / (name + ".so"))
    _build(text.replace(old, new), lib)
    r = _pins(lib, select)
    # (a mistake that makes the oracle read outside its arrays ends the child with a signal: noticed as well)
    assert r.returncode != 0 and (" failed" in r.stdout or r.returncode < 0), \
        "no pin noticed the mistake %s\n%s" % (name, r.stdout[-1500:])
