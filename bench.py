#!/usr/bin/env python3
"""Benchmark of the KiloNeRF rendering path on one MI355X.

A step = one pass of the whole path (march + empty-space skipping, bucketing, grouped MLP, blending
with early termination, wave loop) over one 800x800 frame of the synthetic 16^3-network scene
(workload "cfg3"); the camera cycles through 8 poses on a ring.  Rays, weights and the occupancy
grid are resident in HBM before the timed region.  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MFMA_16BIT = 2.5e15   # FLOP/s, dense fp16 / bf16 MFMA, MI355X
PEAK_MFMA_F32 = 157.3e12   # FLOP/s, fp32 MFMA
PEAK_HBM = 8.0e12          # B/s
MEASURED = {}              # this machine's own limits (paper_2103_13744_amd.peaks), filled by main()


def with_measured(roof, key):
    """Adds the micro-benchmarked peak of the same kind, and the fraction of it, to a roofline block.  key: an entry
    of MEASURED in the block's unit (GB/s or TFLOP/s)."""
    peak = MEASURED.get(key)
    if peak:
        roof["measured_peak"] = peak
        roof["measured_peak_kind"] = key
        roof["frac_of_measured"] = roof["achieved"] / peak
    return roof


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"
# Sec. 3.2's network: 2 * (63 H + H H + H (H + 1) + (H + 27) H + 3 H) FLOP per sample.  The 16-bit kernels take the
# activation-free feature layer and layer 4 as one affine map and execute 2 * (63 H + H H + H + (H + 27) H + 3 H); the
# roofline counts the network as defined (the work the method asks for) and the line states both.
FLOP_PER_SAMPLE = {32: 12160, 64: 36608}
FLOP_PER_SAMPLE_EXECUTED_16BIT = {32: 10112, 64: 28416}
# vector-ALU issue slots of the render variant of k_mlp_mfma per 16 samples, counted in the generated code of its main
# loop (269 / 363 vector instructions per 64 samples, 30 of them transcendental and counted twice)
VALU_SLOTS_PER_16_SAMPLES = {32: 75, 64: 98}


EVENTS_EVERY = 5  # frames of the timed region per frame that carries the dominant kernel's HIP events (coprime to the 8 poses: every pose is timed)
TRAFFIC_FILE = "profiles/hbm_traffic_cfg3_f16.txt"


def read_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE / WRITE_SIZE runs of this
    benchmark, scaled by the copy-kernel calibration stated in the file), and the commit the counters were read at
    (stated in the file): not measured in this run.  ({}, None) if the file is absent."""
    out, commit = {}, None
    try:
        with open(os.path.join(ROOT, TRAFFIC_FILE)) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch":
                    out[parts[1]] = float(parts[2])
                if len(parts) >= 2 and parts[0] == "measured_at_commit":
                    commit = parts[1]
    except OSError:
        pass
    return out, commit


def frames_in_flight(torch, scene, rays, args, R, steps, n, blended_per_frame):
    """Supplementary: the same frames with `n` of them in flight, one stream, workspace and host thread each (frames
    are independent; the kernels of one frame's launch gaps and tails overlap with the other frames' work).  The
    headline value stays the one-frame-at-a-time figure, whose kernels can be timed one by one."""
    import threading
    outs = [torch.empty((R, 3), dtype=torch.float32, device="cuda") for _ in range(n)]
    wss = [torch.empty(scene.workspace_bytes(max_rays=R), dtype=torch.uint8, device="cuda") for _ in range(n)]
    streams = [torch.cuda.Stream() for _ in range(n)]
    per = max(steps // n, 1)

    def worker(t, count):
        with torch.cuda.stream(streams[t]):
            for i in range(count):
                scene.render(*rays[(i * n + t) % 8], *args, out=outs[t], workspace=wss[t])

    for t in range(n):
        worker(t, 2)
    torch.cuda.synchronize()
    best = None
    for _ in range(3):
        th = [threading.Thread(target=worker, args=(t, per)) for t in range(n)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for x in th:
            x.start()
        for x in th:
            x.join()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None or dt < best else best
    frames = per * n
    return {"frames_in_flight": n, "frames": frames, "ms_per_frame": best * 1e3 / frames, "frames_per_sec": frames / best,
            "samples_per_sec": blended_per_frame * frames / best}


def cpu_baseline(cfg, rays_fn, poses, budget_s=12.0):
    """Time the oracle (threaded build, all host cores) on whole frames of the same workload.  cfg: the workload's
    configuration (scene, step, K, ...); rays_fn(azimuth) -> (rays_o, rays_d) as numpy arrays."""
    from oracle import OracleScene
    s = cfg["scene"]
    frame = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    orc = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], s["weights"], s["occupancy"], threads=True)
    samples, t_total, frames = 0, 0.0, 0
    while t_total < budget_s and frames < 64: # whole frames, cycling through the poses, until the time budget is used
        o, d = rays_fn(poses[frames % len(poses)])
        t0 = time.perf_counter()
        _, n_eval, _, _ = orc.render(o, d, *frame)
        t_total += time.perf_counter() - t0
        samples += int(n_eval.sum())
        frames += 1
    # the one-thread build (the oracle as defined) on a sample of the rays of the first pose: a few seconds
    one = OracleScene(s["res"], s["aabb_min"], s["aabb_max"], s["hidden"], s["weights"], s["occupancy"], threads=False)
    o, d = rays_fn(poses[0])
    every = max(4, len(o) // 80000)
    t0 = time.perf_counter()
    _, n1, _, _ = one.render(o[::every], d[::every], *frame)
    t_one = time.perf_counter() - t0
    return {"value": samples / t_total, "unit": "samples/s", "cores": orc.num_threads(), "cpu_model": cpu_model(), "kind": "oracle",
            "sample": "%d whole %dx%d frame(s) of the same scene (%d blended samples, %.1f s)" %
                      (frames, cfg["width"], cfg["height"], samples, t_total),
            "frames_per_sec": frames / t_total,
            "one_thread": {"value": int(n1.sum()) / t_one, "unit": "samples/s", "cores": 1,
                           "sample": "every %dth ray of one frame (%d blended samples, %.1f s)" % (every, int(n1.sum()), t_one)}}


def isolated_mlp(kn, torch, wdtype, iters=10, skewed=False, layered=True):
    """cfg2: the grouped-MLP kernel on its own (2^22 uniform points, 16^3 networks), through kn_eval_grouped; or
    cfg4 (skewed): 2^23 points, 90 % of them in 5 % of the cells."""
    from kn_synth import configs
    cfg = configs.config4(wdtype=wdtype) if skewed else configs.config2(wdtype=wdtype)
    sc = cfg["scene"]
    dt = {"f16": torch.float16, "bf16": torch.bfloat16}[wdtype]
    scene = kn.Scene(sc["res"], sc["aabb_min"], sc["aabb_max"], sc["hidden"], torch.from_numpy(sc["weights"]).to(dt).cuda())
    pts, dirs = torch.from_numpy(cfg["points"]).cuda(), torch.from_numpy(cfg["dirs"]).cuda()
    M = pts.shape[0]
    out = (torch.empty(M, dtype=torch.float32, device="cuda"), torch.empty((M, 3), dtype=torch.float32, device="cuda"))
    for _ in range(3):
        scene.eval_grouped(pts, dirs, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(iters):
        scene.eval_grouped(pts, dirs, out=out)
    torch.cuda.synchronize()
    dt_s = time.perf_counter() - t0            # the whole call, no stage events on the stream
    kn.profile_enable(True)
    kn.profile_read(reset=True)
    for _ in range(iters):
        scene.eval_grouped(pts, dirs, out=out)
    torch.cuda.synchronize()
    prof = kn.profile_read(reset=True)         # the stages (the events add a few microseconds between them)
    kn.profile_enable(False)
    mlp_ms = prof["ms_mlp"] / iters
    tflops = FLOP_PER_SAMPLE[sc["hidden"]] * M / (mlp_ms * 1e-3) / 1e12
    # the same points handed over in grouped order (what the paper's own pipeline feeds its fused kernel after it has
    # physically re-ordered the batch): the kernel then reads positions and directions contiguously
    ids = scene.cell_ids(pts)
    order = torch.argsort(ids.to(torch.int64), stable=True)
    pts_g, dirs_g = pts[order].contiguous(), dirs[order].contiguous()
    for _ in range(2):
        scene.eval_grouped(pts_g, dirs_g, out=out)
    torch.cuda.synchronize()
    kn.profile_enable(True)
    kn.profile_read(reset=True)
    for _ in range(iters):
        scene.eval_grouped(pts_g, dirs_g, out=out)
    prof_g = kn.profile_read(reset=True)
    kn.profile_enable(False)
    mlp_ms_g = prof_g["ms_mlp"] / iters
    tflops_g = FLOP_PER_SAMPLE[sc["hidden"]] * M / (mlp_ms_g * 1e-3) / 1e12
    # the stage call on its own: kn_bucket on the same points' ids (a stable sort of (key, index) pairs)
    # (outputs and workspace allocated once, the library called directly: the host side must not be what is timed)
    b_counts = torch.empty(scene.N + 1, dtype=torch.int32, device="cuda")
    b_offsets = torch.empty(scene.N + 2, dtype=torch.int32, device="cuda")
    b_perm = torch.empty(M, dtype=torch.int32, device="cuda")
    b_ws = torch.empty(scene.workspace_bytes(max_points=M), dtype=torch.uint8, device="cuda")
    ctx_h = kn.default_context().h
    stream = torch.cuda.current_stream().cuda_stream

    def bucket_calls(n):
        for _ in range(n):
            rc = scene.L.kn_bucket(ctx_h, scene.h, stream, ids.data_ptr(), M, b_counts.data_ptr(), b_offsets.data_ptr(), b_perm.data_ptr(),
                                   b_ws.data_ptr(), b_ws.numel())
            assert rc == 0, rc
    bucket_calls(2)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    bucket_calls(4 * iters)
    torch.cuda.synchronize()
    bucket_stage_ms = (time.perf_counter() - t0) * 1e3 / (4 * iters)
    del b_ws, b_perm
    mlp_ms_l = None
    if layered:
        # the comparison point of Sec. 3.5: the same networks one layer at a time (grouped matrix products,
        # activations through device memory), on the grouped-order input
        import ctypes
        nbytes = ctypes.c_int64()
        scene.L.kn_layered_workspace_bytes(scene.h, M, ctypes.byref(nbytes))  # sized once, outside the timed calls
        ws_l = torch.empty(int(nbytes.value), dtype=torch.uint8, device="cuda")
        for _ in range(2):
            scene.eval_grouped_layered(pts_g, dirs_g, out=out, workspace=ws_l)
        torch.cuda.synchronize()
        kn.profile_enable(True)
        kn.profile_read(reset=True)
        for _ in range(iters):
            scene.eval_grouped_layered(pts_g, dirs_g, out=out, workspace=ws_l)
        prof_l = kn.profile_read(reset=True)
        kn.profile_enable(False)
        mlp_ms_l = prof_l["ms_mlp"] / iters
        del ws_l
    # Re-ordering stage (everything between the cell ids and the MLP kernel: two radix passes that move the samples,
    # their count tables and scans, offsets and tile list; and, after the MLP kernel, the copy of the staged results
    # into the caller's arrays).  Algorithmic bytes per point = what a physical re-ordering of the batch has to move
    # once: key 4 + position and direction 24 read, one 32-byte record written, results 16 read and 16 written = 92.
    # What the kernels really move is 164 (first pass 28 in, 36 out; second 36 in, 32 out; results 16 in, 16 out); the
    # figure a sort of indices alone would be charged with, 16 per key (the definition this line used while the stage
    # sorted indices), is kept beside it.  The scattered 16-byte store of each result is inside the MLP kernel's time.
    t_bucket = prof["ms_bucket"] / iters * 1e-3
    return {"workload": ("cfg4: 2^23 points, 90 %% in 5 %% of the cells, 16^3 networks, %s" if skewed else
                         "cfg2: 2^22 points, 16^3 networks, %s") % wdtype, "points": M, "points_per_sec": M / (dt_s / iters),
            "ms_eval_grouped": dt_s * 1e3 / iters, "ms_cell_ids": prof["ms_cell"] / iters,
            "ms_bucket": prof["ms_bucket"] / iters, "ms_mlp_kernel": mlp_ms,
            "mlp_evals_per_sec": M / (mlp_ms * 1e-3), "mlp_tflops": tflops, "mlp_frac_of_mfma_peak": tflops * 1e12 / PEAK_MFMA_16BIT,
            "grouped_order_input": {"ms_mlp_kernel": mlp_ms_g, "mlp_evals_per_sec": M / (mlp_ms_g * 1e-3), "mlp_tflops": tflops_g,
                                    "mlp_frac_of_mfma_peak": tflops_g * 1e12 / PEAK_MFMA_16BIT,
                                    "layer_at_a_time_ms": mlp_ms_l,
                                    "fused_speedup_over_layer_at_a_time": mlp_ms_l / mlp_ms_g if mlp_ms_l else None},
            "roofline_mlp": with_measured({"kernel": "k_mlp_mfma (fused grouped MLP), points in caller order", "bound": "mfma",
                                           "achieved": tflops, "peak": PEAK_MFMA_16BIT / 1e12, "unit": "TFLOP/s",
                                           "frac": tflops * 1e12 / PEAK_MFMA_16BIT, "traffic": None},
                                          "mfma_bf16_tflops" if wdtype == "bf16" else "mfma_f16_tflops"),
            "roofline_bucket": with_measured({"kernel": "k_reorder_scatter x2 + k_key_hist + k_digit_scan x2 + k_offsets_tiles "
                                                        "+ k_split_results (stable re-ordering of the samples by network, results back in caller order)",
                                              "bound": "hbm", "achieved": 92.0 * M / t_bucket / 1e9,
                                              "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                                              "frac": 92.0 * M / t_bucket / PEAK_HBM, "traffic": None,
                                              "bytes_per_point_algorithmic": 92, "bytes_per_point_moved": 164,
                                              "moved_gbps": 164.0 * M / t_bucket / 1e9},
                                             "hbm_copy_gbps"),
            "bucket_gbps_algorithmic": 92.0 * M / t_bucket / 1e9,
            "bucket_gbps_at_16_bytes_per_key": 16.0 * M / t_bucket / 1e9,
            # kn_bucket alone (index sort): key read by the count and by the scatter of each of the two passes, key and
            # index written by each scatter, index read by the second: counted as 16 B per key
            "kn_bucket_stage": with_measured({"kernel": "kn_bucket: k_ids_to_keys + (k_key_hist + k_digit_scan + k_index_scatter) x2 + k_offsets_tiles",
                                              "bound": "hbm", "ms": bucket_stage_ms, "achieved": 16.0 * M / (bucket_stage_ms * 1e-3) / 1e9,
                                              "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": 16.0 * M / (bucket_stage_ms * 1e-3) / PEAK_HBM,
                                              "traffic": None}, "hbm_copy_gbps"),
            "mlp_hbm_gbps_algorithmic": (32.0 + 16.0 + 16.0 + 16.0 + 3.5) * M / (mlp_ms * 1e-3) / 1e9}


def occupancy_extraction(kn, torch, scene, sc, occ_res, iters=5):
    """Occupancy grid extraction (the step that produces the grid the renderer skips with): 27 density probes per voxel
    of a grid of the workload's size, from the workload's own networks, tau as in the paper's Sec. 4.1."""
    import numpy as np
    out = torch.empty(tuple(occ_res), dtype=torch.uint8, device="cuda")
    for _ in range(2):
        scene.extract_occupancy(occ_res, 10.0, out=out)
    torch.cuda.synchronize()
    kn.profile_enable(True)
    kn.profile_read(reset=True)
    for _ in range(iters):
        scene.extract_occupancy(occ_res, 10.0, out=out)
    prof = kn.profile_read(reset=True)
    kn.profile_enable(False)
    H = sc["hidden"]
    probes = 27 * int(np.prod(occ_res))
    flop = 2 * (63 * H + H * H + H)          # layers 1 and 2 and the density row of layer 3
    ms = prof["ms_mlp"] / iters
    tf = flop * probes / (ms * 1e-3) / 1e12
    return {"workload": "%dx%dx%d voxels x 27 probes, %s networks of width %d, %s, tau = 10" %
                        (*occ_res, "x".join(str(r) for r in sc["res"]), H, sc["wdtype"]),
            "probes": probes, "ms_probe_kernel": ms, "ms_setup": prof["ms_setup"] / iters, "probes_per_sec": probes / (ms * 1e-3),
            "voxels_marked_frac": float(out.float().mean().item()),
            "roofline": {"kernel": "k_probe_mfma (density of the probe points)", "bound": "mfma", "achieved": tf,
                         "peak": PEAK_MFMA_16BIT / 1e12, "unit": "TFLOP/s", "frac": tf * 1e12 / PEAK_MFMA_16BIT, "traffic": None}
                        if not MEASURED else with_measured(
                            {"kernel": "k_probe_mfma (density of the probe points)", "bound": "mfma", "achieved": tf,
                             "peak": PEAK_MFMA_16BIT / 1e12, "unit": "TFLOP/s", "frac": tf * 1e12 / PEAK_MFMA_16BIT, "traffic": None},
                            "mfma_bf16_tflops" if sc["wdtype"] == "bf16" else "mfma_f16_tflops")}


def render_variant(kn, torch, scene, rays, args, out, steps, seeded):
    """Frames of a variant of the render (stratified sampling: a new seed per frame; or another scene): ms per frame
    without events, then the stages with events."""
    def frames(n):
        for i in range(n):
            scene.render(*rays[i % len(rays)], *args, out=out, seed=(1000 + i) if seeded else None)
    frames(4)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    frames(steps)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    kn.profile_enable(1)
    kn.profile_read(reset=True)
    frames(steps)
    prof = kn.profile_read(reset=True)
    kn.profile_enable(0)
    return {"ms_per_frame": ms, "frames_per_sec": 1e3 / ms,
            "stage_ms_per_frame": {k: prof[k] / steps for k in ("ms_setup", "ms_march", "ms_bucket", "ms_mlp", "ms_blend")},
            "samples_evaluated_per_frame": prof["mlp_samples"] / steps}


def sparse_grid(kn, torch, configs, poses, size, wdtype, steps):
    """A network grid finer than a dense scene may be (48^3 cells) with networks only in the cells that hold occupied
    voxels, same camera and lattice as the default workload."""
    cfg = configs.config_sparse(size, size, azimuth=poses[0], wdtype=wdtype)
    sc = cfg["scene"]
    dt = {"f16": torch.float16, "bf16": torch.bfloat16}[wdtype]
    scene = kn.Scene(sc["res"], sc["aabb_min"], sc["aabb_max"], sc["hidden"], torch.from_numpy(sc["weights"]).to(dt).cuda(),
                     torch.from_numpy(sc["occupancy"]).cuda(), cell_net=torch.from_numpy(sc["cell_net"]).cuda())
    rays = []
    for az in poses:
        o, d = configs.camera_rays(size, size, 40.0, 4.0, az, 30.0)
        rays.append((torch.from_numpy(o).cuda(), torch.from_numpy(d).cuda()))
    out = torch.empty((size * size, 3), dtype=torch.float32, device="cuda")
    res = render_variant(kn, torch, scene, rays, (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"]), out, steps,
                         False)
    res["workload"] = ("%dx%d render, %d networks (H=%d, %s) in a %s grid, %s occupancy grid (%.1f %% occupied), step diag/512, "
                       "eps 0.01, %d camera poses" % (size, size, len(sc["weights"]), sc["hidden"], wdtype,
                                                      "x".join(str(r) for r in sc["res"]),
                                                      "x".join(str(r) for r in sc["occupancy"].shape),
                                                      100.0 * sc["occupancy"].mean(), len(poses)))
    return res


def measure_render(kn, torch, np, configs, cfg, wdtype, steps, warmup, poses, traffic):
    """The whole path on one render workload: per-pose sample counts, then three passes of `steps` frames (all stage
    events / events around the dominant kernel only = the timed region / no events) -> dict of figures, and the
    objects the supplementary measurements go on with."""
    width, height = cfg["width"], cfg["height"]
    rays_fn = lambda az: configs.camera_rays(width, height, cfg.get("fov", 40.0), cfg.get("radius", 4.0), az, cfg.get("elevation", 30.0),
                                             **({"center": cfg["center"]} if "center" in cfg else {}))
    sc = cfg["scene"]
    dt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[wdtype]
    occ = sc["occupancy"]
    scene = kn.Scene(sc["res"], sc["aabb_min"], sc["aabb_max"], sc["hidden"], torch.from_numpy(sc["weights"]).to(dt).cuda(),
                     None if occ is None else torch.from_numpy(occ).cuda())
    rays = []
    for az in poses:
        o, d = rays_fn(az)
        rays.append((torch.from_numpy(o).cuda(), torch.from_numpy(d).cuda()))
    R = width * height
    out = torch.empty((R, 3), dtype=torch.float32, device="cuda")
    args = (cfg["t_near"], cfg["step"], cfg["K"], cfg["term_eps"], cfg["bg"])
    n_p = len(poses)

    stats = []  # per-pose sample counts (untimed)
    for o, d in rays:
        _, st = scene.render(o, d, *args, want_stats=True, out=out)
        stats.append(st)
    for i in range(warmup):
        scene.render(*rays[i % n_p], *args, out=out)
    torch.cuda.synchronize()

    def run_frames(profile_mode, every=1):
        kn.default_context().set_option(kn.OPT_PROFILE_EVERY, every)
        kn.profile_enable(profile_mode)
        kn.profile_read(reset=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            scene.render(*rays[i % n_p], *args, out=out)
        torch.cuda.synchronize()
        dt_ = time.perf_counter() - t0
        prof = kn.profile_read(reset=True)
        kn.profile_enable(0)
        kn.default_context().set_option(kn.OPT_PROFILE_EVERY, 1)
        return dt_, prof

    # untimed: frames with HIP events around every stage, to find the kernel that takes the most time
    _, prof_all = run_frames(1)
    stage_ms = {k: prof_all[k] for k in ("ms_setup", "ms_march", "ms_bucket", "ms_mlp", "ms_blend")}
    dominant = max(("ms_march", "ms_bucket", "ms_mlp", "ms_blend"), key=lambda k: stage_ms[k])
    # timed region: HIP events (recorded by the library on the stream it launches on) only around the dominant
    # kernel, so that the measurement disturbs the frame as little as possible
    # ... and only on one frame in EVENTS_EVERY (an event pair costs about 5 us on the stream): the kernel's average launch
    # is taken over the launches of those frames, the samples counted are theirs
    mode = {"ms_mlp": 2, "ms_march": 3}.get(dominant, 1)
    dt_s, prof = run_frames(mode, EVENTS_EVERY)
    dt_plain_s, _ = run_frames(0)  # the same frames without any events, for reference

    blended = sum(stats[i % n_p]["samples_blended"] for i in range(steps))
    evaluated = sum(stats[i % n_p]["samples_evaluated"] for i in range(steps))
    waves = sum(stats[i % n_p]["waves"] for i in range(steps))
    launches = waves  # one launch of each per-wave kernel per wave
    timed = range(0, steps, EVENTS_EVERY)  # the frames of the timed region that carried events
    timed_counts = {"evaluated": sum(stats[i % n_p]["samples_evaluated"] for i in timed),
                    "blended": sum(stats[i % n_p]["samples_blended"] for i in timed),
                    "launches": sum(stats[i % n_p]["waves"] for i in timed), "frames": len(timed)}
    all_counts = {"evaluated": evaluated, "blended": blended, "launches": launches, "frames": steps}
    H = sc["hidden"]
    f32 = wdtype == "f32"
    mfma_peak = PEAK_MFMA_F32 if f32 else PEAK_MFMA_16BIT
    mfma_key = {"f32": "mfma_f32_tflops", "f16": "mfma_f16_tflops", "bf16": "mfma_bf16_tflops"}[wdtype]

    def roof_mlp(p, n=None):
        n = n or all_counts
        s_ = p["ms_mlp"] * 1e-3
        tf = FLOP_PER_SAMPLE[H] * n["evaluated"] / s_ / 1e12 if s_ > 0 else 0.0
        r = {"kernel": "k_mlp_f32 (fused grouped MLP, fp32 MFMA)" if f32 else "k_mlp_mfma (fused grouped MLP)", "bound": "mfma",
             "achieved": tf, "peak": mfma_peak / 1e12, "unit": "TFLOP/s", "frac": tf * 1e12 / mfma_peak,
             "traffic": traffic.get("k_mlp_mfma"), "avg_launch_ms": p["ms_mlp"] / max(n["launches"], 1), "launches": n["launches"],
             "frames_with_events": n["frames"], "samples_per_launch": n["evaluated"] / max(n["launches"], 1),
             # the same kernel on the samples the method itself evaluates (those in front of the termination point)
             "achieved_on_blended_samples": tf * n["blended"] / max(n["evaluated"], 1)}
        r["flop_per_sample"] = FLOP_PER_SAMPLE[H]
        r["flop_per_sample_executed"] = FLOP_PER_SAMPLE[H] if f32 else FLOP_PER_SAMPLE_EXECUTED_16BIT[H]
        if not f32:
            # second view: its vector-ALU issue slots (counted in the generated code, transcendental instructions
            # twice) against what 1024 SIMDs can issue at 2.4 GHz, one slot per 4 cycles
            slots = VALU_SLOTS_PER_16_SAMPLES[H] / 16.0 * n["evaluated"]
            r["valu_issue_frac"] = slots / (s_ * 1024 * 2.4e9 / 4.0) if s_ > 0 else 0.0
        return with_measured(r, mfma_key)

    def roof_hbm(p, key, kernel, nbytes, traffic_key, n):
        s_ = p[key] * 1e-3
        return with_measured({"kernel": kernel, "bound": "hbm", "achieved": nbytes / s_ / 1e9 if s_ > 0 else 0.0,
                              "peak": PEAK_HBM / 1e9, "unit": "GB/s", "frac": nbytes / s_ / PEAK_HBM if s_ > 0 else 0.0,
                              "traffic": traffic.get(traffic_key), "avg_launch_ms": p[key] / max(n["launches"], 1),
                              "launches": n["launches"], "frames_with_events": n["frames"]}, "hbm_copy_gbps")

    def roof_march(p, n=None):
        n = n or all_counts
        # algorithmic bytes: 24 B per ray read + the packed occupancy grid read, once per frame, and 8 B (key,
        # record) written per kept sample
        occ_bytes = 0 if occ is None else int(np.prod(occ.shape)) / 8
        return roof_hbm(p, "ms_march", "k_march_wave (march + empty-space skipping)",
                        n["frames"] * (occ_bytes + 24.0 * R) + 8.0 * n["evaluated"], "k_march_wave", n)

    def roof_group(p):
        # algorithmic bytes: every sample's key is read twice (count, fill) and its slot number written: 12 B
        return roof_hbm(p, "ms_bucket", "k_group_pass (order-free grouping by network)", 12.0 * evaluated, "k_group_pass", all_counts)

    def roof_blend(p):
        # algorithmic bytes: 16 B read per evaluated sample, 12 B written per ray of the frame; the per-ray state of the
        # live rays (32 B per wave) is not credited here
        return roof_hbm(p, "ms_blend", "k_composite_wave / k_composite_group (blend, early termination)",
                        16.0 * evaluated + 12.0 * R * steps, "k_composite_wave", all_counts)

    roofline = (roof_mlp(prof, timed_counts) if dominant == "ms_mlp" else roof_march(prof, timed_counts) if dominant == "ms_march"
                else roof_mlp(prof_all))
    roofline["events_on_one_frame_in"] = EVENTS_EVERY
    res = {
        "value": blended / dt_s, "unit": "samples/s", "steps": steps, "warmup": warmup, "ms_per_step": dt_s * 1e3 / steps,
        "dtype": wdtype, "frames_per_sec": steps / dt_s,
        "ms_per_step_without_events": dt_plain_s * 1e3 / steps,
        "samples_blended_per_frame": blended / steps, "samples_evaluated_per_frame": evaluated / steps,
        "evaluated_over_blended": evaluated / max(blended, 1),
        "waves_per_frame": waves / steps,
        "stage_ms_per_frame": {k: v / steps for k, v in stage_ms.items()},
        "dominant_kernel_stage": dominant,
        "roofline": roofline,
        "roofline_mlp_all_events": roof_mlp(prof_all), "roofline_march_all_events": roof_march(prof_all),
        "roofline_group_all_events": roof_group(prof_all), "roofline_blend_all_events": roof_blend(prof_all),
    }
    return res, dict(scene=scene, rays=rays, args=args, out=out, R=R, rays_fn=rays_fn, blended_per_frame=blended / steps)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", default="cfg3", choices=["cfg3", "cfg5"],
                    help="cfg3: the 800x800 frame the headline metric is quoted on (default); cfg5: 1920x1080, 32^3 networks of "
                         "width 64, 512^3 occupancy grid, K = 1024 (the largest configuration; bf16 unless --wdtype is given)")
    ap.add_argument("--wdtype", default=None)
    ap.add_argument("--size", type=int, default=800, help="cfg3: frame width and height")
    ap.add_argument("--wave", default="", help="first_wave_samples,slots_per_ray,growth (experiment knob)")
    ap.add_argument("--in-flight", type=int, default=3,
                    help="frames in flight (one stream and host thread each) of the supplementary throughput pass; 0 = skip")
    ap.add_argument("--frames-only", action="store_true",
                    help="stop after the timed frames of the workload (no supplementary measurements): for counter runs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--bucket-only", action="store_true",
                    help="only the cfg2 eval_grouped calls (for counter runs on the re-ordering kernels)")
    ap.add_argument("--skewed", action="store_true", help="with --bucket-only: cfg4 (load skew) instead of cfg2")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path would shard by rays, every GPU holding the whole scene); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2103_13744_amd as kn
    from kn_synth import configs
    from paper_2103_13744_amd import peaks

    torch.cuda.set_device(0)
    kn.load_library(build_if_missing=True)
    if a.calibrate_copy:  # first, so that the counter runs find it as the largest copy dispatch whatever follows
        src_buf = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst_buf = torch.empty_like(src_buf)
        dst_buf.copy_(src_buf)
        torch.cuda.synchronize()
        del src_buf, dst_buf
    if a.bucket_only:
        r = isolated_mlp(kn, torch, a.wdtype or "f16", iters=4, skewed=a.skewed, layered=False)
        print(json.dumps({"isolated_mlp": r}))
        return
    if a.wave:
        kn.set_render_params(*[int(v) for v in a.wave.split(",")])
    if not a.frames_only:
        MEASURED.update(peaks.measure_peaks())
    poses = [45.0 * i for i in range(8)]
    if a.wdtype is None:
        a.wdtype = "f16" if a.workload == "cfg3" else "bf16"
    if a.workload == "cfg3":
        cfg = configs.config3(a.size, a.size, azimuth=poses[0], wdtype=a.wdtype)
        workload = ("cfg3: %dx%d render, 16^3 networks (H=32), 256^3 occupancy grid (8%% occupied), step diag/512, eps 0.01, "
                    "8 camera poses" % (a.size, a.size))
    else:
        cfg = configs.config5(azimuth=poses[0], wdtype=a.wdtype)
        workload = ("cfg5: 1920x1080 render, 32^3 networks (H=64), 512^3 occupancy grid (5% occupied), step diag/1024, "
                    "eps 0.01, 8 camera poses")
    default_workload = a.workload == "cfg3" and a.wdtype == "f16" and a.size == 800
    # (the committed counter summary is of the default workload)
    traffic, traffic_commit = read_traffic() if default_workload else ({}, None)
    m, ctx = measure_render(kn, torch, np, configs, cfg, a.wdtype, a.steps, a.warmup, poses, traffic)
    res = {"metric": "MLP sample evals/sec + frames/sec at 800x800", "value": m["value"], "unit": m["unit"], "n_gpus": 1,
           "steps": a.steps, "warmup": a.warmup, "ms_per_step": m["ms_per_step"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": a.wdtype, "data": "synthetic", "config": {"workload": workload}}
    res.update({k: v for k, v in m.items() if k not in res})
    if traffic:
        res["roofline"]["traffic_source"] = {"file": TRAFFIC_FILE, "measured_at_commit": traffic_commit,
                                             "note": "rocprofv3 FETCH_SIZE / WRITE_SIZE runs of this command, not re-measured in this run"}
    if MEASURED:
        res["measured_peaks"] = dict(MEASURED, note="micro-benchmarks of this GPU (csrc/kn_peaks.hip): plain 1 GiB copy (read + written), "
                                                    "read-only sweep, register-only MFMA / FMA / sine loops")
    scene, rays, args, out, R = ctx["scene"], ctx["rays"], ctx["args"], ctx["out"], ctx["R"]
    sc = cfg["scene"]
    if a.in_flight > 1 and not a.frames_only:
        res["frames_in_flight"] = frames_in_flight(torch, scene, rays, args, R, a.steps, a.in_flight, ctx["blended_per_frame"])
    if a.wdtype in ("f16", "bf16") and a.workload == "cfg3" and not a.frames_only:
        # the same frames with stratified sampling (Sec. 3.4), a new seed per frame
        res["stratified_sampling"] = render_variant(kn, torch, scene, rays, args, out, a.steps, True)
        res["occupancy_extraction"] = occupancy_extraction(kn, torch, scene, sc, sc["occupancy"].shape)
        res["sparse_grid"] = sparse_grid(kn, torch, configs, poses, a.size, a.wdtype, a.steps)
    del scene, ctx
    torch.cuda.empty_cache()
    if default_workload and not a.frames_only:
        # the other workloads of the benchmark's configuration list, shorter: cfg1 (tiny fp32 render), cfg2 (isolated
        # grouped MLP), cfg4 (load skew), cfg5 (large render, 8 frames, no CPU leg)
        others = {}
        c1 = dict(configs.config1(), radius=2.5, elevation=20.0, center=(0.5, 0.5, 0.5))
        others["cfg1"], _ = measure_render(kn, torch, np, configs, c1, "f32", a.steps, 4, [30.0], {})
        others["cfg1"]["workload"] = "cfg1: 64x64 render, 2^3 networks (H=32), fp32, 32 samples per ray, no occupancy grid, no termination"
        others["cfg2"] = isolated_mlp(kn, torch, "f16")
        others["cfg4"] = isolated_mlp(kn, torch, "bf16", iters=5, skewed=True, layered=False)
        torch.cuda.empty_cache()
        c5 = configs.config5(azimuth=poses[0], wdtype="bf16")
        others["cfg5"], c5ctx = measure_render(kn, torch, np, configs, c5, "bf16", 8, 2, poses, {})
        others["cfg5"]["workload"] = ("cfg5: 1920x1080 render, 32^3 networks (H=64), 512^3 occupancy grid (5% occupied), step diag/1024, "
                                      "eps 0.01, bf16, 8 camera poses, 8 frames")
        del c5ctx
        torch.cuda.empty_cache()
        res["other_workloads"] = others
        res["isolated_mlp"] = others["cfg2"]
    if not a.no_cpu_baseline and not a.frames_only:
        res["cpu_baseline"] = cpu_baseline(cfg, ctx_rays_fn(configs, cfg), poses)
    print(json.dumps(res))


def ctx_rays_fn(configs, cfg):
    return lambda az: configs.camera_rays(cfg["width"], cfg["height"], 40.0, 4.0, az, 30.0)


if __name__ == "__main__":
    main()
