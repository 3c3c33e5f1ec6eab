"""Benchmark of the pxr hot path on one MI355X.

One "step" = one pxr_render_batch call over the whole batch of the headline
workload (all frames of all environments), inputs already resident in HBM.
Prints ONE JSON line: rendered frames/s, the ALU roofline fraction of the
render kernel (timed live with HIP events on the launch stream), the HBM
figure next to it, and the CPU oracle timed on the host cores on a bounded
sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--envs B] [--threads NT]
"""
import argparse
import json
import os
import sys
import threading
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2502_00021_amd import workloads  # noqa: E402

# MI355X: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz = 39.32 T lane-operations/s for
# plain (non-packed) VALU work, one fp32 FMA or one integer op per lane per cycle.  The
# published 157.3 TFLOP/s fp32 vector figure is this x 2 (FMA) x 2 (packed), which an
# integer-heavy, order-fixed path cannot use.
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12
HBM_PEAK_GBS = 8000.0

# HBM bytes per launch, measured with two rocprofv3 --pmc passes (FETCH_SIZE x 2.000 + WRITE_SIZE x
# 1.000, the factors a plain 1 GiB copy gives for the same counters); see profiles/.  Others: null.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {("cfg5", 65536): 2516.8e6, ("cfg4", 16384): 403.5e6}


def algorithmic_ops_per_frame(V, T, npix, mode):
    """Lane-operations per frame that the method itself prescribes.

    Counted from the operation list of the specification, not from the kernel's
    instruction stream (an IEEE fp32 division counts as 10, memory and address
    work as 0): 39 per template vertex, 40 per triangle (gather, box,
    pixel-range test, area sign), 46 per pixel (ground ray, z-resolve, colour,
    quantise, pack), plus 9 per pixel with a distractor bound.  The
    data-dependent raster term (a few percent) is left out, which can only
    understate the achieved figure.
    """
    per_pixel = 46 + (9 if mode in ("color", "video") else 0)
    return 39 * V + 40 * T + per_pixel * npix


def algorithmic_bytes_per_frame(K, npix, mode, has_shapes, S):
    b = K * 28 + 3 * npix
    if has_shapes:
        b += K * 16 / S
    if mode == "video":
        b += 3 * npix
    return b


def cpu_baseline(w, budget_frames_1core=6144, budget_frames_per_thread=6144):
    """The oracle as it stands on the host cores: 1 core, then one single-threaded instance per core."""
    from oracle import orc
    scene = orc.Scene(w["desc"])
    S = w["poses"].shape[1]
    B = w["poses"].shape[0]

    def run(e0, e1):
        sh = None if w["shapes"] is None else w["shapes"][e0:e1]
        scene_local = orc.Scene(w["desc"])
        scene_local.render(w["poses"][e0:e1], sh, step0=0, env0=e0, distractor=w["distractor"], want_ids=False)

    n1 = max(1, min(B, budget_frames_1core // S))
    t0 = time.perf_counter()
    run(0, n1)
    t1 = time.perf_counter() - t0
    one_core = n1 * S / t1
    cores = len(os.sched_getaffinity(0))
    per = max(1, min(B // cores, budget_frames_per_thread // S))
    threads = [threading.Thread(target=run, args=(i * per, (i + 1) * per)) for i in range(cores)]
    t0 = time.perf_counter()
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    tn = time.perf_counter() - t0
    del scene
    return {"value": cores * per * S / tn, "unit": "frames/s", "cores": cores, "kind": "oracle",
            "sample": f"{cores} single-threaded oracle instances x {per} envs x {S} steps of the same workload "
                      f"(disjoint env slices); 1 core alone: {one_core:.1f} frames/s on the first {n1} envs",
            "value_1core": one_core}


def time_next_stages(torch, pxr, w, reps=10):
    """The stages in front of and behind the renderer on the headline workload: joint angles -> poses
    (pxr_pose_batch) and frame stack -> first conv layer of the policy (pxr_conv_forward, matrix cores), each
    timed on its own with HIP events, and the three enqueued back to back (angles in, features out)."""
    fk = w["fk"]
    scene = pxr.Scene(w["desc"])
    scene.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    dis = w["distractor"]
    if dis is not None:
        d = dict(dis)
        if d["mode"] == "video":
            d["video"] = torch.from_numpy(d["video"]).cuda()
        scene.apply_distractor(d)
    free = torch.from_numpy(fk["free_poses"]).cuda()
    ang = torch.from_numpy(fk["angles"]).cuda()
    shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
    B, S = free.shape[0], free.shape[1]
    K = scene.K
    poses = torch.empty((B, S, K, 7), dtype=torch.float32, device="cuda")
    frames = torch.empty((B, S, scene.H, scene.W, 3), dtype=torch.uint8, device="cuda")
    rng = np.random.default_rng(0)
    conv = pxr.Conv(scene.H, scene.W, S, (rng.standard_normal((3, 3, 3 * S, 32)) * 0.1).astype(np.float32),
                    np.zeros(32, np.float32))
    feat = torch.empty((B, conv.Ho, conv.Wo, 32), dtype=torch.bfloat16, device="cuda")

    def timed(fn):
        for _ in range(2):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    ms_fk = timed(lambda: scene.pose_batch(free, ang, poses=poses))
    scene.render_batch(poses, shapes, frames=frames)
    ms_conv = timed(lambda: conv.forward(frames, out=feat))

    def whole():
        scene.render_batch_kinematic(free, ang, shapes, poses=poses, frames=frames)
        conv.forward(frames, out=feat)

    ms_all = timed(whole)
    n = B * S
    fk_bytes = 4 * (free[0, 0].numel() + ang[0, 0].numel() + K * 7) * n
    conv_bytes = frames.numel() + feat.numel() * 2
    conv_flops = 2.0 * B * conv.Ho * conv.Wo * 32 * 27 * S
    pk = pxr.measure_peaks()
    # the time this machine's HBM needs for the layer's bytes: reads at its read-stream rate plus writes at its write-stream rate
    conv_bound_ms = 1e3 * (frames.numel() / (pk["read_gbs"] * 1e9) + feat.numel() * 2 / (pk["write_gbs"] * 1e9))
    out = {
        "kinematics-" + w["name"]: {"kernel": "fk_kernel", "avg_launch_ms": ms_fk, "frames_per_s": n / (1e-3 * ms_fk),
                                   "roofline": {"bound": "hbm", "achieved": fk_bytes / ms_fk / 1e6, "peak": HBM_PEAK_GBS,
                                                "unit": "GB/s", "frac": fk_bytes / ms_fk / 1e6 / HBM_PEAK_GBS}},
        "conv-consumer-" + w["name"]: {"kernel": "conv_kernel", "avg_launch_ms": ms_conv,
                                      "stacks_per_s": B / (1e-3 * ms_conv), "frames_per_s": n / (1e-3 * ms_conv),
                                      "tflops_bf16": conv_flops / ms_conv / 1e9,
                                      "roofline": {"bound": "hbm", "achieved": conv_bytes / ms_conv / 1e6,
                                                   "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                                   "frac": conv_bytes / ms_conv / 1e6 / HBM_PEAK_GBS,
                                                   "algorithmic_bytes_per_stack": conv_bytes / B,
                                                   "measured_stream_bound_ms": conv_bound_ms,
                                                   "frac_of_measured_stream_bound": conv_bound_ms / ms_conv}},
        "angles-to-features-" + w["name"]: {"ms_per_step": ms_all, "frames_per_s": n / (1e-3 * ms_all),
                                           "kernels": "fk_kernel + render_kernel + conv_kernel on one stream"},
    }
    conv.close()
    scene.close()
    return out


def time_small_batch_graph(torch, pxr, reps=200):
    """A launch-bound step (cfg2: 256 environments; angles -> poses -> frames -> conv features = three small
    kernels) enqueued eagerly and replayed from a HIP graph captured once."""
    w = workloads.make(2)
    fk = w["fk"]
    scene = pxr.Scene(w["desc"])
    scene.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    rng = np.random.default_rng(0)
    conv = pxr.Conv(scene.H, scene.W, 1, (rng.standard_normal((3, 3, 3, 32)) * 0.1).astype(np.float32), np.zeros(32, np.float32))
    free = torch.from_numpy(fk["free_poses"]).cuda()
    ang = torch.from_numpy(fk["angles"]).cuda()
    B = free.shape[0]
    poses = torch.empty((B, 1, scene.K, 7), dtype=torch.float32, device="cuda")
    frames = torch.empty((B, 1, scene.H, scene.W, 3), dtype=torch.uint8, device="cuda")
    feat = torch.empty((B, conv.Ho, conv.Wo, 32), dtype=torch.bfloat16, device="cuda")

    def step():
        scene.render_batch_kinematic(free, ang, None, poses=poses, frames=frames)
        conv.forward(frames, out=feat)

    def wall(fn):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return 1e6 * (time.perf_counter() - t0) / reps

    us_eager = wall(step)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    us_graph = wall(graph.replay)
    conv.close()
    scene.close()
    return {"small-batch-step-" + w["name"]: {"envs": B, "us_per_step_eager": us_eager, "us_per_step_hip_graph": us_graph,
                                            "frames_per_s_hip_graph": B / (1e-6 * us_graph),
                                            "kernels": "fk_kernel + render_kernel + conv_kernel, wall clock per step"}}


def time_paper_loop(torch, pxr, env_counts=(1, 10, 100, 1000, 10000), seconds=0.25):
    """The shape of the paper's throughput experiment (its steps-per-second figure): for each of its four
    environments (stand-in skeletons) and each number of parallel environments, one step = joint angles ->
    poses -> one 64x64 frame per environment -> one convolutional layer, all on the device, physics left out.
    Steps are enqueued back to back and the clock stops after a final synchronisation."""
    out = {}
    rng = np.random.default_rng(0)
    wgt = (rng.standard_normal((3, 3, 3, 32)) * 0.1).astype(np.float32)
    for name, make in workloads.PAPER_ENVIRONMENTS.items():
        row = {}
        for n in env_counts:
            w = make(n)
            fk = w["fk"]
            scene = pxr.Scene(w["desc"])
            scene.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
            conv = pxr.Conv(scene.H, scene.W, 1, wgt, np.zeros(32, np.float32))
            free = torch.from_numpy(fk["free_poses"]).cuda()
            ang = torch.from_numpy(fk["angles"]).cuda()
            poses = torch.empty((n, 1, scene.K, 7), dtype=torch.float32, device="cuda")
            frames = torch.empty((n, 1, scene.H, scene.W, 3), dtype=torch.uint8, device="cuda")
            feat = torch.empty((n, conv.Ho, conv.Wo, 32), dtype=torch.bfloat16, device="cuda")

            def run(k):
                for i in range(k):
                    scene.render_batch_kinematic(free, ang, None, step0=i, poses=poses, frames=frames)
                    conv.forward(frames, out=feat)
                torch.cuda.synchronize()

            run(20)
            t0 = time.perf_counter()
            run(50)
            per = (time.perf_counter() - t0) / 50
            k = max(50, min(5000, int(seconds / per)))
            t0 = time.perf_counter()
            run(k)
            dt = time.perf_counter() - t0
            row[str(n)] = {"env_steps_per_s": n * k / dt, "iterations_per_s": k / dt}
            conv.close()
            scene.close()
        out[name] = row
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--envs", type=int, default=None, help="override the number of environments")
    ap.add_argument("--threads", type=int, default=0, help="threads per frame workgroup (0 = library default)")
    ap.add_argument("--no-distractor", action="store_true")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy kernel (the known-size reference that "
                         "scales the FETCH_SIZE / WRITE_SIZE counters of a profiler run)")
    ap.add_argument("--next-stages-only", action="store_true",
                    help="time only the kinematics and conv-consumer stages of the chosen workload (for profiler runs)")
    ap.add_argument("--extras", action="store_true", help="also time the other configurations (reported under 'others')")
    ap.add_argument("--profile-lib", default=None, metavar="FILE",
                    help="profiling only: load this build of the library (paper_2502_00021_amd/build.py --define ... --out FILE) "
                         "instead of the in-tree one; the numbers of such a run are not the product's")
    ap.add_argument("--phase-clocks", action="store_true",
                    help="with --profile-lib naming a build made with --define PXR_PHASE_TIMING: "
                         "report the shader-clock ticks per frame a workgroup spends in each phase of the render kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build renders on ONE GPU (environments are independent, so B shards trivially "
                 "across GPUs with no exchange, but no multi-GPU run is part of it); use --gpus 1")

    import torch
    from paper_2502_00021_amd import pxr

    if args.profile_lib:
        pxr.use_library_file(args.profile_lib)
    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)

    if args.calibrate_copy:
        n = 1 << 30
        src = torch.full((n,), 7, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": 3}))
        return

    def time_workload(cfg, envs, steps, warmup, distract=True, threads=0):
        w = workloads.make(cfg, B=envs)
        scene = pxr.Scene(w["desc"])
        if threads:
            scene.set_block_threads(threads)
        dis = w["distractor"] if distract else None
        mode = "none" if dis is None else dis["mode"]
        if dis is not None:
            d = dict(dis)
            if mode == "video":
                d["video"] = torch.from_numpy(d["video"]).cuda()
            scene.apply_distractor(d)
        poses = torch.from_numpy(w["poses"]).cuda()
        shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
        B, S, K = poses.shape[0], poses.shape[1], poses.shape[2]
        frames = torch.empty((B, S, scene.H, scene.W, 3), dtype=torch.uint8, device="cuda")
        for i in range(warmup):
            scene.render_batch(poses, shapes, step0=i, frames=frames)
        torch.cuda.synchronize()
        if args.phase_clocks:
            import ctypes
            L = pxr.lib()
            if not hasattr(L, "pxr_debug_phase_cycles"):
                sys.exit("bench.py --phase-clocks: the loaded library is not a PXR_PHASE_TIMING build (give one with --profile-lib)")
            L.pxr_debug_phase_cycles.argtypes = [ctypes.c_void_p, ctypes.c_int]
            L.pxr_debug_wave_arrival.argtypes = [ctypes.c_void_p]
            scratch = (ctypes.c_ulonglong * 128)()
            L.pxr_debug_phase_cycles(None, 1)
            L.pxr_debug_wave_arrival(scratch)  # (reading resets)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        ev[0].record()
        for i in range(steps):
            scene.render_batch(poses, shapes, step0=warmup + i, frames=frames)
            ev[i + 1].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        kernel_ms = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
        info = scene.info()
        res = dict(w=w, B=B, S=S, K=K, H=scene.H, W=scene.W, mode=mode, wall=wall, kernel_ms=kernel_ms, info=info,
                   checksum=int(frames[:: max(1, B // 64)].to(torch.int64).sum().item()))
        if args.phase_clocks:
            names = ["0 setup", "1 vertices", "2a coarse", "2b exact", "key clear", "3 raster", "4 resolve"]
            out = (ctypes.c_ulonglong * 16)()
            L.pxr_debug_phase_cycles(out, 0)
            n = float(steps * B * S)
            res["phase_clocks"] = {"ticks_per_frame": {nm: out[i] / n for i, nm in enumerate(names)}}
            L.pxr_debug_wave_arrival(scratch)
            if any(scratch):  # only a PXR_WAVE_ARRIVAL build fills these
                res["phase_clocks"]["wave_arrival_after_first"] = {
                    nm: [scratch[i * 16 + k] / n for k in range(16)] for i, nm in enumerate(names[:6])}
        scene.close()
        del frames, poses, shapes
        return res

    cfg = int(args.workload[3:])
    if args.next_stages_only:
        print(json.dumps(time_next_stages(torch, pxr, workloads.make(cfg, B=args.envs), reps=args.steps)))
        return
    r = time_workload(cfg, args.envs, args.steps, args.warmup, not args.no_distractor, args.threads)
    n_frames = r["B"] * r["S"]
    ms_per_step = 1e3 * r["wall"] / args.steps
    value = n_frames * args.steps / r["wall"]
    avg_kernel_s = 1e-3 * float(np.mean(r["kernel_ms"]))
    V, T, npix = r["info"]["n_verts"], r["info"]["n_tris"], r["H"] * r["W"]
    ops = algorithmic_ops_per_frame(V, T, npix, r["mode"]) * n_frames
    byts = algorithmic_bytes_per_frame(r["K"], npix, r["mode"], r["w"]["shapes"] is not None, r["S"]) * n_frames
    achieved_tops = ops / avg_kernel_s / 1e12
    out = {
        "metric": "rendered frames/sec (envs x steps) at 64x64 RGB",
        "value": value, "unit": "frames/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32+i32 -> u8", "data": "synthetic",
        "config": {"workload": r["w"]["name"], "envs": r["B"], "steps_per_call": r["S"], "image": [r["H"], r["W"], 3],
                   "bodies": r["K"], "vertices_per_frame": V, "triangles_per_frame": T, "distractor": r["mode"],
                   "block_threads": r["info"]["block_threads"], "lds_bytes_per_frame": r["info"]["lds_bytes"],
                   "frames_per_step": n_frames},
        "roofline": {"bound": "alu", "achieved": achieved_tops, "peak": ALU_PEAK_TOPS, "unit": "Tlane-op/s",
                     "frac": achieved_tops / ALU_PEAK_TOPS, "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get((args.workload, r["B"])),
                     "kernel": "render_kernel", "avg_launch_ms": 1e3 * avg_kernel_s,
                     "algorithmic_ops_per_frame": ops // n_frames,
                     "hbm": {"achieved": byts / avg_kernel_s / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                             "frac": byts / avg_kernel_s / 1e9 / HBM_PEAK_GBS,
                             "algorithmic_bytes_per_frame": byts / n_frames}},
        "kernel_frames_per_s": n_frames / avg_kernel_s,
        "checksum": r["checksum"],
    }
    if "phase_clocks" in r:
        out["phase_clocks"] = r["phase_clocks"]  # (a profiling build: `value` is not the product's rate)
    if args.extras:
        # the same fractions against what this GPU sustains right now (microbenchmarks in the library)
        pk = pxr.measure_peaks()
        out["measured_peaks"] = dict(pk, alu_frac_of_measured_fma=achieved_tops / pk["fma_tlaneops"],
                                     hbm_frac_of_measured_copy=out["roofline"]["hbm"]["achieved"] / pk["copy_gbs"])
        others = {}
        others.update(time_next_stages(torch, pxr, r["w"]))
        others.update(time_small_batch_graph(torch, pxr))
        out["paper_loop_steps_per_s"] = time_paper_loop(torch, pxr)
        for name, c, envs, dis in [("cfg2-chain-64", 2, 256, True), ("cfg3-quadruped-64-colour", 3, 4096, True),
                                   ("cfg3-quadruped-64-no-distractor", 3, 4096, False),
                                   ("cfg4-humanoid-84-video", 4, 16384, True),
                                   ("cfg4-humanoid-84-no-distractor", 4, 16384, False),
                                   ("cfg5-humanoid-box-64-stack3-16384envs", 5, 16384, True)]:
            o = time_workload(c, envs, 10, 2, dis)
            others[name] = {"frames_per_s": o["B"] * o["S"] / (1e-3 * float(np.mean(o["kernel_ms"]))),
                            "avg_launch_ms": float(np.mean(o["kernel_ms"]))}
        out["others"] = others
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(r["w"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
