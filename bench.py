"""Benchmark of the pxr hot path on one MI355X.

One "step" = one pxr_render_batch call over the whole batch of the headline workload (all frames of all
environments), inputs already resident in HBM.  Prints ONE JSON line:

  value / roofline    rendered frames/s of the headline workload and the render kernel's fraction of the ALU
                      roofline, the kernel timed live with HIP events on the launch stream
  configs             the other configurations at their full sizes (frames/s, launch time, ALU and HBM fractions),
                      the target point "64x64 at 16 384 environments", the distractor-on / distractor-off ratios,
                      larger frames, and the stages around the renderer (kinematics, conv consumer, the overlapped
                      render + conv pipeline); the two launch-bound configurations also by wall clock over launches
                      made back to back and over the same launches replayed from a HIP graph; the same figures,
                      flat, under config["others.*"]
  env_sweep           the paper's throughput figure on this path: angles -> poses -> frames -> conv features of the
                      headline scene over 1 .. 10 000 parallel environments, launches back to back and as a HIP graph
  measured_peaks      what this GPU sustains right now (dependent-free FMA loop, integer mad loop, copy / read /
                      write streams), and the headline fractions against those
  cpu_baseline        the CPU oracle on the host cores, on a bounded sample of the headline workload

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5] [--envs B] [--threads NT]
                    [--no-others] [--no-cpu]
Profiling aids (not the product's numbers): --profile-lib FILE [--phase-clocks], --calibrate-copy, --only STAGE.
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

# Figures that only a profiler run can give, copied from the summaries under profiles/ (each names its
# command): HBM bytes per launch from two rocprofv3 --pmc passes (FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, the
# factors a plain 1 GiB copy gives for the same counters), and the counter-side view of the vector units
# (share of issue slots busy, share of lanes active per instruction, wave-instructions per frame).
PROFILED = {
    ("cfg5", 65536): {"traffic_bytes_per_launch": 2516.8e6, "valu_busy": 0.908, "lane_use": 0.825,
                      "valu_wave_instructions_per_frame": 9933,
                      "source": "profiles/render_kernel_cfg5_humanoid_box_64x64.md"},
    ("cfg4", 16384): {"traffic_bytes_per_launch": 403.5e6, "valu_busy": 0.795, "lane_use": 0.823,
                      "valu_wave_instructions_per_frame": 14651,
                      "source": "profiles/render_kernel_cfg4_humanoid_84x84_video.md"},
}

OP_CONVENTION = ("algorithmic lane-operations per frame = 39 per template vertex + 40 per triangle + 46 per pixel "
                 "(+9 with a distractor), counted from the method's operation list: an IEEE fp32 division counts as "
                 "10 (its cost on this ISA), loads, stores and addressing as 0, the data-dependent raster term is "
                 "left out; with a division counted as 1 the figures are 0.87x these")


def algorithmic_ops_per_frame(V, T, npix, mode):
    """Lane-operations per frame that the method itself prescribes (see OP_CONVENTION)."""
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
    return {"value": cores * per * S / tn, "unit": "frames/s", "cores": cores, "kind": "oracle",
            "sample": f"{cores} single-threaded oracle instances x {per} envs x {S} steps of the same workload "
                      f"(disjoint env slices); 1 core alone: {one_core:.1f} frames/s on the first {n1} envs",
            "value_1core": one_core}


def _bind(torch, scene, dis):
    if dis is None:
        return "none"
    d = dict(dis)
    if d["mode"] == "video":
        d["video"] = torch.from_numpy(d["video"]).cuda()
    scene.apply_distractor(d)
    return d["mode"]


def _event_ms(torch, fn, reps, warm=2):
    """Mean time of fn() in ms by HIP events on torch's current stream (the stream fn launches on)."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def time_env_sweep(torch, pxr, workloads, cfg, sizes=(1, 10, 100, 1000, 10000), launches=32):
    """The paper's throughput figure (its section 2: steps per second of the whole loop over 1 to 1000 parallel
    environments, a conv forward at the end of every step) on this path: joint angles -> poses -> frames -> conv
    features of the headline scene for B environments, `launches` steps made back to back on one stream (wall
    clock), and the same steps recorded once in a HIP graph and replayed."""
    import time
    out = {}
    for B in sizes:
        w = workloads.make(cfg, B=B)
        fk = w["fk"]
        scene = pxr.Scene(w["desc"])
        scene.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
        _bind(torch, scene, w["distractor"])
        free = torch.from_numpy(fk["free_poses"]).cuda()
        ang = torch.from_numpy(fk["angles"]).cuda()
        shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
        S = free.shape[1]
        poses = torch.empty((B, S, scene.K, 7), dtype=torch.float32, device="cuda")
        frames = torch.empty((B, S, scene.H, scene.W, 3), dtype=torch.uint8, device="cuda")
        rng = np.random.default_rng(0)
        conv = pxr.Conv(scene.H, scene.W, S, (rng.standard_normal((3, 3, 3 * S, 32)) * 0.1).astype(np.float32),
                        np.zeros(32, np.float32))
        feat = torch.empty((B, conv.Ho, conv.Wo, 32), dtype=torch.bfloat16, device="cuda")
        side = torch.cuda.Stream()  # (default priority; capture needs a stream of its own)

        def steps():
            for i in range(launches):
                scene.render_batch_kinematic(free, ang, shapes, step0=i, poses=poses, frames=frames)
                conv.forward(frames, out=feat)

        def wall(fn, reps=5):
            fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) / (reps * launches)

        with torch.cuda.stream(side):
            t_eager = wall(steps)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            steps()
        t_graph = wall(graph.replay)
        out[str(B)] = {"envs": B, "frames_per_step": B * S, "frames_per_s": B * S / t_eager,
                       "frames_per_s_graph_replay": B * S / t_graph, "us_per_step": 1e6 * t_eager,
                       "us_per_step_graph_replay": 1e6 * t_graph}
        del graph
        conv.close()
        scene.close()
    return out


def time_next_stages(torch, pxr, w, reps=10, chunks=(2, 4, 8)):
    """The stages in front of and behind the renderer on the headline workload: joint angles -> poses
    (pxr_pose_batch) and frame stack -> first conv layer of the policy (pxr_conv_forward, matrix cores), each
    timed on its own with HIP events; the three enqueued back to back on one stream; and the same step with the
    render and the conv layer overlapped chunk by chunk on two streams (pxr_pipeline_step)."""
    fk = w["fk"]
    scene = pxr.Scene(w["desc"])
    scene.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    _bind(torch, scene, w["distractor"])
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

    ms_fk = _event_ms(torch, lambda: scene.pose_batch(free, ang, poses=poses), reps)
    ms_render = _event_ms(torch, lambda: scene.render_batch(poses, shapes, frames=frames), reps)
    ms_conv = _event_ms(torch, lambda: conv.forward(frames, out=feat), reps)

    def serial():
        scene.render_batch_kinematic(free, ang, shapes, poses=poses, frames=frames)
        conv.forward(frames, out=feat)

    ms_serial = _event_ms(torch, serial, reps)
    check = feat[:: max(1, B // 256)].clone()
    overlapped = {}
    for n in chunks:
        pipe = pxr.Pipeline(scene, conv, n)

        def piped():
            scene.pose_batch(free, ang, poses=poses)
            pipe.step(poses, shapes, frames, feat)

        overlapped[n] = _event_ms(torch, piped, reps)
        assert torch.equal(check.view(torch.int16), feat[:: max(1, B // 256)].view(torch.int16)), "pipeline output differs"
        pipe.close()
    best = min(overlapped, key=overlapped.get)
    n = B * S
    fk_bytes = 4 * (free[0, 0].numel() + ang[0, 0].numel() + K * 7) * n
    conv_bytes = frames.numel() + feat.numel() * 2
    conv_flops = 2.0 * B * conv.Ho * conv.Wo * 32 * 27 * S
    out = {
        "kinematics": {"kernel": "fk_kernel", "avg_launch_ms": ms_fk, "frames_per_s": n / (1e-3 * ms_fk),
                       "bound": "hbm", "hbm_gbs": fk_bytes / ms_fk / 1e6, "hbm_frac": fk_bytes / ms_fk / 1e6 / HBM_PEAK_GBS},
        "conv_consumer": {"kernel": "conv_kernel", "avg_launch_ms": ms_conv, "stacks_per_s": B / (1e-3 * ms_conv),
                          "frames_per_s": n / (1e-3 * ms_conv), "tflops_bf16": conv_flops / ms_conv / 1e9,
                          "bound": "hbm", "hbm_gbs": conv_bytes / ms_conv / 1e6,
                          "hbm_frac": conv_bytes / ms_conv / 1e6 / HBM_PEAK_GBS,
                          "algorithmic_bytes_per_stack": conv_bytes / B},
        "angles_to_features": {"render_alone_ms": ms_render, "serial_ms": ms_serial,
                               "overlapped_ms": overlapped[best], "overlap_chunks": best,
                               "overlapped_ms_by_chunks": {str(k): v for k, v in overlapped.items()},
                               "frames_per_s_serial": n / (1e-3 * ms_serial),
                               "frames_per_s_overlapped": n / (1e-3 * overlapped[best]),
                               "kernels": "fk_kernel + render_kernel + conv_kernel; overlapped = pxr_pipeline_step "
                                          "(chunk c's conv layer on a second stream beside chunk c+1's render)"},
    }
    conv.close()
    scene.close()
    return out


def _round(x, sig=4):
    if isinstance(x, float):
        return float(f"{x:.{sig}g}")
    if isinstance(x, dict):
        return {k: _round(v, sig) for k, v in x.items()}
    if isinstance(x, list):
        return [_round(v, sig) for v in x]
    return x


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
    ap.add_argument("--envs", type=int, default=None, help="override the number of environments")
    ap.add_argument("--size", type=int, default=None, help="override the frame's width and height")
    ap.add_argument("--threads", type=int, default=0, help="threads per frame workgroup (0 = library default)")
    ap.add_argument("--no-distractor", action="store_true")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-others", action="store_true", help="only the headline workload (no 'configs' block, no peaks)")
    ap.add_argument("--extras", action="store_true", help=argparse.SUPPRESS)  # (the 'configs' block is the default now)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device-to-device copy kernel (the known-size reference that "
                         "scales the FETCH_SIZE / WRITE_SIZE counters of a profiler run)")
    ap.add_argument("--only", default=None, choices=["next-stages"],
                    help="time only the kinematics / conv-consumer / pipeline stages of the chosen workload (for profiler runs)")
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

    def time_workload(cfg, envs, steps, warmup, distract=True, threads=0, size=None, graph_launches=0):
        w = workloads.make(cfg, B=envs)
        if size:
            w["desc"]["width"] = w["desc"]["height"] = size
            if w["distractor"] is not None and w["distractor"]["mode"] == "video":
                w["distractor"] = dict(w["distractor"], video=workloads.make_video(
                    np.random.default_rng(size), w["distractor"]["video"].shape[0], size, size))
        scene = pxr.Scene(w["desc"])
        if threads:
            scene.set_block_threads(threads)
        mode = _bind(torch, scene, w["distractor"] if distract else None)
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
        if graph_launches:
            # Launch-bound batches: the same launches recorded once in a HIP graph (the entry point only enqueues) and
            # replayed, against the same number made one by one; wall clock around both, nothing between the launches.
            side = torch.cuda.Stream()  # (default priority; capture needs a stream of its own)

            def launches():
                for i in range(graph_launches):
                    scene.render_batch(poses, shapes, step0=i, frames=frames)
            with torch.cuda.stream(side):
                launches()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(10):
                    launches()
                torch.cuda.synchronize()
                res["eager_s_per_launch"] = (time.perf_counter() - t0) / (10 * graph_launches)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                launches()
            graph.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                graph.replay()
            torch.cuda.synchronize()
            res["graph_s_per_launch"] = (time.perf_counter() - t0) / (10 * graph_launches)
            del graph
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

    def figures(r):
        """Throughput and roofline fractions of one timed workload (kernel time by HIP events)."""
        n = r["B"] * r["S"]
        s = 1e-3 * float(np.mean(r["kernel_ms"]))
        V, T, npix = r["info"]["n_verts"], r["info"]["n_tris"], r["H"] * r["W"]
        ops = algorithmic_ops_per_frame(V, T, npix, r["mode"])
        byts = algorithmic_bytes_per_frame(r["K"], npix, r["mode"], r["w"]["shapes"] is not None, r["S"])
        f = {"envs": r["B"], "steps_per_call": r["S"], "image": r["H"], "distractor": r["mode"],
             "block_threads": r["info"]["block_threads"], "frames_per_s": n / s, "avg_launch_ms": 1e3 * s,
             "alu_frac": ops * n / s / 1e12 / ALU_PEAK_TOPS, "hbm_frac": byts * n / s / 1e9 / HBM_PEAK_GBS,
             "ops_per_frame": ops}
        if "graph_s_per_launch" in r:  # (wall clock over launches made back to back: no event between them)
            f["frames_per_s_back_to_back"] = n / r["eager_s_per_launch"]
            f["frames_per_s_graph_replay"] = n / r["graph_s_per_launch"]
        return f

    cfg = int(args.workload[3:])
    if args.only == "next-stages":
        print(json.dumps(time_next_stages(torch, pxr, workloads.make(cfg, B=args.envs), reps=args.steps)))
        return
    r = time_workload(cfg, args.envs, args.steps, args.warmup, not args.no_distractor, args.threads, args.size)
    n_frames = r["B"] * r["S"]
    ms_per_step = 1e3 * r["wall"] / args.steps
    value = n_frames * args.steps / r["wall"]
    avg_kernel_s = 1e-3 * float(np.mean(r["kernel_ms"]))
    V, T, npix = r["info"]["n_verts"], r["info"]["n_tris"], r["H"] * r["W"]
    ops = algorithmic_ops_per_frame(V, T, npix, r["mode"]) * n_frames
    byts = algorithmic_bytes_per_frame(r["K"], npix, r["mode"], r["w"]["shapes"] is not None, r["S"]) * n_frames
    achieved_tops = ops / avg_kernel_s / 1e12
    prof = PROFILED.get((args.workload, r["B"])) if not (args.size or args.no_distractor or args.threads) else None
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
                     "frac": achieved_tops / ALU_PEAK_TOPS,
                     "traffic": prof["traffic_bytes_per_launch"] if prof else None,
                     "kernel": "render_kernel", "avg_launch_ms": 1e3 * avg_kernel_s,
                     "algorithmic_ops_per_frame": ops // n_frames, "op_count_convention": OP_CONVENTION,
                     "hbm_achieved_gbs": byts / avg_kernel_s / 1e9, "hbm_frac": byts / avg_kernel_s / 1e9 / HBM_PEAK_GBS,
                     "algorithmic_bytes_per_frame": byts / n_frames},
        "kernel_frames_per_s": n_frames / avg_kernel_s,
        "checksum": r["checksum"],
    }
    if prof:  # (from a profiler run of this same workload, not measured live: see PROFILED)
        out["roofline"].update({"profiled_valu_busy": prof["valu_busy"], "profiled_lane_use": prof["lane_use"],
                                "profiled_valu_wave_instructions_per_frame": prof["valu_wave_instructions_per_frame"],
                                "profile": prof["source"]})
    if "phase_clocks" in r:
        out["phase_clocks"] = r["phase_clocks"]  # (a profiling build: `value` is not the product's rate)
    if not args.no_others and not args.profile_lib:
        # what this GPU sustains right now (microbenchmarks in the library), and the headline fractions against it
        pk = pxr.measure_peaks()
        out["measured_peaks"] = _round(dict(pk, alu_frac_of_measured_fma=achieved_tops / pk["fma_tlaneops"],
                                            hbm_frac_of_measured_copy=out["roofline"]["hbm_achieved_gbs"] / pk["copy_gbs"]))
        configs = {}
        for name, c, envs, dis, size in [("cfg1", 1, 16, True, None), ("cfg2", 2, 256, True, None),
                                         ("cfg3", 3, 4096, True, None), ("cfg3_no_distractor", 3, 4096, False, None),
                                         ("cfg4", 4, 16384, True, None), ("cfg4_no_distractor", 4, 16384, False, None),
                                         ("cfg5_16384envs", 5, 16384, True, None),
                                         ("cfg5_128px", 5, 4096, True, 128), ("cfg5_256px", 5, 1024, True, 256),
                                         ("cfg5_512px", 5, 256, True, 512)]:
            # (launches of 0.01-2.5 ms; the two launch-bound ones also as 32 launches in a HIP graph)
            configs[name] = figures(time_workload(c, envs, 40, 5, dis, 0, size, graph_launches=32 if name in ("cfg1", "cfg2") else 0))
        configs["cfg3_distractor_on_over_off"] = configs["cfg3"]["frames_per_s"] / configs["cfg3_no_distractor"]["frames_per_s"]
        configs["cfg4_distractor_on_over_off"] = configs["cfg4"]["frames_per_s"] / configs["cfg4_no_distractor"]["frames_per_s"]
        configs.update(time_next_stages(torch, pxr, r["w"]))
        sweep = time_env_sweep(torch, pxr, workloads, cfg)
        out["configs"] = _round(configs)
        # the same, flat (scalars only), for readers that keep only the scalar entries of `config`
        flat = out["config"]
        for name, v in configs.items():
            if not isinstance(v, dict):
                flat[f"others.{name}"] = _round(v)
            else:
                for k in ("frames_per_s", "avg_launch_ms", "alu_frac", "hbm_frac", "serial_ms", "overlapped_ms",
                          "frames_per_s_back_to_back", "frames_per_s_graph_replay"):
                    if k in v:
                        flat[f"others.{name}.{k}"] = _round(v[k])
        flat["others.alu_frac_of_measured_fma"] = out["measured_peaks"]["alu_frac_of_measured_fma"]
        out["env_sweep"] = _round(sweep)
        for b, v in sweep.items():
            flat[f"others.env_sweep.{b}.frames_per_s"] = _round(v["frames_per_s"])
            flat[f"others.env_sweep.{b}.frames_per_s_graph_replay"] = _round(v["frames_per_s_graph_replay"])
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(r["w"])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
