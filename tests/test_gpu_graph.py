"""The hot calls only enqueue kernels on the caller's stream (no allocation, no synchronisation, no memset), so
a whole step - joint angles -> poses -> frames -> conv features - can be captured in a HIP graph and replayed.
Every replay is checked against the eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest

from paper_2502_00021_amd import workloads as wl

pytestmark = pytest.mark.gpu


def test_captured_step_replays_like_eager_calls():
    import torch
    assert torch.cuda.is_available()
    from paper_2502_00021_amd import pxr
    w = wl.make(3, B=48)
    fk = w["fk"]
    scene = pxr.Scene(w["desc"])
    scene.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    scene.apply_distractor(dict(w["distractor"]))
    rng = np.random.default_rng(8)
    conv = pxr.Conv(scene.H, scene.W, 1, (rng.standard_normal((3, 3, 3, 32)) * 0.15).astype(np.float32),
                    (rng.standard_normal(32) * 0.1).astype(np.float32))
    free = torch.from_numpy(fk["free_poses"]).cuda()
    ang = torch.from_numpy(fk["angles"]).cuda()
    B = free.shape[0]
    poses = torch.empty((B, 1, scene.K, 7), dtype=torch.float32, device="cuda")
    frames = torch.empty((B, 1, scene.H, scene.W, 3), dtype=torch.uint8, device="cuda")
    feat = torch.empty((B, conv.Ho, conv.Wo, 32), dtype=torch.bfloat16, device="cuda")

    def step():
        scene.render_batch_kinematic(free, ang, None, step0=7, poses=poses, frames=frames)
        conv.forward(frames, out=feat)

    def eager(a):
        ang.copy_(a)
        step()
        torch.cuda.synchronize()
        return poses.clone(), frames.clone(), feat.clone()

    angle_sets = [ang.clone()] + [torch.from_numpy(rng.uniform(-1, 1, tuple(ang.shape)).astype(np.float32)).cuda() for _ in range(3)]
    expected = [eager(a) for a in angle_sets]
    assert not torch.equal(expected[0][1], expected[1][1])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(8):
        k = rep % len(angle_sets)
        ang.copy_(angle_sets[k])
        frames.zero_()  # eager work between replays; the graph must overwrite it
        feat.zero_()
        graph.replay()
        torch.cuda.synchronize()
        p, f, c = expected[k]
        assert torch.equal(poses.view(torch.int32), p.view(torch.int32)), rep
        assert torch.equal(frames, f), rep
        assert torch.equal(feat.view(torch.int16), c.view(torch.int16)), rep
    conv.close()
    scene.close()


@pytest.mark.parametrize("cfg,B", [(2, 48), (5, 20)])
def test_entry_point_that_allocates_nothing_under_capture(cfg, B):
    """pxr_render_batch_kinematic_static is the entry point for callers under graph capture: recorded with the conv
    layer, replayed with eager work in between, every replay against the eager, allocating, calls."""
    import torch
    from paper_2502_00021_amd import pxr
    assert torch.cuda.is_available(), "this test needs the MI355X"
    w = wl.make(cfg, B=B)
    fk = w["fk"]
    sc = pxr.Scene(w["desc"])
    sc.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    free = torch.from_numpy(fk["free_poses"]).cuda()
    ang = torch.from_numpy(fk["angles"]).cuda()
    shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
    S = free.shape[1]
    rng = np.random.default_rng(cfg)
    conv = pxr.Conv(sc.H, sc.W, S, rng.standard_normal((3, 3, 3 * S, 32)).astype(np.float32) * 0.15,
                    rng.standard_normal(32).astype(np.float32) * 0.1)
    frames = torch.zeros((B, S, sc.H, sc.W, 3), dtype=torch.uint8, device="cuda")
    feats = torch.zeros_like(conv.forward(frames))
    ang_in = ang.clone()  # the graph reads these buffers at every replay
    torch.cuda.synchronize()

    side = torch.cuda.Stream()  # (default priority)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sc.render_batch_kinematic_static(free, ang_in, shapes, step0=2, frames=frames)
        conv.forward(frames, out=feats)
    for trial in range(4):
        print(f"graph replay {trial}: cfg{cfg} B={B}", flush=True)
        ang_in.copy_(ang + 0.05 * trial)           # eager work between the replays
        frames.fill_(0x5A)
        feats.fill_(1.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref_frames, _, _ = sc.render_batch_kinematic(free, ang_in, shapes, step0=2)
        ref_feats = conv.forward(ref_frames)
        torch.cuda.synchronize()
        assert torch.equal(frames, ref_frames)
        assert torch.equal(feats.view(torch.int16), ref_feats.view(torch.int16))
    assert not torch.equal(ref_frames, torch.full_like(ref_frames, 0x5A))
    conv.close()
    sc.close()


def test_two_scenes_on_two_streams_and_two_host_threads():
    """Scenes are independent objects and the hot calls keep no hidden state: two host threads, each with its own
    scene and its own (default-priority) stream, interleave launches; every result equals the single-stream one."""
    import threading
    import torch
    from paper_2502_00021_amd import pxr
    from test_gpu_parity import _bind
    results, errors = {}, []

    def reference(cfg, B):
        w = wl.make(cfg, B=B)
        sc = pxr.Scene(w["desc"])
        _bind(torch, sc, w["distractor"])
        poses = torch.from_numpy(w["poses"]).cuda()
        shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
        out = [sc.render_batch(poses, shapes, step0=s)[0].clone() for s in range(6)]
        torch.cuda.synchronize()
        sc.close()
        return out

    refs = {3: reference(3, 64), 5: reference(5, 24)}

    def worker(cfg, B):
        try:
            torch.cuda.set_device(0)
            w = wl.make(cfg, B=B)
            sc = pxr.Scene(w["desc"])
            _bind(torch, sc, w["distractor"])
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                poses = torch.from_numpy(w["poses"]).cuda()
                shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
                outs = []
                for rep in range(4):
                    outs = [sc.render_batch(poses, shapes, step0=s, stream=stream.cuda_stream)[0] for s in range(6)]
                stream.synchronize()
                results[cfg] = [o.clone() for o in outs]
                stream.synchronize()
            sc.close()
        except Exception as e:  # surfaced in the main thread
            errors.append(repr(e))

    threads = [threading.Thread(target=worker, args=(3, 64)), threading.Thread(target=worker, args=(5, 24))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for cfg in (3, 5):
        for a, b in zip(results[cfg], refs[cfg]):
            assert torch.equal(a, b)
    # an error on one thread does not leak into another thread's message
    L = pxr.lib()
    seen = {}

    def bad_call():
        L.pxr_destroy_scene(None)
        L.pxr_scene_info(None, None, None, None, None)
        seen["bad"] = L.pxr_last_error()

    t = threading.Thread(target=bad_call)
    t.start()
    t.join()
    assert b"pxr_scene_info" in seen["bad"]
