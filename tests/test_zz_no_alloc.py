"""pxr_render_batch_kinematic_static (the entry point that allocates nothing) against pxr_render_batch_kinematic,
through the C ABI: frames and ids bit for bit, on two calls in a row, the second with a smaller input (the static
pose buffer then still holds the first call's poses behind the second call's)."""
import ctypes as C

import numpy as np
import pytest

from paper_2502_00021_amd import workloads as wl

pytestmark = pytest.mark.gpu

STATIC_BYTES = 32 << 20


def _setup(torch, pxr, cfg, B):
    w = wl.make(cfg, B=B)
    fk = w["fk"]
    sc = pxr.Scene(w["desc"])
    sc.set_skeleton(fk["skel"], fk["free_poses"].shape[-2], fk["angles"].shape[-1])
    d = w["distractor"]
    if d is not None:
        d = dict(d)
        if d["mode"] == "video":
            d["video"] = torch.from_numpy(d["video"]).cuda()
        sc.apply_distractor(d)
    free = torch.from_numpy(fk["free_poses"]).cuda()
    ang = torch.from_numpy(fk["angles"]).cuda()
    shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
    return sc, free, ang, shapes


def test_static_entry_point_matches_the_allocating_one_twice_in_a_row():
    import torch
    from paper_2502_00021_amd import pxr
    assert torch.cuda.is_available(), "this test needs the MI355X"
    L = pxr.lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    for cfg, B in ((5, 300), (5, 37)):  # 900 frames, then 111: the second call is the smaller one
        print(f"static entry point: cfg{cfg} B={B}", flush=True)
        sc, free, ang, shapes = _setup(torch, pxr, cfg, B)
        S = free.shape[1]
        ref_frames, ref_ids, _ = sc.render_batch_kinematic(free, ang, shapes, step0=5, env0=3, want_ids=True)
        frames = torch.full((B, S, sc.H, sc.W, 3), 0xAB, dtype=torch.uint8, device="cuda")
        ids = torch.full((B, S, sc.H, sc.W), 0x55, dtype=torch.int32, device="cuda")
        rc = L.pxr_render_batch_kinematic_static(sc._h, free.data_ptr(), ang.data_ptr(), shapes.data_ptr(), B, S, 5, 3,
                                                 frames.data_ptr(), ids.data_ptr(), stream)
        assert rc == pxr.OK, L.pxr_last_error().decode()
        torch.cuda.synchronize()
        assert torch.equal(frames, ref_frames) and torch.equal(ids, ref_ids)
        sc.close()
    # a video-distractor scene with a banded frame, through the binding, ids not wanted
    sc, free, ang, shapes = _setup(torch, pxr, 4, 21)
    ref_frames, _, _ = sc.render_batch_kinematic(free, ang, shapes, step0=1)
    frames = torch.zeros_like(ref_frames)
    sc.render_batch_kinematic_static(free, ang, shapes, step0=1, frames=frames)
    torch.cuda.synchronize()
    assert torch.equal(frames, ref_frames)
    sc.close()


def test_static_entry_point_rejects_what_does_not_fit():
    import torch
    from paper_2502_00021_amd import pxr
    L = pxr.lib()
    sc, free, ang, shapes = _setup(torch, pxr, 5, 4)
    K, S = sc.K, 3
    too_many = STATIC_BYTES // (S * K * 28) + 1  # environments whose poses no longer fit
    frames = torch.zeros((4, S, sc.H, sc.W, 3), dtype=torch.uint8, device="cuda")
    # (the size check comes before any buffer is touched, so the small buffers are never read past their end)
    rc = L.pxr_render_batch_kinematic_static(sc._h, free.data_ptr(), ang.data_ptr(), None, too_many, S, 0, 0,
                                             frames.data_ptr(), None, None)
    assert rc == pxr.ERR_UNSUPPORTED and b"static buffer" in L.pxr_last_error()
    assert L.pxr_render_batch_kinematic_static(sc._h, free.data_ptr(), ang.data_ptr(), None, 0, S, 0, 0,
                                               frames.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    assert L.pxr_render_batch_kinematic_static(None, free.data_ptr(), ang.data_ptr(), None, 4, S, 0, 0,
                                               frames.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    sc.set_skeleton(None, 0, 0)
    assert L.pxr_render_batch_kinematic_static(sc._h, free.data_ptr(), ang.data_ptr(), None, 4, S, 0, 0,
                                               frames.data_ptr(), None, None) == pxr.ERR_INVALID_ARG
    torch.cuda.synchronize()
    sc.close()
