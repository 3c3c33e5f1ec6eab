"""pxr_pipeline_step (render and conv layer overlapped chunk by chunk on two streams) against the serial order
pxr_render_batch -> pxr_conv_forward: frames and features byte for byte.  The serial order itself is checked
against the oracle in test_gpu_parity.py / test_gpu_conv.py."""
import numpy as np
import pytest

from paper_2502_00021_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch as _torch
    assert _torch.cuda.is_available(), "these tests need the MI355X"
    return _torch


@pytest.fixture(scope="module")
def pxr():
    from paper_2502_00021_amd import pxr as _pxr
    _pxr.lib()
    return _pxr


def _make(torch, pxr, cfg, B):
    w = wl.make(cfg, B=B)
    sc = pxr.Scene(w["desc"])
    d = w["distractor"]
    if d is not None:
        d = dict(d)
        if d["mode"] == "video":
            d["video"] = torch.from_numpy(d["video"]).cuda()
            # per-environment offsets given by the caller: a chunk must pick up its own environments' entries
            d["env_offset"] = torch.from_numpy(np.random.default_rng(3).integers(0, 64, B).astype(np.int32)).cuda()
        sc.apply_distractor(d)
    poses = torch.from_numpy(w["poses"]).cuda()
    shapes = None if w["shapes"] is None else torch.from_numpy(w["shapes"]).cuda()
    S = poses.shape[1]
    rng = np.random.default_rng(cfg)
    conv = pxr.Conv(sc.H, sc.W, S, (rng.standard_normal((3, 3, 3 * S, 32)) * 0.15).astype(np.float32),
                    (rng.standard_normal(32) * 0.1).astype(np.float32))
    return sc, conv, poses, shapes


@pytest.mark.parametrize("cfg,B,chunks", [(5, 203, 4), (5, 64, 16), (5, 3, 4), (4, 50, 3), (3, 130, 2), (2, 37, 1)])
def test_pipeline_equals_serial_order(torch, pxr, cfg, B, chunks):
    sc, conv, poses, shapes = _make(torch, pxr, cfg, B)
    S = poses.shape[1]
    ref_frames, _ = sc.render_batch(poses, shapes, step0=7, env0=5)
    ref_feat = conv.forward(ref_frames)
    torch.cuda.synchronize()
    pipe = pxr.Pipeline(sc, conv, chunks)
    frames = torch.full_like(ref_frames, 0x5A)
    feat = torch.full_like(ref_feat, -1.0)
    for rep in range(3):  # steps in a row share the second stream and the events
        pipe.step(poses, shapes, frames, feat, step0=7, env0=5)
    torch.cuda.synchronize()
    assert torch.equal(frames, ref_frames)
    assert torch.equal(feat.view(torch.int16), ref_feat.view(torch.int16))
    # on a stream of the caller's own
    side = torch.cuda.Stream()
    frames.fill_(0)
    feat.fill_(0)
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pipe.step(poses, shapes, frames, feat, step0=7, env0=5)
    side.synchronize()
    assert torch.equal(frames, ref_frames) and torch.equal(feat.view(torch.int16), ref_feat.view(torch.int16))
    pipe.close()
    conv.close()
    sc.close()


def test_pipeline_argument_errors(torch, pxr):
    sc, conv, poses, shapes = _make(torch, pxr, 5, 8)
    L = pxr.lib()
    import ctypes as C
    h = C.c_void_p()
    assert L.pxr_pipeline_create(sc._h, conv._h, 0, C.byref(h)) == pxr.ERR_INVALID_ARG
    assert L.pxr_pipeline_create(sc._h, conv._h, 17, C.byref(h)) == pxr.ERR_INVALID_ARG
    assert L.pxr_pipeline_create(None, conv._h, 2, C.byref(h)) == pxr.ERR_INVALID_ARG
    other = pxr.Conv(32, 32, 3, np.zeros((3, 3, 9, 32), np.float32), np.zeros(32, np.float32))
    assert L.pxr_pipeline_create(sc._h, other._h, 2, C.byref(h)) == pxr.ERR_INVALID_ARG
    other.close()
    pipe = pxr.Pipeline(sc, conv, 2)
    frames = torch.empty((8, 3, sc.H, sc.W, 3), dtype=torch.uint8, device="cuda")
    feat = torch.empty((8, conv.Ho, conv.Wo, 32), dtype=torch.bfloat16, device="cuda")
    assert L.pxr_pipeline_step(pipe._h, None, None, 8, 0, 0, frames.data_ptr(), feat.data_ptr(), None) == pxr.ERR_INVALID_ARG
    assert L.pxr_pipeline_step(pipe._h, poses.data_ptr(), None, 0, 0, 0, frames.data_ptr(), feat.data_ptr(), None) == pxr.ERR_INVALID_ARG
    assert L.pxr_pipeline_step(pipe._h, poses.data_ptr(), None, 8, 0, 0, frames.data_ptr(), feat.data_ptr() + 2, None) == pxr.ERR_INVALID_ARG
    assert L.pxr_pipeline_destroy(None) == pxr.OK
    torch.cuda.synchronize()
    pipe.close()
    conv.close()
    sc.close()
