"""GPU parity of the frame consumer (pxr_conv_forward, MFMA) against the float64 oracle.

Tolerance (written out here, derived from the arithmetic): the inputs (bytes) and the bf16 weights are exact
in the matrix unit and so is every product (8 x 8 significant bits); the fp32 accumulation of at most 108 terms
and the final fma contribute at most ~110 * 2^-24 relative to the sum of magnitudes A = bias + sum |x w| / 255;
the output is then rounded once to bfloat16: half an ulp = 2^-9 relative to the result.  Bound asserted:
|got - ref| <= 2^-8 |ref| + 2^-16 A + 1e-30 (the first term is twice the rounding step, to leave room for results whose fp32
value sits next to a rounding boundary).
"""
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


def _layer(rng, S, scale=0.15):
    w = (rng.standard_normal((3, 3, 3 * S, 32)) * scale).astype(np.float32)
    b = (rng.standard_normal(32) * 0.1).astype(np.float32)
    return w, b


def _magnitude(oc, frames, w, b):
    return oc.conv_first_layer(frames, np.abs(oc.round_to_bf16(w)), np.abs(b), relu=False)


def assert_conv_parity(oc, got, frames, w, b, relu=True):
    ref = oc.conv_first_layer(frames, w, b, relu=relu)
    A = _magnitude(oc, frames, w, b)
    got = got.astype(np.float64)
    assert got.shape == ref.shape
    err = np.abs(got - ref)
    bound = 2.0 ** -8 * np.abs(ref) + 2.0 ** -16 * A + 1e-30
    bad = np.argwhere(err > bound)
    assert len(bad) == 0, f"{len(bad)} outputs off, first {bad[0]}: gpu {got[tuple(bad[0])]} oracle {ref[tuple(bad[0])]}"
    # and the typical error is the single bf16 rounding: half an ulp
    big = np.abs(ref) > 1e-2
    if big.any():
        assert np.median(err[big] / np.abs(ref[big])) < 2.0 ** -9


def _run(torch, pxr, frames, w, b, relu=True, tuning=None):
    B, S, H, W, _ = frames.shape
    c = pxr.Conv(H, W, S, w, b, relu=relu)
    if tuning:
        c.set_tuning(*tuning)
    out = c.forward(torch.from_numpy(frames).cuda())
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    c.close()
    return got


@pytest.mark.parametrize("S,H,W,B", [(1, 32, 32, 5), (3, 64, 64, 6), (1, 84, 84, 4), (2, 33, 40, 7), (4, 64, 64, 3),
                                     (3, 9, 8, 9), (1, 3, 4, 2), (2, 128, 128, 2), (1, 17, 132, 3)])
def test_random_frames_match_oracle(torch, pxr, S, H, W, B):
    """Shapes spanning one and several 32-pixel tiles per row, ragged tiles, several bands and a ragged last band."""
    from oracle import conv as oc
    rng = np.random.default_rng(S * 1000 + H * 10 + W)
    frames = rng.integers(0, 256, (B, S, H, W, 3), dtype=np.uint8)
    w, b = _layer(rng, S)
    assert_conv_parity(oc, _run(torch, pxr, frames, w, b), frames, w, b)
    assert_conv_parity(oc, _run(torch, pxr, frames, w, b, relu=False), frames, w, b, relu=False)


def test_exact_cases(torch, pxr):
    """Results that are exactly representable must come out bit-exact: delta kernels with weight 255/256... and bias."""
    from oracle import conv as oc
    rng = np.random.default_rng(3)
    S, H, W, B = 3, 20, 24, 4
    frames = rng.integers(0, 256, (B, S, H, W, 3), dtype=np.uint8)
    # all-zero weights: the output is relu(bias) rounded to bf16
    b = (rng.standard_normal(32)).astype(np.float32)
    got = _run(torch, pxr, frames, np.zeros((3, 3, 9, 32), np.float32), b)
    assert np.array_equal(got, np.broadcast_to(np.maximum(oc.round_to_bf16(b), 0), got.shape))
    # each output channel o picks one tap (ky,kx,s,c): out = x/255 rounded to bf16 via fma(x, 1/255, 0)
    w = np.zeros((3, 3, 9, 32), np.float32)
    taps = [(o % 3, (o // 3) % 3, (o // 9) % 3, o % 3) for o in range(32)]
    for o, (ky, kx, s, c) in enumerate(taps):
        w[ky, kx, 3 * s + c, o] = 1.0
    got = _run(torch, pxr, frames, w, np.zeros(32, np.float32), relu=False)
    Ho, Wo = got.shape[1:3]
    for o, (ky, kx, s, c) in enumerate(taps):
        x = frames[:, s, ky:ky + 2 * Ho - 1:2, kx:kx + 2 * Wo - 1:2, c].astype(np.float32)
        expect = oc.round_to_bf16(x * np.float32(1.0 / 255.0))  # one product, exactly what the kernel's fma computes
        assert np.array_equal(got[..., o], expect), o


def test_tuning_does_not_change_output(torch, pxr):
    rng = np.random.default_rng(4)
    frames = rng.integers(0, 256, (9, 3, 64, 64, 3), dtype=np.uint8)
    w, b = _layer(rng, 3)
    base = _run(torch, pxr, frames, w, b)
    for tuning in [(1, 0), (3, 7), (10, 1), (8, 100000), (5, 2)]:
        assert np.array_equal(_run(torch, pxr, frames, w, b, tuning=tuning), base), tuning


def test_rendered_stack_through_the_layer(torch, pxr, orc):
    """Render cfg5's three-frame stacks, then feed them to the layer on the device; oracle: oracle frames -> oracle conv."""
    from oracle import conv as oc
    from test_gpu_parity import _bind
    w5 = wl.make(5, B=12)
    sc = pxr.Scene(w5["desc"])
    _bind(torch, sc, w5["distractor"])
    frames, _ = sc.render_batch(torch.from_numpy(w5["poses"]).cuda(), torch.from_numpy(w5["shapes"]).cuda(), step0=1)
    rng = np.random.default_rng(5)
    w, b = _layer(rng, 3)
    c = pxr.Conv(64, 64, 3, w, b)
    out = c.forward(frames)
    torch.cuda.synchronize()
    ref_frames = orc.Scene(w5["desc"]).render(w5["poses"], w5["shapes"], step0=1, distractor=w5["distractor"])["frames"]
    assert np.array_equal(frames.cpu().numpy(), ref_frames)
    assert_conv_parity(oc, out.float().cpu().numpy(), ref_frames, w, b)
    c.close()
    sc.close()


def test_full_size_sampled(torch, pxr):
    """65536 environments x 3 frames of 64x64 (the headline batch) in the default launch configuration; the
    oracle checks sampled environments, and the whole output is compared with a second run."""
    from oracle import conv as oc
    B = 65536
    g = torch.Generator(device="cuda").manual_seed(11)
    frames = torch.randint(0, 256, (B, 3, 64, 64, 3), dtype=torch.uint8, device="cuda", generator=g)
    rng = np.random.default_rng(11)
    w, b = _layer(rng, 3)
    c = pxr.Conv(64, 64, 3, w, b)
    out = c.forward(frames)
    again = c.forward(frames)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), again.view(torch.int16))
    n_groups = c.info()["n_groups"]
    picks = sorted(set([0, 1, B - 1, B // 2, n_groups // 4, n_groups // 4 + 1] + [int(e) for e in rng.integers(0, B, 20)]))
    idx = torch.tensor(picks, device="cuda")
    assert_conv_parity(oc, out[idx].float().cpu().numpy(), frames[idx].cpu().numpy(), w, b)
    c.close()


def test_conv_argument_errors(torch, pxr):
    rng = np.random.default_rng(6)
    w, b = _layer(rng, 1)
    for kw in (dict(c_out=16), dict(kernel=5), dict(stride=1)):
        with pytest.raises((pxr.PxrError, AssertionError)):
            ww = w if "c_out" not in kw else w[..., :16]
            bb = b if "c_out" not in kw else b[:16]
            if "kernel" in kw:
                ww = np.zeros((5, 5, 3, 32), np.float32)
            pxr.Conv(32, 32, 1, ww, bb, **kw)
    with pytest.raises(pxr.PxrError):
        pxr.Conv(32, 30, 1, w, b)  # width not a multiple of 4
    with pytest.raises(pxr.PxrError):
        pxr.Conv(2, 32, 1, w, b)
    bad = w.copy()
    bad[0, 0, 0, 0] = np.nan
    with pytest.raises(pxr.PxrError):
        pxr.Conv(32, 32, 1, bad, b)
    c = pxr.Conv(32, 32, 1, w, b)
    L = pxr.lib()
    fr = torch.zeros((2, 1, 32, 32, 3), dtype=torch.uint8, device="cuda")
    out = torch.empty((2, 15, 15, 32), dtype=torch.bfloat16, device="cuda")
    assert L.pxr_conv_forward(c._h, None, 2, out.data_ptr(), None) == pxr.ERR_INVALID_ARG
    assert L.pxr_conv_forward(c._h, fr.data_ptr(), 0, out.data_ptr(), None) == pxr.ERR_INVALID_ARG
    assert L.pxr_conv_forward(c._h, fr.data_ptr(), 2, out.data_ptr() + 2, None) == pxr.ERR_INVALID_ARG
    assert L.pxr_conv_forward(c._h, fr.data_ptr() + 1, 2, out.data_ptr(), None) == pxr.ERR_INVALID_ARG
    assert b"pxr_conv_forward" in L.pxr_last_error()
    c.forward(fr, out=out)
    torch.cuda.synchronize()
    assert np.array_equal(out.float().cpu().numpy()[0, 0, 0], np.maximum(out.float().cpu().numpy()[0, 0, 0], 0))
    c.close()
