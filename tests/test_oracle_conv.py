"""Pins for the oracle's first-conv-layer consumer (oracle/conv.py): bf16 rounding and the convolution itself."""
import numpy as np
import pytest

from oracle import conv as oc


def test_bf16_rounding_known_patterns():
    # value -> bf16 bit pattern (sign 1, exponent 8, mantissa 7), ties to even
    cases = [(1.0, 0x3F80), (-2.0, 0xC000), (0.0, 0x0000), (3.14159265, 0x4049), (255.0, 0x437F),
             (1.0 + 2.0 ** -8, 0x3F80),            # exact tie, even mantissa stays
             (1.0 + 2.0 ** -7 + 2.0 ** -8, 0x3F82),  # exact tie, odd mantissa rounds up
             (1.0 + 2.0 ** -8 + 2.0 ** -20, 0x3F81),  # just above the tie
             (np.float32(3.3895314e38), 0x7F7F)]   # largest finite bf16
    for v, bits in cases:
        assert int(oc.bf16_bits(np.float32(v)).ravel()[0]) == bits, v
    assert np.isinf(oc.round_to_bf16(np.float32(3.4e38)))  # rounds up past the largest bf16
    assert np.isnan(oc.round_to_bf16(np.float32(np.nan)))


def test_bf16_rounding_against_torch():
    import torch
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 20000),
                        np.arange(0, 256, dtype=np.float32)]).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oc.round_to_bf16(x), ref)
    assert np.array_equal(oc.round_to_bf16(np.arange(256, dtype=np.float32)), np.arange(256, dtype=np.float32))


@pytest.mark.parametrize("S,H,W,O,k,st", [(1, 16, 16, 8, 3, 2), (3, 20, 24, 32, 3, 2), (2, 13, 17, 5, 3, 1), (1, 12, 12, 4, 5, 3)])
def test_conv_against_torch_float64(S, H, W, O, k, st):
    import torch
    rng = np.random.default_rng(S * 100 + H)
    B = 3
    frames = rng.integers(0, 256, (B, S, H, W, 3), dtype=np.uint8)
    w = rng.standard_normal((k, k, 3 * S, O)).astype(np.float32) * 0.2
    b = rng.standard_normal(O).astype(np.float32)
    got = oc.conv_first_layer(frames, w, b, stride=st, relu=False)
    x = torch.from_numpy(frames).double().div(255.0).permute(0, 1, 4, 2, 3).reshape(B, 3 * S, H, W)  # channel = 3s + c
    w16 = torch.from_numpy(w).to(torch.bfloat16).double().permute(3, 2, 0, 1)  # OIHW
    ref = torch.nn.functional.conv2d(x, w16, torch.from_numpy(b).double(), stride=st).permute(0, 2, 3, 1).numpy()
    assert got.shape == ref.shape == (B, oc.out_size(H, k, st), oc.out_size(W, k, st), O)
    assert np.abs(got - ref).max() < 1e-12
    assert np.array_equal(oc.conv_first_layer(frames, w, b, stride=st, relu=True), np.maximum(got, 0.0))


def test_conv_closed_forms():
    S, H, W, O = 2, 11, 14, 3
    frames = np.full((1, S, H, W, 3), 51, np.uint8)  # 51/255 = 0.2
    w = np.ones((3, 3, 3 * S, O), np.float32)
    out = oc.conv_first_layer(frames, w, np.zeros(O, np.float32), stride=2, relu=False)
    assert out.shape == (1, 5, 6, O) and np.allclose(out, 0.2 * 9 * 3 * S, rtol=0, atol=1e-13)
    # bias only
    out = oc.conv_first_layer(frames, np.zeros_like(w), np.array([0.5, -1.0, 2.0], np.float32), stride=2, relu=True)
    assert np.array_equal(out[0, 0, 0], [0.5, 0.0, 2.0])
    # a delta kernel picks one tap: strided sub-sampling of one channel of one frame
    rng = np.random.default_rng(5)
    frames = rng.integers(0, 256, (2, S, H, W, 3), dtype=np.uint8)
    for (ky, kx, s, c) in [(0, 0, 0, 0), (2, 1, 1, 2), (1, 2, 0, 1)]:
        w = np.zeros((3, 3, 3 * S, 1), np.float32)
        w[ky, kx, 3 * s + c, 0] = 1.0
        out = oc.conv_first_layer(frames, w, np.zeros(1, np.float32), stride=2, relu=False)
        assert np.array_equal(out[..., 0], frames[:, s, ky:ky + 9:2, kx:kx + 11:2, c] / 255.0)


def test_conv_is_linear_in_the_weights_and_uses_bf16_weights():
    rng = np.random.default_rng(6)
    frames = rng.integers(0, 256, (2, 1, 9, 9, 3), dtype=np.uint8)
    w1 = oc.round_to_bf16(rng.standard_normal((3, 3, 3, 4)).astype(np.float32))
    w2 = oc.round_to_bf16(rng.standard_normal((3, 3, 3, 4)).astype(np.float32))
    z = np.zeros(4, np.float32)
    a = oc.conv_first_layer(frames, w1, z, relu=False)
    b = oc.conv_first_layer(frames, w2, z, relu=False)
    # 2*w1 and -w2 stay representable, so linearity is exact up to float64 summation
    ab = oc.conv_first_layer(frames, 2.0 * w1, z, relu=False) + oc.conv_first_layer(frames, -w2, z, relu=False)
    assert np.abs(ab - (2.0 * a - b)).max() < 1e-12
    # weights are rounded: a perturbation below half a bf16 ulp changes nothing, one above does
    w = np.ones((3, 3, 3, 1), np.float32)
    base = oc.conv_first_layer(frames, w, np.zeros(1, np.float32), relu=False)
    assert np.array_equal(oc.conv_first_layer(frames, w * np.float32(1.001), np.zeros(1, np.float32), relu=False), base)
    assert not np.array_equal(oc.conv_first_layer(frames, w * np.float32(1.01), np.zeros(1, np.float32), relu=False), base)
