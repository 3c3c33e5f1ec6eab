"""CPU oracle of the frame consumer: the first convolutional layer of the policy applied to the frame stack.

TEST INFRASTRUCTURE ONLY (same rules as orc.h: nothing in the product path imports this).

The paper's throughput loop runs, at every environment step, a forward pass through one convolutional layer
on the rendered observations (section 2, the paragraph on the steps-per-second figure); it does not give the
layer's hyper-parameters.  Reading used here: a VALID, strided, square-kernel convolution over the S frames of
an environment stacked on the channel axis (channel s*3 + c), inputs scaled to [0,1] by 1/255, plus bias,
optional ReLU; the weights are stored in bfloat16 (round to nearest even from the given fp32 values), because
that is the precision the device's matrix units consume; everything else is evaluated here in float64 and is
the plain definition of the operation:

    out[b,oy,ox,o] = act( bias[o] + sum_{ky,kx,s,c} frames[b,s,st*oy+ky,st*ox+kx,c]/255 * w16[ky,kx,3s+c,o] )

Pins (tests/test_oracle_conv.py): the bf16 rounding against printed bit patterns and torch's conversion;
the convolution against torch.nn.functional.conv2d in float64, against closed forms (box kernel on a constant
image, delta kernels = strided sub-sampling, bias only) and linearity.
"""
import numpy as np


def round_to_bf16(x):
    """fp32 -> nearest bfloat16 (ties to even), returned as fp32 values with the low 16 bits clear."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = ((bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = (rounded & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32).reshape(x.shape)
    return np.where(np.isnan(x), x, out)


def bf16_bits(x):
    """The 16-bit patterns of round_to_bf16(x)."""
    return (round_to_bf16(x).view(np.uint32) >> 16).astype(np.uint16)


def out_size(n, kernel, stride):
    return (n - kernel) // stride + 1


def conv_first_layer(frames, weights, bias, stride=2, relu=True):
    """frames uint8 [B,S,H,W,3]; weights fp32 [k,k,3S,O] (rounded to bf16 here); bias fp32 [O] -> float64 [B,Ho,Wo,O]."""
    frames = np.asarray(frames)
    assert frames.dtype == np.uint8 and frames.ndim == 5 and frames.shape[-1] == 3
    B, S, H, W, _ = frames.shape
    w = round_to_bf16(weights).astype(np.float64)
    k = w.shape[0]
    assert w.shape[:3] == (k, k, 3 * S), w.shape
    O = w.shape[3]
    Ho, Wo = out_size(H, k, stride), out_size(W, k, stride)
    x = frames.astype(np.float64) / 255.0
    out = np.zeros((B, Ho, Wo, O), np.float64)
    for ky in range(k):
        for kx in range(k):
            for s in range(S):
                win = x[:, s, ky:ky + stride * (Ho - 1) + 1:stride, kx:kx + stride * (Wo - 1) + 1:stride, :]  # [B,Ho,Wo,3]
                out += win @ w[ky, kx, 3 * s:3 * s + 3, :]
    out += np.asarray(bias, dtype=np.float32).astype(np.float64)
    return np.maximum(out, 0.0) if relu else out
