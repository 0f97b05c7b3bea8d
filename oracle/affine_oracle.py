"""CPU oracle of the reference forward with affine (asymmetric) uint8 activations
(test infrastructure only: tests, smoke() and bench.py's cpu_baseline may import
it; the product never does).

Section 5 of the paper delegates the int8 arithmetic to the framework's
quantisation (static for convolutional networks, dynamic for language models).
That framework's default for activations is an affine uint8 code with a zero
point, weights staying symmetric int8.  The paper prints no formula; the reading
taken here is the framework's min/max observer followed by its per-tensor
quantiser, every operation an IEEE float32 one:

    hi    = max(max x, 0),  lo = min(min x, 0)         zero is always a code
    scale = max((hi - lo) / 255, 2^-23)                float32 subtraction, division
    zp    = clamp(0 - rne(lo / scale), 0, 255)         float32 division, ties to even
    q     = clamp(rne(x * (1 / scale)) + zp, 0, 255)   float32 reciprocal and product
    x^    = (q - zp) * scale

A linear or convolution layer multiplies the centred codes, which is exact in
integers, and finishes like the symmetric reference:

    acc = sum_k (q_k - zp) * w_k                       int32
    y   = act( fma((float) acc, scale * s_w, bias) [+ x^_block] )

Zero padding of a 3x3 window pads the *real* value zero, i.e. the centred code 0.
The Transformer glue (attention, GELU, layer norm) is the fp32 one of the
symmetric oracle.
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as F

from . import oracle as sym        # weight quantiser, epilogue, attention, layer norm: no activation codes in them

ACT_NONE, ACT_RELU, ACT_GELU = sym.ACT_NONE, sym.ACT_RELU, sym.ACT_GELU
EPS = np.float32(2.0 ** -23)


def qparams(x):
    """(scale float32, zero point int) of a tensor, from its extrema."""
    x = np.asarray(x, np.float32)
    if not np.isfinite(x).all():
        raise sym.NonFiniteInput("input holds NaN or Inf")
    hi = np.float32(max(float(x.max()) if x.size else 0.0, 0.0))
    lo = np.float32(min(float(x.min()) if x.size else 0.0, 0.0))
    scale = np.float32(np.float32(hi - lo) / np.float32(255.0))
    scale = max(scale, EPS)
    zp = int(np.clip(0 - np.rint(np.float32(lo / scale)), 0, 255))
    return np.float32(scale), zp


def quantize(x):
    """uint8 codes, scale and zero point of `x` (any shape)."""
    x = np.asarray(x, np.float32)
    scale, zp = qparams(x)
    inv = np.float32(np.float32(1.0) / scale)
    q = np.clip(np.rint(x * inv).astype(np.int64) + zp, 0, 255).astype(np.uint8)
    return q, scale, zp


def dequantize(q, scale, zp):
    return ((q.astype(np.int32) - zp).astype(np.float32) * np.float32(scale)).astype(np.float32)


def _centred(q, zp):
    return q.astype(np.float64) - float(zp)


def linear(x, wq, sw, bias, act=ACT_NONE, taps=None, tag=""):
    shp = x.shape
    x2 = np.asarray(x, np.float32).reshape(-1, shp[-1])
    q, sx, zp = quantize(x2)
    acc = (_centred(q, zp) @ wq.astype(np.float64).T).astype(np.int32)      # exact: |acc| < 2^53
    y = sym.dequant_bias_act(acc, sx, sw, bias, act)
    if taps is not None:
        taps[tag + "xq"], taps[tag + "sx"], taps[tag + "zp"], taps[tag + "acc"], taps[tag + "y"] = q, sx, zp, acc, y
    return y.reshape(shp[:-1] + (wq.shape[0],))


def _conv(q, sx, zp, wq, sw, bias, pad, act, residual, taps, tag):
    acc = F.conv2d(torch.from_numpy(_centred(q, zp)), torch.from_numpy(wq.astype(np.float64)), padding=pad).numpy()
    acc = acc.astype(np.int32)
    y = sym.dequant_bias_act(acc, sx, sw, bias, act, residual)
    taps[tag + "xq"], taps[tag + "sx"], taps[tag + "zp"], taps[tag + "acc"], taps[tag + "y"] = q, sx, zp, acc, y
    return y


def fc_relu(x, qw, biases):
    taps = {}
    (wq, sw), = qw
    taps["a_ref"] = linear(x, wq, sw, biases[0], ACT_RELU, taps, "l0.")
    return taps


def basic_block(x, qw, biases, has_residual=True):
    taps = {}
    q, sx, zp = quantize(x)
    xhat = dequantize(q, sx, zp) if has_residual else None
    h = _conv(q, sx, zp, qw[0][0], qw[0][1], biases[0], 1, ACT_RELU, None, taps, "l0.")
    hq, sh, zh = quantize(h)
    taps["a_ref"] = _conv(hq, sh, zh, qw[1][0], qw[1][1], biases[1], 1, ACT_RELU, xhat, taps, "l1.")
    return taps


def bottleneck(x, qw, biases, has_residual=True):
    taps = {}
    q, sx, zp = quantize(x)
    xhat = dequantize(q, sx, zp) if has_residual else None
    h1 = _conv(q, sx, zp, qw[0][0], qw[0][1], biases[0], 0, ACT_RELU, None, taps, "l0.")
    q1, s1, z1 = quantize(h1)
    h2 = _conv(q1, s1, z1, qw[1][0], qw[1][1], biases[1], 1, ACT_RELU, None, taps, "l1.")
    q2, s2, z2 = quantize(h2)
    taps["a_ref"] = _conv(q2, s2, z2, qw[2][0], qw[2][1], biases[2], 0, ACT_RELU, xhat, taps, "l2.")
    return taps


def bert_layer(x, qw, biases, heads, ln_eps, taps, tag):
    qkv = linear(x, qw[0][0], qw[0][1], biases[0], ACT_NONE, taps, tag + "l0.")
    ctx = sym.attention(qkv, heads)
    o = linear(ctx, qw[1][0], qw[1][1], biases[1], ACT_NONE, taps, tag + "l1.")
    y = sym.layernorm(x, o, eps=ln_eps)
    f = linear(y, qw[2][0], qw[2][1], biases[2], ACT_GELU, taps, tag + "l2.")
    z = linear(f, qw[3][0], qw[3][1], biases[3], ACT_NONE, taps, tag + "l3.")
    return sym.layernorm(y, z, eps=ln_eps)


def ref_forward(wl, qw=None):
    """Reference forward of a synthetic workload with affine uint8 activations.
    Taps per linear layer: `xq` (uint8), `sx`, `zp`, `acc`, `y`; `a_ref` the
    module's activation (a list, one per layer, for the Transformer kinds)."""
    if qw is None:
        qw = sym.quantize_weights(wl.weights)
    k = wl.kind
    if k == 0:
        return fc_relu(wl.x, qw, wl.biases)
    if k == 1:
        return basic_block(wl.x, qw, wl.biases, bool(wl.dims["has_residual"]))
    if k == 2:
        return bottleneck(wl.x, qw, wl.biases, bool(wl.dims["has_residual"]))
    d = wl.dims
    taps, cur, outs = {}, np.asarray(wl.x, np.float32), []
    for l in range(d["n_layers"] if k == 4 else 1):
        cur = bert_layer(cur, qw[4 * l:4 * l + 4], wl.biases[4 * l:4 * l + 4], d["heads"], d["ln_eps"], taps, f"L{l}.")
        outs.append(cur)
    taps["a_ref"] = outs
    return taps
