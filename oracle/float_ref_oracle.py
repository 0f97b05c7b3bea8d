"""CPU oracle of the reference forward at float16 and float32 precision (test
infrastructure only: tests, smoke() and bench.py's cpu_baseline may import it;
the product never does).

Section 6.4 of the paper ("Impact of the reference model's precision", Table 2)
runs the reference model at float16 and float32 besides int8 and keeps the
higher precisions as the fallback when int8 fails.  The paper leaves the
arithmetic to its framework; the reading taken here, for a layer with input x,
weight w and bias:

    r(.)  = round to nearest even to the reference precision (identity for float32)
    acc   = sum_k r(x)_k * r(w)_k      exact products, accumulated in float64,
                                       rounded once to float32
    y     = act( acc + bias [+ r(x_block)] )   float32 additions in this order

i.e. weights and every layer's input live in the reference precision, sums are
kept in (at least) float32, and the skip connection adds the block's input as
the reference model holds it.  Convolutions use the library's float64
convolution as the contraction step.  Module kinds: FC + ReLU, basic block,
bottleneck (the paper's Table 2 is measured on a ResNet) and the Transformer
encoder layer / stack.  In an encoder layer only the four linear layers run in
the reference precision, exactly the four the int8 reference quantises
(Section 5): the attention between them, the GELU and the two layer norms take
and give float32 and are evaluated in float64, rounded once:

    gelu(v) = v/2 * (1 + erf(v / sqrt 2))      on the float32 output of the
                                               first feed-forward layer
"""
from __future__ import annotations

import numpy as np
import torch
import torch.nn.functional as F
from scipy.special import erf

from . import oracle as _int8_oracle       # its float32 attention and layer norm (no int8 arithmetic)

PRECISIONS = ("f16", "f32")


def r(a, precision):
    """`a` rounded to the reference precision, returned as float32."""
    a = np.asarray(a, np.float32)
    if precision == "f32":
        return a
    assert precision == "f16"
    return a.astype(np.float16).astype(np.float32)      # IEEE round to nearest even


def _finish(acc64, bias, residual, relu, channel_axis):
    y = acc64.astype(np.float32)                          # the sum, rounded once
    if bias is not None:
        shape = [1] * y.ndim
        shape[channel_axis] = -1
        y = y + np.asarray(bias, np.float32).reshape(shape)
    if residual is not None:
        y = y + residual
    return np.maximum(y, np.float32(0)) if relu else y


def linear(x, w, bias, precision, relu=True):
    xr, wr = r(x, precision), r(w, precision)
    acc = xr.astype(np.float64) @ wr.astype(np.float64).T
    return _finish(acc, bias, None, relu, 1), xr, acc.astype(np.float32)


def conv(x, w, bias, precision, pad, residual=None, relu=True):
    xr, wr = r(x, precision), r(w, precision)
    acc = F.conv2d(torch.from_numpy(xr).double(), torch.from_numpy(wr).double(), padding=pad).numpy()
    return _finish(acc, bias, residual, relu, 1), xr, acc.astype(np.float32)


def gelu(v):
    """erf-form GELU of float32 values, evaluated in float64 and rounded once."""
    v64 = np.asarray(v, np.float32).astype(np.float64)
    return (0.5 * v64 * (1.0 + erf(v64 / np.sqrt(2.0)))).astype(np.float32)


def bert_layer(x, W, B, heads, precision, ln_eps, taps, tag):
    """Post-LN encoder layer, inference mode: x [b, s, hidden] -> [b, s, hidden]."""
    b, s, hd = x.shape

    def lin(i, v):
        y, xr, acc = linear(v.reshape(b * s, -1), W[i], B[i], precision, relu=False)
        taps[f"{tag}l{i}.x"], taps[f"{tag}l{i}.acc"] = xr, acc
        return y

    qkv = lin(0, x)
    taps[tag + "l0.y"] = qkv
    ctx = _int8_oracle.attention(qkv.reshape(b, s, 3 * hd), heads)
    o = lin(1, ctx)
    taps[tag + "l1.y"] = o
    y1 = _int8_oracle.layernorm(x, o.reshape(b, s, hd), eps=ln_eps)
    f = gelu(lin(2, y1))
    taps[tag + "l2.y"] = f
    z = lin(3, f)
    taps[tag + "l3.y"] = z
    return _int8_oracle.layernorm(y1, z.reshape(b, s, hd), eps=ln_eps)


def ref_forward(wl, precision):
    """Taps of the float-precision reference forward of a synthetic workload:
    per layer the rounded input `l<i>.x`, the float32 sum `l<i>.acc` and the
    output `l<i>.y` (prefixed `L<layer>.` for the Transformer kinds); `a_ref` is
    the module's activation (a list, one per layer, for the Transformer kinds)."""
    assert precision in PRECISIONS
    k, W, B = wl.kind, wl.weights, wl.biases
    t = {}

    def keep(i, out):
        t[f"l{i}.y"], t[f"l{i}.x"], t[f"l{i}.acc"] = out
        return out[0]

    if k == 0:
        y = keep(0, linear(wl.x, W[0], B[0], precision))
    elif k == 1:
        res = r(wl.x, precision) if wl.dims["has_residual"] else None
        h = keep(0, conv(wl.x, W[0], B[0], precision, 1))
        y = keep(1, conv(h, W[1], B[1], precision, 1, res))
    elif k == 2:
        res = r(wl.x, precision) if wl.dims["has_residual"] else None
        h1 = keep(0, conv(wl.x, W[0], B[0], precision, 0))
        h2 = keep(1, conv(h1, W[1], B[1], precision, 1))
        y = keep(2, conv(h2, W[2], B[2], precision, 0, res))
    else:
        d = wl.dims
        n_layers = d["n_layers"] if k == 4 else 1
        cur, outs = np.asarray(wl.x, np.float32), []
        for l in range(n_layers):
            cur = bert_layer(cur, W[4 * l:4 * l + 4], B[4 * l:4 * l + 4], d["heads"], precision, d["ln_eps"], t,
                             f"L{l}.")
            outs.append(cur)
        t["a_ref"] = outs
        return t
    t["a_ref"] = y
    return t
