"""numpy front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Loads `libegeria_oracle.so` (built from `egeria_oracle.c` in this folder) and
composes its primitives into the reference forward of each layer-module kind.
Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; it imports nothing from the GPU package.

Every block driver returns a dict of *taps*: each quantised tensor with its
scale, each int32 accumulator and each fp32 intermediate, so that a second
implementation can be compared step by step.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "egeria_oracle.c")
_LIB = os.path.join(_HERE, "libegeria_oracle.so")
_lib = None

_i8p = ctypes.POINTER(ctypes.c_int8)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_i64 = ctypes.c_int64


def build(force: bool = False) -> str:
    """Compile the oracle's C file with gcc (plain -O2, OpenMP on outer loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        L.orc_absmax_f32.restype = ctypes.c_float
        L.orc_absmax_f32.argtypes = [_f32p, _i64]
        L.orc_quantize_f32.restype = ctypes.c_int
        L.orc_quantize_f32.argtypes = [_f32p, _i64, _f32p, _i8p, _f32p]
        L.orc_dequantize.restype = None
        L.orc_dequantize.argtypes = [_i8p, ctypes.c_float, _i64, _f32p]
        L.orc_gemm_i8.restype = None
        L.orc_gemm_i8.argtypes = [_i8p, _i8p, _i64, _i64, _i64, _i32p]
        L.orc_conv2d_i8.restype = None
        L.orc_conv2d_i8.argtypes = [_i8p, _i8p] + [_i64] * 8 + [_i32p]
        L.orc_dequant_bias_act_pc.restype = None
        L.orc_dequant_bias_act_pc.argtypes = [_i32p, _i64, _i64, _i64, ctypes.c_float, _f32p, _f32p, ctypes.c_int,
                                              _f32p, _f32p]
        L.orc_dequant_bias_act.restype = None
        L.orc_dequant_bias_act.argtypes = [_i32p, _i64, _i64, _i64, ctypes.c_float, ctypes.c_float,
                                           _f32p, ctypes.c_int, _f32p, _f32p]
        L.orc_layernorm.restype = None
        L.orc_layernorm.argtypes = [_f32p, _f32p, _i64, _i64, _f32p, _f32p, ctypes.c_double, _f32p]
        L.orc_attention.restype = None
        L.orc_attention.argtypes = [_f32p, _i64, _i64, _i64, _i64, _f32p]
        L.orc_sp_loss_f32.restype = ctypes.c_double
        L.orc_sp_loss_f32.argtypes = [_f32p, _f32p, _i64, _i64, _f64p, _f64p]
        L.orc_num_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def _p(a, t):
    return None if a is None else a.ctypes.data_as(t)


def num_threads() -> int:
    return int(lib().orc_num_threads())


class NonFiniteInput(ValueError):
    pass


# ---- primitives ------------------------------------------------------------

def quantize(x, fixed_scale=None):
    """Per-tensor symmetric int8 codes and the fp32 scale of `x` (any shape)."""
    x = _c(x, np.float32)
    q = np.empty(x.shape, np.int8)
    s = np.zeros(1, np.float32)
    fs = None if fixed_scale is None else np.array([fixed_scale], np.float32)
    rc = lib().orc_quantize_f32(_p(x, _f32p), x.size, _p(fs, _f32p), _p(q, _i8p), _p(s, _f32p))
    if rc != 0:
        raise NonFiniteInput("input holds NaN or Inf")
    return q, np.float32(s[0])


def dequantize(q, scale):
    q = _c(q, np.int8)
    x = np.empty(q.shape, np.float32)
    lib().orc_dequantize(_p(q, _i8p), float(scale), q.size, _p(x, _f32p))
    return x


def gemm_i8(xq, wq):
    xq, wq = _c(xq, np.int8), _c(wq, np.int8)
    M, K = xq.shape
    N, K2 = wq.shape
    assert K == K2
    acc = np.empty((M, N), np.int32)
    lib().orc_gemm_i8(_p(xq, _i8p), _p(wq, _i8p), M, N, K, _p(acc, _i32p))
    return acc


def conv2d_i8(xq, wq, pad):
    xq, wq = _c(xq, np.int8), _c(wq, np.int8)
    B, C, H, W = xq.shape
    OC, C2, KH, KW = wq.shape
    assert C == C2 and KH == 2 * pad + 1 and KW == 2 * pad + 1
    acc = np.empty((B, OC, H, W), np.int32)
    lib().orc_conv2d_i8(_p(xq, _i8p), _p(wq, _i8p), B, C, H, W, OC, KH, KW, pad, _p(acc, _i32p))
    return acc


ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2


def dequant_bias_act(acc, sx, sw, bias=None, act=ACT_NONE, residual=None):
    """acc [outer, channels, *inner] int32 -> fp32 of the same shape."""
    acc = _c(acc, np.int32)
    outer, channels = acc.shape[0], acc.shape[1]
    inner = int(np.prod(acc.shape[2:])) if acc.ndim > 2 else 1
    bias = None if bias is None else _c(bias, np.float32)
    residual = None if residual is None else _c(residual, np.float32)
    if residual is not None:
        assert residual.shape == acc.shape
    y = np.empty(acc.shape, np.float32)
    if np.ndim(sw) == 0:
        lib().orc_dequant_bias_act(_p(acc, _i32p), outer, channels, inner, float(sx), float(sw),
                                   _p(bias, _f32p), int(act), _p(residual, _f32p), _p(y, _f32p))
    else:                                        # one weight scale per output channel
        swv = _c(sw, np.float32)
        assert swv.shape == (channels,)
        lib().orc_dequant_bias_act_pc(_p(acc, _i32p), outer, channels, inner, float(sx), _p(swv, _f32p),
                                      _p(bias, _f32p), int(act), _p(residual, _f32p), _p(y, _f32p))
    return y


def layernorm(x, res=None, gamma=None, beta=None, eps=1e-12):
    x = _c(x, np.float32)
    H = x.shape[-1]
    M = x.size // H
    res = None if res is None else _c(res, np.float32)
    gamma = None if gamma is None else _c(gamma, np.float32)
    beta = None if beta is None else _c(beta, np.float32)
    y = np.empty(x.shape, np.float32)
    lib().orc_layernorm(_p(x, _f32p), _p(res, _f32p), M, H, _p(gamma, _f32p), _p(beta, _f32p),
                        float(eps), _p(y, _f32p))
    return y


def attention(qkv, heads):
    qkv = _c(qkv, np.float32)
    B, S, H3 = qkv.shape
    Hd = H3 // 3
    ctx = np.empty((B, S, Hd), np.float32)
    lib().orc_attention(_p(qkv, _f32p), B, S, Hd, heads, _p(ctx, _f32p))
    return ctx


def sp_loss(a_t, a_r, return_grams=False):
    """Training plasticity (Eq. 1) of two [b, ...] activations, in fp64."""
    a_t, a_r = _c(a_t, np.float32), _c(a_r, np.float32)
    b = a_t.shape[0]
    assert a_r.shape[0] == b
    D = a_t.size // b
    assert a_r.size // b == D
    gt = np.empty((b, b), np.float64) if return_grams else None
    gr = np.empty((b, b), np.float64) if return_grams else None
    p = lib().orc_sp_loss_f32(_p(a_t, _f32p), _p(a_r, _f32p), b, D, _p(gt, _f64p), _p(gr, _f64p))
    return (float(p), gt, gr) if return_grams else float(p)


# ---- layer modules -----------------------------------------------------------

def quantize_per_channel(w):
    """int8 codes of a weight tensor [out, ...] with one symmetric scale per
    output channel: the per-tensor rule applied to every w[o] on its own."""
    w = _c(w, np.float32)
    q = np.empty(w.shape, np.int8)
    s = np.empty(w.shape[0], np.float32)
    for o in range(w.shape[0]):
        q[o], s[o] = quantize(w[o])
    return q, s


def quantize_weights(weights, per_channel=False):
    """Reference-model generation: int8 of every snapshot tensor, with one
    scale per tensor or one per output channel."""
    return [quantize_per_channel(w) if per_channel else quantize(w) for w in weights]


def linear_int8(x, wq, sw, bias, act=ACT_NONE, taps=None, tag="", act_scale=None):
    """Quantised linear layer: quantise the fp32 input per tensor (dynamic scale,
    or the static scale `act_scale`), integer GEMM, dequantising epilogue."""
    shp = x.shape
    x2 = x.reshape(-1, shp[-1])
    xq, sx = quantize(x2, act_scale)
    acc = gemm_i8(xq, wq)
    y = dequant_bias_act(acc, sx, sw, bias, act)
    if taps is not None:
        taps[tag + "xq"], taps[tag + "sx"], taps[tag + "acc"], taps[tag + "y"] = xq, sx, acc, y
    return y.reshape(shp[:-1] + (wq.shape[0],))


def fc_relu(x, qw, biases, act_scales=None):
    taps = {}
    (wq, sw), = qw
    y = linear_int8(x, wq, sw, biases[0], ACT_RELU, taps, "l0.", None if act_scales is None else act_scales[0])
    taps["a_ref"] = y
    return taps


def _conv_int8(xq, sx, wq, sw, bias, pad, act, residual, taps, tag):
    acc = conv2d_i8(xq, wq, pad)
    y = dequant_bias_act(acc, sx, sw, bias, act, residual)
    taps[tag + "xq"], taps[tag + "sx"], taps[tag + "acc"], taps[tag + "y"] = xq, sx, acc, y
    return y


def basic_block(x, qw, biases, has_residual=True, act_scales=None):
    """conv3x3 -> ReLU -> conv3x3 (+ dequantised input) -> ReLU, all NCHW.
    act_scales: static scales of the two quantise points (Section 5: static
    quantisation for convolutional networks), or None for dynamic ones."""
    taps = {}
    st = [None, None] if act_scales is None else act_scales
    xq, sx = quantize(x, st[0])
    xhat = dequantize(xq, sx) if has_residual else None
    h = _conv_int8(xq, sx, qw[0][0], qw[0][1], biases[0], 1, ACT_RELU, None, taps, "l0.")
    hq, sh = quantize(h, st[1])
    y = _conv_int8(hq, sh, qw[1][0], qw[1][1], biases[1], 1, ACT_RELU, xhat, taps, "l1.")
    taps["a_ref"] = y
    return taps


def bottleneck(x, qw, biases, has_residual=True, act_scales=None):
    """conv1x1 -> ReLU -> conv3x3 -> ReLU -> conv1x1 (+ dequantised input) -> ReLU.
    act_scales: static scales of the three quantise points, or None."""
    taps = {}
    st = [None, None, None] if act_scales is None else act_scales
    xq, sx = quantize(x, st[0])
    xhat = dequantize(xq, sx) if has_residual else None
    h1 = _conv_int8(xq, sx, qw[0][0], qw[0][1], biases[0], 0, ACT_RELU, None, taps, "l0.")
    h1q, s1 = quantize(h1, st[1])
    h2 = _conv_int8(h1q, s1, qw[1][0], qw[1][1], biases[1], 1, ACT_RELU, None, taps, "l1.")
    h2q, s2 = quantize(h2, st[2])
    y = _conv_int8(h2q, s2, qw[2][0], qw[2][1], biases[2], 0, ACT_RELU, xhat, taps, "l2.")
    taps["a_ref"] = y
    return taps


def bert_layer(x, qw, biases, heads, ln_eps=1e-12, taps=None, tag=""):
    """Post-LN Transformer encoder layer in inference mode; only the four
    linear layers are quantised (dynamic quantisation), the rest is fp32."""
    taps = {} if taps is None else taps
    qkv = linear_int8(x, qw[0][0], qw[0][1], biases[0], ACT_NONE, taps, tag + "l0.")
    ctx = attention(qkv, heads)
    taps[tag + "ctx"] = ctx
    o = linear_int8(ctx, qw[1][0], qw[1][1], biases[1], ACT_NONE, taps, tag + "l1.")
    y = layernorm(x, o, eps=ln_eps)
    taps[tag + "ln1"] = y
    f = linear_int8(y, qw[2][0], qw[2][1], biases[2], ACT_GELU, taps, tag + "l2.")
    z = linear_int8(f, qw[3][0], qw[3][1], biases[3], ACT_NONE, taps, tag + "l3.")
    out = layernorm(y, z, eps=ln_eps)
    taps[tag + "a_ref"] = out
    return out, taps


def bert_stack(x, qw, biases, heads, n_layers, ln_eps=1e-12, keep_taps=True, progress=None):
    taps = {}
    cur = x
    outs = []
    for l in range(n_layers):
        t = taps if keep_taps else {}
        cur, _ = bert_layer(cur, qw[4 * l:4 * l + 4], biases[4 * l:4 * l + 4], heads, ln_eps, t,
                            f"L{l}.")
        outs.append(cur)
        if progress:
            progress(l)
    taps["a_ref"] = outs
    return taps


def ref_forward(wl, qw=None, keep_taps=True, progress=None, act_scales=None):
    """Reference forward of a synthetic workload (see synth_inputs.Workload).
    act_scales: static activation scales, one per quantise point (FC and conv
    kinds only; the Transformer kinds are dynamically quantised, Section 5)."""
    if qw is None:
        qw = quantize_weights(wl.weights)
    k = wl.kind
    if k == 0:
        return fc_relu(wl.x, qw, wl.biases, act_scales)
    if k == 1:
        return basic_block(wl.x, qw, wl.biases, bool(wl.dims["has_residual"]), act_scales)
    if k == 2:
        return bottleneck(wl.x, qw, wl.biases, bool(wl.dims["has_residual"]), act_scales)
    if act_scales is not None:
        raise ValueError("static activation scales are for the FC and convolution kinds")
    d = wl.dims
    if k == 3:
        out, taps = bert_layer(wl.x, qw, wl.biases, d["heads"], d["ln_eps"], {}, "L0.")
        taps["a_ref"] = [out]
        return taps
    return bert_stack(wl.x, qw, wl.biases, d["heads"], d["n_layers"], d["ln_eps"], keep_taps,
                      progress)
