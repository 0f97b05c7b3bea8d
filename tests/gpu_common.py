"""Helpers shared by the GPU parity tests: run the HIP path of a synthetic
workload through the C-ABI binding and bring its observation points back as
numpy arrays laid out like the oracle's."""
from __future__ import annotations

import numpy as np
import torch

import synth_inputs as si
from paper_2201_06227_amd import binding as eg

DEV = "cuda:0"


def to_dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.to(DEV)


def tap_shapes(wl):
    """Per sub-layer GEMM shapes (M, padded K, N) of a workload."""
    d = wl.dims
    p = eg.padded
    if wl.kind == si.KIND_FC_RELU:
        return [dict(M=d["batch"], kp=p(d["c_in"]), N=d["c_out"])]
    if wl.kind == si.KIND_BASIC_BLOCK:
        M = d["batch"] * d["height"] * d["width"]
        return [dict(M=M, kp=p(d["c_in"]), N=d["c_mid"]), dict(M=M, kp=p(d["c_mid"]), N=d["c_out"])]
    if wl.kind == si.KIND_BOTTLENECK:
        M = d["batch"] * d["height"] * d["width"]
        return [dict(M=M, kp=p(d["c_in"]), N=d["c_mid"]), dict(M=M, kp=p(d["c_mid"]), N=d["c_mid"]),
                dict(M=M, kp=p(d["c_mid"]), N=d["c_out"])]
    M = d["batch"] * d["seq"]
    h, f = d["hidden"], d["ffn"]
    one = [dict(M=M, kp=p(h), N=3 * h), dict(M=M, kp=p(h), N=h), dict(M=M, kp=p(h), N=f),
           dict(M=M, kp=p(f), N=h)]
    return one * d["n_layers"]


def build_reference(wl, act_scales=None):
    W = [to_dev(w) for w in wl.weights]
    B = [None if b is None else to_dev(b) for b in wl.biases]
    st = None if act_scales is None else to_dev(np.asarray(act_scales, np.float32))
    return eg.make_reference(wl.kind, wl.dims, W, B, st)


def a_ref_numel(wl):
    d = wl.dims
    if wl.kind == si.KIND_FC_RELU:
        return d["batch"] * d["c_out"]
    if wl.kind in (si.KIND_BASIC_BLOCK, si.KIND_BOTTLENECK):
        return d["batch"] * d["height"] * d["width"] * d["c_out"]
    return d["n_layers"] * d["batch"] * d["seq"] * d["hidden"]


def run_forward(wl, with_taps=True, act_scales=None):
    """Returns (a_ref [n_layers, b, D] numpy, list of tap dicts of numpy arrays, ref)."""
    ref = build_reference(wl, act_scales)
    x = to_dev(wl.x)
    n_layers = wl.dims.get("n_layers", 1)
    a_ref = torch.empty(a_ref_numel(wl), dtype=torch.float32, device=DEV)
    ws = eg.workspace(eg.workspace_bytes(ref.desc), DEV)
    taps = bufs = None
    if with_taps:
        taps, bufs, _keep = eg.make_taps(ref, tap_shapes(wl), DEV)
    eg.ref_forward(ref, x, a_ref, ws, taps)
    torch.cuda.synchronize()
    assert eg.check(ws) == eg.OK
    out = a_ref.cpu().numpy().reshape(n_layers, wl.batch, -1)
    np_taps = None
    if with_taps:
        np_taps = [{k: v.cpu().numpy() for k, v in b.items()} for b in bufs]
    return out, np_taps, ref


def nhwc(a):
    """Oracle NCHW tensor -> [B*H*W, C] rows as the GPU path lays them out."""
    return np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1))).reshape(-1, a.shape[1])


def assert_int8_rows(gpu_q, want_rows):
    """gpu_q [M, kp] against want [M, K]: equal codes, zero padding."""
    K = want_rows.shape[1]
    assert (gpu_q[:, :K] == want_rows).all()
    assert not gpu_q[:, K:].any()


def assert_conv_q(gpu_q, want_nchw, taps_per_row=1):
    """int8 NHWC [M, cp] against the oracle's NCHW codes."""
    assert_int8_rows(gpu_q, nhwc(want_nchw))


def rel_to_absmax(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


def assert_within_ulp(got, want, max_ulp=1, what=""):
    """fp32 arrays equal up to `max_ulp` units in the last place; returns (and prints, when not zero)
    the number of elements that differ at all.  For tensors that both sides evaluate in fp64 and round
    once: the fp64 values may differ in their last bits (other summation order, another math library),
    which moves a rounded fp32 value by one ulp in about one element in 10^8."""
    got = np.ascontiguousarray(got, dtype=np.float32).reshape(-1)
    want = np.ascontiguousarray(want, dtype=np.float32).reshape(-1)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all() and np.isfinite(want).all(), what
    gi, wi = got.view(np.int32).astype(np.int64), want.view(np.int32).astype(np.int64)
    # order-preserving map of the bit patterns (negative values mirrored)
    gi = np.where(gi < 0, -(gi & 0x7fffffff), gi)
    wi = np.where(wi < 0, -(wi & 0x7fffffff), wi)
    d = np.abs(gi - wi)
    ndiff = int((d != 0).sum())
    assert d.max(initial=0) <= max_ulp, (what, int(d.max()), ndiff)
    if ndiff:
        print(f"{what}: {ndiff} of {d.size} elements differ by one ulp")
    return ndiff
