"""Affine (asymmetric) uint8 activations (Section 5 of the paper: the framework's quantisation, whose
default activation code has a zero point): pins of the CPU oracle, then the library against the oracle
through the C-ABI."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import affine_oracle as ao
from oracle import oracle as orc


# ----------------------------------------------------------------------------- oracle pins

def test_worked_example():
    # extrema -1 and 3: scale = 4/255, lo/scale = -63.75 -> zero point 64; 3 * 63.75 = 191.25 -> 191 + 64 = 255
    x = np.array([-1.0, 0.0, 0.5, 3.0], np.float32)
    q, s, zp = ao.quantize(x)
    assert s == np.float32(np.float32(4.0) / np.float32(255.0)) and zp == 64
    assert q.tolist() == [0, 64, 96, 255]                         # 0.5 * 63.75 = 31.875 -> 32
    assert ao.dequantize(q, s, zp)[1] == 0.0                       # zero is a code
    # all values positive: the range still starts at zero, zero point 0
    q, s, zp = ao.quantize(np.array([2.0, 5.0], np.float32))
    assert zp == 0 and s == np.float32(np.float32(5.0) / np.float32(255.0)) and q.tolist() == [102, 255]
    # all values negative: zero point 255
    q, s, zp = ao.quantize(np.array([-2.0, -5.0], np.float32))
    assert zp == 255 and q.tolist() == [153, 0]
    # a tensor of zeros: the smallest scale, zero point 0, codes 0
    q, s, zp = ao.quantize(np.zeros(5, np.float32))
    assert s == np.float32(2.0 ** -23) and zp == 0 and not q.any()


@pytest.mark.parametrize("seed", range(6))
def test_against_the_frameworks_observer_and_quantiser(seed):
    """The reading is the framework's min/max observer and per-tensor quantiser: same scale, same zero point,
    same codes (another implementation of the same float32 operations)."""
    from torch.ao.quantization.observer import MinMaxObserver
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal(20000) * rng.uniform(0.01, 30) + rng.uniform(-3, 3)).astype(np.float32)
    if seed == 4:
        x = np.abs(x)
    if seed == 5:
        x = -np.abs(x)
    q, s, zp = ao.quantize(x)
    obs = MinMaxObserver(dtype=torch.quint8, qscheme=torch.per_tensor_affine, reduce_range=False)
    obs(torch.from_numpy(x))
    ts, tz = obs.calculate_qparams()
    assert np.float32(ts.item()) == s and int(tz.item()) == zp
    tq = torch.quantize_per_tensor(torch.from_numpy(x), float(s), zp, torch.quint8).int_repr().numpy()
    assert np.array_equal(tq, q)


def test_round_trip_and_monotonicity():
    rng = np.random.default_rng(11)
    x = np.sort((rng.standard_normal(5000) * 2 - 0.7).astype(np.float32))
    q, s, zp = ao.quantize(x)
    assert (np.diff(q.astype(np.int32)) >= 0).all()                # codes are monotone in x
    assert q.min() == 0 and q.max() == 255                         # both ends of the range are used
    err = np.abs(ao.dequantize(q, s, zp).astype(np.float64) - x)
    assert err.max() <= 0.5 * float(s) * (1 + 1e-5) + 1e-7         # half a step inside the range


def test_linear_against_exact_rational_arithmetic():
    """acc = sum (q - zp) w exactly; y = one fma of (float) acc with the float32 product of the scales."""
    rng = np.random.default_rng(12)
    x = rng.standard_normal((3, 7)).astype(np.float32) + 0.4
    w = rng.standard_normal((4, 7)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    wq, sw = orc.quantize(w)
    taps = {}
    y = ao.linear(x, wq, sw, b, ao.ACT_NONE, taps, "")
    q, s, zp = ao.quantize(x)
    for m in range(3):
        for n in range(4):
            acc = sum((int(q[m, k]) - zp) * int(wq[n, k]) for k in range(7))
            assert taps["acc"][m, n] == acc
            exact = Fraction(acc) * Fraction(float(np.float32(s * sw))) + Fraction(float(b[n]))
            want = np.float32(float(exact))                         # the fma rounds once
            assert y[m, n] == want
    # the centred codes times the scale reproduce x to half a step, so y is close to the fp32 layer
    assert np.abs(y - (x @ w.T + b)).max() <= 0.5 * float(s) * np.abs(w).sum(axis=1).max() + 0.5 * float(sw) * np.abs(x).sum(axis=1).max() + 1e-3


def test_padding_is_the_real_value_zero():
    """A 3x3 window over the image border sees centred code 0 there: with weights of ones the accumulator of a
    corner pixel is the sum of the four centred codes inside the image."""
    x = (np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4) - 5.0)
    q, s, zp = ao.quantize(x)
    w = np.ones((1, 1, 3, 3), np.float32)
    wq, sw = orc.quantize(w)
    taps = {}
    ao._conv(q, s, zp, wq, sw, None, 1, ao.ACT_NONE, None, taps, "")
    c = q.astype(np.int32) - zp
    assert zp != 0 and zp != 128
    assert taps["acc"][0, 0, 0, 0] == 127 * (c[0, 0, 0, 0] + c[0, 0, 0, 1] + c[0, 0, 1, 0] + c[0, 0, 1, 1])
    assert taps["acc"][0, 0, 1, 1] == 127 * c[0, 0, :3, :3].sum()


SMALL = [("fc", lambda: si.make_fc(b=5, k=100, n=7, seed=41)),
         ("basic", lambda: si.make_basic_block(b=2, c=20, h=9, w=11, seed=42)),
         ("bottleneck", lambda: si.make_bottleneck(b=2, c_in=24, c_mid=12, h=6, w=5, seed=43)),
         ("bert", lambda: si.make_bert(b=2, s=9, hidden=48, heads=3, ffn=80, n_layers=2, seed=44, train_act_dtype="f32"))]


@pytest.mark.parametrize("name,make", SMALL, ids=[s[0] for s in SMALL])
def test_affine_reference_tracks_the_fp32_model(name, make):
    """End to end the affine reference stays as close to the fp32 module as the symmetric one does (the
    plasticity of identical weights is small), and is not the same computation as the symmetric one."""
    wl = make()
    a = ao.ref_forward(wl)["a_ref"]
    b_ = orc.ref_forward(wl)["a_ref"]
    a = a[-1] if isinstance(a, list) else a
    b_ = b_[-1] if isinstance(b_, list) else b_
    assert a.shape == b_.shape and not np.array_equal(a, b_)
    assert np.abs(a - b_).max() <= 0.2 * np.abs(b_).max()
