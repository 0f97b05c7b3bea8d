"""Reference model at float16 / float32 precision (Section 6.4 of the paper,
Table 2: the higher precisions are the fallback when int8 fails): pins of the
CPU oracle, then the library's kernels against the oracle through the C-ABI."""
import copy

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import float_ref_oracle as fo


def stock_forward(wl):
    """The module in plain fp32 with the framework's own operators (independent of the oracle)."""
    t = lambda a: torch.from_numpy(np.asarray(a, np.float32))
    x, W, B = t(wl.x), [t(w) for w in wl.weights], [None if b is None else t(b) for b in wl.biases]
    with torch.no_grad():
        if wl.kind == si.KIND_FC_RELU:
            return torch.relu(F.linear(x, W[0], B[0])).numpy()
        if wl.kind == si.KIND_BASIC_BLOCK:
            h = torch.relu(F.conv2d(x, W[0], B[0], padding=1))
            y = F.conv2d(h, W[1], B[1], padding=1)
        else:
            h = torch.relu(F.conv2d(x, W[0], B[0]))
            h = torch.relu(F.conv2d(h, W[1], B[1], padding=1))
            y = F.conv2d(h, W[2], B[2])
        return torch.relu(y + x if wl.dims["has_residual"] else y).numpy()


SMALL = [("fc", lambda: si.make_fc(b=5, k=100, n=7, seed=31)),
         ("basic", lambda: si.make_basic_block(b=2, c=20, h=9, w=11, seed=32)),
         ("bottleneck", lambda: si.make_bottleneck(b=2, c_in=24, c_mid=12, h=6, w=5, seed=33))]


# ----------------------------------------------------------------------------- oracle pins

def test_oracle_worked_example():
    # x0 = 1 + 2^-11 lies half way between two float16 values and goes to the even one (1.0);
    # 1365/4096 is a float16 value.  f16: 1*2 + 3*(1365/4096) + 0.5; f32 keeps x0 as it is.
    wl = si.make_fc(b=1, k=2, n=1, seed=1)
    wl.x = np.array([[1.0 + 2.0 ** -11, 3.0]], np.float32)
    wl.weights = [np.array([[2.0, 1365.0 / 4096.0]], np.float32)]
    wl.biases = [np.array([0.5], np.float32)]
    assert fo.ref_forward(wl, "f16")["a_ref"][0, 0] == np.float32(3.499755859375)
    assert fo.ref_forward(wl, "f32")["a_ref"][0, 0] == np.float32(3.500732421875)
    wl.biases = [np.array([-4.0], np.float32)]
    assert fo.ref_forward(wl, "f16")["a_ref"][0, 0] == 0.0            # ReLU


@pytest.mark.parametrize("name,make", SMALL, ids=[s[0] for s in SMALL])
def test_oracle_f32_is_the_plain_fp32_model(name, make):
    wl = make()
    got, want = fo.ref_forward(wl, "f32")["a_ref"], stock_forward(wl)
    assert np.abs(got - want).max() <= 2e-6 * np.abs(want).max()


@pytest.mark.parametrize("name,make", SMALL, ids=[s[0] for s in SMALL])
def test_oracle_f16_rounds_weights_and_layer_inputs(name, make):
    wl = make()
    y16, y32 = fo.ref_forward(wl, "f16"), fo.ref_forward(wl, "f32")
    # first layer: each product carries two roundings of 2^-11 relative, the sum one more of 2^-24
    x, w = np.abs(np.asarray(wl.x, np.float64)), np.abs(np.asarray(wl.weights[0], np.float64))
    if wl.kind == si.KIND_FC_RELU:
        mag = x @ w.T
    else:
        mag = F.conv2d(torch.from_numpy(x), torch.from_numpy(w), padding=w.shape[-1] // 2).numpy()
    bound = (2.0 ** -10 + 2.0 ** -21) * mag + 2.0 ** -22 * np.abs(y32["l0.acc"])
    diff = np.abs(y16["l0.acc"].astype(np.float64) - y32["l0.acc"])
    assert (diff <= bound).all() and diff.max() > 0            # within the bound, and rounding does happen
    # operands that are float16 values already: the two precisions agree bit for bit
    wl2 = copy.copy(wl)
    wl2.x = fo.r(wl.x, "f16")
    wl2.weights = [fo.r(w_, "f16") for w_ in wl.weights]
    if wl.kind == si.KIND_FC_RELU:                             # one layer: nothing is rounded in between
        assert np.array_equal(fo.ref_forward(wl2, "f16")["a_ref"], fo.ref_forward(wl2, "f32")["a_ref"])
    else:
        assert np.array_equal(fo.ref_forward(wl2, "f16")["l0.y"], fo.ref_forward(wl2, "f32")["l0.y"])


def test_oracle_skip_connection_adds_the_rounded_input():
    wl = si.make_basic_block(b=1, c=4, h=3, w=3, seed=34)
    wl.weights = [np.zeros_like(w) for w in wl.weights]
    wl.biases = [np.zeros_like(b) for b in wl.biases]
    assert np.array_equal(fo.ref_forward(wl, "f16")["a_ref"], np.maximum(fo.r(wl.x, "f16"), 0))
    assert np.array_equal(fo.ref_forward(wl, "f32")["a_ref"], np.maximum(wl.x, 0))
