"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests touches the GPU path.  Each pin is chosen so that a
plausible mistake in the oracle (a dropped term, a wrong sign or index, a
transposed operand, a different rounding) fails it: hand-derived values,
closed forms, invariants, exact integer brute force, special cases that reduce
to a library routine, and agreement of the int8 reference forward with the
full-precision forward to within quantisation noise.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- metric

def _read_sp_cases():
    cases, cur = [], None
    for line in open(os.path.join(GOLDEN, "sp_loss_hand_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        if key == "case":
            cur = dict(name=rest[0], b=int(rest[1]), D=int(rest[2]))
            cases.append(cur)
        elif key in ("T", "R"):
            cur[key] = np.array([float(v) for v in rest], np.float32).reshape(cur["b"], cur["D"])
        elif key == "P":
            cur["P"] = float(rest[0])
    return cases


@pytest.mark.parametrize("case", _read_sp_cases(), ids=lambda c: c["name"])
def test_sp_loss_hand_examples(orc, case):
    assert orc.sp_loss(case["T"], case["R"]) == pytest.approx(case["P"], rel=1e-13, abs=1e-15)


def test_sp_loss_hand_example_closed_form():
    # the first golden value is 1 - sqrt2/4 - 1/sqrt5 (derivation in the fixture)
    c = _read_sp_cases()[0]
    assert c["P"] == pytest.approx(1 - math.sqrt(2) / 4 - 1 / math.sqrt(5), rel=1e-14)


def test_sp_loss_identity_is_zero(orc):
    a_t, _ = si.noisy_pair(8, 300, seed=1)
    assert orc.sp_loss(a_t, a_t.copy()) == 0.0


@pytest.mark.parametrize("b", [2, 4, 32, 64, 128])
def test_sp_loss_orthogonal_vs_identical_closed_form(orc, b):
    # G_T = I, G_R = 1/sqrt(b) everywhere  =>  P = (2/b)(1 - 1/sqrt(b))
    rng = np.random.default_rng(b)
    D = b + 5
    q_t = np.zeros((b, D), np.float32)
    q_t[np.arange(b), rng.permutation(D)[:b]] = rng.integers(1, 9, b).astype(np.float32)
    q_r = np.tile(rng.integers(-4, 5, (1, D)).astype(np.float32) + np.float32(0.5), (b, 1))
    assert orc.sp_loss(q_t, q_r) == pytest.approx((2.0 / b) * (1 - 1 / math.sqrt(b)), rel=1e-12)


def test_sp_loss_scale_invariance_per_argument(orc):
    a_t, a_r = si.noisy_pair(6, 257, rel=0.3, seed=2)
    p = orc.sp_loss(a_t, a_r)
    assert p > 0
    # powers of two rescale every product exactly
    assert orc.sp_loss(a_t * np.float32(4), a_r * np.float32(-0.125)) == pytest.approx(p, rel=1e-13)
    # arbitrary factors only add the fp32 rounding of the rescaled inputs
    assert orc.sp_loss(a_t * np.float32(3), a_r * np.float32(-0.7)) == pytest.approx(p, rel=1e-5)


def test_sp_loss_feature_and_sample_permutations(orc):
    a_t, a_r = si.noisy_pair(7, 64, rel=0.2, seed=3)
    p = orc.sp_loss(a_t, a_r)
    rng = np.random.default_rng(0)
    # permuting the feature axis of ONE argument changes nothing
    assert orc.sp_loss(a_t[:, rng.permutation(64)], a_r) == pytest.approx(p, rel=1e-12)
    assert orc.sp_loss(a_t, a_r[:, rng.permutation(64)]) == pytest.approx(p, rel=1e-12)
    # the same sample permutation on BOTH arguments changes nothing ...
    sp = rng.permutation(7)
    assert orc.sp_loss(a_t[sp], a_r[sp]) == pytest.approx(p, rel=1e-12)
    # ... but permuting the samples of one argument only does (pairs are matched)
    assert abs(orc.sp_loss(a_t[sp], a_r) - p) > 1e-3 * p
    # an orthogonal rotation of the feature axis changes nothing either (up to fp32 inputs)
    q, _ = np.linalg.qr(rng.standard_normal((64, 64)))
    rot = (a_t.astype(np.float64) @ q).astype(np.float32)
    assert orc.sp_loss(rot, a_r) == pytest.approx(p, rel=1e-4)


def test_sp_loss_range(orc):
    rng = np.random.default_rng(4)
    for b in (2, 5, 16):
        for _ in range(5):
            a_t = rng.standard_normal((b, 9)).astype(np.float32)
            a_r = rng.standard_normal((b, 9)).astype(np.float32)
            assert 0 <= orc.sp_loss(a_t, a_r) < 4.0 / b
            assert 0 <= orc.sp_loss(np.abs(a_t), np.abs(a_r)) <= 2.0 / b


def test_sp_loss_degenerate_rows(orc):
    a_t, a_r = si.noisy_pair(4, 10, seed=5)
    a_r[2] = 0                                    # a sample whose activation is all zero
    p = orc.sp_loss(a_t, a_r)
    assert np.isfinite(p) and p > 0
    one = np.array([[1.0, -2.0, 3.0]], np.float32)
    assert orc.sp_loss(one, 5 * one[:, ::-1].copy()) == 0.0     # b = 1: G = [1] on both sides


def test_sp_loss_matches_float64_library_formula(orc):
    a_t, a_r = si.noisy_pair(12, 1000, rel=0.05, seed=6)
    def g(a):
        a = a.astype(np.float64)
        m = a @ a.T
        return m / np.linalg.norm(m, axis=1, keepdims=True)
    expect = ((g(a_t) - g(a_r)) ** 2).sum() / 144
    p, gt, gr = orc.sp_loss(a_t, a_r, return_grams=True)
    assert p == pytest.approx(expect, rel=1e-10)
    assert np.allclose(gt, a_t.astype(np.float64) @ a_t.astype(np.float64).T, rtol=1e-12)
    assert np.allclose(gr, gr.T)


def test_sp_loss_distinguishes_arguments(orc):
    # P is symmetric in its two arguments, and grows with the perturbation
    a_t, a_r = si.noisy_pair(8, 128, rel=0.02, seed=7)
    a_t2, _ = si.noisy_pair(8, 128, rel=0.2, seed=7)
    assert orc.sp_loss(a_t, a_r) == pytest.approx(orc.sp_loss(a_r, a_t), rel=1e-12)
    assert orc.sp_loss(a_t2, a_r) > 10 * orc.sp_loss(a_t, a_r)


# --------------------------------------------------------------------------- quantise

def _read_quant_cases():
    cases, cur = [], {}
    for line in open(os.path.join(GOLDEN, "quantize_worked_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *rest = line.split()
        cur[key] = [float(v) for v in rest]
        if key == "scale":
            cases.append(cur)
            cur = {}
    return cases


@pytest.mark.parametrize("case", _read_quant_cases())
def test_quantize_worked_examples(orc, case):
    q, s = orc.quantize(np.array(case["x"], np.float32))
    assert q.tolist() == [int(v) for v in case["q"]]
    assert s == np.float32(np.float64(np.float32(max(abs(v) for v in case["x"]))) / 127.0)
    assert float(s) == pytest.approx(case["scale"][0], rel=1e-6)


def test_quantize_roundtrip_error_at_most_half_a_step(orc):
    rng = np.random.default_rng(10)
    for scale_pow in (-20, 0, 13):
        x = (rng.standard_normal(20000) * 2.0 ** scale_pow).astype(np.float32)
        q, s = orc.quantize(x)
        xh = orc.dequantize(q, s)
        assert np.abs(x.astype(np.float64) - xh.astype(np.float64)).max() <= float(s) / 2 * (1 + 1e-4)
        assert np.abs(q[np.abs(x).argmax()]) == 127
        assert q.min() >= -127


def test_quantize_odd_symmetry_grid_points_and_pow2_rescale(orc):
    rng = np.random.default_rng(11)
    x = rng.standard_normal(5000).astype(np.float32)
    q, s = orc.quantize(x)
    qn, sn = orc.quantize(-x)
    assert (qn == -q).all() and sn == s
    q8, s8 = orc.quantize(x * np.float32(8))
    assert (q8 == q).all() and s8 == s * np.float32(8)
    # grid points k*scale of a tensor with a power-of-two step are recovered exactly
    k = rng.integers(-127, 128, 4000)
    k[0] = 127
    grid = (k * 0.25).astype(np.float32)
    qg, sg = orc.quantize(grid)
    assert sg == np.float32(0.25) and (qg == k).all()


def test_quantize_zero_tiny_static_and_nonfinite(orc):
    q, s = orc.quantize(np.zeros(17, np.float32))
    assert s == 1.0 and not q.any()
    q, s = orc.quantize(np.full(5, 1e-40, np.float32))          # 127/absmax overflows fp32
    assert s == 1.0 and not q.any()
    q, s = orc.quantize(np.array([0.26, -3.0, 100.0, 0.24], np.float32), fixed_scale=0.5)
    assert s == np.float32(0.5) and q.tolist() == [1, -6, 127, 0]   # static scale saturates
    for bad in (np.nan, np.inf, -np.inf):
        with pytest.raises(orc.NonFiniteInput):
            orc.quantize(np.array([1.0, bad], np.float32))


# --------------------------------------------------------------------------- integer contractions

def test_gemm_i8_brute_force_and_bounds(orc):
    rng = np.random.default_rng(20)
    x = rng.integers(-127, 128, (5, 7)).astype(np.int8)
    w = rng.integers(-127, 128, (3, 7)).astype(np.int8)
    acc = orc.gemm_i8(x, w)
    for m in range(5):
        for n in range(3):
            assert acc[m, n] == sum(int(x[m, k]) * int(w[n, k]) for k in range(7))
    # weights are [out, in]: a one-hot weight row n selecting feature k copies column k
    w1 = np.zeros((7, 7), np.int8)
    perm = rng.permutation(7)
    w1[np.arange(7), perm] = 1
    assert (orc.gemm_i8(x, w1) == x[:, perm]).all()
    # extreme values: |acc| reaches K*127^2 without overflow
    K = 3072
    xe = np.full((2, K), 127, np.int8)
    we = np.full((2, K), -127, np.int8)
    assert (orc.gemm_i8(xe, we) == -K * 127 * 127).all()


def test_gemm_i8_matches_float64_matmul(orc):
    rng = np.random.default_rng(21)
    x = rng.integers(-127, 128, (37, 200)).astype(np.int8)
    w = rng.integers(-127, 128, (29, 200)).astype(np.int8)
    ref = x.astype(np.float64) @ w.astype(np.float64).T          # exact below 2^53
    assert (orc.gemm_i8(x, w) == ref.astype(np.int64)).all()


def test_conv_i8_shift_kernels_and_padding(orc):
    rng = np.random.default_rng(22)
    x = rng.integers(-127, 128, (2, 3, 5, 6)).astype(np.int8)
    for kh in range(3):
        for kw in range(3):
            w = np.zeros((3, 3, 3, 3), np.int8)
            for c in range(3):
                w[c, c, kh, kw] = 1
            acc = orc.conv2d_i8(x, w, 1)
            # cross-correlation: out[oh, ow] = in[oh + kh - 1, ow + kw - 1], zero outside
            pad = np.pad(x.astype(np.int32), ((0, 0), (0, 0), (1, 1), (1, 1)))
            assert (acc == pad[:, :, kh:kh + 5, kw:kw + 6]).all()


def test_conv_i8_matches_library_conv_and_im2col(orc):
    rng = np.random.default_rng(23)
    x = rng.integers(-127, 128, (2, 4, 6, 5)).astype(np.int8)
    w = rng.integers(-127, 128, (3, 4, 3, 3)).astype(np.int8)
    acc = orc.conv2d_i8(x, w, 1)
    ref = F.conv2d(torch.from_numpy(x.astype(np.float64)), torch.from_numpy(w.astype(np.float64)),
                   padding=1).numpy()
    assert (acc == ref.astype(np.int64)).all()
    cols = F.unfold(torch.from_numpy(x.astype(np.float64)), 3, padding=1)     # [B, C*9, H*W]
    cols = cols.permute(0, 2, 1).reshape(-1, 36).numpy().astype(np.int8)
    g = orc.gemm_i8(cols, w.reshape(3, 36)).reshape(2, 30, 3).transpose(0, 2, 1).reshape(2, 3, 6, 5)
    assert (acc == g).all()
    # 1x1, no padding
    w1 = rng.integers(-127, 128, (5, 4, 1, 1)).astype(np.int8)
    ref1 = np.einsum("bchw,oc->bohw", x.astype(np.int64), w1[:, :, 0, 0].astype(np.int64))
    assert (orc.conv2d_i8(x, w1, 0) == ref1).all()


# --------------------------------------------------------------------------- epilogue

def _round_f32(fr: Fraction) -> np.float32:
    """Round an exact rational to the nearest fp32 (ties to even)."""
    if fr == 0:
        return np.float32(0)
    sign = -1 if fr < 0 else 1
    fr = abs(fr)
    e = math.floor(math.log2(float(fr)))
    while Fraction(2) ** e > fr:
        e -= 1
    while Fraction(2) ** (e + 1) <= fr:
        e += 1
    ulp = Fraction(2) ** (e - 23)
    n = fr / ulp
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return np.float32(sign * float(lo * ulp))


def test_epilogue_is_single_rounding_fma_then_residual_then_relu(orc):
    rng = np.random.default_rng(30)
    acc = rng.integers(-(1 << 23), 1 << 23, (64, 3)).astype(np.int32)
    sx, sw = np.float32(0.0123456), np.float32(0.00071234)
    bias = rng.standard_normal(3).astype(np.float32)
    res = rng.standard_normal((64, 3)).astype(np.float32)
    s = np.float32(sx * sw)
    y0 = orc.dequant_bias_act(acc, sx, sw, bias)
    y1 = orc.dequant_bias_act(acc, sx, sw, bias, orc.ACT_RELU, res)
    differs_from_two_roundings = 0
    for m in range(64):
        for n in range(3):
            exact = Fraction(int(acc[m, n])) * Fraction(float(s)) + Fraction(float(bias[n]))
            v = _round_f32(exact)
            assert y0[m, n] == v
            two = np.float32(np.float32(acc[m, n]) * s) + bias[n]
            differs_from_two_roundings += int(two != v)
            r = np.float32(v + res[m, n])
            assert y1[m, n] == (r if r > 0 else np.float32(0))
    assert differs_from_two_roundings > 0        # the test can tell fma from mul+add
    # NCHW indexing: bias is per channel (second axis)
    acc4 = rng.integers(-1000, 1000, (2, 3, 2, 2)).astype(np.int32)
    y4 = orc.dequant_bias_act(acc4, 1.0, 1.0, np.array([10, 20, 30], np.float32))
    assert (y4 == acc4 + np.array([10, 20, 30], np.float32)[None, :, None, None]).all()


def test_epilogue_gelu_is_erf_form(orc):
    from scipy.special import erf
    v = np.linspace(-6, 6, 241)
    acc = np.round(v * 1000).astype(np.int32).reshape(-1, 1)
    y = orc.dequant_bias_act(acc, 0.001, 1.0, None, orc.ACT_GELU)[:, 0]
    vin = (acc[:, 0].astype(np.float32) * np.float32(np.float32(0.001) * np.float32(1.0))).astype(np.float64)
    ref = 0.5 * vin * (1 + erf(vin / math.sqrt(2)))
    assert np.allclose(y, ref, rtol=2e-7, atol=1e-12)
    assert y[120] == 0 and y[-1] == pytest.approx(6.0, rel=1e-6) and abs(y[0]) < 1e-7
    # the tanh approximation differs from the erf form by up to ~5e-4: make sure we are not it
    tanh_form = 0.5 * vin * (1 + np.tanh(math.sqrt(2 / math.pi) * (vin + 0.044715 * vin ** 3)))
    assert np.abs(tanh_form - ref).max() > 1e-4 > np.abs(y - ref).max()


# --------------------------------------------------------------------------- fp32 glue

def test_layernorm_matches_library_and_invariants(orc):
    rng = np.random.default_rng(40)
    x = rng.standard_normal((9, 48)).astype(np.float32) * 3 + 1
    r = rng.standard_normal((9, 48)).astype(np.float32)
    g = rng.standard_normal(48).astype(np.float32)
    bt = rng.standard_normal(48).astype(np.float32)
    y = orc.layernorm(x, r, g, bt, eps=1e-12)
    ref = F.layer_norm(torch.from_numpy(x).double() + torch.from_numpy(r).double(), (48,),
                       torch.from_numpy(g).double(), torch.from_numpy(bt).double(), eps=1e-12)
    assert np.allclose(y, ref.numpy(), rtol=1e-6, atol=1e-6)
    y0 = orc.layernorm(x)
    assert np.allclose(y0.mean(1), 0, atol=1e-6) and np.allclose(y0.var(1), 1, rtol=1e-5)


def test_attention_matches_library_and_special_cases(orc):
    rng = np.random.default_rng(41)
    B, S, Hd, nh = 2, 11, 24, 3
    qkv = rng.standard_normal((B, S, 3 * Hd)).astype(np.float32)
    ctx = orc.attention(qkv, nh)
    t = torch.from_numpy(qkv).double()
    q, k, v = [z.reshape(B, S, nh, Hd // nh).permute(0, 2, 1, 3) for z in t.split(Hd, -1)]
    ref = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).reshape(B, S, Hd).numpy()
    assert np.allclose(ctx, ref, rtol=1e-6, atol=1e-6)
    # zero queries: uniform attention, the context is the mean of the values
    z = qkv.copy()
    z[:, :, :Hd] = 0
    assert np.allclose(orc.attention(z, nh), np.broadcast_to(z[:, :, 2 * Hd:].mean(1, keepdims=True),
                                                             (B, S, Hd)), atol=1e-6)


# --------------------------------------------------------------------------- whole layer modules

def _rel_err(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return np.linalg.norm(a - b) / np.linalg.norm(b)


def _fp32_forward_with_ref_weights(wl):
    import copy
    w2 = copy.copy(wl)
    w2.train_weights = wl.weights
    w2.train_act_dtype = "f32"
    return [t.numpy() for t in si.train_forward(w2)]


def _to_nhwc_flat(y):
    return np.ascontiguousarray(np.transpose(y, (0, 2, 3, 1))).reshape(y.shape[0], -1)


def test_fc_block_on_integer_grid_is_exact(orc):
    # inputs already on the int8 grid with absmax 127 quantise losslessly (scale 1),
    # so the reference forward must equal the exact integer product, then ReLU
    rng = np.random.default_rng(50)
    x = rng.integers(-127, 128, (6, 40)).astype(np.float32)
    w = rng.integers(-127, 128, (9, 40)).astype(np.float32)
    x[0, 0], w[0, 0] = 127, -127
    taps = orc.fc_relu(x, orc.quantize_weights([w]), [None])
    assert taps["l0.sx"] == 1.0
    assert (taps["a_ref"] == np.maximum(x.astype(np.int64) @ w.astype(np.int64).T, 0)).all()


@pytest.mark.parametrize("maker,kw,tol", [
    (si.make_fc, dict(b=16, k=96, n=40, seed=51), 0.02),
    (si.make_basic_block, dict(b=3, c=8, h=7, w=6, seed=52), 0.04),
    (si.make_bottleneck, dict(b=2, c_in=32, c_mid=16, h=5, w=5, seed=53), 0.04),
    (si.make_bottleneck, dict(b=2, c_in=32, c_mid=16, h=5, w=5, seed=54, has_residual=0), 0.06),
    (si.make_bert, dict(b=2, s=12, hidden=48, heads=4, ffn=96, n_layers=1, seed=55), 0.04),
    (si.make_bert, dict(b=2, s=12, hidden=48, heads=4, ffn=96, n_layers=3, seed=56), 0.06),
])
def test_int8_reference_tracks_full_precision_forward(orc, maker, kw, tol):
    """The quantised reference must agree with the fp32 model on the same weights
    to within quantisation noise (Section 4.1: the reference stays an accurate
    stand-in).  A dropped bias, residual, activation or a misplaced pad shows up
    as an error an order of magnitude above this."""
    wl = maker(**kw)
    taps = orc.ref_forward(wl)
    full = _fp32_forward_with_ref_weights(wl)
    a_ref = taps["a_ref"]
    if wl.kind in (si.KIND_BASIC_BLOCK, si.KIND_BOTTLENECK):
        a_ref = [_to_nhwc_flat(a_ref)]
    elif wl.kind == si.KIND_FC_RELU:
        a_ref = [a_ref]
    assert len(a_ref) == len(full)
    for got, want in zip(a_ref, full):
        err = _rel_err(got.reshape(want.shape), want)
        assert 0 < err < tol, err


def test_plasticity_of_config_like_blocks_is_small_and_positive(orc):
    wl = si.make_basic_block(b=8, c=8, h=6, w=6, seed=57)
    a_ref = _to_nhwc_flat(orc.ref_forward(wl)["a_ref"])
    a_t = si.train_forward(wl)[0].numpy()
    p = orc.sp_loss(a_t, a_ref)
    assert 0 < p < 1e-3


def test_static_scales_reduce_to_dynamic_and_saturate(orc):
    """Static activation scales (Section 5): with each scale equal to the tensor's own absmax / 127 the
    forward is the dynamic one bit for bit; with a smaller scale values saturate at +-127 and the
    round-trip error of an unsaturated value is still at most scale / 2."""
    import synth_inputs as si
    for wl in (si.make_fc(b=6, k=40, n=9, seed=11), si.make_basic_block(b=2, c=5, h=6, w=5, seed=12),
               si.make_bottleneck(b=2, c_in=12, c_mid=6, h=4, w=5, seed=13)):
        dyn = orc.ref_forward(wl)
        scales = [float(dyn[f"l{i}.sx"]) for i in range(len(wl.weights))]
        st = orc.ref_forward(wl, act_scales=scales)
        for k in dyn:
            assert np.array_equal(np.asarray(dyn[k]), np.asarray(st[k])), k
    x = np.linspace(-3, 3, 61).astype(np.float32)
    q, s = orc.quantize(x, fixed_scale=0.01)
    assert s == np.float32(0.01)
    assert q.min() == -127 and q.max() == 127 and (q[np.abs(x) > 1.28] != 0).all()
    inside = np.abs(x) <= 1.27
    assert (np.abs(x[inside] - q[inside].astype(np.float32) * s) <= 0.005 * (1 + 1e-4)).all()


def test_per_channel_weight_scales(orc):
    """One scale per output channel: every channel obeys the per-tensor rule on its own (its largest
    weight maps to +-127, round-trip error <= scale_c / 2); a channel-wise rescaling of the weights leaves
    the codes unchanged and, with power-of-two factors, rescales the outputs exactly; and a matrix whose rows
    differ by orders of magnitude is represented far better than with one scale."""
    import synth_inputs as si
    rng = np.random.default_rng(3)
    w = rng.standard_normal((12, 40)).astype(np.float32) * np.logspace(-3, 1, 12, dtype=np.float32)[:, None]
    q, s = orc.quantize_per_channel(w)
    assert s.shape == (12,) and (np.abs(q).max(axis=1) == 127).all()
    assert (np.abs(w - q.astype(np.float32) * s[:, None]) <= 0.5 * s[:, None] * (1 + 1e-4)).all()
    for o in range(12):
        qo, so = orc.quantize(w[o])
        assert so == s[o] and np.array_equal(qo, q[o])
    qt, st = orc.quantize(w)
    err_pc = np.abs(w - q.astype(np.float32) * s[:, None]).sum(axis=1) / np.abs(w).sum(axis=1)
    err_pt = np.abs(w - qt.astype(np.float32) * st).sum(axis=1) / np.abs(w).sum(axis=1)
    assert err_pc.max() < 0.02 and err_pt[0] > 0.9          # the small rows vanish under one scale
    # channel-wise power-of-two rescaling: same codes, outputs scaled exactly
    wl = si.make_fc(b=5, k=24, n=6, seed=21)
    f = np.array([1, 2, 0.5, 4, 8, 0.25], np.float32)
    qw1 = orc.quantize_weights(wl.weights, per_channel=True)
    qw2 = orc.quantize_weights([wl.weights[0] * f[:, None]], per_channel=True)
    assert np.array_equal(qw1[0][0], qw2[0][0]) and np.array_equal(qw1[0][1] * f, qw2[0][1])
    nb = [None]
    y1 = orc.fc_relu(wl.x, qw1, nb)["a_ref"]
    y2 = orc.fc_relu(wl.x, qw2, nb)["a_ref"]
    assert np.array_equal(y1 * f[None, :], y2)
    # a uniform scale vector is the per-tensor epilogue
    acc = rng.integers(-5000, 5000, size=(7, 6)).astype(np.int32)
    a = orc.dequant_bias_act(acc, 0.01, np.float32(0.03), None, orc.ACT_RELU)
    b = orc.dequant_bias_act(acc, 0.01, np.full(6, 0.03, np.float32), None, orc.ACT_RELU)
    assert np.array_equal(a, b)
