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
        if wl.kind >= si.KIND_BERT_LAYER:
            d = wl.dims
            b, s, hd, nh = d["batch"], d["seq"], d["hidden"], d["heads"]
            outs = []
            for l in range(d["n_layers"]):
                Wl, Bl = W[4 * l:4 * l + 4], B[4 * l:4 * l + 4]
                q, k, v = F.linear(x, Wl[0], Bl[0]).view(b, s, 3, nh, hd // nh).permute(2, 0, 3, 1, 4)
                ctx = F.scaled_dot_product_attention(q, k, v).permute(0, 2, 1, 3).reshape(b, s, hd)
                y1 = F.layer_norm(x + F.linear(ctx, Wl[1], Bl[1]), (hd,), eps=d["ln_eps"])
                x = F.layer_norm(y1 + F.linear(F.gelu(F.linear(y1, Wl[2], Bl[2])), Wl[3], Bl[3]), (hd,), eps=d["ln_eps"])
                outs.append(x.numpy())
            return outs
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


@pytest.mark.parametrize("precision", ["f16", "f32"])
@pytest.mark.parametrize("pad", [0, 1])
def test_oracle_conv_against_brute_force(precision, pad):
    """The contraction step of `conv` is a library routine; here it is checked against the plain
    definition written out as loops (cross-correlation, stride 1, zero padding) on a tiny shape,
    with exact rational sums so that the only rounding is the oracle's single one to float32."""
    from fractions import Fraction
    rng = np.random.default_rng(77 + pad)
    k = 2 * pad + 1
    B, C, H, W, OC = 2, 3, 4, 5, 2
    x = rng.standard_normal((B, C, H, W)).astype(np.float32)
    w = rng.standard_normal((OC, C, k, k)).astype(np.float32)
    bias = rng.standard_normal(OC).astype(np.float32)
    y, xr, acc = fo.conv(x, w, bias, precision, pad, residual=None, relu=False)
    wr = fo.r(w, precision)
    assert np.array_equal(xr, fo.r(x, precision))
    for b in range(B):
        for oc in range(OC):
            for oh in range(H):
                for ow in range(W):
                    s = Fraction(0)
                    for c in range(C):
                        for kh in range(k):
                            for kw in range(k):
                                ih, iw = oh + kh - pad, ow + kw - pad
                                if 0 <= ih < H and 0 <= iw < W:
                                    s += Fraction(float(xr[b, c, ih, iw])) * Fraction(float(wr[oc, c, kh, kw]))
                    want = np.float32(float(s))          # exact sum, rounded once (double rounding via
                    # fp64 cannot matter here: 27 products of 24-bit values stay far from fp32 ties)
                    assert abs(float(acc[b, oc, oh, ow]) - float(want)) <= 2.0 ** -23 * abs(float(want)) + 1e-30
                    assert y[b, oc, oh, ow] == np.float32(acc[b, oc, oh, ow] + bias[oc])
    # a shifted one-hot kernel reproduces the shifted input (orientation: cross-correlation, not convolution)
    if pad == 1:
        w1 = np.zeros((1, 1, 3, 3), np.float32)
        w1[0, 0, 0, 2] = 1.0                              # tap (kh, kw) = (0, 2): output(oh, ow) = x(oh - 1, ow + 1)
        x1 = fo.r(rng.standard_normal((1, 1, 4, 4)).astype(np.float32), precision)
        y1 = fo.conv(x1, w1, None, precision, 1, relu=False)[0]
        want = np.zeros_like(x1)
        want[0, 0, 1:, :-1] = x1[0, 0, :-1, 1:]
        assert np.array_equal(y1, want)


def test_oracle_skip_connection_adds_the_rounded_input():
    wl = si.make_basic_block(b=1, c=4, h=3, w=3, seed=34)
    wl.weights = [np.zeros_like(w) for w in wl.weights]
    wl.biases = [np.zeros_like(b) for b in wl.biases]
    assert np.array_equal(fo.ref_forward(wl, "f16")["a_ref"], np.maximum(fo.r(wl.x, "f16"), 0))
    assert np.array_equal(fo.ref_forward(wl, "f32")["a_ref"], np.maximum(wl.x, 0))


BERT_SMALL = [("bert_layer", lambda: si.make_bert(b=2, s=9, hidden=48, heads=3, ffn=80, n_layers=1, seed=36,
                                                  train_act_dtype="f32")),
              ("bert_stack", lambda: si.make_bert(b=3, s=20, hidden=64, heads=4, ffn=144, n_layers=3, seed=37,
                                                  train_act_dtype="f32"))]


@pytest.mark.parametrize("name,make", BERT_SMALL, ids=[s[0] for s in BERT_SMALL])
def test_oracle_f32_encoder_is_the_plain_fp32_model(name, make):
    wl = make()
    got, want = fo.ref_forward(wl, "f32")["a_ref"], stock_forward(wl)
    assert len(got) == len(want) == wl.dims["n_layers"]
    for l, (g, w) in enumerate(zip(got, want)):
        # fp32 operators against fp64-evaluated ones: rounding of a few hundred-term sums, growing with depth
        assert np.abs(g - w).max() <= 4e-6 * (l + 1) * np.abs(w).max(), l


def test_oracle_gelu_is_the_erf_form():
    # Phi(1) = 0.8413447460685429..., so gelu(1) = Phi(1), gelu(-1) = -(1 - Phi(1)); the tanh
    # approximation gives 0.8411920 for gelu(1) and is told apart by the first assertion
    assert fo.gelu(np.float32(1.0)) == np.float32(0.8413447460685429)
    assert fo.gelu(np.float32(-1.0)) == np.float32(-0.15865525393145707)
    assert fo.gelu(np.float32(0.0)) == 0.0
    v = np.linspace(-9, 9, 4001).astype(np.float32)
    g, gm = fo.gelu(v).astype(np.float64), fo.gelu(-v).astype(np.float64)
    assert np.abs(g - gm - v).max() <= 2.0 ** -23 * np.abs(v).max()      # gelu(v) - gelu(-v) = v
    want = F.gelu(torch.from_numpy(v).double()).numpy()                  # another library's erf
    assert np.array_equal(fo.gelu(v), want.astype(np.float32))
    assert fo.gelu(np.float32(30.0)) == 30.0 and fo.gelu(np.float32(-30.0)) == 0.0


def test_oracle_encoder_worked_example():
    """One token, hidden = ffn = 2, identity weights, no biases.  With a single key the softmax weight is
    1 and the context is the value vector; a layer norm of two distinct numbers gives (+-1) / sqrt(1 + eps/var).
    x = (3, 1): qkv = (3, 1, 3, 1, 3, 1), ctx = (3, 1), x + ctx = (6, 2) -> ln1 = (1, -1) up to eps;
    first feed-forward output = gelu(+-1) = (Phi(1), Phi(1) - 1); second = the same; ln1 + that =
    (1.8413, -1.1587) -> output (1, -1).  At float16 the second feed-forward layer reads Phi(1) rounded to
    float16: 1723 * 2^-11 (Phi(1) * 2^11 = 1723.07) and -(1299.7 -> 1300) * 2^-13."""
    wl = si.make_bert(b=1, s=1, hidden=2, heads=1, ffn=2, n_layers=1, seed=1, train_act_dtype="f32")
    eye = np.eye(2, dtype=np.float32)
    wl.x = np.array([[[3.0, 1.0]]], np.float32)
    wl.weights = [np.concatenate([eye, eye, eye]), eye, eye, eye]
    wl.biases = [np.zeros(6, np.float32), np.zeros(2, np.float32), np.zeros(2, np.float32), np.zeros(2, np.float32)]
    for prec in fo.PRECISIONS:
        t = fo.ref_forward(wl, prec)
        assert np.array_equal(t["L0.l0.y"], [[3, 1, 3, 1, 3, 1]])
        assert np.array_equal(t["L0.l1.x"], [[3, 1]])                                   # the context
        assert np.abs(t["L0.l2.x"] - np.array([[1, -1]])).max() <= 1e-6                  # ln1, before rounding
        assert np.abs(t["L0.l2.y"] - np.array([[0.8413447460685429, -0.15865525393145707]])).max() <= 1e-7
        assert np.abs(t["a_ref"][0] - np.array([[[1, -1]]])).max() <= 1e-6
    t16 = fo.ref_forward(wl, "f16")
    assert np.array_equal(t16["L0.l3.x"], [[1723 * 2.0 ** -11, -1300 * 2.0 ** -13]])
    # a bias on the first feed-forward layer moves the GELU's argument: gelu is applied after the bias
    wl.biases[2] = np.array([-1.0, 1.0], np.float32)
    assert np.abs(fo.ref_forward(wl, "f32")["L0.l2.y"]).max() <= 1e-6


@pytest.mark.parametrize("name,make", BERT_SMALL, ids=[s[0] for s in BERT_SMALL])
def test_oracle_f16_encoder_rounds_only_the_linear_layers(name, make):
    wl = make()
    y16, y32 = fo.ref_forward(wl, "f16"), fo.ref_forward(wl, "f32")
    assert np.array_equal(y16["L0.l0.x"].reshape(-1), fo.r(wl.x, "f16").reshape(-1))
    assert np.array_equal(y32["L0.l0.x"].reshape(-1), wl.x.reshape(-1))
    diff = np.abs(y16["L0.l0.acc"].astype(np.float64) - y32["L0.l0.acc"])
    x, w = np.abs(wl.x.reshape(-1, wl.dims["hidden"]).astype(np.float64)), np.abs(wl.weights[0].astype(np.float64))
    assert (diff <= (2.0 ** -10 + 2.0 ** -21) * (x @ w.T) + 2.0 ** -22 * np.abs(y32["L0.l0.acc"])).all() and diff.max() > 0
    # operands that are float16 values already: the first layer agrees bit for bit, and with it everything
    # up to the next linear layer's input (attention works on float32 values in both)
    wl2 = copy.copy(wl)
    wl2.x = fo.r(wl.x, "f16")
    wl2.weights = [fo.r(w_, "f16") for w_ in wl.weights]
    a, b = fo.ref_forward(wl2, "f16"), fo.ref_forward(wl2, "f32")
    assert np.array_equal(a["L0.l0.y"], b["L0.l0.y"])
    assert np.array_equal(a["L0.l1.x"], fo.r(b["L0.l1.x"], "f16"))      # the context, rounded only at the layer's input


# ----------------------------------------------------------------------------- GPU parity
# The products are exact on both sides (float16 x float16 and float32 x float32 fit the fp32 /
# fp64 accumulators' inputs); the sums differ in accumulation order and width (fp32 on the matrix
# cores, fp64 in the oracle), so outputs agree to fp32 rounding of a K-term sum, not bit for bit:
#   first layer: |y - y*| <= 4e-6 * max|y*|  (K <= 2304 terms of fp32 accumulation)
#   later layers: an input within that distance of a float16 rounding boundary may round the other
#   way; one such input moves an output by at most one float16 ulp of it times a weight, so
#   |y - y*| <= 4e-6 * max|y*| + 2 * 2^-10 * max|input| * max|weight| (float16; two such inputs in one
#   receptive field are already very unlikely), and 2e-5 * max|y*| at float32.
# The cast operands themselves (pure rounding) must be bit-identical to the oracle's.

def _gpu_float_forward(wl, precision):
    from paper_2201_06227_amd import binding as eg
    import tests.gpu_common as gc
    prec = {"f16": eg.REF_F16, "f32": eg.REF_F32}[precision]
    es = 2 if precision == "f16" else 4
    W = [gc.to_dev(w) for w in wl.weights]
    B = [None if b is None else gc.to_dev(b) for b in wl.biases]
    ref = eg.make_float_reference(wl.kind, wl.dims, W, B, prec)
    shapes = gc.tap_shapes(wl)
    cins = {si.KIND_FC_RELU: ["c_in"], si.KIND_BASIC_BLOCK: ["c_in", "c_mid"],
            si.KIND_BOTTLENECK: ["c_in", "c_mid", "c_mid"]}.get(wl.kind)
    if cins is None:
        cins = ["hidden", "hidden", "hidden", "ffn"] * wl.dims["n_layers"]
    for s, key in zip(shapes, cins):
        s["kp"] = eg.op_row_bytes(wl.dims[key], prec)           # the operand tap holds bytes
    taps, bufs, _keep = eg.make_taps(ref, shapes, gc.DEV)
    a_ref = torch.empty(gc.a_ref_numel(wl), dtype=torch.float32, device=gc.DEV)
    ws = eg.workspace(eg.workspace_bytes(ref.desc), gc.DEV)
    eg.ref_forward(ref, gc.to_dev(wl.x), a_ref, ws, taps)
    plain = torch.empty_like(a_ref)
    eg.ref_forward(ref, gc.to_dev(wl.x), plain, ws)
    torch.cuda.synchronize()
    assert eg.check(ws) == eg.OK
    assert torch.equal(plain, a_ref)                            # observed and unobserved runs agree
    np_dt = np.float16 if precision == "f16" else np.float32
    out = []
    for b_, key in zip(bufs, cins):
        c = wl.dims[key]
        xq = b_["x_q"].cpu().numpy().view(np_dt)[:, :c].astype(np.float32)
        pad = b_["x_q"].cpu().numpy().view(np_dt)[:, c:]
        assert not pad.any()
        out.append(dict(x=xq, acc=b_["acc"].cpu().numpy().view(np.float32), y=b_["y"].cpu().numpy()))
    return a_ref.cpu().numpy(), out, ref, ws


def _rows(a):
    """oracle NCHW / [b, c] tensor -> [M, C] rows as the GPU lays them out"""
    return a if a.ndim == 2 else np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1))).reshape(-1, a.shape[1])


FLOAT_CASES = SMALL + [("fc_cfg1", lambda: si.make_config(1)),
                       ("basic_cfg2", lambda: si.make_config(2)),
                       ("bottleneck_mid", lambda: si.make_bottleneck(b=4, c_in=256, c_mid=64, h=14, w=14, seed=35)),
                       ("bottleneck_cfg3", lambda: si.make_config(3))]


@pytest.mark.gpu
@pytest.mark.parametrize("precision", ["f16", "f32"])
@pytest.mark.parametrize("name,make", FLOAT_CASES, ids=[s[0] for s in FLOAT_CASES])
def test_float_reference_matches_oracle(name, make, precision):
    wl = make()
    ot = fo.ref_forward(wl, precision)
    a_ref, taps, ref, ws = _gpu_float_forward(wl, precision)
    n = len(taps)
    for i, t in enumerate(taps):
        want_y = _rows(ot[f"l{i}.y"])
        if i == 0:
            assert np.array_equal(t["x"], _rows(ot["l0.x"]))                    # the cast: bit for bit
            tol = 4e-6 * np.abs(want_y).max()
        elif precision == "f32":
            tol = 2e-5 * np.abs(want_y).max()
        else:
            flips = (t["x"] != _rows(ot[f"l{i}.x"])).mean()
            # float16 boundary cases only: an input y flips when the fp32 sum's error (about 1e-6 max|y|
            # after K = 1024 terms) exceeds its distance to a float16 boundary (spacing 2^-11 |y|), which
            # happens for the small post-ReLU values: below 1 % of the inputs at K = 1024, 0.1 % at K <= 256
            assert flips <= 2e-2
            tol = 4e-6 * np.abs(want_y).max() + 2 * 2.0 ** -10 * np.abs(ot[f"l{i}.x"]).max() * np.abs(wl.weights[i]).max()
        assert np.abs(t["y"] - want_y).max() <= tol, (i, name)
        assert np.abs(t["acc"] - _rows(ot[f"l{i}.acc"])).max() <= tol, (i, name)
    assert np.abs(a_ref - _rows(ot["a_ref"]).reshape(-1)).max() <= tol


@pytest.mark.gpu
@pytest.mark.parametrize("precision", ["f16", "f32"])
@pytest.mark.parametrize("cfg", [2, 3])
def test_float_reference_score(precision, cfg, orc):
    """Plasticity against a float-precision reference (cfg 2 and cfg 3 at full size).
    (i) The metric itself: the fused call equals the metric on the stored activation bit for bit, and
        is within 1e-4 of the fp64 metric evaluated on that same stored activation.
    (ii) End to end against the oracle chain: here the two A_R differ at fp32-rounding level (fp32 sums on
        the matrix cores against fp64 sums rounded once: relative 1e-6 of max|y| per layer, see the
        tolerances above), and P is the squared difference of two Gram matrices that agree to about
        |A_T - A_R| / |A_R| = 1e-2 (the perturbation of the training weights): a relative change d of
        A_R moves P by about 2 d / 1e-2, i.e. 2e-4 for d = 1e-6 - the bar for this leg is 1e-3."""
    from paper_2201_06227_amd import binding as eg
    import tests.gpu_common as gc
    wl = si.make_config(cfg)
    a_ref, taps, ref, ws = _gpu_float_forward(wl, precision)
    a_t = si.train_forward(wl)
    p = torch.zeros(1, dtype=torch.float32, device=gc.DEV)
    eg.plasticity_eval(ref, gc.to_dev(wl.x), [a_t[0].to(gc.DEV)], p, ws)
    sep = eg.plasticity(a_t[0].to(gc.DEV), torch.from_numpy(a_ref).to(gc.DEV).reshape(wl.batch, -1))
    assert p.item() == sep.item()
    same = orc.sp_loss(a_t[0].numpy().reshape(wl.batch, -1), a_ref.reshape(wl.batch, -1))
    assert abs(p.item() - same) <= 1e-4 * abs(same) + 1e-12 * 4.0 / wl.batch, (p.item(), same)
    want = orc.sp_loss(a_t[0].numpy(), _rows(fo.ref_forward(wl, precision)["a_ref"]).reshape(wl.batch, -1))
    assert p.item() == pytest.approx(want, rel=1e-3)


# Encoder layers.  Per linear layer the same two terms as above: fp32 accumulation against the
# oracle's fp64 sums (4e-6 max|y|), and at float16 inputs that round the other way (one float16 ulp
# of the input times a weight each; rows of 768 / 3072 inputs see a handful of them, adding like a
# random walk).  Between the linear layers the deviation is carried along: the layer norm divides by
# the row's standard deviation (about 1 here) and the softmax is 1-Lipschitz in the scores, so the
# bound grows linearly with the number of linear layers passed; `n` counts them.
BERT_CASES = BERT_SMALL + [("bert_ragged", lambda: si.make_bert(b=3, s=77, hidden=200, heads=5, ffn=328, n_layers=2,
                                                                seed=38, train_act_dtype="f32")),
                           ("bert_cfg4", lambda: si.make_config(4))]


@pytest.mark.gpu
@pytest.mark.parametrize("precision", ["f16", "f32"])
@pytest.mark.parametrize("name,make", BERT_CASES, ids=[s[0] for s in BERT_CASES])
def test_float_encoder_matches_oracle(name, make, precision):
    wl = make()
    ot = fo.ref_forward(wl, precision)
    a_ref, taps, ref, ws = _gpu_float_forward(wl, precision)
    d = wl.dims
    per = d["batch"] * d["seq"] * d["hidden"]
    assert np.array_equal(taps[0]["x"], ot["L0.l0.x"])                              # the cast: bit for bit
    for i, t in enumerate(taps):
        l, j = divmod(i, 4)
        want_y, want_x = ot[f"L{l}.l{j}.y"], ot[f"L{l}.l{j}.x"]
        step = 4e-6 * np.abs(want_y).max()
        if precision == "f16":
            if i < 2:       # deeper inputs already carry earlier flips; their values are bounded through y below
                assert (t["x"] != want_x).mean() <= 2e-2, (i, name)
            step += 4 * 2.0 ** -10 * np.abs(want_x).max() * np.abs(wl.weights[i]).max()
        tol = (i + 1) * step
        assert np.abs(t["y"] - want_y).max() <= tol, (i, name, np.abs(t["y"] - want_y).max(), tol)
        assert np.abs(t["acc"] - ot[f"L{l}.l{j}.acc"]).max() <= tol, (i, name)
    for l in range(d["n_layers"]):
        got, want = a_ref[l * per:(l + 1) * per], ot["a_ref"][l].reshape(-1)
        tol = 4 * (l + 1) * (4e-6 if precision == "f32" else 2.0 ** -9) * np.abs(want).max()
        assert np.abs(got - want).max() <= tol, (l, name, np.abs(got - want).max(), tol)


@pytest.mark.gpu
@pytest.mark.parametrize("precision", ["f16", "f32"])
def test_float_encoder_score(precision, orc):
    """Plasticity of every layer of an encoder stack against a float-precision reference, and of cfg 4."""
    from paper_2201_06227_amd import binding as eg
    import tests.gpu_common as gc
    for wl in (BERT_CASES[2][1](), si.make_config(4)):
        a_ref, taps, ref, ws = _gpu_float_forward(wl, precision)
        n, per = wl.dims["n_layers"], wl.batch * wl.dims["seq"] * wl.dims["hidden"]
        a_t = [a.to(gc.DEV) for a in si.train_forward(wl)]
        p = torch.zeros(n, dtype=torch.float32, device=gc.DEV)
        eg.plasticity_eval(ref, gc.to_dev(wl.x), a_t, p, ws)
        torch.cuda.synchronize()
        ot = fo.ref_forward(wl, precision)
        for l in range(n):
            mine = torch.from_numpy(a_ref[l * per:(l + 1) * per]).to(gc.DEV).reshape(wl.batch, -1)
            assert p[l].item() == eg.plasticity(a_t[l], mine).item()
            at = a_t[l].float().cpu().numpy().reshape(wl.batch, -1)
            same = orc.sp_loss(at, a_ref[l * per:(l + 1) * per].reshape(wl.batch, -1))
            assert abs(p[l].item() - same) <= 1e-4 * abs(same) + 1e-12 * 4.0 / wl.batch
            # against the oracle chain: A_R differs by d = 1e-6 (float32) / 1e-4 (float16, inputs that round
            # the other way) relative, and P moves by about 2 d / (|A_T - A_R| / |A_R|)
            want = orc.sp_loss(at, ot["a_ref"][l].reshape(wl.batch, -1))
            assert p[l].item() == pytest.approx(want, rel=1e-3 if precision == "f32" else 3e-2), (wl.name, l)


@pytest.mark.gpu
def test_float_reference_rejects_what_it_does_not_cover():
    from paper_2201_06227_amd import binding as eg
    import tests.gpu_common as gc
    wl = si.make_fc(b=4, k=32, n=8, seed=3)
    ref = gc.build_reference(wl, act_scales=[0.05])
    ref.desc.ref_precision = eg.REF_F16                        # static int8 scales with a float precision
    ws = eg.workspace(1 << 24, gc.DEV)
    a = torch.empty(gc.a_ref_numel(wl), dtype=torch.float32, device=gc.DEV)
    with pytest.raises(eg.EgeriaError) as e:
        eg.ref_forward(ref, gc.to_dev(wl.x), a, ws)
    assert e.value.code == eg.ERR_UNSUPPORTED
