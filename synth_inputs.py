"""Seeded synthetic inputs for the plasticity-evaluation path.

This module only *draws tensors*: mini-batches, snapshot weights, the
perturbations that turn a snapshot into "training" weights, and the training
model's hooked activation A_T (the paper's Section 4.2 takes A_T as a given: it
is whatever the training framework produced, so here it is produced with stock
framework operators in fp32).  It contains none of the method's arithmetic: no
quantisation, no integer GEMM, no plasticity score.  Both the CPU oracle's
tests and the GPU path's tests draw their inputs from here so that the two
sides see identical host arrays.

Shapes follow the workloads of the paper's Table 1 (ResNet-56 on CIFAR-10,
ResNet-50 on ImageNet, BERT-base) but every value is synthetic: the datasets
themselves are not used.

Draw order inside one workload is fixed (x, weights in forward order, biases,
perturbations in forward order) and each workload owns an independent
`numpy.random.default_rng(SEED_BASE + cfg)` stream.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

SEED_BASE = 20220106

KIND_FC_RELU = 0
KIND_BASIC_BLOCK = 1
KIND_BOTTLENECK = 2
KIND_BERT_LAYER = 3
KIND_BERT_STACK = 4


@dataclass
class Workload:
    """One synthetic evaluation problem.

    weights / train_weights: per sub-layer fp32 arrays in framework layout
    ([out, in] for linear, [oc, ic, kh, kw] for conv).  biases: per sub-layer
    fp32 [out] or None.  For BERT kinds the per-layer order is
    (qkv, attn_out, ffn1, ffn2) repeated n_layers times.
    """
    kind: int
    name: str
    x: np.ndarray
    weights: List[np.ndarray]
    biases: List[Optional[np.ndarray]]
    train_weights: List[np.ndarray]
    dims: dict = field(default_factory=dict)
    train_act_dtype: str = "f32"   # "f32" or "bf16"

    @property
    def batch(self) -> int:
        return int(self.x.shape[0])


def _normal(rng, shape, std):
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def make_fc(b=32, k=512, n=512, seed=SEED_BASE + 1, perturb=0.01) -> Workload:
    rng = np.random.default_rng(seed)
    std = 1.0 / math.sqrt(k)                      # N(0, 1/k): second argument is the variance
    x = _normal(rng, (b, k), 1.0)
    w = _normal(rng, (n, k), std)
    e = _normal(rng, (n, k), std)
    wt = (w + np.float32(perturb) * e).astype(np.float32)
    return Workload(KIND_FC_RELU, f"fc_relu_b{b}_k{k}_n{n}", x, [w], [None], [wt],
                    dims=dict(batch=b, c_in=k, c_out=n))


def make_basic_block(b=128, c=16, h=32, w=32, seed=SEED_BASE + 2, perturb=0.01) -> Workload:
    rng = np.random.default_rng(seed)
    std = math.sqrt(2.0 / (c * 9))                # He init, fan_in = c*3*3
    x = _normal(rng, (b, c, h, w), 1.0)
    w1 = _normal(rng, (c, c, 3, 3), std)
    w2 = _normal(rng, (c, c, 3, 3), std)
    b1 = _normal(rng, (c,), 0.1)                  # folded-BN bias ~ N(0, 0.01)
    b2 = _normal(rng, (c,), 0.1)
    e1 = _normal(rng, (c, c, 3, 3), std)
    e2 = _normal(rng, (c, c, 3, 3), std)
    p = np.float32(perturb)
    return Workload(KIND_BASIC_BLOCK, f"basic_block_b{b}_c{c}_{h}x{w}", x, [w1, w2], [b1, b2],
                    [(w1 + p * e1).astype(np.float32), (w2 + p * e2).astype(np.float32)],
                    dims=dict(batch=b, c_in=c, c_mid=c, c_out=c, height=h, width=w, has_residual=1))


def make_bottleneck(b=64, c_in=1024, c_mid=256, h=14, w=14, seed=SEED_BASE + 3,
                    perturb=0.01, has_residual=1) -> Workload:
    rng = np.random.default_rng(seed)
    x = np.abs(_normal(rng, (b, c_in, h, w), 1.0))            # post-ReLU input
    shapes = [(c_mid, c_in, 1, 1), (c_mid, c_mid, 3, 3), (c_in, c_mid, 1, 1)]
    stds = [math.sqrt(2.0 / (s[1] * s[2] * s[3])) for s in shapes]
    ws = [_normal(rng, s, sd) for s, sd in zip(shapes, stds)]
    bs = [_normal(rng, (s[0],), 0.1) for s in shapes]
    es = [_normal(rng, s, sd) for s, sd in zip(shapes, stds)]
    p = np.float32(perturb)
    wt = [(w_ + p * e_).astype(np.float32) for w_, e_ in zip(ws, es)]
    return Workload(KIND_BOTTLENECK, f"bottleneck_b{b}_c{c_in}_{c_mid}_{h}x{w}", x, ws, bs, wt,
                    dims=dict(batch=b, c_in=c_in, c_mid=c_mid, c_out=c_in, height=h, width=w,
                              has_residual=int(has_residual)))


def make_bert(b=32, s=128, hidden=768, heads=12, ffn=3072, n_layers=1, seed=SEED_BASE + 4,
              perturb=0.02, train_act_dtype="bf16") -> Workload:
    rng = np.random.default_rng(seed)
    x = _normal(rng, (b, s, hidden), 1.0)
    shapes = [(3 * hidden, hidden), (hidden, hidden), (ffn, hidden), (hidden, ffn)]
    ws, es = [], []
    for _ in range(n_layers):
        for (o, i) in shapes:
            ws.append(_normal(rng, (o, i), math.sqrt(2.0 / (i + o))))     # Xavier std
    for l in range(n_layers):
        for (o, i) in shapes:
            es.append(_normal(rng, (o, i), math.sqrt(2.0 / (i + o))))
    p = np.float32(perturb)
    wt = [(w_ + p * e_).astype(np.float32) for w_, e_ in zip(ws, es)]
    bs = [np.zeros((w_.shape[0],), np.float32) for w_ in ws]
    kind = KIND_BERT_LAYER if n_layers == 1 else KIND_BERT_STACK
    return Workload(kind, f"bert_b{b}_s{s}_h{hidden}_L{n_layers}", x, ws, bs, wt,
                    dims=dict(batch=b, seq=s, hidden=hidden, heads=heads, ffn=ffn,
                              n_layers=n_layers, ln_eps=1e-12),
                    train_act_dtype=train_act_dtype)


def make_config(cfg: int) -> Workload:
    """The five evaluation workloads at their full sizes (1-based index)."""
    if cfg == 1:
        return make_fc()
    if cfg == 2:
        return make_basic_block()
    if cfg == 3:
        return make_bottleneck()
    if cfg == 4:
        return make_bert(n_layers=1, seed=SEED_BASE + 4, train_act_dtype="bf16")
    if cfg == 5:
        return make_bert(b=64, s=256, n_layers=12, seed=SEED_BASE + 5, train_act_dtype="f32")
    raise ValueError(f"no such config: {cfg}")


def train_forward(wl: Workload, device: str = "cpu"):
    """Hooked activations A_T of the *training* model: fp32 forward with the
    perturbed weights, stock framework operators.  Returns a list of torch
    tensors, one [b, D] activation per layer module (one entry except for the
    stack), in the layout the reference path hooks (NHWC for conv blocks,
    [b, seq*hidden] for BERT), in `wl.train_act_dtype`."""
    import torch
    import torch.nn.functional as F

    dev = torch.device(device)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    x = t(wl.x)
    W = [t(w) for w in wl.train_weights]
    B = [None if b is None else t(b) for b in wl.biases]
    outs = []
    with torch.no_grad():
        if wl.kind == KIND_FC_RELU:
            outs.append(torch.relu(F.linear(x, W[0], B[0])))
        elif wl.kind == KIND_BASIC_BLOCK:
            h = torch.relu(F.conv2d(x, W[0], B[0], padding=1))
            y = F.conv2d(h, W[1], B[1], padding=1)
            y = torch.relu(y + x) if wl.dims["has_residual"] else torch.relu(y)
            outs.append(y.permute(0, 2, 3, 1).contiguous())
        elif wl.kind == KIND_BOTTLENECK:
            h = torch.relu(F.conv2d(x, W[0], B[0]))
            h = torch.relu(F.conv2d(h, W[1], B[1], padding=1))
            y = F.conv2d(h, W[2], B[2])
            y = torch.relu(y + x) if wl.dims["has_residual"] else torch.relu(y)
            outs.append(y.permute(0, 2, 3, 1).contiguous())
        else:
            d = wl.dims
            hd, nh, eps = d["hidden"], d["heads"], d["ln_eps"]
            b, s = x.shape[0], x.shape[1]
            cur = x
            for l in range(d["n_layers"]):
                wq, wo, w1, w2 = W[4 * l:4 * l + 4]
                bq, bo, b1, b2 = B[4 * l:4 * l + 4]
                qkv = F.linear(cur, wq, bq)
                q, k, v = qkv.split(hd, dim=-1)
                sh = lambda z: z.reshape(b, s, nh, hd // nh).permute(0, 2, 1, 3)
                att = torch.softmax(sh(q) @ sh(k).transpose(-1, -2) / math.sqrt(hd // nh), dim=-1)
                ctx = (att @ sh(v)).permute(0, 2, 1, 3).reshape(b, s, hd)
                y = F.layer_norm(cur + F.linear(ctx, wo, bo), (hd,), eps=eps)
                f = F.gelu(F.linear(y, w1, b1))
                cur = F.layer_norm(y + F.linear(f, w2, b2), (hd,), eps=eps)
                outs.append(cur)
    res = []
    for o in outs:
        o = o.reshape(o.shape[0], -1).contiguous()
        if wl.train_act_dtype == "bf16":
            o = o.to(torch.bfloat16)
        res.append(o)
    return res


def noisy_pair(b: int, D: int, rel: float = 0.02, seed: int = SEED_BASE, nonneg: bool = False):
    """A pair of [b, D] fp32 activations for metric-only tests: a common
    component shared by all samples, a per-sample component, and a small
    relative perturbation separating the 'reference' from the 'training' side."""
    rng = np.random.default_rng(seed)
    common = rng.standard_normal((1, D), dtype=np.float32)
    own = rng.standard_normal((b, D), dtype=np.float32)
    a_r = (np.float32(0.5) * common + own).astype(np.float32)
    a_t = (a_r + np.float32(rel) * rng.standard_normal((b, D), dtype=np.float32)).astype(np.float32)
    if nonneg:
        a_r, a_t = np.maximum(a_r, 0), np.maximum(a_t, 0)
    return a_t, a_r
