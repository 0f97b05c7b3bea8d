"""Pre-allocated driver of one plasticity evaluation: every buffer (quantised
weights, scales, workspaces, scores) is allocated once, so that a step is a
fixed sequence of C-ABI calls with no allocation and no host synchronisation.
Argument marshalling only; all arithmetic is in libegeria's kernels."""
from __future__ import annotations

import ctypes
from typing import Optional, Sequence

import torch

from . import binding as eg


class PlasticityEvaluator:
    """One layer module (or stack): snapshot weights -> int8 reference ->
    reference forward on the mini-batch -> one score per layer.

    step() = reference-model generation (weight quantisation, Section 4.1) +
    reference forward + plasticity (Section 4.2, Eq. 1), all enqueued on the
    current stream; scores land in `self.p_out`."""

    def __init__(self, kind: int, dims: dict, weights: Sequence[torch.Tensor],
                 biases: Sequence[Optional[torch.Tensor]], device="cuda",
                 act_scales: Optional[torch.Tensor] = None, per_channel: bool = False):
        self.weights = [w.contiguous() for w in weights]
        self.biases = list(biases)
        self.desc = eg.make_desc(kind, dims)
        self.n_layers = self.desc.n_layers
        self.w_q, self.scales = [], []
        for w in self.weights:
            if w.dim() == 4:
                o, i, kh, kw = w.shape
                shape = (o, kh, kw, eg.padded(i))
            else:
                shape = (w.shape[0], eg.padded(w.shape[1]))
            self.w_q.append(torch.empty(shape, dtype=torch.int8, device=device))
            self.scales.append(torch.empty(w.shape[0] if per_channel else 1, dtype=torch.float32, device=device))
        self._lin = (eg.QLinear * len(self.weights))()
        for i in range(len(self.weights)):
            self._lin[i].per_channel = 1 if per_channel else 0
            self._lin[i].w_q = self.w_q[i].data_ptr()
            self._lin[i].scale = self.scales[i].data_ptr()
            self._lin[i].bias = 0 if self.biases[i] is None else self.biases[i].data_ptr()
        self.qw = eg.QWeights()
        self.qw.n_linear = len(self.weights)
        self.qw.linear = self._lin
        self.qw.n_norm = 0
        self.qw.norm = None
        # static activation scales (fp32 [n_linear] on the device) or None for dynamic ones
        self.act_scales = act_scales
        self.qw.act_scale = None if act_scales is None else act_scales.data_ptr()
        self.qws = eg.workspace(eg.quantize_weights_workspace_bytes(len(self.weights)), device)
        self._wtab = eg.weight_table(self.weights, self.w_q, self.scales, per_channel)
        nbytes = eg.workspace_bytes(self.desc)
        if nbytes == 0:
            raise ValueError("invalid layer-module description")
        self.ws = eg.workspace(nbytes, device)
        self.p_out = torch.zeros(self.n_layers, dtype=torch.float32, device=device)
        self._lib = eg.lib()

    def quantize_weights(self):
        rc = self._lib.egeria_quantize_weights(self._wtab, len(self.weights), self.qws.data_ptr(), self.qws.numel(),
                                               eg._stream())
        eg._check(rc, "egeria_quantize_weights")

    def evaluate(self, x: torch.Tensor, a_train: Sequence[torch.Tensor]) -> torch.Tensor:
        ptrs = (ctypes.c_void_p * self.n_layers)(*[t.data_ptr() for t in a_train])
        rc = self._lib.egeria_plasticity_eval(ctypes.byref(self.desc), ctypes.byref(self.qw), x.data_ptr(),
                                              eg._dt(x), ptrs, eg._dt(a_train[0]), self.p_out.data_ptr(),
                                              self.ws.data_ptr(), self.ws.numel(), eg._stream())
        eg._check(rc, "egeria_plasticity_eval")
        return self.p_out

    def step(self, x: torch.Tensor, a_train: Sequence[torch.Tensor]) -> torch.Tensor:
        """egeria_refresh_eval: quantize_weights() + evaluate() in one call (same results; the snapshot's
        first pass and the mini-batch's maximum pass share a launch)."""
        ptrs = (ctypes.c_void_p * self.n_layers)(*[t.data_ptr() for t in a_train])
        rc = self._lib.egeria_refresh_eval(self._wtab, len(self.weights), self.qws.data_ptr(), self.qws.numel(),
                                           ctypes.byref(self.desc), ctypes.byref(self.qw), x.data_ptr(), eg._dt(x),
                                           ptrs, eg._dt(a_train[0]), self.p_out.data_ptr(), self.ws.data_ptr(),
                                           self.ws.numel(), eg._stream())
        eg._check(rc, "egeria_refresh_eval")
        return self.p_out

    def step_two_calls(self, x: torch.Tensor, a_train: Sequence[torch.Tensor]) -> torch.Tensor:
        self.quantize_weights()
        return self.evaluate(x, a_train)
