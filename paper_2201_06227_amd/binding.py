"""ctypes binding of libegeria.so: same names as include/egeria.h, argument
marshalling only.  Tensors are torch CUDA tensors (device memory + streams are
all PyTorch is used for); every step of the path runs in the library's kernels.

There is no fallback: if the shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import _build

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_NONFINITE, ERR_HIP = range(6)
F32, BF16 = 0, 1
REF_INT8, REF_F16, REF_F32 = 0, 1, 2
ACT_SYMMETRIC, ACT_AFFINE = 0, 1
FC_RELU, BASIC_BLOCK, BOTTLENECK, BERT_LAYER, BERT_STACK = range(5)

_vp = ctypes.c_void_p
_i64 = ctypes.c_int64
_i32 = ctypes.c_int32
_sz = ctypes.c_size_t


class BlockDesc(ctypes.Structure):
    _fields_ = [("kind", _i32), ("batch", _i32), ("c_in", _i32), ("c_mid", _i32), ("c_out", _i32),
                ("height", _i32), ("width", _i32), ("has_residual", _i32), ("seq", _i32),
                ("hidden", _i32), ("heads", _i32), ("ffn", _i32), ("n_layers", _i32),
                ("ln_eps", ctypes.c_float), ("ref_precision", _i32), ("act_scheme", _i32)]


class QLinear(ctypes.Structure):
    _fields_ = [("w_q", _vp), ("scale", _vp), ("bias", _vp), ("per_channel", _i32), ("colsum", _vp)]


class Norm(ctypes.Structure):
    _fields_ = [("gamma", _vp), ("beta", _vp)]


class QWeights(ctypes.Structure):
    _fields_ = [("n_linear", _i32), ("linear", ctypes.POINTER(QLinear)), ("n_norm", _i32),
                ("norm", ctypes.POINTER(Norm)), ("act_scale", _vp)]


class Tap(ctypes.Structure):
    _fields_ = [("x_q", _vp), ("x_scale", _vp), ("acc", _vp), ("y", _vp), ("x_zp", _vp)]


class Taps(ctypes.Structure):
    _fields_ = [("n", _i32), ("tap", ctypes.POINTER(Tap))]


class Weight(ctypes.Structure):
    _fields_ = [("w", _vp), ("dtype", _i32), ("out", _i32), ("in_", _i32), ("kh", _i32), ("kw", _i32),
                ("w_q", _vp), ("scale", _vp), ("per_channel", _i32), ("precision", _i32), ("colsum", _vp)]


FREEZE_MAX_W = 256
FREEZE_NONE, FREEZE_FREEZE, FREEZE_UNFREEZE_ALL = range(3)


class FreezeState(ctypes.Structure):
    _fields_ = [("n_modules", _i32), ("front", _i32), ("W", _i32), ("stale", _i32), ("lr_annealing", _i32),
                ("has_lr_ref", _i32), ("n_first_slopes", _i32), ("has_T", _i32), ("n_raw", _i64), ("n_smooth", _i64),
                ("T_user", ctypes.c_double), ("T", ctypes.c_double), ("max_first_slope", ctypes.c_double),
                ("lr_ref", ctypes.c_double), ("raw", ctypes.c_double * FREEZE_MAX_W),
                ("smooth", ctypes.c_double * FREEZE_MAX_W)]


class FreezeDecision(ctypes.Structure):
    _fields_ = [("action", _i32), ("front", _i32), ("stale", _i32), ("W", _i32), ("smoothed", ctypes.c_double),
                ("slope", ctypes.c_double), ("T", ctypes.c_double)]


class CacheDesc(ctypes.Structure):
    _fields_ = [("window", _i32), ("batch", _i32), ("row_elems", _i64), ("dtype", _i32)]


class EgeriaError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


_lib = None

EXPORTS = [
    "egeria_padded", "egeria_quantize", "egeria_quantize_rows", "egeria_quantize_nchw",
    "egeria_dequantize", "egeria_quantize_workspace_bytes", "egeria_ref_forward",
    "egeria_plasticity", "egeria_plasticity_workspace_bytes", "egeria_plasticity_eval",
    "egeria_workspace_bytes", "egeria_check", "egeria_status_string", "egeria_profile_begin",
    "egeria_profile_end", "egeria_quantize_weights", "egeria_quantize_weights_workspace_bytes",
    "egeria_freeze_init", "egeria_freeze_observe",
    "egeria_cache_bytes", "egeria_cache_init", "egeria_cache_put", "egeria_cache_get", "egeria_profile_pause",
    "egeria_refresh_eval", "egeria_plasticity_noalloc", "egeria_profile_attention",
    "egeria_quantize_affine", "egeria_quantize_affine_workspace_bytes", "egeria_microbench",
    "egeria_profile_attention_threshold",
]

(KERNEL_NONE, KERNEL_ABSMAX, KERNEL_QUANTIZE, KERNEL_GEMM, KERNEL_GRAM, KERNEL_ATTENTION, KERNEL_LAYERNORM,
 KERNEL_CACHE_COPY) = range(8)


def library_path() -> str:
    return _build.LIB


def lib():
    """The loaded shared library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first "
                           "(python -c 'import __graft_entry__ as g; g.build()')")
    L = ctypes.CDLL(path)
    L.egeria_padded.restype = _i64
    L.egeria_padded.argtypes = [_i64]
    L.egeria_quantize.restype = ctypes.c_int
    L.egeria_quantize.argtypes = [_vp, ctypes.c_int, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    L.egeria_quantize_rows.restype = ctypes.c_int
    L.egeria_quantize_rows.argtypes = [_vp, ctypes.c_int, _i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    L.egeria_quantize_nchw.restype = ctypes.c_int
    L.egeria_quantize_nchw.argtypes = [_vp, ctypes.c_int, _i64, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    L.egeria_quantize_weights.restype = ctypes.c_int
    L.egeria_quantize_weights.argtypes = [ctypes.POINTER(Weight), _i32, _vp, _sz, _vp]
    L.egeria_quantize_weights_workspace_bytes.restype = _sz
    L.egeria_quantize_weights_workspace_bytes.argtypes = [_i32]
    L.egeria_dequantize.restype = ctypes.c_int
    L.egeria_dequantize.argtypes = [_vp, _vp, _i64, _vp, _vp]
    L.egeria_quantize_workspace_bytes.restype = _sz
    L.egeria_quantize_workspace_bytes.argtypes = []
    L.egeria_quantize_affine.restype = ctypes.c_int
    L.egeria_quantize_affine.argtypes = [_vp, ctypes.c_int, _i64, _vp, _vp, _vp, _vp, _sz, _vp]
    L.egeria_quantize_affine_workspace_bytes.restype = _sz
    L.egeria_quantize_affine_workspace_bytes.argtypes = []
    L.egeria_ref_forward.restype = ctypes.c_int
    L.egeria_ref_forward.argtypes = [ctypes.POINTER(BlockDesc), ctypes.POINTER(QWeights), _vp, ctypes.c_int,
                                     _vp, ctypes.POINTER(Taps), _vp, _sz, _vp]
    L.egeria_plasticity.restype = ctypes.c_int
    L.egeria_plasticity.argtypes = [_vp, ctypes.c_int, _vp, ctypes.c_int, _i32, _i64, _vp, _vp, _sz, _vp]
    L.egeria_plasticity_noalloc.restype = ctypes.c_int
    L.egeria_plasticity_noalloc.argtypes = [_vp, ctypes.c_int, _vp, ctypes.c_int, _i32, _i64, _vp, _vp]
    L.egeria_plasticity_workspace_bytes.restype = _sz
    L.egeria_plasticity_workspace_bytes.argtypes = [_i32, _i64]
    L.egeria_plasticity_eval.restype = ctypes.c_int
    L.egeria_plasticity_eval.argtypes = [ctypes.POINTER(BlockDesc), ctypes.POINTER(QWeights), _vp, ctypes.c_int,
                                         ctypes.POINTER(_vp), ctypes.c_int, _vp, _vp, _sz, _vp]
    L.egeria_refresh_eval.restype = ctypes.c_int
    L.egeria_refresh_eval.argtypes = [ctypes.POINTER(Weight), _i32, _vp, _sz, ctypes.POINTER(BlockDesc),
                                      ctypes.POINTER(QWeights), _vp, ctypes.c_int, ctypes.POINTER(_vp), ctypes.c_int,
                                      _vp, _vp, _sz, _vp]
    L.egeria_workspace_bytes.restype = _sz
    L.egeria_workspace_bytes.argtypes = [ctypes.POINTER(BlockDesc)]
    L.egeria_check.restype = ctypes.c_int
    L.egeria_check.argtypes = [_vp, _vp]
    L.egeria_profile_begin.restype = ctypes.c_int
    L.egeria_profile_begin.argtypes = [_i32, _i32]
    L.egeria_profile_pause.restype = ctypes.c_int
    L.egeria_profile_pause.argtypes = [_i32]
    L.egeria_profile_end.restype = ctypes.c_int
    L.egeria_profile_end.argtypes = [ctypes.POINTER(ctypes.c_float), _i32, ctypes.POINTER(_i32)]
    L.egeria_profile_attention.restype = ctypes.c_int
    L.egeria_profile_attention.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp]
    L.egeria_profile_attention_threshold.restype = ctypes.c_double
    L.egeria_profile_attention_threshold.argtypes = [ctypes.c_double]
    L.egeria_microbench.restype = ctypes.c_int
    L.egeria_microbench.argtypes = [_i32, _i32, _vp, _sz, ctypes.POINTER(ctypes.c_float),
                                    ctypes.POINTER(ctypes.c_double), _vp]
    L.egeria_freeze_init.restype = ctypes.c_int
    L.egeria_freeze_init.argtypes = [ctypes.POINTER(FreezeState), _i32, _i32, ctypes.c_double, _i32]
    L.egeria_freeze_observe.restype = ctypes.c_int
    L.egeria_freeze_observe.argtypes = [ctypes.POINTER(FreezeState), ctypes.c_double, ctypes.c_double,
                                        ctypes.POINTER(FreezeDecision)]
    L.egeria_cache_bytes.restype = _sz
    L.egeria_cache_bytes.argtypes = [ctypes.POINTER(CacheDesc)]
    L.egeria_cache_init.restype = ctypes.c_int
    L.egeria_cache_init.argtypes = [ctypes.POINTER(CacheDesc), _vp, _sz, _vp]
    L.egeria_cache_put.restype = ctypes.c_int
    L.egeria_cache_put.argtypes = [ctypes.POINTER(CacheDesc), _vp, _sz, _vp, _i32, _vp, _vp]
    L.egeria_cache_get.restype = ctypes.c_int
    L.egeria_cache_get.argtypes = [ctypes.POINTER(CacheDesc), _vp, _sz, _vp, _i64, _vp, _vp, _vp]
    L.egeria_status_string.restype = ctypes.c_char_p
    L.egeria_status_string.argtypes = [ctypes.c_int]
    _lib = L
    return L


def status_string(code: int) -> str:
    return lib().egeria_status_string(int(code)).decode()


def _check(code: int, where: str):
    if code != OK:
        raise EgeriaError(code, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t: torch.Tensor) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t


def padded(k: int) -> int:
    return int(lib().egeria_padded(int(k)))


def workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ---- quantise -----------------------------------------------------------------------------

def quantize_workspace_bytes() -> int:
    return int(lib().egeria_quantize_workspace_bytes())


def quantize(x: torch.Tensor, fixed_scale: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """egeria_quantize: int8 codes (same shape as x) and the 1-element fp32 scale."""
    x = _dev(x)
    q = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    scale = torch.empty(1, dtype=torch.float32, device=x.device)
    ws = workspace(quantize_workspace_bytes(), x.device) if ws is None else ws
    rc = lib().egeria_quantize(_ptr(x), _dt(x), x.numel(), _ptr(fixed_scale), _ptr(q), _ptr(scale), _ptr(ws),
                               ws.numel(), _stream())
    _check(rc, "egeria_quantize")
    return q, scale


def quantize_rows(x: torch.Tensor, fixed_scale: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """egeria_quantize_rows: [rows, cols] -> int8 [rows, padded(cols)] and scale."""
    x = _dev(x)
    rows, cols = x.shape
    q = torch.empty((rows, padded(cols)), dtype=torch.int8, device=x.device)
    scale = torch.empty(1, dtype=torch.float32, device=x.device)
    ws = workspace(quantize_workspace_bytes(), x.device) if ws is None else ws
    rc = lib().egeria_quantize_rows(_ptr(x), _dt(x), rows, cols, _ptr(fixed_scale), _ptr(q), _ptr(scale),
                                    _ptr(ws), ws.numel(), _stream())
    _check(rc, "egeria_quantize_rows")
    return q, scale


def quantize_nchw(x: torch.Tensor, fixed_scale: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None):
    """egeria_quantize_nchw: [n, c, h, w] -> int8 [n, h, w, padded(c)] and scale."""
    x = _dev(x)
    n, c, h, w = x.shape
    q = torch.empty((n, h, w, padded(c)), dtype=torch.int8, device=x.device)
    scale = torch.empty(1, dtype=torch.float32, device=x.device)
    ws = workspace(quantize_workspace_bytes(), x.device) if ws is None else ws
    rc = lib().egeria_quantize_nchw(_ptr(x), _dt(x), n, c, h, w, _ptr(fixed_scale), _ptr(q), _ptr(scale),
                                    _ptr(ws), ws.numel(), _stream())
    _check(rc, "egeria_quantize_nchw")
    return q, scale


def quantize_affine(x: torch.Tensor):
    """egeria_quantize_affine: uint8 codes (same shape as x), 1-element fp32 scale, 1-element int32 zero point."""
    x = _dev(x)
    n = x.numel()
    q = torch.empty(padded(n), dtype=torch.uint8, device=x.device)
    scale = torch.empty(1, dtype=torch.float32, device=x.device)
    zp = torch.empty(1, dtype=torch.int32, device=x.device)
    ws = workspace(int(lib().egeria_quantize_affine_workspace_bytes()), x.device)
    rc = lib().egeria_quantize_affine(_ptr(x), _dt(x), n, _ptr(q), _ptr(scale), _ptr(zp), _ptr(ws), ws.numel(), _stream())
    _check(rc, "egeria_quantize_affine")
    return q[:n].reshape(x.shape), scale, zp


def colsum_like(w: torch.Tensor) -> torch.Tensor:
    """Buffer for egeria_weight.colsum of a weight tensor: int32 [classes, out]."""
    return torch.empty((16 if w.dim() == 4 and w.shape[2] == 3 else 1, w.shape[0]), dtype=torch.int32, device=w.device)


def weight_table(weights: Sequence[torch.Tensor], w_q: Sequence[torch.Tensor], scales: Sequence[torch.Tensor],
                 per_channel: bool = False, colsums: Optional[Sequence[torch.Tensor]] = None):
    """HOST array of egeria_weight descriptors for egeria_quantize_weights."""
    tab = (Weight * len(weights))()
    for i, (t, w, q, s) in enumerate(zip(tab, weights, w_q, scales)):
        t.colsum = None if colsums is None else colsums[i].data_ptr()
        t.per_channel = 1 if per_channel else 0
        _dev(w)
        if w.dim() == 4:
            t.out, t.in_, t.kh, t.kw = w.shape
        else:
            t.out, t.in_ = w.shape
            t.kh = t.kw = 1
        t.w, t.dtype, t.w_q, t.scale = w.data_ptr(), _dt(w), q.data_ptr(), s.data_ptr()
    return tab


def quantize_weights_workspace_bytes(n: int) -> int:
    return int(lib().egeria_quantize_weights_workspace_bytes(int(n)))


def quantize_weights(weights: Sequence[torch.Tensor], ws: Optional[torch.Tensor] = None, per_channel: bool = False,
                     colsums: Optional[Sequence[torch.Tensor]] = None):
    """egeria_quantize_weights: every tensor of a snapshot in one call.  Returns
    the int8 tensors ([out, padded(in)] or [out, kh, kw, padded(in)]) and scales
    (1 value per tensor, or [out] values with per_channel); colsums (see colsum_like)
    receive the sums of the codes that affine activation codes need."""
    dev = weights[0].device if weights else "cuda"
    w_q, scales = [], []
    for w in weights:
        shape = (w.shape[0], w.shape[2], w.shape[3], padded(w.shape[1])) if w.dim() == 4 else \
            (w.shape[0], padded(w.shape[1]))
        w_q.append(torch.empty(shape, dtype=torch.int8, device=dev))
        scales.append(torch.empty(w.shape[0] if per_channel else 1, dtype=torch.float32, device=dev))
    ws = workspace(quantize_weights_workspace_bytes(len(weights)), dev) if ws is None else ws
    tab = weight_table(weights, w_q, scales, per_channel, colsums)
    rc = lib().egeria_quantize_weights(tab, len(weights), _ptr(ws), ws.numel(), _stream())
    _check(rc, "egeria_quantize_weights")
    return w_q, scales


def dequantize(q: torch.Tensor, scale: torch.Tensor) -> torch.Tensor:
    q = _dev(q)
    x = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    _check(lib().egeria_dequantize(_ptr(q), _ptr(scale), q.numel(), _ptr(x), _stream()), "egeria_dequantize")
    return x


# ---- reference model ------------------------------------------------------------------------

def make_desc(kind: int, dims: dict) -> BlockDesc:
    d = BlockDesc()
    d.kind = kind
    d.batch = dims["batch"]
    for k in ("c_in", "c_mid", "c_out", "height", "width", "has_residual", "seq", "hidden", "heads", "ffn"):
        setattr(d, k, int(dims.get(k, 0)))
    d.n_layers = int(dims.get("n_layers", 1))
    d.ln_eps = float(dims.get("ln_eps", 0.0))
    d.ref_precision = int(dims.get("ref_precision", REF_INT8))
    d.act_scheme = int(dims.get("act_scheme", ACT_SYMMETRIC))
    return d


@dataclass
class ReferenceModel:
    """Device-resident int8 reference model of one layer module: the marshalled
    egeria_qweights plus the tensors that keep its pointers alive."""
    desc: BlockDesc
    qweights: QWeights
    w_q: List[torch.Tensor]
    scales: List[torch.Tensor]
    biases: List[Optional[torch.Tensor]]
    _keep: tuple = ()


def make_reference(kind: int, dims: dict, weights: Sequence[torch.Tensor],
                   biases: Sequence[Optional[torch.Tensor]],
                   act_scales: Optional[torch.Tensor] = None, per_channel: bool = False,
                   act_scheme: int = ACT_SYMMETRIC) -> ReferenceModel:
    """Reference-model generation: quantise every weight tensor of the snapshot
    with the library (egeria_quantize_rows for [out, in], egeria_quantize_nchw for
    [out, in, kh, kw]) and marshal the result.  act_scheme = ACT_AFFINE: affine uint8
    activation codes (the weight-code sums they need are made along with the codes)."""
    w_q, scales = [], []
    colsums = [colsum_like(w) for w in weights] if act_scheme == ACT_AFFINE else None
    if per_channel or colsums is not None:
        w_q, scales = quantize_weights(list(weights), per_channel=per_channel, colsums=colsums)
    else:
        ws = workspace(quantize_workspace_bytes(), weights[0].device)
        for w in weights:
            q, s = quantize_nchw(w, ws=ws) if w.dim() == 4 else quantize_rows(w, ws=ws)
            w_q.append(q)
            scales.append(s)
    arr = (QLinear * len(weights))()
    for i in range(len(weights)):
        arr[i].per_channel = 1 if per_channel else 0
        arr[i].w_q = w_q[i].data_ptr()
        arr[i].scale = scales[i].data_ptr()
        arr[i].bias = 0 if biases[i] is None else biases[i].data_ptr()
        arr[i].colsum = None if colsums is None else colsums[i].data_ptr()
    qw = QWeights()
    qw.n_linear = len(weights)
    qw.linear = arr
    qw.n_norm = 0
    qw.norm = None
    qw.act_scale = None if act_scales is None else _dev(act_scales).data_ptr()   # fp32 [n_linear], static scales
    return ReferenceModel(make_desc(kind, dict(dims, act_scheme=act_scheme)), qw, w_q, scales, list(biases),
                          (arr, act_scales, colsums))


def op_row_bytes(c: int, precision: int) -> int:
    """Bytes of one operand row of c values at a reference precision (padded to 16)."""
    return padded(c * {REF_INT8: 1, REF_F16: 2, REF_F32: 4}[precision])


def make_float_reference(kind: int, dims: dict, weights: Sequence[torch.Tensor],
                         biases: Sequence[Optional[torch.Tensor]], precision: int) -> ReferenceModel:
    """Reference model at float16 / float32 precision: every weight tensor cast by
    egeria_quantize_weights (precision field) into the GEMM's layout."""
    dev = weights[0].device
    w_q = []
    for w in weights:
        taps_ = w.shape[2] * w.shape[3] if w.dim() == 4 else 1
        w_q.append(torch.empty((w.shape[0], taps_ * op_row_bytes(w.shape[1], precision)), dtype=torch.uint8, device=dev))
    tab = weight_table(weights, w_q, [w_q[0]] * len(weights))
    for t in tab:
        t.scale, t.precision = None, precision
    ws = workspace(quantize_weights_workspace_bytes(len(weights)), dev)
    _check(lib().egeria_quantize_weights(tab, len(weights), _ptr(ws), ws.numel(), _stream()), "egeria_quantize_weights")
    arr = (QLinear * len(weights))()
    for i in range(len(weights)):
        arr[i].w_q = w_q[i].data_ptr()
        arr[i].scale = None
        arr[i].bias = 0 if biases[i] is None else biases[i].data_ptr()
    qw = QWeights()
    qw.n_linear, qw.linear, qw.n_norm, qw.norm, qw.act_scale = len(weights), arr, 0, None, None
    return ReferenceModel(make_desc(kind, dict(dims, ref_precision=precision)), qw, w_q, [], list(biases), (arr,))


def workspace_bytes(desc: BlockDesc) -> int:
    return int(lib().egeria_workspace_bytes(ctypes.byref(desc)))


def plasticity_workspace_bytes(b: int, D: int) -> int:
    return int(lib().egeria_plasticity_workspace_bytes(int(b), int(D)))


def make_taps(ref: ReferenceModel, shapes: Sequence[dict], device="cuda"):
    """Allocate observation buffers.  shapes[i] = dict(M=, kp=, N=)."""
    arr = (Tap * len(shapes))()
    bufs = []
    for i, s in enumerate(shapes):
        xq = torch.zeros((s["M"], s["kp"]), dtype=torch.int8, device=device)
        sc = torch.zeros(1, dtype=torch.float32, device=device)
        acc = torch.zeros((s["M"], s["N"]), dtype=torch.int32, device=device)
        y = torch.zeros((s["M"], s["N"]), dtype=torch.float32, device=device)
        zp = torch.zeros(1, dtype=torch.int32, device=device)
        arr[i].x_q, arr[i].x_scale, arr[i].acc, arr[i].y = xq.data_ptr(), sc.data_ptr(), acc.data_ptr(), y.data_ptr()
        arr[i].x_zp = zp.data_ptr()
        bufs.append(dict(x_q=xq, x_scale=sc, acc=acc, y=y, x_zp=zp))
    taps = Taps()
    taps.n = len(shapes)
    taps.tap = arr
    return taps, bufs, arr


def ref_forward(ref: ReferenceModel, x: torch.Tensor, a_ref: torch.Tensor, ws: torch.Tensor,
                taps: Optional[Taps] = None):
    """egeria_ref_forward: enqueue the reference forward; a_ref is written in place."""
    x, a_ref = _dev(x), _dev(a_ref)
    rc = lib().egeria_ref_forward(ctypes.byref(ref.desc), ctypes.byref(ref.qweights), _ptr(x), _dt(x),
                                  _ptr(a_ref), ctypes.byref(taps) if taps is not None else None, _ptr(ws),
                                  ws.numel(), _stream())
    _check(rc, "egeria_ref_forward")
    return a_ref


def plasticity(a_train: torch.Tensor, a_ref: torch.Tensor, p_out: Optional[torch.Tensor] = None,
               ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """egeria_plasticity on two [b, D] activations; returns the 1-element fp32 tensor."""
    a_train, a_ref = _dev(a_train), _dev(a_ref)
    b = a_train.shape[0]
    D = a_train.numel() // b if b else 0
    if a_ref.shape[0] != b or a_ref.numel() != a_train.numel():
        raise ValueError("a_train and a_ref must both be [b, D]")
    if p_out is None:
        p_out = torch.empty(1, dtype=torch.float32, device=a_train.device)
    if ws is None:
        ws = workspace(plasticity_workspace_bytes(b, D), a_train.device)
    rc = lib().egeria_plasticity(_ptr(a_train), _dt(a_train), _ptr(a_ref), _dt(a_ref), b, D, _ptr(p_out),
                                 _ptr(ws), ws.numel(), _stream())
    _check(rc, "egeria_plasticity")
    return p_out


def plasticity_noalloc(a_train: torch.Tensor, a_ref: torch.Tensor, p_out: torch.Tensor) -> torch.Tensor:
    """egeria_plasticity_noalloc: the score into the caller's p_out; nothing is allocated here either."""
    a_train, a_ref = _dev(a_train), _dev(a_ref)
    b = a_train.shape[0]
    D = a_train.numel() // b if b else 0
    if a_ref.shape[0] != b or a_ref.numel() != a_train.numel():
        raise ValueError("a_train and a_ref must both be [b, D]")
    rc = lib().egeria_plasticity_noalloc(_ptr(a_train), _dt(a_train), _ptr(a_ref), _dt(a_ref), b, D, _ptr(p_out),
                                         _stream())
    _check(rc, "egeria_plasticity_noalloc")
    return p_out


def plasticity_eval(ref: ReferenceModel, x: torch.Tensor, a_train: Sequence[torch.Tensor],
                    p_out: torch.Tensor, ws: torch.Tensor) -> torch.Tensor:
    """egeria_plasticity_eval: reference forward + one score per layer."""
    x = _dev(x)
    n = ref.desc.n_layers
    if len(a_train) != n:
        raise ValueError(f"{n} training activations expected")
    ptrs = (_vp * n)(*[_dev(t).data_ptr() for t in a_train])
    rc = lib().egeria_plasticity_eval(ctypes.byref(ref.desc), ctypes.byref(ref.qweights), _ptr(x), _dt(x), ptrs,
                                      _dt(a_train[0]), _ptr(p_out), _ptr(ws), ws.numel(), _stream())
    _check(rc, "egeria_plasticity_eval")
    return p_out


MICRO_KINDS = ["mfma_i32_32x32x32_i8", "mfma_f32_32x32x16_bf16", "mfma_f32_32x32x2_f32", "mfma_f32_16x16x4_f32",
               "mfma_f64_16x16x4_f64", "lds_read_b128", "lds_write_b128", "l2_to_lds_whole_lines", "l2_to_lds_half_lines",
               "hbm_copy", "bf16_dependent_chain", "bf16_chain_plus_8_valu", "bf16_chain_plus_8_valu_2_waves"]


def attention_threshold(min_flops: float = -1.0) -> float:
    """egeria_profile_attention_threshold: sets (if >= 0) and returns the previous threshold."""
    return float(lib().egeria_profile_attention_threshold(float(min_flops)))


def microbench(kind: int, iters: int, scratch: torch.Tensor):
    """egeria_microbench: (milliseconds, work done) of one micro-measurement."""
    ms, work = ctypes.c_float(0), ctypes.c_double(0)
    _check(lib().egeria_microbench(int(kind), int(iters), _ptr(scratch), scratch.numel(), ctypes.byref(ms),
                                   ctypes.byref(work), _stream()), "egeria_microbench")
    return ms.value, work.value


def check(ws: torch.Tensor) -> int:
    """egeria_check: status code (OK or ERR_NONFINITE); synchronises the stream."""
    return int(lib().egeria_check(_ptr(ws), _stream()))


class FreezeController:
    """egeria_freeze_init / egeria_freeze_observe on a state struct owned here."""

    def __init__(self, n_modules: int, W: int, T: float = 0.0, lr_annealing: bool = True):
        self.state = FreezeState()
        _check(lib().egeria_freeze_init(ctypes.byref(self.state), n_modules, W, float(T), 1 if lr_annealing else 0),
               "egeria_freeze_init")

    def observe(self, p: float, lr: float) -> FreezeDecision:
        d = FreezeDecision()
        _check(lib().egeria_freeze_observe(ctypes.byref(self.state), float(p), float(lr), ctypes.byref(d)),
               "egeria_freeze_observe")
        return d


class ActivationCache:
    """egeria_cache_*: the descriptor and the cache memory (a torch byte tensor) held together."""

    def __init__(self, window: int, batch: int, row_elems: int, dtype: torch.dtype = torch.float32,
                 device: str = "cuda:0"):
        self.desc = CacheDesc(int(window), int(batch), int(row_elems), BF16 if dtype == torch.bfloat16 else F32)
        nbytes = int(lib().egeria_cache_bytes(ctypes.byref(self.desc)))
        if nbytes == 0:
            raise EgeriaError(ERR_INVALID_ARG, "egeria_cache_bytes")
        self.mem = torch.empty(nbytes, dtype=torch.uint8, device=device)
        _check(lib().egeria_cache_init(ctypes.byref(self.desc), _ptr(self.mem), nbytes, _stream()), "egeria_cache_init")

    def put(self, ids: torch.Tensor, rows: torch.Tensor) -> None:
        n = int(ids.numel())
        _check(lib().egeria_cache_put(ctypes.byref(self.desc), _ptr(self.mem), self.mem.numel(),
                                      _ptr(_dev(ids)) if n else None, n, _ptr(_dev(rows)) if n else None, _stream()),
               "egeria_cache_put")

    def get(self, ids: torch.Tensor, out: torch.Tensor, hit: torch.Tensor) -> torch.Tensor:
        n = int(ids.numel())
        _check(lib().egeria_cache_get(ctypes.byref(self.desc), _ptr(self.mem), self.mem.numel(),
                                      _ptr(_dev(ids)) if n else None, n, _ptr(_dev(out)) if n else None,
                                      _ptr(hit) if n else None, _stream()), "egeria_cache_get")
        return hit


def profile_attention(qkv: torch.Tensor, heads: int, mode: int):
    """egeria_profile_attention: (ctx [B, S, hidden], records [n, 2] int32 view or None)."""
    qkv = _dev(qkv)
    B, S, h3 = qkv.shape
    hidden = h3 // 3
    ctx = torch.empty((B, S, hidden), dtype=torch.float32, device=qkv.device)
    rec = torch.zeros((B * heads * ((S + 63) // 64), 2), dtype=torch.int32, device=qkv.device) if mode == 1 else None
    _check(lib().egeria_profile_attention(_ptr(qkv), B, S, hidden, heads, mode, _ptr(ctx), _ptr(rec), _stream()),
           "egeria_profile_attention")
    return ctx, rec


def profile_begin(kernel_class: int, max_launches: int) -> None:
    _check(lib().egeria_profile_begin(int(kernel_class), int(max_launches)), "egeria_profile_begin")


def profile_pause(paused: bool) -> None:
    lib().egeria_profile_pause(1 if paused else 0)


def profile_end(capacity: int):
    """egeria_profile_end: list of per-launch durations in ms (waits for them)."""
    buf = (ctypes.c_float * max(capacity, 1))()
    n = _i32(0)
    _check(lib().egeria_profile_end(buf, capacity, ctypes.byref(n)), "egeria_profile_end")
    return [float(buf[i]) for i in range(min(n.value, capacity))]
