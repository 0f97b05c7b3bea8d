"""Host-side checks of the C-ABI that need no GPU: the shared library loads,
exports every function include/egeria.h declares, sizes workspaces sanely and
rejects bad arguments before anything would be launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def eg():
    from paper_2201_06227_amd import _build, binding
    if _build.is_stale():
        _build.build_library()
    binding.lib()
    return binding


def declared_functions():
    """Every function declared by the headers under include/ (the method's interface in egeria.h, the
    benchmark instrumentation in egeria_profile.h)."""
    names = set()
    for h in sorted(os.listdir(os.path.join(ROOT, "include"))):
        if not h.endswith(".h"):
            continue
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(egeria_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_method_header_declares_no_instrumentation():
    text = open(os.path.join(ROOT, "include", "egeria.h")).read()
    assert "egeria_profile_" not in text


def test_library_exports_every_declared_symbol(eg):
    names = declared_functions()
    assert len(names) >= 13
    L = ctypes.CDLL(eg.library_path())
    for n in names:
        assert hasattr(L, n), n
    assert sorted(eg.EXPORTS) == names


def test_status_strings_and_padding(eg):
    assert eg.status_string(eg.OK) == "ok"
    assert len({eg.status_string(c) for c in range(6)}) == 6
    assert [eg.padded(k) for k in (0, 1, 16, 17, 144, 3072)] == [0, 16, 16, 32, 144, 3072]


def test_workspace_sizes(eg):
    d = eg.make_desc(eg.FC_RELU, dict(batch=32, c_in=512, c_out=512))
    assert eg.workspace_bytes(d) >= 32 * 512 + 32 * 512 * 4
    bad = eg.make_desc(eg.FC_RELU, dict(batch=0, c_in=512, c_out=512))
    assert eg.workspace_bytes(bad) == 0
    bad = eg.make_desc(eg.BOTTLENECK, dict(batch=2, c_in=32, c_mid=8, c_out=16, height=4, width=4, has_residual=1))
    assert eg.workspace_bytes(bad) == 0          # the skip connection needs c_out == c_in
    stack = eg.make_desc(eg.BERT_STACK, dict(batch=64, seq=256, hidden=768, heads=12, ffn=3072, n_layers=12,
                                             ln_eps=1e-12))
    one = eg.make_desc(eg.BERT_LAYER, dict(batch=64, seq=256, hidden=768, heads=12, ffn=3072, n_layers=1,
                                           ln_eps=1e-12))
    assert eg.workspace_bytes(stack) > eg.workspace_bytes(one) > 64 * 256 * 3072 * 4
    assert eg.plasticity_workspace_bytes(128, 16384) >= 2 * 128 * 128 * 8
    assert eg.plasticity_workspace_bytes(129, 16) == 0 and eg.plasticity_workspace_bytes(0, 16) == 0
    assert eg.quantize_workspace_bytes() >= 64
    # reference precisions: float operands are 2 / 4 bytes, so the operand buffers grow; BERT kinds have none
    conv = dict(batch=8, c_in=64, c_mid=32, c_out=64, height=14, width=14, has_residual=1)
    sizes = [eg.workspace_bytes(eg.make_desc(eg.BOTTLENECK, dict(conv, ref_precision=p)))
             for p in (eg.REF_INT8, eg.REF_F16, eg.REF_F32)]
    assert 0 < sizes[0] < sizes[1] < sizes[2]
    assert eg.workspace_bytes(eg.make_desc(eg.BOTTLENECK, dict(conv, ref_precision=3))) == 0
    assert eg.workspace_bytes(eg.make_desc(eg.BOTTLENECK, dict(conv, ref_precision=-1))) == 0


def test_bad_arguments_are_rejected_on_the_host(eg):
    L = eg.lib()
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    assert L.egeria_quantize(null, eg.F32, 16, null, fake, fake, fake, 4096, null) == eg.ERR_INVALID_ARG
    assert L.egeria_quantize(fake, eg.F32, -1, null, fake, fake, fake, 4096, null) == eg.ERR_INVALID_ARG
    assert L.egeria_quantize(odd, eg.F32, 16, null, fake, fake, fake, 4096, null) == eg.ERR_INVALID_ARG
    assert L.egeria_quantize(fake, 7, 16, null, fake, fake, fake, 4096, null) == eg.ERR_INVALID_ARG
    assert L.egeria_quantize(fake, eg.F32, 16, null, fake, fake, fake, 8, null) == eg.ERR_WORKSPACE_TOO_SMALL
    assert L.egeria_plasticity(fake, eg.F32, fake, eg.F32, 0, 10, fake, fake, 1 << 20, null) == eg.ERR_INVALID_ARG
    assert L.egeria_plasticity(fake, eg.F32, fake, eg.F32, 129, 10, fake, fake, 1 << 20, null) == eg.ERR_UNSUPPORTED
    assert L.egeria_plasticity(fake, eg.F32, fake, eg.F32, 8, 10, fake, fake, 16, null) == eg.ERR_WORKSPACE_TOO_SMALL
    assert L.egeria_plasticity(fake, eg.F32, null, eg.F32, 8, 10, fake, fake, 1 << 20, null) == eg.ERR_INVALID_ARG
    d = eg.make_desc(eg.FC_RELU, dict(batch=4, c_in=8, c_out=8))
    qw = eg.QWeights()
    qw.n_linear = 2                        # an FC module has exactly one linear layer
    arr = (eg.QLinear * 2)()
    qw.linear = arr
    assert L.egeria_ref_forward(ctypes.byref(d), ctypes.byref(qw), fake, eg.F32, fake, None, fake, 1 << 20,
                                null) == eg.ERR_INVALID_ARG
    qw.n_linear = 1
    assert L.egeria_ref_forward(ctypes.byref(d), ctypes.byref(qw), fake, eg.F32, fake, None, fake, 1 << 20,
                                null) == eg.ERR_INVALID_ARG      # null weight pointers
    arr[0].w_q, arr[0].scale = 0x2000, 0x3000
    assert L.egeria_ref_forward(ctypes.byref(d), ctypes.byref(qw), fake, eg.F32, fake, None, fake, 16,
                                null) == eg.ERR_WORKSPACE_TOO_SMALL
    big = eg.make_desc(eg.BERT_LAYER, dict(batch=2, seq=8, hidden=256, heads=2, ffn=64, n_layers=1))
    qw4 = eg.QWeights()
    arr4 = (eg.QLinear * 4)()
    for i in range(4):
        arr4[i].w_q, arr4[i].scale = 0x2000, 0x3000
    qw4.n_linear, qw4.linear = 4, arr4
    assert L.egeria_ref_forward(ctypes.byref(big), ctypes.byref(qw4), fake, eg.F32, fake, None, fake, 1 << 30,
                                null) == eg.ERR_UNSUPPORTED      # head dimension 128 > 64


def test_refresh_eval_rejects_what_either_call_would(eg):
    """egeria_refresh_eval validates the arguments of both halves on the host before anything is enqueued."""
    L = eg.lib()
    null = ctypes.c_void_p(0)
    fake = ctypes.c_void_p(0x1000)
    d = eg.make_desc(eg.FC_RELU, dict(batch=4, c_in=8, c_out=8))
    qw = eg.QWeights()
    arr = (eg.QLinear * 1)()
    arr[0].w_q, arr[0].scale = 0x2000, 0x3000
    qw.n_linear, qw.linear = 1, arr
    ptrs = (ctypes.c_void_p * 1)(0x4000)
    wtab = (eg.Weight * 1)()
    big = 1 << 30

    def call(w=wtab, n_w=1, ws_w=fake, ws_w_bytes=big, desc=d, x=fake, a_t=ptrs, p_out=fake, ws=fake, ws_bytes=big):
        return L.egeria_refresh_eval(w, n_w, ws_w, ws_w_bytes, ctypes.byref(desc), ctypes.byref(qw), x, eg.F32, a_t,
                                     eg.F32, p_out, ws, ws_bytes, null)

    assert call(x=null) == eg.ERR_INVALID_ARG                      # the evaluation's arguments
    assert call(p_out=null) == eg.ERR_INVALID_ARG
    assert call(ws_bytes=16) == eg.ERR_WORKSPACE_TOO_SMALL
    assert call(a_t=(ctypes.c_void_p * 1)(0)) == eg.ERR_INVALID_ARG
    assert call(n_w=-1) == eg.ERR_INVALID_ARG                      # the snapshot's arguments
    assert call(ws_w=null) == eg.ERR_INVALID_ARG
    assert call(ws_w_bytes=8) == eg.ERR_WORKSPACE_TOO_SMALL
    wtab[0].out, wtab[0].in_, wtab[0].kh, wtab[0].kw = 8, 8, 0, 1  # a kernel of height 0
    assert call() == eg.ERR_INVALID_ARG
    too_big = eg.make_desc(eg.FC_RELU, dict(batch=200, c_in=8, c_out=8))
    assert call(desc=too_big) == eg.ERR_UNSUPPORTED                # the metric takes at most 128 samples


def test_profile_pause_is_harmless_when_nothing_is_armed(eg):
    L = eg.lib()
    assert L.egeria_profile_pause(1) == eg.OK and L.egeria_profile_pause(0) == eg.OK
    n = ctypes.c_int32(-1)
    assert L.egeria_profile_end(None, 0, ctypes.byref(n)) == eg.OK and n.value == 0


def test_missing_library_fails_loudly(eg, monkeypatch, tmp_path):
    from paper_2201_06227_amd import _build
    monkeypatch.setattr(eg, "_lib", None)
    monkeypatch.setattr(_build, "LIB", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError):
        eg.lib()


def test_gelu_table_is_what_its_generator_writes():
    """The table of cubic GELU pieces compiled into the fused quantiser is the committed generator's output,
    and its measured error against the fp64 function stays far inside the bound the kernel certifies with
    (values outside the bound's interval would only cost a fall-back to fp64, never a wrong code, as long as
    the bound holds - which is what the generator measures on 64 points per piece)."""
    import importlib.util
    path = os.path.join(ROOT, "paper_2201_06227_amd", "csrc", "gen_gelu_table.py")
    spec = importlib.util.spec_from_file_location("gen_gelu_table", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    text, worst_abs, worst_rel = mod.table_text()
    assert text == open(os.path.join(ROOT, "paper_2201_06227_amd", "csrc", "gelu_table.inc")).read()
    assert worst_abs < 5e-8 and worst_rel < 2e-7
