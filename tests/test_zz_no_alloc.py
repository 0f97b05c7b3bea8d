"""The entry point that allocates nothing (egeria_plasticity_noalloc) against egeria_plasticity,
through the C-ABI: two calls in a row on one GPU, the second with a smaller input, so that the
library's own scratch array still holds the first call's partials when the second one runs."""
import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu

P_RTOL = 1e-4


def test_noalloc_plasticity_matches_workspace_entry_point():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2201_06227_amd import binding as eg
    from oracle import oracle as orc
    eg.lib()
    dev = "cuda:0"
    p = torch.zeros(1, dtype=torch.float32, device=dev)
    # a large input first (64 x 196608: every split-K chunk and both Gram blocks in use), then a
    # smaller and ragged one, then bf16 training activations, then the large one again
    cases = [(64, 196608, 0.01, False), (24, 5000, 0.05, False), (128, 4099, 0.1, False), (32, 98304, 0.02, True),
             (64, 196608, 0.01, False)]
    for n, (b, D, rel, bf16) in enumerate(cases):
        a_t, a_r = si.noisy_pair(b, D, rel=rel, seed=1234 + b)
        t = torch.from_numpy(a_t).to(dev)
        if bf16:
            t = t.to(torch.bfloat16)
            a_t = t.float().cpu().numpy()
        r = torch.from_numpy(a_r).to(dev)
        want_gpu = eg.plasticity(t, r).item()
        p.fill_(-1.0)
        torch.cuda.synchronize()
        alloc_before = torch.cuda.memory_allocated()
        eg.plasticity_noalloc(t, r, p)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == alloc_before
        got = p.item()
        assert got == want_gpu, (n, b, D, got, want_gpu)                 # same kernels: same bits
        want = orc.sp_loss(a_t, a_r)
        assert abs(got - want) <= P_RTOL * abs(want) + 1e-12 * 4.0 / b, (n, got, want)


def test_noalloc_plasticity_rejects_what_it_cannot_hold():
    import ctypes
    from paper_2201_06227_amd import binding as eg
    L = eg.lib()
    x = torch.zeros(256 * 64, dtype=torch.float32, device="cuda:0")
    p = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.egeria_plasticity_noalloc(vp(x), eg.F32, vp(x), eg.F32, 129, 64, vp(p), None) == eg.ERR_UNSUPPORTED
    assert L.egeria_plasticity_noalloc(None, eg.F32, vp(x), eg.F32, 8, 64, vp(p), None) == eg.ERR_INVALID_ARG
    assert L.egeria_plasticity_noalloc(vp(x), eg.F32, vp(x), eg.F32, 8, 0, vp(p), None) == eg.ERR_INVALID_ARG
    assert L.egeria_plasticity_noalloc(vp(x), 7, vp(x), eg.F32, 8, 64, vp(p), None) == eg.ERR_INVALID_ARG
