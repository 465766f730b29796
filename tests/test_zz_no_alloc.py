"""lime_request_static, the request entry point that takes no workspace and allocates nothing (its scratch is a fixed
array inside the library's device code), against lime_request on a caller's workspace: same kernels, so the link
states and the outputs must be the same bits.  Two calls in a row on the shared scratch, the second on a smaller
problem; then a softmax and an XORA request on a general-kernel shape."""

import ctypes

import numpy as np
import pytest
import torch

from paper_2510_18239_amd import binding, synth
from parity_util import DeviceWorkload

pytestmark = pytest.mark.gpu


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _both(w, xor):
    """(LP, O) of lime_request on a torch-allocated workspace and of lime_request_static, called through the C symbols."""
    g = DeviceWorkload(w)
    lib = binding.lib()
    code = binding.LIME_BF16 if w.dtype == "bf16" else binding.LIME_F32
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    s_h = 1.0 if xor else w.softmax_scale
    s_c = w.softmax_scale
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    outs = []
    for static in (False, True):
        LP = torch.full((w.B, w.m, w.d), 7.0, dtype=tdt, device="cuda")
        O = torch.full((w.B, w.C, w.d), 7.0, dtype=tdt, device="cuda")
        common = (_ptr(g.E), _ptr(g.lens), _ptr(g.L), 0, _ptr(g.Wq), _ptr(g.Wk), _ptr(g.Wv), _ptr(g.T), _ptr(g.L), _ptr(g.Wq),
                  _ptr(g.Wk), _ptr(g.Wv), _ptr(LP), _ptr(O), w.B, w.N, w.C, w.d, w.h, w.m, s_h, s_c, int(xor), code)
        if static:
            st = lib.lime_request_static(*common, stream)
        else:
            need = binding.workspace_bytes(binding.OP_REQUEST, B=w.B, N=w.N, C=w.C, d=w.d, h=w.h, m=w.m, dtype=code)
            ws = torch.empty(need, dtype=torch.uint8, device="cuda")
            st = lib.lime_request(*common, _ptr(ws), need, stream)
        assert st == 0, binding.last_error()
        torch.cuda.synchronize()
        outs.append((LP, O))
    return outs


def _sharp(idx, **kw):
    g = synth.sharp_gain(kw["d"], kw["h"], (kw["d"] // kw["h"]) ** -0.5, 2.0)
    return synth.make_workload(idx, gain=g, value_gain=synth.SHARP_VALUE_GAIN, **kw)


def test_static_request_matches_request_with_a_workspace():
    assert binding.lib().lime_request_static_capacity() == 16 << 20
    # the larger problem first: several history chunks, a ragged candidate tail
    big = _sharp(801, B=2, N=1500, C=5000, d=256, h=4, m=64, dtype="bf16", len_range=(700, 1500), pad_value=np.nan)
    small = _sharp(802, B=1, N=200, C=333, d=256, h=4, m=64, dtype="bf16", len_range=(90, 200), pad_value=np.nan)
    for w in (big, small):
        (LP0, O0), (LP1, O1) = _both(w, xor=False)
        assert torch.isfinite(O1.float()).all() and torch.isfinite(LP1.float()).all()
        assert torch.equal(LP0, LP1), "link states differ"
        assert torch.equal(O0, O1), "candidate outputs differ"
    # the XORA form, and a shape that runs on the general kernels (fp32 storage)
    for w, xor in ((_sharp(803, B=3, N=300, C=100, d=128, h=4, m=64, dtype="bf16", len_range=(1, 300), pad_value=np.nan), True),
                   (_sharp(804, B=2, N=90, C=70, d=64, h=2, m=16, dtype="fp32", len_range=(10, 90), pad_value=np.nan), False)):
        (LP0, O0), (LP1, O1) = _both(w, xor)
        assert torch.equal(LP0, LP1) and torch.equal(O0, O1)


def test_static_request_rejects_what_does_not_fit():
    w = synth.make_workload(805, B=64, N=2048, C=64, d=256, h=4, m=128, dtype="bf16")
    g = DeviceWorkload(w)
    with pytest.raises(binding.LimeError) as e:
        binding.lime_request_static(g.E, None, g.L, g.Wq, g.Wk, g.Wv, g.T, g.L, g.Wq, g.Wk, g.Wv, w.h, 1.0, 1.0)
    assert e.value.status == 2 and "scratch" in str(e.value)
