"""GPU parity of lime_xor_backward (Appendix H.2) against the oracle, element by element, through the C ABI."""

import numpy as np
import pytest
import torch

from oracle import lime_oracle as orc
from paper_2510_18239_amd import binding, synth
from parity_util import assert_close, dev, host

pytestmark = pytest.mark.gpu

NAMES = ("dQS", "dKS", "dVS", "dQT", "dKT", "dVT")
# The gradients are linear in the values and in the upstream gradients: sized so that every gradient entry stays
# below one (sums over thousands of rows, divisions by history lengths of one or two), where the stated absolute
# bar applies; the logits keep their unit standard deviation.
SIZED = dict(value_std=0.5, grad_std=0.1)


def _run(t, h, scale, dtype, with_dos=True):
    g = {k: dev(v, dtype) for k, v in t.items() if k != "lens"}
    lens = None if t["lens"] is None else torch.from_numpy(t["lens"]).cuda()
    got = binding.lime_xor_backward(g["QS"], g["KS"], g["VS"], g["QT"], g["KT"], g["VT"], g["dOT"],
                                    g["dOS"] if with_dos else None, lens, h, scale)
    ref = orc.xor_attention_backward(t["QS"], t["KS"], t["VS"], t["QT"], t["KT"], t["VT"], t["dOT"],
                                     t["dOS"] if with_dos else None, t["lens"], h, scale)
    return [host(x) for x in got], ref


@pytest.mark.parametrize("B,N,m,d,h,dtype,scale", [
    (2, 100, 64, 128, 4, "bf16", 1.0),      # matrix-core form (bf16, d/h = 32), ragged tail in N
    (3, 700, 64, 128, 4, "bf16", 1.0),      # many chunks
    (2, 333, 128, 256, 4, "bf16", 0.7),     # d/h = 64, the widest head; 128 links: the two-kernel form
    (2, 333, 64, 256, 4, "bf16", 0.7),      # d/h = 64 in one pass, two blocks of links
    (3, 700, 24, 128, 2, "bf16", 1.0),      # d/h = 64 in one pass, one ragged block of links
    (2, 50, 40, 128, 4, "bf16", 1.0),       # matrix-core form with m and N that fill no tile
    (2, 300, 32, 128, 4, "bf16", 1.0),      # one block of links
    (3, 1000, 17, 64, 2, "bf16", 0.8),      # one ragged block of links, chunks of several tiles per wave
    (2, 600, 96, 128, 4, "bf16", 1.0),      # three blocks of links in one pass (one wave per SIMD)
    (2, 450, 128, 64, 2, "bf16", 0.9),      # four blocks of links in one pass
    (2, 200, 64, 64, 4, "bf16", 1.0),       # bf16 with d/h = 16: the fp32-arithmetic kernel on bf16 storage
    (1, 65, 5, 24, 1, "fp32", 1.0),         # m and d/h far from any tile size
    (2, 47, 37, 40, 5, "fp32", -0.5),       # d/h = 8, negative scale
    (4, 16, 32, 64, 2, "fp32", 1.3),
    (1, 1, 1, 8, 1, "fp32", 1.0),           # the smallest problem
])
def test_xor_backward_matches_oracle(B, N, m, d, h, dtype, scale):
    """Ragged histories with NaN padding and, from three users on, one empty user; all six gradients."""
    t = synth.backward_inputs(500 + N + m, B, N, m, d, h, dtype, len_range=(1, N), pad_value=np.nan, **SIZED)
    if B >= 3:
        t["lens"][B - 1] = 0
        for k in ("QS", "KS", "VS", "dOS"):
            t[k][B - 1] = np.nan
    print(f"case B={B} N={N} m={m} d={d} h={h} {dtype} lens={t['lens'].tolist()}", flush=True)
    got, ref = _run(t, h, scale, dtype)
    for name, x, r in zip(NAMES, got, ref):
        assert_close(x, r, dtype, name)
    for name, x in zip(NAMES[:3], got[:3]):
        for b in range(B):
            assert not x[b, t["lens"][b]:].any(), f"{name}: padded rows of user {b} must get zero gradients"
    if B >= 3:
        assert not any(x[B - 1].any() for x in got), "a user without history gets zero gradients"


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_xor_backward_without_source_gradient(dtype):
    """dOS absent (O[S] has no consumer, as in a single layer): dQS, dKT and dVT are exactly zero, the other three
    are those of the full call with a zero dOS; all lengths full (lens absent)."""
    t = synth.backward_inputs(77, 2, 130, 64, 128, 4, dtype, **SIZED)
    got, ref = _run(t, 4, 1.0, dtype, with_dos=False)
    for name, x, r in zip(NAMES, got, ref):
        assert_close(x, r, dtype, name)
    assert not got[0].any() and not got[4].any() and not got[5].any()
    t["dOS"][:] = 0.0
    again, _ = _run(t, 4, 1.0, dtype)
    for x, y in zip(got, again):
        np.testing.assert_array_equal(x, y)


def test_xor_backward_at_benchmark_size_is_deterministic():
    """Configuration 4's shape (8 users, d = 128, h = 4, m = 64) at N = 2048, the size bench.py --extras times: every
    element against the oracle, and two runs give the same bits (chunk partial sums are added in a fixed order)."""
    t = synth.backward_inputs(4, 8, 2048, 64, 128, 4, "bf16", len_range=(1024, 2048), **SIZED)
    got, ref = _run(t, 4, 1.0, "bf16")
    for name, x, r in zip(NAMES, got, ref):
        assert_close(x, r, "bf16", name)
    again, _ = _run(t, 4, 1.0, "bf16")
    for x, y in zip(got, again):
        np.testing.assert_array_equal(x, y)


def test_xor_backward_random_shapes():
    """Thirty seeded random shapes of the bf16 forms (d/h = 32 or 64, 1 .. 129 links, histories of up to 2600 rows, full
    or ragged with NaN padding, now and then an empty user, with and without dOS, four scales): every gradient against
    the oracle, padded rows exactly zero.  Every variant of the one-pass form and the two-kernel form are drawn."""
    rng = np.random.default_rng(12345)
    for case in range(30):
        dh, h = int(rng.choice([32, 64])), int(rng.choice([1, 2, 4]))
        m, N, B = int(rng.integers(1, 130)), int(rng.integers(1, 2600)), int(rng.integers(1, 5))
        scale, with_dos, ragged = float(rng.choice([1.0, 0.7, -0.5, 1.3])), bool(rng.integers(0, 4) > 0), bool(rng.integers(0, 3) > 0)
        kw = dict(len_range=(1, N), pad_value=np.nan) if ragged else {}
        t = synth.backward_inputs(1000 + case, B, N, m, dh * h, h, "bf16", **kw, **SIZED)
        if ragged and B >= 2 and case % 5 == 0:
            t["lens"][B - 1] = 0
            for k in ("QS", "KS", "VS", "dOS"):
                t[k][B - 1] = np.nan
        print(f"case {case}: B={B} N={N} m={m} d={dh * h} h={h} scale={scale} dOS={with_dos} "
              f"lens={None if t['lens'] is None else t['lens'].tolist()}", flush=True)
        got, ref = _run(t, h, scale, "bf16", with_dos=with_dos)
        for name, x, r in zip(NAMES, got, ref):
            assert_close(x, r, "bf16", f"case {case} {name}")
        if t["lens"] is not None:
            for name, x in zip(NAMES[:3], got[:3]):
                for b in range(B):
                    assert not x[b, t["lens"][b]:].any(), f"case {case} {name}: padded rows of user {b} must get zero gradients"
