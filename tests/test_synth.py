"""The seeded input generator: determinism, storage rounding, ragged lengths."""

import numpy as np
import torch

from paper_2510_18239_amd import synth


def test_bf16_rounding_matches_torch_rne():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32) * 3
    x[:6] = [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 65504.0]  # includes exact ties
    ours = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(ours, ref)
    back = synth.bf16_bits_to_f32(ours)
    np.testing.assert_array_equal(back, torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    assert np.isnan(synth.round_to(np.array([np.nan], np.float32), "bf16")).all()


def test_workload_is_deterministic_and_shaped():
    a = synth.make_workload(2, B=3, N=40, C=5, d=16, h=4, m=8, dtype="bf16", len_range=(20, 40), pad_value=np.nan)
    b = synth.make_workload(2, B=3, N=40, C=5, d=16, h=4, m=8, dtype="bf16", len_range=(20, 40), pad_value=np.nan)
    for k in ("E", "T", "L", "Wq", "Wk", "Wv", "lens"):
        np.testing.assert_array_equal(getattr(a, k), getattr(b, k))
    assert a.E.shape == (3, 40, 16) and a.T.shape == (3, 5, 16) and a.L.shape == (8, 16)
    assert a.lens.dtype == np.int32 and (a.lens >= 20).all() and (a.lens <= 40).all()
    for i in range(3):
        assert np.isnan(a.E[i, a.lens[i]:]).all() and np.isfinite(a.E[i, : a.lens[i]]).all()
    # values survive a second rounding unchanged (they are already bf16 values)
    np.testing.assert_array_equal(synth.round_to(a.T, "bf16"), a.T)
    c = synth.make_workload(3, B=3, N=40, C=5, d=16, h=4, m=8, dtype="bf16")
    assert not np.array_equal(a.T, c.T) and c.lens is None


def test_distribution_and_sharp_gain():
    w = synth.make_workload(1, B=1, N=4096, C=8, d=64, h=4, m=8, dtype="fp32")
    assert abs(w.E.std() - 64 ** -0.5) < 0.01 * 64 ** -0.5 * 3
    g = synth.sharp_gain(64, 4, w.softmax_scale, 2.0)
    ws = synth.make_workload(1, B=1, N=4096, C=8, d=64, h=4, m=64, dtype="fp32", gain=g)
    q = (ws.L @ ws.Wq).reshape(64, 4, 16)
    k = (ws.E[0] @ ws.Wk).reshape(4096, 4, 16)
    logits = np.einsum("iad,jad->aij", q, k) * ws.softmax_scale
    assert 1.2 < logits.std() < 3.0
