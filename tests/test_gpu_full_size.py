"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times
(same entry points, same shapes, bf16 storage).  The oracle is fast enough to check every
output element of the LIME paths; only the full-target-attention baseline is checked on a
sample of users and candidates (its oracle would need ~0.5 TFLOP in fp64).

Both input families run: the benchmark distribution (gain 1: the bytes bench.py times) and the
sharpened one (logit standard deviation about 2), where the absolute bar is meaningful."""

import numpy as np
import pytest
import torch

from oracle import lime_oracle as orc
from paper_2510_18239_amd import binding, synth
from parity_util import DeviceWorkload, assert_close, host

pytestmark = pytest.mark.gpu


def _workload(idx, gain, **override):
    c = dict(synth.CONFIGS[idx])
    c.update(override)
    if "len_range" in c:
        c["pad_value"] = np.nan
    if gain == "sharp":
        c["gain"] = synth.sharp_gain(c["d"], c["h"], (c["d"] // c["h"]) ** -0.5, 2.0)
        c["value_gain"] = synth.SHARP_VALUE_GAIN
    return synth.make_workload(idx, **c)


@pytest.mark.parametrize("gain", ["bench", "sharp"])
def test_config2_batched_ragged(gain):
    w = _workload(2, gain)
    g = DeviceWorkload(w)
    s = w.softmax_scale
    print(f"config 2 {gain}: lens {w.lens.min()}..{w.lens.max()}", flush=True)
    LP = binding.lime_link_history(g.E, g.lens, g.L, g.Wq, g.Wk, g.Wv, w.h, s)
    O = binding.lime_score_candidates(g.T, g.L, LP, g.Wq, g.Wk, g.Wv, w.h, s)
    assert_close(host(LP), orc.lime_link_history(w.E, w.lens, w.L, w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "LP")
    assert_close(host(O), orc.lime_score_candidates(w.T, w.L, host(LP), w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "O")
    A = binding.mha_target_attention(g.T, g.E, g.lens, g.Wq, g.Wk, g.Wv, w.h, s)
    assert_close(host(A), orc.mha_target_attention(w.T, w.E, w.lens, w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "MHA")


@pytest.mark.parametrize("gain", ["bench", "sharp"])
def test_config3_headline_request(gain):
    """B=1, N=2048, C=32768, d=256, h=4, m=64: the request bench.py times, every element checked."""
    w = _workload(3, gain)
    g = DeviceWorkload(w)
    s = w.softmax_scale
    LP = binding.lime_link_history(g.E, None, g.L, g.Wq, g.Wk, g.Wv, w.h, s)
    O = binding.lime_score_candidates(g.T, g.L, LP, g.Wq, g.Wk, g.Wv, w.h, s)
    LP_ref = orc.lime_link_history(w.E, None, w.L, w.Wq, w.Wk, w.Wv, w.h, s)
    assert_close(host(LP), LP_ref, "bf16", "LP")
    assert_close(host(O), orc.lime_score_candidates(w.T, w.L, host(LP), w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "O")
    assert_close(host(O), orc.lime_score_candidates(w.T, w.L, LP_ref, w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "chain")
    # the same request as the one call bench.py's step makes
    LP1, O1 = binding.lime_request(g.E, None, g.L, g.Wq, g.Wk, g.Wv, g.T, g.L, g.Wq, g.Wk, g.Wv, w.h, s, s)
    assert torch.equal(LP1, LP)
    assert_close(host(O1), orc.lime_score_candidates(w.T, w.L, host(LP1), w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "O in one call")
    assert_close(host(O1), orc.lime_score_candidates(w.T, w.L, LP_ref, w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "chain in one call")


@pytest.mark.parametrize("gain", ["bench", "sharp"])
def test_config2_and_config5_requests_in_one_call(gain):
    """lime_request at the two batched full sizes (ragged lengths; m = 64 and m = 128), every element checked."""
    for idx in (2, 5):
        w = _workload(idx, gain)
        g = DeviceWorkload(w)
        s = w.softmax_scale
        print(f"config {idx} {gain}: lens {w.lens.min()}..{w.lens.max()}", flush=True)
        LP, O = binding.lime_request(g.E, g.lens, g.L, g.Wq, g.Wk, g.Wv, g.T, g.L, g.Wq, g.Wk, g.Wv, w.h, s, s)
        assert_close(host(LP), orc.lime_link_history(w.E, w.lens, w.L, w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "LP")
        assert_close(host(O), orc.lime_score_candidates(w.T, w.L, host(LP), w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "O")


@pytest.mark.parametrize("C", [16, 48, 1000, 4096])
def test_config3_candidate_sweep_points(C):
    """Other points of the candidate sweep, including counts that are not a multiple of the tile."""
    w = _workload(3, "sharp", C=C)
    g = DeviceWorkload(w)
    s = w.softmax_scale
    LPv = synth.per_user_links(3, 1, w.m, w.d, "bf16", gain=w.meta["gain"] * synth.SHARP_VALUE_GAIN)
    O = binding.lime_score_candidates(g.T, g.L, torch.from_numpy(LPv).to(torch.bfloat16).cuda(), g.Wq, g.Wk, g.Wv,
                                      w.h, s)
    assert_close(host(O), orc.lime_score_candidates(w.T, w.L, LPv, w.Wq, w.Wk, w.Wv, w.h, s), "bf16", f"O at C={C}")


@pytest.mark.parametrize("N", [2048, 4096, 8192, 16384])
@pytest.mark.parametrize("gain", ["bench", "sharp"])
def test_config4_long_history_xora(N, gain):
    """8 users, d=128, h=4, m=64, linear XORA pass with both outputs."""
    w = _workload(4, gain, N=N)
    g = DeviceWorkload(w)
    scale = 1.0 if gain == "bench" else w.softmax_scale  # Algorithm 2 uses no scale; sharp inputs need one to stay O(1)
    OT, OS = binding.lime_xor_history(g.E, None, g.L, g.Wq, g.Wk, g.Wv, w.h, scale, want_os=True)
    OT_ref, OS_ref = orc.lime_xor_history(w.E, None, w.L, w.Wq, w.Wk, w.Wv, w.h, scale)
    assert_close(host(OT), OT_ref, "bf16", "O[T]")
    assert_close(host(OS), OS_ref, "bf16", "O[S]")
    O = binding.lime_score_candidates(g.T, g.L, OT, g.Wq, g.Wk, g.Wv, w.h, w.softmax_scale)
    assert_close(host(O), orc.lime_score_candidates(w.T, w.L, host(OT), w.Wq, w.Wk, w.Wv, w.h, w.softmax_scale), "bf16",
                 "O")


@pytest.mark.parametrize("N", [2048, 4096, 8192, 16384])
@pytest.mark.parametrize("gain", ["bench", "sharp"])
def test_config4_stacked_xor_layers(N, gain):
    """8 users, d=128, h=4, m=64: three stacked XOR layers (Eq. 8) at the sizes bench.py --extras times; the gated
    blocks' weights ~N(0, 1/d) like every other weight (the gate projection twice as large on sharp inputs)."""
    w = _workload(4, gain, N=N)
    g = DeviceWorkload(w)
    scale = 1.0 if gain == "bench" else w.softmax_scale
    r = np.random.default_rng(4077)
    rnd = lambda x: torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).float().numpy()  # noqa: E731
    Wu = rnd(r.standard_normal((3, w.d, w.d)) * w.d ** -0.5 * (2.0 if gain == "sharp" else 1.0))
    Wo = rnd(r.standard_normal((3, w.d, w.d)) * w.d ** -0.5)
    to_dev = lambda x: torch.from_numpy(x).to(torch.bfloat16).cuda()  # noqa: E731
    LP = binding.lime_xor_layers(g.E, None, g.L, g.Wq, g.Wk, g.Wv, to_dev(Wu), to_dev(Wo), w.h, scale)
    ref = orc.lime_xor_layers(w.E, None, w.L, w.Wq, w.Wk, w.Wv, Wu, Wo, w.h, scale)
    err = assert_close(host(LP), ref, "bf16", "LP of three XOR layers")
    print(f"N={N} {gain}: max|ref| {np.abs(ref).max():.3e}, max-abs error {err:.3e}", flush=True)


@pytest.mark.parametrize("gain", ["bench", "sharp"])
def test_config5_lime_side(gain):
    """16 users, N=4096 ragged, C=8192, m=128, d=256: the LIME half of the speed-up comparison."""
    w = _workload(5, gain)
    g = DeviceWorkload(w)
    s = w.softmax_scale
    LP = binding.lime_link_history(g.E, g.lens, g.L, g.Wq, g.Wk, g.Wv, w.h, s)
    O = binding.lime_score_candidates(g.T, g.L, LP, g.Wq, g.Wk, g.Wv, w.h, s)
    assert_close(host(LP), orc.lime_link_history(w.E, w.lens, w.L, w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "LP")
    assert_close(host(O), orc.lime_score_candidates(w.T, w.L, host(LP), w.Wq, w.Wk, w.Wv, w.h, s), "bf16", "O")


@pytest.mark.parametrize("gain", ["bench", "sharp"])
def test_config5_target_attention_sampled(gain):
    """The baseline at full size; the oracle checks 3 users x 96 sampled candidates, the first and last
    candidate of each among them."""
    w = _workload(5, gain)
    g = DeviceWorkload(w)
    s = w.softmax_scale
    A = binding.mha_target_attention(g.T, g.E, g.lens, g.Wq, g.Wk, g.Wv, w.h, s)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    users = [0, int(np.argmin(w.lens)), w.B - 1]
    for b in users:
        idx = np.unique(np.concatenate([[0, w.C - 1], rng.integers(0, w.C, 94)]))
        ref = orc.mha_target_attention(w.T[b:b + 1, idx], w.E[b:b + 1], w.lens[b:b + 1], w.Wq, w.Wk, w.Wv, w.h, s)
        assert_close(host(A[b:b + 1, torch.from_numpy(idx).cuda()]), ref, "bf16", f"MHA user {b}")


def test_config4_xor_backward_long_history():
    """8 users, d = 128, h = 4, m = 64 at N = 16384, the larger size bench.py --extras times for lime_xor_backward:
    all six gradients, every element, against the oracle."""
    t = synth.backward_inputs(4, 8, 16384, 64, 128, 4, "bf16", value_std=0.5, grad_std=0.1)  # gradients below one
    g = {k: torch.from_numpy(v).to(torch.bfloat16).cuda() for k, v in t.items() if k != "lens"}
    got = binding.lime_xor_backward(g["QS"], g["KS"], g["VS"], g["QT"], g["KT"], g["VT"], g["dOT"], g["dOS"], None, 4, 1.0)
    ref = orc.xor_attention_backward(t["QS"], t["KS"], t["VS"], t["QT"], t["KT"], t["VT"], t["dOT"], t["dOS"], None, 4, 1.0)
    for name, x, r in zip(("dQS", "dKS", "dVS", "dQT", "dKT", "dVT"), got, ref):
        assert_close(host(x), r, "bf16", name)
