"""Pins for the oracle's scoring pipeline around the two attention stages: layer normalisation before the Q, K, V
projections (Appendix C, "Model Design"), link contextualisation (Eq. 2), the interaction network (Section 3.3) and
their wiring into one request (Eq. 2 -> Eq. 3 -> Eq. 4 -> score).

The paper names these parts without defining them; the readings are stated in the oracle's header.  What is pinned
here is the arithmetic of those readings, against things that are not the oracle's own formula re-typed: scalar
loops with math.sqrt, library routines (torch.nn.functional.layer_norm / linear / relu /
scaled_dot_product_attention, CPU fp64), closed forms, invariants, hand-worked values, and planted mistakes."""

import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import lime_oracle as orc


def _r(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


# ----------------------------------------------------------------------------- layer normalisation

def check_layer_norm_rows_are_standardised():
    X = _r(1, 5, 7, 16) * 3.0 + 2.0
    Y = orc.layer_norm(X, None, None, eps=0.0)
    assert np.abs(Y.mean(axis=-1)).max() < 1e-12
    assert np.abs((Y ** 2).mean(axis=-1) - 1.0).max() < 1e-12  # biased variance: exactly one


def check_layer_norm_hand_values():
    # x = (1, 2, 3, 4): mean 5/2, biased variance 5/4
    y = orc.layer_norm(np.array([[1.0, 2.0, 3.0, 4.0]]), None, None, eps=0.0)[0]
    s = math.sqrt(5.0 / 4.0)
    np.testing.assert_allclose(y, [-1.5 / s, -0.5 / s, 0.5 / s, 1.5 / s], rtol=1e-14)
    # x = (-1, 1): variance 1; eps = 3 sits inside the square root: y = x / 2; then scale and shift
    y = orc.layer_norm(np.array([[-1.0, 1.0]]), np.array([2.0, 4.0]), np.array([10.0, 20.0]), eps=3.0)[0]
    np.testing.assert_allclose(y, [10.0 - 1.0, 20.0 + 2.0], rtol=1e-14)


def check_layer_norm_scalar_loops():
    X, g, b, eps = _r(2, 4, 6), _r(3, 6), _r(4, 6), 1e-5
    Y = orc.layer_norm(X, g, b, eps)
    for i in range(4):
        d = 6
        mean = sum(X[i, k] for k in range(d)) / d
        var = sum((X[i, k] - mean) ** 2 for k in range(d)) / d
        for k in range(d):
            want = (X[i, k] - mean) / math.sqrt(var + eps) * g[k] + b[k]
            assert abs(Y[i, k] - want) < 1e-13


def check_layer_norm_against_library():
    X, g, b = _r(5, 3, 9, 32), _r(6, 32), _r(7, 32)
    want = F.layer_norm(torch.from_numpy(X), (32,), torch.from_numpy(g), torch.from_numpy(b), eps=1e-5).numpy()
    np.testing.assert_allclose(orc.layer_norm(X, g, b, 1e-5), want, rtol=1e-12, atol=1e-12)


def check_layer_norm_shift_and_scale_invariance():
    X = _r(8, 6, 12)
    base = orc.layer_norm(X, None, None, eps=0.0)
    np.testing.assert_allclose(orc.layer_norm(3.5 * X + 11.0, None, None, eps=0.0), base, atol=1e-12)
    # identity on rows that are already standardised, and idempotent
    np.testing.assert_allclose(orc.layer_norm(base, None, None, eps=0.0), base, atol=1e-12)


# ----------------------------------------------------------------------------- Eq. 2

def _ctx_problem(seed, B=3, m=4, d=6, dc=5, dhid=7):
    r = np.random.default_rng(seed)
    return dict(L=r.standard_normal((m, d)), EC=r.standard_normal((B, dc)), W1=r.standard_normal((d + dc, dhid)),
                b1=r.standard_normal(dhid), W2=r.standard_normal((dhid, d)), b2=r.standard_normal(d))


def check_contextualize_scalar_loops():
    p = _ctx_problem(11)
    LC = orc.contextualize_links(**p)
    B, (m, d), dc, dhid = p["EC"].shape[0], p["L"].shape, p["EC"].shape[1], p["W1"].shape[1]
    for b in range(B):
        for i in range(m):
            x = [p["L"][i, k] for k in range(d)] + [p["EC"][b, k] for k in range(dc)]  # link row first, then the context
            hid = [max(0.0, sum(x[k] * p["W1"][k, j] for k in range(d + dc)) + p["b1"][j]) for j in range(dhid)]
            for c in range(d):
                want = sum(hid[j] * p["W2"][j, c] for j in range(dhid)) + p["b2"][c]
                assert abs(LC[b, i, c] - want) < 1e-12


def check_contextualize_against_library():
    p = _ctx_problem(12)
    t = {k: torch.from_numpy(v) for k, v in p.items()}
    for b in range(3):
        X = torch.cat([t["L"], t["EC"][b].expand(4, -1)], dim=1)
        want = F.linear(F.relu(F.linear(X, t["W1"].T, t["b1"])), t["W2"].T, t["b2"]).numpy()
        np.testing.assert_allclose(orc.contextualize_links(**p)[b], want, rtol=1e-12, atol=1e-12)


def check_contextualize_without_context_weights_is_user_independent():
    p = _ctx_problem(13)
    p["W1"][6:] = 0.0  # the rows of W1 that multiply the context vector
    LC = orc.contextualize_links(**p)
    assert np.array_equal(LC[0], LC[1]) and np.array_equal(LC[0], LC[2])
    # ... and with them, users differ
    assert not np.allclose(orc.contextualize_links(**_ctx_problem(13))[0], orc.contextualize_links(**_ctx_problem(13))[1])


def check_contextualize_affine_regime():
    # a large first bias keeps every hidden unit positive: the MLP is then the affine map (X W1 + b1) W2 + b2
    p = _ctx_problem(14)
    p["b1"] = p["b1"] + 100.0
    LC = orc.contextualize_links(**p)
    for b in range(3):
        X = np.concatenate([p["L"], np.tile(p["EC"][b], (4, 1))], axis=1)
        np.testing.assert_allclose(LC[b], (X @ p["W1"] + p["b1"]) @ p["W2"] + p["b2"], rtol=1e-11)
    # a very negative one switches every unit off: the output is b2 for every link
    p["b1"] = p["b1"] - 1000.0
    np.testing.assert_allclose(orc.contextualize_links(**p), np.broadcast_to(p["b2"], (3, 4, 6)))


# ----------------------------------------------------------------------------- the interaction network

def _mlp_problem(seed, d=6, sizes=(5, 4, 3)):
    r = np.random.default_rng(seed)
    dims = (d,) + tuple(sizes) + (1,)
    return [r.standard_normal((dims[i], dims[i + 1])) for i in range(len(dims) - 1)], \
           [r.standard_normal(dims[i + 1]) for i in range(len(dims) - 1)]


def check_interaction_mlp_scalar_loops():
    Ws, bs = _mlp_problem(21)
    O = _r(22, 2, 5, 6)
    got = orc.interaction_mlp(O, Ws, bs)
    assert got.shape == (2, 5)
    for b in range(2):
        for c in range(5):
            x = list(O[b, c])
            for li, (W, bias) in enumerate(zip(Ws, bs)):
                y = [sum(x[k] * W[k, j] for k in range(len(x))) + bias[j] for j in range(W.shape[1])]
                x = y if li + 1 == len(Ws) else [max(0.0, v) for v in y]  # no ReLU on the logit
            assert abs(got[b, c] - x[0]) < 1e-12


def check_interaction_mlp_closed_forms():
    Ws, bs = _mlp_problem(23)
    O = _r(24, 3, 4, 6)
    # all-zero last weights: every score is the last bias
    Wz = Ws[:-1] + [np.zeros_like(Ws[-1])]
    np.testing.assert_allclose(orc.interaction_mlp(O, Wz, bs), np.full((3, 4), bs[-1][0]))
    # no hidden layer: a dot product plus bias, which may be negative (the logit is not rectified)
    w, b0 = _r(25, 6, 1), np.array([-50.0])
    got = orc.interaction_mlp(O, [w], [b0])
    np.testing.assert_allclose(got, O @ w[:, 0] - 50.0)
    assert (got < 0).all()
    # a hidden layer that is switched off (very negative bias) leaves only the biases downstream
    bs2 = [bs[0] - 1e6] + bs[1:]
    a = orc.interaction_mlp(O, Ws, bs2)
    assert np.ptp(a) == 0.0


def check_interaction_mlp_against_library():
    Ws, bs = _mlp_problem(26, d=8, sizes=(16, 4))
    O = _r(27, 7, 8)
    x = torch.from_numpy(O)
    for i, (W, b) in enumerate(zip(Ws, bs)):
        x = F.linear(x, torch.from_numpy(W).T, torch.from_numpy(b))
        if i + 1 < len(Ws):
            x = F.relu(x)
    np.testing.assert_allclose(orc.interaction_mlp(O, Ws, bs), x[:, 0].numpy(), rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- the whole request

def _request(seed, B=2, N=9, C=6, d=8, m=4, dc=3, dhid=5, h=2):
    r = np.random.default_rng(seed)
    w = lambda *s: r.standard_normal(s) / 2  # noqa: E731
    ln = lambda: (1.0 + 0.3 * r.standard_normal(d), 0.3 * r.standard_normal(d))  # noqa: E731
    p = dict(ctx=(w(d + dc, dhid), w(dhid), w(dhid, d), w(d)), hist=(w(d, d), w(d, d), w(d, d)), cand=(w(d, d), w(d, d), w(d, d)),
             ln_hist_q=ln(), ln_hist_kv=ln(), ln_cand_q=ln(), ln_cand_k=ln(), ln_cand_v=ln(),
             mlp=([w(d, 7), w(7, 1)], [w(7), w(1)]))
    return dict(E=r.standard_normal((B, N, d)), lens=np.array([N, 5][:B]), L=r.standard_normal((m, d)), EC=r.standard_normal((B, dc)),
                T=r.standard_normal((B, C, d)), p=p, h=h, scale_hist=0.7, scale_cand=0.4)


def _torch_mha(Q, K, V, Wq, Wk, Wv, h, scale):
    """Eq. 1 with library routines only: projections by F.linear, heads by reshaping, softmax attention by SDPA."""
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x))  # noqa: E731
    q, k, v = F.linear(t(Q), t(Wq).T), F.linear(t(K), t(Wk).T), F.linear(t(V), t(Wv).T)
    split = lambda x: x.reshape(x.shape[0], h, -1).transpose(0, 1)  # noqa: E731
    o = F.scaled_dot_product_attention(split(q), split(k), split(v), scale=scale)
    return o.transpose(0, 1).reshape(Q.shape[0], -1).numpy()


def check_request_wiring_against_library_chain():
    """Eq. 2 -> LN -> Eq. 3 -> LN -> Eq. 4 -> MLP written out with torch's own layer_norm, linear, relu and SDPA."""
    a = _request(31)
    p, h = a["p"], a["h"]
    scores, LC, LP, O = orc.lime_scores(**a, return_all=True)
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x))  # noqa: E731
    ln = lambda x, gb: F.layer_norm(t(x), (x.shape[-1],), t(gb[0]), t(gb[1]), eps=1e-5).numpy()  # noqa: E731
    for b in range(2):
        n = int(a["lens"][b])
        X = torch.cat([t(a["L"]), t(a["EC"][b]).expand(4, -1)], dim=1)
        W1, b1, W2, b2 = (t(x) for x in p["ctx"])
        lc = F.linear(F.relu(F.linear(X, W1.T, b1)), W2.T, b2).numpy()
        np.testing.assert_allclose(LC[b], lc, rtol=1e-11, atol=1e-11)
        Eb = a["E"][b, :n]
        lp = _torch_mha(ln(lc, p["ln_hist_q"]), ln(Eb, p["ln_hist_kv"]), ln(Eb, p["ln_hist_kv"]), *p["hist"], h, a["scale_hist"])
        np.testing.assert_allclose(LP[b], lp, rtol=1e-10, atol=1e-10)
        # decoupled attention: keys from the raw links L, values from the personalised links L^P
        o = _torch_mha(ln(a["T"][b], p["ln_cand_q"]), ln(a["L"], p["ln_cand_k"]), ln(lp, p["ln_cand_v"]), *p["cand"], h, a["scale_cand"])
        np.testing.assert_allclose(O[b], o, rtol=1e-9, atol=1e-9)
        x = t(o)
        for i, (W, bias) in enumerate(zip(*p["mlp"])):
            x = F.linear(x, t(W).T, t(bias))
            if i == 0:
                x = F.relu(x)
        np.testing.assert_allclose(scores[b], x[:, 0].numpy(), rtol=1e-9, atol=1e-9)


def check_request_invariants():
    a = _request(32)
    base = orc.lime_scores(**a)
    assert base.shape == (2, 6)
    # candidates are scored independently: permuting them permutes the scores
    perm = np.array([3, 0, 5, 1, 4, 2])
    a2 = dict(a, T=a["T"][:, perm])
    np.testing.assert_array_equal(orc.lime_scores(**a2), base[:, perm])
    # layer normalisation makes the request blind to a positive rescaling and a shift of every candidate row
    a3 = dict(a, T=2.5 * a["T"] + 1.0)
    np.testing.assert_allclose(orc.lime_scores(**a3, eps=0.0), orc.lime_scores(**a, eps=0.0), rtol=1e-9, atol=1e-9)
    # rows of the history past lens[b] are never read
    a4 = dict(a, E=a["E"].copy())
    a4["E"][1, 5:] = np.nan
    np.testing.assert_array_equal(orc.lime_scores(**a4), base)
    # a user's scores do not depend on another user's context vector
    a5 = dict(a, EC=a["EC"].copy())
    a5["EC"][1] += 1.0
    got = orc.lime_scores(**a5)
    np.testing.assert_array_equal(got[0], base[0])
    assert not np.allclose(got[1], base[1])


PINS = [check_layer_norm_rows_are_standardised, check_layer_norm_hand_values, check_layer_norm_scalar_loops,
        check_layer_norm_against_library, check_layer_norm_shift_and_scale_invariance, check_contextualize_scalar_loops,
        check_contextualize_against_library, check_contextualize_without_context_weights_is_user_independent,
        check_contextualize_affine_regime, check_interaction_mlp_scalar_loops, check_interaction_mlp_closed_forms,
        check_interaction_mlp_against_library, check_request_wiring_against_library_chain, check_request_invariants]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()


# ----------------------------------------------------------------------------- planted mistakes

def _f(x):
    return None if x is None else np.asarray(x, dtype=np.float64)


def _ln_variant(kind):
    def ln(X, gamma, beta, eps=1e-5):
        X = _f(X)
        with np.errstate(invalid="ignore", divide="ignore"):
            mean = X.mean(axis=-1, keepdims=True)
            var = ((X - mean) ** 2).mean(axis=-1, keepdims=True)
            if kind == "unbiased_variance":
                var = var * X.shape[-1] / (X.shape[-1] - 1)
            if kind == "eps_outside_root":
                Y = (X - mean) / (np.sqrt(var) + eps)
            elif kind == "no_mean_subtraction":
                Y = X / np.sqrt((X ** 2).mean(axis=-1, keepdims=True) + eps)
            else:
                Y = (X - mean) / np.sqrt(var + eps)
        if gamma is not None:
            Y = Y * _f(gamma)
        if beta is not None:
            Y = Y * _f(beta) if kind == "shift_multiplies" else Y + _f(beta)
        return Y
    ln.__name__ = f"layer_norm_{kind}"
    return ln


def _ctx_variant(kind):
    def ctx(L, EC, W1, b1, W2, b2):
        L, EC = _f(L), _f(EC)
        out = []
        for b in range(EC.shape[0]):
            e = EC[0] if kind == "first_users_context" else EC[b]
            parts = [np.broadcast_to(e, (L.shape[0], EC.shape[1])), L] if kind == "context_first" else \
                [L, np.broadcast_to(e, (L.shape[0], EC.shape[1]))]
            hid = np.concatenate(parts, axis=1) @ _f(W1) + _f(b1)
            if kind != "no_relu":
                hid = np.maximum(hid, 0.0)
            y = hid @ _f(W2) + _f(b2)
            out.append(np.maximum(y, 0.0) if kind == "relu_on_output" else y)
        return np.stack(out)
    ctx.__name__ = f"contextualize_{kind}"
    return ctx


def _mlp_variant(kind):
    def mlp(O, weights, biases):
        x = _f(O)
        for i, (W, b) in enumerate(zip(weights, biases)):
            x = x @ _f(W) + (0.0 if kind == "no_bias" else _f(b))
            if i + 1 < len(weights) or kind == "relu_on_logit":
                x = np.maximum(x, 0.0)
        return x[..., 0]
    mlp.__name__ = f"interaction_mlp_{kind}"
    return mlp


def _scores_variant(kind):
    def scores(E, lens, L, EC, T, p, h, scale_hist, scale_cand, eps=1e-5, return_all=False):
        ln = orc.layer_norm
        LC = orc.contextualize_links(L, EC, *p["ctx"])
        q_links = L if kind == "raw_links_as_queries" else LC
        LP = orc.lime_link_history(ln(E, *p["ln_hist_kv"], eps), lens, ln(q_links, *p["ln_hist_q"], eps), *p["hist"], h, scale_hist)
        Tn = T if kind == "candidates_not_normalised" else ln(T, *p["ln_cand_q"], eps)
        kg, vg = (p["ln_cand_v"], p["ln_cand_k"]) if kind == "key_value_norms_swapped" else (p["ln_cand_k"], p["ln_cand_v"])
        keys = LP if kind == "personalised_links_as_keys" else L
        O = orc.lime_score_candidates(Tn, ln(keys, *kg, eps), ln(LP, *vg, eps), *p["cand"], h, scale_cand)
        s = orc.interaction_mlp(O, *p["mlp"])
        return (s, LC, LP, O) if return_all else s
    scores.__name__ = f"lime_scores_{kind}"
    return scores


MUTATIONS = [("layer_norm", _ln_variant(k)) for k in ("unbiased_variance", "eps_outside_root", "no_mean_subtraction", "shift_multiplies")] + \
            [("contextualize_links", _ctx_variant(k)) for k in ("context_first", "no_relu", "relu_on_output", "first_users_context")] + \
            [("interaction_mlp", _mlp_variant(k)) for k in ("no_bias", "relu_on_logit")] + \
            [("lime_scores", _scores_variant(k)) for k in ("raw_links_as_queries", "candidates_not_normalised", "key_value_norms_swapped",
                                                           "personalised_links_as_keys")]


def _pins_that_fail():
    failed = []
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin()
        except Exception:  # noqa: BLE001 - any failure counts as "caught"
            failed.append(pin.__name__)
    return failed


@pytest.mark.parametrize("name,mutant", MUTATIONS, ids=[m.__name__ for _, m in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    """A plausible mistake planted in the oracle (on the CPU) must fail at least one pin."""
    assert _pins_that_fail() == []
    monkeypatch.setattr(orc, name, mutant)
    assert _pins_that_fail(), f"mutation {name} survived every pin"
