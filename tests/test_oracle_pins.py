"""Pins for the CPU oracle: things the paper and the mathematics fix, none of
which is the oracle's own formula re-typed with the same library calls.

  * hand-worked closed-form cases (tests/golden/*.json),
  * scalar brute force written from Eq. 1 with math.exp and Python loops,
  * a library routine (torch's scaled_dot_product_attention, CPU fp64),
  * closed forms (uniform attention, identity links, constant logits),
  * invariants (rows sum to one, permutations, zero cross-dependence, masks),
  * planted mistakes: each mutation of the oracle must break at least one pin.
"""

import json
import math
import os

import numpy as np
import pytest

from oracle import lime_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------- helpers

def _val(x):
    if isinstance(x, str):
        return float(eval(x, {"__builtins__": {}}, {"ln": math.log}))
    return float(x)


def _arr(x):
    if x is None:
        return None
    if isinstance(x, list):
        return np.array([_arr(v) for v in x], dtype=np.float64)
    return _val(x)


def _load(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return json.load(f)


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _problem(seed, B=2, N=7, C=5, d=8, m=3):
    r = np.random.default_rng(seed)
    return dict(E=r.standard_normal((B, N, d)), T=r.standard_normal((B, C, d)), L=r.standard_normal((m, d)),
                Wq=r.standard_normal((d, d)) / 2, Wk=r.standard_normal((d, d)) / 2, Wv=r.standard_normal((d, d)) / 2)


# ----------------------------------------------------------------------------- hand-worked cases

def check_golden_eq3():
    g = _load("eq3_link_history.json")
    LP = orc.lime_link_history(_arr(g["E"]), None, _arr(g["LC"]), _arr(g["Wq"]), _arr(g["Wk"]), _arr(g["Wv"]),
                               g["h"], g["scale"])
    np.testing.assert_allclose(LP, _arr(g["LP"]), rtol=0, atol=1e-14)


def check_golden_eq4():
    g = _load("eq4_decoupled_candidates.json")
    O = orc.lime_score_candidates(_arr(g["T"]), _arr(g["L"]), _arr(g["LP"]), None, None, None, g["h"], g["scale"])
    np.testing.assert_allclose(O, _arr(g["O"]), rtol=0, atol=1e-14)


def check_golden_xora():
    g = _load("xora_two_heads.json")
    OT, OS = orc.lime_xor_history(_arr(g["E"]), None, _arr(g["LC"]), _arr(g["Wq"]), _arr(g["Wk"]), _arr(g["Wv"]),
                                  g["h"], g["scale"])
    np.testing.assert_allclose(OT, _arr(g["OT"]), rtol=0, atol=1e-14)
    np.testing.assert_allclose(OS, _arr(g["OS"]), rtol=0, atol=1e-14)
    os_q, ot_q = orc.xora_quadratic(_arr(g["E"])[0], _arr(g["LC"]), _arr(g["Wq"]), _arr(g["Wk"]), _arr(g["Wv"]),
                                    g["h"], g["scale"])
    np.testing.assert_allclose(ot_q, _arr(g["OT"])[0], rtol=0, atol=1e-14)
    np.testing.assert_allclose(os_q, _arr(g["OS"])[0], rtol=0, atol=1e-14)


def check_golden_eq1_masked():
    g = _load("eq1_target_attention_masked.json")
    O = orc.mha_target_attention(_arr(g["T"]), _arr(g["E"]), g["lens"], _arr(g["Wq"]), _arr(g["Wk"]), _arr(g["Wv"]),
                                 g["h"], g["scale"])
    np.testing.assert_allclose(O, _arr(g["O"]), rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- scalar brute force (Eq. 1)

def _brute_attention(Q, K, V, Wq, Wk, Wv, h, scale, phi, denom=1.0):
    """Eq. 1 for one user with scalar loops: no matmul, no vectorised exp."""
    q, d = len(Q), len(Q[0])
    n = len(K)
    dh = d // h

    def proj(X, W):
        return [[sum(X[r][k] * W[k][c] for k in range(d)) for c in range(d)] for r in range(len(X))]

    Qt, Kt, Vt = proj(Q, Wq), proj(K, Wk), proj(V, Wv)
    out = [[0.0] * d for _ in range(q)]
    for a in range(h):
        for i in range(q):
            s = [scale * sum(Qt[i][a * dh + t] * Kt[j][a * dh + t] for t in range(dh)) for j in range(n)]
            if phi == "softmax":
                mx = max(s)
                e = [math.exp(x - mx) for x in s]
                z = sum(e)
                w = [x / z for x in e]
            else:
                w = [x / (1.0 + math.exp(-x)) / denom for x in s]
            for t in range(dh):
                out[i][a * dh + t] = sum(w[j] * Vt[j][a * dh + t] for j in range(n))
    return np.array(out)


def check_brute_force_all_paths():
    p = _problem(11, B=2, N=7, C=5, d=8, m=3)
    lens = [7, 4]
    h, scale = 2, 0.37
    W = (p["Wq"].tolist(), p["Wk"].tolist(), p["Wv"].tolist())
    mha = orc.mha_target_attention(p["T"], p["E"], lens, p["Wq"], p["Wk"], p["Wv"], h, scale)
    LP = orc.lime_link_history(p["E"], lens, p["L"], p["Wq"], p["Wk"], p["Wv"], h, scale)
    O = orc.lime_score_candidates(p["T"], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], h, scale)
    OT, OS = orc.lime_xor_history(p["E"], lens, p["L"], p["Wq"], p["Wk"], p["Wv"], h, 0.8)
    for b in range(2):
        Eb = p["E"][b, : lens[b]].tolist()
        Tb, Lb = p["T"][b].tolist(), p["L"].tolist()
        np.testing.assert_allclose(mha[b], _brute_attention(Tb, Eb, Eb, *W, h, scale, "softmax"), atol=1e-12)
        np.testing.assert_allclose(LP[b], _brute_attention(Lb, Eb, Eb, *W, h, scale, "softmax"), atol=1e-12)
        np.testing.assert_allclose(O[b], _brute_attention(Tb, Lb, LP[b].tolist(), *W, h, scale, "softmax"), atol=1e-12)
        np.testing.assert_allclose(OT[b], _brute_attention(Lb, Eb, Eb, *W, h, 0.8, "silu", denom=lens[b]), atol=1e-12)
        np.testing.assert_allclose(OS[b, : lens[b]], _brute_attention(Eb, Lb, Lb, *W, h, 0.8, "silu", denom=3),
                                   atol=1e-12)
        assert not OS[b, lens[b]:].any()


# ----------------------------------------------------------------------------- library routine

def check_against_torch_sdpa():
    import torch
    import torch.nn.functional as F

    p = _problem(5, B=2, N=33, C=9, d=16, m=6)
    h, scale = 4, 0.41
    t = {k: torch.tensor(v, dtype=torch.float64) for k, v in p.items()}

    def heads(x):  # [r, d] -> [h, r, d/h]
        return x.reshape(x.shape[0], h, -1).transpose(0, 1)

    def sdpa(Q, K, V):
        o = F.scaled_dot_product_attention(heads(Q @ t["Wq"]), heads(K @ t["Wk"]), heads(V @ t["Wv"]), scale=scale)
        return o.transpose(0, 1).reshape(Q.shape[0], -1).numpy()

    lens = [33, 20]
    LP = orc.lime_link_history(p["E"], lens, p["L"], p["Wq"], p["Wk"], p["Wv"], h, scale)
    O = orc.lime_score_candidates(p["T"], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], h, scale)
    A = orc.mha_target_attention(p["T"], p["E"], lens, p["Wq"], p["Wk"], p["Wv"], h, scale)
    for b in range(2):
        Eb = t["E"][b, : lens[b]]
        np.testing.assert_allclose(LP[b], sdpa(t["L"], Eb, Eb), atol=1e-12)
        np.testing.assert_allclose(O[b], sdpa(t["T"][b], t["L"], torch.tensor(LP[b])), atol=1e-12)
        np.testing.assert_allclose(A[b], sdpa(t["T"][b], Eb, Eb), atol=1e-12)


# ----------------------------------------------------------------------------- closed forms

def check_rows_sum_to_one():
    p = _problem(3, B=3, N=12, C=6, d=8, m=4)
    lens = [12, 5, 1]
    _, W = orc.lime_link_history(p["E"], lens, p["L"], p["Wq"], p["Wk"], p["Wv"], 2, 1.3, return_weights=True)
    for b, w in enumerate(W):
        assert w.shape == (2, 4, lens[b])
        np.testing.assert_allclose(w.sum(axis=-1), 1.0, atol=1e-14)
        assert (w >= 0).all()
    LP = _rand(4, 3, 4, 8)
    _, W = orc.lime_score_candidates(p["T"], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], 2, 1.3, return_weights=True)
    for w in W:
        np.testing.assert_allclose(w.sum(axis=-1), 1.0, atol=1e-14)
    # masked form of the primitive: masked keys get weight exactly zero, the rest sums to one
    M = np.zeros((4, 12), dtype=bool)
    M[:, :5] = True
    _, w = orc.mha(p["L"], p["E"][0], p["E"][0], M, p["Wq"], p["Wk"], p["Wv"], 2, 1.3, return_weights=True)
    assert not w[:, :, 5:].any()
    np.testing.assert_allclose(w.sum(axis=-1), 1.0, atol=1e-14)


def check_uniform_attention_closed_form():
    # W_Q = 0 makes every logit 0: softmax is uniform, so the output is the mean of the projected values.
    p = _problem(7, B=2, N=9, C=4, d=8, m=3)
    lens = [9, 6]
    Z = np.zeros((8, 8))
    LP = orc.lime_link_history(p["E"], lens, p["L"], Z, p["Wk"], p["Wv"], 2, 1.0)
    for b in range(2):
        mean_v = (p["E"][b, : lens[b]] @ p["Wv"]).mean(axis=0)
        np.testing.assert_allclose(LP[b], np.tile(mean_v, (3, 1)), atol=1e-13)
    LPin = _rand(8, 2, 3, 8)
    O = orc.lime_score_candidates(p["T"], p["L"], LPin, Z, p["Wk"], p["Wv"], 2, 1.0)
    for b in range(2):
        np.testing.assert_allclose(O[b], np.tile((LPin[b] @ p["Wv"]).mean(axis=0), (4, 1)), atol=1e-13)
    A = orc.mha_target_attention(p["T"], p["E"], lens, Z, p["Wk"], p["Wv"], 2, 1.0)
    for b in range(2):
        np.testing.assert_allclose(A[b], np.tile((p["E"][b, : lens[b]] @ p["Wv"]).mean(axis=0), (4, 1)), atol=1e-13)


def check_identity_links_reduce_to_values():
    # h = 1, d = N = m, E = L^C = c I, W_Q = W_K = I, scale c^2 >= 50: link i attends to item i only,
    # so L^P = E W_V; scoring candidates against those links (keys L = E, values L^P) is then the same
    # as full target attention over the history.
    n, c = 6, 8.0
    I = np.eye(n)
    E = (c * I)[None]
    Wv = _rand(9, n, n)
    LP = orc.lime_link_history(E, None, c * I, I, I, Wv, 1, 1.0)
    np.testing.assert_allclose(LP[0], c * Wv, atol=1e-12)
    T = _rand(10, 1, 5, n)
    Wq, Wk = _rand(12, n, n), _rand(13, n, n)
    # decoupled attention with keys = raw links (= E) and values = L^P, value projection already applied
    O = orc.lime_score_candidates(T, E[0], LP, Wq, Wk, None, 1, 0.3)
    A = orc.mha_target_attention(T, E, None, Wq, Wk, Wv, 1, 0.3)
    np.testing.assert_allclose(O, A, atol=1e-11)


def check_m_equals_n_reduces_to_target_attention():
    # Eq. 4 with L := E_b and L^P := E_b is Eq. 1 with K = V = E_b.
    p = _problem(21, B=1, N=10, C=7, d=8, m=10)
    O = orc.lime_score_candidates(p["T"], p["E"][0], p["E"], p["Wq"], p["Wk"], p["Wv"], 2, 0.6)
    A = orc.mha_target_attention(p["T"], p["E"], None, p["Wq"], p["Wk"], p["Wv"], 2, 0.6)
    np.testing.assert_allclose(O, A, atol=1e-13)


def check_permutations():
    p = _problem(31, B=1, N=11, C=8, d=8, m=4)
    h, s = 2, 0.9
    LP = orc.lime_link_history(p["E"], None, p["L"], p["Wq"], p["Wk"], p["Wv"], h, s)
    perm = np.random.default_rng(1).permutation(8)
    O = orc.lime_score_candidates(p["T"], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], h, s)
    Op = orc.lime_score_candidates(p["T"][:, perm], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], h, s)
    # per-row results must not depend on which other candidates are present
    np.testing.assert_allclose(Op, O[:, perm], rtol=0, atol=1e-15)
    one = orc.lime_score_candidates(p["T"][:, 3:4], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], h, s)
    np.testing.assert_allclose(one[0, 0], O[0, 3], rtol=0, atol=1e-15)
    # no positional term anywhere: permuting the history leaves the link states unchanged
    hperm = np.random.default_rng(2).permutation(11)
    LPp = orc.lime_link_history(p["E"][:, hperm], None, p["L"], p["Wq"], p["Wk"], p["Wv"], h, s)
    np.testing.assert_allclose(LPp, LP, atol=1e-13)
    OT, _ = orc.lime_xor_history(p["E"], None, p["L"], p["Wq"], p["Wk"], p["Wv"], h)
    OTp, OSp = orc.lime_xor_history(p["E"][:, hperm], None, p["L"], p["Wq"], p["Wk"], p["Wv"], h)
    np.testing.assert_allclose(OTp, OT, atol=1e-13)
    _, OS = orc.lime_xor_history(p["E"], None, p["L"], p["Wq"], p["Wk"], p["Wv"], h)
    np.testing.assert_allclose(OSp, OS[:, hperm], atol=1e-13)


# ----------------------------------------------------------------------------- XORA

def check_xor_truth_table():
    # Algorithm 1 for every (i, j): attend iff exactly one index is a source; normaliser = other side's size.
    for n_s, n_t in [(1, 1), (3, 2), (2, 5), (4, 4)]:
        n = n_s + n_t
        for i in range(n):
            for j in range(n):
                m, d = orc.xor_mask_and_denominator(i, j, n_s, n_t)
                src_q, src_k = i < n_s, j < n_s
                assert m == ((src_q and not src_k) or (src_k and not src_q))
                assert d == (n_t if src_q else n_s)
        M = np.array([[orc.xor_mask_and_denominator(i, j, n_s, n_t)[0] for j in range(n)] for i in range(n)])
        # block structure of Eq. 7: zero diagonal blocks, all-ones off-diagonal blocks, symmetric
        assert not M[:n_s, :n_s].any() and not M[n_s:, n_s:].any()
        assert M[:n_s, n_s:].all() and M[n_s:, :n_s].all()
        assert (M == M.T).all() and M.sum() == 2 * n_s * n_t


def check_xor_block_equals_quadratic():
    p = _problem(41, B=2, N=9, C=1, d=8, m=5)
    lens = [9, 3]
    for h in (1, 2, 4):
        OT, OS = orc.lime_xor_history(p["E"], lens, p["L"], p["Wq"], p["Wk"], p["Wv"], h, 0.7)
        for b in range(2):
            os_q, ot_q = orc.xora_quadratic(p["E"][b, : lens[b]], p["L"], p["Wq"], p["Wk"], p["Wv"], h, 0.7)
            np.testing.assert_allclose(OT[b], ot_q, atol=1e-13)
            np.testing.assert_allclose(OS[b, : lens[b]], os_q, atol=1e-13)


def check_xor_closed_forms():
    p = _problem(43, B=1, N=6, C=1, d=4, m=3)
    Z = np.zeros((4, 4))
    # all logits zero: SiLU(0) = 0, both outputs vanish
    OT, OS = orc.lime_xor_history(p["E"], None, p["L"], Z, p["Wk"], p["Wv"], 2)
    assert not OT.any() and not OS.any()
    # constant logit s: h = 1, every projected query and key equals u with <u, u> = s
    d, s = 4, 1.7
    u = np.full(d, math.sqrt(s / d))
    E = np.tile(u, (1, 6, 1))
    L = np.tile(u, (3, 1))
    I = np.eye(d)
    Wv = _rand(44, d, d)
    OT, OS = orc.lime_xor_history(E, None, L, I, I, Wv, 1)
    silu_s = s / (1.0 + math.exp(-s))
    np.testing.assert_allclose(OT[0], np.tile(silu_s * (u @ Wv), (3, 1)), atol=1e-13)  # SiLU(s) * mean(V[S])
    np.testing.assert_allclose(OS[0], np.tile(silu_s * (u @ Wv), (6, 1)), atol=1e-13)  # SiLU(s) * mean(V[T])
    # SiLU is not normalised: doubling the history with copies leaves O[T] unchanged (mean, not sum)
    E2 = np.concatenate([p["E"], p["E"]], axis=1)
    a, _ = orc.lime_xor_history(p["E"], None, p["L"], p["Wq"], p["Wk"], p["Wv"], 2)
    b, _ = orc.lime_xor_history(E2, None, p["L"], p["Wq"], p["Wk"], p["Wv"], 2)
    np.testing.assert_allclose(a, b, atol=1e-13)


def check_xor_zero_cross_dependence():
    # Appendix H.2: O[T] does not depend on Q[S], K[T], V[T]; O[S] not on Q[T], K[S], V[S].
    p = _problem(47, B=1, N=6, C=1, d=4, m=3)
    Eb, Lb = p["E"][0], p["L"]
    os0, ot0 = orc.xora_quadratic(Eb, Lb, p["Wq"], p["Wk"], p["Wv"], 2)

    def quad_with(Qx, Kx, Vx):
        # the quadratic form with separately perturbed query / key / value inputs, projections folded in
        n_s, n_t = 6, 3
        n = n_s + n_t
        M = np.array([[orc.xor_mask_and_denominator(i, j, n_s, n_t)[0] for j in range(n)] for i in range(n)])
        den = np.array([orc.xor_mask_and_denominator(i, 0, n_s, n_t)[1] for i in range(n)])
        O = orc.mha(Qx, Kx, Vx, M, p["Wq"], p["Wk"], p["Wv"], 2, 1.0, "silu", denom=den)
        return O[:n_s], O[n_s:]

    X = np.concatenate([Eb, Lb])
    bump_s = X.copy()
    bump_s[:6] += 1.0  # perturb the source rows only
    bump_t = X.copy()
    bump_t[6:] += 1.0  # perturb the target rows only
    _, ot = quad_with(bump_s, bump_t, bump_t)  # Q[S], K[T], V[T] changed
    np.testing.assert_array_equal(ot, ot0)
    os_, _ = quad_with(bump_t, bump_s, bump_s)  # Q[T], K[S], V[S] changed
    np.testing.assert_array_equal(os_, os0)
    # and the dependence that must be there is there
    _, ot = quad_with(X, bump_s, X)
    assert np.abs(ot - ot0).max() > 1e-3


# ----------------------------------------------------------------------------- masks / ragged

def check_ragged_masking():
    p = _problem(51, B=3, N=10, C=4, d=8, m=3)
    lens = [10, 4, 0]
    h, s = 2, 0.5
    clean = p["E"].copy()
    for b in range(3):
        clean[b, lens[b]:] = 0.0
    outs = []
    for poison in (0.0, np.nan, np.inf, 1e30):
        E = clean.copy()
        for b in range(3):
            E[b, lens[b]:] = poison
        LP = orc.lime_link_history(E, lens, p["L"], p["Wq"], p["Wk"], p["Wv"], h, s)
        OT, OS = orc.lime_xor_history(E, lens, p["L"], p["Wq"], p["Wk"], p["Wv"], h)
        A = orc.mha_target_attention(p["T"], E, lens, p["Wq"], p["Wk"], p["Wv"], h, s)
        outs.append((LP, OT, OS, A))
    for o in outs[1:]:
        for x, y in zip(o, outs[0]):
            np.testing.assert_array_equal(x, y)  # bit-identical whatever the padding holds
    LP, OT, OS, A = outs[0]
    assert np.isfinite(LP).all() and np.isfinite(OT).all() and np.isfinite(OS).all() and np.isfinite(A).all()
    # empty history: zeros, no NaN
    assert not LP[2].any() and not OT[2].any() and not OS[2].any() and not A[2].any()
    # padded O[S] rows are exact zeros
    assert not OS[1, 4:].any()
    # equals the result on truncated tensors
    LPt = orc.lime_link_history(clean[1:2, :4], None, p["L"], p["Wq"], p["Wk"], p["Wv"], h, s)
    np.testing.assert_array_equal(LPt[0], LP[1])
    # equals Eq. 1 with an explicit key mask inside the softmax on the zero-padded tensor
    M = np.zeros((3, 10), dtype=bool)
    M[:, :4] = True
    viaM = orc.mha(p["L"], clean[1], clean[1], M, p["Wq"], p["Wk"], p["Wv"], h, s)
    np.testing.assert_allclose(viaM, LP[1], atol=1e-14)
    # per-user links
    LCu = _rand(52, 3, 3, 8)
    LPu = orc.lime_link_history(clean, lens, LCu, p["Wq"], p["Wk"], p["Wv"], h, s)
    for b in range(2):
        one = orc.lime_link_history(clean[b:b + 1], lens[b:b + 1], LCu[b], p["Wq"], p["Wk"], p["Wv"], h, s)
        np.testing.assert_array_equal(one[0], LPu[b])


def check_softmax_is_shift_invariant_and_stable():
    # logits of a few hundred must not overflow; adding a constant to every logit changes nothing
    S = np.array([[700.0, 699.0, -800.0], [1e4, 1e4, 1e4]])
    A = orc.phi_softmax(S, np.ones_like(S, dtype=bool))
    e = math.exp(-1.0)
    np.testing.assert_allclose(A[0], [1 / (1 + e), e / (1 + e), 0.0], atol=1e-15)
    np.testing.assert_allclose(A[1], [1 / 3] * 3, atol=1e-15)


def check_qk_cache_path():
    # Section 3.3: looking the weights up and summing the personalised links is Eq. 4 itself
    p = _problem(61, B=2, N=5, C=9, d=8, m=4)
    LP = _rand(62, 2, 4, 8)
    h, s = 2, 0.8
    W = orc.qk_cache(p["T"], p["L"], p["Wq"], p["Wk"], h, s)
    assert W.shape == (2, 9, 2, 4)
    np.testing.assert_allclose(W.sum(axis=-1), 1.0, atol=1e-14)
    assert (W >= 0).all()
    direct = orc.lime_score_candidates(p["T"], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], h, s)
    np.testing.assert_allclose(orc.lime_score_candidates_cached(W, LP, p["Wv"], h), direct, atol=1e-13)
    # the cache does not depend on the user's link states or on W_V
    np.testing.assert_array_equal(W, orc.qk_cache(p["T"], p["L"], p["Wq"], p["Wk"], h, s))
    # hand case of the Eq. 4 fixture: logits [ln2, 0] -> weights [2/3, 1/3]; values [[3, 0], [0, 6]] -> [2, 2]
    g = _load("eq4_decoupled_candidates.json")
    Wg = orc.qk_cache(_arr(g["T"]), _arr(g["L"]), None, None, 1, 1.0)
    np.testing.assert_allclose(Wg[0, 0, 0], [2 / 3, 1 / 3], atol=1e-15)
    np.testing.assert_allclose(orc.lime_score_candidates_cached(Wg, _arr(g["LP"]), None, 1), _arr(g["O"]), atol=1e-14)
    # brute force of the weighted sum with scalar loops
    Vt = (LP[1] @ p["Wv"]).tolist()
    out = orc.lime_score_candidates_cached(W, LP, p["Wv"], h)
    for c in range(9):
        for col in range(8):
            a = col // 4
            want = sum(W[1, c, a, i] * Vt[i][col] for i in range(4))
            assert abs(out[1, c, col] - want) < 1e-13


def check_gathered_cache():
    # one cache for the corpus, candidates named by id: the same as scoring the gathered embeddings with Eq. 4
    p = _problem(71, B=1, N=3, C=11, d=8, m=4)  # T[0] plays the corpus of 11 items
    corpus = p["T"][0]
    LP = _rand(72, 3, 4, 8)
    h, s = 2, 0.7
    table = orc.qk_cache(corpus[None], p["L"], p["Wq"], p["Wk"], h, s)[0]
    ids = np.array([[0, 10, 3, 3, 7], [5, 5, 5, 1, 0], [9, 8, 2, 6, 4]])
    got = orc.lime_score_candidates_gathered(table, ids, LP, p["Wv"], h)
    want = orc.lime_score_candidates(corpus[ids], p["L"], LP, p["Wq"], p["Wk"], p["Wv"], h, s)
    np.testing.assert_allclose(got, want, atol=1e-13)
    # equal ids give equal rows; the identity gather is the ungathered stage
    np.testing.assert_array_equal(got[0, 2], got[0, 3])
    all_ids = np.tile(np.arange(11), (3, 1))
    np.testing.assert_allclose(orc.lime_score_candidates_gathered(table, all_ids, LP, p["Wv"], h),
                               orc.lime_score_candidates_cached(np.tile(table[None], (3, 1, 1, 1)), LP, p["Wv"], h), atol=1e-14)
    # ids outside the table: zero rows, the others untouched
    bad = ids.copy()
    bad[1, 2], bad[2, 0] = -1, 11
    out = orc.lime_score_candidates_gathered(table, bad, LP, p["Wv"], h)
    assert not out[1, 2].any() and not out[2, 0].any()
    mask = np.ones(ids.shape, bool)
    mask[1, 2] = mask[2, 0] = False
    np.testing.assert_array_equal(out[mask], got[mask])


def _layer_problem(seed, B=2, N=6, d=8, m=3, n=3):
    p = _problem(seed, B=B, N=N, d=d, m=m)
    r = np.random.default_rng(seed + 1)
    p["Wu"], p["Wo"] = r.standard_normal((n, d, d)) / 2, r.standard_normal((n, d, d)) / 2
    return p


def check_xor_layers_one_layer_from_scalars():
    """n = 1: L^P = (O[T] * SiLU(L^C Wu)) Wo with O[T] from the scalar brute force and the gate and the output
    layer written with math.exp and Python loops."""
    p = _layer_problem(51, n=1)
    lens, h, d = [6, 3], 2, 8
    LP = orc.lime_xor_layers(p["E"], lens, p["L"], p["Wq"], p["Wk"], p["Wv"], p["Wu"], p["Wo"], h, 0.7)
    W = (p["Wq"].tolist(), p["Wk"].tolist(), p["Wv"].tolist())
    Lb, Wu, Wo = p["L"].tolist(), p["Wu"][0].tolist(), p["Wo"][0].tolist()
    for b in range(2):
        Eb = p["E"][b, : lens[b]].tolist()
        OT = _brute_attention(Lb, Eb, Eb, *W, h, 0.7, "silu", denom=lens[b])
        for i in range(3):
            pre = [sum(Lb[i][k] * Wu[k][c] for k in range(d)) for c in range(d)]
            gated = [OT[i][c] * pre[c] / (1.0 + math.exp(-pre[c])) for c in range(d)]
            want = [sum(gated[k] * Wo[k][c] for k in range(d)) for c in range(d)]
            np.testing.assert_allclose(LP[b, i], want, atol=1e-12)


def check_xor_layers_block_equals_quadratic():
    """Three stacked layers in block form = the same three layers on the concatenated sequence with the full
    (n_s + n_t)^2 masked attention of Eq. 6 (the history rows of the last layer, which the block form skips,
    change nothing)."""
    p = _layer_problem(52)
    lens, h = [6, 4], 2
    LP = orc.lime_xor_layers(p["E"], lens, p["L"], p["Wq"], p["Wk"], p["Wv"], p["Wu"], p["Wo"], h, 0.9)
    for b in range(2):
        want = orc.xor_layers_quadratic(p["E"][b, : lens[b]], p["L"], p["Wq"], p["Wk"], p["Wv"], p["Wu"], p["Wo"], h, 0.9)
        np.testing.assert_allclose(LP[b], want, atol=1e-12)


def check_xor_layers_structure():
    """What Eq. 8 fixes whatever the gate is: the layers' link outputs are summed (scaling the last layer's output
    map scales exactly that layer's term); a zero gate projection gives SiLU(0) = 0 and no output; the first
    layer's term is the one-layer result; history rows enter only through sums over the history (permutation
    invariance); rows at or past lens[b] are never read; an empty history gives zeros."""
    p = _layer_problem(53)
    args = (p["Wq"], p["Wk"], p["Wv"])
    lens, h = [5, 6], 2
    f = lambda E, ln, Wu, Wo: orc.lime_xor_layers(E, ln, p["L"], *args, Wu, Wo, h, 0.8)  # noqa: E731
    base = f(p["E"], lens, p["Wu"], p["Wo"])
    Wo2, Wo0 = p["Wo"].copy(), p["Wo"].copy()
    Wo2[2] *= 2.0
    Wo0[2] *= 0.0
    np.testing.assert_allclose(f(p["E"], lens, p["Wu"], Wo2) - base, base - f(p["E"], lens, p["Wu"], Wo0), atol=1e-12)
    assert np.abs(base - f(p["E"], lens, p["Wu"], Wo0)).max() > 1e-3  # the third layer does contribute
    assert not f(p["E"], lens, np.zeros_like(p["Wu"]), p["Wo"]).any()
    # with the later layers' output maps at zero only the first layer's term is left
    Wo1 = p["Wo"].copy()
    Wo1[1:] = 0.0
    np.testing.assert_allclose(f(p["E"], lens, p["Wu"], Wo1), f(p["E"], lens, p["Wu"][:1], p["Wo"][:1]), atol=1e-12)
    # ... but the second layer does see the first one's output: its term differs from a one-layer run
    two = f(p["E"], lens, p["Wu"][:2], p["Wo"][:2]) - f(p["E"], lens, p["Wu"][:1], p["Wo"][:1])
    alone = f(p["E"], lens, p["Wu"][1:2], p["Wo"][1:2])
    assert np.abs(two - alone).max() > 1e-3
    perm = np.random.default_rng(3).permutation(5)
    Ep = p["E"].copy()
    Ep[0, :5] = p["E"][0, perm]
    np.testing.assert_allclose(f(Ep, lens, p["Wu"], p["Wo"])[0], base[0], atol=1e-12)
    Ebad = p["E"].copy()
    Ebad[0, 5:] = np.nan
    np.testing.assert_array_equal(f(Ebad, lens, p["Wu"], p["Wo"]), base)
    np.testing.assert_array_equal(f(p["E"][:, :5], [5, 5], p["Wu"], p["Wo"])[0], base[0])
    assert not f(p["E"], [0, 6], p["Wu"], p["Wo"])[0].any()


def _backward_problem(seed=11, B=2, N=5, m=4, d=6, lens=(5, 3)):
    rng = np.random.default_rng(seed)
    t = {k: rng.standard_normal((B, N, d)) for k in ("QS", "KS", "VS", "dOS")}
    t.update({k: rng.standard_normal((B, m, d)) for k in ("QT", "KT", "VT", "dOT")})
    t["lens"] = np.array(lens, dtype=np.int32)
    return t


def _xora_loss(t, h, scale):
    """sum(O[T] * dOT) + sum(O[S] * dOS) with the forward of Appendix H.1 from the oracle's own MHA (weights absent)."""
    loss = 0.0
    m = t["QT"].shape[1]
    for b, n_s in enumerate(t["lens"]):
        if n_s == 0:
            continue
        OT = orc.mha(t["QT"][b], t["KS"][b, :n_s], t["VS"][b, :n_s], None, None, None, None, h, scale, "silu",
                     denom=np.full(m, n_s))
        OS = orc.mha(t["QS"][b, :n_s], t["KT"][b], t["VT"][b], None, None, None, None, h, scale, "silu",
                     denom=np.full(n_s, m))
        loss += (OT * t["dOT"][b]).sum() + (OS * t["dOS"][b, :n_s]).sum()
    return loss


def check_xor_backward_against_finite_differences():
    """Appendix H.2: every entry of the six gradients equals the central difference of the scalar
    sum(O[T] dOT) + sum(O[S] dOS) through the (separately pinned) forward; padded rows get exactly zero."""
    h, scale = 2, 0.7
    t = _backward_problem()
    grads = dict(zip(("QS", "KS", "VS", "QT", "KT", "VT"),
                     orc.xor_attention_backward(t["QS"], t["KS"], t["VS"], t["QT"], t["KT"], t["VT"], t["dOT"], t["dOS"],
                                                t["lens"], h, scale)))
    eps = 1e-5
    for name, g in grads.items():
        for idx in np.ndindex(*g.shape):
            if name.endswith("S") and idx[1] >= t["lens"][idx[0]]:
                assert g[idx] == 0.0, (name, idx)
                continue
            keep = t[name][idx]
            t[name][idx] = keep + eps
            up = _xora_loss(t, h, scale)
            t[name][idx] = keep - eps
            down = _xora_loss(t, h, scale)
            t[name][idx] = keep
            np.testing.assert_allclose(g[idx], (up - down) / (2 * eps), rtol=2e-6, atol=2e-8, err_msg=f"d{name}{idx}")


def check_xor_backward_closed_forms_and_structure():
    """Zero queries: Z = 0, SiLU(0) = 0 and SiLU'(0) = 1/2, so dV = 0, dK = 0 and dQ = scale ((G V^T) / (2 n)) K.
    Without dOS the three gradients that only O[S] feeds are zero; the gradients are linear in the upstream ones;
    padded rows may hold anything."""
    h, scale = 3, 1.3
    t = _backward_problem(seed=5, d=6, lens=(4, 5))
    z = np.zeros_like
    dQS, dKS, dVS, dQT, dKT, dVT = orc.xor_attention_backward(z(t["QS"]), t["KS"], t["VS"], z(t["QT"]), t["KT"], t["VT"],
                                                              t["dOT"], t["dOS"], t["lens"], h, scale)
    for g in (dVS, dVT, dKS, dKT):
        assert not g.any()
    dh = 2
    for b, n_s in enumerate(t["lens"]):
        for a in range(h):
            c = slice(a * dh, (a + 1) * dh)
            want_t = scale * ((t["dOT"][b, :, c] @ t["VS"][b, :n_s, c].T) / (2 * n_s)) @ t["KS"][b, :n_s, c]
            want_s = scale * ((t["dOS"][b, :n_s, c] @ t["VT"][b, :, c].T) / (2 * 4)) @ t["KT"][b, :, c]
            np.testing.assert_allclose(dQT[b, :, c], want_t, atol=1e-12)
            np.testing.assert_allclose(dQS[b, :n_s, c], want_s, atol=1e-12)
    args = (t["QS"], t["KS"], t["VS"], t["QT"], t["KT"], t["VT"])
    full = orc.xor_attention_backward(*args, t["dOT"], t["dOS"], t["lens"], h, scale)
    only_t = orc.xor_attention_backward(*args, t["dOT"], None, t["lens"], h, scale)
    assert not only_t[0].any() and not only_t[4].any() and not only_t[5].any()
    only_s = orc.xor_attention_backward(*args, z(t["dOT"]), t["dOS"], t["lens"], h, scale)
    for f, a_, b_ in zip(full, only_t, only_s):
        np.testing.assert_allclose(f, a_ + b_, atol=1e-12)
    doubled = orc.xor_attention_backward(*args, 2 * t["dOT"], 2 * t["dOS"], t["lens"], h, scale)
    for f, g in zip(full, doubled):
        np.testing.assert_allclose(g, 2 * f, atol=1e-12)
    bad = [x.copy() for x in args] + [t["dOT"], t["dOS"].copy()]
    for x in (bad[0], bad[1], bad[2], bad[7]):
        x[0, 4:] = np.nan
    for f, g in zip(full, orc.xor_attention_backward(*bad, t["lens"], h, scale)):
        np.testing.assert_array_equal(f, g)
    assert not any(g[1].any() for g in orc.xor_attention_backward(*args, t["dOT"], t["dOS"], [4, 0], h, scale))


PINS = [
    check_xor_backward_against_finite_differences,
    check_xor_backward_closed_forms_and_structure,
    check_xor_layers_one_layer_from_scalars,
    check_xor_layers_block_equals_quadratic,
    check_xor_layers_structure,
    check_gathered_cache,
    check_golden_eq3,
    check_golden_eq4,
    check_golden_xora,
    check_golden_eq1_masked,
    check_brute_force_all_paths,
    check_against_torch_sdpa,
    check_rows_sum_to_one,
    check_uniform_attention_closed_form,
    check_identity_links_reduce_to_values,
    check_m_equals_n_reduces_to_target_attention,
    check_permutations,
    check_xor_truth_table,
    check_xor_block_equals_quadratic,
    check_xor_closed_forms,
    check_xor_zero_cross_dependence,
    check_ragged_masking,
    check_softmax_is_shift_invariant_and_stable,
    check_qk_cache_path,
]


@pytest.mark.parametrize("pin", PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()


# ----------------------------------------------------------------------------- planted mistakes

def _pins_that_fail():
    failed = []
    for pin in PINS:
        try:
            with np.errstate(all="ignore"):
                pin()
        except Exception:  # noqa: BLE001 - any failure counts as "caught"
            failed.append(pin.__name__)
    return failed


def _mut_project_transposed(X, W):
    X = np.asarray(X, dtype=np.float64)
    return X if W is None else X @ np.asarray(W, dtype=np.float64).T


def _mut_silu_wrong_sign(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(x))


def _mut_softmax_ignores_mask(S, M):
    S = np.asarray(S, dtype=np.float64)
    e = np.exp(S - S.max(axis=1, keepdims=True))
    return e / e.sum(axis=1, keepdims=True)


def _mut_softmax_mask_after(S, M):
    # Eq. 1 read literally for softmax: normalise over all keys, then zero the masked ones
    S = np.asarray(S, dtype=np.float64)
    with np.errstate(all="ignore"):
        S = np.nan_to_num(S, nan=0.0, posinf=0.0, neginf=0.0)
        e = np.exp(S - S.max(axis=1, keepdims=True))
    return np.where(M, e / e.sum(axis=1, keepdims=True), 0.0)


def _mut_phi_silu_unnormalised(S, M, denom):
    return np.where(M, _mut_free_silu(S), 0.0)


def _mut_free_silu(x):
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-x))


def _mut_xor_mask_and(n_s, n_t):
    # the formula printed beside Eq. 7 (a conjunction): both indices are sources
    src = np.arange(n_s + n_t) < n_s
    return src[:, None] & src[None, :], np.where(src, n_t, n_s).astype(np.float64)


def _mut_xor_same_side_denominator(n_s, n_t):
    src = np.arange(n_s + n_t) < n_s
    return src[:, None] != src[None, :], np.where(src, n_s, n_t).astype(np.float64)


def _make_mha_mutant(kind):
    real = orc.mha

    def mutant(Q, K, V, M, Wq, Wk, Wv, h, scale, phi="softmax", denom=None, return_weights=False):
        if kind == "no_heads":
            return real(Q, K, V, M, Wq, Wk, Wv, 1, scale, phi, denom, return_weights)
        if kind == "no_scale":
            return real(Q, K, V, M, Wq, Wk, Wv, h, 1.0, phi, denom, return_weights)
        if kind == "keys_from_values":
            return real(Q, V, V, M, Wq, Wk, Wv, h, scale, phi, denom, return_weights)
        if kind == "swap_wk_wv":
            return real(Q, K, V, M, Wq, Wv, Wk, h, scale, phi, denom, return_weights)
        raise AssertionError(kind)

    return mutant


def _mut_gate_without_silu(A, X, Wu, Wo):
    return orc.project(orc._f64(A) * orc.project(orc._f64(X), Wu), Wo)


def _mut_gate_from_attention(A, X, Wu, Wo):
    return orc.project(orc._f64(A) * orc.silu(orc.project(orc._f64(A), Wu)), Wo)


def _mut_gate_after_output(A, X, Wu, Wo):
    return orc.project(orc._f64(A), Wo) * orc.silu(orc.project(orc._f64(X), Wu))


def _make_layers_mutant(kind):
    def mutant(E, lens, LC, Wq, Wk, Wv, Wu, Wo, h, scale=1.0):
        E = orc._f64(E)
        B, N, d = E.shape
        lens_ = orc._lens(lens, B, N)
        m = orc._links_of_user(LC, 0).shape[0]
        LP = np.zeros((B, m, d))
        for b in range(B):
            n_s = int(lens_[b])
            if n_s == 0:
                continue
            Xs, Xt = E[b, :n_s], orc._f64(orc._links_of_user(LC, b))
            for j in range(len(Wu)):
                OT = orc.mha(Xt, Xs, Xs, None, Wq, Wk, Wv, h, scale, "silu", denom=np.full(m, n_s))
                OS = orc.mha(Xs, Xt, Xt, None, Wq, Wk, Wv, h, scale, "silu", denom=np.full(n_s, m))
                Yt, Ys = orc.gated_mlp(OT, Xt, Wu[j], Wo[j]), orc.gated_mlp(OS, Xs, Wu[j], Wo[j])
                if kind == "last_layer_only":
                    LP[b] = Yt
                else:
                    LP[b] += Yt
                if kind == "no_residual":
                    Xs, Xt = Ys, Yt
                elif kind == "links_not_updated":
                    Xs = Xs + Ys
                else:
                    Xs, Xt = Xs + Ys, Xt + Yt
        return LP

    mutant.__name__ = f"layers_{kind}"
    return mutant


def _mut_sigmoid_derivative(x):
    x = np.asarray(x, dtype=np.float64)
    s = 1.0 / (1.0 + np.exp(-x))
    return s * (1.0 - s)


def _mut_silu_derivative_without_sigmoid_factor(x):
    x = np.asarray(x, dtype=np.float64)
    s = 1.0 / (1.0 + np.exp(-x))
    return s * (1.0 - s) * (1.0 + x)


def _make_backward_mutant(kind):
    real = orc.xor_attention_backward

    def mutant(QS, KS, VS, QT, KT, VT, dOT, dOS, lens, h, scale=1.0):
        dQS, dKS, dVS, dQT, dKT, dVT = real(QS, KS, VS, QT, KT, VT, dOT, dOS, lens, h, scale)
        if kind == "queries_without_scale":
            return dQS / scale, dKS, dVS, dQT / scale, dKT, dVT
        if kind == "directions_swapped":  # each direction's key/value gradients land on the other side's tensors
            return real(QT, KT, VT, QS, KS, VS, dOS, dOT, None, h, scale)[3:] + real(QT, KT, VT, QS, KS, VS, dOS, dOT, None, h, scale)[:3]
        if kind == "padding_counted":
            return real(QS, KS, VS, QT, KT, VT, dOT, dOS, None, h, scale)
        raise ValueError(kind)

    mutant.__name__ = f"backward_{kind}"
    return mutant


MUTATIONS = [
    ("silu_derivative", _mut_sigmoid_derivative),
    ("silu_derivative", _mut_silu_derivative_without_sigmoid_factor),
    ("xor_attention_backward", _make_backward_mutant("queries_without_scale")),
    ("xor_attention_backward", _make_backward_mutant("directions_swapped")),
    ("xor_attention_backward", _make_backward_mutant("padding_counted")),
    ("lime_xor_layers", _make_layers_mutant("no_residual")),
    ("lime_xor_layers", _make_layers_mutant("last_layer_only")),
    ("lime_xor_layers", _make_layers_mutant("links_not_updated")),
    ("gated_mlp", _mut_gate_without_silu),
    ("gated_mlp", _mut_gate_from_attention),
    ("gated_mlp", _mut_gate_after_output),
    ("project", _mut_project_transposed),
    ("silu", _mut_silu_wrong_sign),
    ("phi_softmax", _mut_softmax_ignores_mask),
    ("phi_softmax", _mut_softmax_mask_after),
    ("phi_silu", _mut_phi_silu_unnormalised),
    ("xor_mask", _mut_xor_mask_and),
    ("xor_mask", _mut_xor_same_side_denominator),
    ("mha", "no_heads"),
    ("mha", "no_scale"),
    ("mha", "keys_from_values"),
    ("mha", "swap_wk_wv"),
]


@pytest.mark.parametrize("name,mutant", MUTATIONS, ids=[f"{n}:{getattr(m, '__name__', m)}" for n, m in MUTATIONS])
def test_planted_mistake_is_caught(monkeypatch, name, mutant):
    """A plausible mistake planted in the oracle (on the CPU) must fail at least one pin."""
    assert _pins_that_fail() == []
    if isinstance(mutant, str):
        mutant = _make_mha_mutant(mutant)
    monkeypatch.setattr(orc, name, mutant)
    assert _pins_that_fail(), f"mutation {name} survived every pin"
