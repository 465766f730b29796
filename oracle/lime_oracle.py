"""CPU oracle for the LIME inference hot path (arXiv 2510.18239).

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check
and the benchmark's ``cpu_baseline`` leg may import it.  It shares no code with
the HIP library and never imports it.

Everything is evaluated in float64 with numpy, un-fused and un-blocked, in the
order and notation of the paper, so that it can be checked against the paper by
eye.  Inputs are whatever values the caller hands over (bf16-rounded or fp32
values are simply up-cast; no rounding happens in here).

Notation (Appendix A): E history [N, d]; T candidates [C, d]; L raw links
[m, d]; L^C contextualised links; L^P personalised links; theta = {W_Q, W_K,
W_V}, each [d, d] and applied on the right (X~ = X W, Section 3.1, Eq. 1).

Readings of points the paper leaves open (each is repeated where it is used):
  * heads: the d projected columns are cut into h contiguous blocks of d/h; the
    heads are independent and their outputs are concatenated; there is no
    output projection because theta holds only W_Q, W_K, W_V (Eq. 1).
  * "scaled softmax": the logit scale is an explicit argument.
  * ragged histories: a user's result is the result on that user's first
    len_b history rows only; equivalently the mask is applied inside the
    softmax (masked positions take part in neither the maximum nor the sum).
    For phi = SiLU this coincides with Eq. 1's Hadamard mask.
  * an empty history (len_b = 0) gives all-zero link states.
  * XORA: phi(s) = SiLU(s) / (size of the opposite partition) (Appendix I,
    Algorithm 1 and the masking line of Algorithm 2); the mask is the
    exclusive-or of "query is source" and "key is source" (Algorithm 1), which
    is also what Eq. 7 and Appendix H.1 state.

  * stacked XOR layers (Eq. 8): GatedMLP(A; eta)(X) = (A * SiLU(X Wu)) Wo,
    eta = (Wu, Wo), the pointwise gating of the block Eq. 5 summarises without
    its normalisation; the layers form a residual stream X_{j+1} = X_j + Y_j;
    one theta for all layers, eta_j per layer.  The paper defines neither the
    block nor the stacking beyond Eq. 8 and the notation table: this is an
    assumption, and what is pinned below is the arithmetic of this reading.

  * XORA backward (Appendix H.2): the gradients of O = phi(Q K^T) V with the
    factor phi'(Q K^T) applied element-wise (the appendix prints it like a
    matrix factor) and SiLU' written out as the derivative of x sigmoid(x)
    (the expression in the listing of Algorithm 3 is not that derivative).

  * the scoring pipeline around the two attention stages (Appendix C "Model Design", Eq. 2, Section 3.3), for
    which the paper gives names and sizes only:  layer normalisation is the standard one over the d features of a
    row (biased variance, eps inside the square root, learnable scale gamma and shift beta), applied to every
    tensor that enters an MHA, once per tensor and role: the query-side tensor, the key-side tensor and the
    value-side tensor each have their own (gamma, beta), and where keys and values are the same tensor (the
    history in Eq. 3) one normalisation serves both;  Eq. 2's MLP is two affine maps with a ReLU between them,
    applied to each link row concatenated with the user's context vector;  the interaction network is an MLP
    with ReLU after every hidden layer and a last affine map to one logit per candidate, fed with the LIME
    embedding alone.  The arithmetic of these readings is pinned; whether they are the authors' is not ("parity
    unpinned" as to the reading).

Pinned by tests/test_oracle_*.py (closed forms, brute force, a library routine,
invariants, hand-derived fixtures).  Unpinned: the paper's claim that LIME
approximates full target attention (Appendix D), which needs trained links and
is not tested ("parity unpinned"); and whether the reading of GatedMLP and of
"stacking" above is the authors' (lime_xor_layers: "parity unpinned" as to the
reading; its arithmetic is pinned by scalar loops, the quadratic expansion and
the invariants Eq. 8 fixes).
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "project",
    "silu",
    "phi_softmax",
    "phi_silu",
    "mha",
    "xor_mask",
    "xor_mask_and_denominator",
    "lime_link_history",
    "lime_xor_history",
    "xora_quadratic",
    "silu_derivative",
    "xor_attention_backward",
    "gated_mlp",
    "lime_xor_layers",
    "xor_layers_quadratic",
    "lime_score_candidates",
    "mha_target_attention",
    "qk_cache",
    "lime_score_candidates_cached",
    "layer_norm",
    "relu",
    "contextualize_links",
    "interaction_mlp",
    "lime_scores",
]


def _f64(x):
    return None if x is None else np.asarray(x, dtype=np.float64)


def project(X, W):
    """X~ = X W (Eq. 1).  ``W is None`` stands for the identity."""
    X = _f64(X)
    if W is None:
        return X
    return X @ _f64(W)


def silu(x):
    """SiLU(x) = x * sigmoid(x) = x / (1 + exp(-x))."""
    x = _f64(x)
    return x / (1.0 + np.exp(-x))


def phi_softmax(S, M):
    """Row-wise softmax of S over the positions where M is true.

    Masked positions get weight 0 and take part in neither the maximum nor the
    sum, so every row with at least one valid position sums to 1.  A row with
    no valid position gets all-zero weights (reading for an empty history).
    """
    S = _f64(S)
    M = np.asarray(M, dtype=bool)
    with np.errstate(invalid="ignore", over="ignore"):
        row_max = np.where(M, S, -np.inf).max(axis=1, keepdims=True, initial=-np.inf)
        row_max = np.where(np.isfinite(row_max), row_max, 0.0)
        e = np.where(M, np.exp(S - row_max), 0.0)
    row_sum = e.sum(axis=1, keepdims=True)
    return e / np.where(row_sum > 0.0, row_sum, 1.0)


def phi_silu(S, M, denom):
    """S[i,j] <- M[i,j] ? SiLU(S[i,j]) / denom[i] : 0 (Algorithm 2's masking step).

    ``denom`` holds one normaliser per query row (Algorithm 1's d).
    """
    S = _f64(S)
    M = np.asarray(M, dtype=bool)
    denom = _f64(denom).reshape(-1, 1)
    with np.errstate(divide="ignore", invalid="ignore"):
        A = silu(S) / denom
    return np.where(M, A, 0.0)


def mha(Q, K, V, M, Wq, Wk, Wv, h, scale, phi="softmax", denom=None, return_weights=False):
    """MHA(Q, K, V; M; theta) of Eq. 1, with h heads.

    Q [q, d]; K, V [n, d]; M boolean [q, n] (None = the all-ones mask J).
    phi = "softmax": weights = softmax over the unmasked keys of scale * Q~ K~^T.
    phi = "silu":    weights = M ? SiLU(scale * Q~ K~^T) / denom[row] : 0.
    Returns [q, d] (and the per-head weights [h, q, n] on request).
    """
    Qt, Kt, Vt = project(Q, Wq), project(K, Wk), project(V, Wv)
    q, d = Qt.shape
    n = Kt.shape[0]
    assert d % h == 0
    dh = d // h
    if M is None:
        M = np.ones((q, n), dtype=bool)
    out = np.zeros((q, d))
    weights = np.zeros((h, q, n)) if return_weights else None
    for a in range(h):
        cols = slice(a * dh, (a + 1) * dh)
        S = scale * (Qt[:, cols] @ Kt[:, cols].T)
        if phi == "softmax":
            A = phi_softmax(S, M)
        elif phi == "silu":
            A = phi_silu(S, M, denom)
        else:
            raise ValueError(phi)
        if return_weights:
            weights[a] = A
        out[:, cols] = A @ Vt[:, cols]
    return (out, weights) if return_weights else out


def xor_mask(n_s, n_t):
    """M_xor and the per-row normaliser of XORA over X = source (+) target (Eq. 6-7).

    Eq. 7 splits the attention into the two off-diagonal blocks, source queries x target keys and target queries x
    source keys; nothing attends within its own partition.  So with ``is_source`` marking the first n_s of the
    n_s + n_t positions, M[i, j] is true exactly where the two positions lie in different partitions, and a row is
    normalised by the number of keys it can see: the size of the other partition (the "d" of Appendix I).
    Returns (M [n, n] bool, denom [n]).
    """
    is_source = np.arange(n_s + n_t) < n_s
    M = is_source[:, None] != is_source[None, :]
    denom = np.where(is_source, n_t, n_s).astype(np.float64)
    return M, denom


def xor_mask_and_denominator(i, j, n_s, n_t):
    """Entry (i, j) of M_xor and the normaliser of row i (see xor_mask): what Algorithm 1 returns for one pair."""
    M, denom = xor_mask(n_s, n_t)
    return bool(M[i, j]), int(denom[i])


def _lens(lens, B, N):
    if lens is None:
        return np.full(B, N, dtype=np.int64)
    lens = np.asarray(lens, dtype=np.int64)
    assert lens.shape == (B,) and (lens >= 0).all() and (lens <= N).all()
    return lens


def _links_of_user(LC, b):
    LC = _f64(LC)
    return LC if LC.ndim == 2 else LC[b]


def lime_link_history(E, lens, LC, Wq, Wk, Wv, h, scale, return_weights=False):
    """L^P = MHA(L^C, E, E; J; theta) per user (Eq. 3), phi = scaled softmax.

    E [B, N, d]; lens [B] or None; LC [m, d] (shared) or [B, m, d].
    User b sees only E[b, :lens[b]].  Returns [B, m, d].
    """
    E = _f64(E)
    B, N, d = E.shape
    lens = _lens(lens, B, N)
    m = _links_of_user(LC, 0).shape[0]
    LP = np.zeros((B, m, d))
    W = []
    for b in range(B):
        Eb = E[b, : lens[b]]
        if lens[b] == 0:
            W.append(np.zeros((h, m, 0)))
            continue
        r = mha(_links_of_user(LC, b), Eb, Eb, None, Wq, Wk, Wv, h, scale, "softmax", return_weights=return_weights)
        if return_weights:
            LP[b], w = r
            W.append(w)
        else:
            LP[b] = r
    return (LP, W) if return_weights else LP


def lime_xor_history(E, lens, LC, Wq, Wk, Wv, h, scale=1.0, want_os=True):
    """One XORA layer in its block form (Eq. 7, Appendix H.1).

    With source = history (n_s = lens[b] rows) and target = links (n_t = m):
      O[T] = phi(Q[T] K[S]^T) V[S],  phi = SiLU / n_s   -> the link states [B, m, d]
      O[S] = phi(Q[S] K[T]^T) V[T],  phi = SiLU / n_t   -> [B, N, d], rows >= lens[b] zero
    All six projections use the one theta of Eq. 6.  ``scale`` multiplies the
    logits before SiLU (Algorithm 2 uses none, i.e. 1.0).
    """
    E = _f64(E)
    B, N, d = E.shape
    lens = _lens(lens, B, N)
    m = _links_of_user(LC, 0).shape[0]
    OT = np.zeros((B, m, d))
    OS = np.zeros((B, N, d)) if want_os else None
    for b in range(B):
        n_s, n_t = int(lens[b]), m
        if n_s == 0:
            continue
        Eb, Lb = E[b, :n_s], _links_of_user(LC, b)
        OT[b] = mha(Lb, Eb, Eb, None, Wq, Wk, Wv, h, scale, "silu", denom=np.full(n_t, n_s))
        if want_os:
            OS[b, :n_s] = mha(Eb, Lb, Lb, None, Wq, Wk, Wv, h, scale, "silu", denom=np.full(n_s, n_t))
    return OT, OS


def xora_quadratic(Eb, Lb, Wq, Wk, Wv, h, scale=1.0):
    """XORA(X, X, X; theta) = MHA(X, X, X; M_xor; theta), X = E (+) L^C (Eq. 6).

    The full (n_s + n_t)^2 score matrix is formed and masked with M_xor (xor_mask).  One user; Eb holds that user's n_s valid rows.
    Returns (O[S] [n_s, d], O[T] [n_t, d]).
    """
    Eb, Lb = _f64(Eb), _f64(Lb)
    n_s, n_t = Eb.shape[0], Lb.shape[0]
    n = n_s + n_t
    X = np.concatenate([Eb, Lb], axis=0)
    M, denom = xor_mask(n_s, n_t)
    O = mha(X, X, X, M, Wq, Wk, Wv, h, scale, "silu", denom=denom)
    return O[:n_s], O[n_s:]


def silu_derivative(x):
    """d/dx [x sigmoid(x)] = sigmoid(x) (1 + x (1 - sigmoid(x))).

    (The expression printed in the listing of the backward kernel, Algorithm 3, is not this derivative; the
    derivation of Appendix H.2 only needs phi', which is what is written here.)
    """
    x = _f64(x)
    s = 1.0 / (1.0 + np.exp(-x))
    return s * (1.0 + x * (1.0 - s))


def xor_attention_backward(QS, KS, VS, QT, KT, VT, dOT, dOS, lens, h, scale=1.0):
    """Gradients of one XORA layer with respect to its projected inputs (Appendix H.2).

    Forward (Appendix H.1), per user and head, S = source (history rows, n_s = lens[b] valid), T = target
    (links, n_t = m), phi = SiLU(scale .) / n:
      O[T] = phi(Q[T] K[S]^T) V[S]   (normaliser n_s),      O[S] = phi(Q[S] K[T]^T) V[T]   (normaliser n_t).
    O[T] does not depend on Q[S], K[T], V[T] and O[S] not on Q[T], K[S], V[S], so each direction contributes to three
    gradients.  Written for O = phi(Q K^T) V with upstream gradient G = dL/dO and Z = scale Q K^T:
      dL/dV = phi(Z)^T G,     D = (G V^T) * phi'(Z)  (element-wise),     dL/dQ = scale D K,     dL/dK = scale D^T Q,
    phi'(Z) = SiLU'(Z) / n.  (Appendix H.2 prints these with phi' as if it were a matrix factor; the products of its
    total differentials are element-wise in phi', which is the reading taken.)

    QS, KS, VS [B, N, d]; QT, KT, VT [B, m, d]; dOT [B, m, d]; dOS [B, N, d] or None (O[S] unused downstream);
    rows >= lens[b] of the source tensors take no part and get zero gradients.
    Returns dQS, dKS, dVS [B, N, d], dQT, dKT, dVT [B, m, d].
    """
    QS, KS, VS, QT, KT, VT, dOT = (_f64(x) for x in (QS, KS, VS, QT, KT, VT, dOT))
    dOS = None if dOS is None else _f64(dOS)
    B, N, d = QS.shape
    m = QT.shape[1]
    dh = d // h
    lens = _lens(lens, B, N)
    dQS, dKS, dVS = np.zeros((B, N, d)), np.zeros((B, N, d)), np.zeros((B, N, d))
    dQT, dKT, dVT = np.zeros((B, m, d)), np.zeros((B, m, d)), np.zeros((B, m, d))
    for b in range(B):
        n_s, n_t = int(lens[b]), m
        if n_s == 0:
            continue
        for a in range(h):
            c = slice(a * dh, (a + 1) * dh)
            qs, ks, vs = QS[b, :n_s, c], KS[b, :n_s, c], VS[b, :n_s, c]
            qt, kt, vt = QT[b, :, c], KT[b, :, c], VT[b, :, c]
            # O[T]: the links attend over the history
            G = dOT[b, :, c]
            Z = scale * (qt @ ks.T)
            D = (G @ vs.T) * silu_derivative(Z) / n_s
            dVS[b, :n_s, c] = (silu(Z) / n_s).T @ G
            dQT[b, :, c] = scale * (D @ ks)
            dKS[b, :n_s, c] = scale * (D.T @ qt)
            if dOS is None:
                continue
            # O[S]: the history attends back to the links
            G = dOS[b, :n_s, c]
            Z = scale * (qs @ kt.T)
            D = (G @ vt.T) * silu_derivative(Z) / n_t
            dVT[b, :, c] = (silu(Z) / n_t).T @ G
            dQS[b, :n_s, c] = scale * (D @ kt)
            dKT[b, :, c] = scale * (D.T @ qs)
    return dQS, dKS, dVS, dQT, dKT, dVT


def gated_mlp(A, X, Wu, Wo):
    """GatedMLP(A; eta) of an interaction layer (Eq. 5, Eq. 8; the notation table calls it an MLP block that learns
    a gated element-wise product).  The paper gives no formula; the reading taken here is the pointwise gating of
    the block Eq. 5 summarises (HSTU): the attention output A is multiplied element-wise by a gate computed from
    the layer's own input rows, U = SiLU(X Wu), and mapped by a linear output layer:  Y = (A * U) Wo,
    eta = (Wu, Wo), without that block's normalisation (no LayerNorm on this path).

    A, X [rows, d]; Wu, Wo [d, d].  Returns [rows, d].
    """
    A, X = _f64(A), _f64(X)
    return project(A * silu(project(X, Wu)), Wo)


def lime_xor_layers(E, lens, LC, Wq, Wk, Wv, Wu, Wo, h, scale=1.0):
    """L^P of LIME-XOR with n stacked XOR layers (Eq. 8):  L^P = sum_j GatedMLP(XORA(X_j); eta_j) restricted to
    the link rows, X_1 = E (+) L^C.

    Per layer j: A = XORA(X_j, X_j, X_j; theta) in its block form (Eq. 7: the links attend over the valid history
    rows, the history rows over the links, SiLU with Algorithm 1's normalisers), Y_j = GatedMLP(A; eta_j) row by
    row, and - the reading taken for "stacking" - the next layer's input is the residual stream
    X_{j+1} = X_j + Y_j, as in the block of Eq. 5.  One theta for all layers, as Eq. 8 writes it; eta_j per layer.
    The history rows of the last layer feed nothing and are not computed.  A user without history gets zeros.

    E [B, N, d]; LC [m, d] or [B, m, d]; Wu, Wo [n, d, d].  Returns [B, m, d].
    """
    E = _f64(E)
    B, N, d = E.shape
    lens = _lens(lens, B, N)
    Wu, Wo = _f64(Wu), _f64(Wo)
    n_layers = Wu.shape[0]
    m = _links_of_user(LC, 0).shape[0]
    LP = np.zeros((B, m, d))
    for b in range(B):
        n_s, n_t = int(lens[b]), m
        if n_s == 0:
            continue
        Xs, Xt = E[b, :n_s], _f64(_links_of_user(LC, b))
        for j in range(n_layers):
            OT = mha(Xt, Xs, Xs, None, Wq, Wk, Wv, h, scale, "silu", denom=np.full(n_t, n_s))
            Yt = gated_mlp(OT, Xt, Wu[j], Wo[j])
            LP[b] += Yt
            if j + 1 < n_layers:
                OS = mha(Xs, Xt, Xt, None, Wq, Wk, Wv, h, scale, "silu", denom=np.full(n_s, n_t))
                Xs = Xs + gated_mlp(OS, Xs, Wu[j], Wo[j])
                Xt = Xt + Yt
    return LP


def xor_layers_quadratic(Eb, Lb, Wq, Wk, Wv, Wu, Wo, h, scale=1.0):
    """Eq. 8 for one user on the concatenated sequence: every layer runs the full masked (n_s + n_t)^2 attention of
    Eq. 6 (xora_quadratic), the gate and the output layer act on all rows, the stream is X + Y.  Returns the sum
    over the layers of the link rows of Y [n_t, d]."""
    Xs, Xt = _f64(Eb), _f64(Lb)
    n_s = Xs.shape[0]
    Wu, Wo = _f64(Wu), _f64(Wo)
    total = np.zeros_like(Xt)
    for j in range(Wu.shape[0]):
        OS, OT = xora_quadratic(Xs, Xt, Wq, Wk, Wv, h, scale)
        Y = gated_mlp(np.concatenate([OS, OT], axis=0), np.concatenate([Xs, Xt], axis=0), Wu[j], Wo[j])
        total += Y[n_s:]
        Xs, Xt = Xs + Y[:n_s], Xt + Y[n_s:]
    return total


def lime_score_candidates(T, L, LP, Wq, Wk, Wv, h, scale, return_weights=False):
    """O = MHA(T, L, L^P; J; theta) per user (Eq. 4): keys are the raw links L,
    values the personalised links L^P, phi = scaled softmax over the m links.

    T [B, C, d]; L [m, d]; LP [B, m, d].  Any of Wq, Wk, Wv may be None
    (identity), which gives the literal phi(T L^t) L^P.  Returns [B, C, d].
    """
    T, LP = _f64(T), _f64(LP)
    B, C, d = T.shape
    O = np.zeros((B, C, d))
    W = []
    for b in range(B):
        r = mha(T[b], L, LP[b], None, Wq, Wk, Wv, h, scale, "softmax", return_weights=return_weights)
        if return_weights:
            O[b], w = r
            W.append(w)
        else:
            O[b] = r
    return (O, W) if return_weights else O


def mha_target_attention(T, E, lens, Wq, Wk, Wv, h, scale):
    """Full target attention MHA(T, E, E; M; theta) per user (Eq. 1 with the
    candidates as queries and the history as keys and values; the "MHA
    skyline" of Section 4.1).  M masks history rows >= lens[b].

    T [B, C, d]; E [B, N, d].  Returns [B, C, d]; a user with an empty history
    gets zeros.
    """
    T, E = _f64(T), _f64(E)
    B, C, d = T.shape
    lens = _lens(lens, B, E.shape[1])
    O = np.zeros((B, C, d))
    for b in range(B):
        if lens[b] == 0:
            continue
        Eb = E[b, : lens[b]]
        O[b] = mha(T[b], Eb, Eb, None, Wq, Wk, Wv, h, scale, "softmax")
    return O


def qk_cache(T, L, Wq, Wk, h, scale):
    """The user-independent attention weights phi(T L^t) of Eq. 4 (the "QK cache" of Section 3.3):
    W[b, c, a, i] = softmax over the m links i of scale * <(T[b, c] W_Q)_a, (L W_K)[i]_a>.

    T [B, C, d]; L [m, d].  Returns [B, C, h, m].
    """
    T = _f64(T)
    B, C, d = T.shape
    Kt = project(L, Wk)
    m = Kt.shape[0]
    dh = d // h
    W = np.zeros((B, C, h, m))
    for b in range(B):
        Qt = project(T[b], Wq)
        for a in range(h):
            cols = slice(a * dh, (a + 1) * dh)
            S = scale * (Qt[:, cols] @ Kt[:, cols].T)
            W[b, :, a, :] = phi_softmax(S, np.ones_like(S, dtype=bool))
    return W


def lime_score_candidates_cached(W, LP, Wv, h):
    """Online half of the three-stage inference of Section 3.3: the cached weights are looked up and the
    interaction is a weighted sum of the personalised links, O[b, c, head a] = sum_i W[b, c, a, i] (L^P[b] W_V)[i, head a].

    W [B, C, h, m]; LP [B, m, d].  Returns [B, C, d].
    """
    W, LP = _f64(W), _f64(LP)
    B, C, _, m = W.shape
    d = LP.shape[2]
    dh = d // h
    O = np.zeros((B, C, d))
    for b in range(B):
        Vt = project(LP[b], Wv)
        for a in range(h):
            cols = slice(a * dh, (a + 1) * dh)
            O[b][:, cols] = W[b, :, a, :] @ Vt[:, cols]
    return O


def lime_score_candidates_gathered(Wtable, ids, LP, Wv, h):
    """The online stage of Section 3.3 when the cached weights are one table for the whole item corpus and a
    request names its candidates by id: O[b, c] is the weighted sum of user b's projected link states with the
    weights in row ids[b, c] of the table; an id outside the table gives a zero row.

    Wtable [n_items, h, m]; ids [B, C] integers; LP [B, m, d].  Returns [B, C, d].
    """
    Wtable, LP = _f64(Wtable), _f64(LP)
    ids = np.asarray(ids)
    n_items, _, m = Wtable.shape
    B, C = ids.shape
    d = LP.shape[2]
    dh = d // h
    O = np.zeros((B, C, d))
    for b in range(B):
        Vt = project(LP[b], Wv)
        for c in range(C):
            i = int(ids[b, c])
            if not 0 <= i < n_items:
                continue
            for a in range(h):
                O[b, c, a * dh:(a + 1) * dh] = Wtable[i, a] @ Vt[:, a * dh:(a + 1) * dh]
    return O


# ----------------------------------------------------------------------------- the scoring pipeline around the attention stages

def layer_norm(X, gamma, beta, eps=1e-5):
    """Layer normalisation of every row of X over its last axis (Appendix C, "Model Design": applied before the
    Q, K, V projections):  y = (x - mean(x)) / sqrt(var(x) + eps) * gamma + beta, with the biased variance.

    ``gamma`` / ``beta`` [d] (None = 1 / 0).  Rows holding NaN (padding) give NaN rows, which nothing reads.
    """
    X = _f64(X)
    with np.errstate(invalid="ignore"):
        mean = X.mean(axis=-1, keepdims=True)
        var = ((X - mean) ** 2).mean(axis=-1, keepdims=True)
        Y = (X - mean) / np.sqrt(var + eps)
    if gamma is not None:
        Y = Y * _f64(gamma)
    if beta is not None:
        Y = Y + _f64(beta)
    return Y


def relu(x):
    return np.maximum(_f64(x), 0.0)


def contextualize_links(L, EC, W1, b1, W2, b2):
    """Link contextualisation, Eq. 2:  L^C = MLP(L (+) E^C) per user.

    L [m, d] raw links (shared by all users); EC [B, dc] one context vector per user.  Every link row is
    concatenated with the user's context vector ([m, d + dc]) and sent through the MLP, read as
    ReLU(X W1 + b1) W2 + b2 with W1 [d + dc, dhid], W2 [dhid, d].  Returns [B, m, d].
    """
    L, EC = _f64(L), _f64(EC)
    m, d = L.shape
    B = EC.shape[0]
    LC = np.zeros((B, m, d))
    for b in range(B):
        X = np.concatenate([L, np.broadcast_to(EC[b], (m, EC.shape[1]))], axis=1)
        LC[b] = relu(X @ _f64(W1) + _f64(b1)) @ _f64(W2) + _f64(b2)
    return LC


def interaction_mlp(O, weights, biases):
    """The shallow interaction network of Section 3.3 on the LIME embeddings: hidden layers x <- ReLU(x W_i + b_i)
    (sizes as in the hyper-parameter table of Appendix C, e.g. [512, 128, 64]) and a last affine map to one logit.

    O [..., d]; weights[i] [d_in, d_out] with the last d_out = 1.  Returns the logits, shape O.shape[:-1].
    """
    x = _f64(O)
    for i, (W, b) in enumerate(zip(weights, biases)):
        x = x @ _f64(W) + _f64(b)
        if i + 1 < len(weights):
            x = relu(x)
    assert x.shape[-1] == 1
    return x[..., 0]


def lime_scores(E, lens, L, EC, T, p, h, scale_hist, scale_cand, eps=1e-5, return_all=False):
    """One LIME-MHA request from embeddings to scores (Section 3.1 Eq. 2-4, Section 3.3, Appendix C):

      L^C = MLP(L (+) E^C)                                              Eq. 2
      L^P = MHA(LN(L^C), LN(E), LN(E); theta_hist)                      Eq. 3, normalised inputs
      O   = MHA(LN(T), LN(L), LN(L^P); theta_cand)                      Eq. 4, normalised inputs
      score = InteractionMLP(O)                                         Section 3.3

    ``p`` is a dict of parameters: ctx = (W1, b1, W2, b2); hist = (Wq, Wk, Wv); cand = (Wq, Wk, Wv);
    ln_hist_q, ln_hist_kv, ln_cand_q, ln_cand_k, ln_cand_v = (gamma, beta) each; mlp = (weights, biases).
    Returns scores [B, C] (with return_all: also LC, LP, O).
    """
    LC = contextualize_links(L, EC, *p["ctx"])
    LP = lime_link_history(layer_norm(E, *p["ln_hist_kv"], eps), lens, layer_norm(LC, *p["ln_hist_q"], eps), *p["hist"], h,
                           scale_hist)
    O = lime_score_candidates(layer_norm(T, *p["ln_cand_q"], eps), layer_norm(L, *p["ln_cand_k"], eps),
                              layer_norm(LP, *p["ln_cand_v"], eps), *p["cand"], h, scale_cand)
    scores = interaction_mlp(O, *p["mlp"])
    return (scores, LC, LP, O) if return_all else scores
