"""Plain fp64 CPU oracle for DARK attention.  TEST INFRASTRUCTURE ONLY.

This module is the slow, obviously-correct statement of what the HIP library
computes.  Only the test-suite, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product path never does, and this
module imports nothing from the product (numpy only).

Notation follows the paper: per head, queries/keys ``x in R^d``, a learned
geometry ``M in R^{r x d}`` (Sigma = M^T M, Section 4.1), random draws
``w_j ~ N(0, I_r)`` (rows of ``W in R^{m x r}``), and the data-aware directions
``omega~_j = M^T w_j`` (Appendix B, derivation of Eq. (3)).

Readings of points the paper leaves open (each is also listed in the design
notes of the repository):

* The 1/sqrt(d) of scaled dot-product attention is split evenly: every query
  and key is multiplied by ``alpha = d**-0.25`` before the feature map
  (Section 2, footnote on absorbing the scaling), so the estimand is
  ``exp(q^T Sigma k / sqrt(d))``.
* The 1/sqrt(m) factor of the feature map (Section 4.1) is kept.
* No epsilon is added anywhere; the normaliser is the plain sum of the
  estimated kernel values (Section 2, footnote: normalising gives softmax
  attention).
* Causal attention (not spelled out in the paper) lets position i attend to
  keys l <= i.
* Stabilisers: the feature values returned by :func:`featurize` are
  ``exp(logit - c) / sqrt(m)`` with ``c`` the per-row maximum logit for
  queries and the per-head maximum logit for keys.  They cancel exactly in
  every attention output.

Pins (tests/test_oracle_pins.py): Performer special case M = I (Eq. (1)),
Monte-Carlo unbiasedness and closed-form variance (Eq. (3), Lemma 2.1),
causal == bidirectional at the last position, O(L^2) brute force == linear
time, polarisation identity (Section 4.1), convex-hull and gauge invariances,
softmax limit for large m, finite differences for every gradient (Q, K, V, M
and the draws W).
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "alpha_of", "logits", "featurize", "kernel_estimate",
    "attn_bidir", "attn_causal", "attn_brute", "attn_loops",
    "attn_bwd_brute", "attn_row", "whitening_geometry",
]


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def alpha_of(d: int, scale: float | None = None) -> float:
    """Factor applied to each of q and k so that their product carries `scale`.

    scale = 1/sqrt(d) unless given (Section 2: scaled dot-product attention and
    the footnote that q, k absorb the scaling)."""
    s = 1.0 / np.sqrt(float(d)) if scale is None else float(scale)
    return float(np.sqrt(s))


def logits(X, M, W, scale=None):
    """Log of the unnormalised positive random features of the rows of X.

    Section 4.1 (feature map phi_Sigma) with omega~_j = M^T w_j (Appendix B):
    x' = alpha x;  x~ = M x';  logit_j = w_j^T x~ - 1/2 ||x~||^2.
    X: [L, d], M: [r, d], W: [m, r]  ->  [L, m].
    The projection through M is done first and the dot with w_j second, as the
    appendix writes it; nothing is pre-multiplied.
    """
    X, M, W = _f64(X), _f64(M), _f64(W)
    a = alpha_of(X.shape[-1], scale)
    Xp = a * X                      # x'
    Xt = Xp @ M.T                   # x~ = M x'            [L, r]
    n = 0.5 * np.sum(Xt * Xt, axis=-1, keepdims=True)   # 1/2 ||x~||^2
    return Xt @ W.T - n             # w_j^T x~ - n         [L, m]


def featurize(X, M, W, is_query: bool, scale=None):
    """phi_Sigma(x) of Section 4.1 for every row, stabilised.

    Returns (Phi, c) with Phi = exp(logit - c)/sqrt(m); c has shape [L] (row
    maxima) for queries and is a scalar (maximum over the whole head) for keys.
    The unstabilised features are Phi * exp(c).
    """
    lg = logits(X, M, W, scale)
    m = lg.shape[-1]
    if is_query:
        c = lg.max(axis=-1)
        Phi = np.exp(lg - c[:, None]) / np.sqrt(m)
    else:
        c = lg.max()
        Phi = np.exp(lg - c) / np.sqrt(m)
    return Phi, c


def kernel_estimate(q, k, M, W, scale=None):
    """phi(q)^T phi(k): the m-draw estimate of exp(q'^T Sigma k') (Eq. (3))."""
    lq = logits(np.atleast_2d(q), M, W, scale)[0]
    lk = logits(np.atleast_2d(k), M, W, scale)[0]
    return float(np.sum(np.exp(lq + lk)) / lq.shape[0])


def attn_bidir(Q, K, V, M, W, scale=None):
    """Linear-time bidirectional random-feature attention for one head.

    Section 2 ("Efficient attention via random feature kernels"): form
    K'^T V first, then multiply by Q'; divide by Q'(K'^T 1) (footnote on
    normalisation).  Returns out [L, dv]."""
    V = _f64(V)
    PhiQ, _ = featurize(Q, M, W, True, scale)
    PhiK, _ = featurize(K, M, W, False, scale)
    S = PhiK.T @ V                  # [m, dv]
    z = PhiK.sum(axis=0)            # [m]
    return (PhiQ @ S) / (PhiQ @ z)[:, None]


def attn_causal(Q, K, V, M, W, scale=None, rows=None):
    """Causal form: position i uses keys l <= i.  One running (S, z) state,
    updated token by token; no chunking.  `rows` optionally restricts which
    output rows are produced (the state is still advanced over every key)."""
    V = _f64(V)
    PhiQ, _ = featurize(Q, M, W, True, scale)
    PhiK, _ = featurize(K, M, W, False, scale)
    L, m = PhiQ.shape
    dv = V.shape[1]
    want = None if rows is None else set(int(i) for i in rows)
    out = np.zeros((L, dv))
    S = np.zeros((m, dv))
    z = np.zeros(m)
    for i in range(L):
        S += np.outer(PhiK[i], V[i])
        z += PhiK[i]
        if want is None or i in want:
            out[i] = (PhiQ[i] @ S) / (PhiQ[i] @ z)
    if rows is not None:
        return out[np.asarray(list(rows), dtype=np.int64)]
    return out


def attn_brute(Q, K, V, M, W, causal: bool, scale=None):
    """O(L^2) definition: estimated kernel matrix a_il = phi(q_i)^T phi(k_l),
    then out_i = sum_l a_il v_l / sum_l a_il (l <= i if causal)."""
    V = _f64(V)
    lq = logits(Q, M, W, scale)
    lk = logits(K, M, W, scale)
    cq = lq.max(axis=1, keepdims=True)
    ck = lk.max()
    a = np.exp(lq - cq) @ np.exp(lk - ck).T      # [L, L], common factors cancel
    if causal:
        a = np.tril(a)
    return (a @ V) / a.sum(axis=1, keepdims=True)


def attn_loops(Q, K, V, M, W, causal: bool, scale=None):
    """The same definition in scalar Python loops (tiny inputs only)."""
    Q, K, V, M, W = map(_f64, (Q, K, V, M, W))
    L, d = Q.shape
    r = M.shape[0]
    m = W.shape[0]
    dv = V.shape[1]
    al = alpha_of(d, scale)

    def lg(x):
        xt = [sum(M[t, c] * al * x[c] for c in range(d)) for t in range(r)]
        n = 0.5 * sum(v * v for v in xt)
        return [sum(W[j, t] * xt[t] for t in range(r)) - n for j in range(m)]

    lq = [lg(Q[i]) for i in range(L)]
    lk = [lg(K[i]) for i in range(L)]
    out = np.zeros((L, dv))
    for i in range(L):
        den = 0.0
        num = [0.0] * dv
        hi = i + 1 if causal else L
        for l in range(hi):
            a = sum(np.exp(lq[i][j] + lk[l][j]) for j in range(m)) / m
            den += a
            for c in range(dv):
                num[c] += a * V[l, c]
        out[i] = [x / den for x in num]
    return out


def attn_row(Q, K, V, M, W, i: int, causal: bool, scale=None):
    """One output row out_i by its definition (used to sample large problems)."""
    V = _f64(V)
    hi = i + 1 if causal else K.shape[0]
    lq = logits(np.asarray(Q)[i:i + 1], M, W, scale)[0]
    lk = logits(np.asarray(K)[:hi], M, W, scale)
    a = np.exp(lk - lk.max() + (lq - lq.max())[None, :]).sum(axis=1)   # [hi]
    return (a @ V[:hi]) / a.sum()


def attn_bwd_brute(Q, K, V, M, W, G, causal: bool, scale=None, with_dW=False):
    """Gradients of sum(out * G) w.r.t. Q, K, V, M for one head, O(L^2); with_dW adds the gradient
    w.r.t. the draws W [m, r] as a fifth result (Section 6: the learned feature kernel trains the
    projections of Eq. (1) themselves).

    The paper only says M is learnable (Section 4.1); these are the chain-rule
    derivatives of the definition above, written through the literal forward
    (x' -> x~ = M x' -> logits -> exp -> kernel matrix -> ratio):

      out_i = sum_l a_il v_l / D_i,  D_i = sum_l a_il
      d a_il = G_i . (v_l - out_i) / D_i
      a_il   = sum_j exp(lq_ij + lk_lj)/m
      d lq_ij = sum_l d a_il exp(lq_ij + lk_lj)/m     (same for lk with i<->l)
      logit_j = w_j^T x~ - 1/2||x~||^2  =>  d x~ = W^T d logit - (sum_j d logit_j) x~
      x~ = M x', x' = alpha x  =>  dM += d x~ x'^T,  dx = alpha M^T d x~
    Returns dQ, dK, dV, dM (dM summed over both the query and the key path).
    """
    Q, K, V, M, W, G = map(_f64, (Q, K, V, M, W, G))
    L, d = Q.shape
    m = W.shape[0]
    al = alpha_of(d, scale)
    Qp, Kp = al * Q, al * K
    Qt, Kt = Qp @ M.T, Kp @ M.T
    lq = Qt @ W.T - 0.5 * np.sum(Qt * Qt, axis=1, keepdims=True)
    lk = Kt @ W.T - 0.5 * np.sum(Kt * Kt, axis=1, keepdims=True)
    # Work with stabilised factors; a_il = e^{cq_i + ck} * (Eq Ek^T)/m.
    cq = lq.max(axis=1, keepdims=True)
    ck = lk.max()
    Eq, Ek = np.exp(lq - cq), np.exp(lk - ck)
    a = (Eq @ Ek.T) / m                       # a_il / e^{cq_i+ck}
    mask = np.tril(np.ones((L, L))) if causal else np.ones((L, L))
    a = a * mask
    D = a.sum(axis=1, keepdims=True)
    out = (a @ V) / D
    # d(out)/d(a) is homogeneous of degree -1 in the row scale, so the row
    # factor e^{cq_i+ck} cancels between `da` and the exp() it multiplies.
    da = ((G @ V.T) - np.sum(G * out, axis=1, keepdims=True)) / D * mask   # [L, L]
    dV = (a / D).T @ G
    dlq = (da @ Ek) * Eq / m
    dlk = (da.T @ Eq) * Ek / m
    dQt = dlq @ W - dlq.sum(axis=1, keepdims=True) * Qt
    dKt = dlk @ W - dlk.sum(axis=1, keepdims=True) * Kt
    dM = dQt.T @ Qp + dKt.T @ Kp
    dQ = al * (dQt @ M)
    dK = al * (dKt @ M)
    if with_dW:
        # logit_j = w_j^T x~ - ... depends on w_j through the first term only
        return dQ, dK, dV, dM, dlq.T @ Qt + dlk.T @ Kt
    return dQ, dK, dV, dM


def whitening_geometry(Q, K, r=None, floor=1e-6):
    """Geometry that whitens the inputs (Section 4.1 and Proposition C.1: with input covariance Lambda,
    M = Lambda^{-1/2}, Sigma = Lambda^{-1}, makes M q and M k isotropic).

    Q, K: [N, d] rows of one head (the paper assumes Cov(q) = Cov(k) = Lambda, Section 3, so the two are
    pooled).  Readings where the paper is silent: Lambda is estimated as the centred sample covariance of
    the 2N pooled rows (divisor 2N); with Lambda = U diag(lambda) U^T, lambda descending, the result is
    M = diag(lambda_1..r ^ -1/2) U[:, :r]^T (rows = principal directions; for r = d this is Lambda^{-1/2}
    up to a rotation of the rows, which leaves Sigma = M^T M unchanged; for r < d, allowed by Appendix B,
    the r directions of largest variance); eigenvalues below floor * lambda_1 are raised to it.
    Returns (M [r, d], Lambda [d, d]).
    """
    X = np.concatenate([_f64(Q), _f64(K)], axis=0)
    d = X.shape[1]
    r = d if r is None else int(r)
    Xc = X - X.mean(axis=0, keepdims=True)
    Lam = Xc.T @ Xc / X.shape[0]
    w, U = np.linalg.eigh(Lam)
    order = np.argsort(w)[::-1]
    w, U = w[order], U[:, order]
    w = np.maximum(w, floor * w[0])
    M = (U[:, :r] / np.sqrt(w[:r])[None, :]).T
    return M, Lam
