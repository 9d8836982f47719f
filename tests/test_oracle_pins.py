"""Pins for the fp64 oracle against what the paper and the mathematics fix.

None of these tests touches the HIP library.  Each pin is computed by a route
that does not go through the oracle function it checks (a closed form, an
independently written formula, a library routine, scalar loops, or finite
differences)."""
import numpy as np
import pytest
import scipy.special

from oracle import dark_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def _small(seed, L=12, d=6, r=6, m=16, dv=5, scale_x=0.7):
    g = _rng(seed)
    Q = scale_x * g.standard_normal((L, d))
    K = scale_x * g.standard_normal((L, d))
    V = g.standard_normal((L, dv))
    M = g.standard_normal((r, d)) / np.sqrt(d)
    W = g.standard_normal((m, r))
    return Q, K, V, M, W


# --- P1: M = I is the positive-random-feature map of Eq. (1) ---------------
def test_identity_geometry_is_performer_prf():
    g = _rng(1)
    L, d, m = 9, 7, 33
    X = g.standard_normal((L, d))
    W = g.standard_normal((m, d))
    a = d ** -0.25
    # Eq. (1) typed out: h(x)/sqrt(m) * exp(omega_j^T x), h = exp(-|x|^2/2), on x' = a x.
    want = np.empty((L, m))
    for i in range(L):
        xp = a * X[i]
        h = np.exp(-0.5 * np.dot(xp, xp))
        for j in range(m):
            want[i, j] = h / np.sqrt(m) * np.exp(np.dot(W[j], xp))
    Phi, c = O.featurize(X, np.eye(d), W, is_query=True)
    np.testing.assert_allclose(Phi * np.exp(c)[:, None], want, rtol=1e-12)
    PhiK, ck = O.featurize(X, np.eye(d), W, is_query=False)
    np.testing.assert_allclose(PhiK * np.exp(ck), want, rtol=1e-12)


# --- P2: unbiasedness (Eq. (3), Lemma 2.1) and the Gaussian-MGF variance ----
@pytest.mark.parametrize("r,identity", [(6, False), (4, False), (6, True)])
def test_monte_carlo_mean_and_variance(r, identity):
    g = _rng(7)
    d = 6
    M = np.eye(d) if identity else g.standard_normal((r, d)) * 0.6
    q = g.standard_normal(d)
    k = g.standard_normal(d)
    a = d ** -0.25
    qt, kt = M @ (a * q), M @ (a * k)
    v = float(np.dot(qt + kt, qt + kt))
    # The per-draw value is log-normal with log-variance v; at v = 0.5 its kurtosis is
    # about 21, so the sample variance over 1e5 draws has a relative standard error of
    # about 1.4 % and the 10 % band below is a 7-sigma band.
    if v > 0.5:
        s = np.sqrt(0.5 / v)
        q, k = s * q, s * k
        qt, kt = M @ (a * q), M @ (a * k)
        v = float(np.dot(qt + kt, qt + kt))
    Sigma = M.T @ M
    exact = np.exp(q @ Sigma @ k / np.sqrt(d))     # exp(q^T Sigma k / sqrt(d))
    n_draws = 100_000
    W = _rng(11).standard_normal((n_draws, M.shape[0]))
    # each row of W is one independent single-feature estimate
    per_draw = np.exp(O.logits(q[None], M, W)[0] + O.logits(k[None], M, W)[0])
    mean = per_draw.mean()
    se = per_draw.std(ddof=1) / np.sqrt(n_draws)
    assert abs(mean - exact) < 3.0 * se, (mean, exact, se)
    var_closed = exact ** 2 * (np.exp(v) - 1.0)
    assert abs(per_draw.var(ddof=1) / var_closed - 1.0) < 0.10
    # the m-feature estimator is the mean of its per-feature terms
    assert np.isclose(O.kernel_estimate(q, k, M, W[:64]), per_draw[:64].mean(), rtol=1e-12)


# --- P3: causal == bidirectional at the last position ------------------------
def test_causal_last_row_equals_bidirectional():
    Q, K, V, M, W = _small(3)
    np.testing.assert_allclose(O.attn_causal(Q, K, V, M, W)[-1], O.attn_bidir(Q, K, V, M, W)[-1], rtol=1e-12)


# --- P4: O(L^2) definition == linear-time order of summation ---------------
@pytest.mark.parametrize("causal", [False, True])
def test_bruteforce_equals_linear_time(causal):
    Q, K, V, M, W = _small(4, L=17)
    fast = O.attn_causal(Q, K, V, M, W) if causal else O.attn_bidir(Q, K, V, M, W)
    np.testing.assert_allclose(fast, O.attn_brute(Q, K, V, M, W, causal), rtol=1e-11)
    Qs, Ks, Vs, Ms, Ws = _small(5, L=5, d=3, r=3, m=4, dv=2)
    for f in (O.attn_brute(Qs, Ks, Vs, Ms, Ws, causal),
              O.attn_causal(Qs, Ks, Vs, Ms, Ws) if causal else O.attn_bidir(Qs, Ks, Vs, Ms, Ws)):
        np.testing.assert_allclose(f, O.attn_loops(Qs, Ks, Vs, Ms, Ws, causal), rtol=1e-11)
    for i in (0, 3, 16):
        np.testing.assert_allclose(O.attn_row(Q, K, V, M, W, i, causal), fast[i], rtol=1e-11)
    if causal:
        np.testing.assert_allclose(O.attn_causal(Q, K, V, M, W, rows=[2, 9]), fast[[2, 9]], rtol=1e-13)


# --- P5: omega~ = M^T w gives the same logits (Appendix B) -------------------
def test_fused_direction_matrix():
    Q, K, V, M, W = _small(6, r=4)
    A = W @ M                                     # rows omega~_j^T
    a = Q.shape[1] ** -0.25
    Sigma = M.T @ M
    want = (a * Q) @ A.T - 0.5 * np.einsum("ic,ce,ie->i", a * Q, Sigma, a * Q)[:, None]
    np.testing.assert_allclose(O.logits(Q, M, W), want, rtol=1e-11, atol=1e-12)


# --- P6: polarisation identity (Section 4.1) applied to (w_j, x~) ------------
def test_logit_is_gaussian_rbf_form():
    Q, K, V, M, W = _small(8)
    a = Q.shape[1] ** -0.25
    Xt = (a * Q) @ M.T
    dist2 = ((W[None, :, :] - Xt[:, None, :]) ** 2).sum(-1)
    want = 0.5 * (W ** 2).sum(-1)[None, :] - 0.5 * dist2
    lg = O.logits(Q, M, W)
    np.testing.assert_allclose(lg, want, rtol=1e-11, atol=1e-12)
    assert np.all(lg <= 0.5 * (W ** 2).sum(-1)[None, :] + 1e-12)


# --- P7: positivity => outputs are convex combinations of values -------------
@pytest.mark.parametrize("causal", [False, True])
def test_convex_hull(causal):
    Q, K, V, M, W = _small(9, L=20)
    out = O.attn_causal(Q, K, V, M, W) if causal else O.attn_bidir(Q, K, V, M, W)
    for i in range(len(out)):
        Vi = V[: i + 1] if causal else V
        assert np.all(out[i] <= Vi.max(0) + 1e-12) and np.all(out[i] >= Vi.min(0) - 1e-12)
    if causal:
        np.testing.assert_allclose(out[0], V[0], rtol=1e-12)
    Phi, c = O.featurize(Q, M, W, True)
    assert np.all(Phi > 0) and np.allclose(Phi.max(1), 1 / np.sqrt(W.shape[0]))
    PhiK, ck = O.featurize(K, M, W, False)
    assert np.isclose(PhiK.max(), 1 / np.sqrt(W.shape[0])) and np.ndim(ck) == 0


# --- P8: invariances ---------------------------------------------------------
def test_gauge_invariances():
    Q, K, V, M, W = _small(10)
    base = O.attn_bidir(Q, K, V, M, W)
    R = np.linalg.qr(_rng(2).standard_normal((M.shape[0],) * 2))[0]
    np.testing.assert_allclose(O.attn_bidir(Q, K, V, R @ M, W @ R.T), base, rtol=1e-10)
    b = np.arange(V.shape[1], dtype=float)
    np.testing.assert_allclose(O.attn_bidir(Q, K, V + b, M, W), base + b, rtol=1e-10)
    # explicit scale argument == rescaling the inputs by hand
    np.testing.assert_allclose(O.attn_bidir(Q, K, V, M, W, scale=0.3),
                               O.attn_bidir(Q * np.sqrt(0.3) * Q.shape[1] ** 0.25, K * np.sqrt(0.3) * Q.shape[1] ** 0.25, V, M, W),
                               rtol=1e-10)


# --- P11: many features -> exact softmax attention in the geometry M --------
@pytest.mark.parametrize("causal", [False, True])
def test_softmax_limit(causal):
    g = _rng(12)
    L, d, dv, m = 6, 4, 3, 200_000
    Q = 0.25 * g.standard_normal((L, d))
    K = 0.25 * g.standard_normal((L, d))
    V = g.standard_normal((L, dv))
    M = np.eye(d) + 0.2 * g.standard_normal((d, d))
    W = g.standard_normal((m, d))
    scores = (Q @ M.T) @ (K @ M.T).T / np.sqrt(d)
    if causal:
        scores = np.where(np.tril(np.ones((L, L))) > 0, scores, -np.inf)
    want = scipy.special.softmax(scores, axis=1) @ V
    got = O.attn_causal(Q, K, V, M, W) if causal else O.attn_bidir(Q, K, V, M, W)
    a = d ** -0.25
    vmax = max(np.sum((M @ (a * (q + k))) ** 2) for q in Q for k in K)
    tol = 5.0 * np.sqrt((np.exp(vmax) - 1.0) / m) * 2.0 * np.abs(V).max()
    assert np.abs(got - want).max() < tol, (np.abs(got - want).max(), tol)
    assert tol < 0.1


# --- P9 / P10: gradients ------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_backward_finite_differences(causal):
    Q, K, V, M, W = _small(13, L=7, d=5, r=4, m=9, dv=3)
    G = _rng(14).standard_normal(V.shape)

    def loss(Q_, K_, V_, M_):
        return float(np.sum(O.attn_brute(Q_, K_, V_, M_, W, causal) * G))

    dQ, dK, dV, dM = O.attn_bwd_brute(Q, K, V, M, W, G, causal)
    h = 1e-6
    for name, arr, grad, pos in (("Q", Q, dQ, 0), ("K", K, dK, 1), ("V", V, dV, 2), ("M", M, dM, 3)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            args = [Q.copy(), K.copy(), V.copy(), M.copy()]
            args[pos][idx] += h
            up = loss(*args)
            args[pos][idx] -= 2 * h
            dn = loss(*args)
            num[idx] = (up - dn) / (2 * h)
        np.testing.assert_allclose(grad, num, rtol=2e-6, atol=2e-8, err_msg=name)
    # shifting all values by a constant shifts every output by it
    np.testing.assert_allclose(dV.sum(0), G.sum(0), rtol=1e-10)


@pytest.mark.parametrize("causal", [False, True])
def test_gradient_of_the_draws_finite_differences(causal):
    """dW (Section 6: the learned feature kernel trains the projections) against central differences."""
    Q, K, V, M, W = _small(15, L=6, d=5, r=4, m=7, dv=3)
    G = _rng(16).standard_normal(V.shape)
    *_, dW = O.attn_bwd_brute(Q, K, V, M, W, G, causal, with_dW=True)
    assert dW.shape == W.shape
    h = 1e-6
    num = np.zeros_like(W)
    for idx in np.ndindex(W.shape):
        Wp, Wm = W.copy(), W.copy()
        Wp[idx] += h
        Wm[idx] -= h
        num[idx] = (np.sum(O.attn_brute(Q, K, V, M, Wp, causal) * G) - np.sum(O.attn_brute(Q, K, V, M, Wm, causal) * G)) / (2 * h)
    np.testing.assert_allclose(dW, num, rtol=2e-6, atol=2e-8)
    # the four other gradients do not change when dW is asked for
    for a, b in zip(O.attn_bwd_brute(Q, K, V, M, W, G, causal), O.attn_bwd_brute(Q, K, V, M, W, G, causal, with_dW=True)):
        np.testing.assert_array_equal(a, b)


# --- whitening geometry (Section 4.1, Proposition C.1) ----------------------------------------------
def test_whitening_geometry():
    g = _rng(31)
    d, N = 9, 4000
    C = g.standard_normal((d, d))
    C = C @ C.T + 0.05 * np.eye(d)
    Lc = np.linalg.cholesky(C)
    mu = g.standard_normal(d)
    Q = g.standard_normal((N, d)) @ Lc.T + mu
    K = g.standard_normal((N, d)) @ Lc.T + mu
    M, Lam = O.whitening_geometry(Q, K)
    # the estimate is the centred pooled sample covariance (numpy's own routine, bias = divisor N)
    np.testing.assert_allclose(Lam, np.cov(np.concatenate([Q, K]).T, bias=True), rtol=1e-10, atol=1e-12)
    # whitening: Cov(M x) = M Lambda M^T = I, and Sigma = M^T M = Lambda^{-1} (library inverse)
    np.testing.assert_allclose(M @ Lam @ M.T, np.eye(d), atol=1e-9)
    np.testing.assert_allclose(M.T @ M, np.linalg.inv(Lam), rtol=1e-8)
    # close to the population statement M C M^T = I within sampling error
    assert np.abs(M @ C @ M.T - np.eye(d)).max() < 0.12
    # Proposition C.1: |q - k|^2 in the Lambda^{-1} geometry = sum_i delta_i^2 / lambda_i = |Mq - Mk|^2
    lam, U = np.linalg.eigh(Lam)
    q, k = Q[3], K[5]
    delta = U.T @ (q - k)
    want = float(np.sum(delta ** 2 / lam))
    np.testing.assert_allclose((q - k) @ np.linalg.inv(Lam) @ (q - k), want, rtol=1e-9)
    np.testing.assert_allclose(np.sum((M @ q - M @ k) ** 2), want, rtol=1e-9)
    # a common offset of all rows changes nothing
    M2, _ = O.whitening_geometry(Q + 7.0, K + 7.0)
    np.testing.assert_allclose(M2.T @ M2, M.T @ M, rtol=1e-7)
    # r < d: the r directions of largest variance, whitened
    Mr, _ = O.whitening_geometry(Q, K, r=4)
    assert Mr.shape == (4, d)
    np.testing.assert_allclose(Mr @ Lam @ Mr.T, np.eye(4), atol=1e-9)
    top = U[:, np.argsort(lam)[::-1][:4]]
    np.testing.assert_allclose(Mr.T @ Mr @ top, top / np.sort(lam)[::-1][:4][None, :], rtol=1e-8, atol=1e-10)
    # the floor: a direction without variance does not blow up
    Qd = Q.copy(); Kd = K.copy()
    Qd[:, 0] = 1.0; Kd[:, 0] = 1.0
    Mf, Lf = O.whitening_geometry(Qd, Kd, floor=1e-6)
    assert np.isfinite(Mf).all() and np.abs(Mf).max() <= 1.0001 / np.sqrt(1e-6 * np.linalg.eigvalsh(Lf).max())
