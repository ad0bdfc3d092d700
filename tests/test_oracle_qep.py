"""Pins for the oracle's error-propagation (QEP) functions, Sec. 4.3.1 of the paper: the corrected target is
checked against what Eq. (qep_obj) and Eq. (qep) fix independently of the oracle's own formula."""
import numpy as np

from oracle import onecomp_oracle as oc


def _data(seed, T=200, d_in=24, d_out=7, noise=0.05):
    r = np.random.default_rng(seed)
    X = r.standard_normal((T, d_in)) * (1.0 + 4.0 * (r.random(d_in) < 0.1))
    X_hat = X + noise * r.standard_normal((T, d_in))
    W = 0.02 * r.standard_normal((d_out, d_in))
    return X, X_hat, W


def test_crossgram_is_additive_and_reduces_to_the_gram_matrix():
    X, X_hat, _ = _data(0)
    G = oc.crossgram_accumulate(X_hat, X)
    G2 = oc.crossgram_accumulate(X_hat[:77], X[:77])
    G2 = oc.crossgram_accumulate(X_hat[77:], X[77:], G2)
    np.testing.assert_allclose(G2, G, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(oc.crossgram_accumulate(X, X), oc.hessian_accumulate(X), rtol=1e-13)
    # element definition, one entry by explicit summation
    i, k = 3, 11
    assert abs(G[i, k] - 2.0 * sum(X_hat[t, i] * X[t, k] for t in range(X.shape[0]))) <= 1e-9 * abs(G[i, k]) + 1e-12


def test_no_propagation_leaves_the_target_unchanged():
    X, X_hat, W = _data(1)
    H = oc.hessian_accumulate(X_hat)
    G = oc.crossgram_accumulate(X_hat, X)
    assert np.array_equal(oc.qep_target(W, G, H, 0.01, 0.0), W)          # alpha = 0
    Hx = oc.hessian_accumulate(X)
    np.testing.assert_allclose(oc.qep_target(W, Hx, Hx, 0.01, 1.0), W, rtol=0, atol=1e-15)   # X_hat = X: C = 0


def test_full_strength_undamped_target_is_the_least_squares_solution():
    # Eq. (qep_obj): W* minimizes || X_hat B - X W_p ||_F over B (paper orientation, W_p = W^T)
    X, X_hat, W = _data(2)
    H = oc.hessian_accumulate(X_hat)
    G = oc.crossgram_accumulate(X_hat, X)
    Ws = oc.qep_target(W, G, H, 0.0, 1.0)
    B, *_ = np.linalg.lstsq(X_hat, X @ W.T, rcond=None)
    np.testing.assert_allclose(Ws.T, B, rtol=1e-8, atol=1e-12)
    # and any perturbation of it increases the objective
    base = np.linalg.norm(X_hat @ Ws.T - X @ W.T)
    r = np.random.default_rng(5)
    for _ in range(5):
        P = Ws + 1e-3 * r.standard_normal(Ws.shape)
        assert np.linalg.norm(X_hat @ P.T - X @ W.T) > base


def test_damped_target_matches_eq_qep_in_the_paper_s_scaling():
    # Eq. (qep) literally: W_p* = (I + alpha (H_p + lambda_p I)^-1 C) W_p with H_p = X_hat^T X_hat,
    # C = X_hat^T (X - X_hat), lambda_p = eta * mean(diag H_p): checks the factor-2 bookkeeping of H and G
    X, X_hat, W = _data(3, T=150, d_in=12, d_out=5)
    eta, alpha = 0.03, 0.7
    Hp = X_hat.T @ X_hat
    C = X_hat.T @ (X - X_hat)
    lam_p = eta * np.mean(np.diag(Hp))
    Wp_star = (np.eye(12) + alpha * np.linalg.inv(Hp + lam_p * np.eye(12)) @ C) @ W.T
    Ws = oc.qep_target(W, oc.crossgram_accumulate(X_hat, X), oc.hessian_accumulate(X_hat), eta, alpha)
    np.testing.assert_allclose(Ws, Wp_star.T, rtol=1e-9, atol=1e-13)


def test_target_is_affine_in_the_propagation_strength():
    X, X_hat, W = _data(4)
    H = oc.hessian_accumulate(X_hat)
    G = oc.crossgram_accumulate(X_hat, X)
    W1 = oc.qep_target(W, G, H, 0.01, 1.0)
    W3 = oc.qep_target(W, G, H, 0.01, 0.3)
    np.testing.assert_allclose(W3 - W, 0.3 * (W1 - W), rtol=1e-10, atol=1e-16)


def test_target_uses_the_same_damped_matrix_as_the_factor():
    # (H + lambda I)^-1 = U^T U with the U of hessian_factor: the GPU path builds the target from U
    X, X_hat, W = _data(6)
    H = oc.hessian_accumulate(X_hat)
    H[:, 5] = 0.0; H[5, :] = 0.0                     # a dead channel: damp_hessian sets its diagonal to 1
    G = oc.crossgram_accumulate(X_hat, X)
    G[5, :] = 0.0
    f = oc.hessian_factor(H, 0.02)
    U = f["U"]
    ref = W + 0.5 * (W @ (G - H).T) @ (U.T @ U)
    np.testing.assert_allclose(oc.qep_target(W, G, H, 0.02, 0.5), ref, rtol=1e-8, atol=1e-14)
