"""Pins for the float64 oracle: closed forms, invariants, special cases that reduce
to textbook routines, brute force on tiny inputs and hand-worked examples.
Nothing here touches the HIP library."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import onecomp_oracle as oc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")


def _rng(seed):
    return np.random.default_rng(seed)


def _spd(n, seed, cond_boost=0.0):
    r = _rng(seed)
    X = r.standard_normal((3 * n + 5, n))
    X[:, : max(1, n // 8)] *= 1.0 + cond_boost
    return oc.hessian_accumulate(X)


# ------------------------------------------------------------------ Gram ---
def test_gram_additive_over_chunks_and_symmetric():
    r = _rng(1)
    X = r.standard_normal((37, 11))
    H = oc.hessian_accumulate(X)
    H2 = oc.hessian_accumulate(X[20:], oc.hessian_accumulate(X[:20]))
    np.testing.assert_allclose(H, H2, rtol=1e-13, atol=1e-13)
    np.testing.assert_array_equal(H, H.T)


def test_gram_one_hot_rows_give_twice_the_counts():
    idx = np.array([0, 2, 2, 3, 3, 3, 5])
    X = np.zeros((len(idx), 6))
    X[np.arange(len(idx)), idx] = 1.0
    H = oc.hessian_accumulate(X)
    np.testing.assert_array_equal(H, 2.0 * np.diag([1, 0, 2, 3, 0, 1]))


def test_gram_all_ones():
    H = oc.hessian_accumulate(np.ones((9, 4)))
    np.testing.assert_array_equal(H, 18.0 * np.ones((4, 4)))


def test_gram_quadratic_form_is_twice_the_output_energy():
    r = _rng(2)
    X = r.standard_normal((50, 13))
    v = r.standard_normal(13)
    H = oc.hessian_accumulate(X)
    assert np.isclose(v @ H @ v, 2.0 * np.sum((X @ v) ** 2), rtol=1e-12)


def test_gram_not_transposed_and_tile_matches_full():
    r = _rng(3)
    X = r.standard_normal((7, 5))            # n_tokens != d_in: a transposed product has the wrong shape
    H = oc.hessian_accumulate(X)
    assert H.shape == (5, 5)
    # element by element from the definition
    for i in range(5):
        for k in range(5):
            assert np.isclose(H[i, k], 2.0 * sum(X[t, i] * X[t, k] for t in range(7)), rtol=1e-13)
    np.testing.assert_allclose(oc.hessian_tile(X, [1, 3], [0, 2, 4]), H[np.ix_([1, 3], [0, 2, 4])], rtol=1e-13)


# --------------------------------------------------------------- factor ---
def test_damping_rule():
    H = np.diag([1.0, 2.0, 3.0, 6.0])
    Hd, lam = oc.damp_hessian(H, 0.5)
    assert lam == 0.5 * 3.0
    np.testing.assert_array_equal(np.diag(Hd), np.array([1.0, 2.0, 3.0, 6.0]) + 1.5)


def test_dead_channel_gets_unit_diagonal_before_damping():
    H = np.diag([4.0, 0.0, 8.0])
    Hd, lam = oc.damp_hessian(H, 0.3)
    assert np.isclose(lam, 0.3 * (4.0 + 1.0 + 8.0) / 3.0)
    np.testing.assert_allclose(np.diag(Hd), np.array([4.0, 1.0, 8.0]) + lam)


def test_inverse_factor_defining_properties():
    Hd, _ = oc.damp_hessian(_spd(24, 4, cond_boost=20.0), 0.01)
    U, info = oc.inverse_factor(Hd)
    assert info == 0
    assert np.all(np.tril(U, -1) == 0.0)
    assert np.all(np.diag(U) > 0.0)
    np.testing.assert_allclose(U.T @ U @ Hd, np.eye(24), atol=1e-9)
    np.testing.assert_allclose(U @ Hd @ U.T, np.eye(24), atol=1e-9)


def test_inverse_factor_equals_reversed_cholesky_route():
    # Independent route: Hd = M M^T with M upper (Cholesky of the index-reversed
    # matrix, reversed back), then U = M^-1.  Uniqueness of the factor makes them equal.
    Hd, _ = oc.damp_hessian(_spd(17, 5, cond_boost=5.0), 0.01)
    U, _ = oc.inverse_factor(Hd)
    J = np.eye(17)[::-1]
    L = np.linalg.cholesky(J @ Hd @ J)
    M = J @ L @ J
    assert np.all(np.tril(M, -1) == 0.0)
    np.testing.assert_allclose(np.linalg.inv(M), U, rtol=1e-9, atol=1e-12)


def test_inverse_factor_rows_are_schur_complement_rows():
    # Row j of U, scaled by its diagonal, is the first row of the inverse of the
    # trailing sub-matrix Hd[j:, j:], and U_jj^2 is that inverse's first entry.
    Hd, _ = oc.damp_hessian(_spd(12, 6), 0.02)
    U, _ = oc.inverse_factor(Hd)
    for j in range(12):
        S = np.linalg.inv(Hd[j:, j:])
        assert np.isclose(U[j, j] ** 2, S[0, 0], rtol=1e-9)
        np.testing.assert_allclose(U[j, j:] / U[j, j], S[0, :] / S[0, 0], rtol=1e-8, atol=1e-12)


def test_inverse_factor_diagonal_matrix():
    d = np.array([4.0, 0.25, 9.0, 1.0])
    U, info = oc.inverse_factor(np.diag(d))
    assert info == 0
    np.testing.assert_allclose(U, np.diag(1.0 / np.sqrt(d)), rtol=1e-14)


def test_not_positive_definite_reports_first_bad_pivot():
    A = np.diag([1.0, 2.0, -3.0, 4.0])
    U, info = oc.inverse_factor(A)
    assert U is None and info == 3
    assert oc.inverse_factor(-np.eye(3))[1] == 1
    B = np.array([[1.0, 2.0], [2.0, 1.0]])          # second pivot 1 - 4 < 0
    assert oc.inverse_factor(B)[1] == 2
    assert oc.first_bad_pivot(np.eye(5)) == 0


def test_act_order_is_stable_descending():
    H = np.diag([3.0, 7.0, 3.0, 9.0, 7.0])
    np.testing.assert_array_equal(oc.act_order_perm(H), [3, 1, 4, 0, 2])


def test_hessian_factor_with_act_order_factors_the_permuted_matrix():
    H = _spd(10, 7, cond_boost=3.0)
    f = oc.hessian_factor(H, 0.01, act_order=True)
    p = f["perm"]
    assert sorted(p.tolist()) == list(range(10))
    assert np.all(np.diff(np.diag(H)[p]) <= 0)
    Hp = f["Hd"][np.ix_(p, p)]
    np.testing.assert_allclose(f["U"] @ Hp @ f["U"].T, np.eye(10), atol=1e-9)


# ----------------------------------------------------------------- grid ---
def test_hand_worked_grid_examples():
    with open(GOLDEN) as fh:
        gold = json.load(fh)
    for ex in gold["grid"]:
        w = np.array(ex["w"])
        s, z, _ = oc.minmax_params(w.min(), w.max(), ex["bits"])
        q, wh, _ = oc.quantize_scalar(w, s, z, ex["bits"])
        assert float(s) == ex["s"] and float(z) == ex["z"]
        np.testing.assert_array_equal(q, ex["q"])
        np.testing.assert_array_equal(wh, ex["w_hat"])
        # the same through the whole-array routine
        Q, S, Z, WH = oc.rtn_quantize(w[None, :], ex["bits"], len(w))
        np.testing.assert_array_equal(Q[0], ex["q"])
        np.testing.assert_array_equal(WH[0], ex["w_hat"])


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_grid_endpoints_error_bound_and_exact_grid(bits):
    r = _rng(10 + bits)
    W = r.standard_normal((16, 64)) * 0.02
    Q, S, Z, WH = oc.rtn_quantize(W, bits, 32)
    qmax = 2 ** bits - 1
    assert Q.min() >= 0 and Q.max() <= qmax
    Wg, Qg = W.reshape(16, 2, 32), Q.reshape(16, 2, 32)
    # groups that straddle zero have an unclamped zero-point: min -> 0, max -> qmax
    amin = np.take_along_axis(Qg, Wg.argmin(2)[..., None], 2)[..., 0]
    amax = np.take_along_axis(Qg, Wg.argmax(2)[..., None], 2)[..., 0]
    assert np.all(amin == 0) and np.all(amax == qmax)
    # no clipping here, so |w - w^| <= s/2 (text after Eq. (1))
    err = np.abs(W - WH).reshape(16, 2, 32)
    assert np.all(err <= 0.5 * S[:, :, None] * (1 + 1e-12))
    # weights that already lie on a grid s0 (k - z0) are reproduced exactly
    s0, z0 = 0.125, 3
    k = r.integers(0, qmax + 1, size=(5, 32))
    k[:, 0], k[:, 1] = 0, qmax
    Wgrid = s0 * (k - z0)
    Q2, S2, Z2, WH2 = oc.rtn_quantize(Wgrid, bits, 32)
    np.testing.assert_array_equal(WH2, Wgrid)
    if z0 <= qmax:
        np.testing.assert_array_equal(Q2, k)


def test_degenerate_group_takes_unit_scale():
    s, z, _ = oc.minmax_params(np.array([0.75]), np.array([0.75]), 4)
    assert s[0] == 1.0 and z[0] == 0.0           # rne(-0.75) = -1 -> clamp 0
    s, z, _ = oc.minmax_params(np.array([-2.5]), np.array([-2.5]), 4)
    assert s[0] == 1.0 and z[0] == 2.0           # rne(2.5) = 2 (half to even)


def test_dequantize_reproduces_w_hat_exactly():
    r = _rng(20)
    W = r.standard_normal((6, 32)) * 0.02
    f = oc.hessian_factor(_spd(32, 21, cond_boost=4.0), 0.01, act_order=True)
    out = oc.quantize_layer(W, f["U"], 3, 8, perm=f["perm"])
    np.testing.assert_array_equal(
        oc.dequantize(out["Q"], out["scales"], out["zeros"], 8, perm=f["perm"]), out["W_hat"])


# ---------------------------------------------------------------- sweep ---
@pytest.mark.parametrize("bits,G", [(4, 16), (3, 8), (2, 32)])
def test_diagonal_hessian_reproduces_round_to_nearest(bits, G):
    r = _rng(30 + bits)
    W = r.standard_normal((9, 32)) * 0.02
    H = np.diag(r.uniform(0.5, 50.0, size=32))
    f = oc.hessian_factor(H, 0.01)
    out = oc.quantize_layer(W, f["U"], bits, G)
    Q, S, Z, WH = oc.rtn_quantize(W, bits, G)
    np.testing.assert_array_equal(out["Q"], Q)
    np.testing.assert_array_equal(out["scales"], S)
    np.testing.assert_array_equal(out["zeros"], Z)
    np.testing.assert_array_equal(out["W_hat"], WH)


def test_identity_hessian_loss_is_frobenius_error():
    r = _rng(40)
    W = r.standard_normal((7, 24)) * 0.02
    f = oc.hessian_factor(np.eye(24), 0.0)
    np.testing.assert_array_equal(f["U"], np.eye(24))
    out = oc.quantize_layer(W, f["U"], 4, 8)
    assert np.isclose(out["loss"], np.sum((W - out["W_hat"]) ** 2), rtol=1e-13)


def test_sequential_loss_equals_quadratic_form_greedy_and_forced():
    r = _rng(41)
    W = r.standard_normal((5, 24)) * 0.02
    f = oc.hessian_factor(_spd(24, 42, cond_boost=10.0), 0.01)
    out = oc.quantize_layer(W, f["U"], 3, 8)
    assert np.isclose(out["loss"], oc.layer_loss(W, out["W_hat"], f["Hd"]), rtol=1e-9)
    forced = r.integers(0, 8, size=(5, 24))
    out2 = oc.quantize_layer(W, f["U"], 3, 8, forced_codes=forced)
    np.testing.assert_array_equal(out2["Q"], forced)
    assert np.isclose(out2["loss"], oc.layer_loss(W, out2["W_hat"], f["Hd"]), rtol=1e-9)
    assert out2["loss"] > out["loss"]
    # after the sweep W - W^ = E U exactly (each column lands on its grid point)
    np.testing.assert_allclose(W - out["W_hat"], out["E"] @ f["U"], atol=1e-15)


def test_hand_worked_two_column_sweep():
    with open(GOLDEN) as fh:
        ex = json.load(fh)["sweep_2col"]
    Hd = np.array(ex["Hd"])
    U, _ = oc.inverse_factor(Hd)
    out = oc.quantize_layer(np.array([ex["w"]]), U, ex["bits"], ex["group_size"])
    np.testing.assert_array_equal(out["Q"][0], ex["q"])
    np.testing.assert_allclose(out["W_hat"][0], ex["w_hat"], atol=1e-15)
    assert out["scales"][0, 0] == ex["s"] and out["zeros"][0, 0] == ex["z"]
    assert np.isclose(out["loss"], ex["loss"], rtol=1e-12)
    np.testing.assert_array_equal(oc.rtn_quantize(np.array([ex["w"]]), 2, 2)[0][0], ex["rtn_q"])


def test_two_column_closed_form_random():
    r = _rng(43)
    for _ in range(20):
        a, b = r.uniform(1.0, 3.0, size=2)
        c = r.uniform(-0.9, 0.9) * np.sqrt(a * b)
        Hd = np.array([[a, c], [c, b]])
        U, _ = oc.inverse_factor(Hd)
        w = r.standard_normal(2)
        out = oc.quantize_layer(w[None, :], U, 3, 2)
        s, z = out["scales"][0, 0], out["zeros"][0, 0]
        q0 = np.clip(np.rint(w[0] / s) + z, 0, 7)
        d0 = w[0] - s * (q0 - z)
        w1 = w[1] + d0 * c / b
        q1 = np.clip(np.rint(w1 / s) + z, 0, 7)
        d1 = w1 - s * (q1 - z)
        np.testing.assert_array_equal(out["Q"][0], [q0, q1])
        assert np.isclose(out["loss"], d0 * d0 * (a - c * c / b) + b * d1 * d1, rtol=1e-9)


def test_scaling_the_hessian_keeps_codes_and_scales_the_loss():
    r = _rng(44)
    W = r.standard_normal((6, 32)) * 0.02
    H = _spd(32, 45, cond_boost=6.0)
    f1 = oc.hessian_factor(H, 0.01)
    f2 = oc.hessian_factor(8.0 * H, 0.01)          # power of two: exact rescale
    o1 = oc.quantize_layer(W, f1["U"], 4, 16)
    o2 = oc.quantize_layer(W, f2["U"], 4, 16)
    np.testing.assert_array_equal(o1["Q"], o2["Q"])
    assert np.isclose(o2["loss"], 8.0 * o1["loss"], rtol=1e-9)


def test_row_subset_and_explicit_permutation():
    r = _rng(46)
    W = r.standard_normal((10, 32)) * 0.02
    H = _spd(32, 47, cond_boost=8.0)
    f = oc.hessian_factor(H, 0.01, act_order=True)
    p = f["perm"]
    full = oc.quantize_layer(W, f["U"], 3, 8, perm=p)
    sub = oc.quantize_layer(W, f["U"], 3, 8, perm=p, rows=[7, 2])
    np.testing.assert_array_equal(sub["Q"], full["Q"][[7, 2]])
    np.testing.assert_array_equal(sub["W_hat"], full["W_hat"][[7, 2]])
    # running on pre-permuted inputs in natural order, then un-permuting, is the same thing
    pre = oc.quantize_layer(W[:, p], f["U"], 3, 8)
    Q = np.zeros_like(pre["Q"])
    Q[:, p] = pre["Q"]
    np.testing.assert_array_equal(Q, full["Q"])
    np.testing.assert_array_equal(pre["scales"], full["scales"])
    assert np.isclose(full["loss"], oc.layer_loss(W, full["W_hat"], f["Hd"]), rtol=1e-9)


def test_feedback_lowers_the_objective_against_rtn_on_correlated_inputs():
    # Not an identity, but the reason the method exists: with a strongly
    # non-diagonal Hessian the sweep's objective is below plain rounding's.
    r = _rng(48)
    Z = r.standard_normal((400, 32))
    X = Z @ (np.eye(32) + 0.6 * r.standard_normal((32, 32)))
    W = r.standard_normal((64, 32)) * 0.02
    f = oc.hessian_factor(oc.hessian_accumulate(X), 0.01)
    out = oc.quantize_layer(W, f["U"], 3, 32)
    rtn = oc.rtn_quantize(W, 3, 32)
    assert out["loss"] < oc.layer_loss(W, rtn[3], f["Hd"])


def test_brute_force_4x4_two_bit():
    # d_out = d_in = 4, one group of 4 (grid fixed by the original row), b = 2.
    r = _rng(49)
    W = r.standard_normal((4, 4))
    H = _spd(4, 50, cond_boost=2.0)
    f = oc.hessian_factor(H, 0.01)
    U, Hd = f["U"], f["Hd"]
    greedy = oc.quantize_layer(W, U, 2, 4)
    all_codes = np.array(list(itertools.product(range(4), repeat=4)))        # 256 x 4
    for row in range(4):
        Wr = np.repeat(W[row][None, :], 256, axis=0)
        forced = oc.quantize_layer(Wr, U, 2, 4, forced_codes=all_codes)
        # (i) sequential sum of squares == direct quadratic form for every code vector
        s, z = forced["scales"][:, 0:1], forced["zeros"][:, 0:1]
        What = s * (all_codes - z)
        quad = (((Wr - What) @ Hd) * (Wr - What)).sum(axis=1)
        np.testing.assert_allclose(forced["loss_rows"], quad, rtol=1e-10)
        # (iii) the exhaustive minimum is not above the greedy value
        assert quad.min() <= greedy["loss_rows"][row] * (1 + 1e-12)
        # (ii) each greedy code minimises e_j^2 over the 4 codes given the greedy prefix
        gq = greedy["Q"][row]
        for j in range(4):
            best, best_e = None, None
            for c in range(4):
                fc = -np.ones((1, 4), dtype=np.int64)
                fc[0, :j] = gq[:j]
                fc[0, j] = c
                e = oc.quantize_layer(W[row][None, :], U, 2, 4, forced_codes=fc)["E"][0, j]
                if best is None or e * e < best_e:
                    best, best_e = c, e * e
            assert best == gq[j]
    # with a diagonal Hessian greedy IS the exhaustive optimum
    fd = oc.hessian_factor(np.diag(np.diag(H)), 0.01)
    gd = oc.quantize_layer(W, fd["U"], 2, 4)
    for row in range(4):
        Wr = np.repeat(W[row][None, :], 256, axis=0)
        forced = oc.quantize_layer(Wr, fd["U"], 2, 4, forced_codes=all_codes)
        k = int(np.argmin(forced["loss_rows"]))
        assert np.isclose(forced["loss_rows"][k], gd["loss_rows"][row], rtol=1e-12)
        np.testing.assert_array_equal(all_codes[k], gd["Q"][row])


def test_forced_zero_point_is_honoured():
    r = _rng(51)
    W = r.standard_normal((3, 16)) * 0.02
    f = oc.hessian_factor(_spd(16, 52), 0.01)
    base = oc.quantize_layer(W, f["U"], 4, 8)
    fz = -np.ones((3, 2), dtype=np.int64)
    fz[1, 1] = int(base["zeros"][1, 1]) + 1
    out = oc.quantize_layer(W, f["U"], 4, 8, forced_zeros=fz)
    assert out["zeros"][1, 1] == base["zeros"][1, 1] + 1
    np.testing.assert_array_equal(out["Q"][[0, 2]], base["Q"][[0, 2]])
    np.testing.assert_array_equal(out["Q"][1, :8], base["Q"][1, :8])
