"""Pins for the form of the sweep that needs one Cholesky factor only (oracle.direct_factor /
block_feedback_factor / quantize_layer_direct).

The paper's sweep (Sec. 4.3) propagates e_j U_jk with U^T U = (H + lambda I)^-1.  The direct form uses
R = U^-1 instead; it must reproduce the sweep's codes, grid parameters and loss.  The pins below fix R by what
defines it (triangular, positive diagonal, R R^T = Hd, R U = I with U from the independent two-Cholesky route),
the closed form of the 2 x 2 case, and the sweep identity on random layers, act-order and both grids included.
"""
import numpy as np
import pytest

from oracle import onecomp_oracle as oc


def _spd(n, seed, cond=50.0):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((3 * n, n)) * np.linspace(1.0, np.sqrt(cond), n)[None, :]
    A[:, 1:] += 0.6 * A[:, :-1]
    return 2.0 * A.T @ A


@pytest.mark.parametrize("n,seed", [(1, 0), (2, 1), (7, 2), (64, 3), (130, 4)])
def test_direct_factor_defining_properties(n, seed):
    Hd, _ = oc.damp_hessian(_spd(n, seed), 0.01)
    R, info = oc.direct_factor(Hd)
    assert info == 0
    assert np.allclose(R, np.triu(R)) and (np.diag(R) > 0).all()
    assert np.abs(R @ R.T - Hd).max() <= 1e-12 * np.abs(Hd).max()
    U, _ = oc.inverse_factor(Hd)            # independent route: Cholesky, inverse, Cholesky
    assert np.abs(R @ U - np.eye(n)).max() <= 1e-9
    assert np.abs(U @ R - np.eye(n)).max() <= 1e-9


def test_direct_factor_two_by_two_closed_form():
    a, b, c = 5.0, 3.0, 1.5
    R, _ = oc.direct_factor(np.array([[a, c], [c, b]]))
    # R = [[r00, r01], [0, r11]],  R R^T = [[r00^2 + r01^2, r01 r11], [r01 r11, r11^2]]
    r11 = np.sqrt(b)
    r01 = c / r11
    r00 = np.sqrt(a - r01 * r01)
    assert np.allclose(R, [[r00, r01], [0.0, r11]], rtol=1e-14, atol=0)


def test_direct_factor_diagonal_matrix():
    d = np.array([4.0, 9.0, 0.25])
    R, _ = oc.direct_factor(np.diag(d))
    assert np.allclose(R, np.diag(np.sqrt(d)), rtol=1e-15, atol=0)
    U, _ = oc.inverse_factor(np.diag(d))
    F = oc.block_feedback_factor(U, R, 2)
    assert np.allclose(F, np.diag(1.0 / np.sqrt(d)), rtol=1e-15, atol=0)


def test_direct_factor_reports_bad_pivot():
    H = np.array([[1.0, 2.0], [2.0, 1.0]])
    R, info = oc.direct_factor(H)
    assert R is None and info > 0


def test_block_feedback_factor_entries():
    n, B = 12, 4
    Hd, _ = oc.damp_hessian(_spd(n, 11), 0.01)
    R, _ = oc.direct_factor(Hd)
    U, _ = oc.inverse_factor(Hd)
    F = oc.block_feedback_factor(U, R, B)
    for j in range(n):
        for k in range(n):
            if k < j:
                assert F[j, k] == 0.0
            elif j // B == k // B:
                assert F[j, k] == U[j, k]
            else:
                assert F[j, k] == pytest.approx(-U[j, j] * R[j, k] / R[k, k], rel=1e-14)
    # diagonal blocks of U are the inverses of the diagonal blocks of R: nothing else of U is needed
    for b0 in range(0, n, B):
        assert np.abs(U[b0:b0 + B, b0:b0 + B] @ R[b0:b0 + B, b0:b0 + B] - np.eye(B)).max() <= 1e-10
    # a sweep that normalizes a row by its diagonal entry sees -R_jk / R_kk outside the blocks
    assert F[1, 9] / F[1, 1] == pytest.approx(-R[1, 9] / R[9, 9], rel=1e-14)


def test_state_on_entering_a_block():
    """w_B - e_A U_AB = w_B + (w_A - w^_A) R_AB U_BB: checked with explicit matrices on the errors of the sweep."""
    rng = np.random.default_rng(21)
    n, a = 24, 10
    f = oc.hessian_factor(_spd(n, 22), 0.01)
    R, _ = oc.direct_factor(f["Hd"])
    W = rng.standard_normal((4, n))
    ref = oc.quantize_layer(W, f["U"], 3, 2)
    e_A = ref["E"][:, :a]
    dev_A = (W - ref["W_hat"])[:, :a]
    lhs = W[:, a:] - e_A @ f["U"][:a, a:]
    rhs = W[:, a:] + dev_A @ R[:a, a:] @ f["U"][a:, a:]
    assert np.abs(lhs - rhs).max() <= 1e-11


def test_error_identity_of_the_sweep():
    """e = (w - w^) R for the errors of the paper's sweep: the relation the direct form rests on."""
    rng = np.random.default_rng(5)
    n = 48
    H = _spd(n, 6)
    f = oc.hessian_factor(H, 0.01)
    W = rng.standard_normal((6, n))
    ref = oc.quantize_layer(W, f["U"], 3, 16)
    R, _ = oc.direct_factor(f["Hd"])
    E = (W - ref["W_hat"]) @ R
    assert np.abs(E - ref["E"]).max() <= 1e-10 * max(1.0, np.abs(ref["E"]).max())


@pytest.mark.parametrize("bits,G,block,grid,act", [
    (4, 16, 16, "asym", False), (3, 16, 32, "asym", True), (2, 64, 64, "asym", False), (4, 8, 32, "sym", False),
    (3, 32, 64, "sym", True), (4, 32, 32, "asym", True), (4, 16, 64, "asym", False)])
def test_direct_sweep_reproduces_the_sweep(bits, G, block, grid, act):
    rng = np.random.default_rng(100 + bits + G)
    n, rows = 64, 24
    H = _spd(n, 7 + bits)
    f = oc.hessian_factor(H, 0.01, act_order=act)
    W = rng.standard_normal((rows, n)) * 0.05
    ref = oc.quantize_layer(W, f["U"], bits, G, perm=f["perm"], grid=grid)
    Hp = f["Hd"][np.ix_(f["perm"], f["perm"])]
    R, info = oc.direct_factor(Hp)
    assert info == 0
    got = oc.quantize_layer_direct(W, R, bits, G, block, perm=f["perm"], grid=grid)
    # both run in float64: the two forms differ by rounding at the 1e-16 level, so codes can only differ where a
    # pre-rounding value sits within ~1e-12 of a half-integer; none does for these seeds
    assert (got["Q"] == ref["Q"]).all()
    assert np.allclose(got["scales"], ref["scales"], rtol=1e-11, atol=0)
    assert (got["zeros"] == ref["zeros"]).all()
    assert np.allclose(got["W_hat"], ref["W_hat"], rtol=1e-11, atol=1e-15)
    assert got["loss"] == pytest.approx(ref["loss"], rel=1e-9)
    # and the loss is the layer objective on the damped matrix
    assert got["loss"] == pytest.approx(oc.layer_loss(W, got["W_hat"], f["Hd"]), rel=1e-9)


def test_direct_sweep_diagonal_hessian_is_rtn():
    rng = np.random.default_rng(9)
    W = rng.standard_normal((5, 32))
    Hd = np.diag(rng.uniform(0.5, 2.0, 32))
    R, _ = oc.direct_factor(Hd)
    got = oc.quantize_layer_direct(W, R, 4, 8, 16)
    Q, s, z, What = oc.rtn_quantize(W, 4, 8)
    assert (got["Q"] == Q).all() and np.array_equal(got["W_hat"], What)
