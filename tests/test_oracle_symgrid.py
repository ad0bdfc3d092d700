"""Pins for the oracle's symmetric grid (Sec. 2.3.2, Eq. (3)): z fixed, signed codes, s = max|w| / (2^(b-1) - 1)."""
import numpy as np
import pytest

from oracle import onecomp_oracle as oc


def _sym_by_hand(w, bits):
    """Eq. (3) written with signed codes, one group."""
    qs = 2 ** (bits - 1) - 1
    s = max(abs(w.min()), abs(w.max())) / qs
    q = np.clip(np.rint(w / s), -qs, qs)
    return q, s * q, s


@pytest.mark.parametrize("bits", [2, 3, 4, 8])
def test_symmetric_rtn_matches_eq3_with_signed_codes(bits):
    r = np.random.default_rng(bits)
    W = 0.02 * r.standard_normal((5, 64))
    Q, S, Z, What = oc.rtn_quantize(W, bits, 32, grid="sym")
    qs = 2 ** (bits - 1) - 1
    assert np.all(Z == qs)
    assert Q.min() >= 0 and Q.max() <= 2 * qs            # the top unsigned code stays unused
    for row in range(5):
        for g in range(2):
            q, wh, s = _sym_by_hand(W[row, 32 * g:32 * g + 32], bits)
            np.testing.assert_array_equal(Q[row, 32 * g:32 * g + 32] - qs, q)
            np.testing.assert_allclose(What[row, 32 * g:32 * g + 32], wh, rtol=1e-15)
            assert abs(S[row, g] - s) <= 1e-18
    np.testing.assert_allclose(oc.dequantize(Q, S, Z, 32), What, rtol=1e-15)


def test_symmetric_grid_properties():
    r = np.random.default_rng(7)
    W = r.standard_normal((6, 48))
    Q, S, Z, What = oc.rtn_quantize(W, 4, 16, grid="sym")
    Qn, Sn, Zn, Whn = oc.rtn_quantize(-W, 4, 16, grid="sym")
    # odd symmetry: -w gives mirrored codes and -w^ (round half to even is odd)
    np.testing.assert_array_equal(Qn, 2 * 7 - Q)
    np.testing.assert_array_equal(Whn, -What)
    np.testing.assert_array_equal(Sn, S)
    # the element of largest magnitude in a group is reproduced (it sits on the end of the grid)
    Wg = W.reshape(6, 3, 16)
    idx = np.abs(Wg).argmax(axis=2)
    big = np.take_along_axis(Wg, idx[:, :, None], axis=2)[:, :, 0]
    bigh = np.take_along_axis(What.reshape(6, 3, 16), idx[:, :, None], axis=2)[:, :, 0]
    np.testing.assert_allclose(bigh, big, rtol=1e-12)
    # zero is a grid point; inside the range the error is at most s / 2
    W0 = W.copy(); W0[:, 5] = 0.0
    _, S0, _, Wh0 = oc.rtn_quantize(W0, 4, 16, grid="sym")
    assert np.all(Wh0[:, 5] == 0.0)
    assert np.all(np.abs(W0 - Wh0) <= 0.5 * np.repeat(S0, 16, axis=1) * (1 + 1e-12))
    # weights that lie on a symmetric grid are reproduced exactly
    s0 = 0.013
    Wgrid = s0 * r.integers(-7, 8, size=(4, 32)).astype(np.float64)
    Wgrid[:, 0] = 7 * s0
    _, _, _, Whg = oc.rtn_quantize(Wgrid, 4, 32, grid="sym")
    np.testing.assert_allclose(Whg, Wgrid, rtol=1e-12, atol=1e-15)
    # all-zero group: s = 1, codes at the zero-point
    Qz, Sz, Zz, Whz = oc.rtn_quantize(np.zeros((2, 16)), 3, 16, grid="sym")
    assert np.all(Sz == 1.0) and np.all(Qz == 3) and np.all(Whz == 0.0)


def test_symmetric_sweep_special_cases():
    r = np.random.default_rng(11)
    d_out, d_in, G, bits = 6, 64, 16, 4
    W = 0.02 * r.standard_normal((d_out, d_in))
    # diagonal Hessian: no coupling, the sweep is round-to-nearest on the symmetric grid
    Hdiag = np.diag(r.uniform(0.5, 2.0, d_in))
    f = oc.hessian_factor(Hdiag, 0.0)
    out = oc.quantize_layer(W, f["U"], bits, G, grid="sym")
    Q, S, Z, What = oc.rtn_quantize(W, bits, G, grid="sym")
    np.testing.assert_array_equal(out["Q"], Q)
    np.testing.assert_allclose(out["W_hat"], What, rtol=1e-13)
    np.testing.assert_array_equal(out["zeros"], Z)
    # general Hessian: loss identity and dequantization from the returned arrays
    X = r.standard_normal((200, d_in))
    H = oc.hessian_accumulate(X)
    f = oc.hessian_factor(H, 0.01)
    out = oc.quantize_layer(W, f["U"], bits, G, grid="sym")
    assert abs(out["loss"] - oc.layer_loss(W, out["W_hat"], f["Hd"])) <= 1e-9 * out["loss"]
    np.testing.assert_allclose(oc.dequantize(out["Q"], out["scales"], out["zeros"], G), out["W_hat"], rtol=1e-14)
    assert np.all(out["zeros"] == 7) and out["Q"].max() <= 14
    # each step picks the nearest symmetric grid point of the compensated value (clipped to the signed range)
    t = out["T"]
    np.testing.assert_array_equal(out["Q"] - 7, np.clip(np.rint(t), -7, 7).astype(np.int64))
