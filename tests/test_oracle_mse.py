"""Pins for the scale search of the sweep (oracle.mse_search and the scale_search="mse" option).

The paper names the option (Sec. 4.3, "MSE-based grid tuning (mse), which searches over candidate scales to minimize
the mean squared reconstruction error per-group") without a candidate set; this build's reading shrinks the observed
range by p_i = 1 - i / 100, i = 0 .. 79.  Pinned by hand-worked cases (tests/golden/mse_hand_worked.json), by the
special cases that reduce to the plain rule, by invariants, and against the independent whole-array routine."""
import json
import os

import numpy as np
import pytest

from oracle import onecomp_oracle as oc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "mse_hand_worked.json")


@pytest.mark.parametrize("case", json.load(open(GOLDEN))["cases"], ids=lambda c: c["name"])
def test_hand_worked_cases(case):
    w = np.array([case["w"]], dtype=np.float64)
    m = oc.mse_search(w, case["bits"], case["grid"], n_cand=case["n_cand"], step=case["step"])
    assert np.allclose(m["err"][0], case["err"], rtol=1e-12)
    assert int(m["cand"][0]) == case["cand"]
    assert m["s"][0] == pytest.approx(case["s"], rel=1e-14) and m["z"][0] == case["z"]
    q, wh, _ = oc.quantize_scalar(w[0], m["s"][0], m["z"][0], case["bits"], oc.code_range_top(case["bits"], case["grid"]))
    assert q.astype(int).tolist() == case["codes"]
    assert np.allclose(wh, case["w_hat"], rtol=1e-13, atol=1e-15)


@pytest.mark.parametrize("grid", ["asym", "sym"])
def test_candidate_zero_is_the_plain_rule(grid):
    rng = np.random.default_rng(1)
    v = rng.standard_normal((50, 32))
    m = oc.mse_search(v, 4, grid)
    params = oc.minmax_params if grid == "asym" else oc.symmetric_params
    s, z, _ = params(v.min(axis=1), v.max(axis=1), 4)
    assert np.array_equal(m["s_all"][:, 0], s) and np.array_equal(m["z_all"][:, 0], z)
    assert m["err"].shape == (50, oc.MSE_CANDIDATES)
    # the set: both ends shrunk by 1 - i / 100 (the scale is linear in the range for both grids)
    i = np.arange(oc.MSE_CANDIDATES)
    assert np.allclose(m["s_all"], s[:, None] * (1.0 - i / 100.0)[None, :], rtol=1e-12)


def test_values_on_a_grid_keep_the_full_range():
    rng = np.random.default_rng(2)
    s0, z0 = 0.037, 5.0
    q = rng.integers(0, 16, size=(20, 64)).astype(np.float64)
    q[:, 0] = 0.0
    q[:, 1] = 15.0                                # the range is exactly the grid's
    v = s0 * (q - z0)
    m = oc.mse_search(v, 4, "asym")
    assert (m["cand"] == 0).all()
    assert np.all(m["err"][:, 0] <= 1e-28)
    assert np.allclose(m["s"], s0, rtol=1e-12) and (m["z"] == z0).all()


def test_never_worse_than_the_plain_rule_and_argmin():
    rng = np.random.default_rng(3)
    W = rng.standard_normal((30, 128)) * 0.02
    W[:, 7] *= 9.0                                # an outlier column in the first group
    for grid in ("asym", "sym"):
        Q0, s0, z0, W0 = oc.rtn_quantize(W, 3, 32, grid)
        Q1, s1, z1, W1 = oc.rtn_quantize(W, 3, 32, grid, scale_search="mse")
        e0 = ((W - W0) ** 2).reshape(30, 4, 32).sum(axis=2)
        e1 = ((W - W1) ** 2).reshape(30, 4, 32).sum(axis=2)
        assert np.all(e1 <= e0 + 1e-18)
        assert (e1 < e0 - 1e-12).any()            # and it does find better grids somewhere
        assert np.all(s1 <= s0 * (1 + 1e-15)) and np.all(s1 >= 0.21 * s0 * (1 - 1e-12))
        m = oc.mse_search(W[:, :32], 3, grid)
        assert np.array_equal(m["err"][np.arange(30), m["cand"]], m["err"].min(axis=1))
        assert np.allclose(e1[:, 0], m["err"].min(axis=1), rtol=1e-12)


def test_scale_invariance():
    rng = np.random.default_rng(4)
    v = rng.standard_normal((10, 64))
    a = oc.mse_search(v, 4, "asym")
    b = oc.mse_search(4.0 * v, 4, "asym")        # a power of two: every operation scales exactly
    assert np.array_equal(a["cand"], b["cand"])
    assert np.array_equal(4.0 * a["s"], b["s"]) and np.array_equal(a["z"], b["z"])
    assert np.allclose(16.0 * a["err"], b["err"], rtol=1e-14)


def test_sweep_with_diagonal_hessian_is_the_searched_rtn():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((6, 64)) * 0.1
    Hd = np.diag(rng.uniform(0.5, 2.0, 64))
    U, _ = oc.inverse_factor(Hd)
    for grid in ("asym", "sym"):
        out = oc.quantize_layer(W, U, 4, 16, grid=grid, scale_search="mse")
        Q, s, z, What = oc.rtn_quantize(W, 4, 16, grid, scale_search="mse")
        assert (out["Q"] == Q).all() and np.array_equal(out["W_hat"], What)
        assert np.array_equal(out["scales"], s) and np.array_equal(out["zeros"], z)


def test_sweep_records_and_replays_candidates():
    rng = np.random.default_rng(6)
    n = 48
    A = rng.standard_normal((200, n))
    A[:, 1:] += 0.5 * A[:, :-1]
    f = oc.hessian_factor(2.0 * A.T @ A, 0.01)
    W = rng.standard_normal((5, n)) * 0.05
    out = oc.quantize_layer(W, f["U"], 3, 16, scale_search="mse")
    assert out["cand"].shape == (5, 3) and out["Ecand"].shape == (5, 3, oc.MSE_CANDIDATES)
    r = np.arange(5)
    for g in range(3):
        assert np.array_equal(out["scales"][:, g], out["Scand"][r, g, out["cand"][:, g]])
        assert np.array_equal(out["Ecand"][r, g, out["cand"][:, g]], out["Ecand"][:, g, :].min(axis=1))
    # loss identity still holds (the feedback does not care where the grid came from)
    assert out["loss"] == pytest.approx(oc.layer_loss(W, out["W_hat"], f["Hd"]), rel=1e-9)
    # forcing the recorded candidates reproduces the run; forcing another one changes that group's scale only
    fc = out["cand"].copy()
    again = oc.quantize_layer(W, f["U"], 3, 16, scale_search="mse", forced_cand=fc)
    assert (again["Q"] == out["Q"]).all()
    fc2 = -np.ones_like(fc)
    fc2[2, 1] = (out["cand"][2, 1] + 1) % oc.MSE_CANDIDATES
    other = oc.quantize_layer(W, f["U"], 3, 16, scale_search="mse", forced_cand=fc2)
    assert other["scales"][2, 1] != out["scales"][2, 1] and np.array_equal(other["scales"][2, 0], out["scales"][2, 0])
    assert np.array_equal(np.delete(other["Q"], 2, axis=0), np.delete(out["Q"], 2, axis=0))


@pytest.mark.parametrize("case", json.load(open(GOLDEN))["alt_cases"], ids=lambda c: c["name"][:40])
def test_other_neighbour_of_the_zero_point_hand_worked(case):
    """z_alt / err_alt (what the parity protocol may charge a candidate whose zero-point sits at a rounding tie)."""
    m = oc.mse_search(np.array([case["w"]], dtype=np.float64), case["bits"], case["grid"], n_cand=case["n_cand"],
                      step=case["step"])
    assert np.allclose(m["tz_all"][0], case["tz_all"], rtol=1e-12)
    assert m["z_all"][0].tolist() == case["z_all"] and m["z_alt"][0].tolist() == case["z_alt"]
    assert np.allclose(m["err"][0], case["err"], rtol=1e-12) and np.allclose(m["err_alt"][0], case["err_alt"], rtol=1e-12)
    assert int(m["cand"][0]) == case["cand"]


def test_other_neighbour_is_the_other_integer_next_to_tz():
    rng = np.random.default_rng(9)
    v = rng.standard_normal((200, 16)) + 0.3
    m = oc.mse_search(v, 3, "asym")
    tz, z, za = m["tz_all"], m["z_all"], m["z_alt"]
    inside = (tz > 0.0) & (tz < 7.0) & (np.abs(tz - np.rint(tz)) > 1e-9)
    assert inside.any()
    lo, hi = np.floor(tz), np.ceil(tz)
    assert np.all(((z == lo) & (za == hi) | (z == hi) & (za == lo))[inside])
    assert np.all(np.abs(tz - z)[inside] <= np.abs(tz - za)[inside])          # z is the nearer one
    # its error is the error of Eq. (1) on the grid (s, z_alt), recomputed here without the search
    for i, c in ((0, 0), (5, 17), (11, 79)):
        q = np.clip(np.rint(v[i] / m["s_all"][i, c]) + za[i, c], 0, 7)
        assert np.isclose(m["err_alt"][i, c], ((v[i] - m["s_all"][i, c] * (q - za[i, c])) ** 2).sum(), rtol=1e-12)
