"""Pins of the oracle's JointQ local search (Sec. 4.3.2, Eq. (jointq)): hand-worked moves, the gain formula against
least squares on the data matrix itself, monotone descent, scale optimality, local optimality at convergence,
brute force over every code assignment of a tiny group, and the regularizer as an augmented input (Eq. (jointq_reg))."""
import itertools
import json
import os

import numpy as np
import pytest

from oracle import onecomp_oracle as oc

HERE = os.path.dirname(os.path.abspath(__file__))


def _problem(seed, n_rows, d_in, G, bits, n_tok=None, grid="asym"):
    rng = np.random.default_rng(seed)
    n_tok = n_tok or 3 * d_in
    X = rng.standard_normal((n_tok, d_in))
    X[:, 1:] += 0.6 * X[:, :-1]
    W = rng.standard_normal((n_rows, d_in)) * 0.05
    H = oc.hessian_accumulate(X)
    Q, s, z, _ = oc.rtn_quantize(W, bits, G, grid)
    return X, W, H, Q, s, z


def _lstsq_objective(X, w, q, s, z, G, t):
    """Objective 2 |X w - X w^|^2 after refitting the scale of group t by least squares on the data."""
    u = np.zeros_like(w)
    u[t * G:(t + 1) * G] = q[t * G:(t + 1) * G] - z[t]
    others = np.repeat(s, G) * (q - np.repeat(z, G))
    others[t * G:(t + 1) * G] = 0.0
    y = X @ (w - others)
    v = X @ u
    st = np.linalg.lstsq(v[:, None], y, rcond=None)[0][0] if np.any(v) else 0.0
    return 2.0 * float(((y - st * v) ** 2).sum()), st


def test_hand_worked_cases():
    g = json.load(open(os.path.join(HERE, "golden", "jointq_hand_worked.json")))
    A = np.array(g["A"])
    for c in g["cases"]:
        o = oc.jointq_refine(np.array([c["w"]]), A, np.array([g["q0"]]), np.array([[g["s0"]]]), np.array([[g["z"]]]),
                             g["bits"], g["group_size"], n_pass=2, max_scans=4)
        assert o["Q"][0].tolist() == c["q"]
        assert o["scales"][0, 0] == c["s"]
        assert o["f0"][0] == c["f0"] and abs(o["f1"][0] - c["f1"]) < 1e-15
        assert o["moves"][0] == c["moves"]


def test_single_visit_matches_least_squares_on_the_data():
    """Replays one visit move by move with the objective evaluated from X by lstsq: the first improving move of
    the scan (+1 before -1) must be the one the oracle takes, and the refit scale must be the lstsq scale."""
    X, W, H, Q, s, z = _problem(1, 3, 16, 8, 3)
    for t in range(2):
        o = oc.jointq_refine(W, H, Q, s, z, 3, 8, n_pass=1, max_scans=1)
        # reference: group 0 then group 1, one scan each, by brute force on the data
        Qr, sr = Q.astype(np.float64).copy(), s.copy()
        for i in range(3):
            for tt in range(2):
                f_cur, st = _lstsq_objective(X, W[i], Qr[i], sr[i], z[i], 8, tt)
                if not np.any(Qr[i, tt * 8:(tt + 1) * 8] - z[i, tt]):
                    continue
                sr[i, tt] = st
                for j in range(tt * 8, tt * 8 + 8):
                    for d in (1.0, -1.0):
                        if not 0 <= Qr[i, j] + d <= 7:
                            continue
                        Qr[i, j] += d
                        f_new, st_new = _lstsq_objective(X, W[i], Qr[i], sr[i], z[i], 8, tt)
                        if f_new < f_cur * (1 - 1e-13) and np.any(Qr[i, tt * 8:(tt + 1) * 8] - z[i, tt]):
                            f_cur, sr[i, tt] = f_new, st_new
                            break
                        Qr[i, j] -= d
        assert np.array_equal(o["Q"], Qr.astype(np.int64))
        assert np.allclose(o["scales"], sr, rtol=1e-10)


def test_objective_never_rises_and_matches_the_definition():
    X, W, H, Q, s, z = _problem(2, 6, 64, 16, 3)
    prev = oc.row_objective(W, oc.dequantize(Q, s, z, 16), H)
    assert np.allclose(prev, 2.0 * ((X @ (W - oc.dequantize(Q, s, z, 16)).T) ** 2).sum(axis=0), rtol=1e-10)
    cur_Q, cur_s = Q, s
    for _ in range(3):
        o = oc.jointq_refine(W, H, cur_Q, cur_s, z, 3, 16, n_pass=1, max_scans=3)
        assert np.allclose(o["f0"], prev, rtol=1e-12)
        assert np.all(o["f1"] <= prev * (1 + 1e-12))
        assert np.allclose(o["f1"], oc.row_objective(W, oc.dequantize(o["Q"], o["scales"], z, 16), H), rtol=1e-12)
        assert np.array_equal(o["W_hat"], oc.dequantize(o["Q"], o["scales"], z, 16))
        prev, cur_Q, cur_s = o["f1"], o["Q"], o["scales"]
    assert (o["f1"] < 0.9 * oc.row_objective(W, oc.dequantize(Q, s, z, 16), H)).all()   # and it helps
    assert o["Q"].min() >= 0 and o["Q"].max() <= 7


def test_passes_compose():
    X, W, H, Q, s, z = _problem(3, 4, 32, 8, 4)
    two = oc.jointq_refine(W, H, Q, s, z, 4, 8, n_pass=2, max_scans=2)
    one = oc.jointq_refine(W, H, Q, s, z, 4, 8, n_pass=1, max_scans=2)
    again = oc.jointq_refine(W, H, one["Q"], one["scales"], z, 4, 8, n_pass=1, max_scans=2)
    assert np.array_equal(two["Q"], again["Q"]) and np.allclose(two["scales"], again["scales"], rtol=1e-12)


def test_converged_state_is_a_local_optimum_with_optimal_scales():
    X, W, H, Q, s, z = _problem(4, 3, 24, 8, 3)
    o = oc.jointq_refine(W, H, Q, s, z, 3, 8, n_pass=60, max_scans=50)
    o2 = oc.jointq_refine(W, H, o["Q"], o["scales"], z, 3, 8, n_pass=1, max_scans=1)
    assert o2["moves"].sum() == 0                       # converged
    for i in range(3):
        f_here = float(o["f1"][i])
        r = W[i] - o["W_hat"][i]
        for t in range(3):
            u = o["Q"][i, t * 8:(t + 1) * 8] - z[i, t]
            assert abs(u @ (H @ r)[t * 8:(t + 1) * 8]) <= 1e-9 * abs(f_here) + 1e-12   # d f / d s_t = 0
            for j in range(t * 8, t * 8 + 8):
                for d in (1, -1):
                    q2 = o["Q"][i].astype(np.float64).copy()
                    q2[j] += d
                    if not 0 <= q2[j] <= 7:
                        continue
                    f_new, _ = _lstsq_objective(X, W[i], q2, o["scales"][i], z[i], 8, t)
                    assert f_new >= f_here * (1 - 1e-10)


def test_tiny_group_against_every_assignment():
    """One group of 4 columns at 2 bits: 256 assignments, each with its least-squares scale.  The search, started
    from the best assignment, must stay there; started from RTN it must end at a local optimum no worse than its
    start and no better than the global optimum."""
    X, W, H, Q, s, z = _problem(5, 5, 4, 4, 2, n_tok=12)
    for i in range(5):
        best, best_q = np.inf, None
        for q in itertools.product(range(4), repeat=4):
            q = np.array(q, dtype=np.float64)
            if not np.any(q - z[i, 0]):
                continue
            f, _ = _lstsq_objective(X, W[i], q, s[i], z[i], 4, 0)
            if f < best:
                best, best_q = f, q
        o = oc.jointq_refine(W[i:i + 1], H, best_q[None, :], s[i:i + 1], z[i:i + 1], 2, 4, n_pass=3, max_scans=5)
        assert np.array_equal(o["Q"][0], best_q.astype(np.int64)) and abs(o["f1"][0] - best) <= 1e-9 * best + 1e-15
        o = oc.jointq_refine(W[i:i + 1], H, Q[i:i + 1], s[i:i + 1], z[i:i + 1], 2, 4, n_pass=3, max_scans=5)
        assert best * (1 - 1e-9) <= o["f1"][0] <= o["f0"][0] * (1 + 1e-12)


def test_regularizer_is_an_augmented_input():
    """Eq. (jointq_reg): |XW - XW^|^2 + n lam |W - W^|^2 is the plain objective for X stacked on sqrt(n lam) I."""
    X, W, H, Q, s, z = _problem(6, 3, 16, 8, 3)
    n_lam = 0.37 * X.shape[0]
    Xa = np.vstack([X, np.sqrt(n_lam) * np.eye(16)])
    a = oc.jointq_refine(W, oc.hessian_accumulate(Xa), Q, s, z, 3, 8, n_pass=2)
    b = oc.jointq_refine(W, H + 2.0 * n_lam * np.eye(16), Q, s, z, 3, 8, n_pass=2)
    assert np.array_equal(a["Q"], b["Q"]) and np.allclose(a["scales"], b["scales"], rtol=1e-10)


def test_symmetric_grid_zero_group_rows_subset_and_forced_decisions():
    X, W, H, Q, s, z = _problem(7, 6, 32, 16, 3, grid="sym")
    W = W.copy()
    W[2, :16] = 0.0
    Q, s, z, _ = oc.rtn_quantize(W, 3, 16, "sym")
    o = oc.jointq_refine(W, H, Q, s, z, 3, 16, grid="sym", n_pass=2, tie_tol=0.05)
    assert o["Q"].max() <= 6 and o["Q"].min() >= 0            # the top code of the symmetric grid stays unused
    assert np.array_equal(o["Q"][2, :16], Q[2, :16]) and o["scales"][2, 0] == s[2, 0]   # all codes at the zero-point
    sub = oc.jointq_refine(W, H, Q, s, z, 3, 16, grid="sym", n_pass=2, rows=[4, 1])
    assert np.array_equal(sub["Q"], o["Q"][[4, 1]]) and np.array_equal(sub["scales"], o["scales"][[4, 1]])
    # flipping a recorded near-tie changes that decision and nothing before it
    row = next(i for i in range(6) if o["ties"][i])
    key, taken = o["ties"][row][0][:5], o["ties"][row][0][5]
    f = oc.jointq_refine(W, H, Q, s, z, 3, 16, grid="sym", n_pass=2, rows=[row], forced={(0,) + key: True})
    g = oc.jointq_refine(W, H, Q, s, z, 3, 16, grid="sym", n_pass=2, rows=[row], forced={(0,) + key: False})
    assert not (np.array_equal(f["Q"], g["Q"]) and np.array_equal(f["scales"], g["scales"]))
    same = f if taken else g                      # forcing a decision the way it fell changes nothing
    assert np.array_equal(same["Q"][0], o["Q"][row]) and np.allclose(same["scales"][0], o["scales"][row], rtol=1e-12)


def test_column_order_is_the_search_on_permuted_inputs():
    """jointq_refine(perm=p) is the search run on W[:, p], A[p][:, p], Q[:, p] in natural order, un-permuted: groups,
    scan order, scales and zeros follow the sweep's column order, W, A, Q and W_hat stay in the original one."""
    X, W, H, _, _, _ = _problem(11, 5, 48, 16, 3)
    rng = np.random.default_rng(12)
    p = rng.permutation(48)
    # a start in the format the sweep returns under a column order: groups are runs of the permuted order
    Qp, s, z, _ = oc.rtn_quantize(W[:, p], 3, 16)
    Q = np.empty_like(Qp)
    Q[:, p] = Qp
    a = oc.jointq_refine(W, H, Q, s, z, 3, 16, n_pass=2, max_scans=3, perm=p, tie_tol=1e-3)
    b = oc.jointq_refine(W[:, p], H[np.ix_(p, p)], Qp, s, z, 3, 16, n_pass=2, max_scans=3, tie_tol=1e-3)
    assert a["moves"].sum() > 0
    assert np.array_equal(a["Q"][:, p], b["Q"]) and np.array_equal(a["scales"], b["scales"])
    assert np.array_equal(a["W_hat"][:, p], b["W_hat"])
    assert np.array_equal(a["moves"], b["moves"]) and a["ties"] == b["ties"]
    assert np.allclose(a["f0"], b["f0"], rtol=1e-13) and np.allclose(a["f1"], b["f1"], rtol=1e-13)
    # the returned arrays mean what they say in the ORIGINAL order, independently of how perm is implemented
    assert np.array_equal(a["W_hat"], oc.dequantize(a["Q"], a["scales"], z, 16, perm=p))
    assert np.allclose(a["f1"], 2.0 * ((X @ (W - a["W_hat"]).T) ** 2).sum(axis=0), rtol=1e-10)
    # and a different order gives a different search (the order matters)
    c = oc.jointq_refine(W, H, Q, s, z, 3, 16, n_pass=2, max_scans=3)
    assert not np.array_equal(a["Q"], c["Q"])


def _first_decision_terms(X, W, H, Q, s, z, G, i):
    """Row i, first decision of the search (pass 0, group 0, scan 0, column 0, +1), from the definitions: the gain
    N = c' (f_before - f_after) with both objectives by least squares on the data, and the two sums the listing
    rule weighs (sum_k |r_k| |A_k0| and |s*| sum_k |u_k| |A_k0| over the group)."""
    q = Q[i].astype(np.float64)
    f_before, st = _lstsq_objective(X, W[i], q, s[i], z[i], G, 0)
    q2 = q.copy()
    q2[0] += 1.0
    f_after, _ = _lstsq_objective(X, W[i], q2, s[i], z[i], G, 0)
    u2 = q2[:G] - z[i, 0]
    c_new = float(u2 @ H[:G, :G] @ u2)
    r = W[i] - np.repeat(s[i], G) * (q - np.repeat(z[i], G))
    u = q[:G] - z[i, 0]
    b = float(u @ (H[:G] @ r + s[i, 0] * (H[:G, :G] @ u)))
    g_sum = float(np.abs(r) @ np.abs(H[:, 0]))
    a_sum = abs(st) * float(np.abs(u) @ np.abs(H[:G, 0]))
    return c_new * (f_before - f_after), b, g_sum, a_sum


def test_listing_tolerances_only_list_and_forcing_a_listed_decision_changes_only_it():
    """tie_tol / g_tol / a_tol decide which decisions are LISTED as toss-ups, never the result; the list grows with
    each tolerance; a decision that only g_tol (or a_tol) lists can be forced the other way, and then every decision
    before it is the same and that one is not; for the first decision of a row the listing rule is evaluated from
    the definitions (least squares on the data)."""
    X, W, H, Q, s, z = _problem(13, 8, 32, 16, 3)
    kw = dict(bits=3, group_size=16, n_pass=1, max_scans=2)
    plain = oc.jointq_refine(W, H, Q, s, z, **kw)
    runs = {}
    for name, tol in (("t", dict(tie_tol=1e-9)), ("tg", dict(tie_tol=1e-9, g_tol=3e-3)),
                      ("ta", dict(tie_tol=1e-9, a_tol=3e-3)), ("tga", dict(tie_tol=1e-9, g_tol=3e-3, a_tol=3e-3)),
                      ("big", dict(tie_tol=1e-9, g_tol=1e9))):
        o = oc.jointq_refine(W, H, Q, s, z, **kw, **tol)
        assert np.array_equal(o["Q"], plain["Q"]) and np.array_equal(o["scales"], plain["scales"])
        runs[name] = [set(t[:5] for t in row) for row in o["ties"]]
        assert all(len(set(t[:5] for t in row)) == len(row) for row in o["ties"])      # a decision is listed once
    for i in range(8):
        assert runs["t"][i] <= runs["tg"][i] <= runs["tga"][i] and runs["t"][i] <= runs["ta"][i] <= runs["tga"][i]
        assert runs["tga"][i] <= runs["big"][i]
    assert sum(len(r) for r in runs["tg"]) > sum(len(r) for r in runs["t"])
    assert sum(len(r) for r in runs["ta"]) > sum(len(r) for r in runs["t"])
    # an unbounded tolerance lists every decision that was evaluated: at least one per column and scan entered
    assert all(len(r) >= 32 for r in runs["big"])
    # the rule itself, on the first decision of every row, from the definitions
    for i in range(8):
        if not np.any(Q[i, :16] - z[i, 0]) or Q[i, 0] + 1 > 7:
            continue
        N, b, g_sum, a_sum = _first_decision_terms(X, W, H, Q, s, z, 16, i)
        key = (0, 0, 0, 0, 1)
        for g_tol, a_tol in ((3e-3, 0.0), (0.0, 3e-3), (1e-5, 1e-5), (0.3, 0.0)):
            o = oc.jointq_refine(W, H, Q, s, z, rows=[i], tie_tol=1e-300, g_tol=g_tol, a_tol=a_tol, **kw)
            bound = 2.0 * abs(b) * (g_tol * g_sum + a_tol * a_sum)
            if abs(abs(N) - bound) > 1e-6 * bound:                      # away from the edge of the rule
                assert (key in set(t[:5] for t in o["ties"][0])) == (abs(N) <= bound), (i, N, bound)
    # forcing a decision that only g_tol (resp. a_tol) lists; one scan, so that no later scan can undo the move and
    # the code of that column shows the decision
    kw1 = dict(bits=3, group_size=16, n_pass=1, max_scans=1)
    for name in ("tg", "ta"):
        tol = dict(tie_tol=1e-9, g_tol=5e-2) if name == "tg" else dict(tie_tol=1e-9, a_tol=5e-2)
        listed = [set(t[:5] for t in row) for row in oc.jointq_refine(W, H, Q, s, z, **kw1, **tol)["ties"]]
        strict = [set(t[:5] for t in row) for row in oc.jointq_refine(W, H, Q, s, z, **kw1, tie_tol=1e-9)["ties"]]
        i = next(r for r in range(8) if listed[r] - strict[r])
        key = sorted(listed[i] - strict[i])[0]
        base = oc.jointq_refine(W, H, Q, s, z, rows=[i], **kw1, **tol)
        taken = {t[:5]: t[5] for t in base["ties"][0]}[key]
        flip = oc.jointq_refine(W, H, Q, s, z, rows=[i], forced={(0,) + key: not taken}, **kw1, **tol)
        before = [t for t in base["ties"][0] if t[:5] < key]
        assert [t for t in flip["ties"][0] if t[:5] < key] == before     # nothing before it changes
        col = key[1] * 16 + key[3]
        assert np.array_equal(flip["Q"][0, :col], base["Q"][0, :col])
        assert flip["Q"][0, col] != base["Q"][0, col]                    # and that decision does
        same = oc.jointq_refine(W, H, Q, s, z, rows=[i], forced={(0,) + key: taken}, **kw1, **tol)
        assert np.array_equal(same["Q"], base["Q"]) and np.array_equal(same["scales"], base["scales"])


def test_no_move_empties_a_group():
    """A group may not be brought to 'every code at its zero-point' (c' = 0: the refit scale is undefined there and the
    gain reaches 0 from below).  Checked where floating point alone would not settle it: a group with a single code
    away from the zero-point, reached after other moves so that c is a carried sum.  The emptying move is no candidate
    (not even a listed toss-up, and it cannot be forced), the group stays alive, and by the definition the objective
    with the group emptied is indeed no better than what the search returns."""
    rng = np.random.default_rng(3)
    d_in, G, bits = 8, 4, 2
    X = rng.standard_normal((40, d_in))
    X[:, 1:] += 0.7 * X[:, :-1]
    H = oc.hessian_accumulate(X)
    z = np.ones((1, 2))                                   # symmetric 2-bit grid: codes 0..2 around the zero-point 1
    s = np.full((1, 2), 0.05)
    # group 0 wants a single small weight on column 2; it starts with two codes away from the zero-point, so the
    # search first takes one of them back (c becomes a carried sum), and is then one move from emptying the group
    W = np.array([[0.0, 0.0, 0.004, 0.0, 0.05, -0.05, 0.05, 0.0]])
    Q = np.array([[1, 2, 2, 1, 2, 0, 2, 1]])
    o = oc.jointq_refine(W, H, Q, s, z, bits, G, grid="sym", n_pass=1, max_scans=6, tie_tol=1e-3, g_tol=1e-3)
    u0 = o["Q"][0, :G] - 1
    assert np.count_nonzero(u0) == 1                      # the search did reach the single-code state
    j = int(np.nonzero(u0)[0][0])
    d_empty = -int(u0[j])
    assert not any(t[1] == 0 and t[3] == j and t[4] == d_empty for t in o["ties"][0])
    forced = {(0, 0, 0, sc, j, d_empty): True for sc in range(6)}
    o2 = oc.jointq_refine(W, H, Q, s, z, bits, G, grid="sym", n_pass=1, max_scans=6, forced=forced)
    assert np.array_equal(o2["Q"], o["Q"]) and np.array_equal(o2["moves"], o["moves"])
    # by the definition: emptying the group does not lower the objective
    w_hat_empty = o["W_hat"].copy()
    w_hat_empty[0, :G] = 0.0
    assert oc.row_objective(W, w_hat_empty, H)[0] >= o["f1"][0]
