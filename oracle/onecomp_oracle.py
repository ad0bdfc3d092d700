"""Float64 CPU oracle for layer-wise Hessian-aware quantization of one linear layer.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only the tests, the smoke check
and the benchmark's cpu_baseline leg may import it.  It shares no code with the
HIP library and must never be used as a fallback for it.

What it computes (paper sections given in brackets):

  * the calibration Gram / Hessian  H = 2 * X^T X  over token rows of X
    [Sec. 2.5 "Gram matrix H_l = X_l^T X_l"; Sec. 4.3 text after Eq. (layerwise);
     the factor 2 is the constant that makes it the Hessian of ||X(W^-W)||^2,
     cf. Sec. 2.4 "proportional, up to a constant factor, to the local Hessian"]
  * Tikhonov damping  lambda = eta * mean(diag H)  and a Cholesky-based factor
    of (H + lambda I)^-1  [Sec. 4.3.1, text after Eq. (qep)]
  * optional activation ordering: columns sorted by decreasing diag(H)
    [Sec. 4.3, "actorder"]
  * the column-by-column sweep: quantize one column to the per-group
    asymmetric min-max grid (or the symmetric grid of Eq. (3)), propagate its
    residual to the columns not yet quantized  [Sec. 4.3; grid: Eq. (1) scalar
    quantizer, Eq. (2) min-max scale / zero-point, Eq. (4) per-group layout]
  * the layer objective tr((W-W^) H (W-W^)^T)  [Eq. (layerwise), Eq. (activation-aware)]
  * the same sweep without the off-diagonal part of the inverse factor (direct_factor, block_feedback_factor,
    quantize_layer_direct): with R = U^-1, R R^T = H + lambda I, the propagated errors are e = (w - w^) R, so a
    blocked sweep can run on one Cholesky factor of the damped matrix itself and the inverses of its diagonal
    blocks  [a restatement of Sec. 4.3, derived in quantize_layer_direct]
  * the scale search of the sweep ("mse": per group, candidate ranges shrunk from the observed one, the smallest
    squared reconstruction error wins)  [Sec. 4.3; the candidate set is this build's reading, see mse_search]
  * JointQ's local search over codes with the group scale refit in the same move (jointq_refine)
    [Sec. 4.3.2, Eq. (jointq); order of moves and stopping are this build's reading, see the function]
  * the corrected quantization target of error propagation (QEP),
    W* = (I + alpha (H^ + lambda I)^-1 C) W  with  C = X^^T (X - X^)  [Sec. 4.3.1, Eq. (qep)]

Storage convention: W is d_out x d_in (rows = output channels), i.e. the
transpose of the paper's N x M matrix; "column j" is input channel j and a group
is G consecutive input channels inside one output row.

Everything is float64 and unblocked: one column at a time, rank-1 feedback, no
fusion or reordering.  numpy's matmul / Cholesky / triangular solve are used as
library steps.

Pinned by tests/test_oracle_*.py (closed forms, invariants, brute force, a
hand-worked grid example).  Functions without an external pin are marked
"parity unpinned" in their docstring.
"""
from __future__ import annotations

import numpy as np
from scipy.linalg import solve_triangular


# --------------------------------------------------------------------------
# Gram / Hessian
# --------------------------------------------------------------------------
def hessian_accumulate(X, H=None):
    """H + 2 * X^T X in float64 (Gram matrix of Sec. 2.5 / Sec. 4.3, times 2).

    X: [n_tokens, d_in] (any float dtype; widened exactly to float64).
    H: optional running sum [d_in, d_in]; a new array is returned either way.
    """
    X = np.asarray(X, dtype=np.float64)
    G = 2.0 * (X.T @ X)
    return G if H is None else np.asarray(H, dtype=np.float64) + G


def hessian_tile(X, idx_i, idx_k):
    """The sub-matrix H[idx_i][:, idx_k] of 2 * X^T X over all tokens of X."""
    X = np.asarray(X)
    Xi = np.asarray(X[:, idx_i], dtype=np.float64)
    Xk = np.asarray(X[:, idx_k], dtype=np.float64)
    return 2.0 * (Xi.T @ Xk)


# --------------------------------------------------------------------------
# Damping, ordering, inverse factor
# --------------------------------------------------------------------------
def damp_hessian(H, damp):
    """H_d = H + lambda I with lambda = damp * mean(diag H)  [Sec. 4.3.1].

    Reading for a dead input channel (H_jj == 0, on which the paper is silent):
    its diagonal entry is set to 1 before lambda is computed, which keeps H_d
    positive definite and gives that column no feedback.
    Returns (H_d, lambda).
    """
    Hd = np.array(H, dtype=np.float64, copy=True)
    d = np.diag(Hd).copy()
    dead = d == 0.0
    d[dead] = 1.0
    np.fill_diagonal(Hd, d)
    lam = float(damp) * float(d.sum() / d.shape[0])
    Hd[np.diag_indices_from(Hd)] += lam
    return Hd, lam


def act_order_perm(H):
    """Column order by decreasing diag(H); equal keys keep the lower index first
    [Sec. 4.3 "actorder"; the tie rule is this build's choice]."""
    d = np.diag(np.asarray(H, dtype=np.float64))
    return np.argsort(-d, kind="stable").astype(np.int64)


def first_bad_pivot(A):
    """1-based index of the first non-positive pivot met by an unpivoted
    Cholesky of A, or 0 if A is positive definite.  Plain column algorithm."""
    A = np.array(A, dtype=np.float64, copy=True)
    n = A.shape[0]
    for k in range(n):
        p = A[k, k]
        if not (p > 0.0):
            return k + 1
        r = np.sqrt(p)
        col = A[k + 1:, k] / r
        A[k + 1:, k + 1:] -= np.outer(col, col)
    return 0


def inverse_factor(Hd):
    """Upper-triangular U with positive diagonal and U^T U = Hd^-1.

    Steps: lower Cholesky L of Hd; Hd^-1 by two triangular solves against I;
    U = (lower Cholesky of Hd^-1)^T.  Returns (U, info); info = 0 on success,
    else the 1-based index of the first non-positive pivot (U is then None).
    """
    Hd = np.asarray(Hd, dtype=np.float64)
    n = Hd.shape[0]
    try:
        L = np.linalg.cholesky(Hd)
    except np.linalg.LinAlgError:
        return None, first_bad_pivot(Hd)
    Y = solve_triangular(L, np.eye(n), lower=True)          # L Y = I
    Hinv = solve_triangular(L.T, Y, lower=False)            # L^T Hinv = Y
    Hinv = 0.5 * (Hinv + Hinv.T)
    U = np.linalg.cholesky(Hinv).T
    return np.ascontiguousarray(U), 0


def hessian_factor(H, damp, act_order=False):
    """damp -> (optional) permute -> inverse factor.

    Returns dict(U, perm, info, Hd, lam); Hd is the damped matrix in ORIGINAL
    column order, U belongs to the permuted matrix Hd[perm][:, perm]."""
    Hd, lam = damp_hessian(H, damp)
    n = Hd.shape[0]
    perm = act_order_perm(H) if act_order else np.arange(n, dtype=np.int64)
    Hp = Hd[np.ix_(perm, perm)] if act_order else Hd
    U, info = inverse_factor(Hp)
    return {"U": U, "perm": perm, "info": info, "Hd": Hd, "lam": lam}


def direct_factor(Hd):
    """Upper-triangular R with positive diagonal and R R^T = Hd, so that R = U^-1 for the inverse factor U of
    Sec. 4.3.1 (U^T U = Hd^-1  <=>  Hd = U^-1 U^-T).  One Cholesky of the index-reversed matrix:
    J Hd J = L L^T  =>  Hd = (J L J)(J L J)^T  with J L J upper.  Returns (R, info) like inverse_factor."""
    Hd = np.asarray(Hd, dtype=np.float64)
    try:
        L = np.linalg.cholesky(Hd[::-1, ::-1])
    except np.linalg.LinAlgError:
        return None, first_bad_pivot(Hd[::-1, ::-1])
    return np.ascontiguousarray(L[::-1, ::-1]), 0


def block_feedback_factor(U, R, block):
    """The matrix F from which a blocked sweep can run without the off-diagonal part of U (quantize_layer_direct):
    F = U on the block x block diagonal blocks;  F_jk = -U_jj R_jk / R_kk  where j and k lie in different blocks
    (k > j);  0 below the diagonal.  Only the diagonal blocks of U enter, and those are the inverses of the
    diagonal blocks of R."""
    U = np.asarray(U, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    n = R.shape[0]
    d = np.diag(R)
    F = -np.triu(R, 1) / d[None, :] * np.diag(U)[:, None]
    for b0 in range(0, n, block):
        b1 = min(n, b0 + block)
        F[b0:b1, b0:b1] = np.triu(U[b0:b1, b0:b1])
    return np.triu(F)


# --------------------------------------------------------------------------
# Grid (Eq. 1, 2, 4)
# --------------------------------------------------------------------------
def minmax_params(wmin, wmax, bits):
    """Asymmetric min-max scale and zero-point of Eq. (2) for the unsigned
    range 0 .. 2^b - 1.  Rounding is half-to-even.  A degenerate group
    (wmax == wmin, on which the paper is silent) takes s = 1.
    Returns (s, z, tz) with tz = -wmin / s the value before rounding z."""
    qmax = float(2 ** bits - 1)
    wmin = np.asarray(wmin, dtype=np.float64)
    wmax = np.asarray(wmax, dtype=np.float64)
    s = (wmax - wmin) / qmax
    s = np.where(s == 0.0, 1.0, s)
    tz = -wmin / s
    z = np.clip(np.rint(tz), 0.0, qmax)
    return s, z, tz


def symmetric_params(wmin, wmax, bits):
    """Symmetric scale of Eq. (3): s = max(|wmin|, |wmax|) / (2^(b-1) - 1), zero-point fixed, signed codes
    q in {-(2^(b-1)-1), ..., 2^(b-1)-1}, w^ = s q.  Stored in the unsigned format of Eq. (4) as the code
    u = q + (2^(b-1) - 1) with the constant zero-point z = 2^(b-1) - 1, so that w^ = s (u - z) as for the
    asymmetric grid; the highest unsigned code 2^b - 1 is never used.  A degenerate group (all zeros, on which
    the paper is silent) takes s = 1.  Returns (s, z, tz) with tz = z (the zero-point is not rounded)."""
    qs = float(2 ** (bits - 1) - 1)
    m = np.maximum(np.abs(np.asarray(wmin, dtype=np.float64)), np.abs(np.asarray(wmax, dtype=np.float64)))
    s = m / qs
    s = np.where(s == 0.0, 1.0, s)
    z = np.full_like(s, qs)
    return s, z, z.copy()


def code_range_top(bits, grid):
    """Highest unsigned code of the grid: 2^b - 1 (asymmetric, Eq. (1)); 2 (2^(b-1) - 1) (symmetric, Eq. (3))."""
    if grid == "asym":
        return float(2 ** bits - 1)
    if grid == "sym":
        return float(2 * (2 ** (bits - 1) - 1))
    raise ValueError("grid must be 'asym' or 'sym'")


MSE_CANDIDATES = 80     # candidate ranges of the scale search: the min-max range shrunk by p_i = 1 - i / 100,
MSE_STEP = 0.01         # i = 0 .. 79 (down to 21 % of the range); the paper names the search but gives no set


def mse_search(vals, bits, grid="asym", n_cand=MSE_CANDIDATES, step=MSE_STEP):
    """Scale search per group [Sec. 4.3: "MSE-based grid tuning (mse), which searches over candidate scales to
    minimize the mean squared reconstruction error per-group"; the candidate set is this build's reading].

    vals: [rows, G] current values of one group per row.  Candidate i shrinks both ends of the observed range by
    p_i = 1 - i * step and takes (s, z) from it by the rule of the grid (Eq. (2), or Eq. (3) for "sym"); its error
    is sum_k (w_k - w^_k)^2 with w^ from Eq. (1) on that grid.  The smallest error wins, the lower index on a tie;
    candidate 0 is the plain min-max rule.  Returns dict(s, z, tz, cand [rows], err [rows, n_cand],
    s_all, z_all, tz_all [rows, n_cand]) and, for the analysis of ties only (no decision here uses them),
    z_alt [rows, n_cand] = the zero-point a candidate would get were its tz rounded the other way, with
    err_alt [rows, n_cand] the candidate's error on that grid."""
    vals = np.asarray(vals, dtype=np.float64)
    lo = vals.min(axis=1)
    hi = vals.max(axis=1)
    params = minmax_params if grid == "asym" else symmetric_params
    qtop = code_range_top(bits, grid)
    errs, ss, zs, tzs, zas, eas = [], [], [], [], [], []
    for i in range(n_cand):
        p = 1.0 - i * step
        s_i, z_i, tz_i = params(p * lo, p * hi, bits)
        q, wh, _ = quantize_scalar(vals, s_i[:, None], z_i[:, None], bits, qtop)
        errs.append(((vals - wh) ** 2).sum(axis=1))
        ss.append(s_i); zs.append(z_i); tzs.append(tz_i)
        za_i = np.clip(2.0 * np.floor(tz_i) + 1.0 - np.rint(tz_i), 0.0, qtop)   # the other neighbour of tz
        _, wha, _ = quantize_scalar(vals, s_i[:, None], za_i[:, None], bits, qtop)
        zas.append(za_i); eas.append(((vals - wha) ** 2).sum(axis=1))
    err = np.stack(errs, axis=1)
    cand = np.argmin(err, axis=1)          # first minimum
    r = np.arange(vals.shape[0])
    s_all = np.stack(ss, axis=1)
    return {"s": s_all[r, cand], "z": np.stack(zs, axis=1)[r, cand], "tz": np.stack(tzs, axis=1)[r, cand],
            "cand": cand, "err": err, "s_all": s_all, "z_all": np.stack(zs, axis=1), "tz_all": np.stack(tzs, axis=1),
            "z_alt": np.stack(zas, axis=1), "err_alt": np.stack(eas, axis=1)}


def quantize_scalar(w, s, z, bits, qtop=None):
    """Eq. (1): q = clamp(rne(w / s) + z, 0, qtop), w^ = s (q - z); qtop = 2^b - 1 unless given.
    Returns (q, w^, t) with t = w / s the value before rounding."""
    qmax = float(2 ** bits - 1) if qtop is None else float(qtop)
    t = np.asarray(w, dtype=np.float64) / s
    q = np.clip(np.rint(t) + z, 0.0, qmax)
    return q, s * (q - z), t


def rtn_quantize(W, bits, group_size, grid="asym", scale_search=None):
    """Round-to-nearest of W on the per-group min-max grid (Sec. 2.4, Eq.
    (direct weight quant) with the grid of Eq. (2), layout of Eq. (4)).
    Written independently of the sweep (whole-array, no column loop) so that it
    can pin the sweep's diagonal-H special case.  scale_search="mse": the grid of every group comes from
    mse_search instead of the plain range.  Returns (Q, scales, zeros, W^)."""
    W = np.asarray(W, dtype=np.float64)
    d_out, d_in = W.shape
    n_g = d_in // group_size
    Wg = W.reshape(d_out, n_g, group_size)
    lo = Wg.min(axis=2, keepdims=True)
    hi = Wg.max(axis=2, keepdims=True)
    s, z, _ = (minmax_params if grid == "asym" else symmetric_params)(lo, hi, bits)
    if scale_search == "mse":
        for g in range(n_g):
            m = mse_search(Wg[:, g, :], bits, grid)
            s[:, g, 0] = m["s"]
            z[:, g, 0] = m["z"]
    elif scale_search is not None:
        raise ValueError("scale_search must be None or 'mse'")
    qmax = code_range_top(bits, grid)
    Q = np.clip(np.rint(Wg / s) + z, 0.0, qmax)
    What = s * (Q - z)
    return (Q.reshape(d_out, d_in).astype(np.int64), s[:, :, 0], z[:, :, 0],
            What.reshape(d_out, d_in))


# --------------------------------------------------------------------------
# Column sweep (Sec. 4.3: one column at a time, residual propagated)
# --------------------------------------------------------------------------
def quantize_layer(W, U, bits, group_size, perm=None, rows=None,
                   forced_codes=None, forced_zeros=None, grid="asym", scale_search=None, forced_cand=None):
    """Greedy sequential quantization of every row of W with feedback through U.

    W: [d_out, d_in] original column order.  U: upper factor of the (permuted)
    damped inverse Hessian.  perm: column order (None = natural).  rows: optional
    subset of output rows (rows are independent given U).
    forced_codes: optional int array [rows, d_in] in PERMUTED column order,
      entries >= 0 override the rounded code at that step (replay of a tie).
    forced_zeros: optional int array [rows, n_groups], entries >= 0 override z.
    grid: "asym" = min-max grid of Eq. (2) (default), "sym" = symmetric grid of Eq. (3).
    scale_search: None = the grid of a group comes from the plain range of its current values; "mse" = from
      mse_search over those values.  forced_cand: optional int array [rows, n_groups], entries >= 0 override the
      candidate the search picks (replay of a near-tie between candidates).

    Per row, for j = 0 .. d_in-1 in permuted order:
      at a group start: (s, z) from min/max of the CURRENT values of the group
      q_j = clamp(rne(w_j / s) + z), w^_j = s (q_j - z)
      e_j = (w_j - w^_j) / U_jj ;  w_k -= e_j U_jk for k > j
    loss = sum e^2, which equals tr((W - W^) H_d (W - W^)^T) because
    U H_d U^T = I.

    Returns a dict.  Q and W_hat are in ORIGINAL column order; scales / zeros are
    indexed by group number in permuted order; E, T (w/s before rounding) and
    Tz (-wmin/s before rounding) are in permuted order.
    """
    W = np.asarray(W, dtype=np.float64)
    if rows is not None:
        W = W[np.asarray(rows)]
    U = np.asarray(U, dtype=np.float64)
    d_out, d_in = W.shape
    G = int(group_size)
    if d_in % G != 0:
        raise ValueError("d_in must be a multiple of group_size")
    n_g = d_in // G
    qtop = code_range_top(bits, grid)
    params = minmax_params if grid == "asym" else symmetric_params
    if perm is None:
        perm = np.arange(d_in, dtype=np.int64)
    perm = np.asarray(perm, dtype=np.int64)

    w = W[:, perm].copy()                       # working (compensated) values
    Q = np.zeros((d_out, d_in), dtype=np.int64)
    What = np.zeros((d_out, d_in))
    E = np.zeros((d_out, d_in))
    T = np.zeros((d_out, d_in))
    scales = np.zeros((d_out, n_g))
    zeros = np.zeros((d_out, n_g))
    Tz = np.zeros((d_out, n_g))
    n_c = MSE_CANDIDATES if scale_search == "mse" else 0
    Cand = np.zeros((d_out, n_g), dtype=np.int64)
    Ecand = np.zeros((d_out, n_g, n_c))
    Scand = np.zeros((d_out, n_g, n_c))
    Zcand = np.zeros((d_out, n_g, n_c))
    Tzcand = np.zeros((d_out, n_g, n_c))
    Zalt = np.zeros((d_out, n_g, n_c))
    Ealt = np.zeros((d_out, n_g, n_c))
    s = z = None
    for j in range(d_in):
        if j % G == 0:
            g = j // G
            blk = w[:, j:j + G]
            s, z, tz = params(blk.min(axis=1), blk.max(axis=1), bits)
            if scale_search == "mse":
                m = mse_search(blk, bits, grid)
                c = m["cand"]
                if forced_cand is not None:
                    fcd = np.asarray(forced_cand)[:, g]
                    c = np.where(fcd >= 0, fcd, c)
                rr = np.arange(d_out)
                s, z, tz = m["s_all"][rr, c], m["z_all"][rr, c], m["tz_all"][rr, c]
                Cand[:, g] = c
                Ecand[:, g, :] = m["err"]
                Scand[:, g, :] = m["s_all"]
                Zcand[:, g, :] = m["z_all"]
                Tzcand[:, g, :] = m["tz_all"]
                Zalt[:, g, :] = m["z_alt"]
                Ealt[:, g, :] = m["err_alt"]
            elif scale_search is not None:
                raise ValueError("scale_search must be None or 'mse'")
            if forced_zeros is not None:
                fz = np.asarray(forced_zeros)[:, g]
                z = np.where(fz >= 0, fz.astype(np.float64), z)
            scales[:, g] = s
            zeros[:, g] = z
            Tz[:, g] = tz
        wj = w[:, j].copy()
        q, wh, t = quantize_scalar(wj, s, z, bits, qtop)
        if forced_codes is not None:
            fc = np.asarray(forced_codes)[:, j]
            q = np.where(fc >= 0, fc.astype(np.float64), q)
            wh = s * (q - z)
        e = (wj - wh) / U[j, j]
        if j + 1 < d_in:
            w[:, j + 1:] -= e[:, None] * U[j, j + 1:][None, :]
        Q[:, j] = q.astype(np.int64)
        What[:, j] = wh
        E[:, j] = e
        T[:, j] = t
    out_Q = np.zeros_like(Q)
    out_What = np.zeros_like(What)
    out_Q[:, perm] = Q
    out_What[:, perm] = What
    return {
        "Q": out_Q, "W_hat": out_What, "scales": scales, "zeros": zeros,
        "loss": float((E * E).sum()), "loss_rows": (E * E).sum(axis=1),
        "E": E, "T": T, "Tz": Tz, "perm": perm, "cand": Cand, "Ecand": Ecand, "Scand": Scand,
        "Zcand": Zcand, "Tzcand": Tzcand, "Zalt": Zalt, "Ealt": Ealt,
    }


def layer_loss(W, W_hat, Hd):
    """tr((W - W^) Hd (W - W^)^T) evaluated directly (Eq. (layerwise) with the
    Gram matrix written out; all three arguments in the same column order)."""
    D = np.asarray(W, dtype=np.float64) - np.asarray(W_hat, dtype=np.float64)
    return float(((D @ np.asarray(Hd, dtype=np.float64)) * D).sum())


def quantize_layer_direct(W, R, bits, group_size, block, perm=None, grid="asym"):
    """The sweep of Sec. 4.3 arranged so that only ONE Cholesky factor of the damped matrix is needed.

    For one row let w be the original weights, w^ the quantized ones, e the propagated errors of
    quantize_layer and R = U^-1 (upper, R R^T = Hd, direct_factor).  Column j receives sum_{i<j} e_i U_ij and
    its own step removes e_j U_jj, hence  w - w^ = e U  and  e = (w - w^) R.
    Split the columns into those already finished (A) and the rest (B).  The inverse of a block-triangular
    matrix gives U_AB = -U_AA R_AB U_BB, so the compensated values of the unfinished columns are
        w_B - e_A U_AB = w_B + (w_A - w^_A) R_AA U_AA R_AB U_BB = w_B + (w_A - w^_A) R_AB U_BB ,
    and because U_BB is upper triangular its leading block x block part, the inverse of the diagonal block of R,
    is all that the next `block` columns need.  Per block of columns b:
        c    = sum over finished columns i of (w_i - w^_i) R_ib          (deviations from the ORIGINAL weights)
        w'_b = w_b + c (R_bb)^-1                                         (state the paper's sweep has on entering b)
        then the paper's steps inside the block with U_bb = (R_bb)^-1.
    Same greedy rule, same grid, same outputs as quantize_layer in exact arithmetic as long as no group
    straddles a block.  Returns dict(Q, W_hat, scales, zeros, loss), Q and W_hat in original column order.
    Pinned against quantize_layer in tests/test_oracle_direct.py."""
    W = np.asarray(W, dtype=np.float64)
    R = np.asarray(R, dtype=np.float64)
    d_out, d_in = W.shape
    G, B = int(group_size), int(block)
    if B % G != 0 or d_in % B != 0:
        raise ValueError("groups must not straddle blocks")
    n_g = d_in // G
    qtop = code_range_top(bits, grid)
    params = minmax_params if grid == "asym" else symmetric_params
    if perm is None:
        perm = np.arange(d_in, dtype=np.int64)
    perm = np.asarray(perm, dtype=np.int64)
    w0 = W[:, perm]
    dev = np.zeros((d_out, d_in))                # w - w^ of the finished columns
    Q = np.zeros((d_out, d_in), dtype=np.int64)
    What = np.zeros((d_out, d_in))
    scales = np.zeros((d_out, n_g))
    zeros = np.zeros((d_out, n_g))
    loss = 0.0
    for b0 in range(0, d_in, B):
        Ubb = solve_triangular(R[b0:b0 + B, b0:b0 + B], np.eye(B), lower=False)
        c = dev[:, :b0] @ R[:b0, b0:b0 + B]
        w = w0[:, b0:b0 + B] + c @ Ubb
        s = z = None
        for j in range(B):
            if j % G == 0:
                blk = w[:, j:j + G]
                s, z, _ = params(blk.min(axis=1), blk.max(axis=1), bits)
                scales[:, (b0 + j) // G] = s
                zeros[:, (b0 + j) // G] = z
            q, wh, _ = quantize_scalar(w[:, j], s, z, bits, qtop)
            e = (w[:, j] - wh) / Ubb[j, j]
            if j + 1 < B:
                w[:, j + 1:] -= e[:, None] * Ubb[j, j + 1:][None, :]
            loss += float((e * e).sum())
            Q[:, b0 + j] = q.astype(np.int64)
            What[:, b0 + j] = wh
        dev[:, b0:b0 + B] = w0[:, b0:b0 + B] - What[:, b0:b0 + B]
    out_Q = np.zeros_like(Q)
    out_What = np.zeros_like(What)
    out_Q[:, perm] = Q
    out_What[:, perm] = What
    return {"Q": out_Q, "W_hat": out_What, "scales": scales, "zeros": zeros, "loss": loss}


def dequantize(Q, scales, zeros, group_size, perm=None):
    """W^_ij = s_g (q_ij - z_g)  (Eq. (4)); Q in original column order, the
    group of original column c is position_of(c) // G in the sweep order."""
    Q = np.asarray(Q, dtype=np.float64)
    d_out, d_in = Q.shape
    if perm is None:
        perm = np.arange(d_in)
    inv = np.empty(d_in, dtype=np.int64)
    inv[np.asarray(perm)] = np.arange(d_in)
    g = inv // int(group_size)
    return np.asarray(scales, dtype=np.float64)[:, g] * (Q - np.asarray(zeros, dtype=np.float64)[:, g])


# --------------------------------------------------------------------------
# Error propagation (QEP): corrected quantization target  [Sec. 4.3.1, Eq. (qep_obj), Eq. (qep)]
# --------------------------------------------------------------------------
def crossgram_accumulate(X_hat, X, G=None):
    """G + 2 * X_hat^T X in float64.

    X_hat: activations seen by the partly quantized model, X: full-precision activations, both
    [n_tokens, d_in].  With H = 2 X_hat^T X_hat the error-propagation matrix of Sec. 4.3.1 is
    C = X_hat^T (X - X_hat) = (G - H) / 2; the factor 2 is the one of hessian_accumulate.
    """
    X_hat = np.asarray(X_hat, dtype=np.float64)
    X = np.asarray(X, dtype=np.float64)
    P = 2.0 * (X_hat.T @ X)
    return P if G is None else np.asarray(G, dtype=np.float64) + P


def qep_target(W, G, H, damp, alpha):
    """Corrected target of Eq. (qep) in the d_out x d_in storage convention.

    Paper (W_p = W^T is d_in x d_out):  W_p* = (I + alpha (H^_p + lambda_p I)^-1 C) W_p  with
    H^_p = X_hat^T X_hat, C = X_hat^T (X - X_hat), lambda_p = damp * mean(diag H^_p).
    Here H = 2 H^_p and G = 2 X_hat^T X, so 2 C = G - H, lambda = damp * mean(diag H) = 2 lambda_p and
    (H^_p + lambda_p I)^-1 C = (H + lambda I)^-1 (G - H).  Transposed:
        W* = W + alpha * W (G - H)^T (H + lambda I)^-1.
    The damped matrix is the one damp_hessian builds (a dead channel's diagonal entry becomes 1 first).
    The inverse is applied with a symmetric positive definite solve (Cholesky based, as Sec. 4.3.1 says).
    """
    from scipy.linalg import cho_factor, cho_solve
    W = np.asarray(W, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    H = np.asarray(H, dtype=np.float64)
    Hd, _ = damp_hessian(H, damp)
    C2 = G - H                                   # = 2 C
    R = W @ C2.T                                 # d_out x d_in
    cf = cho_factor(Hd, lower=True)
    corr = cho_solve(cf, R.T).T                  # R Hd^-1 (Hd symmetric)
    return W + float(alpha) * corr


# --------------------------------------------------------------------------
# JointQ: local search over integer codes with the group scale refit in the same move  [Sec. 4.3.2, Eq. (jointq)]
# --------------------------------------------------------------------------
def row_objective(W, W_hat, A):
    """Per row (w - w^) A (w - w^)^T: the objective of Eq. (jointq) for one output row when A = X^T X up to the
    constant factor this build carries in H (Eq. (jointq_reg): A = H + lam I, the augmented input matrix)."""
    D = np.asarray(W, dtype=np.float64) - np.asarray(W_hat, dtype=np.float64)
    return ((D @ np.asarray(A, dtype=np.float64)) * D).sum(axis=1)


def jointq_refine(W, A, Q, scales, zeros, bits, group_size, grid="asym", n_pass=1, max_scans=4, rows=None,
                  forced=None, tie_tol=0.0, g_tol=0.0, a_tol=0.0, perm=None):
    """Local search of Sec. 4.3.2 on a solution in the per-group format of Eq. (4), rows independent.

    What the paper fixes: one move changes one integer code by a small amount inside the codebook, the scale of
    that code's group is refit in the same step to the codes, a move is kept iff the objective of Eq. (jointq)
    falls, and the search stops when no move improves; a GPTQ result may serve as the start.  What it leaves open
    and this build reads as follows: the change is +-1; zero-points stay as given; the groups of a row are visited
    in order, n_pass times; inside a visit the columns of the group are scanned in order, for each column +1 is
    tried before -1 and the first improving one is taken at once (at most one per column and scan); the visit ends
    with the first scan that takes no move, or after max_scans scans; on entering a visit the group's scale is
    first refit to its current codes; a group whose codes all equal its zero-point is left alone, and no move may
    bring a group there (the refit scale b / c is undefined at u = 0: c' = 0 and N = -c' b^2 / c reaches 0 from
    below, so by "N > 0 and c' > 0" the move is never taken; deciding it on the integer codes keeps rounding noise
    in a carried c from deciding it).

    One visit, one row, group t with codes q, u = q - z, residual r = w - w^ over the whole row:
        p = (A r)_t + s_old A_tt u     (= (A r0)_t with r0 the residual with group t taken out; fixed in the visit)
        b = u.p,  c = u.A_tt u,        best scale s* = b / c,  objective = r0 A r0^T - b^2 / c .
    Move u' = u + d e_j:  b' = b + d p_j,  c' = c + 2 d a_j + A_jj  with a = A_tt u.  With g = p_j - s* a_j (the
    gradient at the refit scale) and D = c A_jj - a_j^2:
        N = c' (b'^2 / c' - b^2 / c) = 2 d b g + g^2 + 2 s* g a_j - s*^2 D ,
    and the move is taken iff N > 0 and c' > 0 (the objective then falls by N / c').

    W [d_out, d_in]; A symmetric [d_in, d_in]; Q codes, scales / zeros [d_out, n_g] as the sweep returns them.
    perm: the column order of the sweep that produced the start (None = natural): groups, "in order" and the
    column index j of a decision refer to that order, W, A, Q and W_hat are given and returned in the original one.  forced: {(row, pass, t, scan, j, d): bool} overrides single decisions (rows numbered
    within the subset); with tie_tol > 0 every decision with
    |N| <= tie_tol * M + 2 |b| (g_tol (|r| |A|)_j + a_tol |s*| (|u| |A_tt|)_j), M the sum of the absolute values of
    the terms N is built from, is listed in "ties" as (pass, t, scan, j, d, taken) (g_tol, a_tol: the rounding of a
    gradient and of a = A_tt u that are carried along rather than recomputed).
    Returns dict(Q, scales, W_hat, f0, f1 (row objective before / after), moves [rows], ties [list per row])."""
    W = np.asarray(W, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    sel = np.arange(W.shape[0]) if rows is None else np.asarray(rows)
    W = W[sel]
    Q = np.array(np.asarray(Q)[sel], dtype=np.float64, copy=True)
    if perm is not None:
        perm = np.asarray(perm, dtype=np.int64)
        W, Q, A = W[:, perm], Q[:, perm], A[np.ix_(perm, perm)]
    S = np.array(np.asarray(scales)[sel], dtype=np.float64, copy=True)
    Z = np.asarray(zeros, dtype=np.float64)[sel]
    n, d_in = W.shape
    G = int(group_size)
    n_g = d_in // G
    qtop = code_range_top(bits, grid)
    forced = forced or {}
    ties = [[] for _ in range(n)]
    moves = np.zeros(n, dtype=np.int64)

    def dequant():
        return np.repeat(S, G, axis=1) * (Q - np.repeat(Z, G, axis=1))

    f0 = row_objective(W, dequant(), A)
    absA = np.abs(A) if g_tol > 0.0 else None
    for ps in range(int(n_pass)):
        for t in range(n_g):
            cs = slice(t * G, (t + 1) * G)
            r = W - dequant()
            g = r @ A[:, cs]
            gabs = np.abs(r) @ absA[:, cs] if g_tol > 0.0 else np.zeros_like(g)
            Att = A[cs, cs]
            u = Q[:, cs] - Z[:, t][:, None]
            a = u @ Att
            s_old = S[:, t].copy()
            p = g + s_old[:, None] * a
            b = (u * p).sum(axis=1)
            c = (u * a).sum(axis=1)
            live = c > 0.0
            active = live.copy()
            nz = (u != 0.0).sum(axis=1)          # codes of the group away from its zero-point
            for scan in range(int(max_scans)):
                took = np.zeros(n, dtype=bool)
                aabs = np.abs(u) @ np.abs(Att) if a_tol > 0.0 else None
                for j in range(G):
                    done = np.zeros(n, dtype=bool)
                    for d in (1.0, -1.0):
                        qn = Q[:, t * G + j] + d
                        ok = active & ~done & (qn >= 0.0) & (qn <= qtop) & ~((nz == 1) & (u[:, j] == -d))
                        if not ok.any():
                            continue
                        aj, pj, Ajj = a[:, j], p[:, j], Att[j, j]
                        cc = np.where(live, c, 1.0)
                        ss = b / cc
                        gs = pj - ss * aj
                        N = 2.0 * d * b * gs + gs * gs + 2.0 * ss * gs * aj - ss * ss * (cc * Ajj - aj * aj)
                        cn = c + 2.0 * d * aj + Ajj
                        acc = ok & (N > 0.0) & (cn > 0.0)
                        if tie_tol > 0.0 or g_tol > 0.0 or a_tol > 0.0:
                            M = (2.0 * np.abs(b) * (np.abs(pj) + np.abs(ss * aj)) + gs * gs + 2.0 * np.abs(ss * gs * aj)
                                 + ss * ss * (cc * Ajj + aj * aj))
                            slack = g_tol * gabs[:, j]
                            if a_tol > 0.0:
                                slack = slack + a_tol * np.abs(ss) * aabs[:, j]
                            near = ok & (np.abs(N) <= tie_tol * M + 2.0 * np.abs(b) * slack)
                            for i in np.nonzero(near)[0]:
                                ties[i].append((ps, t, scan, j, int(d), bool(acc[i])))
                        for i in np.nonzero(ok)[0] if forced else ():
                            key = (int(i), ps, t, scan, j, int(d))
                            if key in forced:
                                acc[i] = bool(forced[key]) and cn[i] > 0.0
                        if acc.any():
                            nz = nz + np.where(acc, (u[:, j] == 0.0).astype(np.int64) - (u[:, j] + d == 0.0), 0)
                            Q[acc, t * G + j] += d
                            u[acc, j] += d
                            b = np.where(acc, b + d * pj, b)
                            c = np.where(acc, cn, c)
                            a[acc] += d * Att[j][None, :]
                            done |= acc
                            took |= acc
                            moves += acc
                active &= took
                if not active.any():
                    break
            S[:, t] = np.where(live, b / np.where(live, c, 1.0), s_old)
    What = dequant()
    f1 = row_objective(W, What, A)
    if perm is not None:
        Qo, Wo = np.empty_like(Q), np.empty_like(What)
        Qo[:, perm], Wo[:, perm] = Q, What
        Q, What = Qo, Wo
    return {"Q": Q.astype(np.int64), "scales": S, "W_hat": What, "f0": f0, "f1": f1, "moves": moves, "ties": ties}


# --------------------------------------------------------------------------
# Sensitivity proxy for bit-width allocation  [Sec. 4.1, "AutoBit"]
# --------------------------------------------------------------------------
def rtn_sensitivity(W, a_diag, b_diag, bits, group_size, grid="asym"):
    """err = 1/2 tr(B dW A dW^T) with diagonal A (input channels) and B (output rows) and dW = W^ - W from the
    round-to-nearest proxy (rtn_quantize), written for the d_out x d_in storage:
    1/2 sum_r sum_c b_r a_c dW_rc^2.  b_diag None = ones."""
    W = np.asarray(W, dtype=np.float64)
    _, _, _, What = rtn_quantize(W, bits, group_size, grid=grid)
    D = What - W
    a = np.asarray(a_diag, dtype=np.float64)
    b = np.ones(W.shape[0]) if b_diag is None else np.asarray(b_diag, dtype=np.float64)
    return 0.5 * float((b[:, None] * D * D * a[None, :]).sum())
