"""Helpers shared by the GPU parity tests: oracle calls, tie classification and replay."""
import numpy as np
import torch

from oracle import onecomp_oracle as oc

TIE_TOL = 1e-4   # a first mismatch is a legitimate tie flip iff the oracle's pre-rounding value is this close to x.5
CAND_TOL = 1e-4  # scale search: another candidate is a legitimate choice iff its squared error (the oracle's) is within
                 # this relative distance of the smallest one


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def _near_tie(t: np.ndarray) -> np.ndarray:
    return np.abs((t - np.floor(t)) - 0.5) < TIE_TOL


def compare_codes(gpu_Q, gpu_zeros, W, U, bits, G, perm=None, rows=None, max_rounds=64, grid="asym",
                  scale_search=None, gpu_scales=None):
    """GPU codes / zero-points against the oracle with tie replay.

    gpu_Q: [n_rows, d_in] codes in ORIGINAL column order, gpu_zeros: [n_rows, n_g].
    W (full layer, original order) and U are the oracle's inputs; rows selects the compared rows.
    Per row the first disagreement (in sweep order; a group's zero-point comes before its codes)
    must sit at a rounding tie of the oracle (|frac - 0.5| < TIE_TOL, values differ by one);
    the oracle row is then replayed with that decision forced to the GPU's and the comparison
    continues.  With scale_search = "mse" a group's first decision is the candidate of the search: the GPU's
    is read off its scale (gpu_scales, matched against the oracle's candidate scales); a different candidate is
    accepted iff the oracle's own error sums of the two agree to CAND_TOL, and is then forced in the replay.
    Returns stats incl. the final oracle output (after replay)."""
    W = np.asarray(W, dtype=np.float64)
    d_in = W.shape[1]
    if perm is None:
        perm = np.arange(d_in)
    perm = np.asarray(perm, dtype=np.int64)
    rows = np.arange(W.shape[0]) if rows is None else np.asarray(rows)
    gq = np.asarray(gpu_Q, dtype=np.int64)[:, perm]          # sweep order
    gz = np.asarray(gpu_zeros, dtype=np.int64)
    n_rows, n_g = gz.shape
    fc = -np.ones((n_rows, d_in), dtype=np.int64)
    fz = -np.ones((n_rows, n_g), dtype=np.int64)
    fcand = -np.ones((n_rows, n_g), dtype=np.int64)
    mse = scale_search == "mse"
    gs = np.asarray(gpu_scales, dtype=np.float64) if mse else None
    out = oc.quantize_layer(W, U, bits, G, perm=perm, rows=rows, grid=grid, scale_search=scale_search)
    oq = out["Q"][:, perm].copy()
    raw_agree = float((oq == gq).mean())
    res = {k: np.array(v, copy=True) if isinstance(v, np.ndarray) else v for k, v in out.items()}
    tie_flips, cand_flips, real = 0, 0, []
    active = np.arange(n_rows)
    for _ in range(max_rounds):
        redo = []
        for i in active:
            oqi = res["Q"][i][perm]
            ozi = res["zeros"][i].astype(np.int64)
            bad_q = np.nonzero(oqi != gq[i])[0]
            bad_z = np.nonzero(ozi != gz[i])[0]
            jq = bad_q[0] if len(bad_q) else d_in
            jz = bad_z[0] * G if len(bad_z) else d_in
            jc = d_in
            if mse:
                bad_s = np.nonzero(np.abs(gs[i] - res["scales"][i]) > 1e-5 * np.abs(res["scales"][i]))[0]
                jc = bad_s[0] * G if len(bad_s) else d_in
            if jq == d_in and jz == d_in and jc == d_in:
                continue
            if jc <= jz and jc <= jq:
                g = jc // G
                sc, ec = res["Scand"][i, g], res["Ecand"][i, g]
                # a candidate whose zero-point sits at a rounding tie may be charged with either neighbour
                tied = _near_tie(res["Tzcand"][i, g])
                e_hi = np.where(tied, np.maximum(ec, res["Ealt"][i, g]), ec)
                k = int(np.argmin(np.abs(sc - gs[i, g])))
                if gz[i, g] == res["Zcand"][i, g, k]:
                    ek = ec[k]
                elif tied[k] and gz[i, g] == res["Zalt"][i, g, k]:
                    ek = res["Ealt"][i, g, k]
                else:
                    ek = np.inf
                ok = (abs(sc[k] - gs[i, g]) <= 1e-5 * abs(sc[k]) and k != res["cand"][i, g]
                      and ek <= e_hi.min() * (1.0 + CAND_TOL))
                if ok:
                    fcand[i, g] = k
                    if gz[i, g] != res["Zcand"][i, g, k]:
                        fz[i, g] = gz[i, g]
                    cand_flips += 1
                    tie_flips -= 1   # counted separately
            elif jz <= jq:
                g = jz // G
                ok = _near_tie(res["Tz"][i, g]) and abs(int(ozi[g]) - int(gz[i, g])) == 1
                if ok:
                    fz[i, g] = gz[i, g]
            else:
                ok = _near_tie(res["T"][i, jq]) and abs(int(oqi[jq]) - int(gq[i, jq])) == 1
                if ok:
                    fc[i, jq] = gq[i, jq]
            if ok:
                tie_flips += 1
                redo.append(i)
            else:
                real.append((int(rows[i]), int(min(jq, jz, jc))))
        if not redo:
            break
        redo = np.array(redo)
        sub = oc.quantize_layer(W, U, bits, G, perm=perm, rows=rows[redo],
                                forced_codes=fc[redo], forced_zeros=fz[redo], grid=grid, scale_search=scale_search,
                                forced_cand=fcand[redo] if mse else None)
        for k in ("Q", "W_hat", "scales", "zeros", "E", "T", "Tz", "loss_rows", "cand", "Ecand", "Scand", "Zcand", "Tzcand", "Zalt",
                  "Ealt"):
            res[k][redo] = sub[k]
        active = redo
    res["loss"] = float(res["loss_rows"].sum())
    final_agree = float((res["Q"][:, perm] == gq).mean())
    return {"raw_agree": raw_agree, "final_agree": final_agree, "tie_flips": tie_flips, "cand_flips": cand_flips,
            "real_mismatches": real, "oracle": res}


JQ_TIE_TOL = 1e-4   # JointQ: a decision is a legitimate toss-up iff |N| is within this fraction of the terms it sums
JQ_G_TOL = 2e-6     # ... plus this fraction of sum |r_k| |A_kj|, the rounding of the fp32 gradient kept on the GPU
JQ_A_TOL = 2e-6     # ... and, for groups wider than a block, of s* sum |u_k| |A_kj|: there a = A_gg u is carried along too


def _jq_prefix(o, i, gq, gs, G, n_g, pv=None):
    """Number of leading groups (visit order of one pass) in which oracle row i equals the GPU row; pv maps sweep
    positions to columns."""
    oq = o["Q"][i] if pv is None else o["Q"][i][pv]
    gq = gq if pv is None else gq[pv]
    for t in range(n_g):
        same = (np.array_equal(oq[t * G:(t + 1) * G], gq[t * G:(t + 1) * G])
                and abs(o["scales"][i, t] - gs[t]) <= 1e-4 * abs(o["scales"][i, t]))
        if not same:
            return t
    return n_g


def _jq_first_column(o, i, gq, pv):
    """First sweep position at which the codes differ, or -1."""
    bad = np.nonzero(o["Q"][i][pv] != gq[pv])[0]
    return int(bad[0]) if len(bad) else -1


def compare_jointq(gpu_Q, gpu_S, W, A, Q0, S0, Z, bits, G, grid="asym", n_pass=1, max_scans=4, rows=None,
                   max_flips=6, max_tries=24, wide=False, perm=None):
    """GPU result of onecomp_jointq_refine against the oracle's local search from the same start.

    A row must equal the oracle's exactly in its codes (scales to 1e-4), or become equal once decisions the oracle
    itself lists as toss-ups (JQ_TIE_TOL, JQ_G_TOL, JQ_A_TOL) are forced the other way.
    One pass of one scan: every column is decided once, so the GPU's decisions can be read off its codes; the
    first column that differs names the decision, which must be a listed toss-up and is then forced to the GPU's
    (the replay of the sweep's protocol).  Otherwise the decisions are not observable: the oracle is rerun with one
    listed toss-up flipped at a time, and a flip is kept when the rows then agree over more leading groups or, with
    that unchanged, in more codes; up to max_flips flips.  Where no single flip helps, a depth-first search over the
    listed toss-ups of the first differing group follows (a flipped toss-up tends to return as a toss-up of the same
    column in the next scan, so the right replay can be a chain of flips none of which helps alone).
    Returns dict(clean_rows, flipped_rows, flips, real_mismatches, oracle)."""
    W = np.asarray(W, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    rows = np.arange(W.shape[0]) if rows is None else np.asarray(rows)
    gq = np.asarray(gpu_Q, dtype=np.int64)
    gs = np.asarray(gpu_S, dtype=np.float64)
    Q0 = np.asarray(Q0)
    n_g = W.shape[1] // G
    kw = dict(bits=bits, group_size=G, grid=grid, n_pass=n_pass, max_scans=max_scans, tie_tol=JQ_TIE_TOL,
              g_tol=JQ_G_TOL, a_tol=JQ_A_TOL if wide else 0.0, perm=perm)
    pv = np.arange(W.shape[1]) if perm is None else np.asarray(perm, dtype=np.int64)   # sweep position -> column
    o = oc.jointq_refine(W, A, Q0, S0, Z, rows=rows, **kw)
    res = {k: (np.array(v, copy=True) if isinstance(v, np.ndarray) else v) for k, v in o.items()}
    clean, flipped, flips, real = 0, 0, 0, []
    single = n_pass == 1 and max_scans == 1

    def run1(i, forced):
        return oc.jointq_refine(W, A, Q0, S0, Z, rows=rows[i:i + 1], forced=forced, **kw)

    for i in range(len(rows)):
        if _jq_prefix(o, i, gq[i], gs[i], G, n_g, pv) == n_g:
            clean += 1
            continue
        forced, ok = {}, False
        cur = run1(i, forced)
        for _ in range(max_flips if not single else 4 * max_flips):
            pre = _jq_prefix(cur, 0, gq[i], gs[i], G, n_g, pv)
            if pre == n_g:
                ok = True
                break
            listed = {k[:5]: k[5] for k in cur["ties"][0]}
            if single:
                j = _jq_first_column(cur, 0, gq[i], pv)
                if j < 0:
                    break                        # codes equal, a scale differs: not a toss-up
                t, jl = j // G, j % G
                want = int(gq[i, pv[j]] - Q0[rows[i], pv[j]])   # the GPU's decision at this sweep position
                f2 = dict(forced)
                for d in (1, -1):
                    key = (0, t, 0, jl, d)
                    if key in listed and listed[key] != (want == d):
                        f2[(0,) + key] = (want == d)
                if f2 == forced:
                    break                        # the differing decision is not a listed toss-up
                forced, cur = f2, run1(i, f2)
                flips += 1
                continue
            # greedy: one listed toss-up flipped at a time, kept when the rows then agree over more leading groups
            # or, with that unchanged, in more codes
            ham = int((cur["Q"][0] != gq[i]).sum())
            best = None
            for k in [k for k in listed if (0,) + k not in forced and (n_pass > 1 or k[1] == pre)][:max_tries]:
                f2 = dict(forced)
                f2[(0,) + k] = not listed[k]
                trial = run1(i, f2)
                score = (_jq_prefix(trial, 0, gq[i], gs[i], G, n_g, pv), -int((trial["Q"][0] != gq[i]).sum()))
                if score > (pre, -ham) and (best is None or score > best[0]):
                    best = (score, f2, trial)
            if best is not None:
                _, forced, cur = best
                flips += 1
                continue
            # No single flip helps.  A toss-up flipped in one scan usually comes back as a new toss-up of the same
            # column in the next scan, so the right replay can be a chain of flips none of which helps alone:
            # depth-first over the listed toss-ups of the first differing group (of any pass), a branch followed
            # while that group does not move backwards, up to max_flips flips deep and 4 max_tries oracle runs.
            budget = [max_tries * 4]

            def dfs(f, c, depth):
                pre_c = _jq_prefix(c, 0, gq[i], gs[i], G, n_g, pv)
                if pre_c == n_g:
                    return f, c, depth
                if depth >= max_flips:
                    return None
                now = {t[:5]: t[5] for t in c["ties"][0]}
                for k in [k for k in now if k[1] == pre_c and (0,) + k not in f]:
                    if budget[0] <= 0:
                        return None
                    budget[0] -= 1
                    f2 = dict(f)
                    f2[(0,) + k] = not now[k]
                    trial = run1(i, f2)
                    if _jq_prefix(trial, 0, gq[i], gs[i], G, n_g, pv) < pre_c:
                        continue
                    got = dfs(f2, trial, depth + 1)
                    if got is not None:
                        return got
                return None

            got = dfs(forced, cur, 0)
            if got is not None:
                forced, cur, n = got
                flips += n
            break
        ok = ok or _jq_prefix(cur, 0, gq[i], gs[i], G, n_g, pv) == n_g
        if ok:
            flipped += 1
            for k in ("Q", "scales", "W_hat", "f0", "f1", "moves"):
                res[k][i] = cur[k][0]
        else:
            real.append(int(rows[i]))
    return {"clean_rows": clean, "flipped_rows": flipped, "flips": flips, "real_mismatches": real, "oracle": res}


def compare_jointq_by_scan(gpu_Q_by_scan, gpu_S, W, A, Q0, S0, Z, bits, G, grid="asym", rows=None, perm=None):
    """One group per row, one pass, several scans: exact replay of onecomp_jointq_refine against the oracle.

    gpu_Q_by_scan[k - 1]: the GPU's codes after a call with max_scans = k (k = 1 .. S), all from the same start; the
    visit of a row's single group after k scans is the first k scans of the visit with more, so the GPU's decision at
    column j in scan k is the difference of the codes after k and after k - 1 scans.  Scan by scan, the oracle (run
    with max_scans = k and the decisions forced so far) must reproduce the GPU's codes; where it first differs, the
    decision at that column must be one the oracle itself lists as a toss-up (JQ_TIE_TOL, JQ_G_TOL, JQ_A_TOL), which
    is then forced to the GPU's, and the scan is compared again.  gpu_S: the GPU's scales after the last call.
    Returns dict(clean_rows, flipped_rows, flips, real_mismatches [(row, scan, column)], oracle)."""
    W = np.asarray(W, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    rows = np.arange(W.shape[0]) if rows is None else np.asarray(rows)
    d_in = W.shape[1]
    assert G == d_in, "one group per row"
    S = len(gpu_Q_by_scan)
    gq = [np.asarray(q, dtype=np.int64) for q in gpu_Q_by_scan]
    Q0 = np.asarray(Q0)
    pv = np.arange(d_in) if perm is None else np.asarray(perm, dtype=np.int64)
    kw = dict(bits=bits, group_size=G, grid=grid, n_pass=1, tie_tol=JQ_TIE_TOL, g_tol=JQ_G_TOL, a_tol=JQ_A_TOL, perm=perm)
    clean, flipped, flips, real = 0, 0, 0, []
    final = []
    for i in range(len(rows)):
        forced, bad = {}, None
        for k in range(1, S + 1):
            prev = Q0[rows[i]].astype(np.int64) if k == 1 else gq[k - 2][i]
            for _ in range(64):
                cur = oc.jointq_refine(W, A, Q0, S0, Z, rows=rows[i:i + 1], forced=forced, max_scans=k, **kw)
                j = _jq_first_column(cur, 0, gq[k - 1][i], pv)
                if j < 0:
                    break
                want = int(gq[k - 1][i][pv[j]] - prev[pv[j]])          # the GPU's decision at this position in scan k
                listed = {t[:5]: t[5] for t in cur["ties"][0]}
                f2 = dict(forced)
                for d in (1, -1):
                    key = (0, 0, k - 1, j, d)
                    if key in listed and listed[key] != (want == d):
                        f2[(0,) + key] = (want == d)
                if f2 == forced:
                    bad = (int(rows[i]), k - 1, int(j))                  # not a listed toss-up
                    break
                forced = f2
                flips += 1
            else:
                bad = (int(rows[i]), k - 1, -1)
            if bad is not None:
                break
        if bad is not None:
            real.append(bad)
        elif forced:
            flipped += 1
        else:
            clean += 1
        final.append(cur)
    res = {"Q": np.concatenate([c["Q"] for c in final]), "scales": np.concatenate([c["scales"] for c in final])}
    return {"clean_rows": clean, "flipped_rows": flipped, "flips": flips, "real_mismatches": real, "oracle": res}
