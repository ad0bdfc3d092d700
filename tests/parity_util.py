"""Helpers shared by the GPU parity tests: oracle calls, tie classification and replay."""
import numpy as np
import torch

from oracle import onecomp_oracle as oc

TIE_TOL = 1e-4   # a first mismatch is a legitimate tie flip iff the oracle's pre-rounding value is this close to x.5


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def rel_fro(a: np.ndarray, b: np.ndarray) -> float:
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def _near_tie(t: np.ndarray) -> np.ndarray:
    return np.abs((t - np.floor(t)) - 0.5) < TIE_TOL


def compare_codes(gpu_Q, gpu_zeros, W, U, bits, G, perm=None, rows=None, max_rounds=64, grid="asym"):
    """GPU codes / zero-points against the oracle with tie replay.

    gpu_Q: [n_rows, d_in] codes in ORIGINAL column order, gpu_zeros: [n_rows, n_g].
    W (full layer, original order) and U are the oracle's inputs; rows selects the compared rows.
    Per row the first disagreement (in sweep order; a group's zero-point comes before its codes)
    must sit at a rounding tie of the oracle (|frac - 0.5| < TIE_TOL, values differ by one);
    the oracle row is then replayed with that decision forced to the GPU's and the comparison
    continues.  Returns stats incl. the final oracle output (after replay)."""
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
    out = oc.quantize_layer(W, U, bits, G, perm=perm, rows=rows, grid=grid)
    oq = out["Q"][:, perm].copy()
    raw_agree = float((oq == gq).mean())
    res = {k: np.array(v, copy=True) if isinstance(v, np.ndarray) else v for k, v in out.items()}
    tie_flips, real = 0, []
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
            if jq == d_in and jz == d_in:
                continue
            if jz <= jq:
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
                real.append((int(rows[i]), int(min(jq, jz))))
        if not redo:
            break
        redo = np.array(redo)
        sub = oc.quantize_layer(W, U, bits, G, perm=perm, rows=rows[redo],
                                forced_codes=fc[redo], forced_zeros=fz[redo], grid=grid)
        for k in ("Q", "W_hat", "scales", "zeros", "E", "T", "Tz", "loss_rows"):
            res[k][redo] = sub[k]
        active = redo
    res["loss"] = float(res["loss_rows"].sum())
    final_agree = float((res["Q"][:, perm] == gq).mean())
    return {"raw_agree": raw_agree, "final_agree": final_agree, "tie_flips": tie_flips,
            "real_mismatches": real, "oracle": res}
