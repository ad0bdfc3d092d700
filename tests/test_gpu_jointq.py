"""GPU parity of onecomp_jointq_refine (Sec. 4.3.2) against the oracle's local search from the same start."""
import numpy as np
import pytest
import torch

import paper_2603_28845_amd as og
from paper_2603_28845_amd import synth
from oracle import onecomp_oracle as oc
from parity_util import compare_jointq, compare_jointq_by_scan, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _announce(msg):
    print(f"[case] {msg}", flush=True)


def _start(d_out, d_in, bits, G, seed, dtype=torch.float32, grid="asym", start="rtn", act=False):
    """Synthetic layer, its Gram matrix (fp32 values, shared by both sides) and a start from the oracle (act: the
    sweep with activation ordering; the column order is returned as the last element)."""
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=2 * d_in + 13, seed=seed, dtype=dtype,
                       n_outlier=max(1, d_in // 100))
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, "cpu")
    H32 = oc.hessian_accumulate(to_f64(X)).astype(np.float32)
    Wd = to_f64(W)
    if start == "rtn":
        Q0, S0, Z0, _ = oc.rtn_quantize(Wd, bits, G, grid)
    else:
        f = oc.hessian_factor(H32.astype(np.float64), 0.01, act_order=act)
        out = oc.quantize_layer(Wd, f["U"], bits, G, grid=grid, perm=f["perm"] if act else None)
        Q0, S0, Z0 = out["Q"], out["scales"], out["zeros"]
        if act:
            return W, Wd, H32, Q0, S0, Z0, f["perm"]
    return W, Wd, H32, Q0, S0, Z0


def _run(W, Wd, H32, Q0, S0, Z0, bits, G, grid="asym", lam=0.0, n_pass=1, max_scans=4, max_bad_rows=None, perm=None):
    Q = torch.from_numpy(Q0.astype(np.uint8)).to(DEV)
    S = torch.from_numpy(S0.astype(np.float32)).to(DEV)
    Z = torch.from_numpy(Z0.astype(np.float32)).to(DEV)
    H = torch.from_numpy(H32).to(DEV)
    pt = None if perm is None else torch.from_numpy(perm.astype(np.int32)).to(DEV)
    out = og.onecomp_jointq_refine(W, H, Q, S, Z, bits, G, grid="symmetric" if grid == "sym" else "minmax", lam=lam,
                                   n_pass=n_pass, max_scans=max_scans, perm=pt)
    torch.cuda.synchronize()
    gq = out["Q_codes"].cpu().numpy()
    gs = out["scales"].cpu().numpy()
    wh = out["W_hat"].cpu().numpy()
    obj = out["objective"].cpu().numpy().astype(np.float64)
    d_out, d_in = Wd.shape
    A = H32.astype(np.float64) + lam * np.eye(d_in)
    S0f = S0.astype(np.float32).astype(np.float64)      # the start as the GPU received it
    qtop = oc.code_range_top(bits, grid)
    assert gq.max() <= qtop
    grp = (np.arange(d_in) if perm is None else np.argsort(perm)) // G       # group of every original column
    deq = gs[:, grp] * (gq.astype(np.float32) - Z0.astype(np.float32)[:, grp])
    assert np.array_equal(deq.astype(np.float32), wh)
    st = compare_jointq(gq, gs, Wd, A, Q0, S0f, Z0, bits, G, grid=grid, n_pass=n_pass, max_scans=max_scans,
                        wide=G > 128, perm=perm)
    _announce(f"   clean rows {st['clean_rows']}/{d_out}, rows equal after {st['flips']} forced toss-ups: "
              f"{st['flipped_rows']}, real mismatches {len(st['real_mismatches'])}, moves {int(out['n_moves'].item())}")
    assert st["real_mismatches"] == []
    orc = st["oracle"]
    assert np.array_equal(orc["Q"], gq)
    np.testing.assert_allclose(gs, orc["scales"], rtol=1e-4)
    assert abs(obj[0] - orc["f0"].sum()) <= 1e-4 * orc["f0"].sum()
    assert abs(obj[1] - orc["f1"].sum()) <= 1e-3 * orc["f1"].sum()
    assert obj[1] <= obj[0]
    f_gpu = oc.row_objective(Wd, wh.astype(np.float64), A)     # the objective of the GPU's result, by definition
    assert abs(f_gpu.sum() - obj[1]) <= 1e-3 * obj[1]
    # Moves: equal to the oracle's, except that a listed toss-up taken the other way is often undone in the next
    # scan, which leaves the codes alone and changes the count by two.  With equal codes the difference is even, and
    # it is bounded by what the listed toss-ups (of the run before any replay) can account for.
    n_listed = sum(len(t) for t in orc["ties"])
    d_moves = int(out["n_moves"].item()) - int(orc["moves"].sum())
    assert d_moves % 2 == 0 and abs(d_moves) <= 2 * (n_listed + st["flips"])
    if n_listed == 0:
        assert d_moves == 0
    limit = max(2, d_out // 10) if max_bad_rows is None else max_bad_rows
    assert st["flipped_rows"] <= limit
    return out, st


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,grid,start,n_pass,scans,lam", [
    (4, 128, 64, 512, torch.float32, "asym", "rtn", 1, 4, 0.0),
    (3, 64, 37, 384, torch.bfloat16, "asym", "gptq", 1, 3, 0.0),      # rows not a multiple of the workgroup's four
    (2, 32, 50, 256, torch.float32, "asym", "rtn", 1, 6, 0.0),
    (4, 16, 20, 128, torch.bfloat16, "asym", "rtn", 1, 4, 0.0),
    (3, 128, 40, 640, torch.bfloat16, "sym", "gptq", 1, 4, 0.0),
    (4, 64, 33, 256, torch.float32, "sym", "rtn", 1, 2, 0.0),
    (4, 128, 48, 512, torch.bfloat16, "asym", "gptq", 2, 3, 0.0),     # two passes over the groups
    (3, 64, 32, 256, torch.float32, "asym", "rtn", 1, 4, 25.0),       # proximity regularizer (Eq. (jointq_reg))
    (4, 48, 16, 192, torch.float32, "asym", "rtn", 1, 4, 0.0),        # group size not a power of two
    (3, 128, 64, 768, torch.bfloat16, "asym", "rtn", 1, 1, 0.0),      # one scan: decisions replayed exactly
    (4, 128, 520, 2048, torch.bfloat16, "asym", "gptq", 1, 4, 0.0),   # many workgroups, four super-blocks, every row compared
])
def test_jointq_matches_oracle(bits, G, d_out, d_in, dtype, grid, start, n_pass, scans, lam):
    _announce(f"jointq b{bits} g{G} {d_out}x{d_in} {dtype} {grid} start={start} passes={n_pass} scans={scans} lam={lam}")
    W, Wd, H32, Q0, S0, Z0 = _start(d_out, d_in, bits, G, seed=200 + bits + G, dtype=dtype, grid=grid, start=start)
    out, st = _run(W, Wd, H32, Q0, S0, Z0, bits, G, grid=grid, lam=lam, n_pass=n_pass, max_scans=scans)
    # reproducible bit for bit
    Q = torch.from_numpy(Q0.astype(np.uint8)).to(DEV)
    S = torch.from_numpy(S0.astype(np.float32)).to(DEV)
    Z = torch.from_numpy(Z0.astype(np.float32)).to(DEV)
    out2 = og.onecomp_jointq_refine(W, torch.from_numpy(H32).to(DEV), Q, S, Z, bits, G,
                                    grid="symmetric" if grid == "sym" else "minmax", lam=lam, n_pass=n_pass,
                                    max_scans=scans)
    torch.cuda.synchronize()
    for k in ("Q_codes", "scales", "W_hat", "objective", "n_moves"):
        assert torch.equal(out[k], out2[k])


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,grid,start,n_pass,scans,lam", [
    (4, 256, 40, 512, torch.float32, "asym", "rtn", 1, 3, 0.0),        # two blocks per group
    (3, 640, 33, 1280, torch.bfloat16, "asym", "gptq", 1, 4, 0.0),     # a group straddles a 512-column super-block
    (4, 1024, 24, 1024, torch.bfloat16, "sym", "gptq", 1, 4, 0.0),     # one group per row, symmetric: the paper's setting
    (3, 384, 20, 768, torch.float32, "asym", "rtn", 2, 2, 10.0),       # two passes, regularizer
    (4, 1024, 40, 1024, torch.bfloat16, "asym", "rtn", 1, 1, 0.0),     # one scan: decisions replayed exactly
])
def test_jointq_wide_groups(bits, G, d_out, d_in, dtype, grid, start, n_pass, scans, lam):
    """Groups of several 128-column blocks: b, c and a = A_gg u are carried from launch to launch."""
    _announce(f"jointq wide b{bits} g{G} {d_out}x{d_in} {dtype} {grid} start={start} passes={n_pass} scans={scans} lam={lam}")
    W, Wd, H32, Q0, S0, Z0 = _start(d_out, d_in, bits, G, seed=300 + bits + G % 7, dtype=dtype, grid=grid, start=start)
    _run(W, Wd, H32, Q0, S0, Z0, bits, G, grid=grid, lam=lam, n_pass=n_pass, max_scans=scans)


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,grid,n_pass,scans", [
    (4, 128, 48, 512, torch.bfloat16, "asym", 1, 4),
    (3, 64, 33, 384, torch.float32, "sym", 2, 2),
    (4, 256, 24, 768, torch.bfloat16, "asym", 1, 3),       # wide groups in sweep order
    (3, 32, 40, 256, torch.float32, "asym", 1, 1),         # one scan: decisions replayed exactly
])
def test_jointq_after_activation_ordering(bits, G, d_out, d_in, dtype, grid, n_pass, scans):
    """Start from the sweep with activation ordering: groups, scan order, scales and zeros follow the sweep's column
    order, W, H and the codes stay in the original one."""
    _announce(f"jointq act-order b{bits} g{G} {d_out}x{d_in} {dtype} {grid} passes={n_pass} scans={scans}")
    W, Wd, H32, Q0, S0, Z0, perm = _start(d_out, d_in, bits, G, seed=400 + bits + G % 11, dtype=dtype, grid=grid,
                                          start="gptq", act=True)
    assert not np.array_equal(perm, np.arange(d_in))
    _run(W, Wd, H32, Q0, S0, Z0, bits, G, grid=grid, n_pass=n_pass, max_scans=scans, perm=perm)


@pytest.mark.parametrize("bits,G,d_out,d_in,act,lam", [
    (4, 128, 1, 128, False, 0.0),       # one row, one group, one block
    (3, 256, 3, 256, False, 0.0),       # one group per row of two blocks, fewer rows than a workgroup holds
    (4, 16, 5, 48, False, 0.0),         # d_in below one MFMA tile of the products
    (4, 64, 17, 320, True, 5.0),        # regularizer together with a column order
])
def test_jointq_smallest_shapes(bits, G, d_out, d_in, act, lam):
    _announce(f"jointq small b{bits} g{G} {d_out}x{d_in} act={act} lam={lam}")
    r = _start(d_out, d_in, bits, G, seed=500 + G + d_out, start="gptq", act=act)
    perm = r[6] if act else None
    _run(*r[:6], bits, G, lam=lam, n_pass=2, max_scans=3, perm=perm)


def test_jointq_group_with_one_code_left_is_not_emptied():
    """2-bit symmetric grid, groups of 16: one row reaches a group with a single code away from the zero-point.  The
    move that would empty it has c' = 0 and N = 0 in exact arithmetic and rounding noise in fp32; it is no candidate
    (decided on the codes), so codes AND the number of moves equal the oracle's (the kernel once took the move and
    took it back in the next scan: same codes, two moves more)."""
    bits, G, d_out, d_in = 2, 16, 64, 768
    _announce(f"jointq b{bits} g{G} {d_out}x{d_in}: a group with one code left")
    W, Wd, H32, Q0, S0, Z0 = _start(d_out, d_in, bits, G, seed=339, dtype=torch.bfloat16, grid="sym", start="rtn")
    out, st = _run(W, Wd, H32, Q0, S0, Z0, bits, G, grid="sym", n_pass=2, max_scans=2)
    assert st["flips"] == 0 and int(out["n_moves"].item()) == int(st["oracle"]["moves"].sum())


def test_jointq_degenerate_rows_and_zero_passes():
    _announce("jointq: all-zero group, codes at the zero-point; n_pass = 0 returns the start")
    W, Wd, H32, Q0, S0, Z0 = _start(8, 256, 4, 64, seed=77)
    W = W.clone()
    W[0, :64] = 0.0
    Wd = to_f64(W)
    Q0, S0, Z0, _ = oc.rtn_quantize(Wd, 4, 64)
    out, _ = _run(W, Wd, H32, Q0, S0, Z0, 4, 64)
    assert np.array_equal(out["Q_codes"][0, :64].cpu().numpy(), Q0[0, :64])
    Q = torch.from_numpy(Q0.astype(np.uint8)).to(DEV)
    S = torch.from_numpy(S0.astype(np.float32)).to(DEV)
    Z = torch.from_numpy(Z0.astype(np.float32)).to(DEV)
    o0 = og.onecomp_jointq_refine(W, torch.from_numpy(H32).to(DEV), Q, S, Z, 4, 64, n_pass=0)
    torch.cuda.synchronize()
    assert np.array_equal(o0["Q_codes"].cpu().numpy(), Q0) and int(o0["n_moves"].item()) == 0
    assert float(o0["objective"][0]) == float(o0["objective"][1])
    with pytest.raises(og.OnecompError):     # wider than a block and not a multiple of 128
        og.onecomp_jointq_refine(W[:, :192].contiguous(), torch.from_numpy(H32[:192, :192].copy()).to(DEV),
                                 Q[:, :192].contiguous(), S[:, :1].contiguous(), Z[:, :1].contiguous(), 4, 192)


def test_jointq_full_size_sampled():
    """The 4096 x 14336 layer of the benchmark (bf16, 4-bit): the whole layer is refined on the GPU, a sample of rows
    is compared with the oracle, for group 128 on the min-max grid and for one group per row on the symmetric grid
    (the setting of the paper's JointQ table).  The sampled rows start from the oracle's own sweep, the other rows
    from the GPU's (rows are independent); H is the oracle's Gram matrix of 32768 tokens rounded to fp32."""
    cfg = synth.scaled(synth.CONFIGS["c3b"], n_tokens=32768)
    d_out, d_in, bits = cfg.d_out, cfg.d_in, cfg.bits
    _announce(f"jointq full size {d_out}x{d_in} b{bits}: oracle Gram and factor")
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, DEV)
    H32 = oc.hessian_accumulate(to_f64(X)).astype(np.float32)
    del X
    A = H32.astype(np.float64)
    f = oc.hessian_factor(A, cfg.damp)
    Wd = to_f64(W)
    H = torch.from_numpy(H32).to(DEV)
    U32 = torch.from_numpy(f["U"].astype(np.float32)).to(DEV)
    # group 128: four scans per visit, compared through the oracle's listed toss-ups.  One group per row (the setting
    # of the paper's JointQ table, and what bench.py times): four scans as well, replayed exactly scan by scan from
    # GPU calls with max_scans = 1, 2, 3, 4 (the first k scans of a row's only visit do not depend on max_scans).
    for G, grid, n_rows, scans in ((cfg.group_size, "asym", 12, 4), (d_in, "sym", 6, 4)):
        ggrid = "symmetric" if grid == "sym" else "minmax"
        rows = np.sort(np.random.default_rng(11).choice(d_out, size=n_rows, replace=False))
        _announce(f"jointq full size g{G} {grid}: oracle sweep of {n_rows} sampled rows, GPU sweep of the layer")
        o0 = oc.quantize_layer(Wd, f["U"], bits, G, rows=rows, grid=grid)
        g0 = og.onecomp_quantize_layer(W, U32, bits, G, want_w_hat=False, grid=ggrid)
        ridx = torch.from_numpy(rows).to(DEV)
        g0["Q_codes"][ridx] = torch.from_numpy(o0["Q"].astype(np.uint8)).to(DEV)
        g0["scales"][ridx] = torch.from_numpy(o0["scales"].astype(np.float32)).to(DEV)
        g0["zeros"][ridx] = torch.from_numpy(o0["zeros"].astype(np.float32)).to(DEV)
        by_scan = []
        for k in (range(1, scans + 1) if G == d_in else (scans,)):
            _announce(f"jointq full size: GPU refinement, one pass, up to {k} scan(s) per visit")
            Q, S = g0["Q_codes"].clone(), g0["scales"].clone()
            out = og.onecomp_jointq_refine(W, H, Q, S, g0["zeros"], bits, G, grid=ggrid, n_pass=1, max_scans=k,
                                           want_w_hat=False)
            torch.cuda.synchronize()
            obj = out["objective"].cpu().numpy()
            _announce(f"   objective {obj[0]:.4e} -> {obj[1]:.4e}, moves {int(out['n_moves'].item())}")
            by_scan.append(out["Q_codes"][ridx].cpu().numpy())
            gs = out["scales"][ridx].cpu().numpy()
            del out, Q, S
        assert obj[1] < 0.9 * obj[0]
        gq = by_scan[-1]
        del g0
        torch.cuda.empty_cache()
        _announce("jointq full size: oracle refinement of the sampled rows")
        S0f = o0["scales"].astype(np.float32).astype(np.float64)
        if G == d_in:
            st = compare_jointq_by_scan(by_scan, gs, Wd[rows], A, o0["Q"], S0f, o0["zeros"], bits, G, grid=grid)
        else:
            st = compare_jointq(gq, gs, Wd[rows], A, o0["Q"], S0f, o0["zeros"], bits, G, grid=grid, n_pass=1,
                                max_scans=scans, wide=G > 128)
        _announce(f"   clean rows {st['clean_rows']}/{len(rows)}, rows equal after {st['flips']} forced toss-ups: "
                  f"{st['flipped_rows']}, real mismatches {st['real_mismatches']}")
        assert st["real_mismatches"] == []
        assert np.array_equal(st["oracle"]["Q"], gq)
        np.testing.assert_allclose(gs, st["oracle"]["scales"], rtol=1e-4)
