"""GPU parity: every C-ABI call against the float64 oracle on the same seeded inputs.

Bars (from the benchmark spec):
  H            relative Frobenius error <= 1e-4 (fp32 accumulation)
  codes        >= 99.9 % equal; every first-in-row mismatch is a rounding tie (|frac - 0.5| < 1e-4)
               of the oracle and, once that decision is replayed, the rest of the row matches exactly
  loss         relative error <= 1e-3
  W_hat        == scales * (Q - zeros) bit for bit
  U            computed in fp64, rounded once to fp32: relative Frobenius error <= 1e-6 against the
               oracle's U for the same fp32 H (bound: fp32 rounding 6e-8 per entry plus fp64
               factorization error ~ cond * 1e-16)
"""
import numpy as np
import pytest
import torch

import paper_2603_28845_amd as og
from paper_2603_28845_amd import synth
from oracle import onecomp_oracle as oc
from parity_util import compare_codes, rel_fro, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _announce(msg):
    print(f"[case] {msg}", flush=True)


def _gpu_gram(X, chunks=1, ws=None):
    d = X.shape[1]
    H = torch.zeros((d, d), dtype=torch.float32, device=DEV)
    n = X.shape[0]
    step = (n + chunks - 1) // chunks if n else 0
    if n == 0:
        og.onecomp_hessian_accumulate(X, H, workspace=ws)
    for t0 in range(0, n, max(step, 1)):
        og.onecomp_hessian_accumulate(X[t0:t0 + step], H, workspace=ws)
    torch.cuda.synchronize()
    return H


def _check_sweep(W, U32, bits, G, perm=None, rows=None, min_agree=0.999, grid="minmax", F32=None):
    """W: torch tensor on GPU (original order), U32: torch fp32 on GPU: the inverse factor the oracle sweeps with.
    F32: block form of the same factor; when given, the GPU sweeps with it instead of U32."""
    if F32 is None:
        out = og.onecomp_quantize_layer(W, U32, bits, G, perm=perm, grid=grid)
    else:
        out = og.onecomp_quantize_layer(W, F32, bits, G, perm=perm, grid=grid, form="block")
    torch.cuda.synchronize()
    Q = out["Q_codes"].cpu().numpy()
    S = out["scales"].cpu().numpy()
    Z = out["zeros"].cpu().numpy()
    WH = out["W_hat"].cpu().numpy()
    loss = float(out["loss"].item())
    d_out, d_in = W.shape
    p = None if perm is None else perm.cpu().numpy().astype(np.int64)
    sel = np.arange(d_out) if rows is None else np.asarray(rows)
    assert Q.max() <= 2 ** bits - 1
    assert np.all(Z == np.rint(Z)) and Z.min() >= 0 and Z.max() <= 2 ** bits - 1
    # dequantization exactness from the returned arrays, in fp32
    inv = np.arange(d_in) if p is None else np.argsort(p)
    g = inv // G
    deq = (S[:, g] * (Q.astype(np.float32) - Z[:, g])).astype(np.float32)
    assert np.array_equal(deq, WH)
    mse = grid.endswith("_mse")
    st = compare_codes(Q[sel], Z[sel], to_f64(W), to_f64(U32), bits, G, perm=p, rows=sel,
                       grid="sym" if grid.startswith("symmetric") else "asym",
                       scale_search="mse" if mse else None, gpu_scales=S[sel] if mse else None)
    if grid.startswith("symmetric"):
        assert np.all(Z == 2 ** (bits - 1) - 1) and Q.max() <= 2 ** bits - 2
    _announce(f"   raw agreement {st['raw_agree']:.6f}, tie flips {st['tie_flips']}, candidate flips {st['cand_flips']}, "
              f"real {len(st['real_mismatches'])}")
    assert st["real_mismatches"] == []
    assert st["final_agree"] == 1.0
    # Raw agreement: 99.9 % of the entries, before any replay.  A flip at a tie can change every later code of its
    # row, so where fewer than 100 rows are compared one legitimate flip alone may cost more than 0.1 %: only there
    # the bar is what the counted flips can account for (at most one row's worth of entries each).  The number of
    # flips is bounded everywhere.  With the scale search, two candidates whose error sums agree to 1e-4 are either
    # one a valid choice; such a flip changes its group and the rest of the row like a rounding tie does and is
    # counted the same way.
    n_cmp = len(sel)
    flips = st["tie_flips"] + st["cand_flips"]
    if n_cmp >= 100:
        assert st["raw_agree"] >= min_agree
    else:
        assert st["raw_agree"] >= min(min_agree, 1.0 - flips / n_cmp)
    assert st["tie_flips"] <= max(2, n_cmp // 50)
    assert st["cand_flips"] <= max(2, n_cmp // 20)
    if mse:
        # the search can only lower a group's own error against the plain grid at the same compensated values;
        # what the returned arrays allow to check: every scale is one of the shrunk ranges' (<= the plain one's)
        assert np.all(S > 0)
    orc = st["oracle"]
    np.testing.assert_allclose(S[sel], orc["scales"], rtol=1e-5)
    np.testing.assert_array_equal(Z[sel], orc["zeros"])
    np.testing.assert_allclose(WH[sel], orc["W_hat"], rtol=1e-5, atol=1e-9)
    if rows is None:
        assert abs(loss - orc["loss"]) <= 1e-3 * orc["loss"]
    return out, st


# ------------------------------------------------------------------------------------ Gram ---
def test_gram_c1_fp32():
    cfg = synth.CONFIGS["c1"]
    _announce("gram c1 fp32 1024x512")
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X)
    Ho = oc.hessian_accumulate(to_f64(X))
    Hn = H.cpu().numpy()
    assert rel_fro(Hn.astype(np.float64), Ho) <= 1e-4
    assert np.array_equal(Hn, Hn.T)
    # reproducible, and additive over chunks
    H2 = _gpu_gram(X)
    assert torch.equal(H, H2)
    H3 = _gpu_gram(X, chunks=3)
    assert rel_fro(to_f64(H3), Ho) <= 1e-4


@pytest.mark.parametrize("d_in,n_tok,dtype", [
    (128, 77, torch.bfloat16), (384, 1000, torch.bfloat16), (528, 333, torch.bfloat16),
    (1024, 4099, torch.bfloat16), (144, 50, torch.float32), (384, 1001, torch.float32),
    # 128 x 256 direct-to-LDS tiles: ragged channel edge, fewer tokens than the ring holds, odd number of steps
    (1040, 333, torch.bfloat16), (1536, 17, torch.bfloat16), (2304, 1000, torch.bfloat16), (4096, 515, torch.bfloat16),
])
def test_gram_ragged_shapes(d_in, n_tok, dtype):
    _announce(f"gram d_in={d_in} n_tok={n_tok} {dtype}")
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=d_in, n_tokens=n_tok, dtype=dtype, seed=3)
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X)
    Ho = oc.hessian_accumulate(to_f64(X))
    Hn = H.cpu().numpy()
    assert rel_fro(Hn.astype(np.float64), Ho) <= 1e-4
    assert np.array_equal(Hn, Hn.T)


def test_gram_big_tiles_bf16():
    # d_in large enough for the direct-to-LDS tile kernels, several stages and a ragged token tail
    _announce("gram d_in=8192 n_tok=1055 bf16 (direct-to-LDS tiles)")
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=8192, n_tokens=1055, seed=5)
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X)
    Hn = H.cpu().numpy()
    assert np.array_equal(Hn, Hn.T)
    Xd = to_f64(X)
    r = np.random.default_rng(0)
    for _ in range(6):
        i = np.sort(r.choice(8192, size=160, replace=False))
        k = np.sort(r.choice(8192, size=160, replace=False))
        assert rel_fro(Hn[np.ix_(i, k)].astype(np.float64), oc.hessian_tile(Xd, i, k)) <= 1e-4
    d = np.arange(8192)
    np.testing.assert_allclose(Hn[d, d], 2.0 * (Xd * Xd).sum(0), rtol=1e-4)
    # the tiles whose tokens two workgroups share (rows 0 .. 1023, columns from 1024 on): every entry and its mirror
    i = np.arange(0, 1024)
    k = np.arange(1024, 2560)
    assert rel_fro(Hn[np.ix_(i, k)].astype(np.float64), oc.hessian_tile(Xd, i, k)) <= 1e-4
    # additivity over calls on the same path (second call adds onto a non-zero H)
    H2 = _gpu_gram(torch.cat([X, X]), chunks=2)
    assert torch.equal(H2, H2.T)
    assert rel_fro(H2.cpu().numpy().astype(np.float64), 2.0 * Hn.astype(np.float64)) <= 1e-6


@pytest.mark.parametrize("d_in,n_tok,ws_frac", [
    (4096, 17001, 1.0),     # fewer tiles than CUs: every tile (the diagonal ones too) in 8 pieces of the token axis
    (4096, 9000, 1.0),      # fewer tokens: 4 pieces
    (8192, 9001, 1.0),      # two whole rounds plus 16 tiles: those 16 in 4 pieces
    (4096, 17001, 0.3),     # a workspace too small for 8 pieces per tile: fewer pieces
    (4096, 17001, 0.0005),  # a workspace too small for anything: as without one
])
def test_gram_with_workspace(d_in, n_tok, ws_frac):
    """onecomp_hessian_accumulate_ws: partial sums of token pieces parked in a workspace and added in a fixed order."""
    _announce(f"gram with workspace d_in={d_in} n_tok={n_tok} workspace fraction {ws_frac}")
    need = og.onecomp_accumulate_workspace_bytes(torch.bfloat16, d_in)
    assert need > 0 and need % (128 * 256 * 4) == 0    # whole partial sums of a 256 x 256 or a 384 x 256 tile
    ws = torch.empty(max(256, int(need * ws_frac) // 256 * 256), dtype=torch.uint8, device=DEV)
    ws.fill_(0xFF)          # the contents on entry must not matter (0xFFFFFFFF is a NaN)
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=d_in, n_tokens=n_tok, seed=9)
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X, ws=ws)
    assert torch.equal(H, H.T)
    H_again = _gpu_gram(X, ws=ws)
    assert torch.equal(H, H_again)                      # reproducible bit for bit
    Hn = H.cpu().numpy()
    Xd = to_f64(X)
    r = np.random.default_rng(1)
    for _ in range(4):
        i = np.sort(r.choice(d_in, size=200, replace=False))
        k = np.sort(r.choice(d_in, size=200, replace=False))
        assert rel_fro(Hn[np.ix_(i, k)].astype(np.float64), oc.hessian_tile(Xd, i, k)) <= 1e-4
    i = np.arange(0, 300)                               # a diagonal tile and its neighbour, every entry
    assert rel_fro(Hn[np.ix_(i, i)].astype(np.float64), oc.hessian_tile(Xd, i, i)) <= 1e-4
    d = np.arange(d_in)
    np.testing.assert_allclose(Hn[d, d], 2.0 * (Xd * Xd).sum(0), rtol=1e-4)
    # same sums as the call without a workspace, up to fp32 rounding order (each is ~3e-6 from the float64 result)
    H0 = _gpu_gram(X)
    assert rel_fro(Hn.astype(np.float64), H0.cpu().numpy().astype(np.float64)) <= 5e-6
    # additive on a non-zero H
    H2 = _gpu_gram(torch.cat([X, X]), chunks=2, ws=ws)
    assert torch.equal(H2, H2.T)
    assert rel_fro(H2.cpu().numpy().astype(np.float64), 2.0 * Hn.astype(np.float64)) <= 5e-6


@pytest.mark.parametrize("shape", ["wide", "big", "mid"])
@pytest.mark.parametrize("d_in,n_tok,with_ws", [
    (1040, 333, False),     # one ragged tile row and column
    (2304, 1000, True),     # 6 x 9 tiles of 384 x 256, every one in pieces when a workspace is there
    (4096, 9000, True),     # 10 2/3 tile rows of 384: the last one a third full
    (8192, 2063, False),    # more tiles than CUs, whole tiles only, ragged token tail
    (8192, 9001, True),     # whole rounds plus leftover tiles in pieces
])
def test_gram_tile_shapes(monkeypatch, shape, d_in, n_tok, with_ws):
    """Every tile shape of the direct-to-LDS Gram kernel on the same inputs (the library picks one by estimated
    cost; ONECOMP_GRAM_SHAPE forces it): 384 x 256 tiles with pinned accumulator registers, 256 x 256, 128 x 256."""
    _announce(f"gram tile shape {shape}: d_in={d_in} n_tok={n_tok} workspace={with_ws}")
    monkeypatch.setenv("ONECOMP_GRAM_SHAPE", shape)
    ws = None
    if with_ws:
        ws = torch.empty(og.onecomp_accumulate_workspace_bytes(torch.bfloat16, d_in), dtype=torch.uint8, device=DEV)
        ws.fill_(0xFF)
    plan = og.onecomp_accumulate_describe(torch.bfloat16, n_tok, d_in, ws.numel() if with_ws else 0)
    assert plan["tile_rows"] == {"wide": 384, "big": 256, "mid": 128}[shape] and plan["tile_cols"] == 256
    assert plan["launches"] >= 1
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=d_in, n_tokens=n_tok, seed=21)
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X, ws=ws)
    assert torch.equal(H, H.T)
    assert torch.equal(H, _gpu_gram(X, ws=ws))          # reproducible bit for bit
    Hn = H.cpu().numpy()
    Xd = to_f64(X)
    if d_in <= 2304:
        assert rel_fro(Hn.astype(np.float64), oc.hessian_accumulate(Xd)) <= 1e-4
    else:
        r = np.random.default_rng(2)
        for _ in range(4):
            i = np.sort(r.choice(d_in, size=200, replace=False))
            k = np.sort(r.choice(d_in, size=200, replace=False))
            assert rel_fro(Hn[np.ix_(i, k)].astype(np.float64), oc.hessian_tile(Xd, i, k)) <= 1e-4
        # the band along the diagonal, where tiles are cut by it: every entry of a 700-wide window and the far corner
        for lo in (0, 1300, d_in - 700):
            i = np.arange(lo, lo + 700)
            assert rel_fro(Hn[np.ix_(i, i)].astype(np.float64), oc.hessian_tile(Xd, i, i)) <= 1e-4
        d = np.arange(d_in)
        np.testing.assert_allclose(Hn[d, d], 2.0 * (Xd * Xd).sum(0), rtol=1e-4)
    # additive on a non-zero H, two calls of different length
    H2 = _gpu_gram(torch.cat([X, X[: n_tok // 2]]), chunks=2, ws=ws)
    assert torch.equal(H2, H2.T)
    ref2 = Hn.astype(np.float64) + _gpu_gram(X[: n_tok // 2], ws=ws).cpu().numpy().astype(np.float64)
    assert rel_fro(H2.cpu().numpy().astype(np.float64), ref2) <= 1e-5


def test_gram_schedule_of_the_benchmark_layer(monkeypatch):
    """What the library reports for the call bench.py times: with the workspace the 384 x 256 shape in four whole rounds
    plus one launch of pieces, without it 256 x 256 tiles in six rounds plus the split last round."""
    monkeypatch.delenv("ONECOMP_GRAM_SHAPE", raising=False)   # the library's own choice, not a forced shape
    _announce("gram schedule at d_in=14336, 262144 tokens")
    d_in, T = 14336, 262144
    need = og.onecomp_accumulate_workspace_bytes(torch.bfloat16, d_in)
    assert og.onecomp_accumulate_describe(torch.bfloat16, T, d_in, need) == {"tile_rows": 384, "tile_cols": 256, "launches": 5}
    assert og.onecomp_accumulate_describe(torch.bfloat16, T, d_in, 0) == {"tile_rows": 256, "tile_cols": 256, "launches": 7}
    assert og.onecomp_accumulate_describe(torch.float32, T, d_in, 0)["launches"] == 1
    # a call of few tokens (the calibration set handed over sequence by sequence): 256 x 256 tiles in one launch
    monkeypatch.delenv("ONECOMP_GRAM_ROUND_LAUNCHES", raising=False)
    for t in (2048, 16384):
        assert og.onecomp_accumulate_describe(torch.bfloat16, t, d_in, need) == {"tile_rows": 256, "tile_cols": 256, "launches": 1}
    assert og.onecomp_accumulate_describe(torch.bfloat16, 32768, d_in, need) == {"tile_rows": 384, "tile_cols": 256, "launches": 1}
    assert og.onecomp_accumulate_describe(torch.bfloat16, 65536, d_in, need) == {"tile_rows": 384, "tile_cols": 256, "launches": 5}


def test_mfma_rate_probe_runs():
    """The measurement aid: flop count as documented, and a rate between a tenth of the published peak and the peak."""
    _announce("register-only MFMA loops")
    sink = torch.zeros(64, dtype=torch.float32, device=DEV)
    n_cus = torch.cuda.get_device_properties(0).multi_processor_count
    for kind, per_mfma, peak in (("bf16", 2 * 32 * 32 * 16, 2500e12), ("f64", 2 * 16 * 16 * 4, 78.6e12)):
        for w, rnd in ((1, True), (2, True), (2, False)):
            og.onecomp_mfma_rate_probe(kind, w, 500, sink, random_operands=rnd)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = og.onecomp_mfma_rate_probe(kind, w, 4000, sink, random_operands=rnd)
            e1.record()
            torch.cuda.synchronize()
            assert flops == n_cus * w * 4 * 4000 * 8 * per_mfma
            rate = flops / (e0.elapsed_time(e1) * 1e-3)
            _announce(f"   {kind}, {w} wave(s) per SIMD, {'random' if rnd else 'constant'} operands: {rate / 1e12:.1f} TFLOP/s")
            assert 0.1 * peak < rate < 1.02 * peak
    assert float(sink.abs().sum().item()) == 0.0


def test_gram_full_calibration_set_sampled():
    """The Gram launch exactly as bench.py times it: 262144 tokens x 14336 channels (bf16) in ONE call.  The full
    float64 product is out of reach of the host, so the oracle computes sampled index blocks (over all tokens)
    and the diagonal; symmetry and additivity over calls are checked on the whole matrix."""
    cfg = synth.CONFIGS["c3b"]
    d_in = cfg.d_in
    _announce(f"gram full calibration set: {cfg.n_tokens} tokens x {d_in} channels, one call")
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X)
    assert torch.equal(H, H.T)
    r = np.random.default_rng(11)
    for s_i in range(4):
        i = np.sort(r.choice(d_in, size=96, replace=False))
        k = np.sort(r.choice(d_in, size=96, replace=False))
        cols = np.unique(np.concatenate([i, k]))
        Xs = to_f64(X[:, torch.from_numpy(cols).to(DEV)])          # gathered on the GPU: 262144 x <=192
        pos = {c: n for n, c in enumerate(cols)}
        ii = np.array([pos[c] for c in i]); kk = np.array([pos[c] for c in k])
        ref = oc.hessian_tile(Xs, ii, kk)
        got = H[torch.from_numpy(i).to(DEV)][:, torch.from_numpy(k).to(DEV)].cpu().numpy().astype(np.float64)
        err = rel_fro(got, ref)
        _announce(f"   block {s_i}: rel. Frobenius error {err:.2e}")
        assert err <= 1e-4
        if s_i == 0:
            dref = 2.0 * (Xs * Xs).sum(0)
            dgot = H[torch.from_numpy(cols).to(DEV), torch.from_numpy(cols).to(DEV)].cpu().numpy()
            np.testing.assert_allclose(dgot, dref, rtol=1e-4)
        del Xs
    # a block inside the tiles that two workgroups compute by halves of the tokens (tile row 0, tile column 4)
    i = np.arange(40, 136); k = np.arange(1100, 1196)
    cols = np.concatenate([i, k])
    Xs = to_f64(X[:, torch.from_numpy(cols).to(DEV)])
    ref = oc.hessian_tile(Xs, np.arange(96), np.arange(96, 192))
    err = rel_fro(H[40:136, 1100:1196].cpu().numpy().astype(np.float64), ref)
    _announce(f"   block in a token-split tile: rel. Frobenius error {err:.2e}")
    assert err <= 1e-4
    del Xs
    H4 = _gpu_gram(X, chunks=4)
    assert torch.equal(H4, H4.T)
    diff = (H4 - H).double().norm().item() / H.double().norm().item()
    _announce(f"   one call vs four calls: rel. difference {diff:.2e}")
    assert diff <= 1e-5
    del H4
    ws = torch.empty(og.onecomp_accumulate_workspace_bytes(torch.bfloat16, d_in), dtype=torch.uint8, device=DEV)
    Hw = _gpu_gram(X, ws=ws)
    assert torch.equal(Hw, Hw.T)
    diff = (Hw - H).double().norm().item() / H.double().norm().item()
    _announce(f"   with workspace ({ws.numel() >> 20} MiB) vs without: rel. difference {diff:.2e}")
    assert diff <= 5e-6


def test_gram_zero_tokens_and_strided_rows():
    _announce("gram zero tokens / strided X")
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=256, n_tokens=300, seed=4)
    X = synth.make_activations(cfg, DEV)
    H0 = torch.full((256, 256), 3.0, dtype=torch.float32, device=DEV)
    og.onecomp_hessian_accumulate(X[:0], H0)
    torch.cuda.synchronize()
    assert torch.all(H0 == 3.0)
    wide = torch.zeros((300, 512), dtype=X.dtype, device=DEV)
    wide[:, :256] = X
    H = _gpu_gram(wide[:, :256])
    assert rel_fro(to_f64(H), oc.hessian_accumulate(to_f64(X))) <= 1e-4


# ---------------------------------------------------------------------------------- factor ---
def _oracle_H32(d_in, n_tok, seed, outliers=True):
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=d_in, n_tokens=n_tok, seed=seed,
                       n_outlier=(max(1, d_in // 100) if outliers else 0))
    X = synth.make_activations(cfg, "cpu")
    H = oc.hessian_accumulate(to_f64(X))
    return H.astype(np.float32)


@pytest.mark.parametrize("d_in,act", [(128, False), (144, True), (384, False), (512, True), (1040, True), (2048, False)])
def test_factor_against_oracle(d_in, act):
    _announce(f"factor d_in={d_in} act_order={act}")
    H32 = _oracle_H32(d_in, 3 * d_in + 7, seed=11)
    f = oc.hessian_factor(H32.astype(np.float64), 0.01, act_order=act)
    U, perm, info = og.onecomp_hessian_factor(torch.from_numpy(H32).to(DEV), 0.01, act_order=act)
    torch.cuda.synchronize()
    assert int(info.item()) == 0 and f["info"] == 0
    Un = U.cpu().numpy().astype(np.float64)
    if act:
        np.testing.assert_array_equal(perm.cpu().numpy(), f["perm"])
    assert np.all(np.tril(Un, -1) == 0.0) and np.all(np.diag(Un) > 0.0)
    assert rel_fro(Un, f["U"]) <= 1e-6
    p = f["perm"]
    Hp = f["Hd"][np.ix_(p, p)]
    np.testing.assert_allclose(Un @ Hp @ Un.T, np.eye(d_in), atol=2e-5)


def test_factor_dead_channel_and_not_posdef():
    _announce("factor dead channel / not positive definite")
    H32 = _oracle_H32(256, 900, seed=12)
    H32[37, :] = 0.0
    H32[:, 37] = 0.0
    f = oc.hessian_factor(H32.astype(np.float64), 0.01)
    U, _, info = og.onecomp_hessian_factor(torch.from_numpy(H32).to(DEV), 0.01)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    assert rel_fro(U.cpu().numpy().astype(np.float64), f["U"]) <= 1e-6
    Hneg = -torch.eye(256, dtype=torch.float32, device=DEV)
    U, _, info = og.onecomp_hessian_factor(Hneg, 0.0)
    torch.cuda.synchronize()
    assert int(info.item()) > 0
    assert oc.hessian_factor(-np.eye(256), 0.0)["info"] > 0


def _oracle_block_factor(f):
    """Block form (128-column blocks) of the oracle's factor f = oc.hessian_factor(...), in float64."""
    p = f["perm"]
    R, info = oc.direct_factor(f["Hd"][np.ix_(p, p)])
    assert info == 0
    return oc.block_feedback_factor(f["U"], R, 128)


@pytest.mark.parametrize("d_in,act", [(128, False), (384, True), (1024, False), (1152, True), (2048, False)])
def test_block_factor_against_oracle(d_in, act):
    _announce(f"factor, block form, d_in={d_in} act_order={act}")
    H32 = _oracle_H32(d_in, 3 * d_in + 7, seed=13)
    f = oc.hessian_factor(H32.astype(np.float64), 0.01, act_order=act)
    Fo = _oracle_block_factor(f)
    F, perm, info = og.onecomp_hessian_factor(torch.from_numpy(H32).to(DEV), 0.01, act_order=act, form="block")
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Fn = F.cpu().numpy().astype(np.float64)
    if act:
        np.testing.assert_array_equal(perm.cpu().numpy(), f["perm"])
    assert np.all(np.tril(Fn, -1) == 0.0) and np.all(np.diag(Fn) > 0.0)
    assert rel_fro(Fn, Fo) <= 1e-6
    # the diagonal blocks are those of the inverse factor, bit for bit what the inverse form returns
    U, _, _ = og.onecomp_hessian_factor(torch.from_numpy(H32).to(DEV), 0.01, act_order=act)
    torch.cuda.synchronize()
    for b0 in range(0, d_in, 128):
        assert torch.equal(F[b0:b0 + 128, b0:b0 + 128], U[b0:b0 + 128, b0:b0 + 128])
    # outside them the largest entry-wise deviation stays at fp32 rounding of the entry
    off = np.abs(Fn - Fo)
    assert off.max() <= 2e-7 * np.abs(Fo).max()


def test_block_form_argument_checks():
    _announce("block form: rejected arguments")
    H = torch.eye(144, dtype=torch.float32, device=DEV)
    with pytest.raises(og.OnecompError) as ei:
        og.onecomp_hessian_factor(H, 0.01, form="block")          # d_in not a multiple of 128
    assert ei.value.code == 2
    W = torch.zeros((4, 512), dtype=torch.float32, device=DEV)
    F = torch.eye(512, dtype=torch.float32, device=DEV)
    with pytest.raises(og.OnecompError) as ei:
        og.onecomp_quantize_layer(W, F, 4, 256, form="block")     # group wider than a block, not the whole row
    assert ei.value.code == 2


# ----------------------------------------------------------------------------------- sweep ---
def _layer(d_out, d_in, n_tok, seed, dtype=torch.float32, act=False):
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=n_tok, seed=seed, dtype=dtype,
                       n_outlier=max(1, d_in // 100))
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, "cpu")
    H = oc.hessian_accumulate(to_f64(X))
    f = oc.hessian_factor(H, 0.01, act_order=act)
    U32 = torch.from_numpy(f["U"].astype(np.float32)).to(DEV)
    perm = torch.from_numpy(f["perm"].astype(np.int32)).to(DEV) if act else None
    return W, U32, perm


def test_sweep_c1():
    cfg = synth.CONFIGS["c1"]
    _announce("sweep c1 256x512 fp32 b4 g128")
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, "cpu")
    f = oc.hessian_factor(oc.hessian_accumulate(to_f64(X)), cfg.damp)
    U32 = torch.from_numpy(f["U"].astype(np.float32)).to(DEV)
    out, st = _check_sweep(W, U32, cfg.bits, cfg.group_size)
    # reproducible bit for bit
    out2 = og.onecomp_quantize_layer(W, U32, cfg.bits, cfg.group_size)
    torch.cuda.synchronize()
    for k in ("Q_codes", "scales", "zeros", "W_hat", "loss"):
        assert torch.equal(out[k], out2[k])


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,act", [
    (2, 64, 100, 384, torch.bfloat16, True),
    (3, 64, 7, 256, torch.float32, True),
    (8, 128, 64, 256, torch.float32, False),
    (4, 16, 33, 256, torch.bfloat16, False),
    (4, 32, 65, 128, torch.float32, True),
    (3, 256, 130, 512, torch.bfloat16, False),     # group wider than the block
    (4, 384, 1, 384, torch.float32, False),        # per-channel: one group per row
    (4, 128, 300, 1024, torch.bfloat16, True),
    (4, 384, 40, 1920, torch.float32, False),      # groups straddle 512-column boundaries
    (3, 640, 40, 1920, torch.bfloat16, True),      # groups wider than 512 columns, not a multiple of 512
    (4, 256, 70, 1280, torch.bfloat16, False),
    (4, 64, 130, 1664, torch.bfloat16, True),      # several super-blocks, the last one partial (13 blocks)
    (4, 16, 64, 640, torch.float32, False),
    (2, 32, 100, 1152, torch.bfloat16, True),
    (4, 512, 96, 1536, torch.bfloat16, False),     # groups of one super-block each: parameters fixed at the group start
    (3, 1024, 33, 2048, torch.float32, True),      # groups of two super-blocks
    (4, 1664, 130, 1664, torch.bfloat16, False),   # one group per row, last super-block partial
])
def test_sweep_variants(bits, G, d_out, d_in, dtype, act):
    _announce(f"sweep b{bits} g{G} {d_out}x{d_in} {dtype} act={act}")
    W, U32, perm = _layer(d_out, d_in, 2 * d_in + 13, seed=20 + bits + G, dtype=dtype, act=act)
    _check_sweep(W, U32, bits, G, perm=perm)


def _layer_block(d_out, d_in, n_tok, seed, dtype=torch.float32, act=False):
    """As _layer, plus the block form of the factor (from the oracle, rounded to fp32)."""
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=n_tok, seed=seed, dtype=dtype,
                       n_outlier=max(1, d_in // 100))
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, "cpu")
    f = oc.hessian_factor(oc.hessian_accumulate(to_f64(X)), 0.01, act_order=act)
    U32 = torch.from_numpy(f["U"].astype(np.float32)).to(DEV)
    F32 = torch.from_numpy(_oracle_block_factor(f).astype(np.float32)).to(DEV)
    perm = torch.from_numpy(f["perm"].astype(np.int32)).to(DEV) if act else None
    return W, U32, F32, perm


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,act,grid", [
    (4, 128, 256, 512, torch.float32, False, "minmax"),
    (4, 128, 300, 1024, torch.bfloat16, True, "minmax"),
    (3, 64, 7, 256, torch.float32, True, "minmax"),
    (2, 64, 100, 384, torch.bfloat16, True, "minmax"),
    (4, 16, 33, 256, torch.bfloat16, False, "minmax"),
    (4, 32, 65, 128, torch.float32, True, "minmax"),              # a single block: nothing crosses a block
    (4, 64, 130, 1664, torch.bfloat16, True, "minmax"),           # several super-blocks, the last one partial
    (8, 128, 64, 640, torch.float32, False, "minmax"),
    (2, 32, 100, 1152, torch.bfloat16, True, "minmax"),
    (4, 128, 100, 1024, torch.bfloat16, False, "symmetric"),
    (3, 64, 33, 640, torch.float32, True, "symmetric"),
    (4, 1280, 40, 1280, torch.bfloat16, False, "symmetric"),      # one group per row (the setting of the paper's Tables)
    (3, 1152, 65, 1152, torch.float32, True, "minmax"),
])
def test_sweep_block_form(bits, G, d_out, d_in, dtype, act, grid):
    """The sweep fed with the block form of the factor against the oracle's sweep with the inverse factor."""
    _announce(f"sweep, block form, b{bits} g{G} {d_out}x{d_in} {dtype} act={act} {grid}")
    W, U32, F32, perm = _layer_block(d_out, d_in, 2 * d_in + 13, seed=80 + bits + G % 5, dtype=dtype, act=act)
    out, _ = _check_sweep(W, U32, bits, G, perm=perm, grid=grid, F32=F32)
    out2 = og.onecomp_quantize_layer(W, F32, bits, G, perm=perm, grid=grid, form="block")
    torch.cuda.synchronize()
    for k in ("Q_codes", "scales", "zeros", "W_hat", "loss"):
        assert torch.equal(out[k], out2[k])


def test_end_to_end_block_form():
    """Gram, factor in block form and sweep on the GPU against the oracle's path with the inverse factor."""
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=200, d_in=1536, n_tokens=4096, seed=5)
    _announce("end to end, block form, 200x1536 bf16 b4 g128")
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X)
    F, _, info = og.onecomp_hessian_factor(H, cfg.damp, form="block")
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    f = oc.hessian_factor(H.cpu().numpy().astype(np.float64), cfg.damp)
    U32 = torch.from_numpy(f["U"].astype(np.float32)).to(DEV)
    _check_sweep(W, U32, cfg.bits, cfg.group_size, F32=F)


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,act", [
    (4, 128, 100, 1024, torch.bfloat16, False),
    (3, 64, 33, 640, torch.float32, True),
    (2, 16, 64, 256, torch.bfloat16, False),
    (8, 32, 7, 384, torch.float32, False),
    (4, 1280, 40, 1280, torch.bfloat16, False),    # per-channel, symmetric: the setting of the paper's Tables
    (3, 256, 70, 1024, torch.bfloat16, True),
])
def test_sweep_symmetric_grid(bits, G, d_out, d_in, dtype, act):
    _announce(f"sweep symmetric grid b{bits} g{G} {d_out}x{d_in} {dtype} act={act}")
    W, U32, perm = _layer(d_out, d_in, 2 * d_in + 13, seed=60 + bits + G % 7, dtype=dtype, act=act)
    _check_sweep(W, U32, bits, G, perm=perm, grid="symmetric")


def test_sweep_symmetric_all_zero_group():
    _announce("sweep symmetric grid, all-zero group")
    W, U32, _ = _layer(8, 256, 700, seed=33)
    W = W.clone()
    W[0, :] = 0.0             # every group of this row is zero from the start: s = 1, codes at the zero-point
    out, _ = _check_sweep(W, U32, 4, 64, grid="symmetric")
    assert torch.all(out["W_hat"][0] == 0) and torch.all(out["Q_codes"][0] == 7) and torch.all(out["scales"][0] == 1)


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,act,grid,block", [
    (4, 128, 256, 512, torch.float32, False, "minmax_mse", False),
    (3, 64, 100, 384, torch.bfloat16, True, "minmax_mse", False),
    (4, 32, 65, 256, torch.float32, False, "minmax_mse", False),
    (4, 16, 33, 256, torch.bfloat16, True, "minmax_mse", False),       # two groups per quad of lanes
    (3, 16, 64, 640, torch.float32, False, "symmetric_mse", True),
    (2, 128, 64, 1664, torch.bfloat16, True, "minmax_mse", False),     # several super-blocks, the last one partial
    (4, 128, 100, 1024, torch.bfloat16, False, "symmetric_mse", False),
    (3, 64, 33, 640, torch.float32, True, "symmetric_mse", False),
    (4, 1280, 40, 1280, torch.bfloat16, False, "symmetric_mse", False),  # one group per row
    (3, 256, 70, 1024, torch.bfloat16, True, "minmax_mse", False),       # group wider than the block
    (4, 640, 40, 1920, torch.float32, False, "minmax_mse", False),       # groups wider than 512 columns
    (4, 128, 130, 1024, torch.bfloat16, True, "minmax_mse", True),       # block form of the factor
    (4, 1152, 33, 1152, torch.float32, False, "symmetric_mse", True),
])
def test_sweep_scale_search(bits, G, d_out, d_in, dtype, act, grid, block):
    """Grid with the scale search (Sec. 4.3, "mse") against the oracle's sweep with the same search."""
    _announce(f"sweep with scale search b{bits} g{G} {d_out}x{d_in} {dtype} act={act} {grid} block={block}")
    if block:
        W, U32, F32, perm = _layer_block(d_out, d_in, 2 * d_in + 13, seed=120 + bits + G % 5, dtype=dtype, act=act)
    else:
        W, U32, perm = _layer(d_out, d_in, 2 * d_in + 13, seed=120 + bits + G % 5, dtype=dtype, act=act)
        F32 = None
    out, st = _check_sweep(W, U32, bits, G, perm=perm, grid=grid, F32=F32)
    # the search does something: most groups end on a shrunk range
    assert (st["oracle"]["cand"] > 0).mean() > 0.5
    out2 = og.onecomp_quantize_layer(W, U32 if F32 is None else F32, bits, G, perm=perm, grid=grid,
                                     form="inverse" if F32 is None else "block")
    torch.cuda.synchronize()
    for k in ("Q_codes", "scales", "zeros", "W_hat", "loss"):
        assert torch.equal(out[k], out2[k])


def test_sweep_scale_search_degenerate_groups():
    _announce("sweep with scale search: all-zero, constant and one-signed groups")
    W, U32, _ = _layer(8, 256, 700, seed=34)
    W = W.clone()
    W[0, :] = 0.0
    W[1, :] = 0.0125
    W[2, :] = W[2, :].abs() + 0.01
    out, _ = _check_sweep(W, U32, 4, 64, grid="minmax_mse")
    assert torch.all(out["W_hat"][0] == 0) and torch.all(out["scales"][0] == 1)
    _check_sweep(W, U32, 3, 64, grid="symmetric_mse")
    _check_sweep(W, U32, 4, 16, grid="minmax_mse")


def test_sweep_degenerate_and_one_signed_groups():
    _announce("sweep constant / one-signed groups")
    d_out, d_in, G = 8, 256, 64
    W, U32, _ = _layer(d_out, d_in, 700, seed=31)
    W = W.clone()
    W[0, :] = 0.0125            # every group constant at the start (s = 1 for the first group)
    W[1, :] = W[1, :].abs() + 0.01   # one-signed: zero-point clamps to 0
    W[2, 64:128] = -W[2, 64:128].abs() - 0.01
    _check_sweep(W, U32, 4, G)


# ------------------------------------------------------------------------------ end to end ---
def test_end_to_end_c1():
    cfg = synth.CONFIGS["c1"]
    _announce("end to end c1: accumulate -> factor -> quantize, all on the GPU, against the oracle end to end")
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, DEV)
    H = _gpu_gram(X, chunks=2)
    U, _, info = og.onecomp_hessian_factor(H, cfg.damp)
    out = og.onecomp_quantize_layer(W, U, cfg.bits, cfg.group_size)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Ho = oc.hessian_accumulate(to_f64(X))
    f = oc.hessian_factor(Ho, cfg.damp)
    assert rel_fro(to_f64(H), Ho) <= 1e-4
    assert rel_fro(to_f64(U), f["U"]) <= 1e-4
    Q = out["Q_codes"].cpu().numpy()
    Z = out["zeros"].cpu().numpy()
    st = compare_codes(Q, Z, to_f64(W), f["U"], cfg.bits, cfg.group_size)
    _announce(f"   raw agreement {st['raw_agree']:.6f}, tie flips {st['tie_flips']}, real {len(st['real_mismatches'])}")
    assert st["real_mismatches"] == [] and st["final_agree"] == 1.0 and st["raw_agree"] >= 0.999
    loss = float(out["loss"].item())
    assert abs(loss - st["oracle"]["loss"]) <= 1e-3 * st["oracle"]["loss"]
    # the loss the library reports is the layer objective for the damped Hessian
    direct = oc.layer_loss(to_f64(W), to_f64(out["W_hat"]), f["Hd"])
    assert abs(loss - direct) <= 1e-3 * direct


# ------------------------------------------------------------- full size, sampled oracle ---
def _sample_rows(d_out, n, seed=7):
    return np.sort(np.random.default_rng(seed).choice(d_out, size=n, replace=False))


def _full_size_sampled(name, act, sweeps):
    """One full-size layer of the benchmark configurations (bf16, d_in 14336): Gram against the oracle, both forms
    of the factor against the oracle's for the same H, sweeps on sampled rows with tie replay.  The calibration set
    is cut to 32768 tokens (still more than 2 d_in, so H has full rank as in the real workload) so that the float64
    oracle finishes in about a minute.  sweeps: list of (bits, n_rows, grid, form); the bar on raw agreement is
    99.9 % of the compared entries everywhere."""
    cfg = synth.scaled(synth.CONFIGS[name], n_tokens=32768)
    d_out, d_in = cfg.d_out, cfg.d_in
    assert cfg.act_order == act
    _announce(f"full size {name} {d_out}x{d_in} g{cfg.group_size} act={act}: gram ({cfg.n_tokens} tokens)")
    X = synth.make_activations(cfg, DEV)
    W = synth.make_weight(cfg, DEV)
    H = _gpu_gram(X)
    Xd = to_f64(X)
    Ho = oc.hessian_accumulate(Xd)
    Hn = H.cpu().numpy()
    assert np.array_equal(Hn, Hn.T)
    assert rel_fro(Hn.astype(np.float64), Ho) <= 1e-4
    del Xd, X
    _announce("full size: oracle factor")
    H32 = Ho.astype(np.float32)
    del Ho
    f = oc.hessian_factor(H32.astype(np.float64), cfg.damp, act_order=act)
    assert f["info"] == 0
    _announce("full size: GPU factor")
    U, perm, info = og.onecomp_hessian_factor(torch.from_numpy(H32).to(DEV), cfg.damp, act_order=act)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    if act:
        np.testing.assert_array_equal(perm.cpu().numpy(), f["perm"])
    err = rel_fro(U.cpu().numpy().astype(np.float64), f["U"])
    _announce(f"   U rel. Frobenius error {err:.3e}")
    assert err <= 1e-6
    del U
    F = None
    if any(form == "block" for _, _, _, form in sweeps):
        _announce("full size: factor in block form")
        F, _, info = og.onecomp_hessian_factor(torch.from_numpy(H32).to(DEV), cfg.damp, act_order=act, form="block")
        torch.cuda.synchronize()
        assert int(info.item()) == 0
        Fo = _oracle_block_factor(f)
        err = rel_fro(F.cpu().numpy().astype(np.float64), Fo)
        _announce(f"   F rel. Frobenius error {err:.3e}")
        assert err <= 1e-6
        del Fo
    U32 = torch.from_numpy(f["U"].astype(np.float32)).to(DEV)
    for bits, n_rows, grid, form in sweeps:
        _announce(f"full size: sweep b{bits} {grid}, {form} form, {n_rows} sampled rows")
        _, st = _check_sweep(W, U32, bits, cfg.group_size, perm=perm if act else None, rows=_sample_rows(d_out, n_rows),
                             min_agree=0.999, grid=grid, F32=F if form == "block" else None)
        assert st["tie_flips"] <= max(2, n_rows // 50)


def test_full_size_down_projection_sampled():
    """The 4096 x 14336 layer in the launch configuration bench.py times (4-bit, group 128, natural order): 512
    sampled rows with the inverse factor, 128 with the block form and with the scale search."""
    _full_size_sampled("c3b", False, [(4, 512, "minmax", "inverse"), (4, 128, "minmax", "block"),
                                      (4, 128, "minmax_mse", "inverse")])


def test_full_size_act_order_low_bit_sampled():
    """The same layer at 3 bits and at 2 bits, group 64, with activation ordering, either form of the factor."""
    _full_size_sampled("c4_3bit", True, [(3, 128, "minmax", "inverse"), (3, 128, "minmax", "block"),
                                         (2, 128, "minmax", "inverse"), (2, 128, "minmax", "block")])


def test_largest_layer_properties():
    """The widest benchmark layer (8192 x 28672, bf16, 3-bit, group 128): the float64 factorization of a 28672-wide
    matrix is out of the host's reach inside a test, so Gram and factor are
    checked through properties that hold at any size: H symmetric and equal to library-computed sampled entries,
    U^T U (H + lambda I) = I on sampled columns, W_hat = scales (Q - zeros) bit for bit, and the returned loss equal
    to tr((W - W_hat) Hd (W - W_hat)^T), an identity that only holds if every residual was propagated through U
    exactly as the sweep prescribes.  Both forms of the factor; their codes must agree but for tie flips."""
    # (the flips themselves are classified against the oracle in the sampled full-size tests at d_in = 14336)
    cfg = synth.scaled(synth.CONFIGS["c5b"], n_tokens=65536)
    d_out, d_in, G = cfg.d_out, cfg.d_in, cfg.group_size
    _announce(f"largest layer {d_out}x{d_in}: gram ({cfg.n_tokens} tokens)")
    X = synth.make_activations(cfg, DEV)
    W = synth.make_weight(cfg, DEV)
    H = _gpu_gram(X)
    assert torch.equal(H, H.T)
    idx = torch.from_numpy(np.sort(np.random.default_rng(3).choice(d_in, size=64, replace=False))).to(DEV)
    Xs = X[:, idx].double()
    ref = 2.0 * (Xs.T @ Xs)
    got = H[idx][:, idx].double()
    assert ((got - ref).norm() / ref.norm()).item() <= 1e-4
    del X, Xs
    lam = cfg.damp * H.diagonal().double().mean().item()
    Hd = H.double()
    Hd.diagonal().add_(lam)
    outs = {}
    for form in ("inverse", "block"):
        _announce(f"largest layer: factor and sweep, {form} form")
        U, _, info = og.onecomp_hessian_factor(H, cfg.damp, form=form)
        torch.cuda.synchronize()
        assert int(info.item()) == 0
        if form == "inverse":
            E = torch.zeros((d_in, 8), dtype=torch.float64, device=DEV)
            cols = [0, 1, 127, 128, 14335, 20000, 28670, 28671]
            for n, c in enumerate(cols):
                E[c, n] = 1.0
            Ud = U.double()
            V = Hd @ (Ud.T @ (Ud @ E))
            err = (V - E).abs().max().item()
            _announce(f"   max |Hd U^T U e_j - e_j| over 8 columns: {err:.2e}")
            assert err <= 1e-4
            del Ud, V, E
        out = og.onecomp_quantize_layer(W, U, cfg.bits, G, form=form)
        torch.cuda.synchronize()
        if form == "inverse":
            # the sweep itself against the oracle's at this width, on sampled rows, both fed the GPU's factor
            rows = _sample_rows(d_out, 24, seed=5)
            _announce(f"largest layer: oracle sweep of {len(rows)} rows with the GPU's U")
            Ud = U.cpu().numpy().astype(np.float64)
            st = compare_codes(out["Q_codes"][torch.from_numpy(rows).to(DEV)].cpu().numpy(),
                               out["zeros"][torch.from_numpy(rows).to(DEV)].cpu().numpy(), to_f64(W), Ud, cfg.bits, G,
                               rows=rows)
            del Ud
            _announce(f"   raw agreement {st['raw_agree']:.6f}, tie flips {st['tie_flips']}, real {len(st['real_mismatches'])}")
            assert st["real_mismatches"] == [] and st["final_agree"] == 1.0
            assert st["raw_agree"] >= min(0.999, 1.0 - st["tie_flips"] / len(rows)) and st["tie_flips"] <= 2
            np.testing.assert_allclose(out["scales"][torch.from_numpy(rows).to(DEV)].cpu().numpy(), st["oracle"]["scales"],
                                       rtol=1e-5)
        del U
        Q, S, Z, WH = out["Q_codes"], out["scales"], out["zeros"], out["W_hat"]
        assert int(Q.max().item()) <= 2 ** cfg.bits - 1
        assert torch.equal(Z, Z.round()) and Z.min().item() >= 0 and Z.max().item() <= 2 ** cfg.bits - 1
        deq = S.repeat_interleave(G, dim=1) * (Q.float() - Z.repeat_interleave(G, dim=1))
        assert torch.equal(deq, WH)
        del deq
        D = W.double() - WH.double()
        quad = ((D @ Hd) * D).sum().item()
        loss = float(out["loss"].item())
        _announce(f"   loss {loss:.6e}, tr(dW Hd dW^T) {quad:.6e}")
        assert abs(loss - quad) <= 1e-3 * quad
        del D
        outs[form] = Q.clone()
        del out, Q, S, Z, WH
    # The two forms reach the same codes except where a pre-rounding value sits within fp32 noise of a tie; such a
    # flip changes a good part of the rest of its row, and with 28672 columns a few rows in a hundred have one.
    agree = (outs["inverse"] == outs["block"]).float().mean().item()
    rows_equal = (outs["inverse"] == outs["block"]).all(dim=1).float().mean().item()
    _announce(f"   codes, inverse form vs block form: {agree:.6f} of the entries equal, {rows_equal:.4f} of the rows")
    assert agree >= 0.99 and rows_equal >= 0.9
