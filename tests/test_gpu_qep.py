"""GPU parity of the error-propagation (QEP) entry points against the float64 oracle, through the C ABI.

Bars:
  G        relative Frobenius error <= 1e-4 (bf16 products exact in fp32, fp32 accumulation), as for H
  W*       against the oracle's target for the SAME fp32 G, H (isolates the call): relative Frobenius error of
           W* <= 2e-6, and of the correction W* - W <= 1e-4.  The correction is W (G - H)^T (H + lambda I)^-1
           (G - H itself is exact here: both are given in fp32 and agree in their leading digits); three products
           with K up to d_in, each from operands split into two fp16 halves (22 significant bits, fp32
           accumulation), and a factor U rounded to fp32 give ~1e-6 (measured 1e-6 .. 4e-6).
"""
import numpy as np
import pytest
import torch

import paper_2603_28845_amd as og
from paper_2603_28845_amd import synth
from oracle import onecomp_oracle as oc
from parity_util import rel_fro, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _announce(msg):
    print(f"[case] {msg}", flush=True)


def _pair(d_in, n_tok, seed, rel_noise=0.05):
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=d_in, n_tokens=n_tok, seed=seed,
                       n_outlier=max(1, d_in // 100))
    X = synth.make_activations(cfg, DEV)
    Xh = synth.make_perturbed_activations(cfg, X, rel_noise)
    return cfg, X, Xh


def _gpu_cross(Xh, X, chunks=1):
    d = X.shape[1]
    G = torch.zeros((d, d), dtype=torch.float32, device=DEV)
    n = X.shape[0]
    step = (n + chunks - 1) // chunks
    for t0 in range(0, n, step):
        og.onecomp_crossgram_accumulate(Xh[t0:t0 + step], X[t0:t0 + step], G)
    torch.cuda.synchronize()
    return G


@pytest.mark.parametrize("d_in,n_tok", [(128, 77), (528, 333), (1040, 515), (1536, 17), (2304, 1000), (4096, 300)])
def test_crossgram_shapes(d_in, n_tok):
    _announce(f"cross-Gram d_in={d_in} n_tok={n_tok}")
    _, X, Xh = _pair(d_in, n_tok, seed=40 + d_in % 7)
    G = _gpu_cross(Xh, X)
    Go = oc.crossgram_accumulate(to_f64(Xh), to_f64(X))
    assert rel_fro(G.cpu().numpy().astype(np.float64), Go) <= 1e-4
    # additive over calls, and reproducible bit for bit
    G3 = _gpu_cross(Xh, X, chunks=3)
    assert rel_fro(G3.cpu().numpy().astype(np.float64), Go) <= 1e-4
    assert torch.equal(G, _gpu_cross(Xh, X))
    # the same matrix twice gives the symmetric Gram matrix
    H = torch.zeros_like(G)
    og.onecomp_hessian_accumulate(X, H)
    torch.cuda.synchronize()
    Gxx = _gpu_cross(X, X)
    assert rel_fro(Gxx.cpu().numpy().astype(np.float64), H.cpu().numpy().astype(np.float64)) <= 1e-6


@pytest.mark.parametrize("shape", ["wide", "big", "mid"])
@pytest.mark.parametrize("d_in,n_tok", [(1040, 515), (2304, 1000), (4096, 300)])
def test_crossgram_tile_shapes(monkeypatch, shape, d_in, n_tok):
    """Each tile shape of the cross-Gram kernel (384 x 256, 256 x 256, 128 x 256) on the same inputs."""
    _announce(f"cross-Gram tile shape {shape}: d_in={d_in} n_tok={n_tok}")
    monkeypatch.setenv("ONECOMP_GRAM_SHAPE", shape)
    _, X, Xh = _pair(d_in, n_tok, seed=60 + d_in % 7)
    G = _gpu_cross(Xh, X)
    Go = oc.crossgram_accumulate(to_f64(Xh), to_f64(X))
    assert rel_fro(G.cpu().numpy().astype(np.float64), Go) <= 1e-4
    assert torch.equal(G, _gpu_cross(Xh, X))
    G3 = _gpu_cross(Xh, X, chunks=3)
    assert rel_fro(G3.cpu().numpy().astype(np.float64), Go) <= 1e-4


def test_crossgram_strided_rows_and_zero_tokens():
    _announce("cross-Gram strided rows / zero tokens")
    _, X, Xh = _pair(256, 300, seed=3)
    wide = torch.zeros((300, 512), dtype=X.dtype, device=DEV)
    wide[:, :256] = X
    wide_h = torch.zeros((300, 768), dtype=X.dtype, device=DEV)
    wide_h[:, :256] = Xh
    G = _gpu_cross(Xh, X)
    Gs = _gpu_cross(wide_h[:, :256], wide[:, :256])
    assert torch.equal(G, Gs)
    G0 = torch.full((256, 256), 3.0, dtype=torch.float32, device=DEV)
    og.onecomp_crossgram_accumulate(Xh[:0], X[:0], G0)
    torch.cuda.synchronize()
    assert torch.all(G0 == 3.0)


@pytest.mark.parametrize("d_out,d_in,n_tok,dtype,act,alpha", [
    (96, 512, 2000, torch.float32, False, 1.0),
    (200, 1040, 4000, torch.bfloat16, True, 0.5),
    (7, 256, 900, torch.bfloat16, False, 0.25),
    (300, 2304, 6000, torch.bfloat16, True, 1.0),
])
def test_qep_target(d_out, d_in, n_tok, dtype, act, alpha):
    _announce(f"QEP target {d_out}x{d_in} {dtype} act={act} alpha={alpha}")
    cfg, X, Xh = _pair(d_in, n_tok, seed=50 + d_out % 5)
    wcfg = synth.scaled(cfg, d_out=d_out, dtype=dtype)
    W = synth.make_weight(wcfg, DEV)
    H = torch.zeros((d_in, d_in), dtype=torch.float32, device=DEV)
    og.onecomp_hessian_accumulate(Xh, H)
    G = _gpu_cross(Xh, X)
    U, perm, info = og.onecomp_hessian_factor(H, 0.01, act)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Ws = og.onecomp_qep_target(W, G, H, U, alpha, perm=perm)
    torch.cuda.synchronize()
    Wd = to_f64(W)
    ref = oc.qep_target(Wd, G.cpu().numpy().astype(np.float64), H.cpu().numpy().astype(np.float64), 0.01, alpha)
    got = Ws.cpu().numpy().astype(np.float64)
    e_all = rel_fro(got, ref)
    e_corr = rel_fro(got - Wd, ref - Wd)
    _announce(f"   W* rel. error {e_all:.2e}, correction rel. error {e_corr:.2e}, "
              f"|correction| / |W| = {np.linalg.norm(ref - Wd) / np.linalg.norm(Wd):.3f}")
    assert e_all <= 2e-6
    assert e_corr <= 1e-4
    # alpha = 0 returns the weights themselves, exactly
    W0 = og.onecomp_qep_target(W, G, H, U, 0.0, perm=perm)
    torch.cuda.synchronize()
    assert torch.equal(W0, W.to(torch.float32))


def test_qep_full_size_sampled():
    """The error-propagation calls at the 4096 x 14336 layer, in the launch configuration bench.py --qep times
    (bf16, natural order, alpha = 1, accumulate workspace, 384 x 256 cross-Gram tiles): sampled blocks of G against
    the oracle's cross-Gram of the same column subsets, and sampled rows of W* against the oracle's target for the
    SAME fp32 G and H (rows of W are independent in Eq. (qep)).  The calibration set is cut to 32768 tokens, still
    more than 2 d_in, so that the float64 side finishes in about a minute."""
    cfg = synth.scaled(synth.CONFIGS["c3b"], n_tokens=32768)
    d_out, d_in = cfg.d_out, cfg.d_in
    _announce(f"QEP full size {d_out}x{d_in}: activations, Gram and cross-Gram ({cfg.n_tokens} tokens)")
    X = synth.make_activations(cfg, DEV)
    Xh = synth.make_perturbed_activations(cfg, X, 0.05)
    W = synth.make_weight(cfg, DEV)
    ws = torch.empty(og.onecomp_accumulate_workspace_bytes(torch.bfloat16, d_in), dtype=torch.uint8, device=DEV)
    H = torch.zeros((d_in, d_in), dtype=torch.float32, device=DEV)
    og.onecomp_hessian_accumulate(Xh, H, workspace=ws)
    G = torch.zeros((d_in, d_in), dtype=torch.float32, device=DEV)
    og.onecomp_crossgram_accumulate(Xh, X, G)
    torch.cuda.synchronize()
    rng = np.random.default_rng(31)
    for _ in range(6):   # blocks of 64 x 64 entries anywhere in G (it is not symmetric: both triangles)
        i = np.sort(rng.choice(d_in, size=64, replace=False))
        k = np.sort(rng.choice(d_in, size=64, replace=False))
        ref = oc.crossgram_accumulate(to_f64(Xh[:, torch.from_numpy(i).to(DEV)]), to_f64(X[:, torch.from_numpy(k).to(DEV)]))
        got = G[torch.from_numpy(i).to(DEV)][:, torch.from_numpy(k).to(DEV)].cpu().numpy().astype(np.float64)
        assert rel_fro(got, ref) <= 1e-4
    del X, Xh, ws
    _announce("QEP full size: factor and corrected target on the GPU")
    U, perm, info = og.onecomp_hessian_factor(H, cfg.damp, False)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Ws = og.onecomp_qep_target(W, G, H, U, 1.0, perm=None)
    torch.cuda.synchronize()
    del U
    rows = np.sort(rng.choice(d_out, size=64, replace=False))
    _announce("QEP full size: oracle target on 64 sampled rows")
    Wd = to_f64(W)[rows]
    ref = oc.qep_target(Wd, G.cpu().numpy(), H.cpu().numpy(), cfg.damp, 1.0)
    got = Ws.cpu().numpy()[rows].astype(np.float64)
    e_all = rel_fro(got, ref)
    e_corr = rel_fro(got - Wd, ref - Wd)
    _announce(f"   W* rel. error {e_all:.2e}, correction rel. error {e_corr:.2e}, "
              f"|correction| / |W| = {np.linalg.norm(ref - Wd) / np.linalg.norm(Wd):.3f}")
    assert e_all <= 2e-6
    assert e_corr <= 1e-4


def test_qep_reduces_the_output_error_of_the_quantized_layer():
    """The point of the corrected target (Eq. (qep_obj)): quantizing W* reproduces the full-precision output X W^T
    from the perturbed input X_hat better than quantizing W does."""
    d_out, d_in, n_tok = 128, 1024, 4096
    _announce(f"QEP end to end {d_out}x{d_in}")
    cfg, X, Xh = _pair(d_in, n_tok, seed=9, rel_noise=0.1)
    W = synth.make_weight(synth.scaled(cfg, d_out=d_out, dtype=torch.float32), DEV)
    H = torch.zeros((d_in, d_in), dtype=torch.float32, device=DEV)
    og.onecomp_hessian_accumulate(Xh, H)
    G = _gpu_cross(Xh, X)
    U, _, info = og.onecomp_hessian_factor(H, 0.01)
    Ws = og.onecomp_qep_target(W, G, H, U, 1.0)
    q_base = og.onecomp_quantize_layer(W, U, 4, 128)
    q_qep = og.onecomp_quantize_layer(Ws, U, 4, 128)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    Xd, Xhd, Wd = X.double(), Xh.double(), W.double()
    target = Xd @ Wd.T
    err_base = torch.linalg.norm(Xhd @ q_base["W_hat"].double().T - target).item()
    err_qep = torch.linalg.norm(Xhd @ q_qep["W_hat"].double().T - target).item()
    err_unq = torch.linalg.norm(Xhd @ Wd.T - target).item()
    _announce(f"   output error: unquantized W on X_hat {err_unq:.4g}, quantized W {err_base:.4g}, quantized W* {err_qep:.4g}")
    assert err_qep < err_base


@pytest.mark.parametrize("bits,G,d_out,d_in,dtype,grid", [
    (4, 128, 300, 1024, torch.bfloat16, "minmax"),
    (3, 64, 33, 640, torch.float32, "symmetric"),
    (2, 16, 64, 256, torch.bfloat16, "minmax"),
    (8, 32, 7, 384, torch.float32, "minmax"),
    (4, 1280, 40, 1280, torch.bfloat16, "symmetric"),     # per-channel
    (4, 128, 4096, 4096, torch.bfloat16, "minmax"),       # a full-size attention projection
    (3, 128, 4096, 14336, torch.bfloat16, "minmax"),      # the layer bench.py times it on
    (2, 128, 28672, 8192, torch.bfloat16, "symmetric"),   # a 70B-class layer
])
def test_rtn_sensitivity(bits, G, d_out, d_in, dtype, grid):
    """Bit-allocation proxy 1/2 sum b_r a_c dW_rc^2 (Sec. 4.1).  Bar: relative error <= 1e-3 against the float64
    oracle, the bar of the sweep's loss (fp32 grid parameters; an isolated rounding tie moves one element by a
    grid step)."""
    _announce(f"RTN sensitivity b{bits} g{G} {d_out}x{d_in} {dtype} {grid}")
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=16, seed=70 + bits, dtype=dtype)
    W = synth.make_weight(cfg, DEV)
    gen = torch.Generator(device=DEV).manual_seed(5)
    a = (0.5 + 3.0 * torch.rand(d_in, generator=gen, device=DEV)).to(torch.float32)
    b = (0.5 + torch.rand(d_out, generator=gen, device=DEV)).to(torch.float32)
    og_grid = "sym" if grid == "symmetric" else "asym"
    for bd in (None, b):
        e = og.onecomp_rtn_sensitivity(W, a, bits, G, b_diag=bd, grid=grid)
        e2 = og.onecomp_rtn_sensitivity(W, a, bits, G, b_diag=bd, grid=grid)
        torch.cuda.synchronize()
        ref = oc.rtn_sensitivity(to_f64(W), to_f64(a), None if bd is None else to_f64(bd), bits, G, grid=og_grid)
        assert abs(float(e.item()) - ref) <= 1e-3 * ref
        assert torch.equal(e, e2)        # reproducible bit for bit
