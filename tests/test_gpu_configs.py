"""GPU parity at the shapes of the benchmark configurations that test_gpu_parity.py does not cover: the 4096 x 4096
and 14336 x 4096 layers, the 70B-class 28672 x 8192 layer at 2, 3 and 4 bits (the widths of the mixed allocation),
and the whole chain Gram -> factor -> sweep on the GPU against the oracle's chain at 4096 x 14336.  The calibration
sets are cut to 32768 tokens (more than 2 d_in for every width here) so that the float64 oracle finishes within
about a minute per case; the sweeps are compared on sampled rows spread over all output rows."""
import numpy as np
import pytest
import torch

import paper_2603_28845_amd as og
from paper_2603_28845_amd import synth
from oracle import onecomp_oracle as oc
from parity_util import compare_codes, rel_fro, to_f64
from test_gpu_parity import _announce, _check_sweep, _gpu_gram, _sample_rows

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
N_TOK = 32768


def _chain(cfg, bits_list, n_rows, own_h=True):
    """accumulate -> factor -> quantize, every call on the GPU and each fed the GPU's own previous result, against the
    oracle on sampled rows.  Two comparisons:
      stored H   the oracle factors and sweeps from the fp32 H the GPU produced (H is an fp32 array of the interface;
                 it is compared with the oracle's float64 Gram matrix to the 1e-4 bar): raw code agreement >= 99.9 %;
      own H      the oracle's own chain from X in float64 (own_h).  The two chains then differ by the fp32
                 accumulation of H (a few 1e-7 relative), which moves pre-rounding values by ~1e-6 of a grid step, more
                 than the sweep's own arithmetic does (~1e-7): every first difference must still be a rounding tie of
                 the oracle and replay exactly, the raw agreement is reported and bounded below by 99.5 %.
    Returns {bits: statistics of the stored-H comparison}."""
    d_out, d_in, G = cfg.d_out, cfg.d_in, cfg.group_size
    X = synth.make_activations(cfg, DEV)
    W = synth.make_weight(cfg, DEV)
    H = _gpu_gram(X, chunks=2)
    U, perm, info = og.onecomp_hessian_factor(H, cfg.damp, act_order=cfg.act_order)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    _announce("   oracle: Gram in float64, factor of the GPU's H" + (" and of its own" if own_h else ""))
    Ho = oc.hessian_accumulate(to_f64(X))
    del X
    Hg = to_f64(H)
    e_h = rel_fro(Hg, Ho)
    assert np.array_equal(Hg, Hg.T)
    factors = {"stored H": oc.hessian_factor(Hg, cfg.damp, act_order=cfg.act_order)}
    if own_h:
        factors["own H"] = oc.hessian_factor(Ho, cfg.damp, act_order=cfg.act_order)
    del Ho, Hg
    e_u = rel_fro(to_f64(U), factors["stored H"]["U"])
    _announce(f"   H rel. Frobenius error {e_h:.2e}; U against the oracle's factor of the same H {e_u:.2e}")
    assert e_h <= 1e-4 and e_u <= 1e-6
    rows = _sample_rows(d_out, n_rows)
    rt = torch.from_numpy(rows).to(DEV)
    Wd = to_f64(W)
    stats = {}
    for bits in bits_list:
        out = og.onecomp_quantize_layer(W, U, bits, G, perm=perm if cfg.act_order else None)
        torch.cuda.synchronize()
        gq, gz = out["Q_codes"][rt].cpu().numpy(), out["zeros"][rt].cpu().numpy()
        for which, f in factors.items():
            assert f["info"] == 0
            if cfg.act_order:
                np.testing.assert_array_equal(perm.cpu().numpy(), f["perm"])
            st = compare_codes(gq, gz, Wd, f["U"], bits, G, perm=f["perm"] if cfg.act_order else None, rows=rows)
            _announce(f"   b{bits}, oracle from {which}: raw agreement {st['raw_agree']:.6f}, tie flips {st['tie_flips']}, "
                      f"real {len(st['real_mismatches'])}")
            assert st["real_mismatches"] == [] and st["final_agree"] == 1.0
            np.testing.assert_allclose(out["scales"][rt].cpu().numpy(), st["oracle"]["scales"], rtol=1e-4)
            np.testing.assert_array_equal(gz, st["oracle"]["zeros"])
            # loss: the layer objective of the GPU's W_hat on the sampled rows, evaluated with the oracle's damped
            # matrix, against the oracle's sum of e^2 over the same rows
            D = Wd[rows] - to_f64(out["W_hat"][rt])
            lrows = float(((D @ f["Hd"]) * D).sum())
            assert abs(lrows - st["oracle"]["loss"]) <= 1e-3 * st["oracle"]["loss"]
            if which == "stored H":
                assert st["raw_agree"] >= 0.999, (bits, st["raw_agree"])
                assert st["tie_flips"] <= max(2, n_rows // 50)
                stats[bits] = st
            else:
                assert st["raw_agree"] >= 0.995, (bits, st["raw_agree"])
                assert st["tie_flips"] <= max(4, n_rows // 16)
    return stats


def test_config2_attention_projection_chained():
    """4096 x 4096, 4-bit, group 128: the three calls chained on the GPU against the oracle's chain, 256 rows."""
    cfg = synth.scaled(synth.CONFIGS["c2"], n_tokens=N_TOK)
    _announce(f"config 2: {cfg.d_out}x{cfg.d_in} b{cfg.bits} g{cfg.group_size}, chain on the GPU vs chain of the oracle")
    _chain(cfg, [cfg.bits], 256)


def test_config3_up_projection_chained():
    """14336 x 4096 (3.5 times the rows per launch of the square layer), rows sampled over all 14336."""
    cfg = synth.scaled(synth.CONFIGS["c3a"], n_tokens=N_TOK)
    _announce(f"config 3, up/gate shape: {cfg.d_out}x{cfg.d_in} b{cfg.bits} g{cfg.group_size}, chained")
    _chain(cfg, [cfg.bits], 256, own_h=False)


def test_config5_wide_output_layer_at_2_3_4_bits():
    """28672 x 8192 (70B-class up projection) at the three bit-widths of the mixed allocation, chained."""
    cfg = synth.scaled(synth.CONFIGS["c5a"], n_tokens=N_TOK)
    _announce(f"config 5, {cfg.d_out}x{cfg.d_in} g{cfg.group_size} at 2, 3 and 4 bits, chained")
    _chain(cfg, [2, 3, 4], 192, own_h=False)


def test_config3_down_projection_chained():
    """4096 x 14336, the headline layer: GPU Gram -> GPU factor -> GPU sweep against the oracle, from the stored H and
    end to end from its own float64 Gram matrix, loss included."""
    cfg = synth.scaled(synth.CONFIGS["c3b"], n_tokens=N_TOK)
    _announce(f"config 3, down projection {cfg.d_out}x{cfg.d_in} b{cfg.bits} g{cfg.group_size}, chained")
    _chain(cfg, [cfg.bits], 192)
