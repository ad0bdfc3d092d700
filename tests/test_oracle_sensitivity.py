"""Pins for the oracle's bit-allocation sensitivity proxy (Sec. 4.1): err = 1/2 tr(B dW A dW^T), diagonal A, B."""
import numpy as np

from oracle import onecomp_oracle as oc


def test_sensitivity_matches_the_trace_formula_and_its_special_cases():
    r = np.random.default_rng(0)
    W = 0.02 * r.standard_normal((6, 64))
    a = r.uniform(0.5, 3.0, 64)
    b = r.uniform(0.5, 2.0, 6)
    for grid in ("asym", "sym"):
        _, _, _, What = oc.rtn_quantize(W, 3, 16, grid=grid)
        D = What - W
        # the paper's expression with the d_in x d_out matrix dW_p = D^T: 1/2 tr(B dW_p^T A dW_p)
        ref = 0.5 * np.trace(np.diag(b) @ D @ np.diag(a) @ D.T)
        assert abs(oc.rtn_sensitivity(W, a, b, 3, 16, grid=grid) - ref) <= 1e-14 * abs(ref)
        # identity A and B: half the squared Frobenius norm of the perturbation (stated in Sec. 4.1)
        assert abs(oc.rtn_sensitivity(W, np.ones(64), None, 3, 16, grid=grid)
                   - 0.5 * np.linalg.norm(D) ** 2) <= 1e-14
        # B = I: half the layer objective of Eq. (layerwise) for a diagonal Gram matrix
        assert abs(oc.rtn_sensitivity(W, a, None, 3, 16, grid=grid)
                   - 0.5 * oc.layer_loss(W, What, np.diag(a))) <= 1e-14
    # linear in A and in B, and more bits cost less
    e1 = oc.rtn_sensitivity(W, a, b, 4, 16)
    assert abs(oc.rtn_sensitivity(W, 3.0 * a, b, 4, 16) - 3.0 * e1) <= 1e-13 * e1
    assert abs(oc.rtn_sensitivity(W, a, 0.5 * b, 4, 16) - 0.5 * e1) <= 1e-13 * e1
    assert oc.rtn_sensitivity(W, a, b, 2, 16) > oc.rtn_sensitivity(W, a, b, 3, 16) > e1 > oc.rtn_sensitivity(W, a, b, 8, 16)
    # weights already on the grid cost nothing
    Wg = 0.01 * r.integers(0, 16, size=(4, 32)).astype(np.float64)
    Wg[:, 0] = 0.0; Wg[:, 1] = 0.15
    assert oc.rtn_sensitivity(Wg, np.ones(32), None, 4, 32) <= 1e-30
