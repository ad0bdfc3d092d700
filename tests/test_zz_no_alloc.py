"""onecomp_rtn_sensitivity_static, the entry point that takes no workspace and allocates nothing (its partial sums
live in a fixed array of the library's device data), against onecomp_rtn_sensitivity on the same inputs: two calls in
a row, the second on a smaller layer (the array keeps the first call's contents), and against the float64 oracle."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2603_28845_amd as og
from paper_2603_28845_amd import synth
from oracle import onecomp_oracle as oc
from parity_util import to_f64

DEV = "cuda:0"


def _inputs(d_out, d_in, seed, dtype):
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=64, seed=seed, dtype=dtype)
    W = synth.make_weight(cfg, DEV)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    a = (torch.rand(d_in, generator=g) * 3.0 + 0.1).to(DEV)
    b = (torch.rand(d_out, generator=g) + 0.5).to(DEV)
    return W, a, b


@pytest.mark.gpu
def test_static_entry_point_matches_the_workspace_one():
    print("[case] no-allocation sensitivity: 4096x4096 bf16 then 300x768 fp32, through the C ABI", flush=True)
    cases = [(4096, 4096, 1, torch.bfloat16, 4, 128, "minmax"), (300, 768, 2, torch.float32, 3, 64, "symmetric")]
    err_s = torch.zeros(1, dtype=torch.float32, device=DEV)
    for d_out, d_in, seed, dtype, bits, G, grid in cases:
        W, a, b = _inputs(d_out, d_in, seed, dtype)
        ref = og.onecomp_rtn_sensitivity(W, a, bits, G, b_diag=b, grid=grid)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        got = og.onecomp_rtn_sensitivity_static(W, a, bits, G, b_diag=b, grid=grid, err=err_s)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before          # nothing allocated through torch either
        assert got.data_ptr() == err_s.data_ptr()
        # same kernels, same order of the partial sums: bit for bit the workspace variant's value
        assert float(got.item()) == float(ref.item()), (float(got.item()), float(ref.item()))
        want = oc.rtn_sensitivity(to_f64(W), to_f64(a), to_f64(b), bits, G, grid="sym" if grid == "symmetric" else "asym")
        assert abs(float(got.item()) - want) <= 1e-3 * want
        # and once more on the same input (the scratch now holds this call's own partial sums)
        again = og.onecomp_rtn_sensitivity_static(W, a, bits, G, b_diag=b, grid=grid)
        torch.cuda.synchronize()
        assert float(again.item()) == float(ref.item())


def test_static_entry_point_rejects_bad_arguments():
    # host-side checks only: nothing is launched and no device is touched
    lib = og.load_library()
    f = lib.onecomp_rtn_sensitivity_static
    P, NULL = ctypes.c_void_p(0x10000), ctypes.c_void_p(0)
    INVALID, UNSUPPORTED = 1, 2
    assert f(NULL, 1, 64, 256, P, NULL, 4, 128, 0, P, NULL) == INVALID
    assert f(P, 1, 64, 256, P, NULL, 4, 96, 0, P, NULL) == INVALID            # group does not divide d_in
    assert f(P, 1, (1 << 24) + 1, 256, P, NULL, 4, 128, 0, P, NULL) == INVALID  # beyond the size limit
    assert f(P, 1, 64, (1 << 24) + 128, P, NULL, 4, 128, 0, P, NULL) == INVALID
    assert f(P, 1, 64, 256, P, NULL, 5, 128, 0, P, NULL) == UNSUPPORTED
    assert f(ctypes.c_void_p(0x10004), 1, 64, 256, P, NULL, 4, 128, 0, P, NULL) == INVALID
