"""The library allocates nothing, synchronizes nothing and clears its scratch with kernels, so a caller may record
a whole layer step into a HIP graph.  Each replay is checked against the eager result, with eager work and
synchronizations between the replays."""
import pytest
import torch

import paper_2603_28845_amd as og
from paper_2603_28845_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


# the wide case takes the paths of the benchmark layers: 384 x 256 Gram tiles with token pieces parked in the
# accumulate workspace and added by the reduce kernel, Cholesky steps in pairs, the triangular diagonal tile
@pytest.mark.parametrize("form,act,d_out,d_in", [("inverse", False, 130, 640), ("block", True, 130, 640),
                                                 ("inverse", True, 64, 8192)])
def test_layer_step_in_a_hip_graph(form, act, d_out, d_in):
    print(f"[case] graph capture of a layer step {d_out}x{d_in}, factor form {form}, act_order {act}", flush=True)
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=2100, seed=3)
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, DEV)
    d = cfg.d_in
    need = og.onecomp_accumulate_workspace_bytes(X.dtype, d)
    ws_a = torch.empty(need, dtype=torch.uint8, device=DEV) if need else None
    H = torch.zeros((d, d), dtype=torch.float32, device=DEV)
    U = torch.empty((d, d), dtype=torch.float32, device=DEV)
    info = torch.zeros(1, dtype=torch.int32, device=DEV)
    perm = torch.empty(d, dtype=torch.int32, device=DEV)
    ws_f = torch.empty(og.onecomp_factor_workspace_bytes(d), dtype=torch.uint8, device=DEV)
    ws_q = torch.empty(og.onecomp_quantize_workspace_bytes(cfg.d_out, d), dtype=torch.uint8, device=DEV)

    def new_out():
        return {
            "Q_codes": torch.empty((cfg.d_out, d), dtype=torch.uint8, device=DEV),
            "scales": torch.empty((cfg.d_out, d // cfg.group_size), dtype=torch.float32, device=DEV),
            "zeros": torch.empty((cfg.d_out, d // cfg.group_size), dtype=torch.float32, device=DEV),
            "W_hat": torch.empty((cfg.d_out, d), dtype=torch.float32, device=DEV),
            "loss": torch.zeros(1, dtype=torch.float32, device=DEV),
        }

    def step(out):
        H.zero_()                     # a fill kernel, not a memset node
        og.onecomp_hessian_accumulate(X[:1000], H, workspace=ws_a)
        og.onecomp_hessian_accumulate(X[1000:], H, workspace=ws_a)
        og.onecomp_hessian_factor(H, cfg.damp, act, U=U, perm_out=perm, info=info, workspace=ws_f, form=form)
        og.onecomp_quantize_layer(W, U, cfg.bits, cfg.group_size, perm=perm if act else None, workspace=ws_q,
                                  out=out, form=form)

    ref = new_out()
    step(ref)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    H_ref = H.clone()

    out = new_out()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(out)
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            step(out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep in range(3):
        for t in out.values():        # eager work between replays: wipe what the replay must rewrite
            t.zero_()
        H.fill_(7.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(H, H_ref), f"replay {rep}: H"
        for k in ref:
            assert torch.equal(out[k], ref[k]), f"replay {rep}: {k}"


def test_search_sweep_and_jointq_in_a_hip_graph():
    """The sweep with the scale search followed by the JointQ refinement, recorded once and replayed."""
    print("[case] graph capture of sweep (scale search) + JointQ refinement", flush=True)
    cfg = synth.scaled(synth.CONFIGS["c2"], d_out=70, d_in=512, n_tokens=1500, seed=4)
    W = synth.make_weight(cfg, DEV)
    X = synth.make_activations(cfg, DEV)
    d, G = cfg.d_in, 256                       # groups of two blocks: the launches that carry b, c and a along
    H = torch.zeros((d, d), dtype=torch.float32, device=DEV)
    og.onecomp_hessian_accumulate(X, H)
    U, _, info = og.onecomp_hessian_factor(H, cfg.damp)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    ws_q = torch.empty(og.onecomp_quantize_workspace_bytes(cfg.d_out, d), dtype=torch.uint8, device=DEV)
    ws_j = torch.empty(og.onecomp_jointq_workspace_bytes(cfg.d_out, d, G), dtype=torch.uint8, device=DEV)

    def new_out():
        return {
            "Q_codes": torch.empty((cfg.d_out, d), dtype=torch.uint8, device=DEV),
            "scales": torch.empty((cfg.d_out, d // G), dtype=torch.float32, device=DEV),
            "zeros": torch.empty((cfg.d_out, d // G), dtype=torch.float32, device=DEV),
            "W_hat": torch.empty((cfg.d_out, d), dtype=torch.float32, device=DEV),
            "loss": torch.zeros(1, dtype=torch.float32, device=DEV),
            "objective": torch.zeros(2, dtype=torch.float32, device=DEV),
            "n_moves": torch.zeros(1, dtype=torch.int32, device=DEV),
        }

    def step(out):
        og.onecomp_quantize_layer(W, U, cfg.bits, G, workspace=ws_q, out=out, grid="minmax_mse")
        og.onecomp_jointq_refine(W, H, out["Q_codes"], out["scales"], out["zeros"], cfg.bits, G, n_pass=1, max_scans=3,
                                 workspace=ws_j, out=out)

    ref = new_out()
    step(ref)
    torch.cuda.synchronize()
    assert float(ref["objective"][1]) < float(ref["objective"][0]) and int(ref["n_moves"].item()) > 0

    out = new_out()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(out)
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            step(out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(3):
        for t in out.values():
            t.zero_()
        ws_j.fill_(3)                 # stale scratch must not matter
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in ref:
            assert torch.equal(out[k], ref[k]), f"replay {rep}: {k}"
