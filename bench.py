#!/usr/bin/env python3
"""Benchmark of the layer-wise Hessian-aware quantization hot path on one MI355X.

One "step" = the whole hot path for one linear layer on synthetic inputs already resident in HBM:
    onecomp_hessian_accumulate (all calibration tokens) -> onecomp_hessian_factor -> onecomp_quantize_layer
Default workload: the Llama-style down projection W 4096 x 14336 (d_in = 14336), 262144 calibration
tokens, 4-bit, group 128, damp 0.01 (the layer the task's MFMA / HBM targets are quoted on).

Prints ONE JSON line: whole-step throughput in weights/s, per-phase times, the roofline of the dominant
kernel (Gram accumulation, MFMA bound), the sweep's HBM-roofline figure, and the float64 oracle timed on
the host cores over a bounded sample (reported baseline, not the target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# L2 <-> fabric bytes per call from rocprofv3 FETCH_SIZE / WRITE_SIZE (scaled by a plain 4 GiB copy), taken with
# `python bench.py --phase gram|sweep` under rocprofv3 --pmc; see profiles/c3b_hbm_traffic_pmc.md for the commands
GRAM_TRAFFIC_C3B = 69.3e9     # 68.1 GB fetched + 1.2 GB written per accumulate call (384 x 256 tiles, paced launches)
SWEEP_TRAFFIC_C3B = 13.6e9


def sweep_model_bytes_b128(d_out, d_in, B, G, w_bytes):
    """HBM bytes of the plain right-looking lazy-batch schedule with an fp32 working copy (block B):
    per block, the trailing columns are read and written once (8 B / element) and the block's rows of U are
    read (4 B / element); plus W in, codes (1 B) and W^ (4 B) out, scales and zeros.  Reference figure only:
    the library runs the two-level schedule modelled by sweep_model_bytes()."""
    n_b = d_in // B
    total = 0
    for k in range(n_b):
        total += 8 * d_out * (d_in - (k + 1) * B) + 4 * B * (d_in - k * B)
    total += d_out * d_in * (w_bytes + 1 + 4) + 8 * d_out * d_in // G
    return total


def sweep_model_bytes(d_out, d_in, G, w_bytes, SBW=512):
    """HBM bytes of the schedule onecomp_quantize_layer runs for G <= 128 (super-blocks of SBW = 512 columns):
      preparation   W in, fp32 working copy out; the strict upper block triangle of U read twice (maximum, then
                    split) and written once as two fp16 halves
      per super-block  its columns of the working copy (the fp32 feedback sums) and of W in, codes / W^ / scales /
                    zeros out, its residuals out as two fp16 halves (transposed panel), the 128 x 128 diagonal blocks
                    of U in
      far update    the columns beyond the super-block read and written once (8 B / element), the residual panel
                    and the super-block's rows of the split U read once
    Operands that the panel kernel writes and reads back itself (residual fragments) and re-reads of the same
    panel by different workgroups are counted once or not at all: they are served by L2."""
    total = d_out * d_in * (w_bytes + 4)
    upper = d_in * (d_in - 128) // 2
    total += upper * (4 + 4 + 4)
    for s0 in range(0, d_in, SBW):
        s1 = min(d_in, s0 + SBW)
        wdt = s1 - s0
        total += d_out * wdt * (4 + w_bytes + 1 + 4) + 8 * d_out * wdt // G + d_out * wdt * 4 + (wdt // 128) * 128 * 128 * 4
        rest = d_in - s1
        total += 8 * d_out * rest + 4 * d_out * wdt + 4 * wdt * rest
    return total


def _median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


PACED_MIN_TOKENS = 196608   # the library's own constant (gram.hip): long calls of the 384 x 256 shape run its paced form


def gram_kernel_name(d_in, bf16, plan=None, tokens_per_call=0):
    """Kernel onecomp_hessian_accumulate launches for this width; the ring kernel's tile shape (384 x 256, 256 x 256 or
    128 x 256) and how it cuts tiles along the token axis are the library's own choice (estimated rounds over the
    CUs), reported by onecomp_accumulate_describe."""
    if not bf16:
        return "gram_f32_kernel"
    if d_in < 1024:
        return "gram_bf16_kernel<2>"
    shape = {384: "RingWide", 256: "RingBig", 128: "RingMid"}.get(plan["tile_rows"], "?") if plan else "?"
    if shape == "RingWide" and plan["launches"] > 1 and tokens_per_call >= PACED_MIN_TOKENS:
        return "gram_bf16_ring_kernel<RingWide, false, true>"   # third argument: every wave pauses 64 cycles per step
    return f"gram_bf16_ring_kernel<{shape}, false, false>"


def achievable_mfma(og, torch):
    """What the matrix pipes of this box sustain on a register-only loop of independent MFMAs (no LDS, no memory
    traffic), timed with HIP events: the ceiling under which the Gram kernel (bf16) and the factor (fp64) run.  The
    published peaks assume the 2.4 GHz boost clock, which the chip does not hold under MFMA load."""
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    out = {}
    for kind, iters in (("bf16", 40000), ("f64", 16000)):
        for w, rnd in ((1, True), (2, True), (2, False)):
            og.onecomp_mfma_rate_probe(kind, w, 2000, sink, random_operands=rnd)                 # warm-up
            ts = []
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                flops = og.onecomp_mfma_rate_probe(kind, w, iters, sink, random_operands=rnd)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            key = f"{kind}_tflops_{w}_wave_per_simd" + ("" if rnd else "_constant_operands")
            out[key] = flops / (_median(ts) * 1e-3) / 1e12
    out["note"] = ("register-only loops of 8 independent MFMAs per trip (v_mfma_f32_32x32x16_bf16, v_mfma_f64_16x16x4_f64) "
                   "on every CU, 5-15 ms each, operands pseudo-random per lane and MFMA unless marked constant (the pipes "
                   "draw more power on toggling data and the clock follows); published peaks 2500 / 78.6")
    return out


def cpu_baseline(cfg, synth, seconds_hint=20.0):
    """Oracle (float64, numpy) timed per phase on bounded samples of the same workload and extrapolated by
    work: Gram over n_s tokens (linear in tokens), factor at d_s = d_in / 2 (cubic), sweep of r_s rows at
    d_s columns (linear in rows, quadratic in columns)."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import onecomp_oracle as oc

    n_s = min(16384, cfg.n_tokens)
    d_s = max(128, (cfg.d_in // 2) // cfg.group_size * cfg.group_size)
    r_s = min(256, cfg.d_out)
    X = synth.make_activations(cfg, "cpu", n_tokens=n_s).to(dtype=__import__("torch").float64).numpy()
    t0 = time.perf_counter()
    H = oc.hessian_accumulate(X)
    t_gram = time.perf_counter() - t0
    Hs = np.ascontiguousarray(H[:d_s, :d_s])
    del H
    t0 = time.perf_counter()
    # the sample has full rank when it holds at least as many tokens as columns; a shorter one (the widest layers)
    # is held positive definite by heavier damping, which does not change the work
    damp = cfg.damp if n_s >= 2 * d_s else max(cfg.damp, 0.01) * 10.0
    f = oc.hessian_factor(Hs, damp, act_order=cfg.act_order)
    t_factor = time.perf_counter() - t0
    Wc = synth.scaled(cfg, d_out=r_s, d_in=d_s)
    W = synth.make_weight(Wc, "cpu").to(dtype=__import__("torch").float64).numpy()
    t0 = time.perf_counter()
    oc.quantize_layer(W, f["U"], cfg.bits, cfg.group_size, perm=f["perm"])
    t_sweep = time.perf_counter() - t0
    est = (t_gram * cfg.n_tokens / n_s + t_factor * (cfg.d_in / d_s) ** 3 +
           t_sweep * (cfg.d_out / r_s) * (cfg.d_in / d_s) ** 2)
    threads = 1
    for info in threadpool_info():
        if info.get("user_api") == "blas":
            threads = max(threads, int(info.get("num_threads", 1)))
    return {
        "value": cfg.d_out * cfg.d_in / est, "unit": "weights/s", "cores": threads, "kind": "oracle",
        "sample": (f"extrapolated by work from: Gram over {n_s} of {cfg.n_tokens} tokens at d_in={cfg.d_in} "
                   f"({t_gram:.2f} s), factor at d={d_s} ({t_factor:.2f} s, x(d_in/d)^3), sweep of {r_s} rows x {d_s} "
                   f"columns ({t_sweep:.2f} s, x rows x (d_in/d)^2); estimated full step {est:.0f} s"),
        "measured_s": {"gram": t_gram, "factor": t_factor, "sweep": t_sweep},
    }


def bench_jointq(args, cfg, og, W, H, out, perm):
    """JointQ refinement (Sec. 4.3.2) of the sweep's result: args.jointq passes over the groups, four scans per
    visit, on the H of the timed steps.  The refinement works on copies; two timed calls after one warm-up."""
    import torch
    d_out, d_in, G = cfg.d_out, cfg.d_in, cfg.group_size
    base_grid = "symmetric" if args.grid.startswith("symmetric") else "minmax"
    ws = torch.empty(og.onecomp_jointq_workspace_bytes(d_out, d_in, G), dtype=torch.uint8, device=W.device)
    ms = []
    for it in range(3):
        Q, S = out["Q_codes"].clone(), out["scales"].clone()
        e = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        e[0].record()
        r = og.onecomp_jointq_refine(W, H, Q, S, out["zeros"], cfg.bits, G, grid=base_grid, n_pass=args.jointq,
                                     max_scans=4, workspace=ws, want_w_hat=False, perm=perm)
        e[1].record()
        torch.cuda.synchronize()
        if it > 0:
            ms.append(e[0].elapsed_time(e[1]))
    t = _median(ms)
    obj = r["objective"].tolist()
    # products per call: the gradient once; per pass one update per group (groups up to 128 columns) or, for wider
    # groups, a = A_gg u once, one update per scan and the gradient update, each over the group's own columns only
    if G <= 128:
        flops = 2.0 * d_out * d_in * d_in * (1 + args.jointq)
    else:
        flops = 2.0 * d_out * d_in * (d_in + args.jointq * ((1 + 4) * G + d_in))
    return {
        "what": f"onecomp_jointq_refine on the sweep's codes and scales: {args.jointq} pass(es) over the groups, up to 4 "
                "scans per visit, lam 0",
        "ms": t, "weights_per_sec": d_out * d_in / (t * 1e-3),
        "objective_before": obj[0], "objective_after": obj[1], "moves": int(r["n_moves"].item()),
        "roofline": {"kernel": "trailing_kernel (split-fp16 products: gradient R A once, then the rank-group updates) + "
                               "jq_visit_kernel",
                     "bound": "mfma", "achieved": 3.0 * flops / (t * 1e-3) / 1e12, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": 3.0 * flops / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "fp32_equivalent_tflops": flops / (t * 1e-3) / 1e12,
                     "note": "executed fp16 MFMA flops = 3 products x the fp32-equivalent flops of the gradient and its updates "
                             "(2 d_out d_in^2 (1 + passes) for groups up to 128 columns), over the whole call: "
                             "the sequential local search (jq_visit_kernel, no MFMA work) is inside the time"},
    }


def bench_qep(args, cfg, og, synth, W, X, H, U, info, perm, ws_f, ws_q, out, ws_a=None):
    """The layer with error propagation: X_hat = X perturbed by 5 % stands in for the activations of the partly
    quantized model.  One step = H from X_hat, G from (X_hat, X), factor, corrected target W*, sweep of W*."""
    import torch
    d_out, d_in = cfg.d_out, cfg.d_in
    Xh = synth.make_perturbed_activations(cfg, X, 0.05)
    G = torch.zeros_like(H)
    Ws = torch.empty((d_out, d_in), dtype=torch.float32, device=W.device)
    ws_p = torch.empty(og.onecomp_qep_workspace_bytes(d_out, d_in), dtype=torch.uint8, device=W.device)

    def step(rec=None):
        e = [torch.cuda.Event(enable_timing=True) for _ in range(6)]
        H.zero_(); G.zero_()
        e[0].record()
        og.onecomp_hessian_accumulate(Xh, H, workspace=ws_a)
        e[1].record()
        og.onecomp_crossgram_accumulate(Xh, X, G)
        e[2].record()
        og.onecomp_hessian_factor(H, cfg.damp, cfg.act_order, U=U, perm_out=perm, info=info, workspace=ws_f)
        e[3].record()
        og.onecomp_qep_target(W, G, H, U, 1.0, perm=perm, W_star=Ws, workspace=ws_p)
        e[4].record()
        og.onecomp_quantize_layer(Ws, U, cfg.bits, cfg.group_size, perm=perm, workspace=ws_q, out=out)
        e[5].record()
        if rec is not None:
            rec.append(e)

    for _ in range(max(1, args.warmup)):
        step()
    torch.cuda.synchronize()
    rec = []
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    assert int(info.item()) == 0
    # the bit-allocation proxy on the same layer (one candidate = the configured bits / group): memory bound
    a_diag = torch.diagonal(H).contiguous()
    e_s = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    og.onecomp_rtn_sensitivity(W, a_diag, cfg.bits, cfg.group_size)
    e_s[0].record()
    for _ in range(10):
        sens = og.onecomp_rtn_sensitivity(W, a_diag, cfg.bits, cfg.group_size)
    e_s[1].record()
    torch.cuda.synchronize()
    sens_ms = e_s[0].elapsed_time(e_s[1]) / 10
    names = ["hessian_accumulate", "crossgram_accumulate", "hessian_factor", "qep_target", "quantize_layer"]
    ph = {n: _median([e[i].elapsed_time(e[i + 1]) for e in rec]) for i, n in enumerate(names)}
    total = sum(ph.values())
    return {
        "phases_ms": ph, "ms_per_step": total, "weights_per_sec": d_out * d_in / (total * 1e-3),
        "crossgram_tflops": 2.0 * cfg.n_tokens * d_in * d_in / (ph["crossgram_accumulate"] * 1e-3) / 1e12,
        "qep_target_tflops_fp32": 4.0 * d_out * d_in * d_in / (ph["qep_target"] * 1e-3) / 1e12,
        "loss": float(out["loss"].item()),
        "rtn_sensitivity": {"ms": sens_ms, "value": float(sens.item()),
                            "gbs": W.numel() * W.element_size() / (sens_ms * 1e-3) / 1e9,
                            "note": "one candidate configuration; W read once from HBM (second pass from cache)"},
        "note": "X_hat = X * (1 + 0.05 N(0,1)); alpha = 1; cross-Gram flops 2 T d_in^2 (no symmetry to use); target flops "
                "4 d_out d_in^2 (one full and two triangular products)",
    }


def bench_c5(args, og, synth):
    """The 70B-class configuration as stated: six layer instances (three of 28672 x 8192, three of 8192 x 28672) whose
    bit-widths are a seeded shuffle of [2, 3, 4, 2, 3, 4].  One step = the whole hot path (accumulate over all
    calibration tokens, factor, quantize) for each of the six layers in turn, every input resident in HBM; the value
    is allocation-weighted: all six layers' weights over the step's time.  Layers of one shape share H, U, the
    outputs and the workspaces (a layer-wise quantizer holds one layer at a time)."""
    import torch
    dev = "cuda:0"
    layers = synth.c5_allocation(0)
    shapes = {}
    data = []
    for cfg in layers:
        key = (cfg.d_out, cfg.d_in)
        if key not in shapes:
            d_out, d_in = key
            ws_a_bytes = og.onecomp_accumulate_workspace_bytes(cfg.dtype, d_in)
            shapes[key] = {
                "H": torch.zeros((d_in, d_in), dtype=torch.float32, device=dev),
                "U": torch.empty((d_in, d_in), dtype=torch.float32, device=dev),
                "info": torch.zeros(1, dtype=torch.int32, device=dev),
                "ws_a": torch.empty(ws_a_bytes, dtype=torch.uint8, device=dev) if ws_a_bytes > 0 else None,
                "ws_f": torch.empty(og.onecomp_factor_workspace_bytes(d_in), dtype=torch.uint8, device=dev),
                "ws_q": torch.empty(og.onecomp_quantize_workspace_bytes(d_out, d_in, 128), dtype=torch.uint8, device=dev),
                "out": {"Q_codes": torch.empty((d_out, d_in), dtype=torch.uint8, device=dev),
                        "scales": torch.empty((d_out, d_in // cfg.group_size), dtype=torch.float32, device=dev),
                        "zeros": torch.empty((d_out, d_in // cfg.group_size), dtype=torch.float32, device=dev),
                        "W_hat": torch.empty((d_out, d_in), dtype=torch.float32, device=dev),
                        "loss": torch.zeros(1, dtype=torch.float32, device=dev)},
            }
        data.append((cfg, synth.make_weight(cfg, dev), synth.make_activations(cfg, dev)))

    def step(rec=None):
        for i, (cfg, W, X) in enumerate(data):
            b = shapes[(cfg.d_out, cfg.d_in)]
            e = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            b["H"].zero_()
            e[0].record()
            og.onecomp_hessian_accumulate(X, b["H"], workspace=b["ws_a"])
            e[1].record()
            og.onecomp_hessian_factor(b["H"], cfg.damp, cfg.act_order, U=b["U"], info=b["info"], workspace=b["ws_f"],
                                      form=args.factor_form)
            e[2].record()
            og.onecomp_quantize_layer(W, b["U"], cfg.bits, cfg.group_size, workspace=b["ws_q"], out=b["out"],
                                      form=args.factor_form, grid=args.grid)
            e[3].record()
            if rec is not None:
                rec[i].append(e)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    rec = [[] for _ in data]
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(rec)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for b in shapes.values():
        assert int(b["info"].item()) == 0, "Hessian not positive definite"
    ms_per_step = wall * 1e3 / args.steps
    per_layer, weights = [], 0
    for (cfg, W, X), r in zip(data, rec):
        ph = [_median([e[i].elapsed_time(e[i + 1]) for e in r]) for i in range(3)]
        n = cfg.d_out * cfg.d_in
        weights += n
        per_layer.append({"layer": cfg.name, "shape": [cfg.d_out, cfg.d_in], "bits": cfg.bits, "tokens": cfg.n_tokens,
                          "phases_ms": {"hessian_accumulate": ph[0], "hessian_factor": ph[1], "quantize_layer": ph[2]},
                          "ms": sum(ph), "weights_per_sec": n / (sum(ph) * 1e-3),
                          "weights_per_sec_factor_plus_sweep": n / ((ph[1] + ph[2]) * 1e-3)})
    # dominant kernel: the Gram launch of the 28672-wide layers
    wide = [(cfg, p) for (cfg, _, _), p in zip(data, per_layer) if cfg.d_in == 28672]
    cfgw, pw = wide[0]
    gram_ms = _median([p["phases_ms"]["hessian_accumulate"] for _, p in wide])
    flops = float(cfgw.n_tokens) * cfgw.d_in * (cfgw.d_in + 1)
    tfl = flops / (gram_ms * 1e-3) / 1e12
    return {
        "metric": "weights_quantized_per_sec", "value": weights / (ms_per_step * 1e-3), "unit": "weights/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 inputs, f32 accumulate, f64 factor and sweep decisions", "data": "synthetic",
        "config": {"workload": "c5: 70B-class shapes, 3 x (28672x8192) + 3 x (8192x28672) bf16, 131072 tokens each, group 128, "
                               "bit-widths " + ", ".join(f"{c.name.split('_')[0]}={c.bits}" for c, _, _ in data)
                               + f" (seeded shuffle of 2,3,4,2,3,4; mean 3), {args.grid} grid, damp 0.01, factor form {args.factor_form}; "
                               "one step = all six layers"},
        "allocation_weighted_weights_per_sec": weights / (sum(p["ms"] for p in per_layer) * 1e-3),
        "layers": per_layer,
        "roofline": {"kernel": "gram_bf16_ring_kernel", "bound": "mfma", "achieved": tfl, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": tfl / PEAK_BF16_TFLOPS, "traffic": None,
                     "note": "Gram call of the 8192x28672 layers (median of the three): T*d_in*(d_in+1) flops / call time",
                     "call_ms": gram_ms},
        "cpu_baseline": None,
        "cpu_baseline_note": "the oracle is timed for the default workload only (python bench.py)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="c3b",
                    help="synthetic layer config (see paper_2603_28845_amd/synth.py); 'c5' = the six-layer mixed 2/3/4-bit "
                         "allocation of the 70B-class shapes")
    ap.add_argument("--tokens-per-call", type=int, default=0, help="0 = all calibration tokens in one accumulate call")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--phase", default="all", choices=["all", "gram", "factor", "sweep"],
                    help="profiling aid: run only one call in the timed loop (the others run once to prepare its inputs)")
    ap.add_argument("--jointq", type=int, default=1,
                    help="passes of the JointQ refinement (Sec. 4.3.2) timed on the result of the last step and "
                         "reported under 'jointq' (0 = skip); the headline value is unchanged")
    ap.add_argument("--qep", action="store_true",
                    help="also time the layer with error propagation (Sec. 4.3.1): Gram of the perturbed activations, "
                         "cross-Gram, factor, corrected target, sweep of the corrected target; reported under 'qep', "
                         "the headline value is unchanged")
    ap.add_argument("--factor-form", default="inverse", choices=["inverse", "block"],
                    help="inverse: the factor call returns U with U^T U = (H + lambda I)^-1 (Sec. 4.3.1) and the sweep "
                         "propagates through it; block: one Cholesky only, the sweep runs on the block form (same codes "
                         "up to ties; groups up to 128 columns)")
    ap.add_argument("--group-size", type=int, default=0,
                    help="override the workload's group size (d_in = one group per row, the per-channel setting of the "
                         "paper's Table 3); 0 = as configured")
    ap.add_argument("--grid", default="minmax", choices=["minmax", "symmetric", "minmax_mse", "symmetric_mse"],
                    help="grid of the sweep: min-max (Eq. (2), the configured workloads) or symmetric (Eq. (3)); "
                         "_mse adds the scale search of Sec. 4.3")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (accumulate, factor, quantize) in a HIP graph after the warm-up and time "
                         "replays of it; per-phase times are then not available (reported as the eager warm-up's)")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="context only: also time the vendor library's dense bf16 GEMM X^T X (torch.matmul, full d_in x "
                         "d_in output, no symmetry, no accumulate into fp32 H) on the same activations; reported under "
                         "'vendor_gemm_context', the headline value is unchanged")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="profiling aid: also run one plain 4 GiB device-to-device copy kernel (known HBM traffic: "
                         "4 GiB read + 4 GiB written) so that FETCH_SIZE / WRITE_SIZE can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2603_28845_amd as og
    from paper_2603_28845_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    og.load_library()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.workload == "c5":
        print(json.dumps(bench_c5(args, og, synth)))
        return
    cfg = synth.CONFIGS[args.workload]
    if args.group_size > 0:
        cfg = synth.scaled(cfg, group_size=args.group_size)
    d_out, d_in, T = cfg.d_out, cfg.d_in, cfg.n_tokens

    W = synth.make_weight(cfg, dev)
    X = synth.make_activations(cfg, dev)
    H = torch.zeros((d_in, d_in), dtype=torch.float32, device=dev)
    U = torch.empty((d_in, d_in), dtype=torch.float32, device=dev)
    info = torch.zeros(1, dtype=torch.int32, device=dev)
    perm = torch.empty(d_in, dtype=torch.int32, device=dev) if cfg.act_order else None
    ws_a_bytes = og.onecomp_accumulate_workspace_bytes(cfg.dtype, d_in)
    ws_a = torch.empty(ws_a_bytes, dtype=torch.uint8, device=dev) if ws_a_bytes > 0 else None
    ws_f = torch.empty(og.onecomp_factor_workspace_bytes(d_in), dtype=torch.uint8, device=dev)
    ws_q = torch.empty(og.onecomp_quantize_workspace_bytes(d_out, d_in, 128), dtype=torch.uint8, device=dev)
    n_g = d_in // cfg.group_size
    out = {
        "Q_codes": torch.empty((d_out, d_in), dtype=torch.uint8, device=dev),
        "scales": torch.empty((d_out, n_g), dtype=torch.float32, device=dev),
        "zeros": torch.empty((d_out, n_g), dtype=torch.float32, device=dev),
        "W_hat": torch.empty((d_out, d_in), dtype=torch.float32, device=dev),
        "loss": torch.zeros(1, dtype=torch.float32, device=dev),
    }
    tpc = args.tokens_per_call if args.tokens_per_call > 0 else T
    n_calls = (T + tpc - 1) // tpc

    def ev():
        return torch.cuda.Event(enable_timing=True)

    phase = args.phase

    def step(record=None, only=None, form=None):
        form = form or args.factor_form

        class _NoEvent:
            def record(self):
                pass
        # events only when the caller wants the phase times (none are recorded into a graph capture)
        e = [ev() for _ in range(4)] if record is not None else [_NoEvent()] * 4
        if only in (None, "gram"):
            H.zero_()
        e[0].record()
        if only in (None, "gram"):
            for t0 in range(0, T, tpc):
                og.onecomp_hessian_accumulate(X[t0:t0 + tpc], H, workspace=ws_a)
        e[1].record()
        if only in (None, "factor"):
            og.onecomp_hessian_factor(H, cfg.damp, cfg.act_order, U=U, perm_out=perm, info=info, workspace=ws_f,
                                      form=form)
        e[2].record()
        if only in (None, "sweep"):
            og.onecomp_quantize_layer(W, U, cfg.bits, cfg.group_size, perm=perm, workspace=ws_q, out=out,
                                      form=form, grid=args.grid)
        e[3].record()
        if record is not None:
            record.append(e)

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    if phase != "all":
        step()          # prepares H and U for a single-phase loop
        torch.cuda.synchronize()

    only = None if phase == "all" else phase
    for _ in range(args.warmup):
        step(only=only)
    torch.cuda.synchronize()
    rec = []
    if args.graph:
        # the library neither allocates nor synchronizes, so a step can be captured as it is; the eager pass
        # before it supplies the per-phase times
        step(rec, only=only)
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step(only=only)                      # warm-up on the capture stream
            side.synchronize()
            with torch.cuda.graph(g, stream=side):
                step(only=only)
        torch.cuda.current_stream().wait_stream(side)
        g.replay()
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
    else:
        t_start = time.perf_counter()
        for _ in range(args.steps):
            step(rec, only=only)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t_start
    assert int(info.item()) == 0, "Hessian not positive definite"
    loss_main = float(out["loss"].item())

    # the same step with the factor in block form (one Cholesky, no triangular inverse), reported next to the headline
    alt = None
    if phase == "all" and args.factor_form == "inverse" and (cfg.group_size <= 128 or cfg.group_size == d_in) \
            and d_in % 128 == 0:
        for _ in range(args.warmup):
            step(form="block")
        torch.cuda.synchronize()
        rec_b = []
        t_b = time.perf_counter()
        for _ in range(args.steps):
            step(rec_b, form="block")
        torch.cuda.synchronize()
        wall_b = time.perf_counter() - t_b
        ms_b = wall_b * 1e3 / args.steps
        alt = {
            "what": "same step through onecomp_hessian_factor_form / onecomp_quantize_layer_form with "
                    "ONECOMP_FACTOR_BLOCK: one Cholesky instead of Cholesky + triangular inverse; same codes up to ties",
            "ms_per_step": ms_b, "value": d_out * d_in / (ms_b * 1e-3),
            "phases_ms": {"hessian_accumulate": _median([e[0].elapsed_time(e[1]) for e in rec_b]),
                          "hessian_factor": _median([e[1].elapsed_time(e[2]) for e in rec_b]),
                          "quantize_layer": _median([e[2].elapsed_time(e[3]) for e in rec_b])},
            "loss": float(out["loss"].item()),
        }

    tiny = 1e-6   # phases skipped by --phase read as ~0; keep the ratios finite
    acc_ms = max(tiny, _median([e[0].elapsed_time(e[1]) for e in rec]))   # per-phase times: medians over the steps
    fac_ms = max(tiny, _median([e[1].elapsed_time(e[2]) for e in rec]))
    swp_ms = max(tiny, _median([e[2].elapsed_time(e[3]) for e in rec]))
    ms_per_step = wall * 1e3 / args.steps
    weights = d_out * d_in

    # Gram kernel.  Algorithmic flops = symmetric half, T d (d + 1).  An accumulate call on a wide layer launches the
    # kernel once per round of tiles (one tile per CU) and once more for the tiles cut along the tokens; the library
    # reports the tile shape it chose and the number of launches.
    gram_ms = acc_ms / n_calls
    gram_plan = og.onecomp_accumulate_describe(cfg.dtype, tpc, d_in, ws_a.numel() if ws_a is not None else 0)
    gram_launches = gram_plan["launches"]
    algo_flops = float(tpc) * d_in * (d_in + 1)
    gram_tflops = algo_flops / (gram_ms * 1e-3) / 1e12
    # Counter-backed traffic of the Gram call.  Counters cannot be read from inside this process: the figure is the one
    # of profiles/c3b_hbm_traffic_pmc.md (rocprofv3 --pmc runs of this file's --phase gram loop), valid for the default
    # workload in one accumulate call with the workspace; null for anything else.
    gram_traffic = GRAM_TRAFFIC_C3B if (cfg.name == "c3b" and n_calls == 1 and gram_plan["tile_rows"] == 384) else None
    roofline = {
        "kernel": gram_kernel_name(d_in, cfg.dtype == torch.bfloat16, gram_plan, tpc),
        "tile": [gram_plan["tile_rows"], gram_plan["tile_cols"]],
        "bound": "mfma", "achieved": gram_tflops, "peak": PEAK_BF16_TFLOPS if cfg.dtype == torch.bfloat16 else 157.3,
        "unit": "TFLOP/s", "frac": gram_tflops / (PEAK_BF16_TFLOPS if cfg.dtype == torch.bfloat16 else 157.3),
        "traffic": gram_traffic,
        "traffic_note": "L2 <-> fabric bytes per accumulate call (all its launches) from rocprofv3 FETCH_SIZE / "
                        "WRITE_SIZE, scaled by a 4 GiB copy (profiles/c3b_hbm_traffic_pmc.md); measured for the default "
                        "workload only, else null",
        "algorithmic_bytes": 2.0 * tpc * d_in + 8.0 * d_in * d_in,
        "note": "algorithmic flops = T*d_in*(d_in+1) (upper triangle incl. diagonal, 2 flops per MAC); "
                "dense-equivalent rate is 2x this",
        "call_ms": gram_ms, "launches_per_call": gram_launches, "avg_launch_ms": gram_ms / gram_launches,
        "launch_note": "achieved = flops of one accumulate call / its time; the call is launches_per_call launches of "
                       "the kernel back to back, so rocprofv3's average duration of the kernel is call_ms / launches_per_call",
    }
    w_bytes = 2 if cfg.dtype == torch.bfloat16 else 4
    sweep_bytes = sweep_model_bytes(d_out, d_in, cfg.group_size, w_bytes)
    b128_bytes = sweep_model_bytes_b128(d_out, d_in, 128, cfg.group_size, w_bytes)
    sweep_gbs = sweep_bytes / (swp_ms * 1e-3) / 1e9
    roofline_sweep = {
        "kernel": "onecomp_quantize_layer (panel_far_kernel + trailing_kernel launches)", "bound": "hbm",
        "achieved": sweep_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": sweep_gbs / PEAK_HBM_GBS,
        "traffic": SWEEP_TRAFFIC_C3B if (cfg.name == "c3b" and args.grid == "minmax" and args.group_size == 0
                                          and args.factor_form == "inverse") else None,
        "traffic_note": "FETCH_SIZE + WRITE_SIZE of all the call's launches, profiles/c3b_hbm_traffic_pmc.md; null for "
                        "any other configuration",
        "model_bytes": sweep_bytes,
        "note": "modelled HBM bytes of the two-level schedule actually run (512-column super-blocks) / whole-call "
                "time; the trailing updates are split-fp16 MFMA GEMMs fed from L2, so the call is not HBM bound",
        "b128_model_bytes": b128_bytes,
        "b128_equivalent_gbs": b128_bytes / (swp_ms * 1e-3) / 1e9,
        "b128_equivalent_frac": b128_bytes / (swp_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "b128_note": "bytes the plain right-looking block-128 schedule would move, divided by the measured time: "
                     "the figure the 50 %-of-HBM target for this layer was stated in",
    }

    res = {
        "metric": "weights_quantized_per_sec", "value": weights / (ms_per_step * 1e-3), "unit": "weights/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 inputs, f32 accumulate and sweep, f64 factor" if cfg.dtype == torch.bfloat16 else "f32 (f64 factor)",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: W {d_out}x{d_in} {str(cfg.dtype).split('.')[-1]}, {T} tokens, "
                               f"{cfg.bits}-bit, group {cfg.group_size}, {args.grid} grid, damp {cfg.damp}, act_order {cfg.act_order}, "
                               f"block 128, {n_calls} accumulate call(s) with a {ws_a_bytes >> 20} MiB workspace, "
                               f"factor form {args.factor_form}"
                               + (", HIP graph replay" if args.graph else "")
                               + ("" if phase == "all" else f" [PROFILING RUN: only phase '{phase}' timed, value is not the metric]")},
        "phases_ms": {"hessian_accumulate": acc_ms, "hessian_factor": fac_ms, "quantize_layer": swp_ms},
        "layer_quantize_ms": fac_ms + swp_ms,
        "weights_per_sec_factor_plus_sweep": weights / ((fac_ms + swp_ms) * 1e-3),
        "weights_per_sec_sweep_only": weights / (swp_ms * 1e-3),
        "loss": loss_main,
        "roofline": roofline, "roofline_sweep": roofline_sweep,
    }
    if alt is not None:
        res["block_form"] = alt
    if args.vendor_gemm and cfg.dtype == torch.bfloat16:
        e = [ev() for _ in range(2)]
        torch.matmul(X.t(), X)
        e[0].record()
        for _ in range(3):
            G = torch.matmul(X.t(), X)
        e[1].record()
        torch.cuda.synchronize()
        v_ms = e[0].elapsed_time(e[1]) / 3
        del G
        res["vendor_gemm_context"] = {
            "op": "torch.matmul(X.t(), X), bf16 in and out, all d_in x d_in entries", "ms": v_ms,
            "dense_tflops": 2.0 * T * d_in * d_in / (v_ms * 1e-3) / 1e12,
            "frac_of_bf16_peak": 2.0 * T * d_in * d_in / (v_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "gram_kernel_ms_for_the_same_tokens": acc_ms,
        }
    if phase == "all":
        ach = achievable_mfma(og, torch)
        res["achievable_mfma"] = ach
        if cfg.dtype == torch.bfloat16:
            res["roofline"]["frac_of_achievable"] = gram_tflops / max(ach["bf16_tflops_1_wave_per_simd"],
                                                                      ach["bf16_tflops_2_wave_per_simd"])
        res["factor_fp64"] = {
            "tflops": 2.0 * d_in ** 3 / 3.0 / (fac_ms * 1e-3) / 1e12 * (1.0 if args.factor_form == "inverse" else 0.5),
            "frac_of_peak": 2.0 * d_in ** 3 / 3.0 / (fac_ms * 1e-3) / 1e12 * (1.0 if args.factor_form == "inverse" else 0.5) / 78.6,
            "frac_of_achievable": 2.0 * d_in ** 3 / 3.0 / (fac_ms * 1e-3) / 1e12 * (1.0 if args.factor_form == "inverse" else 0.5)
                                  / max(ach["f64_tflops_1_wave_per_simd"], ach["f64_tflops_2_wave_per_simd"]),
            "note": "2 d^3 / 3 flops (Cholesky + triangular inverse; d^3 / 3 in block form) over the factor call's time",
        }
    if args.jointq > 0 and phase == "all" and (cfg.group_size <= 128 or cfg.group_size % 128 == 0):
        res["jointq"] = bench_jointq(args, cfg, og, W, H, out, perm if cfg.act_order else None)
    if args.qep:
        res["qep"] = bench_qep(args, cfg, og, synth, W, X, H, U, info, perm, ws_f, ws_q, out, ws_a)
    if not args.no_cpu_baseline:
        del X
        torch.cuda.empty_cache()
        res["cpu_baseline"] = cpu_baseline(cfg, synth)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
