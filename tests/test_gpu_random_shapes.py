"""Seeded random-shape parity runs through the C ABI: every entry point on shapes, options and data layouts drawn at
random inside its documented limits, each case held to the same bars as the hand-picked cases of the other GPU test
files (whose helpers do the comparing).  The hand-picked cases cover the corners one thinks of; these cover
combinations nobody picked.  A case prints its parameters before it runs."""
import numpy as np
import pytest
import torch

import test_gpu_jointq as TJ
import test_gpu_parity as TP
import test_gpu_qep as TQ
from oracle import onecomp_oracle as oc
from paper_2603_28845_amd import synth
from parity_util import rel_fro, to_f64
import paper_2603_28845_amd as og

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _announce(msg):
    print(f"[case] {msg}", flush=True)


def _group_sizes(nb):
    """Group sizes the sweep takes at d_in = 128 nb: divisors of a block, or whole blocks dividing the row."""
    return [16, 32, 64, 128] + [128 * m for m in range(2, nb + 1) if nb % m == 0]


@pytest.mark.parametrize("seed", [3, 4])
def test_random_sweeps(seed):
    """Quantize call: width, group size, bits, rows, dtype, column order, grid and factor form at random; half of the
    cases with rows of very different size (three decades), an all-zero row, a one-signed row, a 40-fold outlier
    entry and up to three dead input channels."""
    rng = np.random.default_rng(seed)
    for case in range(40):
        nb = int(rng.choice([1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 12, 13, 16]))
        d_in = 128 * nb
        G = int(rng.choice(_group_sizes(nb)))
        bits = int(rng.choice([2, 3, 4, 8]))
        d_out = int(rng.choice([1, 2, 3, 17, 31, 63, 64, 65, 100, 127, 128, 129, 200]))
        dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
        act = bool(rng.random() < 0.5)
        grid = str(rng.choice(["minmax", "symmetric", "minmax_mse", "symmetric_mse"], p=[0.4, 0.2, 0.25, 0.15]))
        form = "block" if ((G <= 128 or G == d_in) and rng.random() < 0.4) else "inverse"
        shaped = bool(rng.random() < 0.5)
        dead = int(rng.choice([0, 0, 1, 3]))
        _announce(f"seed {seed} case {case}: b{bits} g{G} {d_out}x{d_in} {dtype} act={act} grid={grid} form={form} "
                  f"shaped={shaped} dead={dead}")
        cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=2 * d_in + 13, seed=1000 * seed + case,
                           dtype=dtype, n_outlier=max(1, d_in // 100))
        W = synth.make_weight(cfg, DEV).float()
        X = synth.make_activations(cfg, "cpu")
        if shaped:
            W = W * torch.from_numpy(10.0 ** rng.uniform(-3.0, 0.0, size=d_out)).to(DEV).float()[:, None]
            W[0] = 0.0
            if d_out > 2:
                W[2] = W[2].abs() + 1e-4
                W[1, int(rng.integers(d_in))] *= 40.0
            if dead:
                X = X.clone()
                X[:, rng.choice(d_in, size=dead, replace=False)] = 0
        W = W.to(dtype)
        f = oc.hessian_factor(oc.hessian_accumulate(to_f64(X)), 0.01, act_order=act)
        U32 = torch.from_numpy(f["U"].astype(np.float32)).to(DEV)
        perm = torch.from_numpy(f["perm"].astype(np.int32)).to(DEV) if act else None
        F32 = torch.from_numpy(TP._oracle_block_factor(f).astype(np.float32)).to(DEV) if form == "block" else None
        TP._check_sweep(W, U32, bits, G, perm=perm, grid=grid, F32=F32)


@pytest.mark.parametrize("seed", [1])
def test_random_accumulate_and_factor(seed, monkeypatch):
    """Accumulate: width (any multiple of 16), tokens (0 .. 6000), dtype, calls per matrix, workspace size and tile
    shape at random, the whole matrix against the oracle.  Factor: width, column order and form at random."""
    rng = np.random.default_rng(seed)
    for case in range(60):
        if rng.random() < 0.6:
            d_in = 16 * int(rng.integers(1, 200))
            if rng.random() < 0.3:
                d_in = int(rng.choice([1024, 1040, 1536, 2048, 2304, 3072, 3088, 4096]))
            n_tok = int(rng.choice([0, 1, 15, 16, 17, 100, 333, 1000, 2049, 4099, 6000]))
            dtype = torch.bfloat16 if rng.random() < 0.75 else torch.float32
            chunks = int(rng.integers(1, 4))
            wsf = float(rng.choice([-1.0, 1.0, 0.3, 0.01]))
            shape = str(rng.choice(["", "wide", "big", "mid"]))
            _announce(f"seed {seed} case {case}: accumulate d_in={d_in} n_tok={n_tok} {dtype} calls={chunks} "
                      f"workspace fraction {wsf} tile shape {shape!r}")
            if shape:
                monkeypatch.setenv("ONECOMP_GRAM_SHAPE", shape)
            else:
                monkeypatch.delenv("ONECOMP_GRAM_SHAPE", raising=False)
            cfg = synth.scaled(synth.CONFIGS["c2"], d_out=16, d_in=d_in, n_tokens=max(n_tok, 1), dtype=dtype,
                               seed=100 * seed + case)
            X = synth.make_activations(cfg, DEV)[:n_tok]
            ws = None
            need = og.onecomp_accumulate_workspace_bytes(torch.bfloat16, d_in)
            if wsf > 0 and dtype == torch.bfloat16 and need > 0:
                ws = torch.empty(max(256, int(need * wsf) // 256 * 256), dtype=torch.uint8, device=DEV)
                ws.fill_(0xFF)
            Hn = TP._gpu_gram(X, chunks=chunks, ws=ws).cpu().numpy()
            assert np.array_equal(Hn, Hn.T)
            if n_tok:
                assert rel_fro(Hn.astype(np.float64), oc.hessian_accumulate(to_f64(X))) <= 1e-4
            else:
                assert not Hn.any()
        else:
            d_in = 128 * int(rng.integers(1, 20)) if rng.random() < 0.4 else 16 * int(rng.integers(1, 160))
            act = bool(rng.random() < 0.5)
            form = "block" if (d_in % 128 == 0 and rng.random() < 0.4) else "inverse"
            _announce(f"seed {seed} case {case}: factor d_in={d_in} act_order={act} form={form}")
            H32 = TP._oracle_H32(d_in, 3 * d_in + 7, seed=100 * seed + case)
            f = oc.hessian_factor(H32.astype(np.float64), 0.01, act_order=act)
            F, perm, info = og.onecomp_hessian_factor(torch.from_numpy(H32).to(DEV), 0.01, act_order=act, form=form)
            torch.cuda.synchronize()
            assert int(info.item()) == 0 and f["info"] == 0
            if act:
                np.testing.assert_array_equal(perm.cpu().numpy(), f["perm"])
            Fn = F.cpu().numpy().astype(np.float64)
            assert np.all(np.tril(Fn, -1) == 0.0) and np.all(np.diag(Fn) > 0.0)
            assert rel_fro(Fn, f["U"] if form == "inverse" else TP._oracle_block_factor(f)) <= 1e-6


@pytest.mark.parametrize("seed", [2])
def test_random_next_rows(seed, monkeypatch):
    """Cross-Gram, corrected target, sensitivity proxy and JointQ refinement on random shapes and options."""
    rng = np.random.default_rng(seed)
    for case in range(60):
        kind = str(rng.choice(["cross", "qep", "sens", "jointq"]))
        monkeypatch.delenv("ONECOMP_GRAM_SHAPE", raising=False)
        if kind == "cross":
            d_in = 16 * int(rng.integers(1, 200))
            n_tok = int(rng.choice([1, 16, 17, 100, 333, 1000, 2049]))
            chunks = min(int(rng.integers(1, 4)), n_tok)
            shape = str(rng.choice(["", "wide", "big", "mid"]))
            _announce(f"seed {seed} case {case}: cross-Gram d_in={d_in} n_tok={n_tok} calls={chunks} tile shape {shape!r}")
            if shape:
                monkeypatch.setenv("ONECOMP_GRAM_SHAPE", shape)
            _, X, Xh = TQ._pair(d_in, n_tok, seed=100 * seed + case)
            G = TQ._gpu_cross(Xh, X, chunks=chunks)
            assert rel_fro(G.cpu().numpy().astype(np.float64), oc.crossgram_accumulate(to_f64(Xh), to_f64(X))) <= 1e-4
        elif kind == "qep":
            d_in = 16 * int(rng.integers(2, 120))
            d_out = int(rng.choice([1, 7, 64, 100, 129, 300]))
            dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
            act = bool(rng.random() < 0.5)
            alpha = float(rng.choice([1.0, 0.5, 0.25]))
            _announce(f"seed {seed} case {case}: corrected target {d_out}x{d_in} {dtype} act={act} alpha={alpha}")
            cfg, X, Xh = TQ._pair(d_in, 3 * d_in + 5, seed=100 * seed + case)
            W = synth.make_weight(synth.scaled(cfg, d_out=d_out, dtype=dtype), DEV)
            H = torch.zeros((d_in, d_in), dtype=torch.float32, device=DEV)
            og.onecomp_hessian_accumulate(Xh, H)
            G = TQ._gpu_cross(Xh, X)
            U, perm, info = og.onecomp_hessian_factor(H, 0.01, act)
            Ws = og.onecomp_qep_target(W, G, H, U, alpha, perm=perm)
            torch.cuda.synchronize()
            assert int(info.item()) == 0
            Wd = to_f64(W)
            ref = oc.qep_target(Wd, G.cpu().numpy().astype(np.float64), H.cpu().numpy().astype(np.float64), 0.01, alpha)
            got = Ws.cpu().numpy().astype(np.float64)
            assert rel_fro(got, ref) <= 2e-6 and rel_fro(got - Wd, ref - Wd) <= 1e-4
        elif kind == "sens":
            d_in = 128 * int(rng.integers(1, 30))
            G = int(rng.choice([16, 32, 64, 128, d_in]))
            bits = int(rng.choice([2, 3, 4, 8]))
            d_out = int(rng.choice([1, 7, 33, 64, 300, 1000]))
            dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
            grid = str(rng.choice(["minmax", "symmetric"]))
            _announce(f"seed {seed} case {case}: sensitivity b{bits} g{G} {d_out}x{d_in} {dtype} {grid}")
            cfg = synth.scaled(synth.CONFIGS["c2"], d_out=d_out, d_in=d_in, n_tokens=16, seed=100 * seed + case, dtype=dtype)
            W = synth.make_weight(cfg, DEV)
            gen = torch.Generator(device=DEV).manual_seed(case)
            a = (0.5 + 3.0 * torch.rand(d_in, generator=gen, device=DEV)).to(torch.float32)
            b = (0.5 + torch.rand(d_out, generator=gen, device=DEV)).to(torch.float32)
            for bd in (None, b):
                e = og.onecomp_rtn_sensitivity(W, a, bits, G, b_diag=bd, grid=grid)
                torch.cuda.synchronize()
                ref = oc.rtn_sensitivity(to_f64(W), to_f64(a), None if bd is None else to_f64(bd), bits, G,
                                         grid="sym" if grid == "symmetric" else "asym")
                assert abs(float(e.item()) - ref) <= 1e-3 * ref
        else:
            nb = int(rng.choice([1, 2, 3, 4, 5, 6, 8]))
            d_in = 128 * nb
            G = int(rng.choice(_group_sizes(nb)))
            bits = int(rng.choice([2, 3, 4]))
            d_out = int(rng.choice([1, 3, 17, 37, 64]))
            dtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
            grid = str(rng.choice(["asym", "sym"]))
            start = str(rng.choice(["rtn", "gptq"]))
            n_pass = int(rng.choice([1, 1, 2]))
            scans = int(rng.choice([1, 2, 4]))
            lam = float(rng.choice([0.0, 0.0, 25.0]))
            act = bool(start == "gptq" and rng.random() < 0.4)
            _announce(f"seed {seed} case {case}: jointq b{bits} g{G} {d_out}x{d_in} {dtype} {grid} start={start} "
                      f"passes={n_pass} scans={scans} lam={lam} act={act}")
            r = TJ._start(d_out, d_in, bits, G, seed=100 * seed + case, dtype=dtype, grid=grid, start=start, act=act)
            TJ._run(*r[:6], bits, G, grid=grid, lam=lam, n_pass=n_pass, max_scans=scans, perm=r[6] if act else None)
