"""ctypes binding of libonecomp.so: argument marshalling only.

Each function has the name of the C entry point it calls (include/onecomp.h) and
takes torch tensors that live on the GPU; torch supplies device memory and the
current HIP stream, every step of the computation runs in the library's kernels.
There is no CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch  # imported before the library so that both share one HIP runtime

_PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG_DIR, "libonecomp.so")

ONECOMP_OK = 0
ONECOMP_F32 = 0
ONECOMP_BF16 = 1
ONECOMP_GRID_MINMAX = 0
ONECOMP_GRID_SYMMETRIC = 1
ONECOMP_GRID_MINMAX_MSE = 2
ONECOMP_GRID_SYMMETRIC_MSE = 3
_GRIDS = {"minmax": ONECOMP_GRID_MINMAX, "symmetric": ONECOMP_GRID_SYMMETRIC, "minmax_mse": ONECOMP_GRID_MINMAX_MSE,
          "symmetric_mse": ONECOMP_GRID_SYMMETRIC_MSE}
ONECOMP_FACTOR_INVERSE = 0
ONECOMP_FACTOR_BLOCK = 1

EXPORTED_SYMBOLS = (
    "onecomp_hessian_accumulate",
    "onecomp_hessian_factor",
    "onecomp_quantize_layer",
    "onecomp_quantize_layer_grid",
    "onecomp_hessian_factor_form",
    "onecomp_hessian_accumulate_ws",
    "onecomp_accumulate_workspace_bytes",
    "onecomp_accumulate_describe",
    "onecomp_mfma_rate_probe",
    "onecomp_quantize_layer_form",
    "onecomp_factor_workspace_bytes",
    "onecomp_quantize_workspace_bytes",
    "onecomp_crossgram_accumulate",
    "onecomp_qep_target",
    "onecomp_qep_workspace_bytes",
    "onecomp_rtn_sensitivity",
    "onecomp_sensitivity_workspace_bytes",
    "onecomp_rtn_sensitivity_static",
    "onecomp_jointq_refine",
    "onecomp_jointq_workspace_bytes",
    "onecomp_status_string",
    "onecomp_version",
)

_lib = None


class OnecompError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} (status {code})")


def load_library() -> ctypes.CDLL:
    """Load libonecomp.so (once) and declare its prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_28845_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, i32, f32, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
    lib.onecomp_hessian_accumulate.argtypes = [vp, i32, i64, i64, i64, vp, vp]
    lib.onecomp_hessian_accumulate.restype = i32
    lib.onecomp_hessian_factor.argtypes = [vp, i64, f32, i32, vp, vp, vp, vp, sz, vp]
    lib.onecomp_hessian_factor.restype = i32
    lib.onecomp_hessian_accumulate_ws.argtypes = [vp, i32, i64, i64, i64, vp, vp, sz, vp]
    lib.onecomp_hessian_accumulate_ws.restype = i32
    lib.onecomp_accumulate_workspace_bytes.argtypes = [i32, i64]
    lib.onecomp_accumulate_workspace_bytes.restype = sz
    lib.onecomp_accumulate_describe.argtypes = [i32, i64, i64, i64, sz, vp]
    lib.onecomp_accumulate_describe.restype = i32
    lib.onecomp_mfma_rate_probe.argtypes = [i32, i32, i32, i64, vp, vp, vp]
    lib.onecomp_mfma_rate_probe.restype = i32
    lib.onecomp_hessian_factor_form.argtypes = [vp, i64, f32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.onecomp_hessian_factor_form.restype = i32
    lib.onecomp_quantize_layer_form.argtypes = [vp, i32, i64, i64, vp, i32, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp,
                                                vp, sz, vp]
    lib.onecomp_quantize_layer_form.restype = i32
    lib.onecomp_quantize_layer.argtypes = [vp, i32, i64, i64, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.onecomp_quantize_layer.restype = i32
    lib.onecomp_quantize_layer_grid.argtypes = [vp, i32, i64, i64, vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz,
                                                vp]
    lib.onecomp_quantize_layer_grid.restype = i32
    lib.onecomp_factor_workspace_bytes.argtypes = [i64]
    lib.onecomp_factor_workspace_bytes.restype = sz
    lib.onecomp_quantize_workspace_bytes.argtypes = [i64, i64, i32]
    lib.onecomp_quantize_workspace_bytes.restype = sz
    lib.onecomp_crossgram_accumulate.argtypes = [vp, vp, i32, i64, i64, i64, i64, vp, vp]
    lib.onecomp_crossgram_accumulate.restype = i32
    lib.onecomp_qep_target.argtypes = [vp, i32, i64, i64, vp, vp, vp, vp, f32, vp, vp, sz, vp]
    lib.onecomp_qep_target.restype = i32
    lib.onecomp_qep_workspace_bytes.argtypes = [i64, i64]
    lib.onecomp_qep_workspace_bytes.restype = sz
    lib.onecomp_rtn_sensitivity.argtypes = [vp, i32, i64, i64, vp, vp, i32, i32, i32, vp, vp, sz, vp]
    lib.onecomp_rtn_sensitivity.restype = i32
    lib.onecomp_rtn_sensitivity_static.argtypes = [vp, i32, i64, i64, vp, vp, i32, i32, i32, vp, vp]
    lib.onecomp_rtn_sensitivity_static.restype = i32
    lib.onecomp_sensitivity_workspace_bytes.argtypes = []
    lib.onecomp_sensitivity_workspace_bytes.restype = sz
    lib.onecomp_jointq_refine.argtypes = [vp, i32, i64, i64, vp, vp, f32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp,
                                          vp, sz, vp]
    lib.onecomp_jointq_refine.restype = i32
    lib.onecomp_jointq_workspace_bytes.argtypes = [i64, i64, i32]
    lib.onecomp_jointq_workspace_bytes.restype = sz
    lib.onecomp_status_string.argtypes = [i32]
    lib.onecomp_status_string.restype = ctypes.c_char_p
    lib.onecomp_version.argtypes = []
    lib.onecomp_version.restype = i32
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().onecomp_status_string(int(code)).decode()


def onecomp_version() -> int:
    return int(load_library().onecomp_version())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return ONECOMP_F32
    if t.dtype == torch.bfloat16:
        return ONECOMP_BF16
    raise TypeError(f"unsupported dtype {t.dtype}: float32 or bfloat16 expected")


def _dev(t: torch.Tensor, name: str, dtype=None, contiguous=True):
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if contiguous and not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


def _stream() -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def onecomp_factor_workspace_bytes(d_in: int) -> int:
    return int(load_library().onecomp_factor_workspace_bytes(int(d_in)))


def onecomp_quantize_workspace_bytes(d_out: int, d_in: int, block_size: int = 128) -> int:
    return int(load_library().onecomp_quantize_workspace_bytes(int(d_out), int(d_in), int(block_size)))


def onecomp_accumulate_workspace_bytes(dtype: torch.dtype, d_in: int) -> int:
    code = ONECOMP_BF16 if dtype == torch.bfloat16 else ONECOMP_F32
    return int(load_library().onecomp_accumulate_workspace_bytes(code, int(d_in)))


def onecomp_accumulate_describe(dtype: torch.dtype, n_tokens: int, d_in: int, workspace_bytes: int = 0,
                                ldx: Optional[int] = None) -> dict:
    """How an accumulate call of this size would run: tile shape of its main kernel and launches of it per call."""
    code = ONECOMP_BF16 if dtype == torch.bfloat16 else ONECOMP_F32
    out = (ctypes.c_int32 * 3)()
    rc = load_library().onecomp_accumulate_describe(code, int(n_tokens), int(d_in), int(d_in if ldx is None else ldx),
                                                    int(workspace_bytes), ctypes.cast(out, ctypes.c_void_p))
    if rc != 0:
        raise OnecompError(rc, "onecomp_accumulate_describe")
    return {"tile_rows": int(out[0]), "tile_cols": int(out[1]), "launches": int(out[2])}


def onecomp_mfma_rate_probe(kind: str, waves_per_simd: int, iters: int, sink: torch.Tensor,
                            random_operands: bool = True) -> float:
    """Enqueues the register-only MFMA loop (kind "bf16" or "f64") on the current stream; returns its flop count."""
    flops = ctypes.c_double(0.0)
    rc = load_library().onecomp_mfma_rate_probe({"bf16": 0, "f64": 1}[kind], int(waves_per_simd),
                                                int(bool(random_operands)), int(iters),
                                                _ptr(sink), ctypes.cast(ctypes.byref(flops), ctypes.c_void_p),
                                                _stream())
    if rc != 0:
        raise OnecompError(rc, "onecomp_mfma_rate_probe")
    return float(flops.value)


def onecomp_hessian_accumulate(X: torch.Tensor, H: torch.Tensor, workspace: Optional[torch.Tensor] = None) -> None:
    """H += 2 X^T X.  X: [n_tokens, d_in] fp32/bf16 (rows may be strided), H: [d_in, d_in] fp32.
    workspace (uint8 device tensor, see onecomp_accumulate_workspace_bytes) selects onecomp_hessian_accumulate_ws."""
    lib = load_library()
    if X.dim() != 2 or H.dim() != 2 or H.shape[0] != H.shape[1] or H.shape[0] != X.shape[1]:
        raise ValueError("shapes: X [n_tokens, d_in], H [d_in, d_in]")
    if X.shape[0] > 0 and X.stride(1) != 1:
        raise ValueError("X rows must be dense")
    _dev(X, "X", contiguous=False)
    ldx = X.stride(0) if X.shape[0] > 1 else X.shape[1]
    if workspace is None:
        rc = lib.onecomp_hessian_accumulate(_ptr(X), _dtype_code(X), X.shape[0], X.shape[1], ldx,
                                            _dev(H, "H", torch.float32), _stream())
    else:
        rc = lib.onecomp_hessian_accumulate_ws(_ptr(X), _dtype_code(X), X.shape[0], X.shape[1], ldx,
                                               _dev(H, "H", torch.float32), _dev(workspace, "workspace", torch.uint8),
                                               workspace.numel(), _stream())
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_hessian_accumulate")


def onecomp_hessian_factor(H: torch.Tensor, damp: float, act_order: bool = False,
                           U: Optional[torch.Tensor] = None, perm_out: Optional[torch.Tensor] = None,
                           info: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                           form: str = "inverse") -> Tuple[torch.Tensor, Optional[torch.Tensor], torch.Tensor]:
    """Returns (U, perm, info) as device tensors; perm is None when act_order is False and no perm_out was given.
    form = "inverse" calls onecomp_hessian_factor, "block" onecomp_hessian_factor_form with ONECOMP_FACTOR_BLOCK
    (the matrix returned is then meant for onecomp_quantize_layer(..., form="block") only)."""
    lib = load_library()
    d = H.shape[0]
    if U is None:
        U = torch.empty((d, d), dtype=torch.float32, device=H.device)
    if info is None:
        info = torch.zeros(1, dtype=torch.int32, device=H.device)
    if act_order and perm_out is None:
        perm_out = torch.empty(d, dtype=torch.int32, device=H.device)
    need = onecomp_factor_workspace_bytes(d)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=H.device)
    tail = (_ptr(perm_out), _dev(U, "U", torch.float32), _dev(info, "info", torch.int32),
            _dev(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    if form == "inverse":
        rc = lib.onecomp_hessian_factor(_dev(H, "H", torch.float32), d, float(damp), int(bool(act_order)), *tail)
    elif form == "block":
        rc = lib.onecomp_hessian_factor_form(_dev(H, "H", torch.float32), d, float(damp), int(bool(act_order)),
                                             ONECOMP_FACTOR_BLOCK, *tail)
    else:
        raise ValueError("form must be 'inverse' or 'block'")
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_hessian_factor")
    return U, perm_out, info


def onecomp_quantize_layer(W: torch.Tensor, U: torch.Tensor, bits: int, group_size: int,
                           perm: Optional[torch.Tensor] = None, block_size: int = 128, want_w_hat: bool = True,
                           workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None,
                           grid: str = "minmax", form: str = "inverse") -> dict:
    """Returns dict(Q_codes uint8, scales, zeros, W_hat (or None), loss) of device tensors.
    grid = "minmax" calls onecomp_quantize_layer, "symmetric" onecomp_quantize_layer_grid with that grid;
    "minmax_mse" / "symmetric_mse" (the grid with the scale search) call onecomp_quantize_layer_form;
    form = "block" (U from onecomp_hessian_factor(..., form="block")) calls onecomp_quantize_layer_form."""
    lib = load_library()
    d_out, d_in = W.shape
    dev = W.device
    if out is None:
        n_g = d_in // group_size if group_size > 0 and d_in % group_size == 0 else 1
        out = {
            "Q_codes": torch.empty((d_out, d_in), dtype=torch.uint8, device=dev),
            "scales": torch.empty((d_out, n_g), dtype=torch.float32, device=dev),
            "zeros": torch.empty((d_out, n_g), dtype=torch.float32, device=dev),
            "W_hat": torch.empty((d_out, d_in), dtype=torch.float32, device=dev) if want_w_hat else None,
            "loss": torch.zeros(1, dtype=torch.float32, device=dev),
        }
    need = onecomp_quantize_workspace_bytes(d_out, d_in, block_size)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    if perm is not None:
        _dev(perm, "perm", torch.int32)
    head = (_dev(W, "W"), _dtype_code(W), d_out, d_in, _dev(U, "U", torch.float32), _ptr(perm), int(bits),
            int(group_size), int(block_size))
    tail = (_dev(out["Q_codes"], "Q_codes", torch.uint8), _dev(out["scales"], "scales", torch.float32),
            _dev(out["zeros"], "zeros", torch.float32), _ptr(out["W_hat"]), _dev(out["loss"], "loss", torch.float32),
            _dev(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    if grid not in _GRIDS:
        raise ValueError("grid must be one of " + ", ".join(sorted(_GRIDS)))
    if form not in ("inverse", "block"):
        raise ValueError("form must be 'inverse' or 'block'")
    if form == "block" or grid.endswith("_mse"):
        rc = lib.onecomp_quantize_layer_form(*head[:5], ONECOMP_FACTOR_BLOCK if form == "block" else ONECOMP_FACTOR_INVERSE,
                                             *head[5:], _GRIDS[grid], *tail)
    elif grid == "minmax":
        rc = lib.onecomp_quantize_layer(*head, *tail)
    else:
        rc = lib.onecomp_quantize_layer_grid(*head, ONECOMP_GRID_SYMMETRIC, *tail)
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_quantize_layer")
    return out


def onecomp_qep_workspace_bytes(d_out: int, d_in: int) -> int:
    return int(load_library().onecomp_qep_workspace_bytes(int(d_out), int(d_in)))


def onecomp_crossgram_accumulate(X_hat: torch.Tensor, X: torch.Tensor, G: torch.Tensor) -> None:
    """G += 2 X_hat^T X.  X_hat, X: [n_tokens, d_in] bf16 (rows may be strided), G: [d_in, d_in] fp32."""
    lib = load_library()
    if X.dim() != 2 or X_hat.shape != X.shape or G.dim() != 2 or G.shape[0] != G.shape[1] or G.shape[0] != X.shape[1]:
        raise ValueError("shapes: X_hat, X [n_tokens, d_in], G [d_in, d_in]")
    if X.shape[0] > 0 and (X.stride(1) != 1 or X_hat.stride(1) != 1):
        raise ValueError("rows of X_hat and X must be dense")
    if X_hat.dtype != X.dtype:
        raise TypeError("X_hat and X must have the same dtype")
    _dev(X, "X", contiguous=False)
    _dev(X_hat, "X_hat", contiguous=False)
    ldx = X.stride(0) if X.shape[0] > 1 else X.shape[1]
    ldxh = X_hat.stride(0) if X_hat.shape[0] > 1 else X_hat.shape[1]
    rc = lib.onecomp_crossgram_accumulate(_ptr(X_hat), _ptr(X), _dtype_code(X), X.shape[0], X.shape[1], ldxh, ldx,
                                          _dev(G, "G", torch.float32), _stream())
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_crossgram_accumulate")


def onecomp_qep_target(W: torch.Tensor, G: torch.Tensor, H: torch.Tensor, U: torch.Tensor, alpha: float,
                       perm: Optional[torch.Tensor] = None, W_star: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Returns W* = W + alpha W (G - H)^T (H + lambda I)^-1 as an fp32 device tensor (U, perm from the factor call)."""
    lib = load_library()
    d_out, d_in = W.shape
    if W_star is None:
        W_star = torch.empty((d_out, d_in), dtype=torch.float32, device=W.device)
    need = onecomp_qep_workspace_bytes(d_out, d_in)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=W.device)
    if perm is not None:
        _dev(perm, "perm", torch.int32)
    rc = lib.onecomp_qep_target(_dev(W, "W"), _dtype_code(W), d_out, d_in, _dev(G, "G", torch.float32),
                                _dev(H, "H", torch.float32), _dev(U, "U", torch.float32), _ptr(perm), float(alpha),
                                _dev(W_star, "W_star", torch.float32), _dev(workspace, "workspace", torch.uint8),
                                workspace.numel(), _stream())
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_qep_target")
    return W_star


def onecomp_rtn_sensitivity(W: torch.Tensor, a_diag: torch.Tensor, bits: int, group_size: int,
                            b_diag: Optional[torch.Tensor] = None, grid: str = "minmax",
                            err: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """err = 1/2 sum_r sum_c b_r a_c (RTN(W) - W)_rc^2 as a device fp32 scalar tensor."""
    lib = load_library()
    d_out, d_in = W.shape
    if err is None:
        err = torch.zeros(1, dtype=torch.float32, device=W.device)
    if workspace is None:
        workspace = torch.empty(max(int(lib.onecomp_sensitivity_workspace_bytes()), 256), dtype=torch.uint8,
                                device=W.device)
    if grid not in ("minmax", "symmetric"):
        raise ValueError("grid must be 'minmax' or 'symmetric'")
    rc = lib.onecomp_rtn_sensitivity(_dev(W, "W"), _dtype_code(W), d_out, d_in, _dev(a_diag, "a_diag", torch.float32),
                                     _ptr(b_diag), int(bits), int(group_size),
                                     ONECOMP_GRID_SYMMETRIC if grid == "symmetric" else ONECOMP_GRID_MINMAX,
                                     _dev(err, "err", torch.float32), _dev(workspace, "workspace", torch.uint8),
                                     workspace.numel(), _stream())
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_rtn_sensitivity")
    return err


def onecomp_rtn_sensitivity_static(W: torch.Tensor, a_diag: torch.Tensor, bits: int, group_size: int,
                                   b_diag: Optional[torch.Tensor] = None, grid: str = "minmax",
                                   err: Optional[torch.Tensor] = None) -> torch.Tensor:
    """onecomp_rtn_sensitivity without a workspace (the library's built-in scratch).  Pass `err` (device fp32[1]) to keep
    this wrapper from allocating as well."""
    lib = load_library()
    d_out, d_in = W.shape
    if err is None:
        err = torch.zeros(1, dtype=torch.float32, device=W.device)
    if grid not in ("minmax", "symmetric"):
        raise ValueError("grid must be 'minmax' or 'symmetric'")
    rc = lib.onecomp_rtn_sensitivity_static(_dev(W, "W"), _dtype_code(W), d_out, d_in,
                                            _dev(a_diag, "a_diag", torch.float32), _ptr(b_diag), int(bits), int(group_size),
                                            ONECOMP_GRID_SYMMETRIC if grid == "symmetric" else ONECOMP_GRID_MINMAX,
                                            _dev(err, "err", torch.float32), _stream())
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_rtn_sensitivity_static")
    return err


def onecomp_jointq_workspace_bytes(d_out: int, d_in: int, group_size: int) -> int:
    return int(load_library().onecomp_jointq_workspace_bytes(int(d_out), int(d_in), int(group_size)))


def onecomp_jointq_refine(W: torch.Tensor, H: torch.Tensor, Q_codes: torch.Tensor, scales: torch.Tensor,
                          zeros: torch.Tensor, bits: int, group_size: int, grid: str = "minmax", lam: float = 0.0,
                          n_pass: int = 1, max_scans: int = 4, want_w_hat: bool = True,
                          workspace: Optional[torch.Tensor] = None, out: Optional[dict] = None,
                          perm: Optional[torch.Tensor] = None) -> dict:
    """Refines Q_codes and scales IN PLACE; returns dict(Q_codes, scales, W_hat (or None), objective [2] = row
    objective summed over the layer before and after, n_moves) of device tensors.  out: optional dict with
    preallocated "W_hat" (or None), "objective" (fp32[2]) and "n_moves" (int32[1])."""
    lib = load_library()
    d_out, d_in = W.shape
    dev = W.device
    if grid not in _GRIDS:
        raise ValueError("grid must be one of " + ", ".join(sorted(_GRIDS)))
    if workspace is None:
        workspace = torch.empty(max(onecomp_jointq_workspace_bytes(d_out, d_in, group_size), 256), dtype=torch.uint8,
                                device=dev)
    if out is not None:
        W_hat, objective, n_moves = out.get("W_hat"), out["objective"], out["n_moves"]
    else:
        W_hat = torch.empty((d_out, d_in), dtype=torch.float32, device=dev) if want_w_hat else None
        objective = torch.zeros(2, dtype=torch.float32, device=dev)
        n_moves = torch.zeros(1, dtype=torch.int32, device=dev)
    if perm is not None:
        _dev(perm, "perm", torch.int32)
    rc = lib.onecomp_jointq_refine(_dev(W, "W"), _dtype_code(W), d_out, d_in, _dev(H, "H", torch.float32), _ptr(perm),
                                   float(lam),
                                   int(bits), int(group_size), _GRIDS[grid], int(n_pass), int(max_scans),
                                   _dev(Q_codes, "Q_codes", torch.uint8), _dev(scales, "scales", torch.float32),
                                   _dev(zeros, "zeros", torch.float32), _ptr(W_hat),
                                   _dev(objective, "objective", torch.float32), _dev(n_moves, "n_moves", torch.int32),
                                   _dev(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    if rc != ONECOMP_OK:
        raise OnecompError(rc, "onecomp_jointq_refine")
    return {"Q_codes": Q_codes, "scales": scales, "W_hat": W_hat, "objective": objective, "n_moves": n_moves}
