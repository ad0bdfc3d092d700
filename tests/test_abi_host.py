"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
function the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

import paper_2603_28845_amd as oc_gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "onecomp.h")

OK, INVALID, UNSUPPORTED, NOT_POSDEF, WORKSPACE, HIP = range(6)


@pytest.fixture(scope="module")
def lib():
    return oc_gpu.load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(onecomp_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(lib):
    names = _declared_functions()
    assert set(names) == set(oc_gpu.EXPORTED_SYMBOLS)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_status_strings(lib):
    assert oc_gpu.onecomp_version() >= 100
    seen = {oc_gpu.status_string(c) for c in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert oc_gpu.status_string(99) == "unknown status"


def test_workspace_queries(lib):
    assert oc_gpu.onecomp_factor_workspace_bytes(0) == 0
    assert oc_gpu.onecomp_factor_workspace_bytes(100) == 0          # not a multiple of 16
    assert oc_gpu.onecomp_factor_workspace_bytes(512) >= 3 * 512 * 512 * 8
    assert oc_gpu.onecomp_quantize_workspace_bytes(256, 512, 128) >= 256 * 512 * 4
    assert oc_gpu.onecomp_quantize_workspace_bytes(256, 512, 64) == 0
    assert oc_gpu.onecomp_quantize_workspace_bytes(256, 500, 128) == 0


P = ctypes.c_void_p(0x10000)   # non-null, 256-byte aligned dummy; never dereferenced on these paths
NULL = ctypes.c_void_p(0)


def test_accumulate_argument_checks(lib):
    f = lib.onecomp_hessian_accumulate
    assert f(P, 7, 10, 128, 128, P, NULL) == UNSUPPORTED
    assert f(P, 0, 10, 128, 128, NULL, NULL) == INVALID       # H null
    assert f(NULL, 0, 10, 128, 128, P, NULL) == INVALID       # X null with tokens
    assert f(P, 0, 10, 120, 120, P, NULL) == INVALID          # d_in % 16
    assert f(P, 0, 10, 128, 64, P, NULL) == INVALID           # ldx < d_in
    assert f(P, 0, -1, 128, 128, P, NULL) == INVALID
    assert f(ctypes.c_void_p(0x10004), 1, 10, 128, 128, P, NULL) == INVALID   # misaligned X
    assert f(NULL, 0, 0, 128, 128, P, NULL) == OK             # zero tokens: no-op


def test_accumulate_ws_argument_checks(lib):
    f = lib.onecomp_hessian_accumulate_ws
    big = ctypes.c_size_t(1 << 30)
    assert f(P, 7, 10, 128, 128, P, P, big, NULL) == UNSUPPORTED
    assert f(P, 1, 10, 128, 128, NULL, P, big, NULL) == INVALID                 # H null
    assert f(NULL, 1, 10, 128, 128, P, P, big, NULL) == INVALID                 # X null with tokens
    assert f(P, 1, 10, 120, 120, P, P, big, NULL) == INVALID                    # d_in % 16
    assert f(P, 1, 10, 128, 64, P, P, big, NULL) == INVALID                     # ldx < d_in
    assert f(P, 1, 10, 128, 128, P, ctypes.c_void_p(0x10010), big, NULL) == WORKSPACE   # misaligned workspace
    assert f(P, 1, 0, 128, 128, P, P, big, NULL) == OK                          # no tokens: nothing to do
    assert f(P, 1, 0, 128, 128, P, NULL, ctypes.c_size_t(0), NULL) == OK
    g = lib.onecomp_accumulate_workspace_bytes
    assert g(0, 4096) == 0          # fp32 inputs never use one
    assert g(1, 0) == 0 and g(1, 100) == 0


def test_accumulate_describe_argument_checks(lib):
    out = (ctypes.c_int32 * 3)(-1, -1, -1)
    fn = lib.onecomp_accumulate_describe
    fn.restype = ctypes.c_int
    i64, sz = ctypes.c_int64, ctypes.c_size_t
    assert fn(1, i64(100), i64(512), i64(512), sz(0), None) == INVALID          # no output pointer
    assert fn(7, i64(100), i64(512), i64(512), sz(0), out) == UNSUPPORTED       # dtype
    assert fn(1, i64(100), i64(520), i64(520), sz(0), out) == INVALID           # d_in not a multiple of 16
    assert fn(1, i64(-1), i64(512), i64(512), sz(0), out) == INVALID
    assert fn(1, i64(100), i64(512), i64(256), sz(0), out) == INVALID           # row stride below d_in
    assert list(out) == [-1, -1, -1]
    # narrow layers and fp32 inputs: one launch of a 128 x 128 kernel, known without asking the device
    assert fn(1, i64(100), i64(512), i64(512), sz(0), out) == OK and list(out) == [128, 128, 1]
    assert fn(0, i64(100), i64(4096), i64(4096), sz(0), out) == OK and list(out) == [128, 128, 1]


def test_mfma_rate_probe_argument_checks(lib):
    fn = lib.onecomp_mfma_rate_probe
    fn.restype = ctypes.c_int
    i64 = ctypes.c_int64
    flops = ctypes.c_double(-1.0)
    fp = ctypes.byref(flops)
    sink = ctypes.c_void_p(256)      # never dereferenced: every case below is rejected on the host
    assert fn(2, 1, 1, i64(10), sink, fp, None) == UNSUPPORTED            # kind
    assert fn(0, 3, 1, i64(10), sink, fp, None) == UNSUPPORTED            # waves per SIMD
    assert fn(0, 1, 2, i64(10), sink, fp, None) == INVALID                # operand pattern
    assert fn(0, 1, 1, i64(0), sink, fp, None) == INVALID                 # no trips
    assert fn(1, 2, 0, i64(1 << 25), sink, fp, None) == INVALID           # too many trips
    assert fn(0, 1, 1, i64(10), None, fp, None) == INVALID                # no sink
    assert fn(0, 1, 1, i64(10), sink, None, None) == INVALID              # no flop count
    assert flops.value == -1.0


def test_factor_argument_checks(lib):
    f = lib.onecomp_hessian_factor
    big = ctypes.c_size_t(1 << 40)
    assert f(NULL, 128, 0.01, 0, NULL, P, P, P, big, NULL) == INVALID
    assert f(P, 128, 0.01, 0, NULL, NULL, P, P, big, NULL) == INVALID
    assert f(P, 128, 0.01, 0, NULL, P, NULL, P, big, NULL) == INVALID
    assert f(P, 100, 0.01, 0, NULL, P, P, P, big, NULL) == INVALID
    assert f(P, 128, -1.0, 0, NULL, P, P, P, big, NULL) == INVALID
    assert f(P, 128, float("nan"), 0, NULL, P, P, P, big, NULL) == INVALID
    assert f(P, 128, 0.01, 1, NULL, P, P, P, big, NULL) == INVALID      # act_order needs perm_out
    assert f(P, 128, 0.01, 0, NULL, P, P, NULL, big, NULL) == WORKSPACE
    assert f(P, 128, 0.01, 0, NULL, P, P, P, ctypes.c_size_t(1024), NULL) == WORKSPACE
    assert f(P, 128, 0.01, 0, NULL, P, P, ctypes.c_void_p(0x10010), big, NULL) == WORKSPACE


def test_quantize_argument_checks(lib):
    f = lib.onecomp_quantize_layer
    big = ctypes.c_size_t(1 << 40)

    def call(W=P, dt=1, d_out=64, d_in=256, U=P, perm=NULL, bits=4, G=128, B=128, Q=P, s=P, z=P, wh=P, loss=P,
             ws=P, wsb=big):
        return f(W, dt, d_out, d_in, U, perm, bits, G, B, Q, s, z, wh, loss, ws, wsb, NULL)

    assert call(dt=3) == UNSUPPORTED
    assert call(W=NULL) == INVALID
    assert call(U=NULL) == INVALID
    assert call(Q=NULL) == INVALID
    assert call(loss=NULL) == INVALID
    assert call(d_out=0) == INVALID
    for b in (0, 1, 5, 6, 7, 9, 16):
        assert call(bits=b) == UNSUPPORTED
    assert call(B=64) == UNSUPPORTED
    assert call(d_in=200) == INVALID            # d_in % block
    assert call(G=96) == INVALID                # does not divide d_in
    assert call(d_in=384, G=192) == INVALID     # divides d_in, but neither divides nor is divided by the block
    assert call(G=8) == UNSUPPORTED             # not a multiple of 16
    assert call(G=0) == INVALID
    assert call(ws=NULL) == WORKSPACE
    assert call(wsb=ctypes.c_size_t(16)) == WORKSPACE
    assert call(d_in=65536 + 128) == INVALID    # beyond the 16-bit column limit of the sweep
    assert call(W=ctypes.c_void_p(0x10004)) == INVALID      # misaligned W / U (16 bytes), Q_codes (4), W_hat (16)
    assert call(U=ctypes.c_void_p(0x10008)) == INVALID
    assert call(Q=ctypes.c_void_p(0x10002)) == INVALID
    assert call(wh=ctypes.c_void_p(0x10004)) == INVALID


def test_crossgram_argument_checks(lib):
    f = lib.onecomp_crossgram_accumulate
    f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                  ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
    f.restype = ctypes.c_int
    assert f(P, P, 0, 10, 128, 128, 128, P, NULL) == UNSUPPORTED       # fp32 activations
    assert f(P, P, 1, 10, 128, 128, 128, NULL, NULL) == INVALID        # no G
    assert f(P, P, 1, 10, 120, 120, 120, P, NULL) == INVALID           # d_in % 16
    assert f(P, P, 1, 10, 128, 64, 128, P, NULL) == INVALID            # row stride below d_in
    assert f(NULL, P, 1, 10, 128, 128, 128, P, NULL) == INVALID
    assert f(P, P, 1, -1, 128, 128, 128, P, NULL) == INVALID
    assert f(P, P, 1, 10, 128, 128, 1 << 26, P, NULL) == UNSUPPORTED   # 16 rows not addressable with 32 bits
    assert f(NULL, NULL, 1, 0, 128, 128, 128, P, NULL) == 0            # zero tokens: nothing to do


def test_qep_target_argument_checks(lib):
    f = lib.onecomp_qep_target
    f.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                  ctypes.c_void_p]
    f.restype = ctypes.c_int
    lib.onecomp_qep_workspace_bytes.argtypes = [ctypes.c_int64, ctypes.c_int64]
    lib.onecomp_qep_workspace_bytes.restype = ctypes.c_size_t
    big = ctypes.c_size_t(1 << 40)
    P2 = ctypes.c_void_p(0x20000)

    def call(W=P, dt=1, d_out=64, d_in=256, G=P, H=P, U=P, perm=NULL, alpha=0.5, out=P2, ws=P, wsb=big):
        return f(W, dt, d_out, d_in, G, H, U, perm, alpha, out, ws, wsb, NULL)

    assert call(dt=2) == UNSUPPORTED
    assert call(W=NULL) == INVALID
    assert call(G=NULL) == INVALID
    assert call(U=NULL) == INVALID
    assert call(out=NULL) == INVALID
    assert call(out=P) == INVALID                # W* must not alias W
    assert call(alpha=1.5) == INVALID
    assert call(alpha=-0.1) == INVALID
    assert call(alpha=float("nan")) == INVALID
    assert call(d_in=250) == INVALID
    assert call(ws=NULL) == WORKSPACE
    assert call(wsb=ctypes.c_size_t(1000)) == WORKSPACE
    need = lib.onecomp_qep_workspace_bytes(64, 256)
    assert need >= 4 * 256 * 256 + 3 * 4 * 64 * 256
    assert lib.onecomp_qep_workspace_bytes(64, 250) == 0


def test_quantize_grid_argument_checks(lib):
    f = lib.onecomp_quantize_layer_grid
    f.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                  ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                  ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    f.restype = ctypes.c_int
    big = ctypes.c_size_t(1 << 40)
    assert f(P, 1, 64, 256, P, NULL, 4, 128, 128, 4, P, P, P, P, P, P, big, NULL) == UNSUPPORTED    # unknown grid
    assert f(P, 1, 64, 256, P, NULL, 4, 128, 128, 3, P, P, P, P, P, NULL, big, NULL) == WORKSPACE
    assert f(P, 1, 64, 256, P, NULL, 4, 128, 128, -1, P, P, P, P, P, P, big, NULL) == UNSUPPORTED
    assert f(NULL, 1, 64, 256, P, NULL, 4, 128, 128, 1, P, P, P, P, P, P, big, NULL) == INVALID
    assert f(P, 1, 64, 256, P, NULL, 4, 128, 128, 1, P, P, P, P, P, NULL, big, NULL) == WORKSPACE


def test_factor_form_argument_checks(lib):
    f = lib.onecomp_hessian_factor_form
    big = ctypes.c_size_t(1 << 40)
    BLOCK = 1
    assert f(P, 256, 0.01, 0, 2, NULL, P, P, P, big, NULL) == UNSUPPORTED       # unknown form
    assert f(P, 256, 0.01, 0, -1, NULL, P, P, P, big, NULL) == UNSUPPORTED
    assert f(P, 144, 0.01, 0, BLOCK, NULL, P, P, P, big, NULL) == UNSUPPORTED   # block form needs d_in % 128 == 0
    assert f(P, 100, 0.01, 0, BLOCK, NULL, P, P, P, big, NULL) == INVALID       # d_in % 16 comes first
    assert f(NULL, 256, 0.01, 0, BLOCK, NULL, P, P, P, big, NULL) == INVALID
    assert f(P, 256, 0.01, 0, BLOCK, NULL, NULL, P, P, big, NULL) == INVALID
    assert f(P, 256, 0.01, 1, BLOCK, NULL, P, P, P, big, NULL) == INVALID       # act_order needs perm_out
    assert f(P, 256, -1.0, 0, BLOCK, NULL, P, P, P, big, NULL) == INVALID
    assert f(P, 256, 0.01, 0, BLOCK, NULL, P, P, NULL, big, NULL) == WORKSPACE
    assert f(P, 256, 0.01, 0, BLOCK, NULL, P, P, P, ctypes.c_size_t(1024), NULL) == WORKSPACE


def test_quantize_form_argument_checks(lib):
    f = lib.onecomp_quantize_layer_form
    big = ctypes.c_size_t(1 << 40)
    BLOCK = 1

    def call(W=P, dt=1, d_out=64, d_in=256, F=P, form=BLOCK, perm=NULL, bits=4, G=128, B=128, grid=0, Q=P, s=P, z=P,
             wh=P, loss=P, ws=P, wsb=big):
        return f(W, dt, d_out, d_in, F, form, perm, bits, G, B, grid, Q, s, z, wh, loss, ws, wsb, NULL)

    assert call(form=2) == UNSUPPORTED
    assert call(form=-1) == UNSUPPORTED
    assert call(d_in=512, G=256) == UNSUPPORTED  # block form: groups no wider than a block, or one group per row
    assert call(grid=4) == UNSUPPORTED
    assert call(dt=3) == UNSUPPORTED
    assert call(bits=5) == UNSUPPORTED
    assert call(W=NULL) == INVALID
    assert call(F=NULL) == INVALID
    assert call(d_in=200) == INVALID
    assert call(G=96) == INVALID
    assert call(ws=NULL) == WORKSPACE
    assert call(wsb=ctypes.c_size_t(16)) == WORKSPACE


def test_sensitivity_argument_checks(lib):
    f = lib.onecomp_rtn_sensitivity
    f.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p,
                  ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                  ctypes.c_void_p]
    f.restype = ctypes.c_int
    lib.onecomp_sensitivity_workspace_bytes.restype = ctypes.c_size_t
    big = ctypes.c_size_t(1 << 30)

    def call(W=P, dt=1, d_out=64, d_in=256, a=P, b=NULL, bits=4, G=128, grid=0, err=P, ws=P, wsb=big):
        return f(W, dt, d_out, d_in, a, b, bits, G, grid, err, ws, wsb, NULL)

    assert call(dt=5) == UNSUPPORTED
    assert call(grid=3) == UNSUPPORTED
    assert call(bits=5) == UNSUPPORTED
    assert call(G=24) == INVALID           # does not divide d_in
    assert call(G=8) == UNSUPPORTED        # not a multiple of 16
    assert call(W=NULL) == INVALID
    assert call(a=NULL) == INVALID
    assert call(err=NULL) == INVALID
    assert call(W=ctypes.c_void_p(0x10004)) == INVALID     # W and a_diag are read with 16-byte loads
    assert call(a=ctypes.c_void_p(0x10008)) == INVALID
    assert call(ws=NULL) == WORKSPACE
    assert call(wsb=ctypes.c_size_t(8)) == WORKSPACE
    assert lib.onecomp_sensitivity_workspace_bytes() >= 4


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    """No CPU fallback: with the shared library missing, the first use of the binding raises and names the build step."""
    from paper_2603_28845_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libonecomp.so"))
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.load_library()
    with pytest.raises(RuntimeError, match="missing"):
        binding.onecomp_factor_workspace_bytes(512)


def test_product_never_imports_the_oracle():
    """The oracle is test infrastructure: nothing in the package or its C sources refers to it."""
    pkg = os.path.join(ROOT, "paper_2603_28845_amd")
    for base, _, files in os.walk(pkg):
        if "_build" in base or "__pycache__" in base:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(base, f), errors="ignore").read()
                assert not re.search(r"^\s*(from|import)\s+oracle\b", text, flags=re.M), os.path.join(base, f)
                assert "oracle/" not in text and "onecomp_oracle" not in text, os.path.join(base, f)
    text = open(HEADER).read()
    assert "oracle" not in text.lower()


def test_jointq_argument_checks(lib):
    f = lib.onecomp_jointq_refine
    big = ctypes.c_size_t(1 << 40)

    def call(W=P, dt=1, d_out=64, d_in=256, H=P, lam=0.0, bits=4, G=128, grid=0, n_pass=1, scans=4, Q=P, s=P, z=P,
             wh=NULL, obj=P, mv=P, ws=P, wsb=big):
        return f(W, dt, d_out, d_in, H, NULL, lam, bits, G, grid, n_pass, scans, Q, s, z, wh, obj, mv, ws, wsb, NULL)

    assert call(dt=3) == UNSUPPORTED
    assert call(grid=7) == UNSUPPORTED
    assert call(bits=5) == UNSUPPORTED
    assert call(G=192, d_in=384) == UNSUPPORTED      # wider than 128 and not a multiple of 128
    assert call(G=24, d_in=240) == UNSUPPORTED       # not a multiple of 16
    assert call(W=NULL) == INVALID
    assert call(H=NULL) == INVALID
    assert call(Q=NULL) == INVALID
    assert call(obj=NULL) == INVALID
    assert call(mv=NULL) == INVALID
    assert call(lam=-1.0) == INVALID
    assert call(lam=float("nan")) == INVALID
    assert call(n_pass=-1) == INVALID
    assert call(scans=0) == INVALID
    assert call(G=96) == INVALID                     # does not divide d_in
    assert call(W=ctypes.c_void_p(0x10004)) == INVALID      # misaligned W (16 bytes), H (16), Q_codes (4), W_hat (16)
    assert call(H=ctypes.c_void_p(0x10008)) == INVALID
    assert call(Q=ctypes.c_void_p(0x10002)) == INVALID
    assert call(wh=ctypes.c_void_p(0x10004)) == INVALID
    assert call(ws=NULL) == WORKSPACE
    assert call(wsb=ctypes.c_size_t(1024)) == WORKSPACE
    g = lib.onecomp_jointq_workspace_bytes
    assert g(64, 256, 128) >= 2 * 64 * 256 * 4
    assert g(64, 384, 192) == 0 and g(0, 256, 128) == 0 and g(64, 250, 50) == 0
    assert g(64, 256, 256) > g(64, 256, 128)         # wider groups carry two more matrices


def test_header_is_plain_c_and_links(tmp_path):
    """The boundary is a C header: it must compile as C99 on its own, and a C program must link against the library."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_onecomp.c"
    src.write_text('#include "onecomp.h"\n'
                   '#include <stdio.h>\n'
                   'int main(void) {\n'
                   '    printf("%d %s\\n", onecomp_version(), onecomp_status_string(ONECOMP_OK));\n'
                   '    /* host-side argument check: no GPU is touched */\n'
                   '    return onecomp_hessian_accumulate(0, ONECOMP_BF16, 1, 128, 128, 0, 0) == ONECOMP_ERR_INVALID_ARG ? 0 : 1;\n'
                   '}\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(src)],
                   check=True)
    lib_dir = os.path.dirname(oc_gpu.LIB_PATH)
    exe = tmp_path / "use_onecomp"
    subprocess.run([gcc, "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", lib_dir, "-lonecomp",
                    f"-Wl,-rpath,{lib_dir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == oc_gpu.onecomp_version() and out[1] == "ok"


def test_marker_ranges_are_opt_in(tmp_path):
    """ONECOMP_ROCTX=1 makes the entry points look the ROCTx library up at run time and push a named range per call;
    without it the library loads nothing of the kind.  Checked in child processes through an argument-check path
    (no GPU is touched); skipped where no ROCTx library is installed."""
    import subprocess
    import sys
    if not any(os.path.exists(os.path.join("/opt/rocm/lib", n)) for n in ("librocprofiler-sdk-roctx.so.1", "libroctx64.so.4")):
        pytest.skip("no ROCTx library in this image")
    prog = tmp_path / "probe.py"
    prog.write_text(
        "import ctypes\n"
        f"lib = ctypes.CDLL({oc_gpu.LIB_PATH!r})\n"
        "lib.onecomp_rtn_sensitivity_static.restype = ctypes.c_int\n"
        "rc = lib.onecomp_rtn_sensitivity_static(None, 0, ctypes.c_int64(4), ctypes.c_int64(16), None, None, 4, 16, 0, None, None)\n"
        "print(rc, 'roctx' in open('/proc/self/maps').read())\n")
    for value, expect in (("1", "True"), ("0", "False"), (None, "False")):
        env = dict(os.environ)
        env.pop("ONECOMP_ROCTX", None)
        if value is not None:
            env["ONECOMP_ROCTX"] = value
        out = subprocess.run([sys.executable, str(prog)], env=env, check=True, capture_output=True, text=True).stdout.split()
        assert out == [str(INVALID), expect], (value, out)
