"""Host-side checks of the C-ABI library: it loads, exports every symbol the header declares,
its size queries are right, and argument validation rejects bad calls before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "snip.h")


def lib():
    from paper_2602_01410_amd import snip
    if not os.path.exists(snip.LIB_PATH):
        from paper_2602_01410_amd.build import build_library
        build_library()
    return snip


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(snip_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported():
    snip = lib()
    handle = ctypes.CDLL(snip.LIB_PATH)
    names = declared_functions()
    assert set(names) == set(snip.EXPORTS)
    for n in names:
        assert hasattr(handle, n), n


def test_size_queries():
    snip = lib()
    assert snip.code_bytes(10, 64, snip.FP8) == 640
    assert snip.code_bytes(10, 64, snip.FP4) == 320
    assert snip.code_bytes(10, 48, snip.FP8) == 0          # not a multiple of 32
    assert snip.scale_bytes(10, 64) == 20
    assert snip.scale_g4_bytes(10, 64) == 256 * 1 * 4          # one group of 4 blocks, rows padded to 256
    assert snip.scale_g4_bytes(300, 4096) == 512 * 32 * 4
    assert snip.workspace_bytes(1024, 4096) >= 8192 * 12


def test_validation_rejects_before_launch():
    snip = lib()
    L = snip._lib()
    q = snip._QTensorC(0, 0, 0, 32, 64, 0)
    # null source
    assert L.snip_quantize(None, 32, 64, 64, 0, 0, 0, ctypes.byref(q), None, None, 0, None) == 1
    # a fake but aligned, never dereferenced source pointer: validation only
    fake = ctypes.c_void_p(0x1000)
    assert L.snip_quantize(fake, 32, 48, 48, 0, 0, 0, ctypes.byref(q), None, None, 0, None) == 2   # cols % 32
    assert L.snip_quantize(fake, 32, 64, 64, 7, 0, 0, ctypes.byref(q), None, None, 0, None) == 3   # fmt
    assert L.snip_quantize(fake, 32, 64, 60, 0, 0, 0, ctypes.byref(q), None, None, 0, None) == 2   # ld < cols
    assert L.snip_quantize(fake, 32, 64, 68, 0, 0, 0, ctypes.byref(q), None, None, 0, None) == 4   # ld % 8
    assert L.snip_quantize(fake, 32, 64, 64, 0, 0, 0, ctypes.byref(q), None, None, 0, None) == 1   # null codes
    assert L.snip_quant_error_stats(fake, 32, 64, 64, 0, 0, fake, None, None, 0, None) == 5        # workspace
    assert L.snip_quant_error_stats(fake, 31, 64, 64, 1, 0, fake, None, fake, 1 << 30, None) == 2  # rows % 32 (COL)
    plan = snip.make_plan((0,) * 6)
    assert L.snip_gemm_fwd(ctypes.byref(plan), None, None, fake, 64, 0, None, 0, None) == 1
    assert L.snip_status_string(4).decode().startswith("bad alignment")


def test_grouped_scale_copy_must_be_16_byte_aligned():
    snip = lib()
    L = snip._lib()
    fake = ctypes.c_void_p(0x1000)
    q = snip._QTensorC(0x1000, 0x1000, 0x1004, 32, 64, 0)          # grouped copy only 4-byte aligned
    assert L.snip_quantize(fake, 32, 64, 64, 0, 0, 0, ctypes.byref(q), None, None, 0, None) == 4
    plan = snip.make_plan((0,) * 6)
    ok = snip._QTensorC(0x1000, 0x1000, 0x1000, 32, 64, 0)
    assert L.snip_gemm_fwd(ctypes.byref(plan), ctypes.byref(q), ctypes.byref(ok), fake, 64, 0, None, 0, None) == 4


def test_quantize_both_validation():
    snip = lib()
    L = snip._lib()
    fake = ctypes.c_void_p(0x1000)
    qr = snip._QTensorC(0x1000, 0x1000, 0, 64, 96, 0)
    qc = snip._QTensorC(0x1000, 0x1000, 0, 96, 64, 1)
    br, bc = ctypes.byref(qr), ctypes.byref(qc)
    assert L.snip_quantize_both(None, 64, 96, 96, 0, br, bc, None, None, 0, None, 0, None) == 1          # null source
    assert L.snip_quantize_both(fake, 64, 96, 96, 0, None, bc, None, None, 0, None, 0, None) == 1        # null output
    assert L.snip_quantize_both(fake, 48, 96, 96, 0, br, bc, None, None, 0, None, 0, None) == 2          # rows % 32
    assert L.snip_quantize_both(fake, 64, 80, 80, 0, br, bc, None, None, 0, None, 0, None) == 2          # cols % 32
    assert L.snip_quantize_both(fake, 64, 96, 96, 0, bc, br, None, None, 0, None, 0, None) == 2          # outputs swapped
    assert L.snip_quantize_both(fake, 64, 96, 96, 0, br, bc, fake, None, 0, fake, 1 << 30, None) == 1    # one statistics output
    assert L.snip_quantize_both(fake, 64, 96, 96, 0, br, bc, fake, fake, 0, None, 0, None) == 5          # workspace
    assert L.snip_quantize_both(fake, 64, 96, 96, 0, br, bc, None, None, 7, None, 0, None) == 3           # scope
    bad = snip._QTensorC(0x1000, 0x1000, 0, 96, 64, 5)
    assert L.snip_quantize_both(fake, 64, 96, 96, 0, br, ctypes.byref(bad), None, None, 0, None, 0, None) == 3   # format
    odd = snip._QTensorC(0x1008, 0x1000, 0, 96, 64, 1)
    assert L.snip_quantize_both(fake, 64, 96, 96, 0, br, ctypes.byref(odd), None, None, 0, None, 0, None) == 4   # alignment


def test_gemm_norm_validation_and_workspace_size():
    snip = lib()
    L = snip._lib()
    fake = ctypes.c_void_p(0x1000)
    assert snip.gemm_workspace_bytes(256, 256) >= 4 * 4            # four 128 x 128 tiles, one float each
    assert snip.gemm_workspace_bytes(100, 100) >= 4
    assert snip.gemm_workspace_bytes(16384, 11008) >= 128 * 86 * 4
    assert snip.gemm_workspace_bytes(-1, 5) == 0
    plan = snip.make_plan((0,) * 6)
    qa = snip._QTensorC(0x1000, 0x2000, 0, 64, 64, 0)
    qb = snip._QTensorC(0x3000, 0x4000, 0, 32, 64, 0)
    args = (ctypes.byref(plan), ctypes.byref(qa), ctypes.byref(qb), fake, 32, 0)
    assert L.snip_gemm_fwd_norm(*args, None, fake, 1 << 20, None) == 1      # no place for the norm
    assert L.snip_gemm_dgrad_norm(*args, fake, None, 0, None) == 5          # workspace missing
    assert L.snip_gemm_wgrad_norm(*args, fake, fake, 8, None) == 5          # workspace too small


def test_loss_divergence_host_function_against_oracle():
    """Pure host arithmetic: checked here without a GPU, to 1e-14 (the two sides group the square roots
    differently)."""
    import math
    import numpy as np
    import oracle
    snip = lib()
    rng = np.random.default_rng(60)
    for _ in range(200):
        gx, ex, gw, ew = (float(v) for v in 10.0 ** rng.uniform(-12, 12, size=4))
        m, n, k = (int(v) for v in rng.integers(1, 1 << 20, size=3))
        want = oracle.loss_divergence(gx, ex, m, gw, ew, n, k)
        assert math.isclose(snip.snip_loss_divergence(gx, ex, m, gw, ew, n, k), want, rel_tol=1e-14)
    assert snip.snip_loss_divergence(36.0, 36.0, 16, 16.0, 36.0, 4, 9) == 5.0
    assert snip.snip_loss_divergence(0.0, 0.0, 1, 0.0, 0.0, 1, 1) == 0.0
    assert math.isnan(snip.snip_loss_divergence(1.0, 1.0, 0, 1.0, 1.0, 4, 4))
    assert math.isnan(snip.snip_loss_divergence(-1.0, 1.0, 4, 1.0, 1.0, 4, 4))


def test_weight_divergence_host_function_against_oracle():
    import math
    import numpy as np
    import oracle
    snip = lib()
    rng = np.random.default_rng(61)
    for _ in range(100):
        alpha = float(10.0 ** rng.uniform(-6, -2))
        b1, b2 = float(rng.uniform(0.5, 0.99)), float(rng.uniform(0.9, 0.9999))
        t = int(rng.integers(1, 100000))
        s, e = (float(x) for x in 10.0 ** rng.uniform(-10, 12, size=2))
        n, k = (int(x) for x in rng.integers(1, 1 << 16, size=2))
        want = oracle.weight_divergence(alpha, b1, b2, t, s, e, n, k)
        assert math.isclose(snip.snip_weight_divergence(alpha, b1, b2, t, s, e, n, k), want, rel_tol=1e-13)
    assert math.isnan(snip.snip_weight_divergence(1e-3, 0.9, 0.999, 0, 1.0, 1.0, 4, 4))
    assert math.isnan(snip.snip_weight_divergence(1e-3, 1.0, 0.999, 1, 1.0, 1.0, 4, 4))


def test_adamw_validation():
    snip = lib()
    L = snip._lib()
    fake = ctypes.c_void_p(0x1000)
    ws = snip.workspace_bytes(0, 0)
    assert L.snip_adamw_sensitivity(None, fake, fake, 1, 8, 0.9, 0.999, 1e-8, fake, fake, ws, None) == 1
    assert L.snip_adamw_sensitivity(fake, fake, fake, 1, -1, 0.9, 0.999, 1e-8, fake, fake, ws, None) == 2
    assert L.snip_adamw_sensitivity(fake, fake, fake, 5, 8, 0.9, 0.999, 1e-8, fake, fake, ws, None) == 3
    assert L.snip_adamw_sensitivity(fake, fake, fake, 1, 8, 1.5, 0.999, 1e-8, fake, fake, ws, None) == 3
    assert L.snip_adamw_sensitivity(fake, fake, ctypes.c_void_p(0x1004), 1, 8, 0.9, 0.999, 1e-8, fake, fake, ws, None) == 4
    assert L.snip_adamw_sensitivity(fake, fake, fake, 1, 8, 0.9, 0.999, 1e-8, fake, fake, 16, None) == 5


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    from paper_2602_01410_amd import snip
    monkeypatch.setattr(snip, "_handle", None)
    monkeypatch.setattr(snip, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        snip.workspace_bytes(1, 32)


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 and as C++ without any HIP or torch include, and
    a C program that only includes it must link against the library and run the host-only calls."""
    import subprocess
    snip = lib()
    src = tmp_path / "use.c"
    src.write_text(
        '#include "snip.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "  snip_layer_plan p = {0, 0, 1, 1, 1, 0}; (void)p;\n"
        "  if (snip_qtensor_code_bytes(4, 64, SNIP_FP4_E2M1) != 128) return 1;\n"
        "  if (snip_workspace_bytes(16, 64) == 0) return 2;\n"
        "  if (snip_loss_divergence(36.0, 36.0, 16, 16.0, 36.0, 4, 9) != 5.0) return 3;\n"
        "  if (snip_quantize(0, 32, 64, 64, SNIP_FP8_E4M3, SNIP_AXIS_ROW, SNIP_SCALE_NO_OVERFLOW, 0, 0, 0, 0, 0) != SNIP_ERR_NULL) return 4;\n"
        '  printf("%s\\n", snip_status_string(SNIP_OK));\n  return 0;\n}\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", inc, str(src)], check=True)
    subprocess.run(["g++", "-std=c++11", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)], check=True)
    exe = tmp_path / "use"
    libdir = os.path.dirname(snip.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-lsnip_hip",
                    "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", (out.returncode, out.stdout, out.stderr)


def test_binding_argument_counts_match_the_header():
    """Every prototype of the header against the argument list the ctypes binding declares for it."""
    snip = lib()
    L = snip._lib()
    src = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    protos = re.findall(r"\b(snip_[a-z0-9_]+)\s*\(([^;{]*?)\)\s*;", src, flags=re.S)
    assert len(protos) >= 20
    checked = 0
    for name, params in protos:
        params = params.strip()
        n = 0 if params in ("", "void") else params.count(",") + 1
        fn = getattr(L, name)
        if fn.argtypes is None:
            continue
        assert len(fn.argtypes) == n, (name, len(fn.argtypes), n)
        checked += 1
    assert checked >= 20
