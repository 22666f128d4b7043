"""CPU oracle for the SNIP quantized linear-layer path.  TEST INFRASTRUCTURE ONLY.

A thin ctypes loader around ``snip_oracle.c`` (plain C, IEEE double and integers).  Only
the tests, the smoke check and the benchmark's CPU-baseline leg may import this package;
the GPU library and its Python binding never do, and the two share no code.

Passages followed (SNIP, arXiv 2602.01410): Sec. 2.3 (scaling by the block maximum and the
cast to FPX), Sec. 2.2 (which tensors are quantized before which GEMM), Sec. 4.1 / 4.3.1
(shapes of X, W, dY), Sec. 3.1 Step 1 and Sec. 5.3 (Frobenius-norm statistics and their
row-wise form).  The paper prints no worked numeric example for this path; the pins are the
closed forms, enumerations and brute-force checks in ``tests/test_oracle_*.py``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "snip_oracle.c")
_LIB = os.path.join(_HERE, "libsnip_oracle.so")

FP8, FP4 = 0, 1            # element formats: E4M3, E2M1
ROW, COL = 0, 1            # direction of the 32-element tiles in the source matrix
NO_OVERFLOW, FLOOR = 0, 1  # power-of-two scale rules
TILE = 32


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # SNIP_ORACLE_LIB: an alternative build of this same source (the mutation test of the pins uses it
        # to load copies with a planted mistake); unset in every other use
        lib = ctypes.CDLL(os.environ.get("SNIP_ORACLE_LIB") or build())
        i64, dbl, ci, u16 = ctypes.c_int64, ctypes.c_double, ctypes.c_int, ctypes.c_uint16
        vp = ctypes.c_void_p
        lib.oracle_bf16_to_f64.restype = dbl
        lib.oracle_bf16_to_f64.argtypes = [u16]
        lib.oracle_decode.restype = dbl
        lib.oracle_decode.argtypes = [ci, ctypes.c_uint]
        lib.oracle_fmt_max.restype = dbl
        lib.oracle_fmt_max.argtypes = [ci]
        lib.oracle_encode_rne.restype = ctypes.c_uint
        lib.oracle_encode_rne.argtypes = [ci, dbl]
        lib.oracle_scale_byte.restype = ctypes.c_uint
        lib.oracle_scale_byte.argtypes = [ci, ci, dbl]
        lib.oracle_quantize.restype = ci
        lib.oracle_quantize.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, vp]
        lib.oracle_dequantize.restype = ci
        lib.oracle_dequantize.argtypes = [vp, vp, i64, i64, ci, vp]
        lib.oracle_fake_quant.restype = ci
        lib.oracle_fake_quant.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp]
        for name in ("oracle_gemm_fwd", "oracle_gemm_dgrad", "oracle_gemm_wgrad"):
            fn = getattr(lib, name)
            fn.restype = ci
            fn.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.oracle_stats.restype = ci
        lib.oracle_stats.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp]
        u32p = ctypes.POINTER(ctypes.c_uint32)
        lib.oracle_threefry2x32_20.restype = None
        lib.oracle_threefry2x32_20.argtypes = [u32p, u32p, u32p]
        lib.oracle_sr_byte.restype = ctypes.c_uint
        lib.oracle_sr_byte.argtypes = [ctypes.c_uint64, ctypes.c_uint64]
        lib.oracle_encode_sr_fp4.restype = ctypes.c_uint
        lib.oracle_encode_sr_fp4.argtypes = [dbl, ctypes.c_uint]
        lib.oracle_quantize_sr_fp4.restype = ci
        lib.oracle_quantize_sr_fp4.argtypes = [vp, i64, i64, i64, ci, ci, ctypes.c_uint64, vp, vp]
        lib.oracle_adamw_sensitivity_sq.restype = dbl
        lib.oracle_adamw_sensitivity_sq.argtypes = [vp, vp, vp, i64, dbl, dbl, dbl]
        lib.oracle_weight_divergence.restype = dbl
        lib.oracle_weight_divergence.argtypes = [dbl, dbl, dbl, i64, dbl, dbl, i64, i64]
        lib.oracle_quantize_paper.restype = ci
        lib.oracle_quantize_paper.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, vp]
        lib.oracle_dequantize_paper.restype = ci
        lib.oracle_dequantize_paper.argtypes = [vp, vp, i64, i64, ci, ci, vp]
        lib.oracle_stats_paper.restype = ci
        lib.oracle_stats_paper.argtypes = [vp, i64, i64, i64, ci, ci, vp]
        lib.oracle_round_output.restype = dbl
        lib.oracle_round_output.argtypes = [dbl, ci]
        lib.oracle_output_sum_sq.restype = dbl
        lib.oracle_output_sum_sq.argtypes = [vp, i64, ci]
        lib.oracle_loss_divergence.restype = dbl
        lib.oracle_loss_divergence.argtypes = [dbl, dbl, i64, dbl, dbl, i64, i64]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _bf16_2d(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.uint16)
    if x.ndim != 2:
        raise ValueError("expected a 2-D array of bf16 bit patterns (uint16)")
    return x


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what}: bad argument")


# ---- scalar pieces -------------------------------------------------------------------

def bf16_to_f64(bits: int) -> float:
    return _load().oracle_bf16_to_f64(int(bits) & 0xFFFF)


def decode(fmt: int, code: int) -> float:
    """Value of one element code."""
    return _load().oracle_decode(fmt, int(code))


def fmt_max(fmt: int) -> float:
    return _load().oracle_fmt_max(fmt)


def encode_rne(fmt: int, v: float) -> int:
    """Code of the grid value nearest to v (ties to even mantissa, saturating, sign kept)."""
    return int(_load().oracle_encode_rne(fmt, float(v)))


def scale_byte(fmt: int, rule: int, amax: float) -> int:
    """E8M0 byte of the block scale for a block whose largest magnitude is amax."""
    return int(_load().oracle_scale_byte(fmt, rule, float(amax)))


# ---- tensors -------------------------------------------------------------------------

def stored_shape(rows: int, cols: int, axis: int):
    return (rows, cols) if axis == ROW else (cols, rows)


def quantize(x_bf16_bits, fmt: int, axis: int = ROW, rule: int = NO_OVERFLOW):
    """bf16 bits [rows, cols] -> (codes, scales) in the stored orientation.

    codes: uint8 [SR, SC] (FP8) or [SR, SC//2] (FP4, even element in the low nibble);
    scales: uint8 [SR, SC//32].  (SR, SC) = stored_shape(rows, cols, axis).
    """
    x = _bf16_2d(x_bf16_bits)
    rows, cols = x.shape
    sr, sc = stored_shape(rows, cols, axis)
    codes = np.zeros((sr, sc if fmt == FP8 else sc // 2), dtype=np.uint8)
    scales = np.zeros((sr, sc // TILE), dtype=np.uint8)
    _check(_load().oracle_quantize(_ptr(x), rows, cols, cols, fmt, axis, rule,
                                   _ptr(codes), _ptr(scales)), "quantize")
    return codes, scales


def dequantize(codes, scales, fmt: int) -> np.ndarray:
    """Stored codes + scales -> float64 [SR, SC]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    sr = codes.shape[0]
    sc = codes.shape[1] if fmt == FP8 else codes.shape[1] * 2
    out = np.empty((sr, sc), dtype=np.float64)
    _check(_load().oracle_dequantize(_ptr(codes), _ptr(scales), sr, sc, fmt, _ptr(out)),
           "dequantize")
    return out


def fake_quant(x_bf16_bits, fmt: int, axis: int = ROW, rule: int = NO_OVERFLOW) -> np.ndarray:
    """q(x) as float64 in the source orientation [rows, cols]."""
    x = _bf16_2d(x_bf16_bits)
    rows, cols = x.shape
    out = np.empty((rows, cols), dtype=np.float64)
    _check(_load().oracle_fake_quant(_ptr(x), rows, cols, cols, fmt, axis, rule, _ptr(out)),
           "fake_quant")
    return out


def _f64_2d(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float64)
    if a.ndim != 2:
        raise ValueError("expected a 2-D float64 array")
    return a


def gemm_fwd(Xq, Wq) -> np.ndarray:
    """Y[M,N] = sum_k Xq[m,k] Wq[n,k]."""
    X, W = _f64_2d(Xq), _f64_2d(Wq)
    (M, K), (N, K2) = X.shape, W.shape
    if K != K2:
        raise ValueError("fwd: K mismatch")
    Y = np.empty((M, N), dtype=np.float64)
    _check(_load().oracle_gemm_fwd(_ptr(X), _ptr(W), M, N, K, _ptr(Y)), "gemm_fwd")
    return Y


def gemm_dgrad(dYq, Wq) -> np.ndarray:
    """dX[M,K] = sum_n dYq[m,n] Wq[n,k]."""
    dY, W = _f64_2d(dYq), _f64_2d(Wq)
    (M, N), (N2, K) = dY.shape, W.shape
    if N != N2:
        raise ValueError("dgrad: N mismatch")
    dX = np.empty((M, K), dtype=np.float64)
    _check(_load().oracle_gemm_dgrad(_ptr(dY), _ptr(W), M, N, K, _ptr(dX)), "gemm_dgrad")
    return dX


def gemm_wgrad(dYq, Xq) -> np.ndarray:
    """dW[N,K] = sum_m dYq[m,n] Xq[m,k]."""
    dY, X = _f64_2d(dYq), _f64_2d(Xq)
    (M, N), (M2, K) = dY.shape, X.shape
    if M != M2:
        raise ValueError("wgrad: M mismatch")
    dW = np.empty((N, K), dtype=np.float64)
    _check(_load().oracle_gemm_wgrad(_ptr(dY), _ptr(X), M, N, K, _ptr(dW)), "gemm_wgrad")
    return dW


def stats(x_bf16_bits, axis: int = ROW, rule: int = NO_OVERFLOW, per_line: bool = False):
    """(sum x^2, sum (q4(x)-x)^2, sum (q8(x)-x)^2) as float64[3]; with per_line=True also
    the same sums per stored row, float64 [SR, 3]."""
    x = _bf16_2d(x_bf16_bits)
    rows, cols = x.shape
    sr, _ = stored_shape(rows, cols, axis)
    out = np.zeros(3, dtype=np.float64)
    lines = np.zeros((sr, 3), dtype=np.float64) if per_line else None
    _check(_load().oracle_stats(_ptr(x), rows, cols, cols, axis, rule, _ptr(out),
                                _ptr(lines) if per_line else None), "stats")
    return (out, lines) if per_line else out


OUT_BF16, OUT_FP32 = 0, 1


def round_output(v: float, out_dtype: int = OUT_BF16) -> float:
    """Nearest bf16 (or fp32) value, ties to even."""
    return float(_load().oracle_round_output(float(v), out_dtype))


def output_sum_sq(c, out_dtype: int = OUT_BF16) -> float:
    """Squared Frobenius norm of a GEMM output after rounding every element to the output type."""
    a = np.ascontiguousarray(np.asarray(c, dtype=np.float64))
    return float(_load().oracle_output_sum_sq(_ptr(a), a.size, out_dtype))


def loss_divergence(grad_x_sq: float, err_x_sq: float, M: int, grad_w_sq: float, err_w_sq: float,
                    N: int, K: int) -> float:
    """Loss-divergence estimate of one linear layer from squared Frobenius norms."""
    return float(_load().oracle_loss_divergence(float(grad_x_sq), float(err_x_sq), M,
                                                float(grad_w_sq), float(err_w_sq), N, K))


def threefry2x32_20(ctr, key):
    """Threefry-2x32, 20 rounds: (c0, c1), (k0, k1) -> (x0, x1), all 32-bit."""
    A = ctypes.c_uint32 * 2
    c, k, o = A(*[int(v) & 0xFFFFFFFF for v in ctr]), A(*[int(v) & 0xFFFFFFFF for v in key]), A()
    _load().oracle_threefry2x32_20(c, k, o)
    return int(o[0]), int(o[1])


def sr_byte(seed: int, index: int) -> int:
    """Random byte of stored element `index` under `seed`."""
    return int(_load().oracle_sr_byte(int(seed) & (2 ** 64 - 1), int(index)))


def encode_sr_fp4(v: float, rnd: int) -> int:
    """FP4 code of v (already divided by the block scale) under stochastic rounding with random byte rnd."""
    return int(_load().oracle_encode_sr_fp4(float(v), int(rnd)))


def quantize_sr_fp4(x_bf16_bits, axis: int = ROW, rule: int = NO_OVERFLOW, seed: int = 0):
    """(codes uint8 [SR, SC/2], scales uint8 [SR, SC/32]) with stochastically rounded FP4 elements."""
    x = _bf16_2d(x_bf16_bits)
    rows, cols = x.shape
    sr, sc = stored_shape(rows, cols, axis)
    codes = np.zeros((sr, sc // 2), dtype=np.uint8)
    scales = np.zeros((sr, sc // TILE), dtype=np.uint8)
    _check(_load().oracle_quantize_sr_fp4(_ptr(x), rows, cols, cols, axis, rule, int(seed) & (2 ** 64 - 1),
                                          _ptr(codes), _ptr(scales)), "quantize_sr_fp4")
    return codes, scales


def adamw_sensitivity_sq(m, v, g, beta1: float, beta2: float, eps: float) -> float:
    """Squared Frobenius norm of dh/dg for the AdamW update direction h = m / (sqrt(v) + eps)."""
    a = [np.ascontiguousarray(np.asarray(t, dtype=np.float64)).ravel() for t in (m, v, g)]
    assert a[0].size == a[1].size == a[2].size
    return float(_load().oracle_adamw_sensitivity_sq(_ptr(a[0]), _ptr(a[1]), _ptr(a[2]), a[0].size,
                                                     float(beta1), float(beta2), float(eps)))


def weight_divergence(alpha: float, beta1: float, beta2: float, t: int, sens_sq: float, err_g_sq: float,
                      N: int, K: int) -> float:
    return float(_load().oracle_weight_divergence(float(alpha), float(beta1), float(beta2), int(t),
                                                  float(sens_sq), float(err_g_sq), N, K))


TILE_1x128, BLOCK_128x128 = 1, 128      # group_rows of the paper's two granularities


def quantize_paper(x_bf16_bits, fmt: int, axis: int = ROW, group_rows: int = TILE_1x128):
    """The paper's recipe (real-valued scale FPX_MAX / amax per 1x128 tile or 128x128 block):
    (codes, scales float32 [ceil(SR/group_rows), SC/128]) in the stored orientation."""
    x = _bf16_2d(x_bf16_bits)
    rows, cols = x.shape
    sr, sc = stored_shape(rows, cols, axis)
    codes = np.zeros((sr, sc if fmt == FP8 else sc // 2), dtype=np.uint8)
    scales = np.zeros(((sr + group_rows - 1) // group_rows, sc // 128), dtype=np.float32)
    _check(_load().oracle_quantize_paper(_ptr(x), rows, cols, cols, fmt, axis, group_rows, _ptr(codes), _ptr(scales)),
           "quantize_paper")
    return codes, scales


def dequantize_paper(codes, scales, fmt: int, group_rows: int = TILE_1x128) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    sr = codes.shape[0]
    sc = codes.shape[1] if fmt == FP8 else codes.shape[1] * 2
    out = np.empty((sr, sc), dtype=np.float64)
    _check(_load().oracle_dequantize_paper(_ptr(codes), _ptr(scales), sr, sc, fmt, group_rows, _ptr(out)), "dequantize_paper")
    return out


def stats_paper(x_bf16_bits, axis: int = ROW, group_rows: int = TILE_1x128) -> np.ndarray:
    """(sum x^2, sum (q4(x)-x)^2, sum (q8(x)-x)^2) under the paper's recipe."""
    x = _bf16_2d(x_bf16_bits)
    rows, cols = x.shape
    out = np.zeros(3, dtype=np.float64)
    _check(_load().oracle_stats_paper(_ptr(x), rows, cols, cols, axis, group_rows, _ptr(out)), "stats_paper")
    return out
