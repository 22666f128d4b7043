"""ctypes binding of the C-ABI library declared in include/snip.h.

Argument marshalling only: every step of the path runs in the library's HIP kernels.  PyTorch
is used for device memory and for the current stream, nothing else.  There is no fallback: if
the library has not been built, the first call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsnip_hip.so")

FP8, FP4 = 0, 1
ROW, COL = 0, 1
NO_OVERFLOW, OCP_FLOOR = 0, 1
OUT_BF16, OUT_FP32 = 0, 1

EXPORTS = ("snip_qtensor_code_bytes", "snip_qtensor_scale_bytes", "snip_qtensor_scale_g4_bytes",
           "snip_workspace_bytes",
           "snip_quantize", "snip_gemm_fwd", "snip_gemm_dgrad", "snip_gemm_wgrad",
           "snip_quant_error_stats", "snip_status_string",
           "snip_gemm_workspace_bytes", "snip_gemm_fwd_norm", "snip_gemm_dgrad_norm", "snip_gemm_wgrad_norm",
           "snip_loss_divergence", "snip_quantize_sr_fp4", "snip_quantize_both", "snip_adamw_sensitivity", "snip_weight_divergence",
           "snip_paper_scale_bytes", "snip_paper_workspace_bytes", "snip_quantize_paper",
           "snip_quant_error_stats_paper", "snip_gemm_paper", "snip_quant_error_stats_both",
           "snip_noalloc_max_cols", "snip_quant_error_stats_noalloc")


class _PTensorC(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("rows", ctypes.c_int64),
                ("cols", ctypes.c_int64), ("fmt", ctypes.c_int32), ("group", ctypes.c_int32)]


class SnipError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _lib().snip_status_string(status).decode()
        super().__init__(f"{where}: {msg} (status {status})")


class _QTensorC(ctypes.Structure):
    _fields_ = [("codes", ctypes.c_void_p), ("scales", ctypes.c_void_p), ("scales_g4", ctypes.c_void_p),
                ("rows", ctypes.c_int64), ("cols", ctypes.c_int64), ("fmt", ctypes.c_int32)]


class _PlanC(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("fwd_x", "fwd_w", "dgrad_dy", "dgrad_w", "wgrad_dy", "wgrad_x")]


_handle = None


def _lib():
    global _handle
    if _handle is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2602_01410_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        i64, vp, ci, sz = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        lib.snip_qtensor_code_bytes.restype = sz
        lib.snip_qtensor_code_bytes.argtypes = [i64, i64, ci]
        lib.snip_qtensor_scale_bytes.restype = sz
        lib.snip_qtensor_scale_bytes.argtypes = [i64, i64]
        lib.snip_qtensor_scale_g4_bytes.restype = sz
        lib.snip_qtensor_scale_g4_bytes.argtypes = [i64, i64]
        lib.snip_workspace_bytes.restype = sz
        lib.snip_workspace_bytes.argtypes = [i64, i64]
        lib.snip_quantize.restype = ci
        lib.snip_quantize.argtypes = [vp, i64, i64, i64, ci, ci, ci, ctypes.POINTER(_QTensorC), vp, vp, sz, vp]
        for name in ("snip_gemm_fwd", "snip_gemm_dgrad", "snip_gemm_wgrad"):
            fn = getattr(lib, name)
            fn.restype = ci
            fn.argtypes = [ctypes.POINTER(_PlanC), ctypes.POINTER(_QTensorC), ctypes.POINTER(_QTensorC),
                           vp, i64, ci, vp, sz, vp]
        lib.snip_quantize_both.restype = ci
        lib.snip_quantize_both.argtypes = [vp, i64, i64, i64, ci, ctypes.POINTER(_QTensorC), ctypes.POINTER(_QTensorC),
                                           vp, vp, ci, vp, ctypes.c_size_t, vp]
        lib.snip_quantize_sr_fp4.restype = ci
        lib.snip_quantize_sr_fp4.argtypes = [vp, i64, i64, i64, ci, ci, ctypes.c_uint64, ctypes.POINTER(_QTensorC), vp]
        lib.snip_paper_scale_bytes.restype = sz
        lib.snip_paper_scale_bytes.argtypes = [i64, i64, ci]
        lib.snip_paper_workspace_bytes.restype = sz
        lib.snip_paper_workspace_bytes.argtypes = [i64, i64]
        lib.snip_quantize_paper.restype = ci
        lib.snip_quantize_paper.argtypes = [vp, i64, i64, i64, ci, ci, ci, vp, vp, vp]
        lib.snip_quant_error_stats_paper.restype = ci
        lib.snip_quant_error_stats_paper.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp, sz, vp]
        lib.snip_gemm_paper.restype = ci
        lib.snip_gemm_paper.argtypes = [ctypes.POINTER(_PTensorC), ctypes.POINTER(_PTensorC), vp, i64, ci, vp]
        cf, cd = ctypes.c_float, ctypes.c_double
        lib.snip_adamw_sensitivity.restype = ci
        lib.snip_adamw_sensitivity.argtypes = [vp, vp, vp, ci, i64, cf, cf, cf, vp, vp, sz, vp]
        lib.snip_weight_divergence.restype = cd
        lib.snip_weight_divergence.argtypes = [cd, cd, cd, i64, cd, cd, i64, i64]
        lib.snip_gemm_workspace_bytes.restype = sz
        lib.snip_gemm_workspace_bytes.argtypes = [i64, i64]
        for name in ("snip_gemm_fwd_norm", "snip_gemm_dgrad_norm", "snip_gemm_wgrad_norm"):
            fn = getattr(lib, name)
            fn.restype = ci
            fn.argtypes = [ctypes.POINTER(_PlanC), ctypes.POINTER(_QTensorC), ctypes.POINTER(_QTensorC),
                           vp, i64, ci, vp, vp, sz, vp]
        lib.snip_loss_divergence.restype = ctypes.c_double
        lib.snip_loss_divergence.argtypes = [ctypes.c_double, ctypes.c_double, i64, ctypes.c_double, ctypes.c_double, i64, i64]
        lib.snip_quant_error_stats.restype = ci
        lib.snip_quant_error_stats.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp, vp, sz, vp]
        lib.snip_quant_error_stats_both.restype = ci
        lib.snip_quant_error_stats_both.argtypes = [vp, i64, i64, i64, ci, vp, vp, vp, sz, vp]
        lib.snip_noalloc_max_cols.restype = sz
        lib.snip_noalloc_max_cols.argtypes = []
        lib.snip_quant_error_stats_noalloc.restype = ci
        lib.snip_quant_error_stats_noalloc.argtypes = [vp, i64, i64, i64, ci, ci, vp, vp, vp]
        lib.snip_status_string.restype = ctypes.c_char_p
        lib.snip_status_string.argtypes = [ci]
        _handle = lib
    return _handle


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _alloc_on(stream):
    """Context for the temporaries a wrapper allocates itself (outputs, workspaces): they must belong to the stream
    the kernels run on, or the caching allocator may hand them to other work of the current stream while the kernels
    still use them.  A torch stream is entered; a raw stream handle other than the current stream's cannot be
    (torch cannot allocate on it), so such callers pass every buffer themselves."""
    import contextlib
    if stream is None:
        return contextlib.nullcontext()
    if isinstance(stream, torch.cuda.Stream):
        return torch.cuda.stream(stream)
    if int(stream) != torch.cuda.current_stream().cuda_stream:
        raise ValueError("a raw stream handle that is not the current torch stream was given and a buffer would have to be "
                         "allocated: pass out / workspace / statistics buffers explicitly, or pass a torch.cuda.Stream")
    return contextlib.nullcontext()


def _check(status: int, where: str):
    if status != 0:
        raise SnipError(status, where)


@dataclass
class QTensor:
    """A quantized matrix in its stored orientation (cols = contraction extent)."""
    codes: torch.Tensor      # uint8 [rows, cols] (FP8) or [rows, cols // 2] (FP4)
    scales: torch.Tensor     # uint8 [rows, cols // 32]
    rows: int
    cols: int
    fmt: int
    scales_g4: Optional[torch.Tensor] = None   # uint8 [ceil(cols / 128), rows_pad, 4]: grouped copy for the GEMMs

    def c_struct(self) -> _QTensorC:
        return _QTensorC(self.codes.data_ptr(), self.scales.data_ptr(),
                         self.scales_g4.data_ptr() if self.scales_g4 is not None else None,
                         self.rows, self.cols, self.fmt)


def code_bytes(rows: int, cols: int, fmt: int) -> int:
    return _lib().snip_qtensor_code_bytes(rows, cols, fmt)


def scale_bytes(rows: int, cols: int) -> int:
    return _lib().snip_qtensor_scale_bytes(rows, cols)


def scale_g4_bytes(rows: int, cols: int) -> int:
    return _lib().snip_qtensor_scale_g4_bytes(rows, cols)


def workspace_bytes(rows: int, cols: int) -> int:
    return _lib().snip_workspace_bytes(rows, cols)


def alloc_qtensor(rows: int, cols: int, fmt: int, device="cuda", grouped_scales: bool = True) -> QTensor:
    cb = cols if fmt == FP8 else cols // 2
    g4 = None
    if grouped_scales:
        rows_pad = scale_g4_bytes(rows, cols) // (4 * max(1, (cols + 127) // 128)) if cols else 0
        g4 = torch.empty(((cols + 127) // 128, rows_pad, 4), dtype=torch.uint8, device=device)
    return QTensor(torch.empty((rows, cb), dtype=torch.uint8, device=device),
                   torch.empty((rows, cols // 32), dtype=torch.uint8, device=device), rows, cols, fmt, g4)


def alloc_workspace(rows: int, cols: int, device="cuda") -> torch.Tensor:
    return torch.empty(workspace_bytes(rows, cols), dtype=torch.uint8, device=device)


def alloc_stats(device="cuda") -> torch.Tensor:
    """One snip_stats: float64 [3] = (sum_sq, err_sq_fp4, err_sq_fp8)."""
    return torch.empty(3, dtype=torch.float64, device=device)


def make_plan(entry: Sequence[int]) -> _PlanC:
    return _PlanC(*[int(v) for v in entry])


def _src(x: torch.Tensor):
    if x.dim() != 2 or x.element_size() != 2 or not x.is_cuda:
        raise ValueError("expected a 2-D CUDA tensor of bf16 (or its uint16/int16 bit patterns)")
    if x.stride(1) != 1:
        raise ValueError("rows must be contiguous")
    return x.data_ptr(), x.shape[0], x.shape[1], x.stride(0)


def snip_quantize(x: torch.Tensor, fmt: int, axis: int = ROW, rule: int = NO_OVERFLOW,
                  out: Optional[QTensor] = None, stats: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None) -> QTensor:
    ptr, rows, cols, ld = _src(x)
    if out is None or (stats is not None and workspace is None):
        with _alloc_on(stream):
            if out is None:
                sr, sc = (rows, cols) if axis == ROW else (cols, rows)
                out = alloc_qtensor(sr, sc, fmt, x.device)
            if stats is not None and workspace is None:
                workspace = alloc_workspace(rows, cols, x.device)
    q = out.c_struct()
    _check(_lib().snip_quantize(ptr, rows, cols, ld, fmt, axis, rule, ctypes.byref(q),
                                stats.data_ptr() if stats is not None else None,
                                workspace.data_ptr() if workspace is not None else None,
                                workspace.numel() if workspace is not None else 0, _stream(stream)),
           "snip_quantize")
    return out


def snip_quantize_both(x: torch.Tensor, fmt_row: int, fmt_col: int, rule: int = NO_OVERFLOW,
                       out_row: Optional[QTensor] = None, out_col: Optional[QTensor] = None,
                       stats_row: Optional[torch.Tensor] = None, stats_col: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream=None, both_formats: bool = False):
    """Row-block and column-block quantization of x from one read; returns (out_row, out_col).  With statistics
    outputs and both_formats=True they receive the error sums of both formats, not only of the ones written."""
    ptr, rows, cols, ld = _src(x)
    if out_row is None or out_col is None or (stats_row is not None and workspace is None):
        with _alloc_on(stream):
            if out_row is None:
                out_row = alloc_qtensor(rows, cols, fmt_row, x.device)
            if out_col is None:
                out_col = alloc_qtensor(cols, rows, fmt_col, x.device)
            if stats_row is not None and workspace is None:
                workspace = alloc_workspace(rows, cols, x.device)
    qr, qc = out_row.c_struct(), out_col.c_struct()
    _check(_lib().snip_quantize_both(ptr, rows, cols, ld, rule, ctypes.byref(qr), ctypes.byref(qc),
                                     stats_row.data_ptr() if stats_row is not None else None,
                                     stats_col.data_ptr() if stats_col is not None else None,
                                     1 if both_formats else 0,
                                     workspace.data_ptr() if workspace is not None else None,
                                     workspace.numel() if workspace is not None else 0, _stream(stream)),
           "snip_quantize_both")
    return out_row, out_col


def snip_quantize_sr_fp4(x: torch.Tensor, axis: int = ROW, rule: int = NO_OVERFLOW, seed: int = 0,
                         out: Optional[QTensor] = None, stream=None) -> QTensor:
    """FP4 quantization with stochastic rounding; `seed` (64 bit) selects the random byte stream."""
    ptr, rows, cols, ld = _src(x)
    if out is None:
        with _alloc_on(stream):
            sr, sc = (rows, cols) if axis == ROW else (cols, rows)
            out = alloc_qtensor(sr, sc, FP4, x.device)
    q = out.c_struct()
    _check(_lib().snip_quantize_sr_fp4(ptr, rows, cols, ld, axis, rule, int(seed) & (2 ** 64 - 1), ctypes.byref(q),
                                       _stream(stream)), "snip_quantize_sr_fp4")
    return out


TILE_1x128, BLOCK_128x128 = 1, 128


def snip_quantize_paper(x: torch.Tensor, fmt: int, axis: int = ROW, group: int = TILE_1x128, stream=None):
    """The paper's recipe: returns (codes uint8 [SR, SC or SC/2], scales float32 [SR or ceil(SR/128), SC/128])."""
    ptr, rows, cols, ld = _src(x)
    sr, sc = (rows, cols) if axis == ROW else (cols, rows)
    nbytes = int(_lib().snip_paper_scale_bytes(sr, sc, group))
    with _alloc_on(stream):
        codes = torch.empty((sr, sc if fmt == FP8 else sc // 2), dtype=torch.uint8, device=x.device)
        scales = torch.empty((nbytes // 4 // max(1, sc // 128), sc // 128) if sc >= 128 else (0, 0), dtype=torch.float32,
                             device=x.device)
    _check(_lib().snip_quantize_paper(ptr, rows, cols, ld, fmt, axis, group, codes.data_ptr() if codes.numel() else None,
                                      scales.data_ptr() if scales.numel() else None, _stream(stream)), "snip_quantize_paper")
    return codes, scales


def snip_quant_error_stats_both(x: torch.Tensor, rule: int = NO_OVERFLOW, out_row: Optional[torch.Tensor] = None,
                                out_col: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                                stream=None):
    """Statistics for both block directions from one read; returns (out_row, out_col)."""
    ptr, rows, cols, ld = _src(x)
    if out_row is None or out_col is None or workspace is None:
        with _alloc_on(stream):
            if out_row is None:
                out_row = alloc_stats(x.device)
            if out_col is None:
                out_col = alloc_stats(x.device)
            if workspace is None:
                workspace = alloc_workspace(rows, cols, x.device)
    _check(_lib().snip_quant_error_stats_both(ptr, rows, cols, ld, rule, out_row.data_ptr(), out_col.data_ptr(),
                                              workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "snip_quant_error_stats_both")
    return out_row, out_col


def snip_gemm_paper(a_codes, a_scales, a_fmt, a_group, b_codes, b_scales, b_fmt, b_group, out=None,
                    out_dtype=OUT_BF16, stream=None) -> torch.Tensor:
    """C = dequant(A) dequant(B)^T for operands from snip_quantize_paper (stored orientation, uint8 codes)."""
    def pt(codes, scales, fmt, group):
        rows = codes.shape[0]
        cols = codes.shape[1] if fmt == FP8 else codes.shape[1] * 2
        return _PTensorC(codes.data_ptr() if codes.numel() else None, scales.data_ptr() if scales.numel() else None,
                         rows, cols, fmt, group)
    pa, pb = pt(a_codes, a_scales, a_fmt, a_group), pt(b_codes, b_scales, b_fmt, b_group)
    if out is None:
        with _alloc_on(stream):
            out = torch.empty((pa.rows, pb.rows), dtype=torch.bfloat16 if out_dtype == OUT_BF16 else torch.float32,
                              device=a_codes.device)
    _check(_lib().snip_gemm_paper(ctypes.byref(pa), ctypes.byref(pb), out.data_ptr(), out.stride(0), out_dtype,
                                  _stream(stream)), "snip_gemm_paper")
    return out


def snip_quant_error_stats_paper(x: torch.Tensor, axis: int = ROW, group: int = TILE_1x128,
                                 out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                                 stream=None) -> torch.Tensor:
    ptr, rows, cols, ld = _src(x)
    if out is None or workspace is None:
        with _alloc_on(stream):
            if out is None:
                out = alloc_stats(x.device)
            if workspace is None:
                workspace = torch.empty(int(_lib().snip_paper_workspace_bytes(rows, cols)), dtype=torch.uint8, device=x.device)
    _check(_lib().snip_quant_error_stats_paper(ptr, rows, cols, ld, axis, group, out.data_ptr(), workspace.data_ptr(),
                                               workspace.numel(), _stream(stream)), "snip_quant_error_stats_paper")
    return out


def snip_adamw_sensitivity(m: torch.Tensor, v: torch.Tensor, g: torch.Tensor, beta1: float, beta2: float,
                           eps: float, out: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Squared Frobenius norm of dh/dg of the AdamW update direction; m, v fp32, g fp32 or bf16, contiguous."""
    assert m.dtype == torch.float32 and v.dtype == torch.float32 and g.dtype in (torch.float32, torch.bfloat16)
    assert m.is_contiguous() and v.is_contiguous() and g.is_contiguous() and m.numel() == v.numel() == g.numel()
    if out is None or workspace is None:
        with _alloc_on(stream):
            if out is None:
                out = torch.empty(1, dtype=torch.float64, device=m.device)
            if workspace is None:
                workspace = alloc_workspace(0, 0, m.device)
    n = m.numel()
    _check(_lib().snip_adamw_sensitivity(m.data_ptr() if n else None, v.data_ptr() if n else None,
                                         g.data_ptr() if n else None,
                                         OUT_BF16 if g.dtype == torch.bfloat16 else OUT_FP32, n,
                                         float(beta1), float(beta2), float(eps), out.data_ptr(),
                                         workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "snip_adamw_sensitivity")
    return out


def snip_weight_divergence(alpha: float, beta1: float, beta2: float, t: int, sens_sq: float, err_g_sq: float,
                           n: int, k: int) -> float:
    return float(_lib().snip_weight_divergence(float(alpha), float(beta1), float(beta2), int(t), float(sens_sq),
                                               float(err_g_sq), n, k))


def _gemm(fn_name: str, plan, a: QTensor, b: QTensor, out, out_dtype, stream):
    if not isinstance(plan, _PlanC):
        plan = make_plan(plan)
    if out is None:
        with _alloc_on(stream):
            out = torch.empty((a.rows, b.rows), dtype=torch.bfloat16 if out_dtype == OUT_BF16 else torch.float32,
                              device=a.codes.device)
    qa, qb = a.c_struct(), b.c_struct()
    _check(getattr(_lib(), fn_name)(ctypes.byref(plan), ctypes.byref(qa), ctypes.byref(qb), out.data_ptr(),
                                    out.stride(0), out_dtype, None, 0, _stream(stream)), fn_name)
    return out


def gemm_workspace_bytes(out_rows: int, out_cols: int) -> int:
    return int(_lib().snip_gemm_workspace_bytes(out_rows, out_cols))


def _gemm_norm(fn_name, plan, a: QTensor, b: QTensor, out, out_dtype, sum_sq, workspace, stream):
    if not isinstance(plan, _PlanC):
        plan = make_plan(plan)
    dt = torch.bfloat16 if out_dtype == OUT_BF16 else torch.float32
    if out is None or sum_sq is None or workspace is None:
        with _alloc_on(stream):
            if out is None:
                out = torch.empty((a.rows, b.rows), dtype=dt, device=a.codes.device)
            if sum_sq is None:
                sum_sq = torch.empty(1, dtype=torch.float64, device=a.codes.device)
            if workspace is None:
                workspace = torch.empty(gemm_workspace_bytes(a.rows, b.rows), dtype=torch.uint8, device=a.codes.device)
    qa, qb = a.c_struct(), b.c_struct()
    _check(getattr(_lib(), fn_name)(ctypes.byref(plan), ctypes.byref(qa), ctypes.byref(qb),
                                    out.data_ptr(), out.stride(0), out_dtype, sum_sq.data_ptr(), workspace.data_ptr(),
                                    workspace.numel(), _stream(stream)), fn_name)
    return out, sum_sq


def snip_gemm_fwd_norm(plan, xq_row: QTensor, wq_row: QTensor, out=None, out_dtype=OUT_BF16, sum_sq=None,
                       workspace=None, stream=None):
    """snip_gemm_fwd plus the squared Frobenius norm of Y as stored; returns (Y, sum_sq float64[1])."""
    return _gemm_norm("snip_gemm_fwd_norm", plan, xq_row, wq_row, out, out_dtype, sum_sq, workspace, stream)


def snip_gemm_dgrad_norm(plan, dyq_row: QTensor, wq_col: QTensor, out=None, out_dtype=OUT_BF16, sum_sq=None,
                         workspace=None, stream=None):
    return _gemm_norm("snip_gemm_dgrad_norm", plan, dyq_row, wq_col, out, out_dtype, sum_sq, workspace, stream)


def snip_gemm_wgrad_norm(plan, dyq_col: QTensor, xq_col: QTensor, out=None, out_dtype=OUT_BF16, sum_sq=None,
                         workspace=None, stream=None):
    return _gemm_norm("snip_gemm_wgrad_norm", plan, dyq_col, xq_col, out, out_dtype, sum_sq, workspace, stream)


def snip_loss_divergence(grad_x_sq: float, err_x_sq: float, m: int, grad_w_sq: float, err_w_sq: float,
                         n: int, k: int) -> float:
    return float(_lib().snip_loss_divergence(float(grad_x_sq), float(err_x_sq), m, float(grad_w_sq),
                                             float(err_w_sq), n, k))


def snip_gemm_fwd(plan, xq_row: QTensor, wq_row: QTensor, out=None, out_dtype=OUT_BF16, stream=None):
    """Y[M,N] from quantize(X, ROW) and quantize(W, ROW)."""
    return _gemm("snip_gemm_fwd", plan, xq_row, wq_row, out, out_dtype, stream)


def snip_gemm_dgrad(plan, dyq_row: QTensor, wq_col: QTensor, out=None, out_dtype=OUT_BF16, stream=None):
    """dX[M,K] from quantize(dY, ROW) and quantize(W, COL)."""
    return _gemm("snip_gemm_dgrad", plan, dyq_row, wq_col, out, out_dtype, stream)


def snip_gemm_wgrad(plan, dyq_col: QTensor, xq_col: QTensor, out=None, out_dtype=OUT_BF16, stream=None):
    """dW[N,K] from quantize(dY, COL) and quantize(X, COL)."""
    return _gemm("snip_gemm_wgrad", plan, dyq_col, xq_col, out, out_dtype, stream)


def snip_quant_error_stats(x: torch.Tensor, axis: int = ROW, rule: int = NO_OVERFLOW,
                           out: Optional[torch.Tensor] = None, per_line: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    ptr, rows, cols, ld = _src(x)
    if out is None or workspace is None:
        with _alloc_on(stream):
            if out is None:
                out = alloc_stats(x.device)
            if workspace is None:
                workspace = alloc_workspace(rows, cols, x.device)
    _check(_lib().snip_quant_error_stats(ptr, rows, cols, ld, axis, rule, out.data_ptr(),
                                         per_line.data_ptr() if per_line is not None else None,
                                         workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "snip_quant_error_stats")
    return out


def snip_quant_error_stats_noalloc(x: torch.Tensor, axis: int, rule: int, out: torch.Tensor,
                                   per_line: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """snip_quant_error_stats on the library's resident scratch array: the binding allocates nothing either, so
    `out` (and `per_line`, if wanted) must be passed in."""
    ptr, rows, cols, ld = _src(x)
    _check(_lib().snip_quant_error_stats_noalloc(ptr, rows, cols, ld, axis, rule, out.data_ptr(),
                                                 per_line.data_ptr() if per_line is not None else None,
                                                 _stream(stream)), "snip_quant_error_stats_noalloc")
    return out
