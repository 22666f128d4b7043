/*
 * snip.h -- C ABI of the MI355X (gfx950) library for the quantized linear-layer hot path
 * of SNIP (arXiv 2602.01410).
 *
 * The library implements what runs on every GPU in every training step of a mixed-precision
 * linear layer (paper Sec. 2.2, Fig. "mixed precision training"): the inputs, weights and
 * output gradients are quantized to FP8 or FP4 before each of the three GEMMs
 *     forward      Y [M,N] = X [M,K] * W[N,K]^T
 *     data grad    dX[M,K] = dY[M,N] * W[N,K]
 *     weight grad  dW[N,K] = dY[M,N]^T * X[M,K]
 * (shapes as in Sec. 4.1 / 4.3.1), the GEMM output stays in BF16, and the Frobenius norms of
 * the tensors and of their quantization error are collected (Sec. 3.1, Step 1) as input to
 * the loss- and weight-divergence estimates of Sec. 4.  Which format each operand uses is the
 * per-layer decision of the paper's ILP (Sec. 4.2); here it arrives as a snip_layer_plan.
 *
 * Quantization (Sec. 2.3): every group of 32 consecutive elements along the contraction
 * dimension of the consuming GEMM shares one power-of-two scale 2^e stored as an E8M0 byte
 * (value 2^(byte-127)); elements are FP8 E4M3 (no infinities, max 448) or FP4 E2M1 (max 6),
 * rounded to nearest with ties to the even mantissa.  This is the paper's
 * "scale = FPX_MAX / max|x|" with the scale restricted to a power of two.
 *
 * General conventions
 *  - Every pointer argument marked "device" is GPU memory owned by the caller; the library
 *    never allocates, frees or keeps a pointer, and holds no global state.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All work is
 *    enqueued on it; no call synchronizes.  Outputs are valid once the stream has reached
 *    the end of the call.
 *  - Arguments are validated on the host before anything is launched: a call that returns
 *    an error has had no effect.  Errors are reported by return code only.
 *  - Calls are re-entrant; calls on different streams may overlap if their outputs and
 *    workspaces do not.
 *  - Blocks that contain an infinity or a NaN get scale byte 0xFF and all-zero codes; no
 *    error is raised for them.
 */
#ifndef SNIP_H
#define SNIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SNIP_OK = 0,
    SNIP_ERR_NULL = 1,       /* a required pointer is NULL */
    SNIP_ERR_SHAPE = 2,      /* negative extent, blocked extent not a multiple of 32, ld too small */
    SNIP_ERR_FORMAT = 3,     /* unknown enum value, or an operand's format differs from the plan */
    SNIP_ERR_LAYOUT = 4,     /* misaligned pointer / leading dimension, operands' contraction extents differ */
    SNIP_ERR_WORKSPACE = 5,  /* workspace missing or too small */
    SNIP_ERR_HIP = 6         /* a kernel launch failed */
} snip_status;

typedef enum { SNIP_FP8_E4M3 = 0, SNIP_FP4_E2M1 = 1 } snip_fmt;

/* Direction of the 32-element blocks in the SOURCE matrix. */
typedef enum {
    SNIP_AXIS_ROW = 0,       /* along a row (contiguous elements); stored matrix = source */
    SNIP_AXIS_COL = 1        /* down a column; stored matrix = transpose of the source */
} snip_axis;

/* How the power-of-two scale 2^e is derived from the block maximum amax = m * 2^n, 1 <= m < 2. */
typedef enum {
    SNIP_SCALE_NO_OVERFLOW = 0, /* smallest 2^e with amax / 2^e <= FPX_MAX (the paper's scale,
                                   rounded so that the block maximum stays representable) */
    SNIP_SCALE_OCP_FLOOR = 1    /* e = n - emax(FPX); elements above FPX_MAX saturate */
} snip_scale_rule;

typedef enum { SNIP_OUT_BF16 = 0, SNIP_OUT_FP32 = 1 } snip_out_dtype;

/* Scaling groups of the paper's own recipe, in the stored orientation. */
typedef enum {
    SNIP_GROUP_TILE_1x128 = 1,      /* 128 consecutive elements of a stored row (activations, gradients) */
    SNIP_GROUP_BLOCK_128x128 = 128  /* 128 stored rows x 128 elements (weights) */
} snip_group;

/* A quantized matrix in its stored orientation: `cols` is the blocked (contraction) extent.
 *   codes : device. FP8: rows*cols bytes, row-major. FP4: rows*cols/2 bytes, row-major, element
 *           2i in the low nibble and 2i+1 in the high nibble of byte i. 16-byte aligned.
 *   scales: device. E8M0 bytes, [rows][cols/32] row-major. 4-byte aligned.
 *   scales_g4: device or NULL.  A second copy of the same scale bytes, grouped for the GEMMs:
 *           [ceil(cols/128)][rows_pad][4], i.e. the four scales of 128 consecutive contraction
 *           elements of a row in one dword, rows contiguous; rows_pad = rows rounded up to a
 *           multiple of 256 (dwords of rows >= `rows`, and bytes of blocks >= cols/32, are
 *           unspecified).  16-byte aligned (the quantize kernels write it with 16-byte stores;
 *           SNIP_ERR_LAYOUT otherwise).  snip_quantize fills it when it is not NULL; when both
 *           operands of a GEMM carry one and cols is a multiple of 128 the GEMM copies its scales
 *           from it with fully coalesced loads, otherwise it falls back to a slower kernel that
 *           gathers from `scales`.  Size: snip_qtensor_scale_g4_bytes.
 *   rows, cols: extents of the stored matrix; cols must be a multiple of 32. */
typedef struct {
    void*    codes;
    uint8_t* scales;
    uint8_t* scales_g4;
    int64_t  rows, cols;
    int32_t  fmt;            /* snip_fmt */
} snip_qtensor;

/* Element format of each operand of each GEMM of one linear layer.  The paper's option set
 * (Sec. 4.2: one format each for inputs, weights, gradients) is the special case
 * fwd_x == wgrad_x, fwd_w == dgrad_w, dgrad_dy == wgrad_dy. */
typedef struct {
    int32_t fwd_x, fwd_w, dgrad_dy, dgrad_w, wgrad_dy, wgrad_x;   /* snip_fmt each */
} snip_layer_plan;

/* Squared Frobenius norms (Sec. 3.1 Step 1): of the tensor, and of q(x) - x for both candidate
 * formats.  A fused quantize call fills sum_sq and the chosen format's field and writes NaN
 * into the other.
 * Range: differences are exact and squares are formed and added per lane in fp32 (wave and
 * workgroup partials in fp32, everything above in double), so the stated 1e-5 relative accuracy
 * holds for tensors whose nonzero magnitudes lie within [2^-56, 2^48]: below, the squares of
 * the errors (about 2^-5 |x| for FP8) leave the fp32 normal range and count as less than they
 * are; above, sums of squares overflow to infinity.  A lane adds at most rows / 64 (column
 * blocks) or cols / 8 (row blocks) groups of 8 squares before its sum moves to the next level,
 * which keeps the rounding of a sum of n equal terms below 1e-5 up to about 2^22 rows. */
typedef struct { double sum_sq, err_sq_fp4, err_sq_fp8; } snip_stats;

/* ---- sizes (host, pure) ------------------------------------------------------------- */

/* Bytes of codes / scales for a stored matrix of rows x cols; 0 on a bad argument. */
size_t snip_qtensor_code_bytes(int64_t rows, int64_t cols, snip_fmt fmt);
size_t snip_qtensor_scale_bytes(int64_t rows, int64_t cols);
size_t snip_qtensor_scale_g4_bytes(int64_t rows, int64_t cols);

/* Workspace (device bytes) sufficient for any call below on a source matrix of at most
 * rows x cols, including per-line statistics. */
size_t snip_workspace_bytes(int64_t rows, int64_t cols);

/* ---- quantize (Sec. 2.3; which tensors: Sec. 2.2) ------------------------------------ */

/* Quantize a bf16 matrix.
 *   x     : device, bf16 [rows][ld], 16-byte aligned; ld >= cols, ld a multiple of 8.
 *   axis  : SNIP_AXIS_ROW: blocks along rows; cols % 32 == 0; out is rows x cols.
 *           SNIP_AXIS_COL: blocks down columns; rows % 32 == 0, cols even; out is stored
 *           transposed, cols x rows, so that it equals quantize(transpose(x), ROW).
 *   out   : host struct whose codes/scales point to device buffers of at least
 *           snip_qtensor_code_bytes / snip_qtensor_scale_bytes; out->rows, out->cols and
 *           out->fmt must already describe the stored matrix and `fmt`.
 *   stats : device or NULL.  If given, the squared norms of x and of the quantization error
 *           of `fmt` are produced by the same pass (then `workspace` is required).
 *   workspace: device, >= snip_workspace_bytes(rows, cols) bytes, 16-byte aligned; may be
 *           NULL when stats is NULL.
 * Column-block calls are worked on by one workgroup per 128-column unit; the environment variable
 * SNIP_QUANT_COL_UNIT=wave|workgroup, read at every call, fixes the work distribution for tests and
 * measurements (codes and scales do not depend on it; fused statistics are summed in another
 * fixed order). */
snip_status snip_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld,
                          snip_fmt fmt, snip_axis axis, snip_scale_rule rule,
                          const snip_qtensor* out, snip_stats* stats,
                          void* workspace, size_t workspace_bytes, void* stream);

/* Which error sums the fused statistics of snip_quantize_both deliver. */
typedef enum { SNIP_STATS_CHOSEN_FORMAT = 0, SNIP_STATS_BOTH_FORMATS = 1 } snip_stats_scope;

/* Both orientations of one tensor from one pass over it (Sec. 2.2: every GEMM input is quantized
 * for two GEMMs that contract different axes, e.g. X along its rows for Y = X W^T and down its
 * columns for dW = dY^T X).  Produces exactly what
 *     snip_quantize(x, ..., out_row->fmt, SNIP_AXIS_ROW, rule, out_row, stats_row, ...) and
 *     snip_quantize(x, ..., out_col->fmt, SNIP_AXIS_COL, rule, out_col, stats_col, ...)
 * produce (codes, scales and grouped scale copies bit for bit; the statistics summed in another
 * fixed order), reading x from HBM once.  The two formats may differ.
 *   rows, cols: both multiples of 32; other arguments as for snip_quantize.
 *   out_row : stored rows x cols;  out_col : stored cols x rows.
 *   stats_row, stats_col: device, both or neither (SNIP_ERR_NULL for just one).
 *   scope   : SNIP_STATS_CHOSEN_FORMAT: as the fused statistics of snip_quantize (the field of the
 *             format not written is NaN).  SNIP_STATS_BOTH_FORMATS: all three fields, i.e. what
 *             snip_quant_error_stats_both delivers, out of the same pass: the complete Step-1
 *             record of a tensor (Sec. 3.1; the ILP needs the error of the option not in use,
 *             Sec. 4.2) together with its two quantized orientations from one read.  Ignored
 *             without statistics outputs.
 * Small tensors are worked on by one workgroup per 128-column unit, large ones by one wave per unit;
 * the environment variable SNIP_QUANT_BOTH_UNIT=wave|workgroup, read at every call, fixes the choice
 * for tests and measurements (codes and scales do not depend on it; the statistics are summed in
 * another fixed order). */
snip_status snip_quantize_both(const void* x, int64_t rows, int64_t cols, int64_t ld,
                               snip_scale_rule rule, const snip_qtensor* out_row,
                               const snip_qtensor* out_col, snip_stats* stats_row,
                               snip_stats* stats_col, snip_stats_scope scope, void* workspace,
                               size_t workspace_bytes, void* stream);

/* Quantize to FP4 with stochastic rounding (Sec. 5.1 "Quantization Format and Implementation":
 * FP4 output gradients are rounded probabilistically to the two nearest values).  Arguments,
 * layout, scales (bit-identical to snip_quantize with SNIP_FP4_E2M1) and error behaviour as for
 * snip_quantize; out->fmt must be SNIP_FP4_E2M1.  The rounding is a pure function of (x, seed):
 *   - element i (row-major position in the STORED matrix) draws the random byte rnd = byte
 *     (i mod 8) of the 64 bits Threefry-2x32-20(counter = i div 8, key = seed) (Salmon et al.,
 *     SC'11; counter and key low word first; output word 0 first, least significant byte first);
 *   - with lo <= |v| <= hi the grid magnitudes next to the scaled element v and
 *     p = (|v| - lo) / (hi - lo), the magnitude becomes hi iff rnd < floor(256 p), else lo.
 * Grid values are kept for every seed; the expectation over rnd equals v exactly for
 * |v| >= 0.25 (p then has at most 8 bits) and lies within 0.5/256 below |v| otherwise.
 * Use a fresh seed per tensor and step. */
snip_status snip_quantize_sr_fp4(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                 snip_axis axis, snip_scale_rule rule, uint64_t seed,
                                 const snip_qtensor* out, void* stream);

/* ---- the three GEMMs (Sec. 2.2; shapes Sec. 4.1 / 4.3.1) ----------------------------- */
/* All three contract the stored `cols` of both operands: C[i][j] = sum_r A[i][r] * B[j][r]
 * with a = code * 2^(scale-127), accumulated in fp32 and rounded once (nearest even) to the
 * output type.  Operands must have equal cols (SNIP_ERR_LAYOUT otherwise) and the formats the
 * plan names for that GEMM (SNIP_ERR_FORMAT otherwise).  The output is row-major with leading
 * dimension ld_out (elements), 16-byte aligned rows.  `workspace` is reserved (may be NULL).
 *
 *   fwd  : Xq  = quantize(X,  ROW) [M,K],  Wq  = quantize(W,  ROW) [N,K]  ->  Y  [M,N]
 *   dgrad: dYq = quantize(dY, ROW) [M,N],  Wq  = quantize(W,  COL) [K,N]  ->  dX [M,K]
 *   wgrad: dYq = quantize(dY, COL) [N,M],  Xq  = quantize(X,  COL) [K,M]  ->  dW [N,K]
 *
 * Every output element sums its products in one fixed order, whichever kernel and workgroup tile
 * the launcher picks for the shape.  The matrix-core kernel has two tiles (256 x 256 and 256 x 128
 * outputs per workgroup); the environment variable SNIP_GEMM_TILE=big|wide, read at every call,
 * fixes the tile for measurements and tests and never changes a result. */
snip_status snip_gemm_fwd(const snip_layer_plan* plan, const snip_qtensor* xq_row,
                          const snip_qtensor* wq_row, void* y, int64_t ld_out,
                          snip_out_dtype out_dtype, void* workspace, size_t workspace_bytes,
                          void* stream);
snip_status snip_gemm_dgrad(const snip_layer_plan* plan, const snip_qtensor* dyq_row,
                            const snip_qtensor* wq_col, void* dx, int64_t ld_out,
                            snip_out_dtype out_dtype, void* workspace, size_t workspace_bytes,
                            void* stream);
snip_status snip_gemm_wgrad(const snip_layer_plan* plan, const snip_qtensor* dyq_col,
                            const snip_qtensor* xq_col, void* dw, int64_t ld_out,
                            snip_out_dtype out_dtype, void* workspace, size_t workspace_bytes,
                            void* stream);

/* ---- GEMMs that also deliver the norm of their output (Sec. 3.1 Step 1) --------------- */
/* Step 1 of the paper collects the Frobenius norms of Y, dX and dW next to those of the GEMM
 * inputs; ||dX|| and ||dW|| are the gradient factors of the loss-divergence estimate (Sec. 4.2
 * "Loss Divergence in Forward Pass").  These variants compute exactly what the plain calls do and,
 * from the same accumulators, the squared Frobenius norm of the output AS STORED (every element
 * rounded to the output type first; elements outside the matrix do not count).
 *   sum_sq   : device, one double.
 *   workspace: device, required, >= snip_gemm_workspace_bytes(out rows, out cols) bytes, 16-byte
 *              aligned, no initialisation needed; calls that overlap in time must not share it.
 * The sum is formed per lane (128 or 64 squares), per wave and per workgroup in fp32 and across
 * workgroups in double, all in a fixed order: results are identical from run to run. */
size_t snip_gemm_workspace_bytes(int64_t out_rows, int64_t out_cols);
snip_status snip_gemm_fwd_norm(const snip_layer_plan* plan, const snip_qtensor* xq_row,
                               const snip_qtensor* wq_row, void* y, int64_t ld_out,
                               snip_out_dtype out_dtype, double* sum_sq, void* workspace,
                               size_t workspace_bytes, void* stream);
snip_status snip_gemm_dgrad_norm(const snip_layer_plan* plan, const snip_qtensor* dyq_row,
                                 const snip_qtensor* wq_col, void* dx, int64_t ld_out,
                                 snip_out_dtype out_dtype, double* sum_sq, void* workspace,
                                 size_t workspace_bytes, void* stream);
snip_status snip_gemm_wgrad_norm(const snip_layer_plan* plan, const snip_qtensor* dyq_col,
                                 const snip_qtensor* xq_col, void* dw, int64_t ld_out,
                                 snip_out_dtype out_dtype, double* sum_sq, void* workspace,
                                 size_t workspace_bytes, void* stream);

/* Host, pure.  The paper's estimate of the loss change caused by quantizing the inputs X [m,k]
 * and weights W [n,k] of one linear layer (Sec. 4.2 "Loss Divergence in Forward Pass"):
 *     sqrt( (||dX|| ||q(X)-X|| / sqrt(m k))^2 + (||dW|| ||q(W)-W|| / sqrt(n k))^2 )
 * from SQUARED Frobenius norms: grad_x_sq / grad_w_sq are the sum_sq of the dgrad / wgrad calls
 * above, err_x_sq / err_w_sq the err_sq_* fields of snip_stats for the format in question.
 * Returns NaN for a non-positive extent or a negative or NaN argument. */
double snip_loss_divergence(double grad_x_sq, double err_x_sq, int64_t m,
                            double grad_w_sq, double err_w_sq, int64_t n, int64_t k);

/* ---- the paper's own quantization recipe (Sec. 2.3, Sec. 5.1) -------------------------- */
/* Sec. 2.3 scales a group by the real number s = FPX_MAX / max|x|, casts x * s to FPX and divides
 * by s afterwards; Sec. 5.1 uses 1x128 tiles for activations and gradients and 128x128 blocks
 * for weights.  These calls implement exactly that, next to the power-of-two 32-element blocks
 * of snip_quantize, so that the error statistics of the paper's configuration can be produced.
 * s and x * s are formed in fp32 (one correctly rounded division, one correctly rounded
 * product), then rounded to nearest even onto the FPX grid, saturating; s = 1 for an all-zero
 * group, s is capped at 2^126, and a group with an infinity or NaN gets s = NaN and zero codes.
 *   x, rows, cols, ld, axis: as for snip_quantize, but the blocked extent (cols for AXIS_ROW,
 *           rows for AXIS_COL) must be a multiple of 128.
 *   codes : device, layout as snip_qtensor.codes (stored orientation), 16-byte aligned.
 *   scales: device, fp32, [stored rows][stored cols / 128] for tiles,
 *           [ceil(stored rows / 128)][stored cols / 128] for blocks; snip_paper_scale_bytes.
 * The codes are consumed by snip_gemm_paper below, not by snip_gemm_fwd/dgrad/wgrad (the matrix
 * instruction applies power-of-two scales to 32-element blocks only). */
size_t snip_paper_scale_bytes(int64_t stored_rows, int64_t stored_cols, snip_group group);
snip_status snip_quantize_paper(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                snip_fmt fmt, snip_axis axis, snip_group group,
                                void* codes, float* scales, void* stream);

/* A matrix quantized by snip_quantize_paper, in its stored orientation (cols = contraction extent,
 * a multiple of 128); scales as that call lays them out for `group`. */
typedef struct {
    const void*  codes;
    const float* scales;
    int64_t      rows, cols;
    int32_t      fmt;      /* snip_fmt */
    int32_t      group;    /* snip_group */
} snip_ptensor;

/* C[i][j] = sum_r (A[i][r] / sa) * (B[j][r] / sb) for operands of that recipe: the real-valued
 * scales are applied in software once per 128-element slab of the contraction (the codes of a
 * slab are multiplied on the matrix cores with unit scales into a fresh fp32 accumulator, which
 * is folded into the result with the factor (1/sa)(1/sb)); fp32 accumulation, one rounding to
 * the output type.  The three GEMMs of a linear layer are this call with the operand pairs
 * listed for snip_gemm_fwd / dgrad / wgrad.  A NaN scale makes the rows or columns it covers NaN.
 * Output layout and alignment as for the other GEMMs. */
snip_status snip_gemm_paper(const snip_ptensor* a, const snip_ptensor* b, void* c, int64_t ld_out,
                            snip_out_dtype out_dtype, void* stream);

/* Squared Frobenius norms of x and of q(x) - x for both formats under that recipe (q(x) = code / s).
 *   out: device, one snip_stats.  workspace: device, required,
 *   >= snip_paper_workspace_bytes(rows, cols), 16-byte aligned. */
size_t snip_paper_workspace_bytes(int64_t rows, int64_t cols);
snip_status snip_quant_error_stats_paper(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                         snip_axis axis, snip_group group, snip_stats* out,
                                         void* workspace, size_t workspace_bytes, void* stream);

/* ---- AdamW factor of the weight-divergence estimate (Sec. 4.3.2) ---------------------- */
/* With m = beta1 m' + (1-beta1) g and v = beta2 v' + (1-beta2) g^2 (the AdamW moments after the
 * step's update) the update direction h(g) = m / (sqrt(v) + eps) has the element-wise derivative
 *     (1-beta1) / (sqrt(v)+eps)  -  (1-beta2) m g / ( sqrt(v) (sqrt(v)+eps)^2 );
 * Step 1 collects the Frobenius norm of that term (Sec. 4.3.2 "Impact on Weight Divergence").
 * This call writes its SQUARE to *sum_sq.
 *   m, v : device, fp32 [n], 16-byte aligned.  Where v is zero the second part counts as zero.
 *   g    : device, [n], fp32 (g_dtype = SNIP_OUT_FP32, 16-byte aligned) or bf16 (SNIP_OUT_BF16,
 *          8-byte aligned; e.g. the dW a wgrad call produced).
 *   beta1, beta2 in [0, 1), eps >= 0 (SNIP_ERR_FORMAT otherwise).
 *   sum_sq: device, one double.  workspace: device, required, >= snip_workspace_bytes(0, 0).
 * fp32 arithmetic with correctly rounded division and square root; fixed summation order. */
snip_status snip_adamw_sensitivity(const float* m, const float* v, const void* g,
                                   snip_out_dtype g_dtype, int64_t n, float beta1, float beta2,
                                   float eps, double* sum_sq, void* workspace,
                                   size_t workspace_bytes, void* stream);

/* Host, pure.  The per-layer weight-divergence estimate the factor feeds (same section):
 *     alpha sqrt(1 - beta2^t) / (1 - beta1^t) * sqrt(sens_sq) * sqrt(err_g_sq) / sqrt(n k)
 * for a weight of n x k elements at optimizer step t >= 1; sens_sq from snip_adamw_sensitivity,
 * err_g_sq the squared Frobenius norm of the perturbation of the weight gradient.  NaN on a
 * bad argument. */
double snip_weight_divergence(double alpha, double beta1, double beta2, int64_t t, double sens_sq,
                              double err_g_sq, int64_t n, int64_t k);

/* ---- quantization-error statistics (Sec. 3.1 Step 1; row-wise form: Sec. 5.3) -------- */

/* One read of a bf16 matrix; for blocks along `axis` produces the squared Frobenius norm of x
 * and of q(x) - x for BOTH formats (the ILP needs the error of options that are not currently
 * selected, Sec. 4.2).
 *   out      : device, one snip_stats.
 *   per_line : device or NULL; float [L][3] = {sum x^2, err^2 fp4, err^2 fp8} for every line of
 *              the stored matrix: L = rows (one per source row) for AXIS_ROW, L = cols (one per
 *              source column) for AXIS_COL.
 *   workspace: device, required, >= snip_workspace_bytes(rows, cols). */
snip_status snip_quant_error_stats(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                   snip_axis axis, snip_scale_rule rule,
                                   snip_stats* out, float* per_line,
                                   void* workspace, size_t workspace_bytes, void* stream);

/* The same statistics for BOTH block directions from one read of the matrix: *out_row is what
 * snip_quant_error_stats(..., SNIP_AXIS_ROW, ...) delivers and *out_col what SNIP_AXIS_COL
 * delivers (to the tolerance of the statistics; the sums are grouped differently).  A tensor's
 * forward operand is blocked along rows and its backward operands down columns (Sec. 2.2), so
 * this is the complete Step-1 record of a tensor.  rows and cols must both be multiples of 32;
 * no per-line sums.  workspace: >= snip_workspace_bytes(rows, cols). */
snip_status snip_quant_error_stats_both(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                        snip_scale_rule rule, snip_stats* out_row,
                                        snip_stats* out_col, void* workspace,
                                        size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory or pass a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): snip_quant_error_stats with its workspace
 * taken from an array that is part of the library's device image (about 24 MiB, resident on every
 * GPU the library is used on until the process ends).  Same arguments, results and error behaviour
 * as snip_quant_error_stats without the workspace pair, except:
 *   - cols must not exceed snip_noalloc_max_cols() (32768): SNIP_ERR_WORKSPACE otherwise;
 *   - the device is the current one (hipGetDevice) and `stream` must belong to it;
 *   - all calls on one GPU share the array: calls that overlap in time on one GPU (different
 *     streams, different threads) race and must be serialized by the caller.  Nothing in the
 *     array has to start at zero; every word a call reads it has written itself.
 * The call allocates nothing and frees nothing; the first call on a device looks up the array's
 * device address (hipGetSymbolAddress), later calls reuse it. */
size_t snip_noalloc_max_cols(void);
snip_status snip_quant_error_stats_noalloc(const void* x, int64_t rows, int64_t cols, int64_t ld,
                                           snip_axis axis, snip_scale_rule rule,
                                           snip_stats* out, float* per_line, void* stream);

const char* snip_status_string(snip_status s);

#ifdef __cplusplus
}
#endif
#endif /* SNIP_H */
