// C-ABI layer: argument validation and dispatch.  No kernel code here.
#include "../../include/snip.h"
#include "snip_internal.h"
#include <cmath>
#include <mutex>

using namespace snip;

// Scratch of snip_quant_error_stats_noalloc: the workspace of the statistics kernels for a source of up to
// kNoallocMaxCols columns, resident on every device the library is used on.  In host code this name is only a
// handle for hipGetSymbolAddress; kernels and launchers get the device address kept in g_scratch_ptr.
constexpr int64_t kNoallocMaxCols = 32768;
constexpr size_t kScratchBytes = stream_workspace_bytes(kNoallocMaxCols);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool valid_fmt(int f) { return f == SNIP_FP8_E4M3 || f == SNIP_FP4_E2M1; }

snip_status check_source(const void* x, int64_t rows, int64_t cols, int64_t ld, int axis, int rule)
{
    if (!x && rows > 0 && cols > 0) return SNIP_ERR_NULL;   // an empty matrix may have no storage
    if (axis != SNIP_AXIS_ROW && axis != SNIP_AXIS_COL) return SNIP_ERR_FORMAT;
    if (rule != SNIP_SCALE_NO_OVERFLOW && rule != SNIP_SCALE_OCP_FLOOR) return SNIP_ERR_FORMAT;
    if (rows < 0 || cols < 0 || ld < cols) return SNIP_ERR_SHAPE;
    if (axis == SNIP_AXIS_ROW && cols % 32 != 0) return SNIP_ERR_SHAPE;
    if (axis == SNIP_AXIS_COL && (rows % 32 != 0 || cols % 2 != 0)) return SNIP_ERR_SHAPE;
    // kernels index work units with 32-bit integers
    if (rows >= (int64_t)1 << 31 || cols >= (int64_t)1 << 31) return SNIP_ERR_SHAPE;
    if ((rows + 31) / 32 * ((cols + 127) / 128) >= (int64_t)1 << 31) return SNIP_ERR_SHAPE;
    if (rows * ((cols + 511) / 512) >= (int64_t)1 << 31) return SNIP_ERR_SHAPE;
    if (!aligned16(x) || ld % 8 != 0) return SNIP_ERR_LAYOUT;
    return SNIP_OK;
}

snip_status check_qtensor(const snip_qtensor* q)
{
    if (!q) return SNIP_ERR_NULL;
    if ((!q->codes || !q->scales) && q->rows > 0) return SNIP_ERR_NULL;      // an empty matrix may have no storage
    if (!valid_fmt(q->fmt)) return SNIP_ERR_FORMAT;
    if (q->rows < 0 || q->cols <= 0 || q->cols % 32 != 0) return SNIP_ERR_SHAPE;
    if (q->rows >= (int64_t)1 << 31 || q->cols >= (int64_t)1 << 31) return SNIP_ERR_SHAPE;
    if (!aligned16(q->codes)) return SNIP_ERR_LAYOUT;
    if (q->scales_g4 && !aligned16(q->scales_g4)) return SNIP_ERR_LAYOUT;      // written with 16-byte stores
    if (reinterpret_cast<uintptr_t>(q->scales) & 3u) return SNIP_ERR_LAYOUT;
    return SNIP_OK;
}

size_t gemm_ws_bytes(int64_t I, int64_t J) { return (size_t)gemm_norm_partials(I, J) * sizeof(float) + 16; }

snip_status gemm(const snip_qtensor* a, int fmt_a, const snip_qtensor* b, int fmt_b, void* c, int64_t ldc,
                 int out_dtype, void* stream, bool want_norm = false, double* sum_sq = nullptr,
                 void* workspace = nullptr, size_t workspace_bytes_ = 0)
{
    snip_status st = check_qtensor(a);
    if (st != SNIP_OK) return st;
    st = check_qtensor(b);
    if (st != SNIP_OK) return st;
    if (!c && a->rows > 0 && b->rows > 0) return SNIP_ERR_NULL;
    if (!valid_fmt(fmt_a) || !valid_fmt(fmt_b)) return SNIP_ERR_FORMAT;
    if (out_dtype != SNIP_OUT_BF16 && out_dtype != SNIP_OUT_FP32) return SNIP_ERR_FORMAT;
    if (a->fmt != fmt_a || b->fmt != fmt_b) return SNIP_ERR_FORMAT;
    if (a->cols != b->cols) return SNIP_ERR_LAYOUT;
    if (ldc < b->rows) return SNIP_ERR_SHAPE;
    if ((a->rows + 127) / 128 * ((b->rows + 127) / 128) >= (int64_t)1 << 31) return SNIP_ERR_SHAPE;
    const int64_t align_elems = out_dtype == SNIP_OUT_BF16 ? 8 : 4;
    if (!aligned16(c) || ldc % align_elems != 0) return SNIP_ERR_LAYOUT;
    GemmArgs g;
    g.a_codes = (const uint8_t*)a->codes; g.a_scales = a->scales; g.a_scales_g4 = a->scales_g4; g.fmt_a = fmt_a;
    g.b_codes = (const uint8_t*)b->codes; g.b_scales = b->scales; g.b_scales_g4 = b->scales_g4; g.fmt_b = fmt_b;
    g.I = a->rows; g.J = b->rows; g.R = a->cols;
    g.c = c; g.ldc = ldc; g.out_fp32 = out_dtype == SNIP_OUT_FP32;
    if (want_norm) {
        if (!sum_sq) return SNIP_ERR_NULL;
        if (!workspace || workspace_bytes_ < gemm_ws_bytes(g.I, g.J)) return SNIP_ERR_WORKSPACE;
        if (!aligned16(workspace)) return SNIP_ERR_LAYOUT;
        g.norm_partials = (float*)workspace;
        g.norm_out = sum_sq;
    }
    return launch_gemm(g, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

}  // namespace

extern "C" {

size_t snip_qtensor_code_bytes(int64_t rows, int64_t cols, snip_fmt fmt)
{
    if (rows < 0 || cols < 0 || cols % 32 != 0 || !valid_fmt(fmt)) return 0;
    const size_t n = (size_t)rows * (size_t)cols;
    return fmt == SNIP_FP8_E4M3 ? n : n / 2;
}

size_t snip_qtensor_scale_bytes(int64_t rows, int64_t cols)
{
    if (rows < 0 || cols < 0 || cols % 32 != 0) return 0;
    return (size_t)rows * (size_t)(cols / 32);
}

size_t snip_qtensor_scale_g4_bytes(int64_t rows, int64_t cols)
{
    if (rows < 0 || cols < 0 || cols % 32 != 0) return 0;
    return (size_t)g4_pitch(rows) * (size_t)((cols + 127) / 128) * 4;
}

size_t snip_workspace_bytes(int64_t rows, int64_t cols)
{
    if (rows < 0 || cols < 0) return 0;
    return workspace_bytes(rows, cols);
}

snip_status snip_quantize(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_fmt fmt, snip_axis axis,
                          snip_scale_rule rule, const snip_qtensor* out, snip_stats* stats, void* workspace,
                          size_t workspace_bytes_, void* stream)
{
    if (!valid_fmt(fmt)) return SNIP_ERR_FORMAT;
    snip_status st = check_source(x, rows, cols, ld, axis, rule);
    if (st != SNIP_OK) return st;
    if (!out) return SNIP_ERR_NULL;
    if ((!out->codes || !out->scales) && rows > 0 && cols > 0) return SNIP_ERR_NULL;
    if (out->fmt != (int32_t)fmt) return SNIP_ERR_FORMAT;
    const int64_t sr = axis == SNIP_AXIS_ROW ? rows : cols, sc = axis == SNIP_AXIS_ROW ? cols : rows;
    if (out->rows != sr || out->cols != sc) return SNIP_ERR_SHAPE;
    if (!aligned16(out->codes)) return SNIP_ERR_LAYOUT;
    if (out->scales_g4 && !aligned16(out->scales_g4)) return SNIP_ERR_LAYOUT;
    if (reinterpret_cast<uintptr_t>(out->scales) & 3u) return SNIP_ERR_LAYOUT;
    if (stats) {
        if (!workspace || workspace_bytes_ < workspace_bytes(rows, cols)) return SNIP_ERR_WORKSPACE;
        if (!aligned16(workspace)) return SNIP_ERR_LAYOUT;
    }
    QuantArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld;
    a.fmt = fmt; a.axis = axis; a.rule = rule;
    a.codes = (uint8_t*)out->codes; a.scales = out->scales; a.scales_g4 = out->scales_g4;
    a.stats = (double*)stats; a.workspace = workspace;
    return launch_quantize(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

snip_status snip_quantize_both(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_scale_rule rule,
                               const snip_qtensor* out_row, const snip_qtensor* out_col, snip_stats* stats_row,
                               snip_stats* stats_col, snip_stats_scope scope, void* workspace, size_t workspace_bytes_,
                               void* stream)
{
    if (scope != SNIP_STATS_CHOSEN_FORMAT && scope != SNIP_STATS_BOTH_FORMATS) return SNIP_ERR_FORMAT;
    // both orientations: every extent constraint of the two single-orientation calls at once
    snip_status st = check_source(x, rows, cols, ld, SNIP_AXIS_ROW, rule);
    if (st == SNIP_OK) st = check_source(x, rows, cols, ld, SNIP_AXIS_COL, rule);
    if (st != SNIP_OK) return st;
    if (!out_row || !out_col) return SNIP_ERR_NULL;
    if ((stats_row == nullptr) != (stats_col == nullptr)) return SNIP_ERR_NULL;
    const snip_qtensor* outs[2] = {out_row, out_col};
    for (int i = 0; i < 2; ++i) {
        const snip_qtensor* o = outs[i];
        if ((!o->codes || !o->scales) && rows > 0 && cols > 0) return SNIP_ERR_NULL;
        if (!valid_fmt((snip_fmt)o->fmt)) return SNIP_ERR_FORMAT;
        if (o->rows != (i == 0 ? rows : cols) || o->cols != (i == 0 ? cols : rows)) return SNIP_ERR_SHAPE;
        if (!aligned16(o->codes)) return SNIP_ERR_LAYOUT;
        if (o->scales_g4 && !aligned16(o->scales_g4)) return SNIP_ERR_LAYOUT;
        if (reinterpret_cast<uintptr_t>(o->scales) & 3u) return SNIP_ERR_LAYOUT;
    }
    if (stats_row) {
        if (!workspace || workspace_bytes_ < workspace_bytes(rows, cols)) return SNIP_ERR_WORKSPACE;
        if (!aligned16(workspace)) return SNIP_ERR_LAYOUT;
    }
    QuantBothArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld; a.rule = rule;
    a.fmt_r = out_row->fmt; a.codes_r = (uint8_t*)out_row->codes; a.scales_r = out_row->scales; a.g4_r = out_row->scales_g4;
    a.fmt_c = out_col->fmt; a.codes_c = (uint8_t*)out_col->codes; a.scales_c = out_col->scales; a.g4_c = out_col->scales_g4;
    a.stats_r = (double*)stats_row; a.stats_c = (double*)stats_col; a.workspace = workspace;
    a.both_formats = scope == SNIP_STATS_BOTH_FORMATS;
    return launch_quantize_both(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

snip_status snip_quantize_sr_fp4(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_axis axis,
                                 snip_scale_rule rule, uint64_t seed, const snip_qtensor* out, void* stream)
{
    snip_status st = check_source(x, rows, cols, ld, axis, rule);
    if (st != SNIP_OK) return st;
    if (!out) return SNIP_ERR_NULL;
    if ((!out->codes || !out->scales) && rows > 0 && cols > 0) return SNIP_ERR_NULL;
    if (out->fmt != (int32_t)SNIP_FP4_E2M1) return SNIP_ERR_FORMAT;
    const int64_t sr = axis == SNIP_AXIS_ROW ? rows : cols, sc = axis == SNIP_AXIS_ROW ? cols : rows;
    if (out->rows != sr || out->cols != sc) return SNIP_ERR_SHAPE;
    if (!aligned16(out->codes)) return SNIP_ERR_LAYOUT;
    if (out->scales_g4 && !aligned16(out->scales_g4)) return SNIP_ERR_LAYOUT;
    if (reinterpret_cast<uintptr_t>(out->scales) & 3u) return SNIP_ERR_LAYOUT;
    QuantArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld;
    a.fmt = SNIP_FP4_E2M1; a.axis = axis; a.rule = rule;
    a.codes = (uint8_t*)out->codes; a.scales = out->scales; a.scales_g4 = out->scales_g4;
    a.stats = nullptr; a.workspace = nullptr;
    a.stochastic = true; a.sr_seed = seed;
    return launch_quantize(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

snip_status snip_gemm_fwd(const snip_layer_plan* plan, const snip_qtensor* xq_row, const snip_qtensor* wq_row,
                          void* y, int64_t ld_out, snip_out_dtype out_dtype, void*, size_t, void* stream)
{
    if (!plan) return SNIP_ERR_NULL;
    return gemm(xq_row, plan->fwd_x, wq_row, plan->fwd_w, y, ld_out, out_dtype, stream);
}

snip_status snip_gemm_dgrad(const snip_layer_plan* plan, const snip_qtensor* dyq_row, const snip_qtensor* wq_col,
                            void* dx, int64_t ld_out, snip_out_dtype out_dtype, void*, size_t, void* stream)
{
    if (!plan) return SNIP_ERR_NULL;
    return gemm(dyq_row, plan->dgrad_dy, wq_col, plan->dgrad_w, dx, ld_out, out_dtype, stream);
}

snip_status snip_gemm_wgrad(const snip_layer_plan* plan, const snip_qtensor* dyq_col, const snip_qtensor* xq_col,
                            void* dw, int64_t ld_out, snip_out_dtype out_dtype, void*, size_t, void* stream)
{
    if (!plan) return SNIP_ERR_NULL;
    return gemm(dyq_col, plan->wgrad_dy, xq_col, plan->wgrad_x, dw, ld_out, out_dtype, stream);
}

size_t snip_gemm_workspace_bytes(int64_t out_rows, int64_t out_cols)
{
    if (out_rows < 0 || out_cols < 0) return 0;
    return gemm_ws_bytes(out_rows, out_cols);
}

snip_status snip_gemm_fwd_norm(const snip_layer_plan* plan, const snip_qtensor* xq_row, const snip_qtensor* wq_row,
                               void* y, int64_t ld_out, snip_out_dtype out_dtype, double* sum_sq, void* workspace,
                               size_t workspace_bytes_, void* stream)
{
    if (!plan) return SNIP_ERR_NULL;
    return gemm(xq_row, plan->fwd_x, wq_row, plan->fwd_w, y, ld_out, out_dtype, stream, true, sum_sq, workspace, workspace_bytes_);
}

snip_status snip_gemm_dgrad_norm(const snip_layer_plan* plan, const snip_qtensor* dyq_row, const snip_qtensor* wq_col,
                                 void* dx, int64_t ld_out, snip_out_dtype out_dtype, double* sum_sq, void* workspace,
                                 size_t workspace_bytes_, void* stream)
{
    if (!plan) return SNIP_ERR_NULL;
    return gemm(dyq_row, plan->dgrad_dy, wq_col, plan->dgrad_w, dx, ld_out, out_dtype, stream, true, sum_sq, workspace, workspace_bytes_);
}

snip_status snip_gemm_wgrad_norm(const snip_layer_plan* plan, const snip_qtensor* dyq_col, const snip_qtensor* xq_col,
                                 void* dw, int64_t ld_out, snip_out_dtype out_dtype, double* sum_sq, void* workspace,
                                 size_t workspace_bytes_, void* stream)
{
    if (!plan) return SNIP_ERR_NULL;
    return gemm(dyq_col, plan->wgrad_dy, xq_col, plan->wgrad_x, dw, ld_out, out_dtype, stream, true, sum_sq, workspace, workspace_bytes_);
}

double snip_loss_divergence(double grad_x_sq, double err_x_sq, int64_t m, double grad_w_sq, double err_w_sq,
                            int64_t n, int64_t k)
{
    if (m <= 0 || n <= 0 || k <= 0 || !(grad_x_sq >= 0.0) || !(err_x_sq >= 0.0) || !(grad_w_sq >= 0.0) || !(err_w_sq >= 0.0))
        return std::nan("");
    // each term is a product of two Frobenius norms over the square root of the element count
    const double tx = std::sqrt(grad_x_sq * err_x_sq / ((double)m * (double)k));
    const double tw = std::sqrt(grad_w_sq * err_w_sq / ((double)n * (double)k));
    return std::hypot(tx, tw);
}

static snip_status check_paper(const void* x, int64_t rows, int64_t cols, int64_t ld, int axis, int group)
{
    snip_status st = check_source(x, rows, cols, ld, axis, SNIP_SCALE_NO_OVERFLOW);
    if (st != SNIP_OK) return st;
    if (group != SNIP_GROUP_TILE_1x128 && group != SNIP_GROUP_BLOCK_128x128) return SNIP_ERR_FORMAT;
    if ((axis == SNIP_AXIS_ROW ? cols : rows) % 128 != 0) return SNIP_ERR_SHAPE;
    return SNIP_OK;
}

size_t snip_paper_scale_bytes(int64_t stored_rows, int64_t stored_cols, snip_group group)
{
    if (stored_rows < 0 || stored_cols < 0 || stored_cols % 128 != 0) return 0;
    if (group != SNIP_GROUP_TILE_1x128 && group != SNIP_GROUP_BLOCK_128x128) return 0;
    const int64_t gr = group == SNIP_GROUP_TILE_1x128 ? stored_rows : (stored_rows + 127) / 128;
    return (size_t)gr * (size_t)(stored_cols / 128) * sizeof(float);
}

size_t snip_paper_workspace_bytes(int64_t rows, int64_t cols)
{
    if (rows < 0 || cols < 0) return 0;
    return paper_workspace_bytes(rows, cols);
}

snip_status snip_quantize_paper(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_fmt fmt, snip_axis axis,
                                snip_group group, void* codes, float* scales, void* stream)
{
    if (!valid_fmt(fmt)) return SNIP_ERR_FORMAT;
    snip_status st = check_paper(x, rows, cols, ld, axis, group);
    if (st != SNIP_OK) return st;
    if ((!codes || !scales) && rows > 0 && cols > 0) return SNIP_ERR_NULL;
    if (!aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3u)) return SNIP_ERR_LAYOUT;
    PaperArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld; a.fmt = fmt; a.axis = axis;
    a.blocks = group == SNIP_GROUP_BLOCK_128x128;
    a.codes = (uint8_t*)codes; a.scales = scales; a.stats = nullptr; a.workspace = nullptr;
    return launch_paper(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

snip_status snip_quant_error_stats_paper(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_axis axis,
                                         snip_group group, snip_stats* out, void* workspace, size_t workspace_bytes_,
                                         void* stream)
{
    snip_status st = check_paper(x, rows, cols, ld, axis, group);
    if (st != SNIP_OK) return st;
    if (!out) return SNIP_ERR_NULL;
    if (!workspace || workspace_bytes_ < paper_workspace_bytes(rows, cols)) return SNIP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SNIP_ERR_LAYOUT;
    PaperArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld; a.fmt = SNIP_FP8_E4M3; a.axis = axis;
    a.blocks = group == SNIP_GROUP_BLOCK_128x128;
    a.codes = nullptr; a.scales = nullptr; a.stats = (double*)out; a.workspace = workspace;
    return launch_paper(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

static snip_status check_ptensor(const snip_ptensor* q)
{
    if (!q) return SNIP_ERR_NULL;
    if ((!q->codes || !q->scales) && q->rows > 0) return SNIP_ERR_NULL;
    if (!valid_fmt(q->fmt)) return SNIP_ERR_FORMAT;
    if (q->group != SNIP_GROUP_TILE_1x128 && q->group != SNIP_GROUP_BLOCK_128x128) return SNIP_ERR_FORMAT;
    if (q->rows < 0 || q->cols <= 0 || q->cols % 128 != 0) return SNIP_ERR_SHAPE;
    if (q->rows >= (int64_t)1 << 31 || q->cols >= (int64_t)1 << 31) return SNIP_ERR_SHAPE;
    if (!aligned16(q->codes) || (reinterpret_cast<uintptr_t>(q->scales) & 3u)) return SNIP_ERR_LAYOUT;
    return SNIP_OK;
}

snip_status snip_gemm_paper(const snip_ptensor* a, const snip_ptensor* b, void* c, int64_t ld_out,
                            snip_out_dtype out_dtype, void* stream)
{
    snip_status st = check_ptensor(a);
    if (st != SNIP_OK) return st;
    st = check_ptensor(b);
    if (st != SNIP_OK) return st;
    if (!c && a->rows > 0 && b->rows > 0) return SNIP_ERR_NULL;
    if (out_dtype != SNIP_OUT_BF16 && out_dtype != SNIP_OUT_FP32) return SNIP_ERR_FORMAT;
    if (a->cols != b->cols) return SNIP_ERR_LAYOUT;
    if (ld_out < b->rows) return SNIP_ERR_SHAPE;
    if ((a->rows + 127) / 128 * ((b->rows + 127) / 128) >= (int64_t)1 << 31) return SNIP_ERR_SHAPE;
    if (!aligned16(c) || ld_out % (out_dtype == SNIP_OUT_BF16 ? 8 : 4) != 0) return SNIP_ERR_LAYOUT;
    GemmPaperArgs g;
    g.a_codes = (const uint8_t*)a->codes; g.a_scales = a->scales; g.a_group = a->group; g.fmt_a = a->fmt;
    g.b_codes = (const uint8_t*)b->codes; g.b_scales = b->scales; g.b_group = b->group; g.fmt_b = b->fmt;
    g.I = a->rows; g.J = b->rows; g.R = a->cols;
    g.c = c; g.ldc = ld_out; g.out_fp32 = out_dtype == SNIP_OUT_FP32;
    return launch_gemm_paper(g, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

snip_status snip_adamw_sensitivity(const float* m, const float* v, const void* g, snip_out_dtype g_dtype,
                                   int64_t n, float beta1, float beta2, float eps, double* sum_sq,
                                   void* workspace, size_t workspace_bytes_, void* stream)
{
    if (n < 0) return SNIP_ERR_SHAPE;
    if ((!m || !v || !g) && n > 0) return SNIP_ERR_NULL;
    if (!sum_sq) return SNIP_ERR_NULL;
    if (g_dtype != SNIP_OUT_BF16 && g_dtype != SNIP_OUT_FP32) return SNIP_ERR_FORMAT;
    if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f)) return SNIP_ERR_FORMAT;
    if (!aligned16(m) || !aligned16(v)) return SNIP_ERR_LAYOUT;
    if (reinterpret_cast<uintptr_t>(g) & (g_dtype == SNIP_OUT_BF16 ? 7u : 15u)) return SNIP_ERR_LAYOUT;
    if (!workspace || workspace_bytes_ < workspace_bytes(0, 0)) return SNIP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SNIP_ERR_LAYOUT;
    AdamwArgs a;
    a.m = m; a.v = v; a.g = g; a.g_bf16 = g_dtype == SNIP_OUT_BF16; a.n = n;
    a.beta1 = beta1; a.beta2 = beta2; a.eps = eps; a.out = sum_sq; a.workspace = workspace;
    return launch_adamw_sensitivity(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

double snip_weight_divergence(double alpha, double beta1, double beta2, int64_t t, double sens_sq,
                              double err_g_sq, int64_t n, int64_t k)
{
    if (t <= 0 || n <= 0 || k <= 0 || !(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0) ||
        !(sens_sq >= 0.0) || !(err_g_sq >= 0.0))
        return std::nan("");
    const double corr = std::sqrt(1.0 - std::pow(beta2, (double)t)) / (1.0 - std::pow(beta1, (double)t));
    return alpha * corr * std::sqrt(sens_sq * err_g_sq / ((double)n * (double)k));
}

snip_status snip_quant_error_stats(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_axis axis,
                                   snip_scale_rule rule, snip_stats* out, float* per_line, void* workspace,
                                   size_t workspace_bytes_, void* stream)
{
    snip_status st = check_source(x, rows, cols, ld, axis, rule);
    if (st != SNIP_OK) return st;
    if (!out) return SNIP_ERR_NULL;
    if (!workspace || workspace_bytes_ < workspace_bytes(rows, cols)) return SNIP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SNIP_ERR_LAYOUT;
    StatsArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld; a.axis = axis; a.rule = rule;
    a.stats = (double*)out; a.per_line = per_line; a.workspace = workspace;
    return launch_stats(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

snip_status snip_quant_error_stats_both(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_scale_rule rule,
                                        snip_stats* out_row, snip_stats* out_col, void* workspace,
                                        size_t workspace_bytes_, void* stream)
{
    snip_status st = check_source(x, rows, cols, ld, SNIP_AXIS_ROW, rule);
    if (st != SNIP_OK) return st;
    st = check_source(x, rows, cols, ld, SNIP_AXIS_COL, rule);
    if (st != SNIP_OK) return st;
    if (!out_row || !out_col) return SNIP_ERR_NULL;
    if (!workspace || workspace_bytes_ < workspace_bytes(rows, cols)) return SNIP_ERR_WORKSPACE;
    if (!aligned16(workspace)) return SNIP_ERR_LAYOUT;
    StatsArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld; a.axis = SNIP_AXIS_ROW; a.rule = rule;
    a.stats = (double*)out_row; a.per_line = nullptr; a.workspace = workspace;
    return launch_stats_both(a, (double*)out_col, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

size_t snip_noalloc_max_cols(void) { return (size_t)kNoallocMaxCols; }

snip_status snip_quant_error_stats_noalloc(const void* x, int64_t rows, int64_t cols, int64_t ld, snip_axis axis,
                                           snip_scale_rule rule, snip_stats* out, float* per_line, void* stream)
{
    snip_status st = check_source(x, rows, cols, ld, axis, rule);
    if (st != SNIP_OK) return st;
    if (!out) return SNIP_ERR_NULL;
    if (cols > kNoallocMaxCols) return SNIP_ERR_WORKSPACE;         // the resident scratch array is sized for this many columns
    // device address of this device's copy of the array, looked up once per device
    constexpr int kMaxDevices = 64;
    static void* g_scratch_ptr[kMaxDevices] = {};
    static std::mutex g_scratch_mutex;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SNIP_ERR_HIP;
    void* ptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SNIP_ERR_HIP;
            g_scratch_ptr[dev] = p;
        }
        ptr = g_scratch_ptr[dev];
    }
    StatsArgs a;
    a.x = (const uint16_t*)x; a.rows = rows; a.cols = cols; a.ld = ld; a.axis = axis; a.rule = rule;
    a.stats = (double*)out; a.per_line = per_line; a.workspace = ptr;
    return launch_stats(a, (hipStream_t)stream) == hipSuccess ? SNIP_OK : SNIP_ERR_HIP;
}

const char* snip_status_string(snip_status s)
{
    switch (s) {
        case SNIP_OK: return "ok";
        case SNIP_ERR_NULL: return "null pointer";
        case SNIP_ERR_SHAPE: return "bad shape";
        case SNIP_ERR_FORMAT: return "bad format or enum";
        case SNIP_ERR_LAYOUT: return "bad alignment or mismatched operands";
        case SNIP_ERR_WORKSPACE: return "workspace missing or too small";
        case SNIP_ERR_HIP: return "kernel launch failed";
    }
    return "unknown status";
}

}  // extern "C"
