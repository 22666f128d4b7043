// Internal launcher interface between the C-ABI layer (api.hip) and the kernel files.
// Nothing here is exported.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace snip {

constexpr int kFP8 = 0;   // E4M3
constexpr int kFP4 = 1;   // E2M1
constexpr int kBlock = 32;  // elements per scale

// Number of waves the streaming kernels are launched with; also the number of per-wave
// partial-sum slots at the start of the workspace.  Fixed (not device dependent) so that
// reductions run in the same order everywhere.
constexpr int kStreamBlocks = 2048;
constexpr int kWavesPerBlock = 4;
constexpr int kStreamWaves = kStreamBlocks * kWavesPerBlock;
constexpr int kMaxColSplits = 64;    // row splits of the column-statistics kernel
// Workspace of the streaming kernels: [kStreamWaves][6] fp32 wave partials ([..][3] for one block direction),
// then [kMaxColSplits][cols][3] fp32 per-column partials for the per-line column statistics.
constexpr size_t kPartialBytes = (size_t)kStreamWaves * 6 * sizeof(float);
constexpr size_t stream_workspace_bytes(int64_t cols) { return kPartialBytes + (size_t)kMaxColSplits * (size_t)cols * 3 * sizeof(float); }
constexpr int kG4Align = 256;    // row pitch (in dwords) of the grouped scale copy is a multiple of this
__host__ __device__ inline int64_t g4_pitch(int64_t rows) { return (rows + kG4Align - 1) / kG4Align * kG4Align; }

struct QuantArgs {
    const uint16_t* x;
    int64_t rows, cols, ld;
    int fmt, axis, rule;
    uint8_t* codes;
    uint8_t* scales;
    uint8_t* scales_g4;       // [ceil(stored cols / 128)][g4_pitch(stored rows)][4] or nullptr
    double* stats;        // device snip_stats (3 doubles) or nullptr
    void* workspace;
    bool stochastic = false;  // FP4 only: stochastic rounding with the byte stream of sr_seed
    uint64_t sr_seed = 0;
};

// One source matrix quantized in both orientations by one pass (snip_quantize_both).
struct QuantBothArgs {
    const uint16_t* x;
    int64_t rows, cols, ld;
    int rule;
    int fmt_r, fmt_c;                        // row-direction output [rows][cols], column-direction output [cols][rows]
    uint8_t *codes_r, *scales_r, *g4_r;
    uint8_t *codes_c, *scales_c, *g4_c;
    double *stats_r, *stats_c;               // both or neither
    bool both_formats = false;               // statistics: also the error of the format not written
    void* workspace;
};

struct StatsArgs {
    const uint16_t* x;
    int64_t rows, cols, ld;
    int axis, rule;
    double* stats;        // device, 3 doubles
    float* per_line;      // device [L][3] or nullptr
    void* workspace;
};

struct GemmArgs {
    const uint8_t* a_codes; const uint8_t* a_scales; const uint8_t* a_scales_g4; int fmt_a;
    const uint8_t* b_codes; const uint8_t* b_scales; const uint8_t* b_scales_g4; int fmt_b;
    int64_t I, J, R;      // C[I][J] = sum_r A[I][r] B[J][r]
    void* c; int64_t ldc; int out_fp32;
    // optional: squared Frobenius norm of the stored output.  norm_partials has room for
    // gemm_norm_partials(I, J) floats (one per workgroup of the launch); norm_out is one double.
    float* norm_partials = nullptr;
    double* norm_out = nullptr;
};
// Upper bound of the number of partials either GEMM kernel writes for an I x J output (128 x 128 tiles).
inline int64_t gemm_norm_partials(int64_t I, int64_t J) { return ((I + 127) / 128) * ((J + 127) / 128); }

struct AdamwArgs {
    const float* m; const float* v; const void* g; int g_bf16;
    int64_t n;
    float beta1, beta2, eps;
    double* out;          // device, one double
    void* workspace;      // room for kStreamWaves floats
};

// The paper's own recipe (real-valued scale per 1x128 tile or 128x128 block): quantize (stats == nullptr)
// or statistics of both formats (stats != nullptr; codes / scales unused).
struct PaperArgs {
    const uint16_t* x;
    int64_t rows, cols, ld;
    int fmt, axis;
    bool blocks;           // false: 1x128 tiles, true: 128x128 blocks (stored orientation)
    uint8_t* codes;
    float* scales;
    double* stats;         // device, 3 doubles
    void* workspace;       // statistics only: paper_workspace_bytes(rows, cols)
};
struct GemmPaperArgs {
    const uint8_t* a_codes; const float* a_scales; int a_group; int fmt_a;     // group: 1 (tiles) or 128 (blocks)
    const uint8_t* b_codes; const float* b_scales; int b_group; int fmt_b;
    int64_t I, J, R;      // C[I][J] = sum_r (A[I][r] / sa) (B[J][r] / sb)
    void* c; int64_t ldc; int out_fp32;
};
hipError_t launch_gemm_paper(const GemmPaperArgs& a, hipStream_t s);
size_t paper_workspace_bytes(int64_t rows, int64_t cols);
hipError_t launch_paper(const PaperArgs& a, hipStream_t s);

size_t workspace_bytes(int64_t rows, int64_t cols);
hipError_t launch_adamw_sensitivity(const AdamwArgs& a, hipStream_t s);
// out[0] = sum of partials[0..n) in index order, in double (one workgroup); n may be 0
hipError_t launch_sum_partials(const float* partials, int64_t n, double* out, hipStream_t s);
hipError_t launch_quantize(const QuantArgs& a, hipStream_t s);
hipError_t launch_quantize_both(const QuantBothArgs& a, hipStream_t s);
hipError_t launch_stats(const StatsArgs& a, hipStream_t s);
// both block directions from one read: a.stats receives the row-direction record, out_col the column one
// (a.axis and a.per_line are ignored)
hipError_t launch_stats_both(const StatsArgs& a, double* out_col, hipStream_t s);
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
bool gemm_fast_eligible(const GemmArgs& a);          // persistent large-tile kernel (gemm_fast.hip)
hipError_t launch_gemm_fast(const GemmArgs& a, hipStream_t s);
int64_t gemm_fast_partials(const GemmArgs& a);         // partials launch_gemm_fast writes

}  // namespace snip
