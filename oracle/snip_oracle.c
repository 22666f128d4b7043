/*
 * CPU oracle for the SNIP quantized linear-layer path.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, plain definition of what the GPU library must compute.  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline leg, and by
 * nothing else.  It shares no code, header, table or constant with the HIP sources.
 *
 * What it follows (SNIP, arXiv 2602.01410):
 *   - Sec. 2.3 "Quantization granularity": a tensor is scaled so that the largest
 *     magnitude of a scaling group lands on the representable range of FPX, cast to FPX,
 *     and scaled back afterwards (scale = FPX_MAX / max|x|, y = Op(Quant(x*scale))/scale).
 *     Here the scaling group is a 1x32 tile and the scale is restricted to a power of two
 *     (an E8M0 byte), which is the MX layout Sec. 2.3 "Quantization Format" adopts for
 *     its FP4 E2M1 elements.
 *   - Sec. 2.2 / Fig. "mixed precision training": inputs, weights and output gradients
 *     are quantized before each of the three GEMMs of a linear layer.
 *   - Sec. 4.1 / 4.3.1 notation: X in R^{M x K}, W in R^{N x K}, dY in R^{M x N}.
 *   - Sec. 3.1 Step 1: Frobenius norms of the tensors and of their quantization error.
 *   - Sec. 5.3 "Memory Overhead": the row-wise form of those norms.
 *   - Sec. 4.2 "Loss Divergence in Forward Pass": the per-layer estimate built from the
 *     norms of dX, dW and of the quantization errors of X and W.
 *
 * All arithmetic is IEEE double or integer.  Everything a bf16 tensor can hold, and every
 * FP8/FP4 grid value times a power of two, is exact in double, so quantization here has
 * no rounding other than the single round-to-nearest-even onto the FPX grid.
 *
 * Element formats (OCP MX flavours):
 *   fmt 0 = FP8 E4M3: 1 sign, 4 exponent (bias 7), 3 mantissa bits, no infinities,
 *           S.1111.111 is NaN, largest finite 448, smallest subnormal 2^-9.
 *   fmt 1 = FP4 E2M1: 1 sign, 2 exponent (bias 1), 1 mantissa bit, values
 *           {0, .5, 1, 1.5, 2, 3, 4, 6}.
 * Scale rules for the power-of-two block scale 2^e (amax = m * 2^n, 1 <= m < 2):
 *   rule 0 (no overflow): 2^e is the smallest power of two with amax / 2^e <= FPX_MAX,
 *           i.e. the paper's scale rounded in the direction that keeps amax in range.
 *   rule 1 (floor):       e = n - emax(FPX); elements that land above FPX_MAX saturate.
 * Axis: 0 = the 32-element tiles run along a row of the source (contiguous elements),
 *       1 = they run down a column; the quantized tensor is then stored transposed, so
 *           that in both cases the stored matrix has its tiles along its rows.
 *
 * Parity pins for every function here live in tests/test_oracle_*.py (closed forms,
 * enumeration of the grids, brute-force nearest-value search, tie tables, round trips,
 * invariances, numpy's dgemm for the three products).  The paper prints no worked numeric
 * example for this path, so no pin is a value quoted from the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_TILE 32

/* ---- format parameters ------------------------------------------------------------ */

static int fmt_ebits(int fmt) { return fmt == 0 ? 4 : 2; }
static int fmt_mbits(int fmt) { return fmt == 0 ? 3 : 1; }
static int fmt_bias(int fmt)  { return fmt == 0 ? 7 : 1; }

/* Largest finite magnitude: E4M3 gives up only the all-ones pattern to NaN, E2M1 nothing. */
static unsigned fmt_max_code(int fmt) { return fmt == 0 ? 0x7Eu : 0x7u; }

/* bf16 is the upper half of an IEEE single. */
double oracle_bf16_to_f64(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Value of an element code: sign, biased exponent E, mantissa field T.
 * E == 0: subnormal, T * 2^(1 - bias - mbits); otherwise (1 + T/2^mbits) * 2^(E - bias). */
double oracle_decode(int fmt, unsigned code)
{
    const int mb = fmt_mbits(fmt), eb = fmt_ebits(fmt), bias = fmt_bias(fmt);
    const unsigned T = code & ((1u << mb) - 1u);
    const unsigned E = (code >> mb) & ((1u << eb) - 1u);
    const unsigned S = (code >> (mb + eb)) & 1u;
    double mag;
    if (fmt == 0 && E == 15u && T == 7u) return NAN;
    if (E == 0u) mag = ldexp((double)T, 1 - bias - mb);
    else         mag = ldexp(1.0 + ldexp((double)T, -mb), (int)E - bias);
    return S ? -mag : mag;
}

double oracle_fmt_max(int fmt) { return oracle_decode(fmt, fmt_max_code(fmt)); }

/* Round a real v onto the FPX grid: nearest value, ties to the even mantissa, magnitudes
 * beyond the largest finite value saturate, the sign bit is kept (also on zero).
 * The grid spacing around |v| is 2^(floor(log2|v|) - mbits), or the subnormal spacing
 * below the smallest normal; |v| / spacing is rounded to an integer with ties to even,
 * which is ties-to-even-mantissa because spacing * 2^mbits is the binade's lower end. */
unsigned oracle_encode_rne(int fmt, double v)
{
    const int mb = fmt_mbits(fmt), eb = fmt_ebits(fmt), bias = fmt_bias(fmt);
    const unsigned sign = signbit(v) ? 1u << (mb + eb) : 0u;
    double a = fabs(v);
    if (isnan(v)) return fmt == 0 ? 0x7Fu : 0u;
    if (a > oracle_fmt_max(fmt)) return sign | fmt_max_code(fmt);
    if (a == 0.0) return sign;
    int p;
    (void)frexp(a, &p);                 /* a = f * 2^p, 0.5 <= f < 1  =>  floor(log2 a) = p-1 */
    int ex = p - 1;
    if (ex < 1 - bias) ex = 1 - bias;   /* subnormal range shares the spacing of the first binade */
    const int step_exp = ex - mb;
    /* nearbyint under the default rounding mode rounds halves to the even integer */
    double q = nearbyint(ldexp(a, -step_exp));    /* in [0, 2^(mb+1)] */
    /* q counts grid steps from zero inside this binade's spacing; rebuild the value and
     * re-derive its fields (q may have reached the next binade). */
    double r = ldexp(q, step_exp);
    if (r > oracle_fmt_max(fmt)) return sign | fmt_max_code(fmt);
    if (r == 0.0) return sign;
    (void)frexp(r, &p);
    int rex = p - 1;
    unsigned E, T;
    if (rex < 1 - bias) {               /* subnormal result */
        E = 0u;
        T = (unsigned)ldexp(r, -(1 - bias - mb));
    } else {
        E = (unsigned)(rex + bias);
        T = (unsigned)(ldexp(r, -rex + mb)) - (1u << mb);
    }
    return sign | (E << mb) | T;
}

/* Block scale exponent as the stored E8M0 byte (value 2^(byte-127)); 0xFF marks a block
 * that holds a NaN or an infinity.  amax is the largest magnitude in the block. */
unsigned oracle_scale_byte(int fmt, int rule, double amax)
{
    if (isnan(amax) || isinf(amax)) return 0xFFu;
    int e;
    if (amax == 0.0) {
        e = -127;
    } else {
        int p;
        double f = frexp(amax, &p);     /* amax = f * 2^p, f in [0.5, 1) */
        double m = 2.0 * f;             /* in [1, 2) */
        int n = p - 1;
        double top = oracle_fmt_max(fmt);
        int pt;
        double ft = frexp(top, &pt);
        int emax = pt - 1;              /* 8 for E4M3, 2 for E2M1 */
        double mmax = 2.0 * ft;         /* 1.75 / 1.5 */
        e = n - emax;
        if (rule == 0 && m > mmax) e += 1;
    }
    if (e < -127) e = -127;
    if (e > 127) e = 127;
    return (unsigned)(e + 127);
}

/* ---- whole-tensor quantize -------------------------------------------------------- */

/* Element (r, c) of the STORED matrix: for axis 0 the source itself, for axis 1 its
 * transpose.  src is bf16 [rows_src][ld]. */
static uint16_t stored_elem(const uint16_t* src, int64_t ld, int axis, int64_t r, int64_t c)
{
    return axis == 0 ? src[r * ld + c] : src[c * ld + r];
}

/* Quantize a bf16 matrix src[rows][cols] (row stride ld).
 * Stored shape: SR x SC = rows x cols (axis 0) or cols x rows (axis 1); SC must be a
 * multiple of 32.  codes: FP8 one byte per element [SR][SC]; FP4 two per byte
 * [SR][SC/2], even element in the low nibble.  scales: [SR][SC/32] E8M0 bytes.
 * Returns 0, or -1 on a bad argument. */
int oracle_quantize(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld,
                    int fmt, int axis, int rule, uint8_t* codes, uint8_t* scales)
{
    if (!src || !codes || !scales) return -1;
    if ((fmt != 0 && fmt != 1) || (axis != 0 && axis != 1) || (rule != 0 && rule != 1)) return -1;
    if (rows < 0 || cols < 0 || ld < cols) return -1;
    const int64_t SR = axis == 0 ? rows : cols;
    const int64_t SC = axis == 0 ? cols : rows;
    if (SC % ORACLE_TILE) return -1;
    const int64_t nb = SC / ORACLE_TILE;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < SR; ++r) {
        for (int64_t b = 0; b < nb; ++b) {
            double v[ORACLE_TILE];
            double amax = 0.0;
            int bad = 0;
            for (int i = 0; i < ORACLE_TILE; ++i) {
                v[i] = oracle_bf16_to_f64(stored_elem(src, ld, axis, r, b * ORACLE_TILE + i));
                if (isnan(v[i]) || isinf(v[i])) bad = 1;
                else if (fabs(v[i]) > amax) amax = fabs(v[i]);
            }
            unsigned sb = bad ? 0xFFu : oracle_scale_byte(fmt, rule, amax);
            scales[r * nb + b] = (uint8_t)sb;
            for (int i = 0; i < ORACLE_TILE; ++i) {
                unsigned code = 0u;
                if (!bad) code = oracle_encode_rne(fmt, ldexp(v[i], -((int)sb - 127)));
                int64_t e = r * SC + b * ORACLE_TILE + i;
                if (fmt == 0) {
                    codes[e] = (uint8_t)code;
                } else {
                    /* two 4-bit codes per byte; bytes are owned by one thread (same r) */
                    uint8_t* p = &codes[e >> 1];
                    if ((e & 1) == 0) *p = (uint8_t)((*p & 0xF0u) | code);
                    else              *p = (uint8_t)((*p & 0x0Fu) | (code << 4));
                }
            }
        }
    }
    return 0;
}

/* Stored codes + scales -> doubles [SR][SC] (same stored orientation). */
int oracle_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t SR, int64_t SC,
                      int fmt, double* out)
{
    if (!codes || !scales || !out) return -1;
    if ((fmt != 0 && fmt != 1) || SR < 0 || SC < 0 || SC % ORACLE_TILE) return -1;
    const int64_t nb = SC / ORACLE_TILE;
    #pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < SR; ++r) {
        for (int64_t c = 0; c < SC; ++c) {
            unsigned sb = scales[r * nb + c / ORACLE_TILE];
            int64_t e = r * SC + c;
            unsigned code = fmt == 0 ? codes[e] : ((codes[e >> 1] >> ((e & 1) * 4)) & 0xFu);
            out[e] = sb == 0xFFu ? NAN : ldexp(oracle_decode(fmt, code), (int)sb - 127);
        }
    }
    return 0;
}

/* q(x) of Sec. 4.1 (q(x) = x + delta_x): quantize then dequantize, result in the SOURCE
 * orientation out[rows][cols], whatever the tile axis. */
int oracle_fake_quant(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld,
                      int fmt, int axis, int rule, double* out)
{
    const int64_t SR = axis == 0 ? rows : cols;
    const int64_t SC = axis == 0 ? cols : rows;
    if (rows < 0 || cols < 0) return -1;
    size_t n = (size_t)rows * (size_t)cols;
    uint8_t* codes = (uint8_t*)calloc(n ? n : 1, 1);
    uint8_t* scales = (uint8_t*)calloc(n / ORACLE_TILE + 1, 1);
    double* st = (double*)malloc((n ? n : 1) * sizeof(double));
    int rc = -1;
    if (codes && scales && st) {
        rc = oracle_quantize(src, rows, cols, ld, fmt, axis, rule, codes, scales);
        if (rc == 0) rc = oracle_dequantize(codes, scales, SR, SC, fmt, st);
        if (rc == 0) {
            for (int64_t r = 0; r < rows; ++r)
                for (int64_t c = 0; c < cols; ++c)
                    out[r * cols + c] = axis == 0 ? st[r * cols + c] : st[c * rows + r];
        }
    }
    free(codes); free(scales); free(st);
    return rc;
}

/* ---- the three products of a linear layer (Sec. 2.2; shapes of Sec. 4.1 / 4.3.1) ----
 * Operands are q(.) values in double, in their natural orientations:
 * X [M][K], W [N][K], dY [M][N].  One accumulator per output, k ascending. */

int oracle_gemm_fwd(const double* X, const double* W, int64_t M, int64_t N, int64_t K, double* Y)
{
    if (!X || !W || !Y) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k) s += X[m * K + k] * W[n * K + k];
            Y[m * N + n] = s;
        }
    return 0;
}

int oracle_gemm_dgrad(const double* dY, const double* W, int64_t M, int64_t N, int64_t K, double* dX)
{
    if (!dY || !W || !dX) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            double s = 0.0;
            for (int64_t n = 0; n < N; ++n) s += dY[m * N + n] * W[n * K + k];
            dX[m * K + k] = s;
        }
    return 0;
}

int oracle_gemm_wgrad(const double* dY, const double* X, int64_t M, int64_t N, int64_t K, double* dW)
{
    if (!dY || !X || !dW) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            double s = 0.0;
            for (int64_t m = 0; m < M; ++m) s += dY[m * N + n] * X[m * K + k];
            dW[n * K + k] = s;
        }
    return 0;
}

/* ---- Step-1 statistics (Sec. 3.1) -------------------------------------------------- */

/* Squared Frobenius norms of x and of q(x) - x for both candidate formats, tiles along
 * `axis`: out3 = { sum x^2, sum (q_fp4(x)-x)^2, sum (q_fp8(x)-x)^2 }.
 * per_line (optional) holds the same three sums for every stored row, [SR][3]: one per
 * source row for axis 0, one per source column for axis 1 (the row-wise form of
 * Sec. 5.3).  Sums run in index order in double. */
int oracle_stats(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld,
                 int axis, int rule, double* out3, double* per_line)
{
    if (!src || !out3) return -1;
    if ((axis != 0 && axis != 1) || (rule != 0 && rule != 1)) return -1;
    if (rows < 0 || cols < 0 || ld < cols) return -1;
    const int64_t SR = axis == 0 ? rows : cols;
    const int64_t SC = axis == 0 ? cols : rows;
    if (SC % ORACLE_TILE) return -1;
    size_t n = (size_t)rows * (size_t)cols;
    double* q4 = (double*)malloc((n ? n : 1) * sizeof(double));
    double* q8 = (double*)malloc((n ? n : 1) * sizeof(double));
    double* line = (double*)calloc((size_t)(SR ? SR : 1) * 3, sizeof(double));
    int rc = -1;
    if (q4 && q8 && line) {
        rc = oracle_fake_quant(src, rows, cols, ld, 1, axis, rule, q4);
        if (rc == 0) rc = oracle_fake_quant(src, rows, cols, ld, 0, axis, rule, q8);
    }
    if (rc == 0) {
        for (int64_t r = 0; r < SR; ++r) {
            double s0 = 0.0, s4 = 0.0, s8 = 0.0;
            for (int64_t c = 0; c < SC; ++c) {
                int64_t sr = axis == 0 ? r : c, sc = axis == 0 ? c : r;   /* source coords */
                double x = oracle_bf16_to_f64(src[sr * ld + sc]);
                double d4 = q4[sr * cols + sc] - x;
                double d8 = q8[sr * cols + sc] - x;
                s0 += x * x; s4 += d4 * d4; s8 += d8 * d8;
            }
            line[r * 3 + 0] = s0; line[r * 3 + 1] = s4; line[r * 3 + 2] = s8;
        }
        out3[0] = out3[1] = out3[2] = 0.0;
        for (int64_t r = 0; r < SR; ++r)
            for (int j = 0; j < 3; ++j) out3[j] += line[r * 3 + j];
        if (per_line) memcpy(per_line, line, (size_t)SR * 3 * sizeof(double));
    }
    free(q4); free(q8); free(line);
    return rc;
}

/* ---- norms of the GEMM outputs and the loss-divergence estimate ---------------------- */

/* Nearest value representable in the GEMM's output type, ties to even: out_dtype 0 = bf16
 * (8 significant bits, the exponent range of an IEEE single), 1 = IEEE single.  The bf16
 * rounding is done on the double directly (scale so that one unit in the last place is 1,
 * round to the nearest integer with ties to even, scale back).  Magnitudes beyond the
 * type's largest finite value are outside what the path produces and are not handled. */
double oracle_round_output(double v, int out_dtype)
{
    if (out_dtype == 1) return (double)(float)v;
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    (void)frexp(fabs(v), &e);                /* |v| = f * 2^e, 0.5 <= f < 1  =>  exponent of v is e-1 */
    int ex = e - 1;
    if (ex < -126) ex = -126;                /* subnormal range: fixed quantum 2^-133 */
    double quantum = ldexp(1.0, ex - 7);     /* 8 significant bits */
    return nearbyint(v / quantum) * quantum; /* default rounding mode: to nearest, ties to even */
}

/* Squared Frobenius norm of a GEMM output as the path stores it (Sec. 3.1 Step 1 lists the
 * norms of Y, dX and dW among the collected statistics): every element of the exact product
 * c[0..n) is rounded to the output type, squared and summed in index order in double. */
double oracle_output_sum_sq(const double* c, int64_t n, int out_dtype)
{
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double r = oracle_round_output(c[i], out_dtype);
        s += r * r;
    }
    return s;
}

/* Estimated change of the loss when the inputs X [M,K] and weights W [N,K] of one linear
 * layer are quantized (Sec. 4.2 "Loss Divergence in Forward Pass"):
 *     sqrt( (|grad_X L| |delta_X| / sqrt(M K))^2 + (|grad_W L| |delta_W| / sqrt(N K))^2 )
 * with Frobenius norms; the arguments are SQUARED norms, as the statistics deliver them
 * (grad_X L is the dgrad output, grad_W L the wgrad output, delta = q(.) - .). */
double oracle_loss_divergence(double grad_x_sq, double err_x_sq, int64_t M,
                              double grad_w_sq, double err_w_sq, int64_t N, int64_t K)
{
    double tx = sqrt(grad_x_sq) * sqrt(err_x_sq) / sqrt((double)M * (double)K);
    double tw = sqrt(grad_w_sq) * sqrt(err_w_sq) / sqrt((double)N * (double)K);
    return sqrt(tx * tx + tw * tw);
}

/* ---- stochastic rounding of FP4 output gradients (Sec. 5.1 "Quantization Format and
 *      Implementation": values are rounded probabilistically to the two nearest values) ---- */

/* Threefry-2x32 with 20 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
 * as 1, 2, 3", SC'11): a counter-based generator, out = f(counter, key).  Written out from the
 * published description: the key is extended by a third word (XOR of the key words with the
 * parity constant 0x1BD11BDA); a round adds word 1 into word 0, rotates word 1 left by the
 * round's constant and XORs word 0 into it; after every fourth round the next two key words
 * (cyclically) are added, the second one together with the injection number. */
static uint32_t rotl32(uint32_t v, int r) { return (v << r) | (v >> (32 - r)); }

void oracle_threefry2x32_20(const uint32_t ctr[2], const uint32_t key[2], uint32_t out[2])
{
    static const int rot[8] = { 13, 15, 26, 6, 17, 29, 16, 24 };
    uint32_t ks[3] = { key[0], key[1], 0x1BD11BDAu ^ key[0] ^ key[1] };
    uint32_t x0 = ctr[0] + ks[0], x1 = ctr[1] + ks[1];
    for (int round = 0; round < 20; ++round) {
        x0 += x1;
        x1 = rotl32(x1, rot[round % 8]);
        x1 ^= x0;
        if (round % 4 == 3) {
            int inj = round / 4 + 1;                 /* 1 .. 5 */
            x0 += ks[inj % 3];
            x1 += ks[(inj + 1) % 3] + (uint32_t)inj;
        }
    }
    out[0] = x0; out[1] = x1;
}

/* The random byte of stored element number `index` (row-major position in the STORED matrix)
 * under `seed`: elements are served in groups of eight by one generator call with counter =
 * index / 8 (low word first) and key = seed (low word first); element j of a group takes
 * byte j of the 64 output bits, word 0 first, least significant byte first. */
unsigned oracle_sr_byte(uint64_t seed, uint64_t index)
{
    uint64_t group = index / 8;
    uint32_t ctr[2] = { (uint32_t)group, (uint32_t)(group >> 32) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[2];
    oracle_threefry2x32_20(ctr, key, out);
    unsigned j = (unsigned)(index % 8);
    return (out[j / 4] >> (8 * (j % 4))) & 0xFFu;
}

/* Stochastic rounding of v (already divided by the block scale) onto the FP4 E2M1 grid with
 * the random byte rnd (0..255).  lo <= |v| <= hi are the two nearest grid magnitudes; the
 * magnitude goes up to hi with probability p = (|v| - lo) / (hi - lo), realised as
 *     up  <=>  rnd < floor(256 p).
 * Grid values stay where they are for every rnd; magnitudes at or beyond the largest grid
 * value give the largest code (they only occur under the saturating scale rule); the sign is
 * kept (so a negative value that rounds to zero gives the code of -0).  Returns the 4-bit code. */
unsigned oracle_encode_sr_fp4(double v, unsigned rnd)
{
    unsigned sign = signbit(v) ? 8u : 0u;
    double a = fabs(v);
    if (isnan(a)) return sign;           /* not produced by the path: blocks with NaN/Inf get zero codes */
    unsigned top = fmt_max_code(1);
    if (a >= oracle_decode(1, top)) return sign | top;
    unsigned lo_code = 0;
    while (oracle_decode(1, lo_code + 1) <= a) ++lo_code;        /* largest grid magnitude <= a */
    double lo = oracle_decode(1, lo_code), hi = oracle_decode(1, lo_code + 1);
    double p = (a - lo) / (hi - lo);                             /* exact: hi - lo is a power of two */
    double threshold = floor(256.0 * p);
    return sign | (lo_code + ((double)rnd < threshold ? 1u : 0u));
}

/* Quantize a bf16 matrix to FP4 with stochastic rounding.  Layout, scale rule, axis and the
 * treatment of zero and non-finite blocks are those of oracle_quantize (the scale does not
 * depend on the rounding mode); fmt is fixed to FP4. */
int oracle_quantize_sr_fp4(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld,
                           int axis, int rule, uint64_t seed, uint8_t* codes, uint8_t* scales)
{
    if (!src || !codes || !scales) return -1;
    if ((axis != 0 && axis != 1) || (rule != 0 && rule != 1)) return -1;
    if (rows < 0 || cols < 0 || ld < cols) return -1;
    const int64_t SR = axis == 0 ? rows : cols;
    const int64_t SC = axis == 0 ? cols : rows;
    if (SC % ORACLE_TILE) return -1;
    const int64_t nb = SC / ORACLE_TILE;
    memset(codes, 0, (size_t)(SR * SC / 2));
    for (int64_t r = 0; r < SR; ++r)
        for (int64_t b = 0; b < nb; ++b) {
            double amax = 0.0;
            int bad = 0;
            for (int k = 0; k < ORACLE_TILE; ++k) {
                double x = oracle_bf16_to_f64(stored_elem(src, ld, axis, r, b * ORACLE_TILE + k));
                if (isnan(x) || isinf(x)) bad = 1;
                else if (fabs(x) > amax) amax = fabs(x);
            }
            unsigned byte = bad ? 0xFFu : oracle_scale_byte(1, rule, amax);
            scales[r * nb + b] = (uint8_t)byte;
            if (bad) continue;                                   /* codes stay zero */
            double scale = ldexp(1.0, (int)byte - 127);
            for (int k = 0; k < ORACLE_TILE; ++k) {
                int64_t c = b * ORACLE_TILE + k;
                double x = oracle_bf16_to_f64(stored_elem(src, ld, axis, r, c));
                uint64_t index = (uint64_t)r * (uint64_t)SC + (uint64_t)c;
                unsigned code = oracle_encode_sr_fp4(x / scale, oracle_sr_byte(seed, index));
                codes[(r * SC + c) / 2] |= (uint8_t)(code << (4 * (c % 2)));
            }
        }
    return 0;
}

/* ---- AdamW factor of the weight-divergence estimate (Sec. 4.3.2 "Impact on Weight Divergence") ---- */

/* With m = beta1 m' + (1-beta1) g and v = beta2 v' + (1-beta2) g^2 the update direction
 * h(g) = m / (sqrt(v) + eps) has the element-wise derivative
 *     dh/dg = (1-beta1) / (sqrt(v)+eps)  -  (1-beta2) m g / ( sqrt(v) (sqrt(v)+eps)^2 ),
 * and Step 1 collects the Frobenius norm of that term.  Returns its SQUARE, summed in index
 * order in double.  Where v is zero the second part is taken as zero (AdamW has m = g = 0
 * there; the expression itself would be 0/0). */
double oracle_adamw_sensitivity_sq(const double* m, const double* v, const double* g, int64_t n,
                                   double beta1, double beta2, double eps)
{
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double root = sqrt(v[i]);
        double first = (1.0 - beta1) / (root + eps);
        double second = 0.0;
        if (v[i] > 0.0) second = (1.0 - beta2) * m[i] * g[i] / (root * (root + eps) * (root + eps));
        double t = first - second;
        s += t * t;
    }
    return s;
}

/* The per-layer weight-divergence estimate that the factor feeds (same section):
 *     alpha * sqrt(1 - beta2^t) / (1 - beta1^t) * ||dh/dg||_F * ||eps_g||_F / sqrt(N K)
 * from squared norms; eps_g is the perturbation of the weight gradient. */
double oracle_weight_divergence(double alpha, double beta1, double beta2, int64_t t,
                                double sens_sq, double err_g_sq, int64_t N, int64_t K)
{
    double corr = sqrt(1.0 - pow(beta2, (double)t)) / (1.0 - pow(beta1, (double)t));
    return alpha * corr * sqrt(sens_sq) * sqrt(err_g_sq) / sqrt((double)N * (double)K);
}

/* ---- the paper's own quantization recipe (Sec. 2.3 and Sec. 5.1) ---------------------- */

/* Sec. 2.3: scale = FPX_MAX / max|x| over a scaling group, y = Quant(x * scale), and the
 * value the GEMM sees is y / scale.  Sec. 5.1: the groups are 1x128 tiles for activations and
 * gradients and 128x128 blocks for weights.  Unlike the power-of-two block scales above, this
 * scale is a real number and x * scale is not exact, so the precision of those two steps is
 * part of the definition.  The paper gives the formula, not the arithmetic; its experiments
 * fake-quantize inside a training framework (Sec. 5.1), where such a scale is held as an fp32
 * tensor and multiplied in fp32.  The reading taken here is therefore fp32: one correctly
 * rounded division, one correctly rounded product:
 *     s = (float)FPX_MAX / amax          (amax = 0: s = 1;  s is capped at 2^126 so that a
 *                                         group of denormal-sized values does not overflow it)
 *     t = (float)x * s
 *     code = nearest FPX value to t, ties to even, saturating
 * The scale array holds s as fp32, one per group, in the stored orientation:
 *     group_rows = 1   (tiles):  [SR][SC/128]
 *     group_rows = 128 (blocks): [ceil(SR/128)][SC/128]
 * SC must be a multiple of 128.  A group that contains an infinity or a NaN gets scale NaN and
 * zero codes.  Codes are laid out as in oracle_quantize. */
static float paper_group_scale(const uint16_t* src, int64_t ld, int axis, int fmt,
                               int64_t r0, int64_t r1, int64_t c0, int64_t c1)
{
    float amax = 0.0f;
    int bad = 0;
    for (int64_t r = r0; r < r1; ++r)
        for (int64_t c = c0; c < c1; ++c) {
            float x = (float)oracle_bf16_to_f64(stored_elem(src, ld, axis, r, c));
            if (isnan(x) || isinf(x)) bad = 1;
            else if (fabsf(x) > amax) amax = fabsf(x);
        }
    if (bad) return NAN;
    if (amax == 0.0f) return 1.0f;
    float s = (float)oracle_fmt_max(fmt) / amax;
    if (!(s <= 0x1p126f)) s = 0x1p126f;
    return s;
}

int oracle_quantize_paper(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld,
                          int fmt, int axis, int group_rows, uint8_t* codes, float* scales)
{
    if (!src || !codes || !scales) return -1;
    if ((fmt != 0 && fmt != 1) || (axis != 0 && axis != 1) || (group_rows != 1 && group_rows != 128)) return -1;
    if (rows < 0 || cols < 0 || ld < cols) return -1;
    const int64_t SR = axis == 0 ? rows : cols;
    const int64_t SC = axis == 0 ? cols : rows;
    if (SC % 128) return -1;
    const int64_t ng = SC / 128;
    if (fmt == 1) memset(codes, 0, (size_t)(SR * SC / 2));
    for (int64_t r0 = 0; r0 < SR; r0 += group_rows) {
        int64_t r1 = r0 + group_rows < SR ? r0 + group_rows : SR;
        for (int64_t gcol = 0; gcol < ng; ++gcol) {
            float s = paper_group_scale(src, ld, axis, fmt, r0, r1, gcol * 128, gcol * 128 + 128);
            scales[(r0 / group_rows) * ng + gcol] = s;
            for (int64_t r = r0; r < r1; ++r)
                for (int64_t c = gcol * 128; c < gcol * 128 + 128; ++c) {
                    unsigned code = 0u;
                    if (!isnan(s)) {
                        float x = (float)oracle_bf16_to_f64(stored_elem(src, ld, axis, r, c));
                        float t = x * s;
                        code = oracle_encode_rne(fmt, (double)t);
                    }
                    int64_t e = r * SC + c;
                    if (fmt == 0) codes[e] = (uint8_t)code;
                    else codes[e >> 1] |= (uint8_t)(code << (4 * (e & 1)));
                }
        }
    }
    return 0;
}

/* Value the GEMM sees for every element: decode(code) / s, in double, stored orientation. */
int oracle_dequantize_paper(const uint8_t* codes, const float* scales, int64_t SR, int64_t SC,
                            int fmt, int group_rows, double* out)
{
    if (!codes || !scales || !out || SC % 128 || (fmt != 0 && fmt != 1)) return -1;
    const int64_t ng = SC / 128;
    for (int64_t r = 0; r < SR; ++r)
        for (int64_t c = 0; c < SC; ++c) {
            int64_t e = r * SC + c;
            unsigned code = fmt == 0 ? codes[e] : (codes[e >> 1] >> (4 * (e & 1))) & 0xFu;
            double s = (double)scales[(r / group_rows) * ng + c / 128];
            out[e] = isnan(s) ? NAN : oracle_decode(fmt, code) / s;
        }
    return 0;
}

/* Step-1 statistics under the paper's recipe: out3 = { sum x^2, sum (q4(x)-x)^2, sum (q8(x)-x)^2 }
 * with q = dequantize(quantize(x)) as above, sums in index order in double. */
int oracle_stats_paper(const uint16_t* src, int64_t rows, int64_t cols, int64_t ld,
                       int axis, int group_rows, double* out3)
{
    if (!src || !out3) return -1;
    const int64_t SR = axis == 0 ? rows : cols;
    const int64_t SC = axis == 0 ? cols : rows;
    if (rows < 0 || cols < 0 || ld < cols || SC % 128) return -1;
    size_t n = (size_t)SR * (size_t)SC;
    size_t ngroups = (size_t)((SR + group_rows - 1) / group_rows) * (size_t)(SC / 128);
    uint8_t* codes = (uint8_t*)malloc(n ? n : 1);
    float* scales = (float*)malloc((ngroups ? ngroups : 1) * sizeof(float));
    double* q = (double*)malloc((n ? n : 1) * sizeof(double));
    int rc = (codes && scales && q) ? 0 : -1;
    out3[0] = out3[1] = out3[2] = 0.0;
    for (int fmt = 1; fmt >= 0 && rc == 0; --fmt) {
        rc = oracle_quantize_paper(src, rows, cols, ld, fmt, axis, group_rows, codes, scales);
        if (rc == 0) rc = oracle_dequantize_paper(codes, scales, SR, SC, fmt, group_rows, q);
        if (rc != 0) break;
        double s0 = 0.0, se = 0.0;
        for (int64_t r = 0; r < SR; ++r)
            for (int64_t c = 0; c < SC; ++c) {
                double x = oracle_bf16_to_f64(stored_elem(src, ld, axis, r, c));
                double d = q[r * SC + c] - x;
                s0 += x * x; se += d * d;
            }
        out3[0] = s0;
        out3[fmt == 1 ? 1 : 2] = se;
    }
    free(codes); free(scales); free(q);
    return rc;
}
