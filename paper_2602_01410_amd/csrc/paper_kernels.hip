// The paper's own quantization recipe (SNIP Sec. 2.3 and Sec. 5.1): a real-valued scale
// s = FPX_MAX / max|x| per scaling group, codes = RNE_FPX(x * s), value seen by the GEMM = code / s;
// groups are 1x128 tiles (activations, gradients) or 128x128 blocks (weights), both in the STORED
// orientation (blocks along rows, or down columns with the result stored transposed).
//
// Unlike the power-of-two block scales of the main path, s and x * s are not exact, so their precision is
// part of the definition: fp32, one correctly rounded division and one correctly rounded product, which is
// what these kernels compute (v_div_* sequence, v_mul_f32) before gfx950's v_cvt_scalef32_pk_{fp8,fp4}_f32
// rounds to the element format (scale operand 1.0; the FP8 form does not saturate, so x * s is clamped to
// +-448 first: the product can exceed 448 by one rounding).
//
// Kernels: quantize along rows (tile maxima by a 16-lane DPP reduction inside the pass), quantize down
// columns (a lane owns two columns, so tile maxima never leave the lane; the unit is read twice, the
// second time from cache), a block-maximum pre-pass for the 128x128 groups, and the matching statistics
// kernels (both formats from one read).  All are streaming kernels bound by HBM bandwidth or VALU rate.
#include "snip_internal.h"

namespace snip {
namespace {

typedef short short2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));
typedef unsigned v4u __attribute__((ext_vector_type(4)));

// Streaming (non-temporal) loads for sources that are read once.
__device__ __forceinline__ uint4 ld16_stream(const void* p)
{
    const v4u v = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ unsigned ld4_stream(const void* p) { return __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(p)); }

constexpr int kGroup = 128;              // scaling-group extent along the blocked dimension
constexpr int kSeg = 512;                // elements of a row one wave handles per load
constexpr int kUnroll = 4;               // rows in flight per wave (row kernels)
constexpr int kColsPerWave = 128;        // columns per unit (column kernels)

template <int FMT> __device__ __forceinline__ float fmt_max() { return FMT == kFP8 ? 448.f : 6.f; }

__device__ __forceinline__ unsigned pk_max_u16(unsigned a, unsigned b)
{
    return __builtin_bit_cast(unsigned, __builtin_elementwise_max(__builtin_bit_cast(ushort2_t, a),
                                                                  __builtin_bit_cast(ushort2_t, b)));
}
__device__ __forceinline__ float wave_sum(float v)
{
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ unsigned umax(unsigned a, unsigned b) { return a > b ? a : b; }

// Scale of a group from the 15 magnitude bits of its bf16 maximum: MAX / amax in fp32, 1 for an all-zero
// group, capped at 2^126 (a group of denormal-sized values would overflow it), NaN for a group that holds
// an infinity or a NaN.
template <int FMT>
__device__ __forceinline__ float group_scale(unsigned amax_bits)
{
    if (amax_bits >= 0x7F80u) return __builtin_nanf("");
    if (amax_bits == 0u) return 1.f;
    const float s = __fdiv_rn(fmt_max<FMT>(), __uint_as_float(amax_bits << 16));
    return s <= 0x1p126f ? s : 0x1p126f;
}

// Magnitude bits of the largest of the 8 bf16 values of one 16-byte load.
__device__ __forceinline__ unsigned amax8(const uint4& v)
{
    const unsigned m = pk_max_u16(pk_max_u16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu),
                                  pk_max_u16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu));
    return umax(m & 0xFFFFu, m >> 16);
}
// Maximum over the 16 lanes of a DPP row: quad permutes, then rotations by 4 and 8 inside the row.
__device__ __forceinline__ unsigned row16_max(unsigned m)
{
    m = umax(m, (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0xB1, 0xF, 0xF, true));     // quad_perm [1,0,3,2]
    m = umax(m, (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0x4E, 0xF, 0xF, true));     // quad_perm [2,3,0,1]
    m = umax(m, (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0x124, 0xF, 0xF, true));    // row_ror:4
    m = umax(m, (unsigned)__builtin_amdgcn_update_dpp(0, (int)m, 0x128, 0xF, 0xF, true));    // row_ror:8
    return m;
}

// x * s for the two bf16 halves of a word.
__device__ __forceinline__ void scaled2(unsigned w, float s, float& lo, float& hi)
{
    lo = __fmul_rn(__uint_as_float(w << 16), s);
    hi = __fmul_rn(__uint_as_float(w & 0xFFFF0000u), s);
}
__device__ __forceinline__ float clamp448(float t) { return fminf(fmaxf(t, -448.f), 448.f); }

// Four words (8 consecutive elements) -> 8 FP8 bytes (c0, c1) or 8 FP4 nibbles (c0).
template <int FMT>
__device__ __forceinline__ void encode8(const unsigned* w, float s, unsigned& c0, unsigned& c1)
{
    float t[8];
#pragma unroll
    for (int i = 0; i < 4; ++i) scaled2(w[i], s, t[2 * i], t[2 * i + 1]);
    if (FMT == kFP8) {
        short2_t a = {0, 0}, b = {0, 0};
        a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(a, clamp448(t[0]), clamp448(t[1]), 1.0f, false);
        a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(a, clamp448(t[2]), clamp448(t[3]), 1.0f, true);
        b = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(b, clamp448(t[4]), clamp448(t[5]), 1.0f, false);
        b = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(b, clamp448(t[6]), clamp448(t[7]), 1.0f, true);
        c0 = __builtin_bit_cast(unsigned, a);
        c1 = __builtin_bit_cast(unsigned, b);
    } else {
        unsigned r = 0;
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[0], t[1], 1.0f, 0);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[2], t[3], 1.0f, 1);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[4], t[5], 1.0f, 2);
        r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[6], t[7], 1.0f, 3);
        c0 = r;
        c1 = 0;
    }
}

// Error sums of 8 elements for one format: (code / s - x)^2 with code = RNE(x * s); also sum x^2 if asked.
template <int FMT>
__device__ __forceinline__ void err8(const unsigned* w, float s, float inv_s, float& s0, float& se, bool want_s0)
{
    unsigned c0, c1;
    encode8<FMT>(w, s, c0, c1);
    float2_t qq[4];
    if (FMT == kFP8) {
        qq[0] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c0, 1.0f, false);
        qq[1] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c0, 1.0f, true);
        qq[2] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c1, 1.0f, false);
        qq[3] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c1, 1.0f, true);
    } else {
        qq[0] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c0, 1.0f, 0);
        qq[1] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c0, 1.0f, 1);
        qq[2] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c0, 1.0f, 2);
        qq[3] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c0, 1.0f, 3);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float2_t q = qq[i];
        const float xl = __uint_as_float(w[i] << 16), xh = __uint_as_float(w[i] & 0xFFFF0000u);
        const float dl = q[0] * inv_s - xl, dh = q[1] * inv_s - xh;
        se = fmaf(dl, dl, se);
        se = fmaf(dh, dh, se);
        if (want_s0) { s0 = fmaf(xl, xl, s0); s0 = fmaf(xh, xh, s0); }
    }
}

// ------------------------------------------------------------------------------------------
// Block maxima for the 128x128 groups.  One wave per 128 x 128 block of the SOURCE; a lane reads
// two adjacent columns of every row.  Output: the block's scale for FP8 and for FP4 at
// scales8 / scales4 [index], index in the stored orientation (transposed for the column variant).
// ------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void block_scale_kernel(const uint16_t* __restrict__ x, int rows, int cols, int64_t ld,
                                                          int transpose_index, float* __restrict__ scales8,
                                                          float* __restrict__ scales4)
{
    const int lane = threadIdx.x & 63;
    const int nbr = (rows + kGroup - 1) / kGroup, nbc = (cols + kGroup - 1) / kGroup;
    const int nblocks = nbr * nbc;
    const int wave0 = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    for (int b = wave0; b < nblocks; b += gridDim.x * kWavesPerBlock) {
        const int br = b / nbc, bc = b - br * nbc;
        const int c = bc * kGroup + lane * 2;
        const int r0 = br * kGroup, r1 = min(r0 + kGroup, rows);
        // 128 loads in flight, none under a condition: rows past the end repeat the last row (a maximum does not
        // mind), lanes past the last column read column 0 and are discarded
        const uint16_t* const base = x + (c < cols ? c : 0);
        unsigned v[4][32];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int i = 0; i < 32; ++i) v[k][i] = *reinterpret_cast<const unsigned*>(base + (int64_t)min(r0 + k * 32 + i, r1 - 1) * ld);
        unsigned m = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int i = 0; i < 32; ++i) m = pk_max_u16(m, v[k][i] & 0x7FFF7FFFu);
        if (c >= cols) m = 0;
        unsigned am = umax(m & 0xFFFFu, m >> 16);
        for (int off = 32; off > 0; off >>= 1) am = umax(am, (unsigned)__shfl_xor((int)am, off, 64));
        if (lane == 0) {
            const int idx = transpose_index ? bc * nbr + br : br * nbc + bc;
            if (scales8) scales8[idx] = group_scale<kFP8>(am);
            if (scales4) scales4[idx] = group_scale<kFP4>(am);
        }
    }
}

// ------------------------------------------------------------------------------------------
// Blocks along rows.  A lane owns 8 consecutive elements, 16 lanes own a 128-element tile.
// BLOCKS: the scale comes from block_scales [row / 128][col / 128]; otherwise it is the tile's own
// and is written to scales [row][col / 128].
// MODE 0: write codes (+ tile scales).  MODE 1: statistics of both formats, nothing written but partials.
// ------------------------------------------------------------------------------------------
template <int FMT, bool BLOCKS, int MODE>
__global__ __launch_bounds__(256) void paper_row_kernel(const uint16_t* __restrict__ x, int rows, int cols, int64_t ld,
                                                        uint8_t* __restrict__ codes, float* __restrict__ scales,
                                                        const float* __restrict__ block_scales8,
                                                        const float* __restrict__ block_scales4,
                                                        float* __restrict__ partials)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int nwaves = gridDim.x * kWavesPerBlock;
    const int spr = (cols + kSeg - 1) / kSeg;
    const int units = ((rows + kUnroll - 1) / kUnroll) * spr;
    const int ng = cols / kGroup;
    float s0 = 0.f, e4 = 0.f, e8 = 0.f;
    for (int u = wave; u < units; u += nwaves) {
        const int rg = u / spr;
        const int col = (u - rg * spr) * kSeg + lane * 8;
        uint4 v[kUnroll];
        bool act[kUnroll];
#pragma unroll
        for (int j = 0; j < kUnroll; ++j) {
            const int row = rg * kUnroll + j;
            act[j] = row < rows && col < cols;
            v[j] = make_uint4(0, 0, 0, 0);
            if (act[j]) v[j] = ld16_stream(x + (int64_t)row * ld + col);
        }
#pragma unroll
        for (int j = 0; j < kUnroll; ++j) {
            const int row = rg * kUnroll + j;
            const unsigned w[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            const int gidx = BLOCKS ? (row >> 7) * ng + (col >> 7) : row * ng + (col >> 7);
            float s8 = 1.f, s4 = 1.f;
            if (BLOCKS) {
                if (act[j]) {
                    if (MODE == 1 || FMT == kFP8) s8 = block_scales8[gidx];
                    if (MODE == 1 || FMT == kFP4) s4 = block_scales4[gidx];
                }
            } else {
                const unsigned am = row16_max(amax8(v[j]));
                if (MODE == 1 || FMT == kFP8) s8 = group_scale<kFP8>(am);
                if (MODE == 1 || FMT == kFP4) s4 = group_scale<kFP4>(am);
            }
            if (MODE == 0) {
                const float s = FMT == kFP8 ? s8 : s4;
                const bool bad = s != s;
                unsigned c0, c1;
                encode8<FMT>(w, s, c0, c1);
                if (bad) { c0 = 0; c1 = 0; }
                const int64_t e0 = (int64_t)row * cols + col;
                if (act[j]) {
                    if (FMT == kFP8) *reinterpret_cast<uint2*>(codes + e0) = make_uint2(c0, c1);
                    else             *reinterpret_cast<unsigned*>(codes + (e0 >> 1)) = c0;
                    if (!BLOCKS && (lane & 15) == 0) scales[gidx] = s;
                }
            } else if (act[j]) {
                float dummy = 0.f;
                err8<kFP8>(w, s8, __fdiv_rn(1.f, s8), s0, e8, true);
                err8<kFP4>(w, s4, __fdiv_rn(1.f, s4), dummy, e4, false);
            }
        }
    }
    if (MODE == 1) {
        s0 = wave_sum(s0); e4 = wave_sum(e4); e8 = wave_sum(e8);
        if (lane == 0) { partials[wave] = s0; partials[kStreamWaves + wave] = e4; partials[2 * kStreamWaves + wave] = e8; }
    }
}

// ------------------------------------------------------------------------------------------
// Blocks down columns, result stored transposed.  A wave owns 128 columns x 128 rows (one tile per
// column); a lane owns two adjacent columns.  First pass: column maxima (never leave the lane).
// Second pass (the same 32 KB again, from cache): scale, round, and stage the codes in LDS as a
// [128 stored rows][ROWB] image (ROWB = 128 bytes FP8, 64 bytes FP4) whose 16-byte chunks are XOR-swizzled,
// then store it with 16 bytes per lane so that whole 128- / 64-byte runs are written.
// ------------------------------------------------------------------------------------------
template <int FMT>
__device__ __forceinline__ void encode_column(const unsigned* v, int half, float s, uint8_t* __restrict__ lds_row,
                                              int k, int swz)
{
    // rows 2j, 2j+1 of this column are adjacent in the stored row
    float t[32];
#pragma unroll
    for (int i = 0; i < 32; ++i)
        t[i] = __fmul_rn(half ? __uint_as_float(v[i] & 0xFFFF0000u) : __uint_as_float(v[i] << 16), s);
    const bool bad = s != s;
    if (FMT == kFP8) {
        unsigned c[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            short2_t a = {0, 0};
            a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(a, clamp448(t[4 * q]), clamp448(t[4 * q + 1]), 1.0f, false);
            a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(a, clamp448(t[4 * q + 2]), clamp448(t[4 * q + 3]), 1.0f, true);
            c[q] = bad ? 0u : __builtin_bit_cast(unsigned, a);
        }
        *reinterpret_cast<uint4*>(lds_row + (((k * 2 + 0) ^ swz) * 16)) = make_uint4(c[0], c[1], c[2], c[3]);
        *reinterpret_cast<uint4*>(lds_row + (((k * 2 + 1) ^ swz) * 16)) = make_uint4(c[4], c[5], c[6], c[7]);
    } else {
        unsigned c[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            unsigned r = 0;
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[8 * q], t[8 * q + 1], 1.0f, 0);
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[8 * q + 2], t[8 * q + 3], 1.0f, 1);
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[8 * q + 4], t[8 * q + 5], 1.0f, 2);
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[8 * q + 6], t[8 * q + 7], 1.0f, 3);
            c[q] = bad ? 0u : r;
        }
        *reinterpret_cast<uint4*>(lds_row + ((k ^ swz) * 16)) = make_uint4(c[0], c[1], c[2], c[3]);
    }
}

// Error sums of one column's 32 rows for one format.
template <int FMT>
__device__ __forceinline__ void err_column(const unsigned* v, int half, float s, float inv_s, float& s0, float& se, bool want_s0)
{
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        float x[4], t[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[i] = half ? __uint_as_float(v[4 * q + i] & 0xFFFF0000u) : __uint_as_float(v[4 * q + i] << 16);
            t[i] = __fmul_rn(x[i], s);
        }
        float2_t q01, q23;
        if (FMT == kFP8) {
            short2_t a = {0, 0};
            a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(a, clamp448(t[0]), clamp448(t[1]), 1.0f, false);
            a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(a, clamp448(t[2]), clamp448(t[3]), 1.0f, true);
            const unsigned c = __builtin_bit_cast(unsigned, a);
            q01 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c, 1.0f, false);
            q23 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(c, 1.0f, true);
        } else {
            unsigned r = 0;
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[0], t[1], 1.0f, 0);
            r = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(r, t[2], t[3], 1.0f, 1);
            q01 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r, 1.0f, 0);
            q23 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(r, 1.0f, 1);
        }
        const float d0 = q01[0] * inv_s - x[0], d1 = q01[1] * inv_s - x[1];
        const float d2 = q23[0] * inv_s - x[2], d3 = q23[1] * inv_s - x[3];
        se = fmaf(d0, d0, se); se = fmaf(d1, d1, se); se = fmaf(d2, d2, se); se = fmaf(d3, d3, se);
        if (want_s0) { s0 = fmaf(x[0], x[0], s0); s0 = fmaf(x[1], x[1], s0); s0 = fmaf(x[2], x[2], s0); s0 = fmaf(x[3], x[3], s0); }
    }
}

template <int FMT, bool BLOCKS, int MODE>
__global__ __launch_bounds__(256) void paper_col_kernel(const uint16_t* __restrict__ x, int rows, int cols, int64_t ld,
                                                        uint8_t* __restrict__ codes, float* __restrict__ scales,
                                                        const float* __restrict__ block_scales8,
                                                        const float* __restrict__ block_scales4,
                                                        float* __restrict__ partials)
{
    constexpr int ROWB = FMT == kFP8 ? 128 : 64;
    constexpr int CPR = ROWB / 16;
    __shared__ __attribute__((aligned(16))) uint8_t stage[MODE == 0 ? kWavesPerBlock : 1][MODE == 0 ? kColsPerWave * ROWB : 16];
    const int lane = threadIdx.x & 63;
    uint8_t* const reg = stage[MODE == 0 ? (threadIdx.x >> 6) : 0];
    const int wave = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    const int nwaves = gridDim.x * kWavesPerBlock;
    const int ncg = (cols + kColsPerWave - 1) / kColsPerWave;
    const int nru = rows / kGroup;                       // rows is a multiple of 128
    const int units = ncg * nru;
    const int64_t out_row_bytes = FMT == kFP8 ? rows : rows / 2;
    float s0 = 0.f, e4 = 0.f, e8 = 0.f;
    for (int u = wave; u < units; u += nwaves) {
        const int ru = u / ncg, cg = u - ru * ncg;
        const int c = cg * kColsPerWave + lane * 2;
        const bool act = c < cols;
        // The unit's 128 rows of this lane's two columns stay in registers: one read serves the group maximum
        // and the encoding, and all 128 loads are in flight together.  They carry no condition (a lane past the
        // last column reads column 0 of the same rows and is zeroed under a wave-uniform test).
        const uint16_t* const base = x + (int64_t)ru * kGroup * ld + (act ? c : 0);
        unsigned v[4][32];
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int i = 0; i < 32; ++i) v[k][i] = ld4_stream(base + (int64_t)(k * 32 + i) * ld);
        if ((cg + 1) * kColsPerWave > cols) {
#pragma unroll
            for (int k = 0; k < 4; ++k)
#pragma unroll
                for (int i = 0; i < 32; ++i) v[k][i] = act ? v[k][i] : 0u;
        }
        float s8[2] = {1.f, 1.f}, s4[2] = {1.f, 1.f};
        unsigned m = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int i = 0; i < 32; ++i) m = pk_max_u16(m, v[k][i] & 0x7FFF7FFFu);
        if (BLOCKS) {
            // the unit is one 128 x 128 block: its maximum is the maximum over the wave
            unsigned bm = umax(m & 0xFFFFu, m >> 16);
            for (int off = 32; off > 0; off >>= 1) bm = umax(bm, (unsigned)__shfl_xor((int)bm, off, 64));
            if (MODE == 1 || FMT == kFP8) s8[0] = s8[1] = group_scale<kFP8>(bm);
            if (MODE == 1 || FMT == kFP4) s4[0] = s4[1] = group_scale<kFP4>(bm);
            if (MODE == 0 && lane == 0) scales[cg * nru + ru] = FMT == kFP8 ? s8[0] : s4[0];   // stored orientation: [column group][row group]
        } else {
            const unsigned am[2] = {m & 0xFFFFu, m >> 16};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                if (MODE == 1 || FMT == kFP8) s8[h] = group_scale<kFP8>(am[h]);
                if (MODE == 1 || FMT == kFP4) s4[h] = group_scale<kFP4>(am[h]);
            }
            if (MODE == 0 && act) {
                scales[(int64_t)c * nru + ru] = FMT == kFP8 ? s8[0] : s4[0];
                scales[(int64_t)(c + 1) * nru + ru] = FMT == kFP8 ? s8[1] : s4[1];
            }
        }
        const int swz = lane & (CPR - 1);
        float inv8[2], inv4[2];
        if (MODE == 1) {
#pragma unroll
            for (int h = 0; h < 2; ++h) { inv8[h] = __fdiv_rn(1.f, s8[h]); inv4[h] = __fdiv_rn(1.f, s4[h]); }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (MODE == 0) {
                encode_column<FMT>(v[k], 0, FMT == kFP8 ? s8[0] : s4[0], reg + (2 * lane) * ROWB, k, swz);
                encode_column<FMT>(v[k], 1, FMT == kFP8 ? s8[1] : s4[1], reg + (2 * lane + 1) * ROWB, k, swz);
            } else if (act) {
                float dummy = 0.f;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    err_column<kFP8>(v[k], h, s8[h], inv8[h], s0, e8, true);
                    err_column<kFP4>(v[k], h, s4[h], inv4[h], dummy, e4, false);
                }
            }
        }
        if (MODE == 0) {
#pragma unroll
            for (int it = 0; it < kColsPerWave * CPR / 64; ++it) {
                const int idx = it * 64 + lane;
                const int row = idx / CPR, chunk = idx % CPR;
                const uint4 val = *reinterpret_cast<const uint4*>(reg + row * ROWB + ((chunk ^ ((row >> 1) & (CPR - 1))) * 16));
                const int cc = cg * kColsPerWave + row;
                if (cc < cols)
                    *reinterpret_cast<uint4*>(codes + (int64_t)cc * out_row_bytes + (int64_t)ru * ROWB + chunk * 16) = val;
            }
        }
    }
    if (MODE == 1) {
        s0 = wave_sum(s0); e4 = wave_sum(e4); e8 = wave_sum(e8);
        if (lane == 0) { partials[wave] = s0; partials[kStreamWaves + wave] = e4; partials[2 * kStreamWaves + wave] = e8; }
    }
}

int blocks_for(int64_t units)
{
    if (units <= 0) return 1;
    const int64_t per_wave = (units + kStreamWaves - 1) / kStreamWaves;
    const int64_t waves = (units + per_wave - 1) / per_wave;
    return (int)((waves + kWavesPerBlock - 1) / kWavesPerBlock);
}

template <int FMT, bool BLOCKS, int MODE>
int launch_one(const PaperArgs& a, const float* bs8, const float* bs4, float* partials, hipStream_t s)
{
    int blocks;
    if (a.axis == 0) {
        blocks = blocks_for(((a.rows + kUnroll - 1) / kUnroll) * ((a.cols + kSeg - 1) / kSeg));
        hipLaunchKernelGGL((paper_row_kernel<FMT, BLOCKS, MODE>), dim3(blocks), dim3(256), 0, s,
                           a.x, (int)a.rows, (int)a.cols, a.ld, a.codes, a.scales, bs8, bs4, partials);
    } else {
        blocks = blocks_for(((a.cols + kColsPerWave - 1) / kColsPerWave) * (a.rows / kGroup));
        hipLaunchKernelGGL((paper_col_kernel<FMT, BLOCKS, MODE>), dim3(blocks), dim3(256), 0, s,
                           a.x, (int)a.rows, (int)a.cols, a.ld, a.codes, a.scales, bs8, bs4, partials);
    }
    return blocks;
}

}  // namespace

size_t paper_workspace_bytes(int64_t rows, int64_t cols)
{
    const size_t nblocks = (size_t)((rows + kGroup - 1) / kGroup) * (size_t)((cols + kGroup - 1) / kGroup);
    return 3 * (size_t)kStreamWaves * sizeof(float) + 2 * nblocks * sizeof(float);
}

// Workspace layout: [3][kStreamWaves] float partial sums, then the FP8 and the FP4 block-scale arrays.
hipError_t launch_paper(const PaperArgs& a, hipStream_t s)
{
    const bool stats = a.stats != nullptr;
    float* partials = (float*)a.workspace;
    const bool empty = a.rows == 0 || a.cols == 0;
    const size_t nblocks = (size_t)((a.rows + kGroup - 1) / kGroup) * (size_t)((a.cols + kGroup - 1) / kGroup);
    float* bs8 = nullptr;
    float* bs4 = nullptr;
    if (a.blocks && !empty && a.axis == 0) {       // the column kernel finds its blocks' maxima itself
        if (stats) { bs8 = partials + 3 * kStreamWaves; bs4 = bs8 + nblocks; }
        else       { bs8 = a.fmt == kFP8 ? a.scales : nullptr; bs4 = a.fmt == kFP4 ? a.scales : nullptr; }   // the output array itself
        hipLaunchKernelGGL(block_scale_kernel, dim3(blocks_for((int64_t)nblocks)), dim3(256), 0, s,
                           a.x, (int)a.rows, (int)a.cols, a.ld, a.axis == 1 ? 1 : 0, bs8, bs4);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    int blocks = 0;
    if (!empty) {
        if (stats) {
            blocks = a.blocks ? launch_one<kFP8, true, 1>(a, bs8, bs4, partials, s) : launch_one<kFP8, false, 1>(a, bs8, bs4, partials, s);
        } else if (a.fmt == kFP8) {
            blocks = a.blocks ? launch_one<kFP8, true, 0>(a, bs8, bs4, partials, s) : launch_one<kFP8, false, 0>(a, bs8, bs4, partials, s);
        } else {
            blocks = a.blocks ? launch_one<kFP4, true, 0>(a, bs8, bs4, partials, s) : launch_one<kFP4, false, 0>(a, bs8, bs4, partials, s);
        }
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (stats) {
        const int64_t n = (int64_t)blocks * kWavesPerBlock;
        for (int j = 0; j < 3; ++j) {
            const hipError_t e = launch_sum_partials(partials + (size_t)j * kStreamWaves, n, a.stats + j, s);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace snip
