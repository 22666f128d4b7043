// GEMM on operands quantized with the paper's own recipe (SNIP Sec. 2.3 / 5.1: real-valued scale per
// 1x128 tile or 128x128 block): C[I][J] = sum_r (A[i][r] / sa) * (B[j][r] / sb).
//
// The matrix instruction applies only power-of-two scales to 32-element blocks, so the real-valued scales
// are applied in software: the contraction runs in slabs of 128 elements (one scaling group of either
// operand); the codes of a slab are multiplied on the matrix cores with unit scales into a fresh fp32
// accumulator, which is then folded into the running result with the factor (1/sa) * (1/sb) of that slab.
// A's factor is per output row (tiles) or per 128 rows (blocks), B's per output column or per 128 columns;
// both cases read their factor through the same index function.
//
// 128 x 128 workgroup tile, 4 waves of 64 x 64 (two accumulator sets of 64 registers), operands staged
// global -> registers -> LDS with the next slab's loads in flight during the current slab's MFMAs.  The fold
// costs about as many VALU cycles as the slab's FP8 MFMAs take, so this kernel runs well below the
// block-scaled path; it exists so that the paper's configuration can be reproduced end to end.
// Register layout of the instruction: see gemm.hip.
#include "snip_internal.h"

namespace snip {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

constexpr int BM = 128, BN = 128, WM = 64, WN = 64, NTHREADS = 256;
constexpr int KE = 128;                         // contraction elements per slab = per stage
constexpr unsigned kUnitScale = 0x7F7F7F7Fu;    // E8M0 127 = 2^0 in every byte

template <int F> struct Op {
    static constexpr int SB = F == kFP8 ? KE : KE / 2;      // code bytes per row per slab
    static constexpr int PITCH = SB + 16;                   // padded LDS row pitch
    static constexpr int CPR = SB / 16;
    static constexpr int NCH = BM * CPR / NTHREADS;         // 16-byte chunks per thread
};

template <int F>
__device__ __forceinline__ void gload(uint4* r, const uint8_t* __restrict__ codes, int64_t row_bytes, int row0,
                                      int nrows, int64_t kbyte0)
{
#pragma unroll
    for (int i = 0; i < Op<F>::NCH; ++i) {
        const int q = threadIdx.x + NTHREADS * i;
        const int row = q / Op<F>::CPR, ch = q % Op<F>::CPR;
        r[i] = make_uint4(0, 0, 0, 0);
        if (row0 + row < nrows) r[i] = *reinterpret_cast<const uint4*>(codes + (int64_t)(row0 + row) * row_bytes + kbyte0 + ch * 16);
    }
}
template <int F>
__device__ __forceinline__ void sstore(const uint4* r, uint8_t* lds)
{
#pragma unroll
    for (int i = 0; i < Op<F>::NCH; ++i) {
        const int q = threadIdx.x + NTHREADS * i;
        const int row = q / Op<F>::CPR, ch = q % Op<F>::CPR;
        *reinterpret_cast<uint4*>(lds + row * Op<F>::PITCH + ch * 16) = r[i];
    }
}
template <int F>
__device__ __forceinline__ v8i load_frag(const uint8_t* lds, int row, int g, int ks)
{
    v8i f = {0, 0, 0, 0, 0, 0, 0, 0};
    if (F == kFP8) {
        const uint4 a = *reinterpret_cast<const uint4*>(lds + row * Op<F>::PITCH + ks * 64 + 16 * g);
        const uint4 b = *reinterpret_cast<const uint4*>(lds + row * Op<F>::PITCH + ks * 64 + 32 + 16 * g);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    } else {
        const uint4 a = *reinterpret_cast<const uint4*>(lds + row * Op<F>::PITCH + ks * 32 + 16 * g);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    }
    return f;
}

// Scale of (row, slab) as stored; +infinity for rows past the end, whose reciprocal (the factor used) is zero.
// The reciprocal is taken one slab later, when the load has landed anyway: a use right after the load would make
// the wave wait for every load in flight, the next slab's operands included.
__device__ __forceinline__ float raw_scale(const float* __restrict__ scales, int row, int nrows, int group_rows,
                                           int ng, int slab)
{
    if (row >= nrows) return __builtin_inff();
    return scales[(int64_t)(group_rows == 1 ? row : row >> 7) * ng + slab];
}

template <int FA, int FB, bool OUT_F32>
__global__ __launch_bounds__(NTHREADS) void gemm_paper_kernel(const uint8_t* __restrict__ a_codes, const float* __restrict__ a_scales,
                                                              int a_group, const uint8_t* __restrict__ b_codes,
                                                              const float* __restrict__ b_scales, int b_group,
                                                              int I, int J, int R, void* __restrict__ c_out, int64_t ldc,
                                                              int tiles_j)
{
    __shared__ __attribute__((aligned(16))) uint8_t lds_a[BM * Op<FA>::PITCH];
    __shared__ __attribute__((aligned(16))) uint8_t lds_b[BN * Op<FB>::PITCH];
    __shared__ __attribute__((aligned(16))) float lds_db[2][BN];          // B's factors of a slab, double-buffered

    const int ti = blockIdx.x / tiles_j, tj = blockIdx.x % tiles_j;
    const int i0 = ti * BM, j0 = tj * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r32 = lane & 31, g = lane >> 5;
    const int64_t a_row_bytes = FA == kFP8 ? R : R / 2, b_row_bytes = FB == kFP8 ? R : R / 2;
    const int nslab = R / KE;

    uint4 ra[Op<FA>::NCH], rb[Op<FB>::NCH];
    v16f acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[a][b][k] = 0.f;

    int arow[2];
#pragma unroll
    for (int ib = 0; ib < 2; ++ib) arow[ib] = i0 + wm * WM + ib * 32 + r32;
    const int bcol = j0 + (threadIdx.x & (BN - 1));            // the column whose factor this thread fetches

    float sa_n[2] = {raw_scale(a_scales, arow[0], I, a_group, nslab, 0), raw_scale(a_scales, arow[1], I, a_group, nslab, 0)};
    float sb_n = raw_scale(b_scales, bcol, J, b_group, nslab, 0);
    gload<FA>(ra, a_codes, a_row_bytes, i0, I, 0);
    gload<FB>(rb, b_codes, b_row_bytes, j0, J, 0);

    for (int s = 0; s < nslab; ++s) {
        __syncthreads();                                       // the previous slab's LDS reads are done
        sstore<FA>(ra, lds_a);
        sstore<FB>(rb, lds_b);
        if (threadIdx.x < BN) lds_db[s & 1][threadIdx.x] = __fdiv_rn(1.f, sb_n);
        const float da[2] = {__fdiv_rn(1.f, sa_n[0]), __fdiv_rn(1.f, sa_n[1])};
        __syncthreads();
        if (s + 1 < nslab) {
            sa_n[0] = raw_scale(a_scales, arow[0], I, a_group, nslab, s + 1);
            sa_n[1] = raw_scale(a_scales, arow[1], I, a_group, nslab, s + 1);
            sb_n = raw_scale(b_scales, bcol, J, b_group, nslab, s + 1);
            gload<FA>(ra, a_codes, a_row_bytes, i0, I, (int64_t)(s + 1) * Op<FA>::SB);
            gload<FB>(rb, b_codes, b_row_bytes, j0, J, (int64_t)(s + 1) * Op<FB>::SB);
        }
        // the slab's products with unit scales, into a fresh accumulator
        v16f tmp[2][2];
        constexpr int ca = FB == kFP8 ? 0 : 4, cb = FA == kFP8 ? 0 : 4;     // first operand = B tile
#pragma unroll
        for (int ks = 0; ks < KE / 64; ++ks) {
            v8i fa[2], fb[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                fa[b] = load_frag<FA>(lds_a, wm * WM + b * 32 + r32, g, ks);
                fb[b] = load_frag<FB>(lds_b, wn * WN + b * 32 + r32, g, ks);
            }
#pragma unroll
            for (int ib = 0; ib < 2; ++ib)
#pragma unroll
                for (int jb = 0; jb < 2; ++jb) {
                    v16f c0;
                    if (ks == 0) {
#pragma unroll
                        for (int k = 0; k < 16; ++k) c0[k] = 0.f;
                    } else {
                        c0 = tmp[ib][jb];
                    }
                    tmp[ib][jb] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[jb], fa[ib], c0, ca, cb, 0, (int)kUnitScale,
                                                                                  0, (int)kUnitScale);
                }
        }
        // fold: lane (r32, g) holds C[row r32][column 8q + 4g + t] in register 4q + t of each 32 x 32 block
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 db = *reinterpret_cast<const float4*>(&lds_db[s & 1][wn * WN + jb * 32 + 8 * q + 4 * g]);
                const float dbv[4] = {db.x, db.y, db.z, db.w};
#pragma unroll
                for (int ib = 0; ib < 2; ++ib)
#pragma unroll
                    for (int t = 0; t < 4; ++t)
                        acc[ib][jb][4 * q + t] = fmaf(tmp[ib][jb][4 * q + t], __fmul_rn(da[ib], dbv[t]), acc[ib][jb][4 * q + t]);
            }
    }

    // epilogue: lane owns row i, register quad q owns columns 8q + 4g .. +3 of each 32-wide block
#pragma unroll
    for (int ib = 0; ib < 2; ++ib) {
        const int i = i0 + wm * WM + ib * 32 + r32;
        if (i >= I) continue;
#pragma unroll
        for (int jb = 0; jb < 2; ++jb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = j0 + wn * WN + jb * 32 + 8 * q + 4 * g;
                const float v0 = acc[ib][jb][4 * q + 0], v1 = acc[ib][jb][4 * q + 1];
                const float v2 = acc[ib][jb][4 * q + 2], v3 = acc[ib][jb][4 * q + 3];
                if (OUT_F32) {
                    float* p = reinterpret_cast<float*>(c_out) + (int64_t)i * ldc + j;
                    if (j + 3 < J) *reinterpret_cast<float4*>(p) = make_float4(v0, v1, v2, v3);
                    else { if (j < J) p[0] = v0; if (j + 1 < J) p[1] = v1; if (j + 2 < J) p[2] = v2; }
                } else {
                    __bf16* p = reinterpret_cast<__bf16*>(c_out) + (int64_t)i * ldc + j;
                    if (j + 3 < J) {
                        const float2_t lo = {v0, v1}, hi = {v2, v3};
                        const bf16x2 blo = __builtin_convertvector(lo, bf16x2), bhi = __builtin_convertvector(hi, bf16x2);
                        *reinterpret_cast<uint2*>(p) = make_uint2(__builtin_bit_cast(unsigned, blo), __builtin_bit_cast(unsigned, bhi));
                    } else {
                        if (j < J) p[0] = (__bf16)v0;
                        if (j + 1 < J) p[1] = (__bf16)v1;
                        if (j + 2 < J) p[2] = (__bf16)v2;
                    }
                }
            }
    }
}

template <int FA, int FB>
hipError_t launch_t(const GemmPaperArgs& a, hipStream_t s)
{
    const int ti = (int)((a.I + BM - 1) / BM), tj = (int)((a.J + BN - 1) / BN);
    const dim3 grid((unsigned)(ti * tj)), block(NTHREADS);
    if (a.out_fp32)
        hipLaunchKernelGGL((gemm_paper_kernel<FA, FB, true>), grid, block, 0, s, a.a_codes, a.a_scales, a.a_group, a.b_codes,
                           a.b_scales, a.b_group, (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, tj);
    else
        hipLaunchKernelGGL((gemm_paper_kernel<FA, FB, false>), grid, block, 0, s, a.a_codes, a.a_scales, a.a_group, a.b_codes,
                           a.b_scales, a.b_group, (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, tj);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_paper(const GemmPaperArgs& a, hipStream_t s)
{
    if (a.I == 0 || a.J == 0) return hipSuccess;
    if (a.fmt_a == kFP8 && a.fmt_b == kFP8) return launch_t<kFP8, kFP8>(a, s);
    if (a.fmt_a == kFP8 && a.fmt_b == kFP4) return launch_t<kFP8, kFP4>(a, s);
    if (a.fmt_a == kFP4 && a.fmt_b == kFP8) return launch_t<kFP4, kFP8>(a, s);
    return launch_t<kFP4, kFP4>(a, s);
}

}  // namespace snip
