// Block-scaled FP8/FP4 GEMM on gfx950 scaled MFMA: C[I][J] = sum_r A[I][r] * B[J][r] with
// a = code * 2^(scale-127) (SNIP Sec. 2.2: the three GEMMs of a linear layer all take this
// form once each operand is stored with its contraction dimension contiguous).
//
// Instruction: v_mfma_scale_f32_32x32x64_f8f6f4.  Register layout (established with one-hot
// probes on the hardware):
//   - 64 contraction elements per instruction = two 32-element scale blocks.
//   - lane l supplies row (l % 32) of its operand; g = l / 32.
//     FP8: 32 bytes per lane: VGPR0-3 = bytes [16g, 16g+16) and VGPR4-7 = bytes
//          [32+16g, 32+16g+16) of the row's 64-byte slab.
//     FP4: 16 bytes per lane (VGPR0-3) = bytes [16g, 16g+16) of the row's 32-byte slab, i.e.
//          elements [32g, 32g+32), low nibble first.
//   - the scale of (row r, block b) is read from lane 32*b + r, byte `opsel` of its scale VGPR.
//   - result: lane l holds column (l % 32) of the second operand's rows; register q*4+t holds
//     row 8q + 4(l/32) + t of the first operand's rows.
// The B tile is fed as the first operand and the A tile as the second, so that a lane ends up
// with 4 consecutive output columns per register quad.
#include "snip_internal.h"

namespace snip {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

constexpr int BM = 128, BN = 128;          // workgroup tile (A rows x B rows)
constexpr int WM = 64, WN = 64;            // wave tile
constexpr int NTHREADS = 256;

template <int FA, int FB> struct Cfg {
    static constexpr int KE = (FA == kFP4 && FB == kFP4) ? 256 : 128;   // contraction elements per stage
    static constexpr int SBA = FA == kFP8 ? KE : KE / 2;                 // code bytes per row per stage
    static constexpr int SBB = FB == kFP8 ? KE : KE / 2;
    static constexpr int PA = SBA + 16, PB = SBB + 16;                   // padded LDS row pitch
    static constexpr int KS = KE / 64;                                   // MFMA steps per stage
    static constexpr int NSD = KE / 128;                                 // scale dwords per row per stage
};

// Four scale bytes of `row` starting at block kb (zero beyond nkb).
__device__ __forceinline__ unsigned load_scale4(const uint8_t* __restrict__ srow, int kb, int nkb, bool row_ok, bool aligned)
{
    if (!row_ok || kb >= nkb) return 0u;
    if (aligned) return *reinterpret_cast<const unsigned*>(srow + kb);
    unsigned s = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        if (kb + i < nkb) s |= (unsigned)srow[kb + i] << (8 * i);
    return s;
}

template <int F, int SB, int PITCH, int ROWS>
struct TileLoader {
    static constexpr int CPR = SB / 16;                   // 16-byte chunks per row
    static constexpr int NCH = ROWS * CPR / NTHREADS;     // chunks per thread
    uint4 r[NCH];
    __device__ __forceinline__ void gload(const uint8_t* __restrict__ codes, int64_t row_bytes, int row0, int nrows,
                                          int64_t kbyte0)
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int q = threadIdx.x + NTHREADS * i;
            const int row = q / CPR, ch = q % CPR;
            const int64_t kb = kbyte0 + ch * 16;
            r[i] = make_uint4(0, 0, 0, 0);
            if (row0 + row < nrows && kb < row_bytes)
                r[i] = *reinterpret_cast<const uint4*>(codes + (int64_t)(row0 + row) * row_bytes + kb);
        }
    }
    __device__ __forceinline__ void sstore(uint8_t* lds) const
    {
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const int q = threadIdx.x + NTHREADS * i;
            const int row = q / CPR, ch = q % CPR;
            *reinterpret_cast<uint4*>(lds + row * PITCH + ch * 16) = r[i];
        }
    }
};

// Operand registers of one 32-row block for MFMA step ks, read from the LDS tile.
template <int F, int PITCH>
__device__ __forceinline__ v8i load_frag(const uint8_t* lds, int row, int g, int ks)
{
    v8i f = {0, 0, 0, 0, 0, 0, 0, 0};
    if (F == kFP8) {
        const uint4 a = *reinterpret_cast<const uint4*>(lds + row * PITCH + ks * 64 + 16 * g);
        const uint4 b = *reinterpret_cast<const uint4*>(lds + row * PITCH + ks * 64 + 32 + 16 * g);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w; f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
    } else {
        const uint4 a = *reinterpret_cast<const uint4*>(lds + row * PITCH + ks * 32 + 16 * g);
        f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
    }
    return f;
}

template <int FA, int FB, int OP>
__device__ __forceinline__ v16f mfma(const v8i& bfrag, const v8i& afrag, v16f acc, unsigned sb, unsigned sa)
{
    constexpr int ca = FB == kFP8 ? 0 : 4;   // first operand = B tile
    constexpr int cb = FA == kFP8 ? 0 : 4;   // second operand = A tile
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bfrag, afrag, acc, ca, cb, OP, (int)sb, OP, (int)sa);
}

template <int FA, int FB, bool OUT_F32>
__global__ __launch_bounds__(NTHREADS) void gemm_kernel(const uint8_t* __restrict__ a_codes,
                                                        const uint8_t* __restrict__ a_scales,
                                                        const uint8_t* __restrict__ b_codes,
                                                        const uint8_t* __restrict__ b_scales,
                                                        int I, int J, int R, void* __restrict__ c_out, int64_t ldc,
                                                        int tiles_i, int tiles_j, float* __restrict__ norm_partials)
{
    using C = Cfg<FA, FB>;
    __shared__ __attribute__((aligned(16))) uint8_t lds_a[BM * C::PA];
    __shared__ __attribute__((aligned(16))) uint8_t lds_b[BN * C::PB];

    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
    // tiles so that tiles sharing an operand meet in the same L2.
    const int nblk = tiles_i * tiles_j;
    int bid = blockIdx.x;
    {
        const int per = nblk / 8;
        if (bid < per * 8) bid = (bid % 8) * per + bid / 8;
    }
    // Walk J fastest inside bands of 8 tile rows.
    const int band = 8;
    const int band_sz = band * tiles_j;
    const int b0 = bid / band_sz;
    const int rem = bid - b0 * band_sz;
    const int rows_in_band = min(band, tiles_i - b0 * band);
    const int ti = b0 * band + rem % rows_in_band;
    const int tj = rem / rows_in_band;

    const int i0 = ti * BM, j0 = tj * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int r32 = lane & 31, g = lane >> 5;

    const int64_t a_row_bytes = FA == kFP8 ? R : R / 2;
    const int64_t b_row_bytes = FB == kFP8 ? R : R / 2;
    const int nkb = R / kBlock;
    const bool sc_aligned = (nkb & 3) == 0;

    TileLoader<FA, C::SBA, C::PA, BM> la;
    TileLoader<FB, C::SBB, C::PB, BN> lb;

    v16f acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[a][b][k] = 0.f;

    const int nstage = (R + C::KE - 1) / C::KE;
    la.gload(a_codes, a_row_bytes, i0, I, 0);
    lb.gload(b_codes, b_row_bytes, j0, J, 0);

    // scale rows owned by this lane
    int arow[2], brow[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) { arow[b] = i0 + wm * WM + b * 32 + r32; brow[b] = j0 + wn * WN + b * 32 + r32; }
    unsigned sa[2][C::NSD], sb[2][C::NSD], sa_n[2][C::NSD], sb_n[2][C::NSD];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int d = 0; d < C::NSD; ++d) {
            sa_n[b][d] = load_scale4(a_scales + (int64_t)arow[b] * nkb, d * 4, nkb, arow[b] < I, sc_aligned);
            sb_n[b][d] = load_scale4(b_scales + (int64_t)brow[b] * nkb, d * 4, nkb, brow[b] < J, sc_aligned);
        }

    for (int s = 0; s < nstage; ++s) {
        __syncthreads();
        la.sstore(lds_a);
        lb.sstore(lds_b);
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int d = 0; d < C::NSD; ++d) { sa[b][d] = sa_n[b][d] >> (8 * g); sb[b][d] = sb_n[b][d] >> (8 * g); }
        __syncthreads();
        if (s + 1 < nstage) {
            la.gload(a_codes, a_row_bytes, i0, I, (int64_t)(s + 1) * C::SBA);
            lb.gload(b_codes, b_row_bytes, j0, J, (int64_t)(s + 1) * C::SBB);
            const int kb0 = (s + 1) * (C::KE / kBlock);
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int d = 0; d < C::NSD; ++d) {
                    sa_n[b][d] = load_scale4(a_scales + (int64_t)arow[b] * nkb, kb0 + d * 4, nkb, arow[b] < I, sc_aligned);
                    sb_n[b][d] = load_scale4(b_scales + (int64_t)brow[b] * nkb, kb0 + d * 4, nkb, brow[b] < J, sc_aligned);
                }
        }
#pragma unroll
        for (int ks = 0; ks < C::KS; ++ks) {
            v8i fa[2], fb[2];
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                fa[b] = load_frag<FA, C::PA>(lds_a, wm * WM + b * 32 + r32, g, ks);
                fb[b] = load_frag<FB, C::PB>(lds_b, wn * WN + b * 32 + r32, g, ks);
            }
            const int d = ks >> 1;
#pragma unroll
            for (int ib = 0; ib < 2; ++ib)
#pragma unroll
                for (int jb = 0; jb < 2; ++jb) {
                    if ((ks & 1) == 0) acc[ib][jb] = mfma<FA, FB, 0>(fb[jb], fa[ib], acc[ib][jb], sb[jb][d], sa[ib][d]);
                    else               acc[ib][jb] = mfma<FA, FB, 2>(fb[jb], fa[ib], acc[ib][jb], sb[jb][d], sa[ib][d]);
                }
        }
    }

    // Optional: sum of squares of the tile as it will be stored (rounded to the output type), elements
    // outside the matrix excluded; one partial per workgroup, combined by reduce_norm_kernel.
    if (norm_partials) {
        float ss = 0.f;
#pragma unroll
        for (int ib = 0; ib < 2; ++ib) {
            const bool row_ok = i0 + wm * WM + ib * 32 + r32 < I;
#pragma unroll
            for (int jb = 0; jb < 2; ++jb)
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    const int col = j0 + wn * WN + jb * 32 + 8 * (k >> 2) + 4 * g + (k & 3);
                    float v = acc[ib][jb][k];
                    if (!OUT_F32) v = (float)(__bf16)v;
                    ss = (row_ok && col < J) ? fmaf(v, v, ss) : ss;
                }
        }
        for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
        __shared__ float wave_ss[NTHREADS / 64];
        if (lane == 0) wave_ss[wave] = ss;
        __syncthreads();
        if (threadIdx.x == 0) {
            float t = 0.f;
            for (int w = 0; w < NTHREADS / 64; ++w) t += wave_ss[w];
            norm_partials[blockIdx.x] = t;
        }
    }

    // Epilogue: lane owns row i, register quad q owns columns 8q + 4g .. +3 of each 32-wide block.
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
hipError_t launch_t(const GemmArgs& a, hipStream_t s)
{
    const int ti = (int)((a.I + BM - 1) / BM), tj = (int)((a.J + BN - 1) / BN);
    const dim3 grid((unsigned)(ti * tj)), block(NTHREADS);
    if (a.out_fp32)
        hipLaunchKernelGGL((gemm_kernel<FA, FB, true>), grid, block, 0, s, a.a_codes, a.a_scales, a.b_codes, a.b_scales,
                           (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, ti, tj, a.norm_partials);
    else
        hipLaunchKernelGGL((gemm_kernel<FA, FB, false>), grid, block, 0, s, a.a_codes, a.a_scales, a.b_codes, a.b_scales,
                           (int)a.I, (int)a.J, (int)a.R, a.c, a.ldc, ti, tj, a.norm_partials);
    return hipGetLastError();
}

}  // namespace

// Sum of n workgroup partials in index order, in double: one workgroup, thread t adds t, t + 1024, ...,
// then a shared-memory tree.
constexpr int kNormThreads = 1024;
__global__ __launch_bounds__(kNormThreads) void reduce_norm_kernel(const float* __restrict__ partials, int64_t n,
                                                                   double* __restrict__ out)
{
    __shared__ double sh[kNormThreads];
    double a = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += kNormThreads) a += (double)partials[i];
    sh[threadIdx.x] = a;
    __syncthreads();
    for (int st = kNormThreads / 2; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) sh[threadIdx.x] += sh[threadIdx.x + st];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = sh[0];
}

hipError_t launch_sum_partials(const float* partials, int64_t n, double* out, hipStream_t s)
{
    hipLaunchKernelGGL(reduce_norm_kernel, dim3(1), dim3(kNormThreads), 0, s, partials, n, out);
    return hipGetLastError();
}

static hipError_t launch_gemm_kernel(const GemmArgs& a, hipStream_t s)
{
    if (gemm_fast_eligible(a)) return launch_gemm_fast(a, s);
    if (a.fmt_a == kFP8 && a.fmt_b == kFP8) return launch_t<kFP8, kFP8>(a, s);
    if (a.fmt_a == kFP8 && a.fmt_b == kFP4) return launch_t<kFP8, kFP4>(a, s);
    if (a.fmt_a == kFP4 && a.fmt_b == kFP8) return launch_t<kFP4, kFP8>(a, s);
    return launch_t<kFP4, kFP4>(a, s);
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s)
{
    const bool empty = a.I == 0 || a.J == 0;
    if (!empty) {
        const hipError_t e = launch_gemm_kernel(a, s);
        if (e != hipSuccess) return e;
    }
    if (a.norm_out) {
        int64_t n = 0;
        if (!empty)
            n = gemm_fast_eligible(a) ? gemm_fast_partials(a)
                                      : ((a.I + BM - 1) / BM) * ((a.J + BN - 1) / BN);
        return launch_sum_partials(a.norm_partials, n, a.norm_out, s);
    }
    return hipSuccess;
}

}  // namespace snip
